"""Training-side operators (Sec. III Eqs. 3-9) through the C ABI against the CPU oracle: APB(w) bit for bit,
the straight-through gradient bit for bit, the size of the binarized set exactly, and the two float64
reductions dL/dalpha, dL/ddelta within 1e-6 relative of the oracle's (the terms are formed by the same
float64 operations; only the order of the additions differs)."""
import numpy as np
import pytest
import torch

from oracle import apb_train_oracle as t
from paper_2306_08960_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2306_08960_amd import binding
    binding.load()
    return binding


def _close(got, want, scale):
    # relative to the sum of the magnitudes of the terms is what reordering float64 additions can move;
    # 1e-6 of the value itself is the stated bar, with that floor for sums that cancel
    return abs(got - want) <= 1e-6 * abs(want) + 1e-13 * scale


def _check(b, W, G, alpha, delta, tag):
    print(f"[case] train {tag} n={W.size} alpha={alpha} delta={delta}", flush=True)
    Wd, Gd = torch.from_numpy(W).cuda(), torch.from_numpy(G).cuda()
    out = b.apb_train_forward(Wd, alpha, delta).cpu().numpy()
    assert np.array_equal(out.view(np.uint32), t.apb_operator(W, alpha, delta).view(np.uint32))
    grad_w, sums, count = b.apb_train_backward(Wd, Gd, alpha, delta)
    ref = t.backward(W, G, alpha, delta)
    assert np.array_equal(grad_w.cpu().numpy().view(np.uint32), ref["grad_w"].view(np.uint32))
    assert int(count.item()) == ref["n_binarized"]
    ga, gd = sums.cpu().numpy().tolist()
    mag = float(np.sum(np.abs(G.astype(np.float64)))) / W.size
    assert _close(ga, ref["grad_alpha"], mag), (ga, ref["grad_alpha"])
    assert _close(gd, ref["grad_delta"], mag * (abs(alpha) + float(np.abs(W).max())) / delta), (gd, ref["grad_delta"])
    # deterministic: a second call gives the same bits; without grad_w the sums are the same too
    _, sums2, _ = b.apb_train_backward(Wd, Gd, alpha, delta, want_grad_w=False)
    assert torch.equal(sums, sums2)


@pytest.mark.parametrize("n", [1, 3, 4, 63, 64, 257, 1000, 4099, 1 << 20, (1 << 20) + 3])
def test_sizes_and_ragged_tails(b, n):
    g = np.random.default_rng(n)
    W = (g.standard_normal(n) * 0.05).astype(np.float32)
    G = g.standard_normal(n).astype(np.float32)
    _check(b, W, G, 0.04, 0.06, "ragged")


def test_boundary_values_signed_zeros_and_empty_sets(b):
    lim = np.float32(np.float32(0.25) + np.float32(0.5))
    W = np.array([0.0, -0.0, lim, -lim, np.nextafter(lim, np.float32(1)), -np.nextafter(lim, np.float32(1)), 1e-45, -1e-45,
                  0.25, -0.25, 3.0, -3.0], dtype=np.float32)
    G = np.arange(1, W.size + 1, dtype=np.float32)
    _check(b, W, G, 0.25, 0.5, "boundary")
    big = np.full(1000, 7.0, dtype=np.float32)
    _check(b, big, np.ones(1000, dtype=np.float32), 0.25, 0.5, "nothing binarized")
    _check(b, big, np.ones(1000, dtype=np.float32), 0.25, 100.0, "everything binarized")
    _check(b, W, G, 0.0, 0.5, "alpha zero")


def test_unaligned_views_take_the_scalar_path(b):
    g = np.random.default_rng(5)
    W = (g.standard_normal(4097) * 0.05).astype(np.float32)
    G = g.standard_normal(4097).astype(np.float32)
    Wd, Gd = torch.from_numpy(W).cuda()[1:], torch.from_numpy(G).cuda()[1:]        # 4-byte aligned only
    out = b.apb_train_forward(Wd, 0.04, 0.06)
    assert np.array_equal(out.cpu().numpy(), t.apb_operator(W[1:], 0.04, 0.06))
    _, sums, count = b.apb_train_backward(Wd, Gd, 0.04, 0.06)
    ref = t.backward(W[1:], G[1:], 0.04, 0.06)
    assert int(count.item()) == ref["n_binarized"]
    assert sums[0].item() == pytest.approx(ref["grad_alpha"], rel=1e-6)
    assert sums[1].item() == pytest.approx(ref["grad_delta"], rel=1e-6)


@pytest.mark.parametrize("name", ["C2", "C4", "C5a", "C5b"])
def test_benchmark_layers_at_full_size(b, name):
    cfg = synth.CONFIGS[name]
    W, delta_total = synth.make_weights(cfg)
    g = np.random.default_rng(cfg.index)
    G = g.standard_normal(W.shape).astype(np.float32)
    alpha = float(np.float32(np.mean(np.abs(W))))
    delta = float(np.float32(np.float32(delta_total) - np.float32(alpha)))          # interval = the config's
    _check(b, W, G, alpha, delta, name)


def test_argument_errors(b):
    W = torch.zeros(8, device="cuda")
    with pytest.raises(b.ApbError) as e:
        b.apb_train_backward(W, W, 0.1, 0.0)
    assert e.value.code == b.APB_ERR_VALUE
    with pytest.raises(b.ApbError) as e:
        b.apb_train_forward(W, float("nan"), 0.1)
    assert e.value.code == b.APB_ERR_VALUE
