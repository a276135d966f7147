"""apb_quantize_forward (quantize + forward as one call; one kernel for layers of at most 128 rows)
through the C ABI: Y must equal, bit for bit, apb_quantize_acts followed by apb_forward -- whose parity
with the oracle the other tests establish -- and, directly, the oracle within 1e-5 relative."""
import os

import numpy as np
import pytest
import torch

from oracle import apb_oracle as o
from oracle import capi
from paper_2306_08960_amd import synth

pytestmark = pytest.mark.gpu
THREADS = max(1, min(16, len(os.sched_getaffinity(0))))


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2306_08960_amd import binding
    binding.load()
    return binding


# N <= 128 with 2-, 4- and 8-wave workgroups, ragged K and M, K below one word, a K too long for the
# on-chip strip (falls back to two kernels), N > 128 (falls back), few columns with 8 waves (falls back)
SHAPES = [(1, 1, 1), (5, 33, 3), (16, 64, 64), (30, 100, 65), (33, 257, 130), (64, 300, 700), (64, 576, 5000),
          (70, 520, 129), (128, 1152, 30000), (100, 200, 24001), (128, 9000, 300), (130, 200, 70), (40, 7000, 100),
          # more than 512 strips of columns (several rounds of workgroups on the chip): an odd number of strips,
          # ragged M and K, 8-, 4- and 2-wave row groups, and values of K whose strip takes 15 to 39 KB of LDS
          (128, 1152, 32900), (64, 300, 40000), (20, 97, 33333), (128, 1500, 32800), (64, 1800, 32770),
          (128, 2400, 32800)]


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("N,K,M", SHAPES)
def test_equals_the_two_calls_bit_for_bit(b, N, K, M, bits):
    print(f"[case] quantize_forward N={N} K={K} M={M} bits={bits}", flush=True)
    W, delta, X, step = synth.random_case(N + K + M, N, K, M, bits, rho=0.04)
    Xd = torch.from_numpy(X).cuda()
    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta))
    packed = b.apb_quantize_acts(Xd, bits, float(step))
    Y2 = b.apb_forward(layer, packed, M, bits, float(step))
    scratch = b.alloc_packed(K, M, bits)
    Y1 = torch.full((N, M), float("nan"), device="cuda")
    b.apb_quantize_forward(layer, Xd, bits, float(step), packed=scratch, Y=Y1)
    assert torch.equal(Y1, Y2)
    layer.free()


@pytest.mark.parametrize("bits", [1, 2])
def test_against_the_oracle(b, bits):
    W, delta, X, step = synth.random_case(4321, 90, 300, 24500, bits, rho=0.03)
    X[5, 7] = np.nan                                          # quantizes to code 0 / sign -
    L = o.compress(W, delta)
    c = o.quantize(X, bits, step)
    F = capi.forward(L, o.pack_acts(c, bits), c, bits, step, threads=THREADS)
    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta), alpha=float(L["alpha"]))
    Y = b.apb_quantize_forward(layer, torch.from_numpy(X).cuda(), bits, float(step)).cpu().numpy()
    ref = F["Y"].astype(np.float64)
    assert np.all(np.abs(Y.astype(np.float64) - ref) <= 1e-5 * np.abs(ref))
    layer.free()


@pytest.mark.parametrize("name", ["C1", "C2", "C4", "C5b"])
def test_benchmark_layers_at_full_size(b, name):
    """The step as the benchmark launches it: bit-equal to the two calls, and every output within 1e-5 relative of
    the oracle's directly."""
    cfg = synth.CONFIGS[name]
    W, delta, X, step = synth.make_layer(cfg)
    L = o.compress(W, delta)
    c = o.quantize(X, cfg.bits, step)
    F = capi.forward(L, o.pack_acts(c, cfg.bits), c, cfg.bits, step, threads=THREADS)
    Xd = torch.from_numpy(X).cuda()
    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta), alpha=float(L["alpha"]))
    packed = b.apb_quantize_acts(Xd, cfg.bits, float(step))
    Y2 = b.apb_forward(layer, packed, cfg.M, cfg.bits, float(step))
    Y1 = b.apb_quantize_forward(layer, Xd, cfg.bits, float(step), packed=packed)
    assert torch.equal(Y1, Y2)
    ref = F["Y"].astype(np.float64)
    assert np.all(np.abs(Y1.cpu().numpy().astype(np.float64) - ref) <= 1e-5 * np.abs(ref))
    layer.free()
