"""Parity of the 2/2 routine (Sec. IV "2/2": 2-bit weights x 2-bit activations) with the CPU oracle,
through the C ABI, on the same seeded inputs.  Bars: bit-exact for the packed weight planes and the
integer product D22; max relative error 1e-5 for Y, every element, no floor."""
import numpy as np
import pytest
import torch

from oracle import apb_oracle as o
from paper_2306_08960_amd import synth

pytestmark = pytest.mark.gpu

REL_TOL = 1e-5


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2306_08960_amd import binding
    binding.load()
    return binding


def check_2_2(b, W, step_w, X, step_a, rows=None, tag=""):
    """Pack, multiply and compare; `rows` restricts the oracle product to a sample of weight rows."""
    N, K = W.shape
    M = X.shape[1]
    print(f"[case 2/2] {tag} N={N} K={K} M={M} step_w={float(step_w):.4g} step_a={float(step_a):.4g}", flush=True)
    q = o.quantize_weights_2bit(W, step_w)
    c = o.quantize(X, 2, step_a)
    Wd = torch.from_numpy(W).cuda()
    Xd = torch.from_numpy(X).cuda()
    w2 = b.apb_w2_pack(Wd, float(step_w))
    planes = b.apb_w2_export(w2).cpu().numpy().view(np.uint32)
    assert np.array_equal(planes, o.pack_weight_planes(q))
    packed = b.apb_quantize_acts(Xd, 2, float(step_a))
    D = b.apb_gemm_2_2_int(w2, packed, M).cpu().numpy()
    Y = b.apb_gemm_2_2(w2, packed, M, float(step_a)).cpu().numpy()
    torch.cuda.synchronize()
    sel = np.arange(N) if rows is None else np.asarray(rows)
    ref = o.gemm_2_2(q[sel], c, step_w, step_a)
    assert np.array_equal(D[sel], ref["D"])
    err = np.abs(Y[sel].astype(np.float64) - ref["Y"].astype(np.float64))
    assert np.all(err <= REL_TOL * np.abs(ref["Y"].astype(np.float64))), float(err.max())
    w2.free()


EDGE_SHAPES = [(1, 1, 1), (1, 31, 1), (2, 32, 64), (3, 33, 65), (33, 64, 63), (31, 95, 127), (65, 257, 193),
               (100, 1000, 300), (7, 4100, 5), (130, 200, 70)]


@pytest.mark.parametrize("N,K,M", EDGE_SHAPES)
def test_edge_shapes(b, N, K, M):
    W, _, X, step = synth.random_case(2200 + N * 7 + K + M, N, K, M, 2, rho=0.05)
    check_2_2(b, W, np.float32(0.04), X, step, tag="edge")


# Shapes with 384 or more tiles of 128 x 128: the kernel whose waves share the activation operand through LDS --
# ragged N, K (one step, an odd number of words, a tail past the pipeline's ring of six) and M
SHARED_SHAPES = [(130, 200, 24593), (300, 33, 16500), (128, 64, 49100), (257, 1000, 16400), (513, 832, 9900)]


@pytest.mark.parametrize("N,K,M", SHARED_SHAPES)
def test_shapes_on_the_shared_operand_kernel(b, N, K, M):
    assert ((N + 127) // 128) * ((M + 63) // 64 * 64 + 127) // 128 >= 384
    W, _, X, step = synth.random_case(4100 + N + K + M, N, K, M, 2, rho=0.05)
    check_2_2(b, W, np.float32(0.04), X, step, tag="shared operand")
    # the same kernel computes the integer part D of a binary layer (1- and 2-bit activations)
    for bits in (1, 2):
        Wb, delta, Xb, stepb = synth.random_case(4200 + N + K + M + bits, N, K, M, bits, rho=0.02)
        c = o.quantize(Xb, bits, stepb)
        rows = np.unique(np.concatenate([[0, N - 1], np.random.default_rng(N).choice(N, 24, replace=False)]))
        want = o.int_part_unpacked(o.sign_bits(Wb)[rows], c)
        layer = b.apb_compress(torch.from_numpy(Wb).cuda(), float(delta))
        packed = b.apb_quantize_acts(torch.from_numpy(Xb).cuda(), bits, float(stepb))
        D = b.apb_forward_int(layer, packed, M, bits).cpu().numpy()
        assert np.array_equal(D[rows], want)
        layer.free()


def test_special_values_and_degenerate_steps(b):
    W = np.zeros((4, 70), dtype=np.float32)
    W[0] = [0.0, -0.0, 0.49, 0.5, 0.99, 1.0, 7.0, -1e-30, -0.5, -0.51, -1.0, -1.01, -9.0, np.inf] * 5
    W[1] = np.float32(1e-40)
    W[2] = -np.float32(1e-40)
    W[3] = np.random.default_rng(3).standard_normal(70).astype(np.float32)
    X = np.maximum(np.random.default_rng(4).standard_normal((70, 67)), 0).astype(np.float32) * 2
    check_2_2(b, W, np.float32(0.5), X, np.float32(0.75), tag="boundaries")
    check_2_2(b, W, np.float32(1e6), X, np.float32(0.75), tag="every weight in the two middle cells")
    check_2_2(b, W, np.float32(1e-6), X, np.float32(1e-3), tag="every weight and activation saturated")


@pytest.mark.parametrize("name", ["C2", "C3_r05_b2", "C4", "C5a", "C5b"])
def test_benchmark_shapes(b, name):
    """Every benchmark shape at full size, every row and column against the oracle."""
    cfg = synth.CONFIGS[name]
    W, _, X, step = synth.make_layer(cfg)
    step_w = np.float32(np.std(W))
    check_2_2(b, W, step_w, X, step, tag=name)


def test_k_beyond_the_exact_range_is_refused(b):
    """9*K >= 2^24: the float accumulators of the matrix instruction could no longer hold every partial sum."""
    K = (1 << 24) // 9 + 32
    w2 = b.apb_w2_pack(torch.zeros((1, K), device="cuda"), 1.0)
    packed = b.apb_quantize_acts(torch.zeros((K, 1), device="cuda"), 2, 1.0)
    with pytest.raises(b.ApbError) as e:
        b.apb_gemm_2_2_int(w2, packed, 1)
    assert e.value.code == b.APB_ERR_SHAPE
    w2.free()
