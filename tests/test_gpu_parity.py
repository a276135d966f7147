"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element, on the
same seeded inputs.  Bars: bit-exact for sign words, CSR, packed planes, column sums and the
integer part D; max relative error 1e-5 for the float output Y, every element, no floor
(|y - y_ref| <= 1e-5 * |y_ref|)."""
import os

import numpy as np
import pytest
import torch

from oracle import apb_oracle as o
from oracle import capi
from paper_2306_08960_amd import synth

pytestmark = pytest.mark.gpu

REL_TOL = 1e-5
THREADS = max(1, min(16, len(os.sched_getaffinity(0))))


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2306_08960_amd import binding
    binding.load()
    return binding


def _bits_view(t):
    return t.detach().cpu().numpy()


def check_layer(b, W, delta, X, bits, step, alpha=None, tag=""):
    """Run compress / quantize / forward on both sides and compare everything."""
    print(f"[case] {tag} N={W.shape[0]} K={W.shape[1]} M={X.shape[1]} bits={bits} delta={float(delta):.6g}", flush=True)
    N, K = W.shape
    M = X.shape[1]
    L = o.compress(W, delta, alpha)
    c = o.quantize(X, bits, step)
    packed_ref = o.pack_acts(c, bits)
    F = capi.forward(L, packed_ref, c, bits, step, threads=THREADS)

    Wd = torch.from_numpy(W).cuda()
    Xd = torch.from_numpy(X).cuda()

    # a1: compress with the oracle's alpha -> canonical representation, bit for bit
    layer = b.apb_compress(Wd, float(delta), alpha=float(L["alpha"]))
    ex = b.apb_layer_export(layer)
    nnz = int(L["row_ptr"][-1])
    assert ex["N"] == N and ex["K"] == K and ex["nnz"] == nnz
    assert ex["mem_bits"] == o.mem_bits(N, K, nnz)
    assert np.array_equal(_bits_view(ex["sign_words"]).view(np.uint32), L["sign_words"])
    assert np.array_equal(_bits_view(ex["row_ptr"]), L["row_ptr"])
    assert np.array_equal(_bits_view(ex["col_idx"]), L["col_idx"])
    assert np.array_equal(_bits_view(ex["val"]).view(np.uint32), L["val"].view(np.uint32))
    assert np.array_equal(_bits_view(ex["rowsum"]), L["rowsum"])
    if alpha is None:
        # the library's own default scale: same mean, float64 sum in another order
        lay2 = b.apb_compress(Wd, float(delta))
        a2 = lay2.info()["alpha"]
        assert abs(a2 - float(L["alpha"])) <= 1e-6 * abs(float(L["alpha"]))
        lay2.free()

    # a2: quantize + pack, bit for bit (planes and column sums)
    packed = b.apb_quantize_acts(Xd, bits, float(step))
    got = _bits_view(packed).view(np.uint32)
    assert got.size == packed_ref.size
    assert np.array_equal(got, packed_ref)

    # a3: integer part, exact
    D = _bits_view(b.apb_forward_int(layer, packed, M, bits))
    assert np.array_equal(D, F["D"]), "matrix-core integer part"
    D2 = _bits_view(b.apb_forward_int_popcount(layer, packed, M, bits))
    assert np.array_equal(D2, F["D"]), "popcount integer part"

    # a4 + a5: float output, product path (matrix cores + sparse/epilogue) and popcount path
    ref = F["Y"]
    for name, fn in (("apb_forward", b.apb_forward), ("apb_forward_popcount", b.apb_forward_popcount)):
        Y = _bits_view(fn(layer, packed, M, bits, float(step)))
        err = np.abs(Y.astype(np.float64) - ref.astype(np.float64))
        bound = REL_TOL * np.abs(ref.astype(np.float64))
        bad = err > bound
        assert not bad.any(), (f"{name}: {int(bad.sum())} of {bad.size} outputs off by more than {REL_TOL} "
                               f"relative; worst {float((err / np.maximum(np.abs(ref), 1e-300)).max()):.3g}")
        ulps = err / np.spacing(np.maximum(np.abs(ref), np.float32(1e-30)))
    print(f"        nnz={nnz} max |D|={int(np.abs(D).max())} max ulp diff of Y={float(ulps.max()):.2f}", flush=True)
    layer.free()
    return Y


# ----------------------------------------------------------------------------- small shapes and edges
EDGE_SHAPES = [(1, 1, 1), (1, 31, 1), (2, 32, 64), (3, 33, 65), (33, 64, 63), (31, 95, 127), (32, 96, 128),
               (65, 257, 193), (100, 1000, 300), (7, 4100, 5), (130, 200, 70)]


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("N,K,M", EDGE_SHAPES)
def test_edge_shapes(b, N, K, M, bits):
    W, delta, X, step = synth.random_case(N * 7 + K + M + bits, N, K, M, bits, rho=0.05)
    check_layer(b, W, delta, X, bits, step, tag="edge")


@pytest.mark.parametrize("bits", [1, 2])
def test_degenerate_intervals(b, bits):
    W, _, X, step = synth.random_case(77 + bits, 40, 70, 90, bits)
    check_layer(b, W, np.float32(np.inf), X, bits, step, alpha=np.float32(0.04), tag="no residuals")
    check_layer(b, W, np.float32(-1.0), X, bits, step, tag="every weight a residual (alpha=0)")
    check_layer(b, W, np.float32(-1.0), X, bits, step, alpha=np.float32(0.04), tag="every weight a residual")
    check_layer(b, W, np.float32(0.0), X, bits, step, tag="delta=0")


def test_signed_zeros_denormals_ties_and_boundaries(b):
    W = np.zeros((5, 70), dtype=np.float32)
    W[0] = 0.5                                  # |w| == delta: binarized
    W[1] = -0.5
    W[2, ::2] = -0.0                            # sign(-0.0) is +
    W[2, 1::2] = np.nextafter(np.float32(0.5), np.float32(1.0))
    W[3] = np.float32(-1e-40)                   # negative denormal: sign -
    W[4, 3] = 9.0
    X = np.zeros((70, 67), dtype=np.float32)
    X[:, 0] = -0.0
    X[:, 1] = np.float32(1e-40)
    X[:, 2] = np.float32(-1e-40)
    X[:, 3] = 0.375                             # x/s = 0.5 -> 0 (tie to even) for s = 0.75
    X[:, 4] = 1.125                             # 1.5 -> 2
    X[:, 5] = 1.875                             # 2.5 -> 2
    X[:, 6] = 2.625                             # 3.5 -> 4 -> clamp 3
    X[:, 7] = -3.0
    X[:, 8] = 1e30
    X[:, 66] = np.nan                           # quantizes to code 0 / sign -
    X[:, 9:66] = np.random.default_rng(5).standard_normal((70, 57)).astype(np.float32)
    for bits, step in ((1, 1.0), (2, 0.75), (2, 0.1)):
        check_layer(b, W, np.float32(0.5), X, bits, np.float32(step), alpha=np.float32(0.25), tag="special values")


def test_skewed_rows_small(b):
    cfg = synth.small_variant(synth.CONFIGS["C4"], M=700)
    W, delta, X, step = synth.make_layer(cfg)
    check_layer(b, W, delta, X, cfg.bits, step, tag="C4 rows, M=700")


# ----------------------------------------------------------------------------- the benchmark layers, full size
FULL = ["C1", "C2", "C3_r05_b1", "C3_r20_b1", "C3_r50_b1", "C3_r05_b2", "C3_r20_b2", "C3_r50_b2", "C4", "C5a", "C5b"]


@pytest.mark.parametrize("name", FULL)
def test_benchmark_layers_full_size(b, name):
    cfg = synth.CONFIGS[name]
    W, delta, X, step = synth.make_layer(cfg)
    check_layer(b, W, delta, X, cfg.bits, step, tag=name)
    torch.cuda.empty_cache()


# ----------------------------------------------------------------------------- behaviour of the boundary
def test_errors_and_reuse(b):
    W, delta, X, step = synth.random_case(3, 8, 40, 10, 2)
    Wd, Xd = torch.from_numpy(W).cuda(), torch.from_numpy(X).cuda()
    layer = b.apb_compress(Wd, float(delta))
    packed = b.apb_quantize_acts(Xd, 2, float(step))
    lib = b.load()
    Y = torch.empty((8, 10), dtype=torch.float32, device="cuda")
    assert lib.apb_forward(layer.handle, packed.data_ptr(), 10, 3, 0.75, Y.data_ptr(), None) == b.APB_ERR_BITS
    assert lib.apb_forward(layer.handle, packed.data_ptr(), 0, 2, 0.75, Y.data_ptr(), None) == b.APB_ERR_SHAPE
    assert lib.apb_forward(layer.handle, packed.data_ptr(), 10, 2, float("nan"), Y.data_ptr(), None) == b.APB_ERR_VALUE
    assert lib.apb_forward(layer.handle, packed.data_ptr(), 10, 2, 0.75, None, None) == b.APB_ERR_NULL
    # same layer, same buffers, twice and on a side stream: identical bits
    y1 = b.apb_forward(layer, packed, 10, 2, float(step)).clone()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        p2 = b.apb_quantize_acts(Xd, 2, float(step))
        y2 = b.apb_forward(layer, p2, 10, 2, float(step))
    s.synchronize()
    assert torch.equal(y1, y2) and torch.equal(packed, p2)
    layer.free()
    layer.free()


def test_step_can_be_captured_in_a_graph_and_replayed(b):
    """quantize + forward allocate nothing and record no memset: a captured graph of the step must
    reproduce the eager result on every replay, with eager work and synchronizations in between."""
    W, delta, X, step = synth.random_case(4242, 70, 300, 5000, 2, rho=0.03)
    Wd = torch.from_numpy(W).cuda()
    Xd = torch.from_numpy(X).cuda()
    layer = b.apb_compress(Wd, float(delta))
    packed = b.alloc_packed(300, 5000, 2)
    Y = torch.empty((70, 5000), dtype=torch.float32, device="cuda")

    def one_step():
        b.apb_quantize_acts(Xd, 2, float(step), packed=packed)
        b.apb_forward(layer, packed, 5000, 2, float(step), Y=Y)

    one_step()
    torch.cuda.synchronize()
    y_ref = Y.clone()
    p_ref = packed.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_step()                                       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        one_step()
    for _ in range(3):
        Y.zero_()
        packed.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(packed, p_ref)
        assert torch.equal(Y, y_ref)
        one_step()                                       # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(Y, y_ref)
    layer.free()
