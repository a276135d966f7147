"""apb_forward_requant (one layer's output quantized and packed for the next layer, no float round
trip) against the CPU oracle, through the C ABI.

Bars.  The packed output is integer work decided by a float: both sides take the decision on the
float32 Z with the same float32 quantizer, so the codes must be equal wherever Z is not within the
float tolerance (1e-5, relative to the magnitude of the two parts that were added) of a decision
boundary; such near-ties must be rare (< 0.1 % of the elements) and are the only differences
allowed.  Everything else is exact: the column sums equal the sums of the codes actually written,
padding columns and the bits of rows >= N are zero, and the next layer computed on the GPU from the
GPU's packed output equals the oracle's next layer computed from those same codes to the usual
1e-5."""
import os

import numpy as np
import pytest
import torch

from oracle import apb_oracle as o
from oracle import capi
from paper_2306_08960_amd import synth
from requant_checks import REL_TOL, compare_codes, unpack

pytestmark = pytest.mark.gpu

THREADS = max(1, min(16, len(os.sched_getaffinity(0))))


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2306_08960_amd import binding
    binding.load()
    return binding


def check_requant(b, W, delta, X, bits, step, bits_out, step_out, affine, tag="", W2=None, delta2=None):
    N, K = W.shape
    M = X.shape[1]
    print(f"[case] {tag} N={N} K={K} M={M} bits={bits}->{bits_out} affine={affine}", flush=True)
    L = o.compress(W, delta)
    c = o.quantize(X, bits, step)
    F = capi.forward(L, o.pack_acts(c, bits), c, bits, step, threads=THREADS)
    scale = shift = None
    if affine:
        r = np.random.default_rng(N * 7 + K)
        scale = r.uniform(0.5, 1.5, N).astype(np.float32) * np.where(r.random(N) < 0.1, -1, 1).astype(np.float32)
        shift = (r.standard_normal(N) * float(step_out)).astype(np.float32)
    ref = o.requant(L["alpha"], step, F["D"], F["R"], bits_out, step_out, scale, shift)

    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta), alpha=float(L["alpha"]))
    packed = b.apb_quantize_acts(torch.from_numpy(X).cuda(), bits, float(step))
    out = b.alloc_packed(N, M, bits_out)
    out.fill_(-1)                                            # the call must overwrite everything
    b.apb_forward_requant(layer, packed, M, bits, float(step), bits_out, float(step_out),
                          None if scale is None else torch.from_numpy(scale).cuda(),
                          None if shift is None else torch.from_numpy(shift).cuda(), packed_out=out)
    torch.cuda.synchronize()
    got_words = out.cpu().numpy().view(np.uint32)
    code, colsum = unpack(got_words, N, M, bits_out)
    assert np.array_equal(colsum[:M], code.sum(axis=0)), "column sums of the codes written"

    n_diff = compare_codes(code, ref, L["alpha"], step, F["D"], F["R"], bits_out, step_out, scale, shift)
    if n_diff == 0:
        assert np.array_equal(got_words, ref["packed"])

    if W2 is not None:
        # the next layer, on the GPU from the GPU's packed output, against the oracle on the same codes
        L2 = o.compress(W2, delta2)
        c2 = (2 * code - 1).astype(np.int8) if bits_out == 1 else code.astype(np.int8)
        F2 = capi.forward(L2, o.pack_acts(c2, bits_out), c2, bits_out, step_out, threads=THREADS)
        layer2 = b.apb_compress(torch.from_numpy(W2).cuda(), float(delta2), alpha=float(L2["alpha"]))
        Y2 = b.apb_forward(layer2, out, M, bits_out, float(step_out)).cpu().numpy()
        err = np.abs(Y2.astype(np.float64) - F2["Y"].astype(np.float64))
        assert np.all(err <= REL_TOL * np.abs(F2["Y"].astype(np.float64)))
        layer2.free()
    layer.free()
    return n_diff


EDGE = [(1, 1, 1), (5, 33, 3), (16, 64, 64), (17, 100, 65), (33, 257, 130), (64, 300, 70), (70, 520, 129),
        (130, 200, 70), (257, 96, 40)]


@pytest.mark.parametrize("bits,bits_out", [(2, 2), (1, 1), (2, 1), (1, 2)])
@pytest.mark.parametrize("N,K,M", EDGE)
def test_edge_shapes(b, N, K, M, bits, bits_out):
    W, delta, X, step = synth.random_case(N * 31 + K + M, N, K, M, bits, rho=0.05)
    step_out = np.float32(0.03 * np.sqrt(K))                 # spreads the outputs over all four levels
    W2, delta2, _, _ = synth.random_case(N + 5, 9, N, 1, 2, rho=0.1)
    check_requant(b, W, delta, X, bits, step, bits_out, step_out, affine=(N % 2 == 1), tag="edge", W2=W2, delta2=delta2)


def test_special_values(b):
    """All-outlier and no-outlier layers, zero activations (Y = 0 exactly: code 0, sign +)."""
    W, _, X, step = synth.random_case(5, 40, 130, 90, 2)
    check_requant(b, W, np.float32(-1.0), X, 2, step, 2, np.float32(0.02), affine=False, tag="all outliers")
    check_requant(b, W, np.float32(np.inf), X, 2, step, 2, np.float32(0.02), affine=True, tag="no outliers")
    check_requant(b, W, np.float32(0.1), np.zeros_like(X), 2, step, 1, np.float32(1.0), affine=False, tag="zero acts")
    check_requant(b, W, np.float32(0.1), np.zeros_like(X), 2, step, 2, np.float32(1.0), affine=False, tag="zero acts")


@pytest.mark.parametrize("name,N,K,M", [("C2", None, None, 1500), ("C3_r20_b2", None, None, 700), ("C3_r50_b1", None, None, 300), ("C4", None, None, 900),
                                        ("C5a", 520, 1100, 256), ("C5b", 512, 1200, 300)])
def test_config_shapes_reduced(b, name, N, K, M):
    cfg = synth.small_variant(synth.CONFIGS[name], N=N, K=K, M=M)
    W, delta, X, step = synth.make_layer(cfg)
    W2, delta2, _, _ = synth.random_case(11, 40, W.shape[0], 1, 2, rho=0.03)
    check_requant(b, W, delta, X, cfg.bits, step, 2, np.float32(0.03 * np.sqrt(W.shape[1])), affine=True, tag=name, W2=W2,
                  delta2=delta2)


def test_fc_chain_at_full_size_sampled_columns(b):
    """C5a at its full size in the launch configuration the benchmark times: the layer applied twice
    in a row (N = K); a sample of output columns is checked against the oracle, the rest through
    the column-sum identity."""
    cfg = synth.CONFIGS["C5a"]
    W, delta, X, step = synth.make_layer(cfg)
    N, K = W.shape
    M = X.shape[1]
    L = o.compress(W, delta)
    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta), alpha=float(L["alpha"]))
    packed = b.apb_quantize_acts(torch.from_numpy(X).cuda(), cfg.bits, float(step))
    step_out = np.float32(0.6)
    hop = b.apb_forward_requant(layer, packed, M, cfg.bits, float(step), 2, float(step_out))
    hop2 = b.apb_forward_requant(layer, hop, M, 2, float(step_out), 2, float(step_out))
    torch.cuda.synchronize()
    code1, colsum1 = unpack(hop.cpu().numpy().view(np.uint32), N, M, 2)
    code2, colsum2 = unpack(hop2.cpu().numpy().view(np.uint32), N, M, 2)
    assert np.array_equal(colsum1[:M], code1.sum(axis=0)) and np.array_equal(colsum2[:M], code2.sum(axis=0))
    cols = np.random.default_rng(1).choice(M, 24, replace=False)
    c = o.quantize(X[:, cols], cfg.bits, step)
    F = capi.forward(L, o.pack_acts(c, cfg.bits), c, cfg.bits, step, threads=THREADS)
    ref1 = o.requant(L["alpha"], step, F["D"], F["R"], 2, step_out)
    # equal codes, except within the float tolerance of a decision boundary, then off by one level and rare
    compare_codes(code1[:, cols], ref1, L["alpha"], step, F["D"], F["R"], 2, step_out, None, None)
    c_mid = code1[:, cols].astype(np.int8)                   # second hop from the GPU's own codes
    F2 = capi.forward(L, o.pack_acts(c_mid, 2), c_mid, 2, step_out, threads=THREADS)
    ref2 = o.requant(L["alpha"], step_out, F2["D"], F2["R"], 2, step_out)
    compare_codes(code2[:, cols], ref2, L["alpha"], step_out, F2["D"], F2["R"], 2, step_out, None, None)
    layer.free()


def test_argument_errors(b):
    W, delta, X, step = synth.random_case(1, 20, 64, 10, 2)
    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta))
    packed = b.apb_quantize_acts(torch.from_numpy(X).cuda(), 2, float(step))
    out = b.alloc_packed(20, 10, 2)
    lib = b.load()
    ptr = lambda t: t.data_ptr()
    f = torch.ones(20, device="cuda")
    call = lambda *a: lib.apb_forward_requant(layer.handle, *a)
    assert call(ptr(packed), 10, 2, 0.75, None, None, 3, 1.0, ptr(out), None) == b.APB_ERR_BITS
    assert call(ptr(packed), 10, 3, 0.75, None, None, 2, 1.0, ptr(out), None) == b.APB_ERR_BITS
    assert call(ptr(packed), 10, 2, 0.75, None, None, 2, 0.0, ptr(out), None) == b.APB_ERR_VALUE
    assert call(ptr(packed), 10, 2, float("nan"), None, None, 2, 1.0, ptr(out), None) == b.APB_ERR_VALUE
    assert call(ptr(packed), 10, 2, 0.75, ptr(f), None, 2, 1.0, ptr(out), None) == b.APB_ERR_NULL
    assert call(ptr(packed), 10, 2, 0.75, None, None, 2, 1.0, None, None) == b.APB_ERR_NULL
    assert call(ptr(packed), 0, 2, 0.75, None, None, 2, 1.0, ptr(out), None) == b.APB_ERR_SHAPE
    with pytest.raises(ValueError):
        b.apb_forward_requant(layer, packed, 10, 2, 0.75, 2, 1.0, scale=f)
    with pytest.raises(ValueError):
        b.apb_forward_requant(layer, packed, 10, 2, 0.75, 2, 1.0, packed_out=torch.empty(4, dtype=torch.int32, device="cuda"))
    layer.free()
