"""The rows-in-lanes forward kernel (lanes along the rows of the sparse matrix; layers of 256 rows and more with
enough residuals per row) through apb_forward, against the CPU oracle: integer part exact through the separate
entry point, every output of Y within 1e-5 relative, no floor.  Each case first checks, by the kernel name the
library reports, that it is this kernel that runs.  Shapes: rows not a multiple of 64 (padding slots), K not a
multiple of 128 or of 32 (padded matrix steps, partial last word), column groups with fewer than 16 valid columns,
one column, empty rows and rows of very different lengths (padding entries in the lists), the largest K whose code
table fits on chip, both activation widths.  Every case that runs on this kernel also runs its packed-output
form (apb_forward_requant) and compares the codes and column sums with the oracle's."""
import os

import numpy as np
import pytest
import torch

from oracle import apb_oracle as o
from oracle import capi
from paper_2306_08960_amd import synth
from requant_checks import compare_codes, unpack

pytestmark = pytest.mark.gpu
THREADS = max(1, min(16, len(os.sched_getaffinity(0))))


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2306_08960_amd import binding
    binding.load()
    return binding


def check(b, W, delta, X, bits, step, tag, expect_rows=True):
    N, K = W.shape
    M = X.shape[1]
    print(f"[case] rows kernel {tag} N={N} K={K} M={M} bits={bits}", flush=True)
    L = o.compress(W, delta)
    c = o.quantize(X, bits, step)
    F = capi.forward(L, o.pack_acts(c, bits), c, bits, step, threads=THREADS)
    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta), alpha=float(L["alpha"]))
    name = b.apb_forward_kernel_name(layer, M, bits)
    assert name.startswith("k_forward_rows") == expect_rows, name
    packed = b.apb_quantize_acts(torch.from_numpy(X).cuda(), bits, float(step))
    Y = torch.full((N, M), float("nan"), device="cuda")
    b.apb_forward(layer, packed, M, bits, float(step), Y=Y)
    Y = Y.cpu().numpy().astype(np.float64)
    ref = F["Y"].astype(np.float64)
    bad = ~(np.abs(Y - ref) <= 1e-5 * np.abs(ref))             # (a NaN left in Y counts as bad)
    assert not bad.any(), f"{int(bad.sum())} of {bad.size} outputs off; first at {np.argwhere(bad)[0]}"
    if expect_rows:
        # the same kernel ending in the next layer's quantizer (apb_forward_requant): both output widths, with and
        # without the per-row affine map, into a buffer full of ones
        r = np.random.default_rng(N + K)
        for bits_out in (2, 1):
            step_out = np.float32(np.std(ref) * 0.7 + 1e-3)
            scale = r.uniform(0.5, 1.5, N).astype(np.float32)
            shift = (r.standard_normal(N) * float(step_out)).astype(np.float32)
            for sc, sh in ((None, None), (scale, shift)):
                want = o.requant(L["alpha"], step, F["D"], F["R"], bits_out, step_out, sc, sh)
                out = b.alloc_packed(N, M, bits_out)
                out.fill_(-1)
                b.apb_forward_requant(layer, packed, M, bits, float(step), bits_out, float(step_out),
                                      None if sc is None else torch.from_numpy(sc).cuda(),
                                      None if sh is None else torch.from_numpy(sh).cuda(), packed_out=out)
                torch.cuda.synchronize()
                code, colsum = unpack(out.cpu().numpy().view(np.uint32), N, M, bits_out)
                assert np.array_equal(colsum[:M], code.sum(axis=0))
                compare_codes(code, want, L["alpha"], step, F["D"], F["R"], bits_out, step_out, sc, sh)
    layer.free()


SHAPES = [(256, 128, 16), (257, 100, 1), (300, 97, 15), (320, 1000, 17), (513, 300, 100), (640, 4100, 70),
          (1000, 257, 1000), (256, 2304, 333),
          # a little more than four tasks per compute unit: the remainder's column groups run as the finer tail
          # (2 and 3 row groups, the last one with idle waves, ragged M)
          (512, 300, 8310), (600, 200, 5590),
          # the same with one task per compute unit and a few more: one row group (whose packed-output form stores
          # plainly and takes no tail) and two
          (256, 128, 4340), (300, 97, 2200),
          # few column groups: one workgroup per compute unit already (no sharing), two waves per block of rows to
          # get there, and the doubling more that long rows take
          (4100, 500, 250), (4100, 300, 120), (4100, 4100, 250)]


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("N,K,M", SHAPES)
def test_ragged_shapes(b, N, K, M, bits):
    W, delta, X, step = synth.random_case(9000 + N + K + M + bits, N, K, M, bits, rho=0.12)
    check(b, W, delta, X, bits, step, "ragged")


def test_empty_rows_and_very_uneven_rows(b):
    g = np.random.default_rng(31)
    N, K, M = 384, 700, 90
    W = (g.standard_normal((N, K)) * 0.01).astype(np.float32)   # all inside the interval ...
    delta = np.float32(0.2)
    counts = g.integers(0, 61, size=N)                           # ... except planted residuals: 0 to 60 per row,
    counts[::7] = 0                                              # every seventh row none at all
    for n in range(N):
        cols = g.choice(K, size=counts[n], replace=False)
        W[n, cols] = (0.3 + g.random(counts[n])).astype(np.float32) * g.choice([-1.0, 1.0], size=counts[n]).astype(np.float32)
    for bits, step in ((1, 1.0), (2, 0.75)):
        X = g.standard_normal((K, M)).astype(np.float32)
        if bits == 2:
            np.maximum(X, 0, out=X)
        check(b, W, delta, X, bits, np.float32(step), "uneven rows")


def test_largest_k_whose_table_fits_and_the_fallback_beyond(b):
    g = np.random.default_rng(32)
    for K, expect in ((18432, True), (18464, False)):
        W, delta, X, step = synth.random_case(9100 + K, 256, K, 40, 2, rho=0.01)
        check(b, W, delta, X, 2, step, "largest K" if expect else "K beyond the table", expect_rows=expect)


def test_layers_outside_its_range_take_the_other_kernel(b):
    # one row carrying residuals in every column beside light rows: the lists, padded to the longest row of each
    # block of 64, would be mostly padding
    g = np.random.default_rng(33)
    W = (g.standard_normal((384, 700)) * 0.01).astype(np.float32)
    W[5] = 0.5
    W[::3, :8] = -0.4
    X = np.maximum(g.standard_normal((700, 90)), 0).astype(np.float32)
    check(b, W, np.float32(0.2), X, 2, np.float32(0.75), "one very long row", expect_rows=False)
    W, delta, X, step = synth.random_case(9200, 128, 512, 64, 2, rho=0.05)        # fewer than 4 blocks of 64 rows
    check(b, W, delta, X, 2, step, "128 rows", expect_rows=False)
    W, delta, X, step = synth.random_case(9201, 512, 512, 64, 2, rho=0.001)       # hardly any residuals
    check(b, W, delta, X, 2, step, "0.1 % residuals", expect_rows=False)


@pytest.mark.parametrize("name", ["C3_r05_b1", "C3_r50_b1", "C3_r50_b2", "C5a", "C5b"])
def test_benchmark_layers_run_on_it(b, name):
    cfg = synth.CONFIGS[name]
    W, delta, X, step = synth.make_layer(cfg)
    check(b, W, delta, X, cfg.bits, step, name)
