"""apb_quantize_forward_static (the entry point that allocates nothing: the packed activations pass
through the library's static device array) through the C ABI: Y must equal, bit for bit, what
apb_quantize_forward writes for the same inputs -- the same kernels run, only the workspace differs --
on two calls in a row that share the array, the second on a smaller input, so that contents left by
the first call would show.  The shapes have more than 128 rows: the two-kernel route, the one that
uses the array."""
import pytest
import torch

from paper_2306_08960_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def b():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2306_08960_amd import binding
    binding.load()
    return binding


def _both(b, seed, N, K, M, bits):
    print(f"[case] quantize_forward_static N={N} K={K} M={M} bits={bits}", flush=True)
    W, delta, X, step = synth.random_case(seed, N, K, M, bits, rho=0.04)
    Xd = torch.from_numpy(X).cuda()
    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta))
    assert not b.apb_quantize_forward_is_one_kernel(layer, M, bits)
    Y_ref = b.apb_quantize_forward(layer, Xd, bits, float(step))
    Y = torch.full((N, M), float("nan"), device="cuda")
    b.apb_quantize_forward_static(layer, Xd, bits, float(step), Y)
    torch.cuda.synchronize()
    same = torch.equal(Y, Y_ref)
    layer.free()
    return same


def test_two_calls_in_a_row_second_one_smaller(b):
    # 2-bit, many columns (column sums stored plainly), then 1-bit with few columns (K split across
    # workgroups: column sums cleared by a fill kernel and added atomically) inside the area the first
    # call wrote, then a ragged 2-bit case again
    assert _both(b, 901, 300, 700, 9000, 2)
    assert _both(b, 902, 130, 260, 700, 1)
    assert _both(b, 903, 257, 333, 1234, 2)


def test_sizes_beyond_the_array_are_refused_and_nothing_runs(b):
    N, K, bits = 130, 64, 2
    W, delta, _, step = synth.random_case(904, N, K, 8, bits)
    layer = b.apb_compress(torch.from_numpy(W).cuda(), float(delta))
    M = b.APB_STATIC_SCRATCH_BYTES // (4 * (bits * 2 + 1)) + 64      # one strip of columns too many
    assert b.apb_acts_bytes(K, M, bits) > b.APB_STATIC_SCRATCH_BYTES
    X = torch.zeros((K, M), device="cuda")
    Y = torch.full((N, M), 7.0, device="cuda")
    with pytest.raises(b.ApbError) as e:
        b.apb_quantize_forward_static(layer, X, bits, float(step), Y)
    assert e.value.code == b.APB_ERR_SCRATCH
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all())
    # the largest M that fits is accepted and matches the workspace route
    M = (b.APB_STATIC_SCRATCH_BYTES // (4 * (bits * 2 + 1))) // 64 * 64
    assert b.apb_acts_bytes(K, M, bits) <= b.APB_STATIC_SCRATCH_BYTES
    X = torch.rand((K, M), device="cuda") * 3
    Y = torch.empty((N, M), device="cuda")
    b.apb_quantize_forward_static(layer, X, bits, float(step), Y)
    assert torch.equal(Y, b.apb_quantize_forward(layer, X, bits, float(step)))
    layer.free()
