"""apb_forward_conv3x3 / apb_forward_conv3x3_requant (3x3 convolution over a packed feature map through
an implicit im2col) against the CPU oracle, through the C ABI.

The oracle builds the im2col matrix of the quantized map explicitly (oracle.im2col_codes, pinned against
scipy's cross-correlation) and runs its ordinary forward on it.  Bars as everywhere: Y within 1e-5
relative, element by element; packed outputs as in test_gpu_requant.  At sizes the oracle cannot reach,
the implicit route must reproduce, bit for bit, the library's own explicit route (quantize an explicitly
built float im2col matrix, then apb_forward), whose parity is established by the other tests."""
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


def make_case(seed, N, C, B, H, W, bits, rho=0.03):
    """Weights [N, 9*C] and delta as in the benchmark layers; a float feature map [C, B*H*W]."""
    Wt, delta, _, step = synth.random_case(seed, N, 9 * C, 1, bits, rho=rho)
    r = np.random.default_rng(seed + 99)
    Xmap = r.standard_normal((C, B * H * W)).astype(np.float32)
    if bits == 2:
        Xmap = np.maximum(Xmap, 0)
    return Wt, delta, Xmap, step


def torch_im2col(Xmap_d, C, B, H, W, pad_value):
    """Explicit float im2col [9*C, B*H*W] on the GPU (plain torch indexing; test-side only)."""
    x = torch.full((C, B, H + 2, W + 2), pad_value, dtype=torch.float32, device=Xmap_d.device)
    x[:, :, 1:H + 1, 1:W + 1] = Xmap_d.view(C, B, H, W)
    return torch.cat([x[:, :, ky:ky + H, kx:kx + W].reshape(C, B * H * W) for ky in range(3) for kx in range(3)], dim=0)


SHAPES = [  # N, C, B, H, W
    (20, 64, 2, 5, 7), (64, 64, 3, 8, 8), (130, 128, 1, 9, 13), (256, 64, 5, 8, 8), (40, 64, 1, 1, 1),
    (33, 64, 1, 1, 70), (17, 64, 2, 66, 1), (512, 192, 1, 7, 7), (64, 64, 1, 32, 32),
]


@pytest.mark.parametrize("bits", [2, 1])
@pytest.mark.parametrize("N,C,B,H,W", SHAPES)
def test_conv_matches_oracle(b, N, C, B, H, W, bits):
    print(f"[case] conv N={N} C={C} B={B} H={H} W={W} bits={bits}", flush=True)
    Wt, delta, Xmap, step = make_case(N + C + H * W, N, C, B, H, W, bits)
    P = B * H * W
    L = o.compress(Wt, delta)
    c_map = o.quantize(Xmap, bits, step)
    patches = o.im2col_codes(c_map, B, H, W, bits)
    F = capi.forward(L, o.pack_acts(patches, bits), patches, bits, step, threads=THREADS)

    layer = b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta), alpha=float(L["alpha"]))
    fmap = b.apb_quantize_acts(torch.from_numpy(Xmap).cuda(), bits, float(step))
    assert np.array_equal(fmap.cpu().numpy().view(np.uint32), o.pack_acts(c_map, bits))
    Y = b.apb_forward_conv3x3(layer, fmap, B, H, W, bits, float(step)).cpu().numpy()
    ref = F["Y"].astype(np.float64)
    assert np.all(np.abs(Y.astype(np.float64) - ref) <= REL_TOL * np.abs(ref))

    # packed output map, then a second 3x3 layer on it (only where N can be a channel count)
    step_out = np.float32(0.03 * np.sqrt(9 * C))
    r = np.random.default_rng(N)
    scale = r.uniform(0.5, 1.5, N).astype(np.float32)
    shift = (r.standard_normal(N) * float(step_out)).astype(np.float32)
    for sc, sh in ((None, None), (scale, shift)):
        want = o.requant(L["alpha"], step, F["D"], F["R"], 2, step_out, sc, sh)
        out = b.alloc_packed(N, P, 2)
        out.fill_(-1)
        b.apb_forward_conv3x3_requant(layer, fmap, B, H, W, bits, float(step), 2, float(step_out),
                                      None if sc is None else torch.from_numpy(sc).cuda(),
                                      None if sh is None else torch.from_numpy(sh).cuda(), fmap_out=out)
        torch.cuda.synchronize()
        code, pixsum = unpack(out.cpu().numpy().view(np.uint32), N, P, 2)
        assert np.array_equal(pixsum[:P], code.sum(axis=0))
        compare_codes(code, want, L["alpha"], step, F["D"], F["R"], 2, step_out, sc, sh)
    if N % 64 == 0:
        W2, delta2, _, _ = synth.random_case(N + 1, 24, 9 * N, 1, 2, rho=0.02)
        L2 = o.compress(W2, delta2)
        c2 = code.astype(np.int8)
        patches2 = o.im2col_codes(c2, B, H, W, 2)
        F2 = capi.forward(L2, o.pack_acts(patches2, 2), patches2, 2, step_out, threads=THREADS)
        layer2 = b.apb_compress(torch.from_numpy(W2).cuda(), float(delta2), alpha=float(L2["alpha"]))
        Y2 = b.apb_forward_conv3x3(layer2, out, B, H, W, 2, float(step_out)).cpu().numpy()
        ref2 = F2["Y"].astype(np.float64)
        assert np.all(np.abs(Y2.astype(np.float64) - ref2) <= REL_TOL * np.abs(ref2))
        layer2.free()
    layer.free()


def test_shape_errors(b):
    Wt, delta, _, _ = synth.random_case(3, 8, 9 * 32, 1, 2)              # C = 32: not a multiple of 64
    layer = b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta))
    fmap = b.alloc_packed(32, 16, 2)
    with pytest.raises(b.ApbError) as e:
        b.apb_forward_conv3x3(layer, fmap, 1, 4, 4, 2, 0.75)
    assert e.value.code == b.APB_ERR_SHAPE
    layer.free()


@pytest.mark.parametrize("name,B,H,W", [("C2", 128, 32, 32), ("C4", 64, 28, 28), ("C3_r20_b2", 128, 8, 8),
                                        ("C3_r50_b1", 128, 8, 8), ("C5b", 256, 7, 7)])
def test_full_size_conv_layers_equal_the_explicit_route(b, name, B, H, W):
    """The benchmark's conv layers at full size, in the launch configuration the benchmark times: the
    implicit route on the packed map against apb_quantize_acts on the explicit float im2col matrix +
    apb_forward (bit for bit), and sampled columns against the oracle."""
    cfg = synth.CONFIGS[name]
    Wt, delta = synth.make_weights(cfg)
    N, K = Wt.shape
    C, P, bits, step = K // 9, B * H * W, cfg.bits, np.float32(cfg.step)
    assert P == cfg.M and C % 64 == 0
    Xmap = np.random.default_rng(5).standard_normal((C, P)).astype(np.float32)
    if bits == 2:
        Xmap = np.maximum(Xmap, 0)
    Xd = torch.from_numpy(Xmap).cuda()
    layer = b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta))
    fmap = b.apb_quantize_acts(Xd, bits, float(step))
    Y = b.apb_forward_conv3x3(layer, fmap, B, H, W, bits, float(step))
    explicit = torch_im2col(Xd, C, B, H, W, 0.0 if bits == 2 else -1.0)
    packed = b.apb_quantize_acts(explicit, bits, float(step))
    del explicit
    Y_explicit = b.apb_forward(layer, packed, P, bits, float(step))
    assert torch.equal(Y, Y_explicit)
    out = b.apb_forward_conv3x3_requant(layer, fmap, B, H, W, bits, float(step), 2, 1.0)
    out_explicit = b.apb_forward_requant(layer, packed, P, bits, float(step), 2, 1.0)
    assert torch.equal(out, out_explicit)
    # sampled pixels against the oracle (image corners and edges included)
    L = o.compress(Wt, delta, alpha=np.float32(layer.info()["alpha"]))
    pix = np.unique(np.concatenate([[0, W - 1, (H - 1) * W, H * W - 1, P - 1, P - W],
                                    np.random.default_rng(7).choice(P, 40, replace=False)]))
    c_map = o.quantize(Xmap, bits, step)
    pad = 0 if bits == 2 else -1
    cm = np.full((C, B, H + 2, W + 2), pad, dtype=np.int8)
    cm[:, :, 1:H + 1, 1:W + 1] = c_map.reshape(C, B, H, W)
    bb, yy, xx = pix // (H * W), (pix // W) % H, pix % W
    patches = np.concatenate([cm[:, bb, yy + ky, xx + kx] for ky in range(3) for kx in range(3)], axis=0)
    F = capi.forward(L, o.pack_acts(patches, bits), patches, bits, step, threads=THREADS)
    got = Y[:, torch.from_numpy(pix).cuda()].cpu().numpy().astype(np.float64)
    ref = F["Y"].astype(np.float64)
    assert np.all(np.abs(got - ref) <= REL_TOL * np.abs(ref))
    layer.free()


def test_three_chained_convolutions_in_a_captured_graph(b):
    """quantize -> conv+requant -> conv+requant -> conv (float) recorded into a graph: the chained entry
    points allocate nothing and clear their output with a fill kernel, so every replay must reproduce the
    eager result, with eager work between the replays.  One layer has more than 128 rows (zero fill +
    atomics), the others at most 128 (plain stores)."""
    B, H, W = 3, 9, 11
    P = B * H * W
    shapes = [(64, 64), (192, 64), (128, 192)]               # (N, C) of the three layers
    layers = []
    for i, (N, C) in enumerate(shapes):
        Wt, delta, _, _ = synth.random_case(500 + i, N, 9 * C, 1, 2, rho=0.03)
        layers.append(b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta)))
    Xmap = torch.from_numpy(np.maximum(np.random.default_rng(9).standard_normal((64, P)), 0).astype(np.float32)).cuda()
    f0 = b.alloc_packed(64, P, 2)
    f1 = b.alloc_packed(64, P, 2)
    f2 = b.alloc_packed(192, P, 2)
    Y = torch.empty((128, P), dtype=torch.float32, device="cuda")

    def net():
        b.apb_quantize_acts(Xmap, 2, 0.75, packed=f0)
        b.apb_forward_conv3x3_requant(layers[0], f0, B, H, W, 2, 0.75, 2, 0.6, fmap_out=f1)
        b.apb_forward_conv3x3_requant(layers[1], f1, B, H, W, 2, 0.6, 2, 0.9, fmap_out=f2)
        b.apb_forward_conv3x3(layers[2], f2, B, H, W, 2, 0.9, Y=Y)

    net()
    torch.cuda.synchronize()
    y_ref, f2_ref = Y.clone(), f2.clone()
    assert f2_ref.any() and y_ref.abs().max() > 0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        net()
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        net()
    for _ in range(3):
        Y.zero_()
        f1.fill_(-1)
        f2.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(f2, f2_ref) and torch.equal(Y, y_ref)
        net()
        torch.cuda.synchronize()
        assert torch.equal(Y, y_ref)
    for layer in layers:
        layer.free()
