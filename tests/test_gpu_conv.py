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


def torch_im2col(Xmap_d, C, B, H, W, pad_value, stride=1):
    """Explicit float im2col [9*C, B*Ho*Wo] on the GPU (plain torch indexing; test-side only)."""
    x = torch.full((C, B, H + 2, W + 2), pad_value, dtype=torch.float32, device=Xmap_d.device)
    x[:, :, 1:H + 1, 1:W + 1] = Xmap_d.view(C, B, H, W)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    return torch.cat([x[:, :, ky:ky + stride * (Ho - 1) + 1:stride, kx:kx + stride * (Wo - 1) + 1:stride].reshape(C, B * Ho * Wo)
                      for ky in range(3) for kx in range(3)], dim=0)


SHAPES = [  # N, C, B, H, W, stride
    (20, 64, 2, 5, 7, 1), (64, 64, 3, 8, 8, 1), (130, 128, 1, 9, 13, 1), (256, 64, 5, 8, 8, 1), (40, 64, 1, 1, 1, 1),
    (33, 64, 1, 1, 70, 1), (17, 64, 2, 66, 1, 1), (512, 192, 1, 7, 7, 1), (64, 64, 1, 32, 32, 1),
    # channel counts that are odd multiples of 32 (a matrix step then straddles two taps), down to one word
    (24, 32, 2, 6, 5, 1), (64, 96, 1, 9, 9, 1), (130, 160, 2, 7, 7, 1), (256, 32, 3, 8, 8, 1),
    # stride 2: even and odd image sizes, one-pixel images, few output pixels (K split inside the workgroup)
    (64, 64, 3, 8, 8, 2), (20, 64, 2, 5, 7, 2), (130, 128, 1, 9, 13, 2), (40, 64, 1, 1, 1, 2), (33, 32, 1, 2, 70, 2),
    (128, 64, 2, 16, 16, 2), (256, 96, 5, 15, 14, 2), (512, 160, 1, 7, 7, 2), (64, 64, 1, 32, 31, 2),
]


@pytest.mark.parametrize("bits", [2, 1])
@pytest.mark.parametrize("N,C,B,H,W,stride", SHAPES)
def test_conv_matches_oracle(b, N, C, B, H, W, stride, bits):
    print(f"[case] conv N={N} C={C} B={B} H={H} W={W} stride={stride} bits={bits}", flush=True)
    Wt, delta, Xmap, step = make_case(N + C + H * W, N, C, B, H, W, bits)
    Ho, Wo = o.conv_out_size(H, stride), o.conv_out_size(W, stride)
    P = B * Ho * Wo                                            # output pixels
    L = o.compress(Wt, delta)
    c_map = o.quantize(Xmap, bits, step)
    patches = o.im2col_codes(c_map, B, H, W, bits, stride)
    F = capi.forward(L, o.pack_acts(patches, bits), patches, bits, step, threads=THREADS)

    layer = b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta), alpha=float(L["alpha"]))
    fmap = b.apb_quantize_acts(torch.from_numpy(Xmap).cuda(), bits, float(step))
    assert np.array_equal(fmap.cpu().numpy().view(np.uint32), o.pack_acts(c_map, bits))
    Y = b.apb_forward_conv3x3(layer, fmap, B, H, W, bits, float(step), stride=stride).cpu().numpy()
    assert Y.shape == (N, P)
    ref = F["Y"].astype(np.float64)
    assert np.all(np.abs(Y.astype(np.float64) - ref) <= REL_TOL * np.abs(ref))
    # with a workspace (layers with many residuals per row then multiply the written-out packed patch matrix;
    # the others ignore it): the same bar, and a workspace that is too small is ignored as well
    ws = b.alloc_packed(9 * C, P, bits)
    for w in (ws, ws[: max(1, ws.numel() // 2)]):
        w.fill_(-1)
        Yw = b.apb_forward_conv3x3(layer, fmap, B, H, W, bits, float(step), stride=stride, workspace=w).cpu().numpy()
        assert np.all(np.abs(Yw.astype(np.float64) - ref) <= REL_TOL * np.abs(ref))

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
                                      None if sh is None else torch.from_numpy(sh).cuda(), fmap_out=out, stride=stride)
        torch.cuda.synchronize()
        code, pixsum = unpack(out.cpu().numpy().view(np.uint32), N, P, 2)
        assert np.array_equal(pixsum[:P], code.sum(axis=0))
        compare_codes(code, want, L["alpha"], step, F["D"], F["R"], 2, step_out, sc, sh)
        out_w = b.alloc_packed(N, P, 2)
        out_w.fill_(-1)
        ws.fill_(-1)
        b.apb_forward_conv3x3_requant(layer, fmap, B, H, W, bits, float(step), 2, float(step_out),
                                      None if sc is None else torch.from_numpy(sc).cuda(),
                                      None if sh is None else torch.from_numpy(sh).cuda(), fmap_out=out_w, stride=stride,
                                      workspace=ws)
        torch.cuda.synchronize()
        code_w, pixsum_w = unpack(out_w.cpu().numpy().view(np.uint32), N, P, 2)
        assert np.array_equal(pixsum_w[:P], code_w.sum(axis=0))
        compare_codes(code_w, want, L["alpha"], step, F["D"], F["R"], 2, step_out, sc, sh)
    if N % 32 == 0:
        # (the output map is B images of Ho x Wo pixels; the second layer runs on it with stride 1)
        W2, delta2, _, _ = synth.random_case(N + 1, 24, 9 * N, 1, 2, rho=0.02)
        L2 = o.compress(W2, delta2)
        c2 = code.astype(np.int8)
        patches2 = o.im2col_codes(c2, B, Ho, Wo, 2)
        F2 = capi.forward(L2, o.pack_acts(patches2, 2), patches2, 2, step_out, threads=THREADS)
        layer2 = b.apb_compress(torch.from_numpy(W2).cuda(), float(delta2), alpha=float(L2["alpha"]))
        Y2 = b.apb_forward_conv3x3(layer2, out, B, Ho, Wo, 2, float(step_out)).cpu().numpy()
        ref2 = F2["Y"].astype(np.float64)
        assert np.all(np.abs(Y2.astype(np.float64) - ref2) <= REL_TOL * np.abs(ref2))
        layer2.free()
    layer.free()


def test_shape_errors(b):
    Wt, delta, _, _ = synth.random_case(3, 8, 9 * 16, 1, 2)              # C = 16: not a multiple of 32
    layer = b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta))
    fmap = b.alloc_packed(16, 16, 2)
    with pytest.raises(b.ApbError) as e:
        b.apb_forward_conv3x3(layer, fmap, 1, 4, 4, 2, 0.75)
    assert e.value.code == b.APB_ERR_SHAPE
    layer.free()
    Wt, delta, _, _ = synth.random_case(4, 8, 9 * 32, 1, 2)
    layer = b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta))
    fmap = b.alloc_packed(32, 16, 2)
    Y = torch.empty((8, 16), device="cuda")
    lib = b.load()
    for stride in (0, 3, -1):                                           # only strides 1 and 2
        rc = lib.apb_forward_conv3x3(layer.handle, fmap.data_ptr(), 1, 4, 4, stride, 2, 0.75, None, 0, Y.data_ptr(), None)
        assert rc == b.APB_ERR_SHAPE
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
    ws = torch.full_like(packed, -1)
    assert torch.equal(b.apb_forward_conv3x3(layer, fmap, B, H, W, bits, float(step), workspace=ws), Y)
    if b.apb_forward_kernel_name(layer, P, bits).startswith("k_forward_rows"):
        assert torch.equal(ws, packed)                        # the packed patch matrix, word for word
    assert torch.equal(b.apb_forward_conv3x3_requant(layer, fmap, B, H, W, bits, float(step), 2, 1.0, workspace=ws), out)
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


@pytest.mark.parametrize("N,C,B,H,W,bits", [(128, 64, 64, 56, 56, 2), (256, 128, 64, 28, 28, 2), (512, 256, 128, 14, 14, 1),
                                            (96, 96, 32, 35, 35, 2)])
def test_full_size_stride_2_layers_equal_the_explicit_route(b, N, C, B, H, W, bits):
    """The first convolution of a ResNet stage (stride 2, channels doubled) at the size of the benchmark layers,
    and one with an odd multiple of 32 channels and odd image sizes: the implicit route against apb_quantize_acts
    on the explicit strided float im2col matrix + apb_forward (bit for bit, float and packed outputs), and sampled
    output pixels against the oracle (image corners and edges included)."""
    print(f"[case] stride-2 conv N={N} C={C} B={B} H={H} W={W} bits={bits}", flush=True)
    Wt, delta, Xmap, step = make_case(N + C + H, N, C, B, H, W, bits)
    Ho, Wo = o.conv_out_size(H, 2), o.conv_out_size(W, 2)
    P = B * Ho * Wo
    Xd = torch.from_numpy(Xmap).cuda()
    layer = b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta))
    fmap = b.apb_quantize_acts(Xd, bits, float(step))
    Y = b.apb_forward_conv3x3(layer, fmap, B, H, W, bits, float(step), stride=2)
    explicit = torch_im2col(Xd, C, B, H, W, 0.0 if bits == 2 else -1.0, stride=2)
    packed = b.apb_quantize_acts(explicit, bits, float(step))
    del explicit
    assert torch.equal(Y, b.apb_forward(layer, packed, P, bits, float(step)))
    out = b.apb_forward_conv3x3_requant(layer, fmap, B, H, W, bits, float(step), 2, 1.0, stride=2)
    assert torch.equal(out, b.apb_forward_requant(layer, packed, P, bits, float(step), 2, 1.0))
    # with a workspace: the packed patch matrix written there equals the quantized explicit matrix word for word
    # wherever the layer takes that route, and the outputs stay the same
    ws = torch.full_like(packed, -1)
    Yw = b.apb_forward_conv3x3(layer, fmap, B, H, W, bits, float(step), stride=2, workspace=ws)
    assert torch.equal(Yw, Y)
    if b.apb_forward_kernel_name(layer, P, bits).startswith("k_forward_rows"):
        assert torch.equal(ws, packed)
    assert torch.equal(b.apb_forward_conv3x3_requant(layer, fmap, B, H, W, bits, float(step), 2, 1.0, stride=2, workspace=ws), out)
    L = o.compress(Wt, delta, alpha=np.float32(layer.info()["alpha"]))
    pix = np.unique(np.concatenate([[0, Wo - 1, (Ho - 1) * Wo, Ho * Wo - 1, P - 1, P - Wo],
                                    np.random.default_rng(7).choice(P, 40, replace=False)]))
    c_map = o.quantize(Xmap, bits, step)
    cm = np.full((C, B, H + 2, W + 2), 0 if bits == 2 else -1, dtype=np.int8)
    cm[:, :, 1:H + 1, 1:W + 1] = c_map.reshape(C, B, H, W)
    bb, yy, xx = pix // (Ho * Wo), 2 * ((pix // Wo) % Ho), 2 * (pix % Wo)
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


def test_chain_on_the_rows_kernel_with_a_workspace_in_a_captured_graph(b):
    """Layers with many residuals per row: conv + requant through the packed patch matrix in a workspace (stride 2,
    then stride 1), then a fully-connected chained layer -- all on the rows-in-lanes kernel with its packed-output
    epilogue (LDS merge + atomics into a buffer cleared by a fill kernel or by the patch-packing launch).  Recorded
    into a graph and replayed with eager work in between: every replay must reproduce the eager result."""
    B, H, W = 3, 10, 9
    Ho, Wo = 5, 5
    P0, P1 = B * H * W, B * Ho * Wo
    layers = []
    for i, (N, C) in enumerate([(256, 64), (320, 256)]):
        Wt, delta, _, _ = synth.random_case(700 + i, N, 9 * C, 1, 2, rho=0.05)
        layers.append(b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta)))
    Wt, delta, _, _ = synth.random_case(702, 512, 320, 1, 2, rho=0.05)
    fc = b.apb_compress(torch.from_numpy(Wt).cuda(), float(delta))
    for layer, P in ((layers[0], P1), (layers[1], P1), (fc, P1)):
        assert b.apb_forward_kernel_name(layer, P, 2).startswith("k_forward_rows")
    Xmap = torch.from_numpy(np.maximum(np.random.default_rng(10).standard_normal((64, P0)), 0).astype(np.float32)).cuda()
    f0, f1, f2, f3 = b.alloc_packed(64, P0, 2), b.alloc_packed(256, P1, 2), b.alloc_packed(320, P1, 2), b.alloc_packed(512, P1, 2)
    ws = b.alloc_packed(9 * 256, P1, 2)                       # (the larger of the two patch matrices)
    Y = torch.empty((512, P1), dtype=torch.float32, device="cuda")

    def net():
        b.apb_quantize_acts(Xmap, 2, 0.75, packed=f0)
        b.apb_forward_conv3x3_requant(layers[0], f0, B, H, W, 2, 0.75, 2, 0.6, fmap_out=f1, stride=2, workspace=ws)
        b.apb_forward_conv3x3_requant(layers[1], f1, B, Ho, Wo, 2, 0.6, 2, 0.9, fmap_out=f2, workspace=ws)
        b.apb_forward_requant(fc, f2, P1, 2, 0.9, 2, 1.1, packed_out=f3)
        b.apb_forward(fc, f2, P1, 2, 0.9, Y=Y)

    net()
    torch.cuda.synchronize()
    y_ref, f3_ref = Y.clone(), f3.clone()
    assert f3_ref.any() and y_ref.abs().max() > 0
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
        for t in (f1, f2, f3, ws):
            t.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(f3, f3_ref) and torch.equal(Y, y_ref)
        net()
        torch.cuda.synchronize()
        assert torch.equal(Y, y_ref)
    for layer in layers + [fc]:
        layer.free()
