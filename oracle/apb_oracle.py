"""CPU oracle for the APB layer forward pass -- TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct implementation of what the hot path computes,
written from the paper (arXiv 2306.08960).  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product (the HIP library and
its Python binding) never does, and this file imports nothing from the product.

Notation (the benchmark's, the paper's in brackets): W [A] is the N x K weight
matrix, X [B] the K x M activation matrix, Y [C] the N x M output.  `delta` is
the half-width of the binarization interval, i.e. the paper's alpha + delta in
the definition of the APB operator (Sec. III, Eq. 3).

What is computed, and where it is defined:

  compress        Sec. III Eq. 1 (sign convention), Eq. 3 (partition),
                  "Memory Impact" (binary matrix fully represented),
                  "Inference Considerations" Eqs. 11-12 (mask, A^bin, A^full)
  mem_bits        Sec. III Eq. 10
  quantize        Sec. IV "1/2": a_p = p*s, p in {0,1,2,3};  "1/1": +-beta
  T_transform     Sec. IV Table "transformation T" and its decoding rules
  mbm             Sec. IV Eq. 18
  dot_1_1_xor     Sec. IV Eq. 16
  dot_1_2_mbm     Sec. IV Eq. 19 with the level weights 3/2 and 1/2 that the
                  printed equation leaves out, plus the zero-centering term
                  mu * sum(w), mu = 3s/2
  forward         Sec. III Eq. 13:  C = A^bin * B + A^full * B
  forward_requant Eq. 13 of one layer followed by the activation quantizer
                  (Sec. IV) of the layer it feeds, with an optional per-row
                  affine map in between (a folded batch normalization)
  im2col_codes    Sec. III, footnote on convolutions: a convolution is the matrix
                  product of the layer with the im2col matrix of its input map
  dot_2_2_mbm     Sec. IV "2/2": the 1/2 routine applied twice -- four mbm terms
                  under the and of the two masks, with the level weights 9/4,
                  3/4, 3/4, 1/4 that the printed equation leaves out (and the
                  operands t_w, t_a in its first term)
  gemm_2_2        Sec. IV "2/2": 2-bit weights (zero-centred levels) times
                  2-bit activations a_p = p*s
  brute_force     the plain definition: APB(W) (Eq. 3) times the dequantized
                  activations, as one dense float64 product

Readings taken where the paper is silent (each is listed in the design notes):
the interval test is the exact float32 compare |w| <= delta; sign uses the
compare w >= 0 (so -0.0 is +); the sparse values are the residuals
w - alpha*sign(w) computed as ONE float32 subtraction; default alpha is the
float64 mean of |w| over the binarized set rounded to float32; the 2-bit
quantizer is p = clamp(rint(x * (1/s)), 0, 3) with float32 arithmetic and
round-half-to-even; dequantized activations are the exact reals c*s (float64);
all floating-point accumulation is float64, the output is rounded once to
float32.  For the 2/2 routine the paper takes the quantized weights as given;
here the 2-bit weight quantizer is the uniform mid-rise one with step s_w:
level index q = clamp(floor(w * (1/s_w)) + 2, 0, 3), value (q - 3/2) * s_w
(the zero-centred levels of Sec. IV "2/2"), float32 arithmetic, NaN -> 0.

Packed activation buffer (the library's interface layout, re-stated here
independently): Kw = ceil(K/32), Mp = 64*ceil(M/64); uint32 planes
[bits][Kw][Mp] where bit i of planes[b][j][m] is bit b of the code of element
(k = 32*j + i, m), followed by int32 colsum[Mp] = sum_k code[k, m]; columns
m >= M and bits k >= K are zero.  For 1-bit activations the code is 1 for
x >= 0 and 0 otherwise.
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------- compress


def sign_bits(W: np.ndarray) -> np.ndarray:
    """Eq. 1: +alpha iff w >= 0.  Returns bool [N,K], True <-> +1."""
    return np.asarray(W, dtype=np.float32) >= np.float32(0.0)


def outlier_mask(W: np.ndarray, delta) -> np.ndarray:
    """Eq. 3: a weight is binarized iff |w| <= delta; everything else stays full precision."""
    return np.abs(np.asarray(W, dtype=np.float32)) > np.float32(delta)


def default_alpha(W: np.ndarray, delta) -> np.float32:
    """Mean |w| over the binarized set (float64 sum), 0 if the set is empty."""
    W = np.asarray(W, dtype=np.float32)
    inl = ~outlier_mask(W, delta)
    cnt = int(inl.sum())
    if cnt == 0:
        return np.float32(0.0)
    total = np.abs(W[inl]).astype(np.float64).sum()
    return np.float32(total / cnt)


def pack_bits_rows(bits: np.ndarray) -> np.ndarray:
    """bool [R,C] -> uint32 [R, ceil(C/32)]; bit i of word j <-> column 32*j+i; pad bits 0."""
    R, C = bits.shape
    Cw = (C + 31) // 32
    out = np.zeros((R, Cw), dtype=np.uint32)
    for c in range(C):
        out[:, c // 32] |= bits[:, c].astype(np.uint32) << np.uint32(c % 32)
    return out


def compress(W: np.ndarray, delta, alpha=None) -> dict:
    """Split W into the fully represented sign matrix and the CSR of residuals (Eqs. 11-12)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    bit = sign_bits(W)
    out = outlier_mask(W, delta)
    a = default_alpha(W, delta) if alpha is None else np.float32(alpha)
    signed_alpha = np.where(bit, a, -a).astype(np.float32)          # A^bin, every position
    counts = out.sum(axis=1).astype(np.int64)
    row_ptr = np.zeros(N + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(counts)
    rows, cols = np.nonzero(out)                                     # row-major, columns ascending
    val = (W[rows, cols] - signed_alpha[rows, cols]).astype(np.float32)   # one fp32 subtraction
    sigma = np.where(bit, 1, -1).astype(np.int32)
    return {
        "N": N, "K": K, "alpha": a, "bit": bit, "out": out,
        "sign_words": pack_bits_rows(bit),
        "row_ptr": row_ptr, "col_idx": cols.astype(np.int32), "val": val,
        "rowsum": sigma.sum(axis=1).astype(np.int32),
    }


def position_bits(N: int, K: int) -> int:
    """b_p of Eq. 10 read as the bits of a flat index into the N*K matrix."""
    n = N * K
    return 1 if n <= 2 else int(np.floor(np.log2(n - 1))) + 1


def mem_bits(N: int, K: int, nnz: int) -> int:
    """Eq. 10 in its 'fully represented' form: n + s*(b_v + b_p), b_v = 32."""
    return N * K + nnz * (32 + position_bits(N, K))


def apb_dense(W: np.ndarray, delta, alpha) -> np.ndarray:
    """Eq. 3 applied element-wise; float64 [N,K]."""
    W = np.asarray(W, dtype=np.float32)
    a = np.float64(np.float32(alpha))
    binar = np.where(sign_bits(W), a, -a)
    return np.where(outlier_mask(W, delta), W.astype(np.float64), binar)


# --------------------------------------------------------------------------- activations


def quantize(X: np.ndarray, bits: int, step) -> np.ndarray:
    """Integer activation values c [K,M] int8: +-1 (1-bit) or the level index p (2-bit)."""
    X = np.asarray(X, dtype=np.float32)
    if bits == 1:
        return np.where(X >= np.float32(0.0), 1, -1).astype(np.int8)
    if bits == 2:
        inv = np.float32(1.0) / np.float32(step)
        with np.errstate(invalid="ignore"):
            r = np.rint(X * inv)                   # float32 multiply, ties to even
        r = np.fmax(np.float32(0.0), r)            # fmax: a NaN input falls to 0
        r = np.fmin(np.float32(3.0), r)
        return r.astype(np.int8)
    raise ValueError("bits must be 1 or 2")


def codes_of(c: np.ndarray, bits: int) -> np.ndarray:
    """Stored code of each value: 1-bit {-1,+1} -> {0,1}; 2-bit p -> p."""
    return ((c.astype(np.int32) + 1) // 2).astype(np.uint8) if bits == 1 else c.astype(np.uint8)


def dequantize(c: np.ndarray, step) -> np.ndarray:
    """The reals c*s (1/2: a_p = p*s; 1/1: +-beta), float64."""
    return c.astype(np.float64) * np.float64(np.float32(step))


def pack_acts(c: np.ndarray, bits: int) -> np.ndarray:
    """Packed interface buffer (see module docstring) as a flat uint32 array."""
    K, M = c.shape
    Kw, Mp = (K + 31) // 32, 64 * ((M + 63) // 64)
    code = codes_of(c, bits)
    planes = np.zeros((bits, Kw, Mp), dtype=np.uint32)
    for b in range(bits):
        for k in range(K):
            planes[b, k // 32, :M] |= ((code[k] >> b) & 1).astype(np.uint32) << np.uint32(k % 32)
    colsum = np.zeros(Mp, dtype=np.int32)
    colsum[:M] = code.astype(np.int32).sum(axis=0)
    return np.concatenate([planes.ravel(), colsum.view(np.uint32)])


def acts_words(K: int, M: int, bits: int) -> int:
    Kw, Mp = (K + 31) // 32, 64 * ((M + 63) // 64)
    return Mp * (bits * Kw + 1)


# --------------------------------------------------------------------------- paper's bitwise forms


def popcount(v) -> int:
    return bin(int(v)).count("1")


def dot_1_1_xor(u_bits, v_bits) -> int:
    """Eq. 16 on {0,1}-encoded +-1 vectors: n - 2*popcount(xor(u, v))."""
    u = np.asarray(u_bits).astype(bool)
    v = np.asarray(v_bits).astype(bool)
    return int(u.size - 2 * np.count_nonzero(np.logical_xor(u, v)))


def T_transform(p: np.ndarray):
    """Table of T: level index p (zero-centred value (p - 3/2)) -> bit vectors (t, h, m)."""
    p = np.asarray(p).astype(np.int64)
    t = (p == 3)
    h = (p == 2)
    m = (p == 0) | (p == 3)
    return t, h, m


def T_inverse(t, h, m) -> np.ndarray:
    """Decoding rules below the table of T; returns the level index p."""
    t = np.asarray(t, bool)
    h = np.asarray(h, bool)
    m = np.asarray(m, bool)
    p = np.empty(t.shape, dtype=np.int64)
    p[t] = 3
    p[h] = 2
    p[m & ~t] = 0
    p[~m & ~h] = 1
    return p


def mbm(x, y, z) -> int:
    """Eq. 18: popcount(z) - 2*popcount(and(xor(x, y), z)) on bool vectors."""
    x = np.asarray(x, bool)
    y = np.asarray(y, bool)
    z = np.asarray(z, bool)
    return int(np.count_nonzero(z) - 2 * np.count_nonzero(np.logical_xor(x, y) & z))


def dot_1_2_mbm_twice(w_bits, p) -> int:
    """TWICE the dot product (in units of s) of a +-1 vector and level indices p, the paper's way.

    Zero-centre (a_bar = a - 3s/2), split by T, apply mbm to the three-halves part under m and
    to the one-half part under not-m, weight them 3/2 and 1/2, add back mu * sum(w):
        2 * (w . p) = 3*mbm(w,t,m) + mbm(w,h,~m) + 3*sum(w).
    """
    w = np.asarray(w_bits, bool)
    t, h, m = T_transform(p)
    sum_w = int(2 * np.count_nonzero(w) - w.size)
    return 3 * mbm(w, t, m) + mbm(w, h, ~m) + 3 * sum_w


# --------------------------------------------------------------------------- forward, step by step


def int_part_unpacked(bit: np.ndarray, c: np.ndarray) -> np.ndarray:
    """D[n,m] = sum_k sigma[n,k] * c[k,m], int64 accumulation, returned as int32."""
    sigma = np.where(bit, 1, -1).astype(np.int64)
    return (sigma @ c.astype(np.int64)).astype(np.int32)


def int_part_packed(sign_words: np.ndarray, packed: np.ndarray, K: int, M: int, bits: int) -> np.ndarray:
    """Same D from packed words: Eq. 16 (1-bit) or the AND/popcount bit-plane form (2-bit).

    Pure-Python popcounts: small cases only.
    """
    N, Kw = sign_words.shape
    Mp = 64 * ((M + 63) // 64)
    planes = packed[: bits * Kw * Mp].reshape(bits, Kw, Mp)
    colsum = packed[bits * Kw * Mp:].view(np.int32)
    D = np.zeros((N, M), dtype=np.int32)
    for n in range(N):
        for m in range(M):
            if bits == 1:
                diff = sum(popcount(sign_words[n, j] ^ planes[0, j, m]) for j in range(Kw))
                # pad bits are 0 on both sides and cancel in the xor
                D[n, m] = K - 2 * diff
            else:
                pos = sum((1 << b) * popcount(sign_words[n, j] & planes[b, j, m])
                          for b in range(bits) for j in range(Kw))
                D[n, m] = 2 * pos - int(colsum[m])
    return D


def sparse_part(row_ptr, col_idx, val, c: np.ndarray, step) -> np.ndarray:
    """R[n,m] = sum_{j in row n} val_j * xhat[col_j, m], float64."""
    xhat = dequantize(c, step)
    N = len(row_ptr) - 1
    R = np.zeros((N, c.shape[1]), dtype=np.float64)
    for n in range(N):
        for j in range(int(row_ptr[n]), int(row_ptr[n + 1])):
            R[n] += np.float64(val[j]) * xhat[col_idx[j]]
    return R


def epilogue(alpha, step, D: np.ndarray, R: np.ndarray) -> np.ndarray:
    """Y = alpha*s*D + R in float64, rounded once to float32 (Eq. 13 with the scalars of Sec. IV)."""
    a = np.float64(np.float32(alpha))
    s = np.float64(np.float32(step))
    return (a * s * D.astype(np.float64) + R).astype(np.float32)


def forward(layer: dict, c: np.ndarray, step) -> dict:
    D = int_part_unpacked(layer["bit"], c)
    R = sparse_part(layer["row_ptr"], layer["col_idx"], layer["val"], c, step)
    return {"D": D, "R": R, "Y": epilogue(layer["alpha"], step, D, R)}


def requant(alpha, step, D: np.ndarray, R: np.ndarray, bits_out: int, step_out, scale=None, shift=None) -> dict:
    """The activations the next layer sees, from the two parts of Eq. 13: Z = scale[n]*Y + shift[n]
    (Z = Y without scale) formed in float64 from the float64 Y = alpha*s*D + R, rounded once to float32
    and then quantized as any other activation matrix (N x M: this layer's rows are the next layer's K)."""
    y = np.float64(np.float32(alpha)) * np.float64(np.float32(step)) * D.astype(np.float64) + R
    if scale is not None:
        y = np.asarray(scale, dtype=np.float32).astype(np.float64)[:, None] * y \
            + np.asarray(shift, dtype=np.float32).astype(np.float64)[:, None]
    Z = y.astype(np.float32)
    c_out = quantize(Z, bits_out, step_out)
    return {"Z": Z, "c": c_out, "packed": pack_acts(c_out, bits_out)}


def forward_requant(layer: dict, c: np.ndarray, step, bits_out: int, step_out, scale=None, shift=None) -> dict:
    D = int_part_unpacked(layer["bit"], c)
    R = sparse_part(layer["row_ptr"], layer["col_idx"], layer["val"], c, step)
    return requant(layer["alpha"], step, D, R, bits_out, step_out, scale, shift)


def conv_out_size(H: int, stride: int) -> int:
    """Output rows (or columns) of a 3-wide window with padding 1 moved in steps of `stride` over H inputs."""
    return (H - 1) // stride + 1


def im2col_codes(c_map: np.ndarray, B: int, H: int, W: int, bits: int, stride: int = 1) -> np.ndarray:
    """Patch matrix [9*C, B*Ho*Wo] of a 3x3 convolution (padding 1, the given stride; Ho, Wo = conv_out_size)
    over the integer activation values of a feature map [C, B*H*W] (column = (b*H + y)*W + x).  Row tap*C + ch
    with tap = 3*ky + kx; output column (b, yo, xo) holds the value at (b, stride*yo + ky - 1, stride*xo + kx - 1),
    and outside the image the value whose stored code is 0: 0 for 2-bit activations (zero padding), -1 for
    1-bit ones."""
    C, P = c_map.shape
    assert P == B * H * W and stride >= 1
    Ho, Wo = conv_out_size(H, stride), conv_out_size(W, stride)
    padded = np.full((C, B, H + 2, W + 2), 0 if bits == 2 else -1, dtype=c_map.dtype)
    padded[:, :, 1:H + 1, 1:W + 1] = c_map.reshape(C, B, H, W)
    taps = []
    for ky in range(3):
        for kx in range(3):
            view = padded[:, :, ky:ky + stride * (Ho - 1) + 1:stride, kx:kx + stride * (Wo - 1) + 1:stride]
            assert view.shape == (C, B, Ho, Wo)
            taps.append(view.reshape(C, B * Ho * Wo))
    return np.concatenate(taps, axis=0)


def brute_force(W: np.ndarray, delta, alpha, X: np.ndarray, bits: int, step) -> np.ndarray:
    """The plain definition, float64: APB(W) @ dequantize(quantize(X))."""
    return apb_dense(W, delta, alpha) @ dequantize(quantize(X, bits, step), step)


# --------------------------------------------------------------------------- the 2/2 routine


def quantize_weights_2bit(W: np.ndarray, step_w) -> np.ndarray:
    """Level index q in {0,1,2,3} of every weight; the weight it stands for is (q - 3/2) * s_w."""
    W = np.asarray(W, dtype=np.float32)
    inv = np.float32(1.0) / np.float32(step_w)
    t = np.floor(W * inv) + np.float32(2.0)
    with np.errstate(invalid="ignore"):
        t = np.where(np.isnan(t), np.float32(0.0), t)
    return np.clip(t, 0.0, 3.0).astype(np.uint8)


def pack_weight_planes(q: np.ndarray) -> np.ndarray:
    """uint32 [2][N][Kw]: bit i of word j of plane b = bit b of q[n, 32*j + i]; pad bits 0."""
    q = np.asarray(q, dtype=np.uint8)
    return np.stack([pack_bits_rows((q >> b) & 1) for b in range(2)])


def dot_2_2_mbm_times4(q, p) -> int:
    """FOUR times the dot product, in units of s_w*s_a, of zero-centred 2-bit vectors, the paper's way.

    Both level-index vectors stand for values (q - 3/2) and (p - 3/2).  T splits each into a
    three-halves part (under its mask m) and a one-half part (under not-m); each of the four
    pairings is one mbm under the and of the two masks and carries the product of its levels:
        4 * (w_bar . a_bar) = 9*mbm(t_w,t_a,m_w&m_a) + 3*mbm(t_w,h_a,m_w&~m_a)
                            + 3*mbm(h_w,t_a,~m_w&m_a) + mbm(h_w,h_a,~m_w&~m_a).
    """
    tw, hw, mw = T_transform(q)
    ta, ha, ma = T_transform(p)
    return (9 * mbm(tw, ta, mw & ma) + 3 * mbm(tw, ha, mw & ~ma)
            + 3 * mbm(hw, ta, ~mw & ma) + mbm(hw, ha, ~mw & ~ma))


def int_2_2_unpacked(q: np.ndarray, c: np.ndarray) -> np.ndarray:
    """D22[n,m] = sum_k (2*q[n,k] - 3) * p[k,m]  (= 2/(s_w*s_a) times the product of the zero-centred
    weights with the activations p*s_a).  The matrix product runs in float64, which is exact here
    (every partial sum is an integer far below 2^53)."""
    wq = 2.0 * np.asarray(q).astype(np.float64) - 3.0
    return np.rint(wq @ np.asarray(c).astype(np.float64)).astype(np.int32)


def int_2_2_packed(wplanes: np.ndarray, packed: np.ndarray, K: int, M: int) -> np.ndarray:
    """The same D22 from packed words: sum over the four plane pairs of 2^(a+b) * popcount(W_a & P_b)
    gives sum_k q*p; the zero-centring of the weights takes 3/2 * colsum off.  Small cases only."""
    _, N, Kw = wplanes.shape
    Mp = 64 * ((M + 63) // 64)
    planes = packed[: 2 * Kw * Mp].reshape(2, Kw, Mp)
    colsum = packed[2 * Kw * Mp:].view(np.int32)
    D = np.zeros((N, M), dtype=np.int32)
    for n in range(N):
        for m in range(M):
            qp = sum((1 << (a + b)) * popcount(wplanes[a, n, j] & planes[b, j, m])
                     for a in range(2) for b in range(2) for j in range(Kw))
            D[n, m] = 2 * qp - 3 * int(colsum[m])
    return D


def gemm_2_2(q: np.ndarray, c: np.ndarray, step_w, step_a) -> dict:
    """Y = W_q @ A_q with W_q = (q - 3/2)*s_w and A_q = p*s_a: (s_w*s_a/2) * D22 in float64, rounded
    once to float32."""
    D = int_2_2_unpacked(q, c)
    sw = np.float64(np.float32(step_w))
    sa = np.float64(np.float32(step_a))
    return {"D": D, "Y": (0.5 * sw * sa * D.astype(np.float64)).astype(np.float32)}


def brute_force_2_2(W: np.ndarray, step_w, X: np.ndarray, step_a) -> np.ndarray:
    """The plain definition, float64: dequantized 2-bit weights times dequantized 2-bit activations."""
    q = quantize_weights_2bit(W, step_w).astype(np.float64)
    Wq = (q - 1.5) * np.float64(np.float32(step_w))
    return Wq @ dequantize(quantize(X, 2, step_a), step_a)
