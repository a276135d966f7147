"""Pins for the CPU oracle: every check compares it with something that is NOT the oracle --
values the paper prints, closed forms, hand-worked cases, textbook special cases, or a direct
element-by-element evaluation of the definition written here in the test."""
import os

import numpy as np
import pytest

from oracle import apb_oracle as o
from oracle import capi

rng = np.random.default_rng(20230608)


# ----------------------------------------------------------------------------- Table of T
def _read_T(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "T_table.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a, t, h, m = line.split()
            num, den = a.split("/")
            rows.append((int(num) / int(den), int(t), int(h), int(m)))
    return rows


def test_T_matches_printed_table(golden_dir):
    rows = _read_T(golden_dir)
    assert len(rows) == 4
    for a_bar, t, h, m in rows:
        p = int(a_bar + 1.5)
        tt, hh, mm = o.T_transform(np.array([p]))
        assert (int(tt[0]), int(hh[0]), int(mm[0])) == (t, h, m)


def test_T_bijective_and_decoding_rules(golden_dir):
    triples = {(t, h, m) for _, t, h, m in _read_T(golden_dir)}
    assert len(triples) == 4                               # injective on the four levels
    p = rng.integers(0, 4, 1000)
    t, h, m = o.T_transform(p)
    assert np.array_equal(o.T_inverse(t, h, m), p)
    # decoding rules: t=1 -> 3/2, h=1 -> 1/2, m=1 & t=0 -> -3/2, m=0 & h=0 -> -1/2
    assert np.all(p[t] == 3) and np.all(p[h] == 2)
    assert np.all(p[m & ~t] == 0) and np.all(p[~m & ~h] == 1)


def test_bitplanes_reproduce_T(golden_dir):
    """The stored planes P0 (low bit of p) and P1 (high bit) give t, h, m by pure logic."""
    for a_bar, t, h, m in _read_T(golden_dir):
        p = int(a_bar + 1.5)
        P0, P1 = p & 1, (p >> 1) & 1
        assert (P1 & P0, P1 & (1 - P0), 1 - (P1 ^ P0)) == (t, h, m)


# ----------------------------------------------------------------------------- Eq. 16 / 18 / 19
def test_eq16_all_lengths():
    for n in range(1, 131):
        u = rng.integers(0, 2, n)
        v = rng.integers(0, 2, n)
        direct = int(np.sum((2 * u - 1) * (2 * v - 1)))
        assert o.dot_1_1_xor(u, v) == direct
        assert o.dot_1_1_xor(u, u) == n
        assert o.dot_1_1_xor(u, 1 - u) == -n


def test_mbm_is_masked_signed_agreement():
    for n in (1, 2, 31, 32, 33, 100):
        x, y, z = (rng.integers(0, 2, n) for _ in range(3))
        direct = int(np.sum(((2 * x - 1) * (2 * y - 1))[z == 1]))
        assert o.mbm(x, y, z) == direct


def test_one_two_routine_equals_direct_sum():
    for n in list(range(1, 70)) + [127, 128, 129, 500]:
        w = rng.integers(0, 2, n)
        p = rng.integers(0, 4, n)
        direct = int(np.sum((2 * w - 1) * p))
        assert o.dot_1_2_mbm_twice(w, p) == 2 * direct


def test_printed_eq19_needs_level_weights():
    """n=1, w=+1, a_bar=3/2: the printed sum of the two mbm terms gives 1, the true product is 3/2."""
    w, p = np.array([1]), np.array([3])
    t, h, m = o.T_transform(p)
    assert o.mbm(w, t, m) + o.mbm(w, h, ~m) == 1
    assert o.dot_1_2_mbm_twice(w, p) == 2 * 3              # (3/2 + 3/2) * 2 in units of s


# ----------------------------------------------------------------------------- compress
def test_partition_boundaries_and_sign_convention():
    delta = np.float32(0.5)
    W = np.array([[0.5, -0.5, np.nextafter(np.float32(0.5), np.float32(1)), -0.0, 0.0, -0.75, 2.0, -1e-30]],
                 dtype=np.float32)
    L = o.compress(W, delta, alpha=np.float32(0.25))
    assert L["out"].tolist() == [[False, False, True, False, False, True, True, False]]
    assert L["bit"].tolist() == [[True, False, True, True, True, False, True, False]]
    assert L["row_ptr"].tolist() == [0, 3]
    assert L["col_idx"].tolist() == [2, 5, 6]
    # residuals w - alpha*sign(w), hand-computed (all exact in float32 here)
    assert L["val"].tolist() == [float(np.float32(W[0, 2]) - np.float32(0.25)), -0.5, 1.75]
    assert L["rowsum"].tolist() == [5 - 3]
    assert int(L["sign_words"][0, 0]) == 0b01011101


def test_sign_word_bit_order_and_padding():
    W = -np.ones((2, 70), dtype=np.float32)
    W[0, 0] = W[0, 33] = W[1, 69] = 1.0
    L = o.compress(W, np.float32(10.0), alpha=np.float32(1.0))
    sw = L["sign_words"]
    assert sw.shape == (2, 3)
    assert sw[0].tolist() == [1, 2, 0]
    assert sw[1].tolist() == [0, 0, 1 << 5]


def test_extreme_intervals_and_memory_formula():
    N, K = 8, 128                                          # n = 1024 weights -> flat index needs 10 bits
    W = rng.standard_normal((N, K)).astype(np.float32)
    none = o.compress(W, np.float32(np.inf))
    assert none["row_ptr"][-1] == 0 and none["val"].size == 0
    allo = o.compress(W, np.float32(-1.0))
    assert allo["row_ptr"][-1] == N * K
    assert np.array_equal(allo["col_idx"].reshape(N, K), np.tile(np.arange(K), (N, 1)))
    assert allo["alpha"] == 0.0                            # empty binarized set
    assert np.array_equal(allo["val"].reshape(N, K), W)    # residual of alpha = 0 is w itself
    assert o.position_bits(N, K) == 10
    assert o.mem_bits(N, K, 0) == 1024
    assert o.mem_bits(N, K, 7) == 1024 + 7 * (32 + 10)
    assert o.position_bits(256, 256) == 16 and o.position_bits(4096, 4096) == 24


def test_default_alpha_closed_forms():
    W = np.full((4, 9), 0.125, dtype=np.float32)
    W[::2] *= -1
    assert o.default_alpha(W, np.float32(1.0)) == np.float32(0.125)
    W[0, 0] = 50.0                                         # outlier: must not enter the mean
    assert o.default_alpha(W, np.float32(1.0)) == np.float32(0.125)
    W2 = np.array([[0.1, -0.3, 0.2, 7.0]], dtype=np.float32)
    want = np.float32((np.float64(np.float32(0.1)) + np.float64(np.float32(0.3)) + np.float64(np.float32(0.2))) / 3)
    assert o.default_alpha(W2, np.float32(1.0)) == want


def test_reconstruction_matches_definition():
    """alpha*sigma + scatter(val) must be Eq. 3's matrix: exact inside, within 1 ulp outside."""
    W = (rng.standard_normal((13, 77)) * 0.05).astype(np.float32)
    delta = np.float32(0.08)
    L = o.compress(W, delta)
    a = np.float64(L["alpha"])
    rec = np.where(L["bit"], a, -a)
    for n in range(13):
        for j in range(L["row_ptr"][n], L["row_ptr"][n + 1]):
            rec[n, L["col_idx"][j]] += np.float64(L["val"][j])
    want = np.empty_like(rec)                              # Eq. 3, element by element
    for n in range(13):
        for k in range(77):
            w = W[n, k]
            want[n, k] = (a if w >= 0 else -a) if abs(w) <= delta else np.float64(w)
    inside = np.abs(W) <= delta
    assert np.array_equal(rec[inside], want[inside])
    ulp = np.spacing(np.abs(W[~inside]).astype(np.float32)).astype(np.float64)
    assert np.all(np.abs(rec[~inside] - want[~inside]) <= ulp)
    assert L["row_ptr"][-1] == np.count_nonzero(~inside) > 0
    assert np.array_equal(o.apb_dense(W, delta, L["alpha"]), want)


# ----------------------------------------------------------------------------- quantizer
def test_two_bit_quantizer_hand_cases():
    s = np.float32(0.5)                                    # 1/s = 2 exactly
    x = np.array([[-3.0, -0.0, 0.0, 0.24, 0.25, 0.26, 0.5, 0.75, 1.0, 1.25, 1.4, 1.5, 9.0, np.nan]],
                 dtype=np.float32).T
    #  x/s:          -6    0    0   .48  .5->0 .52  1   1.5->2  2  2.5->2 2.8   3    18   nan->0
    want = [0, 0, 0, 0, 0, 1, 1, 2, 2, 2, 3, 3, 3, 0]
    assert o.quantize(x, 2, s)[:, 0].tolist() == want
    assert np.array_equal(o.dequantize(o.quantize(x, 2, s), s)[:, 0], np.array(want) * 0.5)


def test_one_bit_quantizer_hand_cases():
    x = np.array([[-1.0, -0.0, 0.0, 1e-30, -1e-30]], dtype=np.float32)
    c = o.quantize(x, 1, np.float32(2.0))
    assert c.tolist() == [[-1, 1, 1, 1, -1]]
    assert o.dequantize(c, np.float32(2.0)).tolist() == [[-2.0, 2.0, 2.0, 2.0, -2.0]]
    assert o.codes_of(c, 1).tolist() == [[0, 1, 1, 1, 0]]


def test_pack_acts_layout():
    c = np.zeros((40, 3), dtype=np.int8)
    c[0, 0] = 1
    c[33, 1] = 3
    c[39, 2] = 2
    buf = o.pack_acts(c, 2)
    Kw, Mp = 2, 64
    assert buf.size == o.acts_words(40, 3, 2) == Mp * (2 * Kw + 1)
    planes = buf[: 2 * Kw * Mp].reshape(2, Kw, Mp)
    want = np.zeros((2, Kw, Mp), dtype=np.uint32)
    want[0, 0, 0] = 1
    want[0, 1, 1] = 2
    want[1, 1, 1] = 2
    want[1, 1, 2] = 1 << 7
    assert np.array_equal(planes, want)
    assert buf[2 * Kw * Mp:].view(np.int32)[:4].tolist() == [1, 3, 2, 0]


# ----------------------------------------------------------------------------- integer part
SHAPES = [(1, 1, 1), (3, 5, 2), (7, 31, 9), (5, 32, 64), (4, 33, 65), (9, 100, 70), (2, 130, 1), (1, 64, 129)]


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("N,K,M", SHAPES)
def test_integer_part_three_ways(N, K, M, bits):
    bit = rng.integers(0, 2, (N, K)).astype(bool)
    c = (rng.integers(0, 2, (K, M)) * 2 - 1 if bits == 1 else rng.integers(0, 4, (K, M))).astype(np.int8)
    D = o.int_part_unpacked(bit, c)
    direct = np.zeros((N, M), dtype=np.int64)              # the definition, element by element
    for n in range(N):
        for m in range(M):
            direct[n, m] = sum((1 if bit[n, k] else -1) * int(c[k, m]) for k in range(K))
    assert np.array_equal(D, direct)
    sw = o.pack_bits_rows(bit)
    packed = o.pack_acts(c, bits)
    assert np.array_equal(o.int_part_packed(sw, packed, K, M, bits), direct)
    assert np.array_equal(capi.int_packed(sw, packed, K, M, bits), direct)
    assert np.array_equal(capi.int_packed(sw, packed, K, M, bits, threads=3), direct)
    assert np.array_equal(capi.int_unpacked(bit, c), direct)
    assert np.all(np.abs(direct) <= (3 if bits == 2 else 1) * K)
    if bits == 2:                                          # the paper's T / mbm route, one column
        for n in range(N):
            assert o.dot_1_2_mbm_twice(bit[n], c[:, 0]) == 2 * direct[n, 0]
    else:
        for n in range(N):
            assert o.dot_1_1_xor(bit[n], c[:, 0] > 0) == direct[n, 0]


def test_integer_part_closed_forms():
    N, K, M = 6, 75, 5
    bit = rng.integers(0, 2, (N, K)).astype(bool)
    rowsum = np.where(bit, 1, -1).sum(axis=1)
    c3 = np.full((K, M), 3, dtype=np.int8)
    assert np.array_equal(o.int_part_unpacked(bit, c3), np.repeat(3 * rowsum[:, None], M, 1))
    sw, pk = o.pack_bits_rows(bit), o.pack_acts(c3, 2)
    assert np.array_equal(capi.int_packed(sw, pk, K, M, 2), np.repeat(3 * rowsum[:, None], M, 1))
    c0 = np.zeros((K, M), dtype=np.int8)
    assert not capi.int_packed(sw, o.pack_acts(c0, 2), K, M, 2).any()
    cs = np.where(bit[2], 1, -1).astype(np.int8)[:, None].repeat(M, 1)      # x = row 2 of sigma
    D = capi.int_packed(sw, o.pack_acts(cs, 1), K, M, 1)
    assert np.all(D[2] == K)


# ----------------------------------------------------------------------------- decomposition (Eq. 13)
def _case(N, K, M, bits, rho, seed):
    g = np.random.default_rng(seed)
    W = (g.standard_normal((N, K)) * 0.05).astype(np.float32)
    a = np.sort(np.abs(W).ravel())
    delta = np.float32(a[min(a.size - 1, int((1 - rho) * a.size))])
    X = g.standard_normal((K, M)).astype(np.float32)
    if bits == 2:
        X = np.maximum(X, 0)
    return W, delta, X, np.float32(1.0 if bits == 1 else 0.75)


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("N,K,M", [(1, 1, 1), (4, 37, 3), (16, 64, 5), (11, 100, 66), (3, 257, 2)])
def test_forward_equals_dense_definition(N, K, M, bits):
    W, delta, X, step = _case(N, K, M, bits, 0.1, N * 1000 + K + bits)
    L = o.compress(W, delta)
    c = o.quantize(X, bits, step)
    F = o.forward(L, c, step)
    # (i) exact algebra: alpha*sigma + residual, as one dense float64 matrix, times X_hat
    a = np.float64(L["alpha"])
    What = np.where(L["bit"], a, -a)
    for n in range(N):
        for j in range(L["row_ptr"][n], L["row_ptr"][n + 1]):
            What[n, L["col_idx"][j]] += np.float64(L["val"][j])
    xhat = o.dequantize(c, step)
    Y1 = What @ xhat
    mag = np.abs(What) @ np.abs(xhat) + 1e-300
    assert np.max(np.abs(F["Y"].astype(np.float64) - Y1) / mag) < 2.0 ** -23   # one float32 rounding + fp64 noise
    Yd = a * np.float64(step) * F["D"] + F["R"]
    assert np.max(np.abs(Yd - Y1) / mag) < 1e-13
    # (ii) against the definition (Eq. 3 matrix): differs only by the float32 rounding of each residual
    Y2 = o.brute_force(W, delta, L["alpha"], X, bits, step)
    slack = np.zeros((N, M))
    for n in range(N):
        for j in range(L["row_ptr"][n], L["row_ptr"][n + 1]):
            k = L["col_idx"][j]
            slack[n] += np.spacing(np.float32(abs(W[n, k]))) * np.abs(xhat[k])
    assert np.all(np.abs(Yd - Y2) <= slack + 1e-13 * mag)
    # the C loops agree with numpy bit for bit (same order of operations)
    Fc = capi.forward(L, o.pack_acts(c, bits), c, bits, step, threads=2)
    assert np.array_equal(Fc["D"], F["D"]) and np.array_equal(Fc["R"], F["R"]) and np.array_equal(Fc["Y"], F["Y"])


def test_special_cases_reduce_to_textbook_products():
    W, _, X, step = _case(9, 70, 12, 2, 0.1, 5)
    c = o.quantize(X, 2, step)
    xhat = c.astype(np.float64) * 0.75
    # every weight an outlier, alpha = 0: a plain dense product W @ X_hat
    L = o.compress(W, np.float32(-1.0))
    Y = o.forward(L, c, step)["Y"]
    assert np.allclose(Y, W.astype(np.float64) @ xhat, rtol=1e-6, atol=1e-9)
    # no outliers: XNOR-Net style layer alpha * sign(W) @ X_hat
    L = o.compress(W, np.float32(np.inf), alpha=np.float32(0.03))
    Y = o.forward(L, c, step)["Y"]
    want = np.float64(np.float32(0.03)) * (np.where(W >= 0, 1.0, -1.0) @ xhat)
    assert np.allclose(Y, want, rtol=1e-6, atol=1e-9)
    # 1-bit activations, no outliers: alpha * beta * (K - 2 popcount(xor))
    X1 = rng.standard_normal((70, 12)).astype(np.float32)
    c1 = o.quantize(X1, 1, np.float32(0.5))
    Y = o.forward(L, c1, np.float32(0.5))["Y"]
    n, m = 4, 7
    pc = np.count_nonzero((W[n] >= 0) != (X1[:, m] >= 0))
    assert Y[n, m] == np.float32(np.float64(np.float32(0.03)) * 0.5 * (70 - 2 * pc))


def test_additivity_of_the_two_parts():
    W, delta, X, step = _case(8, 90, 10, 2, 0.1, 11)
    c = o.quantize(X, 2, step)
    L = o.compress(W, delta)
    full = o.forward(L, c, step)
    only_bin = dict(L, row_ptr=np.zeros(9, np.int32), col_idx=L["col_idx"][:0], val=L["val"][:0])
    only_sp = dict(L, alpha=np.float32(0.0))
    yb = o.forward(only_bin, c, step)
    ys = o.forward(only_sp, c, step)
    assert not yb["R"].any()
    tot = np.float64(L["alpha"]) * 0.75 * yb["D"] + ys["R"]
    assert np.array_equal(tot.astype(np.float32), full["Y"])


def test_empty_and_full_rows():
    W = (rng.standard_normal((5, 40)) * 0.01).astype(np.float32)
    W[1] = 5.0                                             # a row made of outliers only
    W[3, 7] = -4.0
    X = np.maximum(rng.standard_normal((40, 6)), 0).astype(np.float32)
    L = o.compress(W, np.float32(1.0))
    assert np.diff(L["row_ptr"]).tolist() == [0, 40, 0, 1, 0]
    c = o.quantize(X, 2, np.float32(0.75))
    F = o.forward(L, c, np.float32(0.75))
    Yb = o.brute_force(W, np.float32(1.0), L["alpha"], X, 2, np.float32(0.75))
    assert np.allclose(F["Y"], Yb, rtol=1e-6, atol=1e-7)


# --------------------------------------------------------------------------- the 2/2 routine (Sec. IV "2/2")

def test_2_2_mbm_form_equals_the_direct_sum_for_every_length():
    r = np.random.default_rng(22)
    for n in range(1, 131):
        q = r.integers(0, 4, n)
        p = r.integers(0, 4, n)
        assert o.dot_2_2_mbm_times4(q, p) == int(np.sum((2 * q - 3) * (2 * p - 3)))


def test_2_2_extremes_and_single_levels():
    n = 37
    for q0, p0 in [(3, 3), (0, 3), (3, 0), (2, 2), (1, 2), (2, 0), (1, 1)]:
        q = np.full(n, q0)
        p = np.full(n, p0)
        assert o.dot_2_2_mbm_times4(q, p) == n * (2 * q0 - 3) * (2 * p0 - 3)


def test_2_2_printed_formula_without_level_weights_is_not_the_product():
    # one element, both vectors at +3/2: the product is 9/4, the four unweighted mbm terms add up to 1
    q = np.array([3])
    p = np.array([3])
    tw, hw, mw = o.T_transform(q)
    ta, ha, ma = o.T_transform(p)
    unweighted = (o.mbm(tw, ta, mw & ma) + o.mbm(tw, ha, mw & ~ma) + o.mbm(hw, ta, ~mw & ma)
                  + o.mbm(hw, ha, ~mw & ~ma))
    assert unweighted == 1
    assert o.dot_2_2_mbm_times4(q, p) == 9


def test_2_2_zero_centring_term_and_integer_form():
    # w . a = w_bar . a_bar + (3/2) * sum(w_bar)  (activations a = p*s are not zero-centred), hence
    # D22 = sum (2q-3) p = ( 4*(w_bar . a_bar) + 3 * sum(2q-3) ) / 2
    r = np.random.default_rng(23)
    q = r.integers(0, 4, (6, 75)).astype(np.uint8)
    p = r.integers(0, 4, (75, 5)).astype(np.int8)
    D = o.int_2_2_unpacked(q, p)
    for n in range(6):
        for m in range(5):
            t4 = o.dot_2_2_mbm_times4(q[n], p[:, m])
            assert 2 * int(D[n, m]) == t4 + 3 * int(np.sum(2 * q[n].astype(int) - 3))


def test_2_2_packed_equals_unpacked_with_ragged_k():
    r = np.random.default_rng(24)
    for N, K, M in [(3, 1, 2), (4, 33, 5), (5, 64, 3), (2, 97, 66)]:
        W = (r.standard_normal((N, K)) * 0.1).astype(np.float32)
        X = np.maximum(r.standard_normal((K, M)), 0).astype(np.float32)
        q = o.quantize_weights_2bit(W, np.float32(0.07))
        c = o.quantize(X, 2, np.float32(0.75))
        D = o.int_2_2_packed(o.pack_weight_planes(q), o.pack_acts(c, 2), K, M)
        assert np.array_equal(D, o.int_2_2_unpacked(q, c))


def test_2_2_with_half_levels_only_is_the_1_2_integer_part():
    # weights restricted to -1/2, +1/2 (q = 1, 2) are a +-1 vector scaled by 1/2: D22 must equal the
    # integer part of the binary layer with the same signs
    r = np.random.default_rng(25)
    bit = r.integers(0, 2, (7, 90)).astype(bool)
    p = r.integers(0, 4, (90, 11)).astype(np.int8)
    assert np.array_equal(o.int_2_2_unpacked(1 + bit.astype(np.uint8), p), o.int_part_unpacked(bit, p))


def test_2_2_weight_quantizer_levels_and_boundaries():
    s = np.float32(0.5)
    w = np.array([0.0, -0.0, 0.49, 0.5, 0.99, 1.0, 7.0, -1e-30, -0.5, -0.51, -1.0, -1.01, -9.0, np.nan, np.inf, -np.inf],
                 dtype=np.float32)
    assert o.quantize_weights_2bit(w, s).tolist() == [2, 2, 2, 3, 3, 3, 3, 1, 1, 0, 0, 0, 0, 0, 3, 0]
    # the dequantized weight is the midpoint of the cell the weight falls in
    r = np.random.default_rng(26)
    w = (r.uniform(-0.999, 0.999, 1000)).astype(np.float32)
    q = o.quantize_weights_2bit(w, s).astype(np.float64)
    assert np.all(np.abs((q - 1.5) * 0.5 - w) <= 0.25 + 1e-7)


def test_2_2_gemm_matches_the_plain_definition():
    r = np.random.default_rng(27)
    W = (r.standard_normal((9, 130)) * 0.1).astype(np.float32)
    X = np.maximum(r.standard_normal((130, 17)), 0).astype(np.float32)
    sw, sa = np.float32(0.08), np.float32(0.75)
    G = o.gemm_2_2(o.quantize_weights_2bit(W, sw), o.quantize(X, 2, sa), sw, sa)
    Yb = o.brute_force_2_2(W, sw, X, sa)
    assert np.allclose(G["Y"], Yb, rtol=1e-6, atol=1e-9)
    assert np.abs(G["D"]).max() <= 3 * 3 * 130


# --------------------------------------------------------------------------- two layers in a row
def test_forward_requant_on_exactly_representable_values():
    """Weights +-1/4 with a few outliers at multiples of 1/2, activations p/2: every Y is a multiple
    of 1/8, so Z and the level index are exact and can be written down with Python's fractions
    (round() on a Fraction rounds halves to even, as the quantizer must)."""
    from fractions import Fraction as Fr
    r = np.random.default_rng(77)
    N, K, M = 7, 45, 9
    W = np.where(r.random((N, K)) < 0.5, 0.25, -0.25).astype(np.float32)
    for (n, k, v) in [(0, 3, 1.5), (0, 44, -2.0), (2, 0, 2.5), (6, 17, -1.5), (6, 18, 3.0)]:
        W[n, k] = v
    p_in = r.integers(0, 4, (K, M))
    X = (p_in * 0.5).astype(np.float32)
    L = o.compress(W, np.float32(0.25), alpha=np.float32(0.25))
    assert np.diff(L["row_ptr"]).tolist() == [2, 0, 1, 0, 0, 0, 2]
    c = o.quantize(X, 2, np.float32(0.5))
    assert np.array_equal(c, p_in)
    scale = np.array([1, 0.5, 2, 1, -1, 0.25, 1], dtype=np.float32)
    shift = np.array([0, 0.25, -1, 0.125, 3, 0, -0.5], dtype=np.float32)
    for sc, sh in ((None, None), (scale, shift)):
        for bits_out, step_out in ((2, 1.0), (2, 0.25), (1, 1.0)):
            got = o.forward_requant(L, c, np.float32(0.5), bits_out, np.float32(step_out), sc, sh)
            want = np.zeros((N, M), dtype=np.int64)
            for n in range(N):
                for m in range(M):
                    y = sum(Fr(float(W[n, k])) * Fr(int(p_in[k, m]), 2) for k in range(K))
                    z = y if sc is None else Fr(float(sc[n])) * y + Fr(float(sh[n]))
                    assert float(got["Z"][n, m]) == float(z)
                    want[n, m] = (1 if z >= 0 else -1) if bits_out == 1 else min(3, max(0, round(z / Fr(step_out))))
            assert np.array_equal(got["c"], want)
            assert np.array_equal(got["packed"], o.pack_acts(want.astype(np.int8), bits_out))
    # ties really occur in this case (otherwise the rounding rule would go untested)
    Z = o.forward_requant(L, c, np.float32(0.5), 2, np.float32(0.25))["Z"].astype(np.float64)
    assert np.any(np.abs(Z / 0.25 - np.floor(Z / 0.25) - 0.5) == 0.0)


def test_two_layer_chain_equals_the_dense_definition():
    """forward_requant of layer 1 feeding forward of layer 2 == APB(W2) @ dequantize(quantize(APB(W1) @ X^))."""
    W1, d1, X, step = _case(12, 70, 10, 2, 0.1, 901)
    W2, d2, _, _ = _case(5, 12, 10, 2, 0.1, 902)
    L1, L2 = o.compress(W1, d1), o.compress(W2, d2)
    c1 = o.quantize(X, 2, step)
    s2 = np.float32(0.05)
    hop = o.forward_requant(L1, c1, step, 2, s2)
    Y2 = o.forward(L2, hop["c"], s2)["Y"]
    Y1 = o.brute_force(W1, d1, L1["alpha"], X, 2, step)                 # float64, the definition
    lvl = Y1.astype(np.float32).astype(np.float64) / np.float64(s2)
    assert np.min(np.abs(lvl - np.floor(lvl) - 0.5)) > 1e-4            # no near-tie: the codes are unambiguous
    c2 = np.clip(np.rint(lvl), 0, 3)
    assert np.array_equal(hop["c"], c2)
    want = o.apb_dense(W2, d2, L2["alpha"]) @ (c2 * np.float64(s2))
    assert np.allclose(Y2, want, rtol=1e-6, atol=1e-9)


# --------------------------------------------------------------------------- convolution as a product
@pytest.mark.parametrize("bits", [1, 2])
def test_im2col_forward_is_the_direct_convolution(bits):
    """forward on im2col_codes == the textbook 3x3 cross-correlation (scipy) of the dequantized map with
    the reconstructed weights, padded with the value of code 0."""
    from scipy.signal import correlate2d
    r = np.random.default_rng(31 + bits)
    N, C, B, H, W = 3, 4, 2, 5, 6
    Wt = (r.standard_normal((N, 9 * C)) * 0.05).astype(np.float32)
    delta = np.float32(0.08)
    step = np.float32(0.75 if bits == 2 else 0.5)
    Xmap = r.standard_normal((C, B * H * W)).astype(np.float32)
    if bits == 2:
        Xmap = np.maximum(Xmap, 0)
    L = o.compress(Wt, delta)
    assert 0 < int(L["row_ptr"][-1]) < N * 9 * C
    c_map = o.quantize(Xmap, bits, step)
    patches = o.im2col_codes(c_map, B, H, W, bits)
    assert patches.shape == (9 * C, B * H * W)
    assert np.array_equal(patches[4 * C:5 * C], c_map)                  # the centre tap is the map itself
    Y = o.forward(L, patches, step)["Y"].reshape(N, B, H, W)
    dense = o.apb_dense(Wt, delta, L["alpha"]).reshape(N, 3, 3, C)      # [n][ky][kx][c]
    xhat = o.dequantize(c_map, step).reshape(C, B, H, W)
    fill = 0.0 if bits == 2 else -float(step)
    for n in range(N):
        for b_ in range(B):
            want = sum(correlate2d(xhat[ch, b_], dense[n, :, :, ch], mode="same", boundary="fill", fillvalue=fill)
                       for ch in range(C))
            assert np.allclose(Y[n, b_], want, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("bits", [1, 2])
@pytest.mark.parametrize("stride,H,W", [(2, 5, 6), (2, 6, 7), (2, 1, 1), (3, 7, 5)])
def test_strided_im2col_is_the_subsampled_direct_convolution(bits, stride, H, W):
    """With a stride the product on im2col_codes is the textbook cross-correlation (scipy, full resolution,
    padded with the value of code 0) read at every stride-th row and column; its centre tap is the map
    subsampled the same way, and stride 1 is the unstrided matrix."""
    from scipy.signal import correlate2d
    r = np.random.default_rng(57 + 10 * bits + stride + H)
    N, C, B = 3, 4, 2
    Wt = (r.standard_normal((N, 9 * C)) * 0.05).astype(np.float32)
    delta = np.float32(0.08)
    step = np.float32(0.75 if bits == 2 else 0.5)
    Xmap = r.standard_normal((C, B * H * W)).astype(np.float32)
    if bits == 2:
        Xmap = np.maximum(Xmap, 0)
    L = o.compress(Wt, delta)
    c_map = o.quantize(Xmap, bits, step)
    Ho, Wo = o.conv_out_size(H, stride), o.conv_out_size(W, stride)
    assert (Ho, Wo) == (len(range(0, H, stride)), len(range(0, W, stride)))
    patches = o.im2col_codes(c_map, B, H, W, bits, stride)
    assert patches.shape == (9 * C, B * Ho * Wo)
    assert np.array_equal(o.im2col_codes(c_map, B, H, W, bits, 1), o.im2col_codes(c_map, B, H, W, bits))
    centre = c_map.reshape(C, B, H, W)[:, :, ::stride, ::stride].reshape(C, B * Ho * Wo)
    assert np.array_equal(patches[4 * C:5 * C], centre)
    Y = o.forward(L, patches, step)["Y"].reshape(N, B, Ho, Wo)
    dense = o.apb_dense(Wt, delta, L["alpha"]).reshape(N, 3, 3, C)
    xhat = o.dequantize(c_map, step).reshape(C, B, H, W)
    fill = 0.0 if bits == 2 else -float(step)
    for n in range(N):
        for b_ in range(B):
            full = sum(correlate2d(xhat[ch, b_], dense[n, :, :, ch], mode="same", boundary="fill", fillvalue=fill)
                       for ch in range(C))
            assert np.allclose(Y[n, b_], full[::stride, ::stride], rtol=1e-6, atol=1e-9)
