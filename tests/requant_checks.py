"""Shared checks for packed outputs written by the re-quantizing forward entry points (not a test module)."""
import numpy as np

from oracle import apb_oracle as o

REL_TOL = 1e-5


def unpack(words: np.ndarray, K: int, M: int, bits: int):
    """codes [K, M] and colsum [Mp] out of a packed buffer; asserts that the padding is zero."""
    Kw, Mp = (K + 31) // 32, 64 * ((M + 63) // 64)
    assert words.size == Mp * (bits * Kw + 1)
    planes = words[: bits * Kw * Mp].reshape(bits, Kw, Mp)
    colsum = words[bits * Kw * Mp:].view(np.int32)
    assert not planes[:, :, M:].any() and not colsum[M:].any()
    code = np.zeros((Kw * 32, M), dtype=np.int32)
    for pl in range(bits):
        for i in range(32):
            code[i::32] += (((planes[pl, :, :M] >> np.uint32(i)) & 1) << pl).astype(np.int32)
    assert not code[K:].any()
    return code[:K], colsum


def compare_codes(code, ref, alpha, step, D, R, bits_out, step_out, scale, shift) -> int:
    """Codes read back from the GPU against the oracle's (`ref` = oracle.requant(...)): equal, except where
    the oracle's Z lies within the float tolerance (relative to the magnitude of the two parts that were
    added) of a decision boundary of the quantizer; such near-ties must be rare and off by one level.
    Returns the number of differing codes."""
    want = o.codes_of(ref["c"], bits_out).astype(np.int32)
    diff = code != want
    if diff.any():
        a_s = np.float64(np.float32(alpha)) * np.float64(np.float32(step))
        mag = np.abs(a_s * D) + np.abs(R)
        if scale is not None:
            mag = np.abs(scale.astype(np.float64))[:, None] * mag + np.abs(shift.astype(np.float64))[:, None]
        Z = ref["Z"].astype(np.float64)
        if bits_out == 1:
            dist = np.abs(Z)
        else:
            lvl = Z / np.float64(np.float32(step_out))
            dist = np.abs(lvl - np.floor(lvl) - 0.5) * np.float64(np.float32(step_out))
        assert np.all(dist[diff] <= REL_TOL * mag[diff]), f"{int(diff.sum())} codes differ away from any boundary"
        assert np.abs(code - want)[diff].max() == 1
        assert diff.mean() < 1e-3
    return int(diff.sum())
