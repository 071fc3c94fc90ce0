"""Helpers shared by the tests: the error metric and bit comparisons."""
import numpy as np

TOL = 1e-6   # the fp32 bar: per-layer max-normalised error


def layer_error(a: np.ndarray, b: np.ndarray, offsets) -> float:
    """max over layers l of  max_e |a_e - b_e| / max(max_e |b_e|, tiny)  with a, b of shape
    [n, pitch] and the layer l occupying columns offsets[l]:offsets[l+1] of every row."""
    worst = 0.0
    a64 = a.astype(np.float64)
    b64 = b.astype(np.float64)
    for l in range(len(offsets) - 1):
        lo, hi = int(offsets[l]), int(offsets[l + 1])
        if hi <= lo:
            continue
        num = np.max(np.abs(a64[:, lo:hi] - b64[:, lo:hi]))
        den = max(np.max(np.abs(b64[:, lo:hi])), 1e-30)
        worst = max(worst, float(num / den))
    return worst


def bit_mismatches(a: np.ndarray, b: np.ndarray) -> int:
    assert a.dtype == b.dtype and a.shape == b.shape
    u = {4: np.uint32, 2: np.uint16, 8: np.uint64}[a.dtype.itemsize]
    return int(np.count_nonzero(np.ascontiguousarray(a).view(u) != np.ascontiguousarray(b).view(u)))
