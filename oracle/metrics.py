"""Error measures used when a low-precision result is compared with the fp64 reference
(test infrastructure only)."""
import numpy as np


def max_abs(x, ref):
    return float(np.max(np.abs(np.asarray(x, dtype=np.float64) - np.asarray(ref, dtype=np.float64))))


def rel_l2(x, ref):
    x = np.asarray(x, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm((x - ref).ravel()) / np.linalg.norm(ref.ravel()))


def mean_signed(x, ref):
    """Mean of (x - ref): the signed-error statistic of Sec. 3.3.2 (a systematic bias shows
    as a mean far outside its sampling noise)."""
    return float(np.mean(np.asarray(x, dtype=np.float64) - np.asarray(ref, dtype=np.float64)))


def mean_signed_noise(x, ref):
    """Standard error of mean_signed under independent errors: std(err)/sqrt(n)."""
    e = (np.asarray(x, dtype=np.float64) - np.asarray(ref, dtype=np.float64)).ravel()
    return float(np.std(e) / np.sqrt(e.size))
