"""TEST INFRASTRUCTURE - not part of the product path.

Plain statement of the paper's analytical latency model (App. A): the regressors of the prefill and
decoding phase times and their least-squares fit, in fp64 numpy.  Only tests may import this module.

  prefill (App. A.2):   T = C1 (4 t h^2 + 2 t h m) + C2 (3 h t2 / b) + C3
  decoding (App. A.3):  T = C4 (4 h^2 + 2 h m) + C5 (3 h t)

with t = sum of lengths, t2 = sum of squared lengths, b the attention block size.  For decoding the
"lengths" are the context lengths of the requests in the batch.
"""
import numpy as np


def prefill_regressors(lens, h, m, b):
    """One row [4 t h^2 + 2 t h m, 3 h t2 / b, 1] for a batch with the given prompt lengths."""
    t = 0.0
    t2 = 0.0
    for l in lens:
        t += float(l)
        t2 += float(l) * float(l)
    return np.array([4.0 * t * h * h + 2.0 * t * h * m, 3.0 * h * t2 / b, 1.0], dtype=np.float64)


def decode_regressors(ctx_lens, h, m):
    """One row [4 h^2 + 2 h m, 3 h t] for a decoding batch with the given context lengths."""
    t = 0.0
    for l in ctx_lens:
        t += float(l)
    return np.array([4.0 * h * h + 2.0 * h * m, 3.0 * h * t], dtype=np.float64)


def fit(rows, times):
    """Ordinary least squares: the coefficient vector minimising |rows @ c - times|_2."""
    a = np.asarray(rows, dtype=np.float64)
    y = np.asarray(times, dtype=np.float64)
    c, *_ = np.linalg.lstsq(a, y, rcond=None)
    return c


def predict(rows, c):
    return np.asarray(rows, dtype=np.float64) @ np.asarray(c, dtype=np.float64)
