"""Per-token confidence statistics over the vocabulary.

The confidence score of a token is the top-1 probability of the softmax over the
vocabulary (Section 3.2, "Offloading Decision Metrics").  The benchmark spec adds
the Shannon entropy (nats, temperature 1) of the same distribution.  Both are
written the naive way: materialise the probability vector, then read it.
"""
import numpy as np


def confidence_row(x, dtype=np.float64):
    """One row of logits -> (argmax id, top-1 probability, entropy, top-2 logit margin).

    Ties in the maximum go to the lowest token id.
    """
    x = np.asarray(x, dtype=dtype)
    idx = int(np.argmax(x))                 # first occurrence == lowest id
    m = x[idx]
    e = np.exp(x - m)
    p = e / e.sum(dtype=dtype)
    nz = p > 0
    H = -(p[nz] * np.log(p[nz])).sum(dtype=dtype)
    if x.size > 1:
        rest = np.delete(x, idx)
        margin = float(m - rest.max())
    else:
        margin = float("inf")
    return idx, float(p[idx]), float(H), margin


def confidence(logits, dtype=np.float64):
    """Rows of logits -> (ids int32[R], top1 prob[R], entropy[R], margin[R])."""
    logits = np.asarray(logits)
    R = logits.shape[0]
    ids = np.empty(R, np.int32)
    p1 = np.empty(R, np.float64)
    H = np.empty(R, np.float64)
    mg = np.empty(R, np.float64)
    for r in range(R):
        ids[r], p1[r], H[r], mg[r] = confidence_row(logits[r], dtype)
    return ids, p1, H, mg
