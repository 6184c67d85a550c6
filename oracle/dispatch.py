"""Selective-offloading statistics that ride on the vocabulary pass (the paper's device-side decision
inputs and the compressed distribution a device sends with a chunk):

* top-k entries of a token's softmax distribution, the compressed form transmitted instead of the full
  vector ("Compression before transmission", Section 4.2), and the top-p (nucleus) cut over the full
  vocabulary;
* the margin score, top-1 minus top-2 probability (layer-wise early exit, Section 4.3);
* the mean confidence of a chunk and the dispatch probability P_conf(c), a scaled sigmoid above a
  threshold c_th and 1 at or below it (first equation of Section 4.2);
* P_imp(i), the three-tier dispatch probability of an importance score (second equation of Section 4.2).

Everything is written the naive way (materialise the probability vector, sort it).
"""
import math

import numpy as np


def softmax_probs(x, dtype=np.float64):
    x = np.asarray(x, dtype=dtype)
    e = np.exp(x - x.max())
    return e / e.sum(dtype=dtype)


def topk_row(x, k, dtype=np.float64):
    """One row of logits -> (ids[k], probs[k]) of the k most probable tokens, most probable first;
    equal logits go by the lower token id first."""
    x = np.asarray(x, dtype=dtype)
    p = softmax_probs(x, dtype)
    order = sorted(range(x.size), key=lambda j: (-x[j], j))[:k]
    return np.array(order, np.int32), p[order]


def margin_row(x, dtype=np.float64):
    """Margin score: top-1 probability minus top-2 probability (0 if the two largest logits tie)."""
    _, p = topk_row(x, 2, dtype)
    return float(p[0] - p[1]) if p.size > 1 else float(p[0])


def topk(logits, k, dtype=np.float64):
    """Rows of logits -> (ids int32[R][k], probs[R][k], margin[R])."""
    logits = np.asarray(logits)
    R = logits.shape[0]
    ids = np.empty((R, k), np.int32)
    pr = np.empty((R, k), np.float64)
    mg = np.empty(R, np.float64)
    for r in range(R):
        ids[r], pr[r] = topk_row(logits[r], k, dtype)
        mg[r] = pr[r, 0] - pr[r, 1] if k > 1 else margin_row(logits[r], dtype)   # the margin is p1 - p2 whatever k is
    return ids, pr, mg


def topp_count(probs_desc, top_p, dtype=np.float32):
    """Top-p (nucleus) truncation of a distribution whose entries are given most probable first: the
    smallest n with probs_desc[0] + ... + probs_desc[n-1] >= top_p, and that sum.  If the given entries
    do not reach top_p (the list is itself a truncation, e.g. the top-k window a device transmits) all of
    them are kept.  The running sum is taken in `dtype`, in list order: the decision is an integer, so the
    precision is part of the definition (float32, as the transmitted probabilities are)."""
    acc = dtype(0.0)
    n = 0
    for v in probs_desc:
        acc = dtype(acc + dtype(v))
        n += 1
        if acc >= dtype(top_p):
            break
    return n, float(acc)


def nucleus_row(x, top_p, dtype=np.float64):
    """Full-vocabulary top-p (nucleus) truncation of one row of logits (Section 4.2 lists top-p beside top-1
    and top-k as the sampling methods whose lists are transmitted; the standard definition is taken): sort the
    softmax probabilities, most probable first (equal logits by the lower id), and keep the smallest prefix
    whose sum reaches top_p.  Returns (n, mass of the n kept, cut logit = the smallest logit kept,
    gap = how close the running sum passes to top_p at the two candidates for the cut: an integer decision
    taken within `gap` of a tie is not unique to rounding)."""
    x = np.asarray(x, dtype=dtype)
    p = softmax_probs(x, dtype)
    order = sorted(range(x.size), key=lambda j: (-x[j], j))
    cum = np.cumsum(p[order], dtype=dtype)
    n = int(np.searchsorted(cum, dtype(top_p), side="left")) + 1
    n = min(n, x.size)                       # rounding may leave the total a hair under top_p = 1
    near = [abs(float(cum[n - 1]) - top_p)] + ([abs(float(cum[n - 2]) - top_p)] if n > 1 else [])
    return n, float(cum[n - 1]), float(x[order[n - 1]]), min(near)


def p_conf(c, c_th, k=10.0):
    """Dispatch probability of a chunk whose mean confidence is c (Section 4.2, first equation):
    1 for c <= c_th, else 1 / (1 + exp(k * norm(c))) with norm(c) = (c - c_th) / (1 - c_th) - 1/2."""
    if c <= c_th:
        return 1.0
    norm = (c - c_th) / (1.0 - c_th) - 0.5
    return 1.0 / (1.0 + math.exp(k * norm))


def p_imp(i, i_th, theta=-10.0):
    """Dispatch probability of an importance score i (Section 4.2, second equation): 0 up to i_th / 2,
    1 above i_th, a sigmoid with slope theta < 0 of norm(i) = (i - i_th/2) / (i_th/2) - 1/2 between."""
    if i <= i_th / 2.0:
        return 0.0
    if i > i_th:
        return 1.0
    norm = (i - i_th / 2.0) / (i_th / 2.0) - 0.5
    return 1.0 / (1.0 + math.exp(theta * norm))


def chunk_dispatch(top1_prob, cu_rows, c_th, k=10.0):
    """Rows grouped into chunks by prefix sums cu_rows[B+1] -> (mean confidence[B], P_conf[B]).
    The confidence of a token is its top-1 probability (Section 3.2); c is its mean over the chunk's
    draft tokens.  An empty chunk has mean confidence 0 and is dispatched (P_conf = 1)."""
    top1_prob = np.asarray(top1_prob, np.float64)
    B = len(cu_rows) - 1
    mean = np.zeros(B)
    pc = np.ones(B)
    for b in range(B):
        seg = top1_prob[cu_rows[b]:cu_rows[b + 1]]
        if seg.size:
            mean[b] = seg.sum() / seg.size
        pc[b] = p_conf(mean[b], c_th, k)
    return mean, pc
