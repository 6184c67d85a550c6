"""Stochastic verification of a draft chunk: speculative sampling.  TEST INFRASTRUCTURE ONLY.

The paper verifies drafts against the LLM's distributions q(x | prefix), ..., q(x | prefix, x_1..x_k) under
"top-1 (greedy), top-k, or top-p" sampling and sends the SLM's distributions p in compressed form
(Section 4.2, "Compression before transmission"; Section 4.5), but it does not write the acceptance rule
down; it cites the speculative-decoding work for it.  The rule taken here is the one that work publishes
(speculative sampling), stated for one request:

  for j = 1 .. k:   accept draft x_j with probability min(1, q_j(x_j) / p_j(x_j));
                    at the first rejection emit a token drawn from norm(max(0, q_j - p_j)) and stop;
  if all k drafts are accepted, emit one more token drawn from q_{k+1}.

Its point: whatever p is, the emitted tokens are distributed exactly as if drawn from q.

Readings: p_j is the distribution the device really sampled from, i.e. its transmitted top-k list
renormalised to sum 1 (tokens outside the list have probability 0; a draft that is not in its own list is
rejected).  q_j is the plain softmax of the LLM's logits row.  Every random decision consumes a uniform
number in [0, 1) that the caller passes in: u_accept[j] for draft j, u_sample for the emitted token, which
is found by inverting the cumulative sums of the target distribution in token-id order:
the smallest v with c_v > u_sample * c_last (c = inclusive cumulative sums).
"""
import numpy as np


def inverse_cdf(weights, u):
    """Token drawn from the (unnormalised, non-negative) weights with the uniform number u in [0, 1):
    the smallest index v whose inclusive cumulative sum exceeds u * total.  Also returns how close the
    target came to a cumulative boundary, relative to the total (for tolerance decisions in tests)."""
    w = np.asarray(weights, np.float64)
    c = np.cumsum(w)
    target = u * c[-1]
    v = int(np.searchsorted(c, target, side="right"))
    v = min(v, len(w) - 1)
    while w[v] == 0.0 and v + 1 < len(w):            # never emit a token of zero weight
        v += 1
    gap = float(np.min(np.abs(c - target))) / float(c[-1])
    return v, gap


def compressed_to_dense(ids, probs, vocab):
    """The distribution a top-k list stands for: its probabilities renormalised to 1, 0 elsewhere."""
    p = np.zeros(vocab, np.float64)
    pr = np.asarray(probs, np.float64)
    p[np.asarray(ids, np.int64)] = pr / pr.sum()
    return p


def speculative_accept(q_rows, p_lists, drafts, u_accept, u_sample):
    """q_rows [k+1][V]: LLM probabilities at the k draft positions and after the last draft.
    p_lists: per draft (ids, probs), the compressed SLM distribution it was sampled from.
    Returns (n accepted, emitted token, info) with info = {"ratio_gap": smallest |u - ratio| over the
    decisions taken, "cdf_gap": closeness of the emitted token's draw to a cumulative boundary}."""
    k = len(drafts)
    V = q_rows.shape[1]
    ratio_gap = np.inf
    for j in range(k):
        x = int(drafts[j])
        p = compressed_to_dense(p_lists[j][0], p_lists[j][1], V)
        q = np.asarray(q_rows[j], np.float64)
        ratio = min(1.0, q[x] / p[x]) if p[x] > 0.0 else 0.0
        ratio_gap = min(ratio_gap, abs(u_accept[j] - ratio))
        if u_accept[j] < ratio:
            continue
        token, gap = inverse_cdf(np.maximum(q - p, 0.0), u_sample)
        return j, token, {"ratio_gap": ratio_gap, "cdf_gap": gap}
    token, gap = inverse_cdf(np.asarray(q_rows[k], np.float64), u_sample)
    return k, token, {"ratio_gap": ratio_gap, "cdf_gap": gap}
