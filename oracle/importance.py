"""Importance score (Section 3.2): the column-wise sum of the attention matrix
softmax(Q K^T / sqrt(d_k)).  TEST INFRASTRUCTURE ONLY.

For a request that forwards n chunk tokens at positions L .. L+n-1, the attention matrix of one head has
one row per chunk token and one column per key position 0 .. L+n-1 (row r sees keys 0 .. L+r).  The
score of key j is the sum over the rows of column j.

What the paper leaves open, and the reading taken here: it names neither the layer nor how heads are
combined.  The scores are those of the LAST decoder layer, averaged over the query heads (so that each
chunk token hands out a total weight of 1, and the scores of a request sum to n).  The mean score "across
draft tokens" that feeds P_imp (Section 4.2, second equation; oracle.dispatch.p_imp) is the mean of the
scores of the k draft positions L+u .. L+u+k-1.
"""
import numpy as np

from .decoder import forward_tokens


def importance_from_attention(P):
    """P [heads, rows, keys] -> scores [keys]: column sums over the rows, mean over the heads."""
    return np.asarray(P).sum(axis=1).mean(axis=0)


def importance_scores(model, kv, items, layer=None):
    """Forward `items` (as oracle.forward_tokens: the K/V of the chunk tokens are appended) and return, per
    item, the importance scores of its key positions 0 .. start+n-1 from `layer` (default: the last)."""
    layer = model.n_layers - 1 if layer is None else layer
    probe = (layer, [])
    forward_tokens(model, kv, items, attn_probe=probe)
    return [importance_from_attention(P) for P in probe[1]]


def mean_draft_importance(scores, ctx_len, n_uncached, n_draft):
    """Mean score of the request's draft positions."""
    a = ctx_len + n_uncached
    return float(np.mean(scores[a:a + n_draft]))
