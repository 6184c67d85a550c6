"""Pins for the importance score of the oracle (Section 3.2: column-wise sum of the attention matrix)."""
import math

import numpy as np

import oracle
import workloads as wl
import gpu_harness as gh

SHAPE = wl.ModelShape("mini", 2, 128, 4, 2, 64, 256, 256)


def _model(seed=9):
    return gh.draw_weights(SHAPE, seed, "cpu")["model"]


def _kv(n_pages=16):
    return oracle.PagedKV(SHAPE.n_layers, n_pages, SHAPE.n_kv_heads, SHAPE.head_dim)


def test_column_sums_of_a_hand_made_attention_matrix():
    P = np.zeros((2, 2, 3))
    P[0] = [[0.25, 0.75, 0.0], [0.5, 0.25, 0.25]]
    P[1] = [[1.0, 0.0, 0.0], [0.0, 0.0, 1.0]]
    # head 0 columns: 0.75, 1.0, 0.25; head 1: 1, 0, 1; mean over heads
    assert np.allclose(oracle.importance_from_attention(P), [0.875, 0.5, 0.625])


def test_scores_of_a_request_sum_to_its_number_of_chunk_tokens_and_respect_causality():
    model, kv = _model(), _kv()
    rng = np.random.default_rng(0)
    row = np.arange(16, dtype=np.int32)
    oracle.forward_tokens(model, kv, [(row[:8], 0, rng.integers(0, 256, 37))])
    items = [(row[:8], 37, rng.integers(0, 256, 9)), (row[8:], 0, rng.integers(0, 256, 5))]
    for layer in (0, 1, None):
        kv2 = oracle.PagedKV(SHAPE.n_layers, 16, SHAPE.n_kv_heads, SHAPE.head_dim)
        kv2.k[:], kv2.v[:] = kv.k, kv.v
        I = oracle.importance_scores(model, kv2, items, layer)
        assert [len(x) for x in I] == [46, 5]
        assert abs(I[0].sum() - 9) < 1e-9 and abs(I[1].sum() - 5) < 1e-9
        assert (I[0] >= 0).all()
        # the last key is visible to the last row only: its score is at most 1 and it is that row's weight
        assert 0 < I[0][-1] <= 1.0 and 0 < I[1][-1] <= 1.0
        assert abs(I[1][0] - 1.0) > 1e-6 and I[1][0] >= 1.0       # key 0: all of row 0's weight, plus more


def test_uniform_attention_gives_the_harmonic_closed_form():
    """With W_q = 0 every score is 0, so row r spreads 1 / (L + r + 1) over its visible keys:
    I_j = sum over rows r with L + r >= j of 1 / (L + r + 1)."""
    model, kv = _model(), _kv()
    for l in range(SHAPE.n_layers):
        model.layer(l)["wq"][:] = 0
    L, n = 21, 6
    row = np.arange(16, dtype=np.int32)
    rng = np.random.default_rng(1)
    oracle.forward_tokens(model, kv, [(row, 0, rng.integers(0, 256, L))])
    I = oracle.importance_scores(model, kv, [(row, L, rng.integers(0, 256, n))])[0]
    want = [sum(1.0 / (L + r + 1) for r in range(n) if L + r >= j) for j in range(L + n)]
    assert np.allclose(I, want, rtol=0, atol=1e-12)


def test_first_layer_matrix_recomputed_literally():
    """Layer 0 depends on nothing but the embeddings: recompute q, the scores against the cached keys and
    the softmax row by row with plain loops, and compare the column sums."""
    model, kv = _model(3), _kv()
    rng = np.random.default_rng(2)
    row = np.arange(16, dtype=np.int32)
    ctx, chunk = rng.integers(0, 256, 19), rng.integers(0, 256, 4)
    oracle.forward_tokens(model, kv, [(row, 0, ctx)])
    I = oracle.importance_scores(model, kv, [(row, 19, chunk)], layer=0)[0]
    w = model.layer(0)
    Hq, Hkv, h = SHAPE.n_q_heads, SHAPE.n_kv_heads, SHAPE.head_dim
    K, _ = kv.gather(0, row, 19 + 4)                         # bf16 cache contents, positions 0..22
    want = np.zeros(23)
    for r, tok in enumerate(chunk):
        x = np.asarray(model.embed[tok], np.float64)
        y = x / math.sqrt(float(np.mean(x * x)) + model.rms_eps) * np.asarray(w["attn_norm"], np.float64)
        q = oracle.rope((np.asarray(w["wq"], np.float64) @ y).reshape(Hq, h), 19 + r, model.rope_base)
        for hq in range(Hq):
            s = [float(np.dot(q[hq], np.asarray(K[j, hq // (Hq // Hkv)], np.float64))) / math.sqrt(h) for j in range(19 + r + 1)]
            z = sum(math.exp(v - max(s)) for v in s)
            for j, v in enumerate(s):
                want[j] += math.exp(v - max(s)) / z / Hq
    assert np.allclose(I, want, rtol=0, atol=1e-9)


def test_mean_over_the_draft_positions():
    I = np.arange(10, dtype=np.float64)
    assert oracle.mean_draft_importance(I, ctx_len=5, n_uncached=1, n_draft=3) == (6 + 7 + 8) / 3
