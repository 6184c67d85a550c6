"""Pins of the CPU oracle against what the method and the mathematics fix.

The paper prints no worked numeric example for the verify path, so the pins are
invariants of partial prefill (Section 3.4), the attention definition
(Section 3.2), the k+1-distribution structure of verification (Section 4.5),
closed forms, brute force on tiny inputs, and a second, independently written
dense decoder (torch float64, no cache, complex-number rotary, library softmax).
"""
import cmath
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import drawn_model, oracle_model, small_shape, to_np

F64 = np.float64


# --------------------------------------------------------------------------- numerics
def test_bf16_round_matches_torch_and_ties_to_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(size=4000), rng.normal(size=2000) * 1e-3,
                        rng.normal(size=2000) * 1e4]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.bf16_round(x), want)
    # exact ties: 1 + 2^-8 is halfway between 1 and 1+2^-7 -> even mantissa (1.0)
    assert oracle.bf16_round(np.float32(1.0 + 2.0 ** -8)) == np.float32(1.0)
    assert oracle.bf16_round(np.float32(1.0 + 3 * 2.0 ** -8)) == np.float32(1.0 + 2.0 ** -6)
    b = oracle.bf16_bits(np.float32([1.0, -2.0, 0.0]))
    assert list(b) == [0x3F80, 0xC000, 0x0000]
    assert np.array_equal(oracle.bf16_from_bits(b), np.float32([1.0, -2.0, 0.0]))


# --------------------------------------------------------------------------- confidence
def test_confidence_closed_forms():
    V = 37
    idx, p, H, mg = oracle.confidence_row(np.full(V, 2.5))
    assert idx == 0 and mg == 0.0                       # tie -> lowest id
    assert p == pytest.approx(1.0 / V, rel=1e-14)
    assert H == pytest.approx(math.log(V), rel=1e-14)
    # one entry raised by D over a constant row
    D, at = 3.0, 11
    x = np.full(V, -1.25)
    x[at] += D
    idx, p, H, mg = oracle.confidence_row(x)
    Z = math.exp(D) + V - 1
    p1, po = math.exp(D) / Z, 1.0 / Z
    assert idx == at and mg == pytest.approx(D)
    assert p == pytest.approx(p1, rel=1e-14)
    assert H == pytest.approx(-(p1 * math.log(p1) + (V - 1) * po * math.log(po)), rel=1e-13)
    # dominant entry: p -> 1, H -> 0; underflowed probabilities are skipped, not NaN
    x = np.zeros(V)
    x[5] = 800.0
    idx, p, H, _ = oracle.confidence_row(x)
    assert idx == 5 and p == 1.0 and H == 0.0


def test_confidence_bruteforce_and_shift_invariance():
    rng = np.random.default_rng(1)
    for V in (2, 3, 17, 64):
        x = rng.normal(size=V) * 3
        idx, p, H, mg = oracle.confidence_row(x)
        es = [math.exp(v) for v in x]
        Z = math.fsum(es)
        ps = [e / Z for e in es]
        best = max(range(V), key=lambda i: (x[i], -i))
        assert idx == best
        assert p == pytest.approx(ps[best], rel=1e-13)
        assert H == pytest.approx(-math.fsum(q * math.log(q) for q in ps), rel=1e-12)
        srt = sorted(x)
        assert mg == pytest.approx(srt[-1] - srt[-2], rel=1e-13)
        # identity the fused GPU reduction uses: H = ln Z' - S/Z' with Z' = sum e^(x-m), S = sum e^(x-m)(x-m)
        m = max(x)
        Zp = math.fsum(math.exp(v - m) for v in x)
        S = math.fsum(math.exp(v - m) * (v - m) for v in x)
        assert H == pytest.approx(math.log(Zp) - S / Zp, rel=1e-12)
        idx2, p2, H2, _ = oracle.confidence_row(x + 123.0)
        assert idx2 == idx and p2 == pytest.approx(p, rel=1e-12) and H2 == pytest.approx(H, rel=1e-11)
    ids, p, H, mg = oracle.confidence(np.array([[0.0, 1.0, 1.0], [5.0, 5.0, 1.0]]))
    assert list(ids) == [1, 0] and mg[0] == 0.0 and mg[1] == 0.0


# --------------------------------------------------------------------------- accept rule
def _accept_independent(d, a):
    """Second formulation: count of leading ones in the match vector."""
    match = (np.asarray(d) == np.asarray(a[:len(d)])).astype(np.int64)
    n = int(np.cumprod(match).sum())
    return n, int(a[n])


def test_accept_prefix_bruteforce_and_properties():
    rng = np.random.default_rng(2)
    for _ in range(2000):
        k = int(rng.integers(1, 17))
        a = rng.integers(0, 4, size=k + 1)
        d = rng.integers(0, 4, size=k)
        assert oracle.accept_prefix(d, a) == _accept_independent(d, a)
    a = [7, 8, 9, 10]
    assert oracle.accept_prefix([7, 8, 9], a) == (3, 10)          # all accepted -> bonus token
    assert oracle.accept_prefix([0, 8, 9], a) == (0, 7)           # first wrong -> anchor is the correction
    assert oracle.accept_prefix([7, 0, 9], a) == (1, 8)           # later matches do not count
    assert oracle.accept_prefix([7, 8, 0], a) == (2, 9)


# --------------------------------------------------------------------------- building blocks
def test_rmsnorm_closed_forms():
    g = np.linspace(0.5, 1.5, 8)
    y = oracle.rmsnorm(np.full(8, 3.0), g, 1e-5)
    assert np.allclose(y, 3.0 / math.sqrt(9.0 + 1e-5) * g, rtol=1e-15)
    x = np.random.default_rng(3).normal(size=8)
    y1, y2 = oracle.rmsnorm(x, g, 0.0), oracle.rmsnorm(5.0 * x, g, 0.0)
    assert np.allclose(y1, y2, rtol=1e-14)                         # scale invariant at eps = 0
    assert np.mean((y1 / g) ** 2) == pytest.approx(1.0, rel=1e-14)
    want = x / math.sqrt(sum(v * v for v in x) / 8 + 0.25) * g
    assert np.allclose(oracle.rmsnorm(x, g, 0.25), want, rtol=1e-14)


def test_rope_against_complex_rotation_and_properties():
    rng = np.random.default_rng(4)
    h = 16
    v = rng.normal(size=(3, h))
    assert np.array_equal(oracle.rope(v, 0), v)                    # position 0 is the identity
    for pos in (1, 17, 4095):
        r = oracle.rope(v, pos, base=10000.0)
        for row in range(3):
            for i in range(h // 2):
                z = complex(v[row, 2 * i], v[row, 2 * i + 1]) * cmath.exp(1j * pos * 10000.0 ** (-2.0 * i / h))
                assert r[row, 2 * i] == pytest.approx(z.real, rel=1e-12, abs=1e-12)
                assert r[row, 2 * i + 1] == pytest.approx(z.imag, rel=1e-12, abs=1e-12)
        assert np.allclose(np.linalg.norm(r, axis=1), np.linalg.norm(v, axis=1), rtol=1e-13)
    q, k = rng.normal(size=h), rng.normal(size=h)
    d1 = oracle.rope(q, 40) @ oracle.rope(k, 33)
    d2 = oracle.rope(q, 107) @ oracle.rope(k, 100)
    assert d1 == pytest.approx(d2, rel=1e-11)                      # depends on the offset only


def test_attention_special_cases_and_dense_bruteforce():
    rng = np.random.default_rng(5)
    Hq, Hkv, h, n = 4, 2, 8, 9
    q = rng.normal(size=(Hq, h))
    K = rng.normal(size=(n, Hkv, h))
    V = rng.normal(size=(n, Hkv, h))
    o = oracle.attention_one_query(q, K[:1], V[:1])                # single key -> o = v
    for hq in range(Hq):
        assert np.allclose(o[hq], V[0, hq // 2], rtol=1e-14)
    Keq = np.repeat(K[:1], n, axis=0)                              # equal keys -> mean of v
    o = oracle.attention_one_query(q, Keq, V)
    for hq in range(Hq):
        assert np.allclose(o[hq], V[:, hq // 2].mean(axis=0), rtol=1e-13)
    o = oracle.attention_one_query(q, K, V)                        # brute force, python floats
    for hq in range(Hq):
        kh = hq // (Hq // Hkv)
        s = [sum(q[hq, c] * K[t, kh, c] for c in range(h)) / math.sqrt(h) for t in range(n)]
        Z = math.fsum(math.exp(v) for v in s)
        for c in range(h):
            want = math.fsum(math.exp(s[t]) / Z * V[t, kh, c] for t in range(n))
            assert o[hq, c] == pytest.approx(want, rel=1e-12, abs=1e-13)
    # G = 1: grouped attention is plain multi-head attention
    K4, V4 = rng.normal(size=(n, Hq, h)), rng.normal(size=(n, Hq, h))
    o = oracle.attention_one_query(q, K4, V4)
    for hq in range(Hq):
        s = K4[:, hq] @ q[hq] / math.sqrt(h)
        p = np.exp(s) / np.exp(s).sum()
        assert np.allclose(o[hq], p @ V4[:, hq], rtol=1e-12)


def test_paged_kv_layout_and_sparse_pool():
    kv = oracle.PagedKV(n_layers=2, n_pages=6, n_kv_heads=2, head_dim=4)
    bt = [4, 2, 5]
    k = np.arange(8, dtype=np.float32).reshape(2, 4) + 1
    v = -(np.arange(8, dtype=np.float32).reshape(2, 4) + 1)
    kv.append(1, bt, 19, k, v)                                     # page bt[1] = 2, slot 3
    assert np.array_equal(oracle.bf16_from_bits(kv.k[1, 2, :, 3, :]), k)
    assert np.array_equal(oracle.bf16_from_bits(kv.v[1, 2, :, :, 3]), v)
    assert kv.k.sum() == oracle.bf16_bits(k).astype(np.int64).sum()      # nothing else written
    assert kv.k[0].sum() == 0
    K, V = kv.gather(1, bt, 20)
    assert np.array_equal(K[19], k) and np.array_equal(V[19], v) and not K[:19].any()
    kv.append(0, bt, 0, np.float32([[1.00390625] * 4] * 2), v)     # 1 + 2^-8 rounds to even -> 1.0
    assert np.all(oracle.bf16_from_bits(kv.k[0, 4, :, 0, :]) == 1.0)
    with pytest.raises(IndexError):
        kv.append(0, [9], 0, k, v)
    sp = oracle.PagedKV(2, 6, 2, 4, pages=[5, 2, 4])
    sp.append(1, bt, 19, k, v)
    K2, V2 = sp.gather(1, bt, 20)
    assert np.array_equal(K, K2) and np.array_equal(V, V2)


# --------------------------------------------------------------------------- second derivation
def _dense_decoder_torch(shape, head, layers, tokens):
    """Independent dense float64 decoder: whole sequence at once, no cache, complex
    rotary, library softmax; K and V pass through torch's bf16 (the cache format)."""
    t64 = lambda w: w.to(torch.float64)                                     # noqa: E731
    S, Hq, Hkv, h = len(tokens), shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    x = t64(head["embed"])[torch.as_tensor(tokens, dtype=torch.long)]
    pos = torch.arange(S, dtype=torch.float64)
    freqs = shape.rope_base ** (-torch.arange(0, h, 2, dtype=torch.float64) / h)
    rot = torch.polar(torch.ones(S, h // 2, dtype=torch.float64), pos[:, None] * freqs[None, :])

    def rotary(z):                                                 # z [S, H, h]
        zc = torch.view_as_complex(z.reshape(S, -1, h // 2, 2).contiguous())
        return torch.view_as_real(zc * rot[:, None, :]).reshape(S, -1, h)

    def norm(z, g):
        return z * torch.rsqrt(z.pow(2).mean(-1, keepdim=True) + shape.rms_eps) * t64(g)

    mask = torch.full((S, S), float("-inf"), dtype=torch.float64).triu(1)
    for w in layers:
        y = norm(x, w["attn_norm"])
        q = rotary((y @ t64(w["wq"]).T).view(S, Hq, h))
        k = rotary((y @ t64(w["wk"]).T).view(S, Hkv, h)).to(torch.bfloat16).to(torch.float64)
        v = (y @ t64(w["wv"]).T).view(S, Hkv, h).to(torch.bfloat16).to(torch.float64)
        k = k.repeat_interleave(Hq // Hkv, dim=1)
        v = v.repeat_interleave(Hq // Hkv, dim=1)
        s = torch.einsum("shc,thc->hst", q, k) / math.sqrt(h) + mask
        o = torch.einsum("hst,thc->shc", torch.softmax(s, dim=-1), v).reshape(S, Hq * h)
        x = x + o @ t64(w["wo"]).T
        y = norm(x, w["mlp_norm"])
        x = x + (torch.nn.functional.silu(y @ t64(w["w_gate"]).T) * (y @ t64(w["w_up"]).T)) @ t64(w["w_down"]).T
    return (norm(x, head["final_norm"]) @ t64(head["lm_head"]).T).numpy()


@pytest.mark.parametrize("shape", [small_shape(), wl.CONFIGS[1].shape], ids=["mini_gqa", "c1_shape"])
def test_chunk_mode_equals_independent_dense_decoder(shape):
    head, layers = drawn_model(shape, 77)
    m = oracle_model(shape, head, layers, F64)
    rng = np.random.default_rng(6)
    toks = rng.integers(0, shape.vocab, size=41)
    kv = oracle.PagedKV(shape.n_layers, 5, shape.n_kv_heads, shape.head_dim)
    bt = [3, 0, 4]
    x = oracle.forward_tokens(m, kv, [(bt, 0, toks)])
    got = oracle.lm_head(m, x)
    want = _dense_decoder_torch(shape, head, layers, toks)
    assert np.abs(got - want).max() < 1e-9
    assert np.array_equal(got.argmax(1), want.argmax(1))


# --------------------------------------------------------------------------- invariants of partial prefill
def _mini():
    shape = small_shape()
    head, layers = drawn_model(shape, 5)
    return shape, oracle_model(shape, head, layers, F64)


def test_chunked_equals_sequential_equals_full_prefill():
    shape, m = _mini()
    rng = np.random.default_rng(7)
    L, k = 21, 6
    ctx, chunk = rng.integers(0, shape.vocab, L), rng.integers(0, shape.vocab, k)
    bt = [2, 5, 1]
    new = lambda: oracle.PagedKV(shape.n_layers, 6, shape.n_kv_heads, shape.head_dim)   # noqa: E731
    # sequential: one token at a time by the literal definition
    kv_a = new()
    xs = [oracle.decode_token(m, kv_a, bt, t, int(tok)) for t, tok in enumerate(np.concatenate([ctx, chunk]))]
    seq = oracle.lm_head(m, np.stack(xs[L:]))
    # partial prefill: cache the context, then the k-token chunk in one pass
    kv_b = new()
    oracle.forward_tokens(m, kv_b, [(bt, 0, ctx)])
    par = oracle.lm_head(m, oracle.forward_tokens(m, kv_b, [(bt, L, chunk)]))
    # full prefill from an empty cache
    kv_c = new()
    full = oracle.lm_head(m, oracle.forward_tokens(m, kv_c, [(bt, 0, np.concatenate([ctx, chunk]))]))[L:]
    assert np.abs(seq - par).max() < 1e-11 and np.abs(full - par).max() < 1e-11
    assert np.array_equal(seq.argmax(1), par.argmax(1))
    assert np.array_equal(kv_a.k, kv_b.k) and np.array_equal(kv_a.v, kv_b.v)
    assert np.array_equal(kv_a.k, kv_c.k) and np.array_equal(kv_a.v, kv_c.v)


def _requests(shape, rng, B, pages_per_req=3):
    reqs = []
    for i in range(B):
        reqs.append({"ctx": rng.integers(0, shape.vocab, int(rng.integers(5, 30))),
                     "drafts": rng.integers(0, shape.vocab, int(rng.integers(1, 9))),
                     "uncached": np.zeros(0, np.int64)})
    return reqs


def _run_batch(shape, m, reqs, bts, n_pages, order=None):
    kv = oracle.PagedKV(shape.n_layers, n_pages, shape.n_kv_heads, shape.head_dim)
    order = range(len(reqs)) if order is None else order
    batch = []
    for i in order:
        anchor = oracle.prefill_context(m, kv, bts[i], reqs[i]["ctx"])
        batch.append({"block_table": bts[i], "ctx_len": len(reqs[i]["ctx"]), "uncached": reqs[i]["uncached"],
                      "drafts": reqs[i]["drafts"], "anchor": anchor})
    return oracle.verify_chunks(m, kv, batch), kv, batch


def test_paging_and_batch_invariance():
    shape, m = _mini()
    rng = np.random.default_rng(8)
    reqs = _requests(shape, rng, 4)
    bts = [list(range(3 * i, 3 * i + 3)) for i in range(4)]
    base, kv0, _ = _run_batch(shape, m, reqs, bts, 12)
    perm = rng.permutation(20)
    bts_p = [[int(perm[p]) for p in bt] for bt in bts]
    moved, kv1, _ = _run_batch(shape, m, reqs, bts_p, 20)
    for key in ("logits", "argmax", "top1_prob", "entropy", "accept_len", "correction"):
        assert np.array_equal(base[key], moved[key]), key          # bit-identical under page relabelling
    for p in range(12):
        assert np.array_equal(kv0.k[:, p], kv1.k[:, perm[p]]) and np.array_equal(kv0.v[:, p], kv1.v[:, perm[p]])
    # a request's outputs do not depend on its batch mates or its place in the batch
    solo, _, _ = _run_batch(shape, m, reqs, bts, 12, order=[2])
    k_before = sum(len(r["drafts"]) for r in reqs[:2])
    k2 = len(reqs[2]["drafts"])
    assert np.abs(solo["logits"] - base["logits"][k_before:k_before + k2]).max() < 1e-11
    assert solo["accept_len"][0] == base["accept_len"][2] and solo["correction"][0] == base["correction"][2]
    rev, _, _ = _run_batch(shape, m, reqs, bts, 12, order=[3, 2, 1, 0])
    assert list(rev["accept_len"]) == list(base["accept_len"][::-1])
    assert list(rev["correction"]) == list(base["correction"][::-1])


def test_uncached_tokens_supply_the_first_distribution():
    """With u >= 1 uncached accepted tokens the row of the last of them replaces the
    anchor; moving tokens between 'cached' and 'uncached' must not change the result."""
    shape, m = _mini()
    rng = np.random.default_rng(9)
    ctx = rng.integers(0, shape.vocab, 19)
    drafts = rng.integers(0, shape.vocab, 5)
    bt = [1, 0, 2]
    kv = oracle.PagedKV(shape.n_layers, 3, shape.n_kv_heads, shape.head_dim)
    anchor = oracle.prefill_context(m, kv, bt, ctx)
    drafts[0] = anchor                                             # make at least one accept
    a = oracle.verify_chunks(m, kv, [{"block_table": bt, "ctx_len": 19, "uncached": [], "drafts": drafts,
                                      "anchor": anchor}])
    kv2 = oracle.PagedKV(shape.n_layers, 3, shape.n_kv_heads, shape.head_dim)
    oracle.prefill_context(m, kv2, bt, ctx[:15])
    b = oracle.verify_chunks(m, kv2, [{"block_table": bt, "ctx_len": 15, "uncached": ctx[15:], "drafts": drafts,
                                       "anchor": -1}])
    assert np.abs(a["logits"] - b["logits"]).max() < 1e-11
    assert a["accept_len"][0] == b["accept_len"][0] >= 1 and a["correction"][0] == b["correction"][0]
    assert np.isfinite(b["first_margin"][0]) and np.isinf(a["first_margin"][0])


def test_verify_reproduces_draft_chain_and_accept_semantics():
    shape, m = _mini()
    rng = np.random.default_rng(10)
    B = 6
    reqs = _requests(shape, rng, B)
    bts = [list(range(3 * i, 3 * i + 3)) for i in range(B)]
    kv = oracle.PagedKV(shape.n_layers, 3 * B, shape.n_kv_heads, shape.head_dim)
    batch = [{"block_table": bts[i], "ctx_len": len(r["ctx"]), "n_draft": len(r["drafts"]),
              "anchor": oracle.prefill_context(m, kv, bts[i], r["ctx"])} for i, r in enumerate(reqs)]
    for p, expect in ((1.0, "all"), (0.0, "none")):
        u = rng.random((B, 32))
        tok = rng.integers(0, shape.vocab, (B, 32))
        drafts, rows = oracle.draft_chain(m, kv, batch, p, u, tok)
        ver = oracle.verify_chunks(m, kv, [dict(b, uncached=[], drafts=d) for b, d in zip(batch, drafts)])
        assert np.abs(ver["logits"] - np.concatenate(rows)).max() < 1e-11   # k-token verify == k decodes
        for i in range(B):
            k = len(drafts[i])
            if expect == "all":
                assert ver["accept_len"][i] == k
                assert ver["correction"][i] == rows[i][-1].argmax()         # bonus token
            else:
                want = oracle.accept_prefix(drafts[i], [batch[i]["anchor"]] + list(np.argmax(rows[i], axis=1)))
                assert (ver["accept_len"][i], ver["correction"][i]) == want
                if drafts[i][0] != batch[i]["anchor"]:
                    assert ver["accept_len"][i] == 0 and ver["correction"][i] == batch[i]["anchor"]


def test_expected_accept_length_is_capped_geometric():
    """Under per-token match probability p and chunk length k the accepted length has
    mean sum_{m=1..k} p^m (cf. the capped geometric of Section 4.4 / Section 5)."""
    shape, m = _mini()
    rng = np.random.default_rng(11)
    B, k, p = 400, 5, 0.7
    bt = [0, 1]
    kv = oracle.PagedKV(shape.n_layers, 2, shape.n_kv_heads, shape.head_dim)
    anchor = oracle.prefill_context(m, kv, bt, rng.integers(0, shape.vocab, 9))
    total = 0
    for b in range(B):                                             # same context, fresh random numbers
        u, tok = rng.random((1, 32)), rng.integers(0, shape.vocab, (1, 32))
        req = [{"block_table": bt, "ctx_len": 9, "n_draft": k, "anchor": anchor}]
        drafts, rows = oracle.draft_chain(m, kv, req, p, u, tok)
        n, _ = oracle.accept_prefix(drafts[0], [anchor] + list(np.argmax(rows[0], axis=1)))
        total += n
    mean = total / B
    want = sum(p ** j for j in range(1, k + 1)) + (1 - p) / shape.vocab   # random token may match by chance
    assert abs(mean - want) < 4 * 1.5 / math.sqrt(B)


def test_float32_mode_tracks_float64():
    shape = wl.CONFIGS[1].shape
    head, layers = drawn_model(shape, 3)
    rng = np.random.default_rng(12)
    toks = rng.integers(0, shape.vocab, 24)
    outs = []
    for dt in (np.float64, np.float32):
        m = oracle_model(shape, head, layers, dt)
        kv = oracle.PagedKV(shape.n_layers, 2, shape.n_kv_heads, shape.head_dim)
        outs.append(oracle.lm_head(m, oracle.forward_tokens(m, kv, [([0, 1], 0, toks)])))
    assert outs[1].dtype == np.float32
    assert np.abs(outs[0] - outs[1]).max() < 2e-3          # bf16 rounding of K/V can differ by one ulp


def test_append_many_equals_single_appends():
    rng = np.random.default_rng(13)
    bt = [3, 0, 2, 1]
    K, V = rng.normal(size=(41, 2, 4)), rng.normal(size=(41, 2, 4))
    a = oracle.PagedKV(1, 4, 2, 4)
    b = oracle.PagedKV(1, 4, 2, 4)
    for t in range(41):
        a.append(0, bt, 5 + t, K[t], V[t])
    b.append_many(0, bt, 5, K, V)
    assert np.array_equal(a.k, b.k) and np.array_equal(a.v, b.v)
