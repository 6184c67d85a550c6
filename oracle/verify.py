"""Greedy verification of offloaded draft chunks (CPU oracle).

After the engine's forward pass, verification uses the LLM's distributions
q(x | prefix), q(x | prefix, d_0), ..., q(x | prefix, d_0..d_{k-1}): k+1
distributions for k drafts (Section 4.5; Section 4.2 "Compression before
transmission" lists the matching SLM side).  The paper leaves the acceptance
formula to the sampling method in use; the benchmark spec fixes top-1 (greedy):
a draft is accepted while it equals the LLM's greedy token at its position, and
the LLM's greedy token at the first mismatch (or after the last draft) is the
correction.

q(x | prefix) is not produced by forwarding the drafts alone.  When a request
carries uncached device-accepted tokens (Section 3.4) it is the row of the last
of them; when it carries none, the caller supplies it as `anchor` (the LLM's
greedy token after the cached context, known from the prefill or from the
previous verification's correction).
"""
import numpy as np

from .confidence import confidence
from .decoder import forward_tokens, lm_head


def accept_prefix(drafts, greedy):
    """drafts d_0..d_{k-1}; greedy a_0..a_k with a_j the LLM's greedy token at the
    position of draft j (a_k follows the last draft).  Returns (n, a_n) where n is
    the length of the longest prefix with d_j == a_j."""
    n = 0
    while n < len(drafts) and int(drafts[n]) == int(greedy[n]):
        n += 1
    return n, int(greedy[n])


def verify_chunks(model, kv, requests):
    """One flattened partial prefill plus verification.

    requests: list of dicts with block_table (row), ctx_len, uncached (token ids,
    may be empty), drafts (token ids, >= 1), anchor (used iff no uncached tokens).
    Returns per-draft-row arrays in flattened request order (logits[R,V], argmax,
    top1_prob, entropy, margin) and per-request accept_len, correction and
    first_margin (top-2 margin of the row that supplies q(x|prefix), inf when the
    anchor is given).
    """
    items = [(r["block_table"], int(r["ctx_len"]),
              np.concatenate([np.asarray(r["uncached"], np.int64), np.asarray(r["drafts"], np.int64)]))
             for r in requests]
    x = forward_tokens(model, kv, items)
    rows, first_rows = [], []
    r0 = 0
    for r in requests:
        u, k = len(r["uncached"]), len(r["drafts"])
        first_rows.append(r0 + u - 1 if u > 0 else -1)
        rows.extend(range(r0 + u, r0 + u + k))
        r0 += u + k
    logits = lm_head(model, x[rows])
    ids, p1, H, mg = confidence(logits, model.dtype)
    accept, corr, first_margin = [], [], []
    at = 0
    for r, fr in zip(requests, first_rows):
        k = len(r["drafts"])
        if fr >= 0:
            a0, _, _, m0 = confidence(lm_head(model, x[fr:fr + 1]), model.dtype)
            a0, m0 = int(a0[0]), float(m0[0])
        else:
            a0, m0 = int(r["anchor"]), float("inf")
        n, c = accept_prefix(r["drafts"], [a0] + [int(t) for t in ids[at:at + k]])
        accept.append(n)
        corr.append(c)
        first_margin.append(m0)
        at += k
    return {"logits": logits, "argmax": ids, "top1_prob": p1, "entropy": H, "margin": mg,
            "accept_len": np.asarray(accept, np.int32), "correction": np.asarray(corr, np.int32),
            "first_margin": np.asarray(first_margin)}


def prefill_context(model, kv, block_table_row, tokens):
    """Fill the cache by forwarding `tokens` from an empty cache; returns the LLM's
    greedy token after them (the anchor of the next verification)."""
    x = forward_tokens(model, kv, [(block_table_row, 0, tokens)])
    return int(np.argmax(lm_head(model, x[-1])))


def draft_chain(model, kv, requests, p_match, u, tok):
    """Draw draft chunks the way an SLM that agrees with the LLM with probability
    p_match would produce them, by sequential single-token decoding.

    requests: list of dicts with block_table, ctx_len, n_draft, anchor.  u[i][j]
    is a uniform in [0,1) and tok[i][j] a random token for request i, position j.
    Draft j is the LLM's greedy token a_j given the context and drafts 0..j-1 when
    u < p_match, else tok.  Forwarding draft j (appending its K/V) yields the row
    that defines a_{j+1}.  Returns (drafts per request, logits rows per request
    [k_i, V]) - the rows are, by construction, what a verification of these
    drafts must reproduce.
    """
    B = len(requests)
    greedy = [int(r["anchor"]) for r in requests]
    drafts = [[] for _ in range(B)]
    rows = [[] for _ in range(B)]
    for j in range(max(int(r["n_draft"]) for r in requests)):
        live = [i for i in range(B) if int(requests[i]["n_draft"]) > j]
        items = []
        for i in live:
            d = greedy[i] if u[i][j] < p_match else int(tok[i][j])
            drafts[i].append(d)
            items.append((requests[i]["block_table"], int(requests[i]["ctx_len"]) + j, [d]))
        logits = lm_head(model, forward_tokens(model, kv, items))
        for n, i in enumerate(live):
            rows[i].append(logits[n])
            greedy[i] = int(np.argmax(logits[n]))
    return ([np.asarray(d, np.int32) for d in drafts], [np.stack(r) for r in rows])
