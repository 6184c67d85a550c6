"""Builds a verify workload on the GPU, runs the HIP path, and compares it with the CPU oracle.

Per request the oracle either takes part (a *sampled* request: the oracle computes its
context K/V at the last context position, its anchor, its draft chain and the
expected rows) or not (its drafts come from the HIP path's own greedy chain and only
size-independent properties are checked).  Inputs of sampled requests never come from
the HIP path.  KV pools start filled with bf16 NaN so that any read of a slot that was
never written (a masking or page-indexing mistake) poisons the outputs.
"""
import math
import time
from dataclasses import dataclass, field

import numpy as np
import torch

import oracle
import paper_2511_07423_amd as synera
import workloads as wl
import progress
from helpers import oracle_model, to_np

LOGIT_TOL = 2e-2          # max |delta| on logits (task statement)
MARGIN = 1e-2             # ids exact unless the oracle's top-2 margin is below this
ENTROPY_RTOL = 1e-3
NAN_BITS = 0x7FC0


@dataclass
class Case:
    recipe: object
    shape: object
    device: str
    batch: dict
    head: dict
    layers: list
    verifier: object
    k_pool: torch.Tensor
    v_pool: torch.Tensor
    sampled: list
    model: object = None
    okv: object = None
    anchor: np.ndarray = None            # int32 [B]: input to verify
    drafts: list = None                  # per request int32 arrays
    want_rows: dict = field(default_factory=dict)   # sampled request -> oracle logits [k, V]
    n_uncached: np.ndarray = None
    timing: dict = field(default_factory=dict)


def nan_pool(shape, n_pages, device, transposed):
    dims = (shape.n_layers, n_pages, shape.n_kv_heads, shape.head_dim, wl.PAGE_SIZE) if transposed else \
           (shape.n_layers, n_pages, shape.n_kv_heads, wl.PAGE_SIZE, shape.head_dim)
    t = torch.empty(dims, dtype=torch.int16, device=device)
    t.fill_(NAN_BITS)
    return t.view(torch.bfloat16)


def pick_sample(batch, n):
    """Requests the oracle follows: extremes of context length and chunk length first."""
    B = len(batch["ctx_len"])
    if n >= B:
        return list(range(B))
    L, k = batch["ctx_len"], batch["n_draft"]
    order = [int(np.argmin(L)), int(np.argmax(L)), int(np.argmin(k)), int(np.argmax(k))]
    rng = np.random.default_rng(12345)
    order += [int(i) for i in rng.permutation(B)]
    out = []
    for i in order:
        if i not in out:
            out.append(i)
        if len(out) == n:
            break
    return sorted(out)


def _oracle_pool_to_device(okv, device):
    k = torch.from_numpy(okv.k.view(np.int16)).to(device).view(torch.bfloat16)
    v = torch.from_numpy(okv.v.view(np.int16)).to(device).view(torch.bfloat16)
    return k, v


def gpu_chain(case, reqs, anchors):
    """Drafts for `reqs` from the HIP path's own greedy tokens: draft j is the current greedy
    token with probability p_match, else a random token; the chunk so far is re-verified to
    get the next greedy token."""
    rec, b = case.recipe, case.batch
    rnd = wl.draw_draft_randoms(rec, len(b["ctx_len"]))
    drafts = {i: [] for i in reqs}
    greedy = {i: int(anchors[i]) for i in reqs}
    dev = case.device
    for j in range(int(max(b["n_draft"][i] for i in reqs))):
        live = [i for i in reqs if b["n_draft"][i] > j]
        for i in live:
            drafts[i].append(greedy[i] if rnd["u"][i][j] < rec.p_match else int(rnd["tok"][i][j]))
        toks = torch.tensor([t for i in live for t in drafts[i]], dtype=torch.int32, device=dev)
        out = case.verifier.verify(
            b["ctx_len"][live], np.zeros(len(live), np.int32), np.full(len(live), j + 1, np.int32), toks,
            torch.tensor([int(anchors[i]) for i in live], dtype=torch.int32, device=dev),
            b["block_table"][live], b["n_pages"], case.k_pool, case.v_pool, want_logits=False)
        am = out["argmax"].cpu().numpy()
        for n, i in enumerate(live):
            greedy[i] = int(am[(n + 1) * (j + 1) - 1])
    return {i: np.asarray(d, np.int32) for i, d in drafts.items()}


def draw_weights(shape, seed, device, oracle_dtype=None, lazy_oracle=False):
    """Weights on the device plus the oracle's widened host copy of the same bytes.  Tests of several
    configs with one model shape may share the result.  lazy_oracle: the oracle widens one layer at a
    time from the device copy (for models whose fp32 copy does not fit in host memory)."""
    if oracle_dtype is None:
        # float64, the exact arithmetic of the definition: a float32 run of the oracle is no arbiter for a deep
        # decoder (bf16 KV-cache rounding decisions flip and attention carries them on; measured at the 70B
        # shape with all 80 layers, float32 run vs float64 run: 4e-3 to 1e-1 depending on the requests looked at)
        oracle_dtype = np.float64
    head = wl.draw_head_weights(shape, seed, device)
    layers = [wl.draw_layer_weights(shape, seed, l, device) for l in range(shape.n_layers)]
    src = (lambda l: layers[l]) if lazy_oracle else layers
    return {"head": head, "layers": layers, "model": oracle_model(shape, head, src, oracle_dtype)}


def build_case(recipe, device="cuda:0", n_oracle=None, batch_size=None, oracle_dtype=None, verbose=False,
               weights=None):
    shape = recipe.shape
    t0 = time.time()
    say = (lambda *a: progress.say("[case]", *a, f"(+{time.time() - t0:.1f}s)")) if verbose else (lambda *a: None)
    b = wl.draw_batch(recipe, batch_size)
    B = len(b["ctx_len"])
    rnd = wl.draw_draft_randoms(recipe, B)
    if weights is None:
        weights = draw_weights(shape, recipe.seed, device, oracle_dtype)
    head, layers = weights["head"], weights["layers"]
    say("weights drawn")
    k_pool = nan_pool(shape, b["n_pages"], device, False)
    v_pool = nan_pool(shape, b["n_pages"], device, True)
    ver = synera.Verifier(shape, head, layers, max_batch=B, max_tokens=int(b["n_draft"].sum()) + B,
                          max_pages=b["max_pages"])
    sampled = pick_sample(b, B if n_oracle is None else n_oracle)
    model = weights["model"]
    pages = [p for i in sampled for p in b["block_table"][i] if p >= 0]
    okv = oracle.PagedKV(shape.n_layers, b["n_pages"], shape.n_kv_heads, shape.head_dim,
                         pages=None if len(sampled) == B and shape.d_model <= 512 else pages)
    case = Case(recipe, shape, device, b, head, layers, ver, k_pool, v_pool, sampled, model, okv)
    case.n_uncached = np.zeros(B, np.int32)
    anchors = np.zeros(B, np.int32)
    L = b["ctx_len"]

    if recipe.real_prefill:
        # cached context = a real prefill of random ids by the oracle; the GPU pools start from those bytes
        assert len(sampled) == B and okv.slot_of is None
        ctx = wl.draw_context_tokens(recipe, L)
        for i in range(B):
            anchors[i] = oracle.prefill_context(model, okv, b["block_table"][i], ctx[i])
        kd, vd = _oracle_pool_to_device(okv, device)
        for i in range(B):                       # copy exactly the cached positions 0..L-1
            for t0 in range(0, int(L[i]), wl.PAGE_SIZE):
                page, m = int(b["block_table"][i][t0 // wl.PAGE_SIZE]), min(wl.PAGE_SIZE, int(L[i]) - t0)
                k_pool[:, page, :, :m, :] = kd[:, page, :, :m, :]
                v_pool[:, page, :, :, :m] = vd[:, page, :, :, :m]
    else:
        # stand-in context: N(0,1) K/V rows at positions 0..L-2, then a true decode of a random token
        # at position L-1 (each side computes its own), which also yields the anchor
        n_fill = (L - 1).astype(np.int32)
        starts = np.concatenate([[0], np.cumsum(n_fill)])
        zeros = np.zeros(B, np.int32)
        for l in range(shape.n_layers):
            kr, vr = wl.draw_context_kv(shape, recipe.seed, l, int(n_fill.sum()), device)
            ver.kv_append(l, zeros, n_fill, kr, vr, b["block_table"], b["n_pages"], k_pool, v_pool)
            for i in sampled:
                sl = slice(int(starts[i]), int(starts[i + 1]))
                okv.append_many(l, b["block_table"][i], 0, to_np(kr[sl]), to_np(vr[sl]))
            torch.cuda.synchronize()
        say("context K/V filled")
        last = torch.from_numpy(rnd["last_ctx_tok"]).to(device)
        out = ver.verify(n_fill, zeros, np.ones(B, np.int32), last, torch.zeros(B, dtype=torch.int32, device=device),
                         b["block_table"], b["n_pages"], k_pool, v_pool, want_logits=False)
        anchors[:] = out["argmax"].cpu().numpy()
        items = [(b["block_table"][i], int(L[i]) - 1, [int(rnd["last_ctx_tok"][i])]) for i in sampled]
        lg = oracle.lm_head(model, oracle.forward_tokens(model, okv, items))
        for n, i in enumerate(sampled):
            anchors[i] = int(np.argmax(lg[n]))
        # sampled requests: the GPU cache takes the oracle's K/V at position L-1, so both sides verify
        # against bit-identical caches
        sub = np.asarray(sampled)
        for l in range(shape.n_layers):
            kr = np.stack([oracle.bf16_from_bits(okv.k[l, okv._backing(b["block_table"][i][(L[i] - 1) // 16]), :,
                                                       (L[i] - 1) % 16, :]) for i in sampled])
            vr = np.stack([oracle.bf16_from_bits(okv.v[l, okv._backing(b["block_table"][i][(L[i] - 1) // 16]), :, :,
                                                       (L[i] - 1) % 16]) for i in sampled])
            ver.kv_append(l, n_fill[sub], np.ones(len(sub), np.int32),
                          torch.from_numpy(kr).to(device, torch.bfloat16), torch.from_numpy(vr).to(device, torch.bfloat16),
                          b["block_table"][sub], b["n_pages"], k_pool, v_pool)
        torch.cuda.synchronize()
        say("last context token decoded on both sides")

    reqs = [{"block_table": b["block_table"][i], "ctx_len": int(L[i]), "n_draft": int(b["n_draft"][i]),
             "anchor": int(anchors[i])} for i in sampled]
    t1 = time.time()
    plain_layers, passes = model._layers, [0]

    def layer_and_say(l):                     # one line per pass of the oracle over the decoder
        if l == 0:
            passes[0] += 1
            say(f"oracle draft chain: forward pass {passes[0]}")
        return plain_layers(l) if callable(plain_layers) else plain_layers[l]
    model._layers = layer_and_say
    try:
        dr, rows = oracle.draft_chain(model, okv, reqs, recipe.p_match, rnd["u"][sampled], rnd["tok"][sampled])
    finally:
        model._layers = plain_layers
    case.timing["oracle_chain_s"] = time.time() - t1
    say("oracle draft chain done")
    drafts = [None] * B
    for n, i in enumerate(sampled):
        drafts[i] = dr[n]
        case.want_rows[i] = rows[n]
    rest = [i for i in range(B) if i not in sampled]
    if rest:
        for i, d in gpu_chain(case, rest, anchors).items():
            drafts[i] = d
        say("HIP-path chain for the other requests done")
    case.anchor, case.drafts = anchors, drafts
    return case


def run_verify(case, want_logits=True):
    b = case.batch
    dev = case.device
    toks = torch.from_numpy(np.concatenate(case.drafts).astype(np.int32)).to(dev)
    anchor = torch.from_numpy(case.anchor.astype(np.int32)).to(dev)
    out = case.verifier.verify(b["ctx_len"], case.n_uncached, b["n_draft"], toks, anchor, b["block_table"],
                               b["n_pages"], case.k_pool, case.v_pool, want_logits=want_logits)
    torch.cuda.synchronize()
    return {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}


def compare_with_oracle(case, out, logit_tol=LOGIT_TOL):
    """Element-wise comparison on the sampled requests plus size-independent properties on all."""
    b, shape = case.batch, case.shape
    B = len(b["ctx_len"])
    k = b["n_draft"]
    cu = np.concatenate([[0], np.cumsum(k)])
    rep = {"ok": True, "fail": [], "max_logit_err": 0.0, "max_entropy_rel": 0.0, "max_prob_rel": 0.0,
           "exempt_rows": 0, "exempt_requests": 0, "rows_checked": 0, "requests_checked": 0}

    def fail(msg):
        rep["ok"] = False
        if len(rep["fail"]) < 12:
            rep["fail"].append(msg)

    for name in ("argmax", "top1_prob", "entropy", "accept_len", "correction", "logits"):
        if out.get(name) is not None and not np.all(np.isfinite(out[name])):
            fail(f"non-finite values in {name}")
    # properties that hold for every request
    for i in range(B):
        am = out["argmax"][cu[i]:cu[i + 1]]
        n, c = oracle.accept_prefix(case.drafts[i], [int(case.anchor[i])] + [int(t) for t in am])
        if (n, c) != (int(out["accept_len"][i]), int(out["correction"][i])):
            fail(f"request {i}: accept/correction {out['accept_len'][i]}/{out['correction'][i]} "
                 f"inconsistent with its own argmax rows ({n}/{c})")
    p, H = out["top1_prob"], out["entropy"]
    if not (np.all(p > 0) and np.all(p <= 1 + 1e-6)):
        fail("top1_prob outside (0,1]")
    if not (np.all(H >= -1e-5) and np.all(H <= math.log(shape.vocab) + 1e-4)):
        fail("entropy outside [0, ln V]")
    if not np.all(p >= np.exp(-H) * (1 - 1e-4)):
        fail("top1_prob < exp(-H)")
    if out.get("logits") is not None:
        if not np.array_equal(out["logits"].argmax(axis=1).astype(np.int32), out["argmax"]):
            fail("argmax differs from the argmax of the returned logits")
    # element-wise against the oracle
    for i in case.sampled:
        want = case.want_rows[i]
        ids, p1, Hw, mg = oracle.confidence(want, case.model.dtype)
        sl = slice(int(cu[i]), int(cu[i + 1]))
        rep["rows_checked"] += int(k[i])
        if out.get("logits") is not None:
            err = float(np.abs(out["logits"][sl].astype(np.float64) - want).max())
            rep["max_logit_err"] = max(rep["max_logit_err"], err)
            if err > logit_tol:
                fail(f"request {i}: logits off by {err:.3e}")
        for j in range(int(k[i])):
            if mg[j] < MARGIN:
                rep["exempt_rows"] += 1
            elif int(out["argmax"][sl][j]) != int(ids[j]):
                fail(f"request {i} row {j}: argmax {out['argmax'][sl][j]} != {ids[j]} (margin {mg[j]:.3g})")
        prel = np.abs(out["top1_prob"][sl] - p1) / p1
        hrel = np.abs(out["entropy"][sl] - Hw) / np.maximum(Hw, 1e-30)
        rep["max_prob_rel"] = max(rep["max_prob_rel"], float(prel.max()))
        rep["max_entropy_rel"] = max(rep["max_entropy_rel"], float(hrel.max()))
        if np.any(np.abs(out["top1_prob"][sl] - p1) > 2.5e-2 * p1 + 1e-6):
            fail(f"request {i}: top1_prob off by rel {prel.max():.3e}")
        if np.any(hrel > ENTROPY_RTOL):
            fail(f"request {i}: entropy off by rel {hrel.max():.3e}")
        n, c = oracle.accept_prefix(case.drafts[i], [int(case.anchor[i])] + [int(t) for t in ids])
        rep["requests_checked"] += 1
        if np.all(mg[:min(n + 1, int(k[i]))] >= MARGIN):
            if (n, c) != (int(out["accept_len"][i]), int(out["correction"][i])):
                fail(f"request {i}: accept/correction {out['accept_len'][i]}/{out['correction'][i]} != {n}/{c}")
        else:
            rep["exempt_requests"] += 1
    return rep


def compare_kv(case, atol=LOGIT_TOL):
    """KV pool after the verify, sampled requests: context positions bit-identical to the oracle's, every
    slot of their pages beyond the chunk still untouched, chunk positions within |d| <= atol + 2^-6 |value|
    of the oracle's.  Where that tolerance comes from: a K/V entry is a projection of the same residual
    stream through weights of the same scale as a logit (N(0, 0.02) rows of length d), so before its
    rounding it is held to the logits tolerance (atol = 2e-2); each side then rounds to bf16, which moves
    the value by at most half a step of 2^-7 |value| -- two values that close can land on bf16 numbers up
    to 2^-6 |value| + atol apart.  In the first layer both sides see identical inputs and nearly every entry is
    bit-identical (the count is reported); deeper in, entries near a rounding boundary fall either way."""
    b = case.batch
    rep = {"ok": True, "fail": [], "max_kv_err": 0.0, "chunk_entries": 0, "chunk_entries_differing": 0,
           "layer0_entries": 0, "layer0_entries_differing": 0}
    kp = case.k_pool.view(torch.int16)
    vp = case.v_pool.view(torch.int16)
    for i in case.sampled:
        L, kk = int(b["ctx_len"][i]), int(b["n_draft"][i]) + int(case.n_uncached[i])
        for pg_i, page in enumerate(b["block_table"][i]):
            if page < 0:
                continue
            ob = case.okv._backing(page)
            gk = kp[:, page].cpu().numpy().view(np.uint16)      # [layers, Hkv, 16, hd]
            gv = vp[:, page].cpu().numpy().view(np.uint16)      # [layers, Hkv, hd, 16]
            for s in range(wl.PAGE_SIZE):
                t = pg_i * wl.PAGE_SIZE + s
                wk, wv = case.okv.k[:, ob, :, s, :], case.okv.v[:, ob, :, :, s]
                if t < L:
                    if not (np.array_equal(gk[:, :, s, :], wk) and np.array_equal(gv[:, :, :, s], wv)):
                        rep["ok"] = False
                        rep["fail"].append(f"request {i} position {t}: cached K/V changed")
                elif t < L + kk:
                    ek = np.abs(oracle.bf16_from_bits(gk[:, :, s, :]) - oracle.bf16_from_bits(wk))
                    ev = np.abs(oracle.bf16_from_bits(gv[:, :, :, s]) - oracle.bf16_from_bits(wv))
                    tol_k = atol + 2.0 ** -6 * np.abs(oracle.bf16_from_bits(wk))
                    tol_v = atol + 2.0 ** -6 * np.abs(oracle.bf16_from_bits(wv))
                    rep["max_kv_err"] = max(rep["max_kv_err"], float(ek.max()), float(ev.max()))
                    # entries whose bf16 rounding fell the other way than the oracle's (layer 0 sees identical
                    # inputs on both sides, so its count measures the projection's own precision)
                    dk, dv = gk[:, :, s, :] != wk, gv[:, :, :, s] != wv
                    rep["chunk_entries"] += dk.size + dv.size
                    rep["chunk_entries_differing"] += int(dk.sum()) + int(dv.sum())
                    rep["layer0_entries"] += dk[0].size + dv[0].size
                    rep["layer0_entries_differing"] += int(dk[0].sum()) + int(dv[0].sum())
                    if not (np.all(np.isfinite(ek)) and np.all(ek <= tol_k) and np.all(ev <= tol_v)):
                        rep["ok"] = False
                        rep["fail"].append(f"request {i} position {t}: appended K/V off (k {ek.max():.3e}, v {ev.max():.3e})")
                else:
                    if not (np.all(gk[:, :, s, :] == NAN_BITS) and np.all(gv[:, :, :, s] == NAN_BITS)):
                        rep["ok"] = False
                        rep["fail"].append(f"request {i} position {t}: slot beyond the chunk was written")
        if len(rep["fail"]) > 12:
            break
    return rep


def one_pass_parity(recipe, weights, device="cuda:0", n_requests=None, float32_too=False, tag=""):
    """Element-wise parity of ONE partial prefill over the whole batch, every input drawn independently of the
    HIP path: request i carries its last context token as one uncached token (the row that supplies
    q(x | prefix)) plus its k_i drafts, drawn uniformly at random (so nearly every chunk is rejected at once:
    accepted prefixes are what the chain-based cases cover).  The cached context is the stand-in K/V at
    positions 0..L-2 on both sides.  The oracle follows `n_requests` of the batch (all by default) through the
    same partial prefill; logits, ids, probabilities, entropies, accept lengths, corrections and the appended
    K/V of those requests are compared.  weights["model"] may widen its layers lazily (70B shape).
    float32_too: also run the oracle in float32 and report how far it lands from its float64 run."""
    shape = recipe.shape
    t0 = time.time()
    say = lambda *a: progress.say(f"[{tag or recipe.name}]", *a, f"(+{time.time() - t0:.0f}s)")   # noqa: E731
    b = wl.draw_batch(recipe)
    B = len(b["ctx_len"])
    k = b["n_draft"].astype(np.int32)
    rnd = wl.draw_draft_randoms(recipe, B)
    chosen = pick_sample(b, B if n_requests is None else n_requests)
    k_pool = nan_pool(shape, b["n_pages"], device, False)
    v_pool = nan_pool(shape, b["n_pages"], device, True)
    ver = synera.Verifier(shape, weights["head"], weights["layers"], max_batch=B, max_tokens=int(k.sum()) + B,
                          max_pages=b["max_pages"])
    model = weights["model"]
    pages = [p for i in chosen for p in b["block_table"][i] if p >= 0]
    okv = oracle.PagedKV(shape.n_layers, b["n_pages"], shape.n_kv_heads, shape.head_dim, pages=pages)
    okv32 = oracle.PagedKV(shape.n_layers, b["n_pages"], shape.n_kv_heads, shape.head_dim, pages=pages) if float32_too else None
    L = b["ctx_len"]
    n_fill = (L - 1).astype(np.int32)
    starts = np.concatenate([[0], np.cumsum(n_fill)])
    zeros, ones = np.zeros(B, np.int32), np.ones(B, np.int32)
    for l in range(shape.n_layers):
        kr, vr = wl.draw_context_kv(shape, recipe.seed, l, int(n_fill.sum()), device)
        ver.kv_append(l, zeros, n_fill, kr, vr, b["block_table"], b["n_pages"], k_pool, v_pool)
        for i in chosen:
            sl = slice(int(starts[i]), int(starts[i + 1]))
            okv.append_many(l, b["block_table"][i], 0, to_np(kr[sl]), to_np(vr[sl]))
            if okv32 is not None:
                okv32.append_many(l, b["block_table"][i], 0, to_np(kr[sl]), to_np(vr[sl]))
        torch.cuda.synchronize()
    say("context K/V filled")
    drafts = [np.asarray(rnd["tok"][i][:k[i]], np.int32) for i in range(B)]
    toks = np.concatenate([np.concatenate([[rnd["last_ctx_tok"][i]], drafts[i]]) for i in range(B)]).astype(np.int32)
    out = ver.verify(n_fill, ones, k, torch.from_numpy(toks).to(device), torch.zeros(B, dtype=torch.int32, device=device),
                     b["block_table"], b["n_pages"], k_pool, v_pool, want_logits=True)
    torch.cuda.synchronize()
    out = {n: (v.cpu().numpy() if v is not None else None) for n, v in out.items()}
    say("HIP path done")
    reqs = [{"block_table": b["block_table"][i], "ctx_len": int(L[i]) - 1, "uncached": [int(rnd["last_ctx_tok"][i])],
             "drafts": drafts[i], "anchor": -1} for i in chosen]
    widen = model._layers

    def layer_and_say(l):                     # a line every few layers: a pass over a 70B model takes minutes
        if l % 8 == 0:
            say(f"oracle at layer {l}")
        return widen(l) if callable(widen) else widen[l]
    model._layers = layer_and_say
    want = oracle.verify_chunks(model, okv, reqs)
    say("oracle done")
    rep = {"ok": True, "fail": [], "requests_checked": 0, "rows_checked": 0, "max_logit_err": 0.0,
           "max_entropy_rel": 0.0, "max_prob_rel": 0.0, "exempt_rows": 0, "exempt_requests": 0, "float32_floor": None,
           "worst_request": -1}
    if float32_too:
        model32 = oracle.OracleModel(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                                     shape.d_ffn, shape.vocab, model.embed, model._layers, model.final_norm,
                                     model.lm_head_w, rope_base=shape.rope_base, rms_eps=shape.rms_eps, dtype=np.float32)
        want32 = oracle.verify_chunks(model32, okv32, reqs)
        rep["float32_floor"] = float(np.abs(want32["logits"].astype(np.float64) - want["logits"]).max())
        say(f"float32 oracle done: max|dlogit| float32 oracle vs float64 oracle = {rep['float32_floor']:.3e}")
    model._layers = widen

    def fail(msg):
        rep["ok"] = False
        if len(rep["fail"]) < 12:
            rep["fail"].append(msg)

    for name in ("logits", "top1_prob", "entropy"):
        if not np.all(np.isfinite(out[name])):
            fail(f"non-finite values in {name}")
    if not np.array_equal(out["logits"].argmax(axis=1).astype(np.int32), out["argmax"]):
        fail("argmax differs from the argmax of the returned logits")
    cu = np.concatenate([[0], np.cumsum(k)])
    at = 0
    for n, i in enumerate(chosen):
        sl = slice(int(cu[i]), int(cu[i + 1]))
        w = slice(at, at + int(k[i]))
        at += int(k[i])
        rep["requests_checked"] += 1
        rep["rows_checked"] += int(k[i])
        err = float(np.abs(out["logits"][sl].astype(np.float64) - want["logits"][w]).max())
        if err > rep["max_logit_err"]:
            rep["max_logit_err"], rep["worst_request"] = err, i
        if err > LOGIT_TOL:
            fail(f"request {i}: logits off by {err:.3e}")
        mg = want["margin"][w]
        for j in range(int(k[i])):
            if mg[j] < MARGIN:
                rep["exempt_rows"] += 1
            elif int(out["argmax"][sl][j]) != int(want["argmax"][w][j]):
                fail(f"request {i} row {j}: argmax {out['argmax'][sl][j]} != {want['argmax'][w][j]} (margin {mg[j]:.3g})")
        p1, Hw = want["top1_prob"][w], want["entropy"][w]
        prel = np.abs(out["top1_prob"][sl] - p1) / p1
        hrel = np.abs(out["entropy"][sl] - Hw) / np.maximum(Hw, 1e-30)
        rep["max_prob_rel"] = max(rep["max_prob_rel"], float(prel.max()))
        rep["max_entropy_rel"] = max(rep["max_entropy_rel"], float(hrel.max()))
        if np.any(np.abs(out["top1_prob"][sl] - p1) > 2.5e-2 * p1 + 1e-6):
            fail(f"request {i}: top1_prob off by rel {prel.max():.3e}")
        if np.any(hrel > ENTROPY_RTOL):
            fail(f"request {i}: entropy off by rel {hrel.max():.3e}")
        # accept length / correction: exact when every row that decides them is outside the margin exemption
        n_acc = int(want["accept_len"][n])
        if want["first_margin"][n] >= MARGIN and np.all(mg[:min(n_acc, int(k[i]))] >= MARGIN):
            if (int(out["accept_len"][i]), int(out["correction"][i])) != (n_acc, int(want["correction"][n])):
                fail(f"request {i}: accept/correction {out['accept_len'][i]}/{out['correction'][i]} != "
                     f"{n_acc}/{want['correction'][n]}")
        else:
            rep["exempt_requests"] += 1
    case = Case(recipe, shape, device, dict(b, ctx_len=n_fill), weights["head"], weights["layers"], ver, k_pool, v_pool,
                chosen, model, okv)
    case.n_uncached = ones
    kv = compare_kv(case)
    ver.close()
    print(f"[{tag or recipe.name}] one pass, {rep['requests_checked']} of {B} requests, rows={rep['rows_checked']} "
          f"max|dlogit|={rep['max_logit_err']:.3e} (request {rep['worst_request']}) max rel dH={rep['max_entropy_rel']:.3e} "
          f"max rel dp={rep['max_prob_rel']:.3e} exempt rows/requests={rep['exempt_rows']}/{rep['exempt_requests']} "
          f"max|dKV|={kv['max_kv_err']:.3e} KV roundings differing: {kv['chunk_entries_differing']}/{kv['chunk_entries']} "
          f"(layer 0: {kv['layer0_entries_differing']}/{kv['layer0_entries']})"
          + (f" float32 oracle vs float64 oracle: {rep['float32_floor']:.3e}" if float32_too else ""), flush=True)
    return rep, kv
