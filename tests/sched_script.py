"""A scripted serving session for the scheduler tests, produced on the CPU by the oracle alone:
SchedulerOracle drives oracle.verify_chunks on a small decoder while a seeded stand-in for the device
side submits prompts and verification requests.  Its drafts come from sequential greedy decoding with the
same oracle model from the request's current state, replaced by a random token at seeded positions, so
accept lengths vary; some rounds first "accept locally" 33 more tokens so that the partial prefill spans
several 32-token chunks, and even-numbered requests send their first verification without uncached
tokens (anchor form).  The script records every arrival and every engine call with its tokens, anchors
and results; the GPU test replays it against the C-ABI scheduler + synera_verify."""
import random
from dataclasses import dataclass, field

import numpy as np

import oracle
from oracle.scheduler import SchedulerOracle


@dataclass
class ScriptCall:
    kind: str
    items: list                 # EngineItem
    tokens: list                # per item: token ids of the chunk (uncached then LM-head rows)
    anchors: list               # per item: anchor token (used when the chunk has no uncached tokens)
    argmax: list                # per item: oracle greedy token after each LM-head row
    margin: list                # per item: oracle top-2 logit margins of those rows
    first_margin: list          # per item: margin of the row that supplies q(x | prefix) (inf with an anchor)
    accept_len: list            # per item (None unless final_verify)
    correction: list
    logits: object = None       # oracle logits of all LM-head rows of the call, request-major [R][V]


@dataclass
class Script:
    calls: list = field(default_factory=list)
    arrivals: list = field(default_factory=list)   # one list of (what, id, a, b) per arrival point: one before
                                                   # every iteration and one inside every engine call
    iterations: list = field(default_factory=list) # engine calls per iteration (0 = idle)
    prompt_len: dict = field(default_factory=dict)
    final_cached: dict = field(default_factory=dict)


def make_script(model, shape, seed, n_requests=8, n_pages=80, max_pages=12, max_batch=4, max_tokens=96,
                horizon=60, steps=120):
    rng = random.Random(seed)
    sched = SchedulerOracle(n_pages, max_pages, max_batch, max_tokens)
    kv = oracle.PagedKV(shape.n_layers, n_pages + 16 * n_requests, shape.n_kv_heads, shape.head_dim)
    script = Script()
    prompts, emitted, sub, last_row = {}, {}, {}, {}
    for i in range(n_requests):
        prompts[i] = [rng.randrange(shape.vocab) for _ in range(rng.choice([3, 17, 33, 40, 70]))]
        script.prompt_len[i] = len(prompts[i])
    state = {"to_submit": list(range(n_requests)), "done": set()}

    def table(pages):
        row = np.full(max_pages, -1, np.int32)
        row[:len(pages)] = pages
        return row

    def decode(i, pos, tokens):
        """Greedy token after forwarding `tokens` at positions pos.. (writes K/V that the verification of
        the same positions overwrites)."""
        x = oracle.forward_tokens(model, kv, [(table(sched.requests[i].pages + spare[i]), pos, tokens)])
        return int(np.argmax(oracle.lm_head(model, x[-1])))

    spare = {}                                               # scratch pages for the stand-in's lookahead

    def arrivals():
        ev = []
        script.arrivals.append(ev)
        if state["to_submit"] and rng.random() < 0.5:
            i = state["to_submit"].pop(0)
            sched.submit_prefill(i, len(prompts[i]))
            sub[i] = list(prompts[i])
            ev.append(("prefill", i, len(prompts[i]), 0))
        for i in list(sched.B):
            r = sched.requests[i]
            if r.completed or r.waiting is not None or r.running or i in state["done"] or rng.random() < 0.4:
                continue
            if r.cached + 60 > max_pages * 16 or emitted[i] > horizon:
                sched.finish(i)
                ev.append(("finish", i, 0, 0))
                state["done"].add(i)
                continue
            # lookahead pages beyond the request's own, so that drafting never touches another request
            need = -(-(r.cached + 50) // 16) - len(r.pages)
            spare[i] = list(range(n_pages + 16 * i, n_pages + 16 * i + max(need, 0)))
            k = rng.randint(1, 8)
            if r.cached == len(prompts[i]) and i % 2 == 0:   # first round, no uncached token: anchor form
                unc, g = [], last_row[i]
            else:                                            # the last emitted token is not cached yet
                unc = [last_tok[i]]
                g = decode(i, r.cached, unc)
                for _ in range(rng.choice([0, 0, 0, 33])):   # plus tokens the device accepted by itself
                    unc.append(g)
                    g = decode(i, r.cached + len(unc) - 1, [g])
            drafts = []
            for j in range(k):
                d = g if rng.random() < 0.7 else (g + 1 + rng.randrange(shape.vocab - 1)) % shape.vocab
                drafts.append(d)
                if j + 1 < k:
                    g = decode(i, r.cached + len(unc) + j, [d])
            sched.submit_verify(i, len(unc), len(drafts))
            sub[i] = unc + drafts
            ev.append(("verify", i, len(unc), len(drafts)))

    last_tok = {}                                            # the LLM's newest token, not cached yet

    def engine(call):
        reqs, toks, anchors = [], [], []
        for it in call:
            n = it.n_uncached + it.n_draft
            t = sub[it.request_id][it.token_begin:it.token_begin + n]
            a = last_row.get(it.request_id, 0)
            reqs.append({"block_table": table(it.pages), "ctx_len": it.ctx_len, "uncached": t[:it.n_uncached],
                         "drafts": t[it.n_uncached:], "anchor": a})
            toks.append(t)
            anchors.append(a)
        out = oracle.verify_chunks(model, kv, reqs)
        acc, am, mg, corr = [], [], [], []
        at = 0
        for j, it in enumerate(call):
            rows = slice(at, at + it.n_draft)
            at += it.n_draft
            am.append([int(x) for x in out["argmax"][rows]])
            mg.append([float(x) for x in out["margin"][rows]])
            last_row[it.request_id] = am[-1][-1]             # greedy token after the chunk's last row
            i = it.request_id
            if it.final_verify:
                a = int(out["accept_len"][j])
                acc.append(a)
                corr.append(int(out["correction"][j]))
                last_tok[i] = corr[-1]
                emitted[i] = (it.ctx_len + it.n_uncached - len(prompts[i])) + a + 1
            else:
                acc.append(None)
                corr.append(None)
                if it.ctx_len + it.n_uncached + it.n_draft == len(prompts[i]) and it.ctx_len < len(prompts[i]):
                    emitted[i] = 1                           # prompt consumed: the anchor is known
                    last_tok[i] = am[-1][-1]
        script.calls.append(ScriptCall(sched.log[-1][0], list(call), toks, anchors, am, mg,
                                       [float(x) for x in out["first_margin"]], acc, corr, np.asarray(out["logits"])))
        arrivals()
        return acc

    for _ in range(steps):
        arrivals()
        n0 = len(script.calls)
        sched.iteration(engine)
        script.iterations.append(len(script.calls) - n0)
    script.final_cached = {i: r.cached for i, r in sched.requests.items()}
    return script
