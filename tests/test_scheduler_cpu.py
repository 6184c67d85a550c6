"""The C-ABI scheduler (include/synera_sched.h, host code only) against the scheduler oracle on seeded
arrival traces: the same engine calls in the same order -- kind, requests, cached lengths, uncached and
draft counts, token offsets, final-verify flags -- and valid page tables (page ids may differ: any free
page is a correct choice).  Arrivals are injected between engine calls, also in the middle of an
iteration."""
import random

import numpy as np
import pytest

import paper_2511_07423_amd as synera
from oracle.scheduler import SchedulerOracle

KIND = {"prefill": synera.SCHED_PREFILL, "verify": synera.SCHED_VERIFY, "idle": synera.SCHED_IDLE}


def _trace(seed, n_pages, max_pages, max_batch, max_tokens, steps=160):
    """Drive the oracle; record its engine calls and, per arrival point (one before every iteration, one
    inside every engine call), the events that arrived there."""
    rng = random.Random(seed)
    o = SchedulerOracle(n_pages, max_pages, max_batch, max_tokens)
    calls, events, state = [], [], {"next_id": 0, "waiting": set()}

    def arrivals():
        events.append([])
        r = rng.random()
        if r < 0.3:
            n, i = rng.choice([1, 5, 31, 32, 33, 70, 200]), state["next_id"]
            state["next_id"] += 1
            try:
                o.submit_prefill(i, n)
                events[-1].append(("prefill", i, n, 0, synera.OK))
            except MemoryError:
                events[-1].append(("prefill", i, n, 0, synera.ENOSPC))
        elif r < 0.75 and o.B:
            i = rng.choice(o.B)
            u, k = rng.choice([0, 0, 1, 2, 30, 45]), rng.randint(1, 32 if rng.random() < 0.2 else 8)
            try:
                o.submit_verify(i, u, k)
                events[-1].append(("verify", i, u, k, synera.OK))
            except ValueError:
                events[-1].append(("verify", i, u, k, synera.EINVAL))
            except MemoryError:
                events[-1].append(("verify", i, u, k, synera.ENOSPC))
        elif r < 0.85 and o.B:
            i = rng.choice(o.B)
            try:
                o.finish(i)
                events[-1].append(("finish", i, 0, 0, synera.OK))
            except ValueError:
                events[-1].append(("finish", i, 0, 0, synera.EINVAL))

    def engine(call):
        acc = [rng.randint(0, it.n_draft) if it.final_verify else None for it in call]
        calls.append((list(call), acc))
        arrivals()                                   # lands in the middle of the oracle's iteration
        return acc

    kinds = []
    for _ in range(steps):
        arrivals()
        n0 = len(calls)
        kind = o.iteration(engine)
        kinds.append((kind, len(calls) - n0))
    return o, calls, events, kinds


@pytest.mark.parametrize("seed,n_pages,max_pages,max_batch,max_tokens", [
    (0, 4096, 64, 64, 2048), (1, 64, 16, 4, 64), (2, 40, 8, 3, 40), (3, 512, 32, 16, 100),
    (4, 30, 30, 64, 2048), (5, 4096, 64, 2, 33)])
def test_same_engine_calls_as_the_oracle(seed, n_pages, max_pages, max_batch, max_tokens):
    o, calls, events, kinds = _trace(seed, n_pages, max_pages, max_batch, max_tokens)
    assert len(calls) > 20
    s = synera.Scheduler(n_pages, max_pages, max_batch, max_tokens)

    def replay():
        for what, i, a, b, status in events.pop(0):
            try:
                {"prefill": lambda: s.submit_prefill(i, a), "verify": lambda: s.submit_verify(i, a, b),
                 "finish": lambda: s.finish(i)}[what]()
                got = synera.OK
            except synera.SyneraError as e:
                got = e.status
            assert got == status, (what, i, a, b)

    n_call = 0
    owner = {}                                       # page -> request, to check that tables stay valid
    for kind, n_calls in kinds:
        for p in [p for p, r in owner.items() if s.cached_len(r) < 0]:
            del owner[p]                             # pages of requests that left may be handed out again
        replay()
        if n_calls == 0:
            k, out = s.next()
            assert k == synera.SCHED_IDLE and len(out["request_id"]) == 0
            continue
        for _ in range(n_calls):
            k, out = s.next()
            want, acc = calls[n_call]
            assert k == KIND[kind]
            assert out["request_id"].tolist() == [it.request_id for it in want]
            assert out["ctx_len"].tolist() == [it.ctx_len for it in want]
            assert out["n_uncached"].tolist() == [it.n_uncached for it in want]
            assert out["n_draft"].tolist() == [it.n_draft for it in want]
            assert out["token_begin"].tolist() == [it.token_begin for it in want]
            assert out["final_verify"].tolist() == [int(it.final_verify) for it in want]
            bt = out["block_table"]
            ok = synera.validate_batch(ctx_len=out["ctx_len"], n_first=out["n_draft"], n_second=out["n_uncached"],
                                       block_table=bt, n_pages_in_pool=n_pages, max_batch=max_batch,
                                       max_tokens=max_tokens, chunk_limit=32)
            assert ok == synera.OK                   # exactly what synera_verify would check
            for row, it in zip(bt, want):
                have = [int(p) for p in row if p >= 0]
                assert len(have) == len(it.pages)
                for p in have:
                    assert owner.setdefault(p, it.request_id) == it.request_id
            n_call += 1
            replay()                                 # arrivals during the iteration
            s.commit([0 if a is None else a for a in acc])
    st = s.stats()
    assert st["engine_calls"] == len(calls)
    assert st["free_pages"] == len(o.free_pages) and st["active_requests"] == len(o.B)
    for i, r in o.requests.items():
        assert s.cached_len(i) == r.cached
    assert st["iterations_prefill"] == sum(1 for k, n in kinds if k == "prefill")
    assert st["iterations_verify"] == sum(1 for k, n in kinds if k == "verify")


def test_protocol_errors():
    s = synera.Scheduler(64, 16, 8, 256)
    with pytest.raises(synera.SyneraError):
        s.commit()                                   # nothing outstanding
    s.submit_prefill(1, 10)
    with pytest.raises(synera.SyneraError):
        s.submit_prefill(1, 10)                      # id in use
    with pytest.raises(synera.SyneraError):
        s.submit_verify(1, 0, 4)                     # not prefilled yet
    k, out = s.next()
    assert k == synera.SCHED_PREFILL
    with pytest.raises(synera.SyneraError):
        s.next()                                     # commit first
    s.commit()
    s.submit_verify(1, 2, 4)
    with pytest.raises(synera.SyneraError):
        s.submit_verify(1, 0, 1)                     # one at a time
    with pytest.raises(synera.SyneraError):
        s.finish(1)                                  # work pending
    k, out = s.next()
    assert k == synera.SCHED_VERIFY and out["ctx_len"].tolist() == [10] and out["n_uncached"].tolist() == [2]
    with pytest.raises(synera.SyneraError):
        s.commit([5])                                # accept length beyond k: refused, state kept
    s.commit([3])
    assert s.cached_len(1) == 10 + 2 + 3
    with pytest.raises(synera.SyneraError) as e:
        s.submit_prefill(2, 16 * 16 + 1)             # more pages than a block-table row holds
    assert e.value.status == synera.ENOSPC
    s.finish(1)
    assert s.next()[0] == synera.SCHED_IDLE
    assert s.cached_len(1) == -1 and s.stats()["free_pages"] == 64


def test_scripted_session_gives_the_same_engine_calls():
    """The serving session the GPU test replays (oracle scheduler + oracle verify + a seeded device stand-in),
    here against the C-ABI scheduler alone."""
    import gpu_harness as gh
    import sched_script as ss
    import workloads as wl
    shape = wl.ModelShape("mini", 2, 128, 4, 2, 64, 256, 256)
    sc = ss.make_script(gh.draw_weights(shape, 9, "cpu")["model"], shape, 1)
    assert sum(1 for c in sc.calls if c.kind == "verify" for it in c.items if not it.final_verify) >= 3   # chunked
    assert sum(1 for c in sc.calls for it in c.items if it.final_verify and it.n_uncached == 0) >= 2      # anchor form
    s = synera.Scheduler(80, 12, 4, 96)
    arrivals, n_call = list(sc.arrivals), 0

    def replay():
        for what, i, a, b in arrivals.pop(0):
            {"prefill": lambda: s.submit_prefill(i, a), "verify": lambda: s.submit_verify(i, a, b),
             "finish": lambda: s.finish(i)}[what]()

    for n_calls in sc.iterations:
        replay()
        if n_calls == 0:
            assert s.next()[0] == synera.SCHED_IDLE
        for _ in range(n_calls):
            kind, out = s.next()
            call = sc.calls[n_call]
            assert kind == KIND[call.kind]
            for name in ("request_id", "ctx_len", "n_uncached", "n_draft", "token_begin"):
                assert out[name].tolist() == [getattr(it, name) for it in call.items]
            n_call += 1
            replay()
            s.commit([0 if a is None else a for a in call.accept_len])
    assert n_call == len(sc.calls) > 30


def test_golden_session_worked_from_the_listing_of_algorithm_1():
    """The hand-worked session of tests/golden/scheduler_trace.txt through the C-ABI scheduler: iteration kinds,
    requests and uncached counts per engine call, cached lengths after every iteration, free pages and the active
    batch at the end."""
    from test_oracle_scheduler import _golden_session
    steps = _golden_session()
    s = synera.Scheduler(*[int(v) for v in steps[0][1:]])
    accept = {}
    for st in steps[1:]:
        if st[0] == "prefill":
            s.submit_prefill(int(st[1]), int(st[2]))
        elif st[0] == "verify":
            s.submit_verify(int(st[1]), int(st[2]), int(st[3]))
        elif st[0] == "finish":
            s.finish(int(st[1]))
        elif st[0] == "accept":
            accept = {int(a): int(b) for a, b in zip(st[1::2], st[2::2])}
        else:
            f = dict(x.split("=") for x in st[2:])
            want_len = {int(a): int(b) for a, b in (item.split(":") for item in f["len"].split(","))}
            if st[1] == "idle":
                kind, out = s.next()
                assert kind == synera.SCHED_IDLE and len(out["request_id"]) == 0, st
            else:
                ids = [int(v) for v in f["ids"].split(",")]
                seen = []
                for _ in range(4):                      # an iteration is one engine call per 32-token chunk
                    kind, out = s.next()
                    assert kind == KIND[st[1]], st
                    for i in out["request_id"].tolist():
                        if i not in seen:
                            seen.append(i)
                    if st[1] == "verify":
                        assert out["n_uncached"].tolist() == [int(v) for v in f["unc"].split(",")], st
                        s.commit([accept[int(i)] for i in out["request_id"]])
                    else:
                        s.commit()
                    if all(s.cached_len(i) == L for i, L in want_len.items() if i in ids):
                        break
                assert seen == ids, st
            for rid, L in want_len.items():
                assert s.cached_len(rid) == L, st
            last = f
    # the module closes an iteration (B <- B_prefill U B, remove_completed) when the next one is asked for: the
    # session ends on an idle iteration, after which its counters are those of the last line
    assert s.next()[0] == synera.SCHED_IDLE
    stats = s.stats()
    assert stats["free_pages"] == int(last["free"]) and stats["active_requests"] == len(last["B"].split(","))
    assert stats["iterations_prefill"] == 3 and stats["iterations_verify"] == 3
