"""Pins for the scheduler oracle (Section 4.5, Algorithm 1): hand-worked traces of what the text says an
iteration does (prefill first and alone, else all waiting verifications with their uncached counts,
completed requests leave afterwards), the chunk arithmetic in closed form, and conservation invariants
on seeded random arrival traces."""
import random

import pytest

from oracle.scheduler import SchedulerOracle


class Recorder:
    """Engine stand-in: records every engine call; accept lengths come from a seeded generator."""

    def __init__(self, seed=0, accept=None):
        self.rng = random.Random(seed)
        self.calls = []
        self.accept = accept

    def __call__(self, call):
        self.calls.append(call)
        out = []
        for it in call:
            if not it.final_verify:
                out.append(None)
            elif self.accept is not None:
                out.append(min(self.accept, it.n_draft))
            else:
                out.append(self.rng.randint(0, it.n_draft))
        return out


def make(**kw):
    args = dict(n_pages=4096, max_pages_per_request=256, max_batch=64, max_tokens=2048)
    args.update(kw)
    return SchedulerOracle(**args)


def test_prefill_has_priority_and_runs_alone():
    s, e = make(), Recorder(accept=2)
    s.submit_prefill(1, 40)
    assert s.iteration(e) == "prefill"
    s.submit_verify(1, 0, 4)
    s.submit_prefill(2, 10)                    # arrives while a verification is waiting
    assert s.iteration(e) == "prefill"         # ... and goes first
    assert s.log[-1] == ("prefill", [2], None)
    assert all(it.request_id == 2 for it in e.calls[-1])
    assert s.iteration(e) == "verify"          # only now the verification
    assert s.log[-1] == ("verify", [1], [0])
    assert s.iteration(e) == "idle"
    assert s.B == [2, 1]                       # B <- B_prefill U B: the newer prefill is in front


def test_all_waiting_verifications_form_one_batch_with_their_uncached_counts():
    s, e = make(), Recorder(accept=0)
    for i, n in enumerate([5, 17, 33]):
        s.submit_prefill(i, n)
    assert s.iteration(e) == "prefill"
    assert s.log[-1] == ("prefill", [0, 1, 2], None)
    s.submit_verify(2, 3, 4)
    s.submit_verify(0, 0, 8)
    s.submit_verify(1, 7, 1)
    n_before = len(e.calls)
    assert s.iteration(e) == "verify"
    assert s.log[-1] == ("verify", [2, 0, 1], [3, 0, 7])      # arrival order, u of every request
    assert len(e.calls) == n_before + 1                        # all fit one chunk: one engine call
    call = e.calls[-1]
    assert [(it.request_id, it.ctx_len, it.n_uncached, it.n_draft, it.final_verify) for it in call] == \
        [(2, 33, 3, 4, True), (0, 5, 0, 8, True), (1, 17, 7, 1, True)]


def test_cached_length_after_a_verification_is_L_plus_u_plus_accepted():
    s = make()
    s.submit_prefill(7, 20)
    s.iteration(Recorder())
    for u, k, a in [(0, 4, 4), (1, 6, 0), (3, 5, 2)]:
        L = s.requests[7].cached
        e = Recorder(accept=a)
        s.submit_verify(7, u, k)
        s.iteration(e)
        assert e.calls[-1][0].ctx_len == L
        assert s.requests[7].cached == L + u + a
    assert s.requests[7].cached == 20 + 4 + 1 + 5


def test_completed_requests_leave_after_a_verification_iteration_and_return_their_pages():
    s, e = make(n_pages=8), Recorder(accept=1)
    s.submit_prefill(1, 30)
    s.submit_prefill(2, 30)
    s.iteration(e)
    assert len(s.free_pages) == 8 - 4
    s.finish(1)
    s.submit_prefill(3, 16)
    assert s.iteration(e) == "prefill"          # a prefill iteration ends before remove_completed
    assert 1 in s.B and len(s.free_pages) == 3
    assert s.iteration(e) == "idle"             # the next one reaches it
    assert s.B == [3, 2] and 1 not in s.requests and len(s.free_pages) == 5
    with pytest.raises(ValueError):
        s.submit_verify(1, 0, 1)


@pytest.mark.parametrize("u,k", [(0, 1), (0, 32), (1, 32), (20, 16), (31, 2), (33, 31), (33, 32), (64, 32), (63, 2), (100, 5)])
def test_verification_chunks_closed_form(u, k):
    s, e = make(), Recorder(accept=k)
    s.submit_prefill(0, 3)
    s.iteration(e)
    e.calls.clear()
    s.submit_verify(0, u, k)
    s.iteration(e)
    rho = u % 32
    assert len(e.calls) == u // 32 + (1 if rho + k <= 32 else 2) == -(-(u + k) // 32)
    items = [c[0] for c in e.calls]
    pos = 0
    for it in items:                             # every token once, in order, at its position
        assert it.token_begin == pos and it.ctx_len == 3 + pos
        assert 1 <= it.n_uncached + it.n_draft <= 32
        pos += it.n_uncached + it.n_draft
    assert pos == u + k
    assert [it.final_verify for it in items] == [False] * (len(items) - 1) + [True]
    assert items[-1].n_draft == k and all(it.n_draft == 1 for it in items[:-1])


@pytest.mark.parametrize("n", [1, 31, 32, 33, 64, 1000])
def test_prefill_chunks_closed_form(n):
    s, e = make(), Recorder()
    s.submit_prefill(0, n)
    s.iteration(e)
    assert len(e.calls) == -(-n // 32)
    assert sum(c[0].n_uncached + c[0].n_draft for c in e.calls) == n
    assert all(c[0].n_draft == 1 and not c[0].final_verify for c in e.calls)
    assert s.requests[0].cached == n and len(s.requests[0].pages) == -(-n // 16)


def test_limits_admit_in_arrival_order_without_overtaking():
    s, e = make(max_batch=2), Recorder(accept=0)
    for i in range(3):
        s.submit_prefill(i, 4)
    assert s.iteration(e) == "prefill" and s.log[-1][1] == [0, 1]
    assert s.iteration(e) == "prefill" and s.log[-1][1] == [2]
    # token limit: chunks of 20 + 20 fit 40, a third does not
    s = make(max_tokens=40)
    for i in range(3):
        s.submit_prefill(i, 20)
    s.iteration(e); assert s.log[-1][1] == [0, 1]
    s.iteration(e); assert s.log[-1][1] == [2]
    # pages: 4 pages in the pool; request 0 holds 2, request 1 needs 3 and blocks request 2 behind it
    s = make(n_pages=4)
    s.submit_prefill(0, 32); s.submit_prefill(1, 40); s.submit_prefill(2, 1)
    s.iteration(e); assert s.log[-1][1] == [0]
    assert s.iteration(e) == "idle"
    s.finish(0)
    assert s.iteration(e) == "idle"              # this one frees the pages (after the gathering)
    assert s.iteration(e) == "prefill" and s.log[-1][1] == [1, 2]
    with pytest.raises(MemoryError):
        s.submit_prefill(9, 16 * 4 + 1)


def test_random_traces_conserve_tokens_pages_and_kinds():
    for seed in range(20):
        rng = random.Random(seed)
        s = make(n_pages=rng.choice([64, 256]), max_batch=rng.choice([3, 8, 64]), max_tokens=rng.choice([64, 256]))
        e = Recorder(seed)
        submitted = {}                            # id -> list of (u, k) verifications forwarded
        next_id, waiting = 0, set()
        for step in range(200):
            r = rng.random()
            if r < 0.25:
                n = rng.randint(1, 120)
                try:
                    s.submit_prefill(next_id, n)
                    submitted[next_id] = [n]
                except MemoryError:
                    pass
                next_id += 1
            elif r < 0.7 and s.B:
                i = rng.choice(s.B)
                if i not in waiting and not s.requests[i].completed:
                    u, k = rng.choice([0, 0, 1, 3, 40]), rng.randint(1, 16)
                    try:
                        s.submit_verify(i, u, k)
                        waiting.add(i)
                    except MemoryError:
                        s.finish(i)
            elif r < 0.75 and s.B:
                i = rng.choice(s.B)
                if i not in waiting and not s.requests[i].completed:
                    s.finish(i)
            n_calls = len(e.calls)
            kind = s.iteration(e)
            new_calls = e.calls[n_calls:]
            if kind == "idle":
                assert not new_calls
            for call in new_calls:
                assert 1 <= len(call) <= s.max_batch
                assert sum(it.n_uncached + it.n_draft for it in call) <= s.max_tokens
                ids = [it.request_id for it in call]
                assert len(set(ids)) == len(ids)
                assert all(it.final_verify or it.n_draft == 1 for it in call)
                if kind == "prefill":            # never mixed with verifications
                    assert not any(it.final_verify for it in call)
                    assert all(it.ctx_len == it.token_begin for it in call)
                used = [p for it in call for p in it.pages]
                assert len(set(used)) == len(used)                       # no page shared between requests
                for it in call:
                    assert len(it.pages) * 16 >= it.ctx_len + it.n_uncached + it.n_draft
                    if it.final_verify:
                        waiting.discard(it.request_id)
            live = [p for r_ in s.requests.values() for p in r_.pages]
            assert len(set(live)) == len(live) and not set(live) & set(s.free_pages)
            assert len(live) + len(s.free_pages) == s.n_pages
        assert e.calls


def test_a_submission_arriving_while_the_iteration_still_runs_waits_for_the_next_one():
    """Request 1 finishes its single chunk while request 2 still has chunks to go; its next verification
    arrives in between.  It must not be swept into the running iteration (Algorithm 1 gathers only at the
    start of an iteration), and it gets the page its longer context needs."""
    s = make()
    s.submit_prefill(1, 204)
    s.submit_prefill(2, 10)
    s.iteration(Recorder())
    calls = []

    def engine(call):
        calls.append(call)
        if len(calls) == 2:
            s.submit_verify(1, 1, 6)                 # request 1's first verification ended with call 1
        return [it.n_draft if it.final_verify else None for it in call]

    s.submit_verify(1, 0, 2)                         # one chunk: 204 -> 206 cached
    s.submit_verify(2, 70, 4)                        # three chunks
    assert s.iteration(engine) == "verify"
    assert [[it.request_id for it in c] for c in calls] == [[1, 2], [2], [2]]
    assert s.iteration(engine) == "verify"
    it = calls[-1][0]
    assert (it.request_id, it.ctx_len, it.n_uncached, it.n_draft) == (1, 206, 1, 6)
    assert len(it.pages) == 14                       # 213 tokens


def _golden_session():
    """tests/golden/scheduler_trace.txt parsed into steps."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "scheduler_trace.txt")
    steps = []
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            steps.append(line.split())
    return steps


def test_golden_session_worked_from_the_listing_of_algorithm_1():
    """Prefill priority, B <- B_prefill U B, the iteration that ends before remove_completed, L_uncached in
    batch order, a request that waits for pages, and pages of removed requests reused: the oracle against a
    session worked by hand from the listing (tests/golden/scheduler_trace.txt)."""
    steps = _golden_session()
    assert steps[0][0] == "pool"
    s = SchedulerOracle(*[int(v) for v in steps[0][1:]])
    accept, owners, n_iter = {}, {}, 0

    def engine(call):
        return [accept[it.request_id] if it.final_verify else None for it in call]

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
            assert st[0] == "iter"
            kind = st[1]
            f = dict(x.split("=") for x in st[2:])
            n_log = len(s.log)
            assert s.iteration(engine) == kind, st
            ids = [] if f["ids"] == "-" else [int(v) for v in f["ids"].split(",")]
            if kind == "idle":
                assert len(s.log) == n_log
            else:
                unc = None if f["unc"] == "-" else [int(v) for v in f["unc"].split(",")]
                assert s.log[-1] == (kind, ids, unc), st
            assert s.B == [int(v) for v in f["B"].split(",")], st
            assert len(s.free_pages) == int(f["free"]), st
            for item in f["len"].split(","):
                rid, L = item.split(":")
                assert s.requests[int(rid)].cached == int(L), st
            # a page belongs to one live request at a time, and freed pages do come back into use
            held = [p for r in s.requests.values() for p in r.pages]
            assert len(held) == len(set(held)) and not set(held) & set(s.free_pages)
            for r in s.requests.values():
                for p in r.pages:
                    owners.setdefault(p, set()).add(r.rid if hasattr(r, "rid") else id(r))
            n_iter += 1
    assert n_iter == 9
    assert any(len(v) > 1 for v in owners.values())          # some page served two requests in turn
