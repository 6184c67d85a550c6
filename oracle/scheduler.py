"""Oracle for the verification-aware scheduler (Section 4.5, Algorithm 1).  TEST INFRASTRUCTURE ONLY.

Plain Python on lists and dicts, in the algorithm's own order and names: one call of `iteration()` is one
pass of the algorithm's outer loop.  Prefill requests have priority: if any is waiting, the iteration
executes them and ends; otherwise every waiting verification request is gathered into B_verify with
its number of uncached tokens (L_uncached) and executed as one partial prefill; completed requests
leave the active batch B at the end of an iteration that reached that step.

What the algorithm leaves open, and the reading taken here (the product's host module takes the same):

  * `execute_prefill` / `execute_partialprefill` are given as opaque calls.  Here each is a sequence of
    engine calls on fixed chunks of at most `chunk` = 32 tokens per request (Section 4.5, chunked partial
    prefill): a request with n tokens to forward takes ceil(n / chunk) engine calls, requests of one batch
    advance together, and the draft tokens of a verification request ride in its last chunk.  Because
    the engine call needs at least one row that goes through the LM head per request, the last token
    of a chunk without drafts is marked as that row (`n_draft` = 1, result unused except after the last
    prompt token, whose greedy token is the request's first anchor).
  * The listing reads `get_num_uncached` after fetching the *next* request, which would skip the first
    request's count and query the empty one; L_uncached here holds u of every request of B_verify, in
    batch order.
  * The listing's `break` after a prefill ends the iteration, not the scheduler.
  * Capacity is not part of the algorithm.  Requests are admitted in arrival order while they fit:
    at most `max_batch` requests per batch, at most `max_tokens` chunk tokens in an engine call, and
    KV pages for the request's whole new length (ceil((L + n) / page) pages of `page` = 16 tokens)
    from a pool of `n_pages`; the first request that does not fit stays at the head of its queue and
    ends the gathering (no overtaking).  A request that could never fit is refused when submitted.
  * After a verification with accept length a, the request's cached length becomes L + u + a: the
    rejected drafts' KV entries are dead and are overwritten by the next chunk.

The `engine` callback stands for the model: it receives one engine call (a list of EngineItem) and
returns the accept length for every item whose `final_verify` is set (None elsewhere).
"""
from collections import deque
from dataclasses import dataclass, field


@dataclass
class EngineItem:
    request_id: int
    ctx_len: int          # L: tokens of this request whose KV is cached before the call
    n_uncached: int       # u: forwarded for their KV only
    n_draft: int          # k: rows that go through the LM head
    token_begin: int      # index of the chunk's first token in the request's submitted token list
    final_verify: bool    # the chunk carries the request's drafts: the accept length is read from it
    pages: tuple          # page ids of the request, in order, covering L + u + k tokens


@dataclass
class _Request:
    request_id: int
    cached: int = 0                    # L
    pages: list = field(default_factory=list)
    completed: bool = False
    # the request waiting in a queue or being executed
    n_prompt: int = 0
    u: int = 0
    k: int = 0
    done: int = 0                      # tokens of the current submission already forwarded


class SchedulerOracle:
    def __init__(self, n_pages, max_pages_per_request, max_batch, max_tokens, chunk=32, page=16):
        self.chunk, self.page = chunk, page
        self.max_batch, self.max_tokens, self.max_pages_per_request = max_batch, max_tokens, max_pages_per_request
        self.free_pages = list(range(n_pages))
        self.n_pages = n_pages
        self.requests = {}
        self.prefill_queue = deque()
        self.verify_queue = deque()
        self.B = []                    # the active batch of Algorithm 1: ids in the order they joined
        self.log = []                  # ("prefill" | "verify", [ids], L_uncached or None) per executed iteration

    # ---- arrivals -------------------------------------------------------------------------------
    def _pages_for(self, n_tokens):
        return -(-n_tokens // self.page)

    def submit_prefill(self, request_id, n_prompt):
        if request_id in self.requests or n_prompt < 1:
            raise ValueError("bad prefill request")
        if self._pages_for(n_prompt) > min(self.max_pages_per_request, self.n_pages):
            raise MemoryError("prompt can never fit")
        r = _Request(request_id, n_prompt=n_prompt)
        self.requests[request_id] = r
        self.prefill_queue.append(r)

    def submit_verify(self, request_id, u, k):
        r = self.requests.get(request_id)
        if r is None or request_id not in self.B or r.completed or u < 0 or k < 1 or k > self.chunk:
            raise ValueError("bad verification request")
        if r in self.verify_queue or r.k:
            raise ValueError("request already has a verification pending")
        if self._pages_for(r.cached + u + k) > min(self.max_pages_per_request, self.n_pages):
            raise MemoryError("request can never fit")
        r.u, r.k, r.done = u, k, 0
        self.verify_queue.append(r)

    def finish(self, request_id):
        r = self.requests[request_id]
        if r.k or r.n_prompt:
            raise ValueError("request still has work pending")
        r.completed = True

    # ---- the two fetch operations of the algorithm, with the admission rule ---------------------
    def _admit(self, r, n_new_tokens, batch, first_call_tokens):
        """Pages for the request's whole new length, if batch, token and page limits allow."""
        if len(batch) + 1 > self.max_batch:
            return False
        if first_call_tokens + min(self.chunk, n_new_tokens) > self.max_tokens:
            return False
        need = self._pages_for(r.cached + n_new_tokens) - len(r.pages)
        if need > len(self.free_pages):
            return False
        for _ in range(max(need, 0)):
            r.pages.append(self.free_pages.pop(0))
        return True

    def get_next_prefill_request(self, B_prefill):
        if not self.prefill_queue:
            return None
        r = self.prefill_queue[0]
        tokens = sum(min(self.chunk, q.n_prompt) for q in B_prefill)
        if not self._admit(r, r.n_prompt, B_prefill, tokens):
            return None
        return self.prefill_queue.popleft()

    def get_next_verification_request(self, B_verify):
        if not self.verify_queue:
            return None
        r = self.verify_queue[0]
        tokens = sum(min(self.chunk, q.u + q.k) for q in B_verify)
        if not self._admit(r, r.u + r.k, B_verify, tokens):
            return None
        return self.verify_queue.popleft()

    # ---- execution: fixed chunks through the engine ---------------------------------------------
    def _engine_calls(self, batch, total_of, engine, verify):
        while any(r.done < total_of(r) for r in batch):
            call = []
            for r in batch:
                total = total_of(r)
                if r.done >= total:
                    continue
                remaining = total - r.done
                if verify and remaining <= self.chunk:     # the rest of the uncached tokens and all drafts
                    n, k, last = remaining, r.k, True
                else:                                      # tokens forwarded for their KV only
                    n, k, last = min(self.chunk, remaining - (r.k if verify else 0)), 1, False
                call.append(EngineItem(r.request_id, r.cached + r.done, n - k, k, r.done, last, tuple(r.pages)))
            accept = engine(call)
            for item, a in zip(call, accept):
                r = self.requests[item.request_id]
                n = item.n_uncached + item.n_draft
                if item.final_verify:
                    assert 0 <= a <= item.n_draft
                    r.cached += r.done + item.n_uncached + a
                    r.done = total_of(r)                   # submission consumed
                else:
                    r.done += n
            for r in batch:
                if r.done >= total_of(r) and (r.n_prompt or r.k):
                    if not verify:
                        r.cached += r.n_prompt
                    r.n_prompt = r.u = r.k = r.done = 0

    def execute_prefill(self, B_prefill, engine):
        self._engine_calls(B_prefill, lambda r: r.n_prompt, engine, verify=False)

    def execute_partialprefill(self, B_verify, L_uncached, engine):
        assert L_uncached == [r.u for r in B_verify]
        self._engine_calls(B_verify, lambda r: r.u + r.k, engine, verify=True)

    def remove_completed(self, B):
        keep = []
        for i in B:
            r = self.requests[i]
            if r.completed:
                self.free_pages.extend(r.pages)
                self.free_pages.sort()
                del self.requests[i]
            else:
                keep.append(i)
        return keep

    # ---- one pass of the algorithm's outer loop --------------------------------------------------
    def iteration(self, engine):
        """Returns "prefill", "verify" or "idle"."""
        B_prefill, B_verify = [], []
        R_new = self.get_next_prefill_request(B_prefill)
        while R_new is not None:
            B_prefill.append(R_new)
            R_new = self.get_next_prefill_request(B_prefill)

        if B_prefill:
            ids = [r.request_id for r in B_prefill]
            self.log.append(("prefill", ids, None))
            self.execute_prefill(B_prefill, engine)
            self.B = ids + self.B
            return "prefill"

        L_uncached = []
        R_verify = self.get_next_verification_request(B_verify)
        while R_verify is not None:
            B_verify.append(R_verify)
            L_uncached.append(R_verify.u)
            R_verify = self.get_next_verification_request(B_verify)

        kind = "idle"
        if B_verify:
            ids = [r.request_id for r in B_verify]
            self.log.append(("verify", ids, list(L_uncached)))
            self.execute_partialprefill(B_verify, L_uncached, engine)
            self.B = self.B + [i for i in ids if i not in self.B]
            kind = "verify"

        self.B = self.remove_completed(self.B)
        return kind
