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
    waiting: object = None             # the submission waiting in a queue: _Work, or None
    running: bool = False              # a submission of this request is being executed


@dataclass
class _Work:
    """One submission of a request: a prompt (u = n_prompt, k = 0) or a verification (u uncached, k drafts)."""
    r: _Request
    u: int
    k: int
    verify: bool
    done: int = 0                      # tokens already forwarded

    @property
    def total(self):
        return self.u + self.k


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
        r = _Request(request_id)
        r.waiting = _Work(r, n_prompt, 0, verify=False)
        self.requests[request_id] = r
        self.prefill_queue.append(r.waiting)

    def submit_verify(self, request_id, u, k):
        r = self.requests.get(request_id)
        if r is None or request_id not in self.B or r.completed or u < 0 or k < 1 or k > self.chunk:
            raise ValueError("bad verification request")
        if r.waiting is not None or r.running:
            raise ValueError("request already has a verification pending")
        if self._pages_for(r.cached + u + k) > min(self.max_pages_per_request, self.n_pages):
            raise MemoryError("request can never fit")
        r.waiting = _Work(r, u, k, verify=True)
        self.verify_queue.append(r.waiting)

    def finish(self, request_id):
        r = self.requests[request_id]
        if request_id not in self.B or r.waiting is not None or r.running:
            raise ValueError("request still has work pending")
        r.completed = True

    # ---- the two fetch operations of the algorithm, with the admission rule ---------------------
    def _get_next(self, queue, batch):
        """Head of the queue if batch, token and page limits allow it (it then gets the pages for the
        request's whole new length), else nothing: no overtaking."""
        if not queue:
            return None
        w = queue[0]
        if len(batch) + 1 > self.max_batch:
            return None
        if sum(min(self.chunk, q.total) for q in batch) + min(self.chunk, w.total) > self.max_tokens:
            return None
        need = self._pages_for(w.r.cached + w.total) - len(w.r.pages)
        if need > len(self.free_pages):
            return None
        for _ in range(max(need, 0)):
            w.r.pages.append(self.free_pages.pop(0))
        w.r.waiting, w.r.running = None, True
        return queue.popleft()

    def get_next_prefill_request(self, B_prefill):
        return self._get_next(self.prefill_queue, B_prefill)

    def get_next_verification_request(self, B_verify):
        return self._get_next(self.verify_queue, B_verify)

    # ---- execution: fixed chunks through the engine ---------------------------------------------
    def _engine_calls(self, batch, engine):
        while any(w.done < w.total for w in batch):
            call = []
            for w in batch:
                remaining = w.total - w.done
                if remaining == 0:
                    continue
                if w.verify and remaining <= self.chunk:   # the rest of the uncached tokens and all drafts
                    n, k, last = remaining, w.k, True
                else:                                      # tokens forwarded for their KV only
                    n, k, last = min(self.chunk, remaining - w.k), 1, False
                call.append((w, EngineItem(w.r.request_id, w.r.cached + w.done, n - k, k, w.done, last,
                                           tuple(w.r.pages))))
            accept = engine([item for _, item in call])
            for (w, item), a in zip(call, accept):
                w.done += item.n_uncached + item.n_draft
                if w.done == w.total:                      # submission consumed
                    if item.final_verify:
                        assert 0 <= a <= w.k
                        w.r.cached += w.u + a
                    else:
                        w.r.cached += w.u
                    w.r.running = False

    def execute_prefill(self, B_prefill, engine):
        self._engine_calls(B_prefill, engine)

    def execute_partialprefill(self, B_verify, L_uncached, engine):
        assert L_uncached == [w.u for w in B_verify]
        self._engine_calls(B_verify, engine)

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
            ids = [w.r.request_id for w in B_prefill]
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
            ids = [w.r.request_id for w in B_verify]
            self.log.append(("verify", ids, list(L_uncached)))
            self.execute_partialprefill(B_verify, L_uncached, engine)
            self.B = self.B + [i for i in ids if i not in self.B]
            kind = "verify"

        self.B = self.remove_completed(self.B)
        return kind
