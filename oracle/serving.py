"""TEST INFRASTRUCTURE -- oracle for serving inside the task graph (paper Section 6.1, "supporting
runtime dynamism": continuous batching and a paged KV cache; a task on the graph's start event
prepares each decoding iteration by (1) removing completed requests, (2) admitting newly arrived
ones and (3) updating the per-request KV-cache metadata, which attention tasks read from device
memory).

Three parts, each the plain definition written out:

PagedDecoderOracle   the decoder oracle with its cache kept in pages.  A page table maps
                     (sequence, row // page_size) to a page of a per-layer pool
                     [n_pages][n_kv][page_size][d]; a step gathers the rows a sequence owns into
                     the contiguous form the layer function takes, runs the very same layer
                     function, and puts the appended row back into its page.  Paging is pure
                     indirection: the result is bit-identical to the contiguous oracle for ANY
                     page table that gives every (sequence, block) a page of its own.

ServeState           the start-event task as a state machine over slots (one slot per batch row),
                     a FIFO queue of requests, and a stack of free pages.  The paper names the three
                     steps and fixes no policy; the policy here is this library's contract:
                       * a request is (prompt tokens, max_new_tokens); it is finished when it has
                         produced max_new_tokens tokens or the end-of-sequence token.  Prompts are
                         consumed one token per iteration through the decode path (the sampled
                         token is ignored while prompt tokens remain): prefill is not a separate
                         kernel here.
                       * retire: slots in ascending order; a finished request gives its pages
                         back in page-table order (pushed onto the free stack).
                       * compact: the requests still running move, in order, to the lowest slots
                         (a slot is only metadata -- the rows stay in their pages), so the
                         running requests always occupy slots 0 .. n-1 and a task graph compiled
                         for fewer slots can serve them.
                       * admit: free slots in ascending order take requests in arrival order; a
                         request is admitted only if the pages it can ever need,
                         ceil((prompt_len + max_new - 1) / page_size), are free and not promised
                         to running requests.  The first request that does not fit stops admission
                         for the iteration (no overtaking).
                       * metadata: a running slot whose position reaches a page boundary pops one
                         page (ascending slot order); an idle slot computes on token 0 at position
                         0 in a page reserved for it (page number = slot number), so the graph of
                         the full batch runs whatever the number of live requests.

ServingOracle        ServeState + PagedDecoderOracle + greedy sampling: whole iterations.

Nothing here is imported by the GPU library.
"""
from __future__ import annotations

import numpy as np

from .decoder import DecoderOracle

BF16_NAN = 0x7FC0
PENDING, RUNNING, DONE = 0, 1, 2


class PagedDecoderOracle(DecoderOracle):
    """provider.kv_pool(l) -> (K, V) uint16 [n_pages][n_kv][page_size][d] (copied, then owned).
    Set `page_table` (int [B][max_seq // page_size]) before every step."""

    def __init__(self, shape, provider, page_size, prec="f32", n_layers=None):
        super().__init__(shape, provider, prec, n_layers)
        assert shape.max_seq % page_size == 0
        self.ps = int(page_size)
        self.page_table = None
        self.pool = {}

    def _kv(self, l):
        if l not in self.pool:
            k, v = self.p.kv_pool(l)
            self.pool[l] = (np.ascontiguousarray(k).copy(), np.ascontiguousarray(v).copy())
        return self.pool[l]

    def _rows_in(self, l, b, Kp, Vp, pos):
        s, ps = self.s, self.ps
        # rows the sequence does not own yet read as NaN: a read past `pos` would show
        Kc = np.full((s.n_kv_heads, s.max_seq, s.head_dim), BF16_NAN, np.uint16)
        Vc = np.full_like(Kc, BF16_NAN)
        for t in range(pos):
            page = int(self.page_table[b][t // ps])
            Kc[:, t, :] = Kp[page, :, t % ps, :]
            Vc[:, t, :] = Vp[page, :, t % ps, :]
        return Kc, Vc

    def _rows_out(self, l, b, Kc, Vc, pos):
        Kp, Vp = self.pool[l]
        page = int(self.page_table[b][pos // self.ps])
        Kp[page, :, pos % self.ps, :] = Kc[:, pos, :]
        Vp[page, :, pos % self.ps, :] = Vc[:, pos, :]


class Request:
    def __init__(self, prompt, max_new):
        self.prompt = [int(t) for t in prompt]
        self.max_new = int(max_new)
        self.out = []
        self.state = PENDING


class ServeState:
    """The metadata the start-event task keeps, and its three steps (see the module header)."""

    def __init__(self, batch, page_size, n_pages, max_seq, eos):
        assert n_pages > batch and max_seq % page_size == 0
        self.B, self.ps, self.n_pages, self.max_seq, self.eos = batch, page_size, n_pages, max_seq, eos
        self.max_blocks = max_seq // page_size
        self.slot_req = [-1] * batch          # request in the slot, -1 = idle
        self.slot_pos = [0] * batch           # rows cached = position of the token fed this iteration
        self.slot_next = [0] * batch          # token fed this iteration
        self.slot_held = [0] * batch          # pages the slot's request holds
        self.table = [[-1] * self.max_blocks for _ in range(batch)]
        for b in range(batch):
            self.table[b][0] = b              # the slot's own idle page
        # free stack: pop takes the last element; the lowest page number comes out first
        self.free = list(range(n_pages - 1, batch - 1, -1))
        self.promised = 0                     # pages running requests may still ask for
        self.requests = []
        self.q_head = 0                       # next request to admit

    # ---- host side
    def need(self, r):
        q = self.requests[r]
        return -(-(len(q.prompt) + q.max_new - 1) // self.ps)

    def submit(self, prompt, max_new):
        assert len(prompt) >= 1 and max_new >= 1
        assert len(prompt) + max_new - 1 <= self.max_seq
        self.requests.append(Request(prompt, max_new))
        assert self.need(len(self.requests) - 1) <= self.n_pages - self.B
        return len(self.requests) - 1

    # ---- the start-event task
    def begin_iteration(self, sampled):
        """sampled[b]: the token the previous iteration sampled for slot b (ignored for idle
        slots and while the slot still has prompt tokens to feed).  Returns the iteration's
        (tokens[B], positions[B]); self.table holds its page tables."""
        B, ps = self.B, self.ps
        # (1) completed requests leave
        for b in range(B):
            r = self.slot_req[b]
            if r < 0:
                continue
            q = self.requests[r]
            cached = self.slot_pos[b] + 1
            if cached < len(q.prompt):
                nxt = q.prompt[cached]
            else:
                tok = int(sampled[b])
                q.out.append(tok)
                nxt = tok
                if tok == self.eos or len(q.out) == q.max_new:
                    for i in range(self.slot_held[b]):
                        self.free.append(self.table[b][i])
                        self.table[b][i] = -1
                    self.promised -= self.need(r) - self.slot_held[b]
                    self.table[b][0] = b
                    self.slot_req[b], self.slot_held[b] = -1, 0
                    q.state = DONE
                    continue
            self.slot_pos[b], self.slot_next[b] = cached, nxt
        # (1b) the running requests close ranks
        running = [b for b in range(B) if self.slot_req[b] >= 0]
        for dst, src in enumerate(running):
            if dst == src:
                continue
            held = self.slot_held[src]
            self.slot_req[dst], self.slot_pos[dst] = self.slot_req[src], self.slot_pos[src]
            self.slot_next[dst], self.slot_held[dst] = self.slot_next[src], held
            self.table[dst] = self.table[src][:held] + [-1] * (self.max_blocks - held)
            self.slot_req[src], self.slot_held[src] = -1, 0
            self.table[src] = [src] + [-1] * (self.max_blocks - 1)
        # (2) arrivals enter, in order, while their pages are there
        for b in range(B):
            if self.slot_req[b] >= 0:
                continue
            if self.q_head == len(self.requests):
                break
            r = self.q_head
            if len(self.free) - self.promised < self.need(r):
                break
            self.q_head += 1
            self.requests[r].state = RUNNING
            self.slot_req[b], self.slot_pos[b], self.slot_held[b] = r, 0, 0
            self.slot_next[b] = self.requests[r].prompt[0]
            self.promised += self.need(r)
        # (3) metadata of the iteration
        tokens, positions = [0] * B, [0] * B
        for b in range(B):
            if self.slot_req[b] < 0:
                continue
            if self.slot_pos[b] % ps == 0:
                self.table[b][self.slot_pos[b] // ps] = self.free.pop()
                self.slot_held[b] += 1
                self.promised -= 1
            tokens[b], positions[b] = self.slot_next[b], self.slot_pos[b]
        return tokens, positions

    def n_running(self):
        return sum(r >= 0 for r in self.slot_req)

    def drained(self):
        """Nothing running and nothing queued (after an iteration's start-event task)."""
        return self.n_running() == 0 and self.q_head == len(self.requests)

    def snapshot(self):
        """The state as plain integers (what a device-side implementation must reproduce)."""
        return {"slot_req": list(self.slot_req),
                "slot_pos": [p if r >= 0 else 0 for p, r in zip(self.slot_pos, self.slot_req)],
                "slot_held": list(self.slot_held),
                "table": [list(row) for row in self.table],
                "free": list(self.free), "promised": self.promised, "q_head": self.q_head}


class ServingOracle:
    """Whole serving iterations on the CPU: start-event task, one decode step of the full batch
    through the page tables, greedy sampling."""

    def __init__(self, shape, provider, page_size, n_pages, eos, prec="f32"):
        self.state = ServeState(shape.batch, page_size, n_pages, shape.max_seq, eos)
        self.dec = PagedDecoderOracle(shape, provider, page_size, prec)
        self.sampled = [0] * shape.batch
        self.last_logits = None

    def submit(self, prompt, max_new):
        return self.state.submit(prompt, max_new)

    def iteration(self):
        tokens, positions = self.state.begin_iteration(self.sampled)
        self.dec.page_table = self.state.table
        lg = self.dec.step(tokens, positions)
        self.sampled = [self.dec.ops.argmax(lg[b]) for b in range(len(tokens))]
        self.last_logits = lg
        return tokens, positions

    def launch(self, n):
        """One launch of up to n iterations: the kernel runs until its workload is done (paper
        Section 5), i.e. the iteration whose start-event task finds nothing running and nothing
        queued is the launch's last.  Returns the number of iterations run."""
        for i in range(n):
            self.iteration()
            if self.state.drained():
                return i + 1
        return n

    def outputs(self, r):
        q = self.state.requests[r]
        return list(q.out), q.state
