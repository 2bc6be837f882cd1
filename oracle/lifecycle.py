"""Exact definition of the closed-loop request life cycle (TEST INFRASTRUCTURE ONLY).

Sections 4.4, 4.5.1 and 4.5.2 of the paper: a request first waits for KV blocks (the decode side
owns the only cache manager and sizes a prompt's blocks from its length), its block ids go to the
prefill side, which serves prompts first come first served and never chunks them; completion of
the prefill is a notification, after which the request joins the running decode batch; blocks are
released when the request ends or is preempted.

Readings where the paper is silent:
  * a prompt's prefill yields the request's first output token; every decode step one more;
  * a request ends with its max_new-th token or with the end-of-sequence token, which it keeps;
  * one prefill pass is in flight at a time; it takes, in arrival order, as many whole prompts as
    fit the prefill token budget (at least one, never part of one); the decode batch is capped and
    filled in arrival order;
  * when a running request's next token has no block, the most recently arrived request that
    holds blocks and is not being prefilled at that moment (possibly the starved request itself)
    is preempted: its blocks are released, it waits again at its original place in the arrival
    order, and its next prefill covers prompt + tokens generated so far (recomputation); if the
    starved request is the only block holder the pool is simply too small;
  * here every sampled token is visible to the scheduler at the next step (no lag).

Hybrid batching (`hybrid_chunk` > 0; section 3.1 describes the scheme the paper compares with: a
prompt is cut into chunks of 512 or 1024 tokens and every chunk shares a batch with the running
decode tokens).  Readings: `hybrid_chunk` is a step's budget of prompt tokens (the decode rows come on
top); prompts are served first come first served and the budget is filled in that order -- the
rest of the prompt in progress first, then the next prompts that have their blocks, the last of
them possibly in part; a part that is not the end of its prompt is a multiple of 16 tokens (so that
every later part starts on a block boundary), which may leave a few tokens of the budget unused; at
most `max_prefill_reqs` prompts have a part in one step; these parts and the decode step of all
running requests form one batch; the step that takes a prompt's last part also yields its first
output token, which the scheduler sees at the next step, after that step's decode tokens; a request
with a part taken and its first token not yet seen is "being prefilled" for the preemption rule.
Everything else -- block accounting, promotion, retirement, preemption -- is unchanged, so the
tokens a request receives are the same under either policy.

The tokens themselves come from outside: `script[req]` is the sequence of tokens the request's
successive sampling events yield (a missing entry yields 0).  Everything is integer and exact.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Tuple

from .kv_alloc import KVAllocator, NoBlocks

WAITING, PREFILL_READY, PREFILLING, PREFILL_DONE, RUNNING, FINISHED = range(6)


class _Req:
    def __init__(self, rid, prompt_len, max_new, script):
        self.id, self.prompt_len, self.max_new = rid, prompt_len, max_new
        self.script = list(script)
        self.events = 0          # sampling events consumed
        self.out: List[int] = []
        self.state = WAITING
        self.n_prefill = prompt_len
        self.ctx = 0
        self.complete = False


class Lifecycle:
    def __init__(self, n_blocks: int, max_batch: int, eos: int = -1,
                 split: Optional[Callable[[int, int, bool], Tuple[int, int]]] = None,
                 max_prefill_tokens: int = 1 << 30, max_prefill_reqs: int = 64, hybrid_chunk: int = 0):
        self.max_prefill_tokens, self.max_prefill_reqs = max_prefill_tokens, max_prefill_reqs
        self.hybrid_chunk = hybrid_chunk
        self.hyb_cur: Optional[int] = None   # the prompt of which a part, not yet the last, has been taken
        self.chunk_done = 0                  # tokens of that prompt that earlier steps took
        self.hyb_finishing: List[int] = []   # prompts whose last part the previous step took
        self.alloc = KVAllocator(n_blocks)
        self.max_batch, self.eos = max_batch, eos
        self.split = split
        self.reqs: Dict[int, _Req] = {}
        self.arrival: List[int] = []
        self.running: List[int] = []
        self.prefilling: List[int] = []      # the prompts of the pass in flight
        self.pass_done = False
        self.last_tokens: List[int] = []   # requests whose decode-step token is still to be read

    def submit(self, rid: int, prompt_len: int, max_new: int, script=()):
        self.reqs[rid] = _Req(rid, prompt_len, max_new, script)
        self.arrival.append(rid)

    def complete_prefill(self, rid: int):
        """The pass that contains rid has finished."""
        assert self.reqs[rid].state == PREFILLING and rid in self.prefilling
        self.pass_done = True

    def _sample(self, r: _Req):
        tok = r.script[r.events] if r.events < len(r.script) else 0
        r.events += 1
        if r.complete:
            return
        r.out.append(tok)
        if tok == self.eos or len(r.out) >= r.max_new:
            r.complete = True

    def _finish(self, r: _Req):
        r.state = FINISHED
        if r.id in self.alloc.owned:
            self.alloc.release(r.id)

    def step(self) -> dict:
        o = dict(n_promoted=0, n_finished=0, n_preempted=0, prefill_started_req=-1, prefill_started_tokens=0)
        for rid in self.last_tokens:                       # tokens of the previous decode step
            self._sample(self.reqs[rid])
        self.last_tokens = []
        for rid in self.hyb_finishing:                     # hybrid batching: first tokens of the previous step
            r = self.reqs[rid]
            r.state, r.ctx = PREFILL_DONE, r.n_prefill
            self._sample(r)
            if r.complete:
                self._finish(r)
                o["n_finished"] += 1
        self.hyb_finishing = []
        if self.prefilling and self.pass_done:
            self.pass_done = False
            for rid in self.prefilling:
                r = self.reqs[rid]
                r.state, r.ctx = PREFILL_DONE, r.n_prefill
                self._sample(r)
                if r.complete:
                    self._finish(r)
                    o["n_finished"] += 1
            self.prefilling = []
        for rid in list(self.running):
            if self.reqs[rid].complete:
                self._finish(self.reqs[rid])
                self.running.remove(rid)
                o["n_finished"] += 1
        while self.arrival and self.reqs[self.arrival[0]].state == FINISHED:
            self.arrival.pop(0)
        for rid in self.arrival:
            r = self.reqs[rid]
            if r.state == PREFILL_DONE and len(self.running) < self.max_batch:
                r.state = RUNNING
                self.running.append(rid)
                o["n_promoted"] += 1
        for rid in self.arrival:
            r = self.reqs[rid]
            if r.state != WAITING:
                continue
            try:
                self.alloc.alloc(rid, r.n_prefill)
            except NoBlocks:
                break
            r.state = PREFILL_READY
        while True:                                        # room for every running request's next token
            stuck = None
            for rid in self.running:
                try:
                    self.alloc.alloc(rid, self.reqs[rid].ctx + 1)
                except NoBlocks:
                    stuck = rid
                    break
            if stuck is None:
                break
            v = next(self.reqs[rid] for rid in reversed(self.arrival)
                     if self.reqs[rid].state in (RUNNING, PREFILL_DONE, PREFILL_READY))
            if v.id == stuck and all(not b for rid, b in self.alloc.owned.items() if rid != stuck):
                raise NoBlocks()
            if v.state == RUNNING:
                self.running.remove(v.id)
            self.alloc.release(v.id)
            v.state, v.n_prefill, v.ctx = WAITING, v.prompt_len + len(v.out), 0
            o["n_preempted"] += 1
        o["n_waiting"] = sum(1 for rid in self.arrival if self.reqs[rid].state == WAITING)
        if self.hybrid_chunk:
            return self._hybrid_tail(o)
        nxt: List[int] = []
        if not self.prefilling:
            total = 0
            for rid in self.arrival:
                r = self.reqs[rid]
                if r.state != PREFILL_READY:
                    continue
                if nxt and (total + r.n_prefill > self.max_prefill_tokens or len(nxt) >= self.max_prefill_reqs):
                    break
                nxt.append(rid)
                total += r.n_prefill
        pending = bool(self.prefilling) or bool(nxt)
        o["decode_batch"] = len(self.running)
        o["decode_sum_ctx"] = sum(self.reqs[rid].ctx for rid in self.running)
        o["batch_ids"] = list(self.running)
        p_cus = 256
        if self.split is not None and (self.running or pending):
            p_cus, d_cus = self.split(len(self.running), o["decode_sum_ctx"], pending)
            o["split"] = (p_cus, d_cus)
        for rid in self.running:                           # the decode step
            self.reqs[rid].ctx += 1
        self.last_tokens = list(self.running)
        o["prefill_started_count"] = 0
        if nxt and p_cus > 0:
            for rid in nxt:
                self.reqs[rid].state = PREFILLING
            self.prefilling = nxt
            o["prefill_started_req"] = nxt[0]
            o["prefill_started_tokens"] = sum(self.reqs[rid].n_prefill for rid in nxt)
            o["prefill_started_count"] = len(nxt)
            o["prefill_started_ids"] = list(nxt)
        return o

    def _hybrid_tail(self, o: dict) -> dict:
        """The rest of a step under hybrid batching: the prompt parts and the decode step, one batch."""
        o["prefill_started_count"] = 0
        o["decode_batch"] = len(self.running)
        o["decode_sum_ctx"] = sum(self.reqs[rid].ctx for rid in self.running)
        o["batch_ids"] = list(self.running)
        chunks: List[Tuple[int, int, int]] = []
        budget = self.hybrid_chunk
        while budget > 0 and len(chunks) < self.max_prefill_reqs:
            rid = self.hyb_cur
            if rid is None:                                # the next prompt that has its blocks, if any
                rid = next((q for q in self.arrival if self.reqs[q].state == PREFILL_READY), None)
                if rid is None:
                    break
            r = self.reqs[rid]
            done = self.chunk_done if self.hyb_cur is not None else 0
            rest = r.n_prefill - done
            n = min(budget, rest)
            if n < rest:
                n -= n % 16
            if n == 0:                                     # what is left of the budget is less than a block
                break
            if self.hyb_cur is None:                       # taken up with its first part
                r.state = PREFILLING
                self.hyb_cur, self.chunk_done = rid, 0
                if o["prefill_started_req"] < 0:
                    o["prefill_started_req"] = rid
                o["prefill_started_tokens"] += r.n_prefill
                o["prefill_started_count"] += 1
                o.setdefault("prefill_started_ids", []).append(rid)
                o.setdefault("prefill_started_lens", []).append(r.n_prefill)
            chunks.append((rid, done, n))
            self.chunk_done += n
            budget -= n
            if self.chunk_done == r.n_prefill:
                self.hyb_finishing.append(rid)             # its first token is seen at the next step
                self.hyb_cur = None
        o["chunks"] = chunks
        for rid in self.running:                           # the decode rows of the same batch
            self.reqs[rid].ctx += 1
        self.last_tokens = list(self.running)
        return o
