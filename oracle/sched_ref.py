"""Reference model of the scheduler / block manager -- TEST INFRASTRUCTURE ONLY.

A plain, slow transcription of the engine iteration that arXiv 2602.07878 describes in
Sec. 5.1 ("Revisiting vLLM Scheduler"): FIFO free-block queue and persistent blocks
(Sec. 5.1.1), strict first-come-first-served admission that stops at the first request
that does not fit (Sec. 5.1.1, head-of-line blocking), last-in-first-out preemption with
the victim put at the front of the waiting queue and recovery by swapping or by
recomputation (Sec. 5.1.2).  With chunked=True the prefill of a request is spread over
iterations under the shared token budget (the paper's section "Effects of Chunked Prefill":
a fixed budget of tokens per iteration, prefill chunks interleaved with the decoding steps of
the other requests, KV-cache use rising chunk by chunk).  Python lists only; no code shared
with the C++ model.
"""
from __future__ import annotations

SWAP, RECOMPUTE = 0, 1


class Request:
    def __init__(self, rid, prompt, max_new):
        self.rid, self.prompt, self.max_new = rid, prompt, max_new
        self.generated = 0       # output tokens produced so far
        self.computed = 0        # tokens whose K/V sit in GPU blocks
        self.blocks = []         # physical GPU blocks, in logical order
        self.cpu_blocks = []     # host blocks while swapped out
        self.swapped = False
        self.prefilling = False  # chunked mode: part of the prompt is still to be prefilled
        self.target = 0          # ... up to this many tokens
        self.chunk = 0           # ... of which this many in the current iteration


class RefScheduler:
    def __init__(self, num_gpu_blocks, num_cpu_blocks, block_size, max_num_seqs,
                 max_num_batched_tokens, max_blocks_per_seq, watermark_blocks=0, mode=SWAP,
                 chunked=False):
        if chunked and max_num_batched_tokens < max_num_seqs:
            raise ValueError("the token budget must cover one decode token per running request")
        self.chunked = chunked
        self.bs = block_size
        self.max_seqs, self.budget = max_num_seqs, max_num_batched_tokens
        self.max_blocks, self.watermark, self.mode = max_blocks_per_seq, watermark_blocks, mode
        self.num_gpu_blocks = num_gpu_blocks
        self.free_gpu = list(range(num_gpu_blocks))     # FIFO: take from the front, return to the back
        self.free_cpu = list(range(num_cpu_blocks))
        self.waiting, self.running, self.known = [], [], set()
        self.totals = dict(steps=0, preemptions=0, swap_out=0, swap_in=0, recomputed=0,
                           finished=0, blocked=0, decoded=0)

    def add_request(self, rid, prompt, max_new):
        full = -(-(prompt + max_new - 1) // self.bs)      # blocks at full length
        # a request evicted at its full length returns only if its blocks fit beside the watermark
        if prompt < 1 or max_new < 1 or (prompt > self.budget and not self.chunked) \
                or full > self.max_blocks or full + self.watermark > self.num_gpu_blocks:
            raise ValueError("request can never run")
        if rid in self.known:
            raise KeyError(rid)
        self.known.add(rid)
        self.waiting.append(Request(rid, prompt, max_new))

    def _preempt(self, r, out):
        self.totals["preemptions"] += 1
        out["preempted"].append(r.rid)
        if self.mode == SWAP and len(self.free_cpu) >= len(r.blocks):
            for b in r.blocks:
                c = self.free_cpu.pop(0)
                out["swap_out"].append((b, c))
                r.cpu_blocks.append(c)
                self.free_gpu.append(b)
            self.totals["swap_out"] += len(r.blocks)
            r.swapped = True
        else:                                            # recomputation: the cache is dropped
            self.free_gpu.extend(r.blocks)
            r.computed = 0
            r.prefilling = False                         # it starts over when it is admitted again
        r.blocks = []
        self.waiting.insert(0, r)                        # front of the queue

    def _finish(self, r, out):
        self.free_gpu.extend(r.blocks)
        r.blocks = []
        out["finished"].append(r.rid)
        self.totals["finished"] += 1

    def step(self):
        if self.chunked:
            return self._step_chunked()
        out = dict(decode=[], prefill=[], preempted=[], swap_out=[], swap_in=[], finished=[],
                   head_blocked=False)
        self.totals["steps"] += 1
        # 1. a slot for the next token of every running request, in scheduling order
        i = 0
        while i < len(self.running):
            r = self.running[i]
            need = 1 if r.computed % self.bs == 0 else 0
            evicted_self = False
            while len(self.free_gpu) < need:
                victim = self.running.pop()              # most recently scheduled
                self._preempt(victim, out)
                if victim is r:
                    evicted_self = True
                    break
            if evicted_self:
                break
            if need:
                r.blocks.append(self.free_gpu.pop(0))
            i += 1
        # 2. first-come-first-served admission, unless this iteration had to preempt
        admitted = []
        if not out["preempted"]:
            budget = self.budget
            while self.waiting and len(self.running) + len(admitted) < self.max_seqs:
                r = self.waiting[0]
                if r.swapped:
                    nb = len(r.cpu_blocks)
                    if len(self.free_gpu) < nb + self.watermark:
                        out["head_blocked"] = True
                        break
                    for c in r.cpu_blocks:
                        g = self.free_gpu.pop(0)
                        out["swap_in"].append((c, g))
                        r.blocks.append(g)
                        self.free_cpu.append(c)
                    self.totals["swap_in"] += nb
                    r.cpu_blocks, r.swapped = [], False
                    self.waiting.pop(0)
                    admitted.append(r)
                    continue
                tokens = r.prompt if r.generated == 0 else r.prompt + r.generated - 1
                nb = -(-tokens // self.bs)
                # Sec. "Effects of Chunked Prefill": without chunking a prefill is atomic.  A
                # re-prefill that exceeds the budget of a whole iteration is not split and not
                # dropped: it is the only prefill of its iteration.
                oversized = r.generated > 0 and tokens > self.budget
                fits_budget = (budget == self.budget) if oversized else (tokens <= budget)
                if not fits_budget or len(self.free_gpu) < nb + self.watermark:
                    out["head_blocked"] = True
                    break
                r.blocks = [self.free_gpu.pop(0) for _ in range(nb)]
                r.computed = tokens
                budget = 0 if oversized else budget - tokens
                if r.generated == 0:
                    r.generated = 1                      # the prefill yields the first token
                else:
                    self.totals["recomputed"] += tokens
                out["prefill"].append((r.rid, tokens))
                self.waiting.pop(0)
                if r.generated >= r.max_new:
                    self._finish(r, out)
                else:
                    admitted.append(r)
        out["swap_in"].sort(key=lambda pair: pair[1])   # reported by ascending pool block
        if out["head_blocked"]:
            self.totals["blocked"] += 1
        # 3. one decode token for everything that was running before the admissions
        still = []
        for r in self.running:
            r.computed += 1
            out["decode"].append((r.rid, r.computed, list(r.blocks)))
            r.generated += 1
            self.totals["decoded"] += 1
            if r.generated >= r.max_new:
                self._finish(r, out)
            else:
                still.append(r)
        self.running = still + admitted
        out["free_blocks"] = len(self.free_gpu)
        out["running"], out["waiting"] = len(self.running), len(self.waiting)
        out["swapped"] = sum(1 for r in self.waiting if r.swapped)
        return out

    def _step_chunked(self):
        """The iteration with chunked prefill.  One token budget per iteration pays for the
        decode tokens (one per decoding request) and for prefill chunks.  prefill records are
        (request, tokens of the chunk, cached tokens after it): first the chunks of requests
        already running, in running order, then the admissions."""
        out = dict(decode=[], prefill=[], preempted=[], swap_out=[], swap_in=[], finished=[],
                   head_blocked=False)
        self.totals["steps"] += 1
        # decode tokens come first in the budget: one per running request that decodes
        budget = self.budget - sum(1 for r in self.running if not r.prefilling)
        # 1. in scheduling order, every running request reserves what it needs this iteration:
        #    a decoding one the slot of its next token, a prefilling one the blocks of its next
        #    chunk (as much of the rest of its prompt as the budget still allows)
        i = 0
        while i < len(self.running):
            r = self.running[i]
            if r.prefilling:
                r.chunk = min(r.target - r.computed, budget)
                need = -(-(r.computed + r.chunk) // self.bs) - len(r.blocks)
                cost = r.chunk
            else:
                need = 1 if r.computed % self.bs == 0 else 0
                cost = 0
            evicted_self = False
            while len(self.free_gpu) < need:
                victim = self.running.pop()
                self._preempt(victim, out)
                if victim is r:
                    evicted_self = True
                    break
            if evicted_self:
                break
            for _ in range(need):
                r.blocks.append(self.free_gpu.pop(0))
            budget -= cost
            i += 1
        # 2. admission from the head of the waiting queue, unless this iteration had to preempt
        admitted, admitted_records = [], []
        if not out["preempted"]:
            while self.waiting and len(self.running) + len(admitted) < self.max_seqs:
                r = self.waiting[0]
                if r.swapped:
                    nb = len(r.cpu_blocks)
                    if len(self.free_gpu) < nb + self.watermark:
                        out["head_blocked"] = True
                        break
                    for c in r.cpu_blocks:
                        g = self.free_gpu.pop(0)
                        out["swap_in"].append((c, g))
                        r.blocks.append(g)
                        self.free_cpu.append(c)
                    self.totals["swap_in"] += nb
                    r.cpu_blocks, r.swapped = [], False
                    r.chunk = 0
                    self.waiting.pop(0)
                    admitted.append(r)
                    continue
                total = r.prompt if r.generated == 0 else r.prompt + r.generated - 1
                chunk = min(total, budget)
                nb = -(-chunk // self.bs)
                if chunk == 0 or len(self.free_gpu) < nb + self.watermark:
                    out["head_blocked"] = True
                    break
                r.blocks = [self.free_gpu.pop(0) for _ in range(nb)]
                r.target, r.computed, r.chunk = total, chunk, 0
                budget -= chunk
                if r.generated > 0:
                    self.totals["recomputed"] += chunk
                admitted_records.append((r.rid, chunk, chunk))
                self.waiting.pop(0)
                r.prefilling = chunk < total
                if not r.prefilling and r.generated == 0:
                    r.generated = 1                      # the last chunk yields the first token
                if not r.prefilling and r.generated >= r.max_new:
                    self._finish(r, out)
                else:
                    admitted.append(r)
        out["swap_in"].sort(key=lambda pair: pair[1])
        if out["head_blocked"]:
            self.totals["blocked"] += 1
        # 3. the requests that were running before the admissions take their step
        still = []
        for r in self.running:
            if r.prefilling:
                if r.chunk > 0:
                    r.computed += r.chunk
                    if r.generated > 0:
                        self.totals["recomputed"] += r.chunk
                    out["prefill"].append((r.rid, r.chunk, r.computed))
                    if r.computed == r.target:
                        r.prefilling = False
                        if r.generated == 0:
                            r.generated = 1
                if not r.prefilling and r.generated >= r.max_new:
                    self._finish(r, out)
                else:
                    still.append(r)
                continue
            r.computed += 1
            out["decode"].append((r.rid, r.computed, list(r.blocks)))
            r.generated += 1
            self.totals["decoded"] += 1
            if r.generated >= r.max_new:
                self._finish(r, out)
            else:
                still.append(r)
        out["prefill"].extend(admitted_records)
        self.running = still + admitted
        out["free_blocks"] = len(self.free_gpu)
        out["running"], out["waiting"] = len(self.running), len(self.waiting)
        out["swapped"] = sum(1 for r in self.waiting if r.swapped)
        return out
