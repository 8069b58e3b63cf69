"""Scheduler / block-manager model: the Python reference (oracle/sched_ref.py) pinned to what
the paper fixes (Sec. 5.1.1: FIFO free queue, persistent blocks, strict FCFS admission with
head-of-line blocking; Sec. 5.1.2: LIFO victim, victim to the front of the queue, swap or
recompute recovery) by hand-worked traces and invariants, then the C++ library held to the
reference, iteration by iteration and bit for bit.  CPU only."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle.sched_ref import RefScheduler, SWAP, RECOMPUTE
from paper_2602_07878_amd import binding, sched, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def ref(**kw):
    d = dict(num_gpu_blocks=4, num_cpu_blocks=4, block_size=2, max_num_seqs=8,
             max_num_batched_tokens=64, max_blocks_per_seq=8, watermark_blocks=0, mode=RECOMPUTE)
    d.update(kw)
    return RefScheduler(**d)


# ---- pins of the reference ------------------------------------------------------------------
def test_head_of_line_blocking_small_request_waits_behind_a_big_one():
    s = ref(block_size=4)
    s.add_request(1, 8, 100 - 91)      # 2 blocks
    s.add_request(2, 12, 4)            # 3 blocks: does not fit beside request 1
    s.add_request(3, 4, 4)             # 1 block: would fit, but is behind request 2
    o = s.step()
    assert o["prefill"] == [(1, 8)] and o["head_blocked"] and o["waiting"] == 2
    assert o["free_blocks"] == 2       # capacity for request 3 is there, and stays unused
    o = s.step()
    assert [d[0] for d in o["decode"]] == [1] and o["prefill"] == [] and o["head_blocked"]


def test_hand_worked_trace_lifo_victim_goes_to_the_front_and_is_recomputed():
    s = ref()                          # 4 blocks of 2 tokens, recompute mode
    for rid in (1, 2, 3):
        s.add_request(rid, 2, 6)       # 7 tokens at full length: the whole pool
    o = s.step()                       # all three prefilled: blocks 0, 1, 2; block 3 free
    assert o["prefill"] == [(1, 2), (2, 2), (3, 2)] and o["decode"] == [] and o["free_blocks"] == 1
    s.add_request(4, 2, 6)             # arrives before the victim is preempted
    o = s.step()
    # every request needs a second block: 1 takes block 3; for 2 the pool is empty, so the most
    # recently scheduled request (3) is evicted and its block 2 serves request 2
    assert o["preempted"] == [3]
    assert o["decode"] == [(1, 3, [0, 3]), (2, 3, [1, 2])]
    assert o["prefill"] == [] and o["free_blocks"] == 0          # no admission while preempting
    assert [r.rid for r in s.waiting] == [3, 4]                   # victim ahead of the newcomer
    o = s.step()                       # nobody needs a block; request 3 cannot come back yet
    assert o["decode"] == [(1, 4, [0, 3]), (2, 4, [1, 2])] and o["head_blocked"] and not o["preempted"]
    o = s.step()                       # request 1 needs a third block: victim is request 2
    assert o["preempted"] == [2] and o["decode"] == [(1, 5, [0, 3, 1])] and o["free_blocks"] == 1
    assert [r.rid for r in s.waiting] == [2, 3, 4]
    o = s.step()                       # request 2 (3 generated tokens) needs prompt + 2 = 4 tokens = 2 blocks
    assert o["head_blocked"] and o["decode"] == [(1, 6, [0, 3, 1])]
    assert s.totals["recomputed"] == 0


def test_recompute_prefills_prompt_plus_generated_minus_one_and_resumes_decoding():
    s = ref(num_gpu_blocks=3)
    s.add_request(1, 2, 3)
    s.add_request(2, 2, 4)
    s.step()                           # both prefilled (blocks 0, 1), block 2 free, generated = 1 each
    o = s.step()                       # 1 takes block 2; 2 finds none and is evicted itself
    assert o["preempted"] == [2] and o["decode"] == [(1, 3, [0, 2])]
    o = s.step()                       # request 2 returns into its old block: it had produced 1 token,
    assert o["prefill"] == [(2, 2)]    # so prompt + 1 - 1 tokens are prefilled again;
    assert o["finished"] == [1] and o["decode"] == [(1, 4, [0, 2])]   # request 1 ends with its third token
    o = s.step()
    assert o["decode"] == [(2, 3, [1, 0])]   # request 2 goes on where it stopped: context 3
    assert s.totals["recomputed"] == 2 and s.totals["preemptions"] == 1


def test_swap_moves_blocks_out_and_back_to_other_physical_blocks():
    s = ref(mode=SWAP)
    for rid in (1, 2, 3):
        s.add_request(rid, 2, 6)
    s.step()
    o = s.step()
    assert o["preempted"] == [3] and o["swap_out"] == [(2, 0)]    # pool block 2 -> host block 0
    assert s.waiting[0].rid == 3 and s.waiting[0].swapped and s.waiting[0].computed == 2
    for _ in range(2):
        o = s.step()
    assert o["preempted"] == [2] and o["swap_out"] == [(1, 1), (2, 2)]
    # request 1 runs to its end (6 tokens), then the victims return in queue order: 2, then 3
    seen_in = []
    for _ in range(12):
        o = s.step()
        seen_in += o["swap_in"]
    # request 2 (host blocks 1, 2) is served first and gets pool blocks 0 and 3, the first two
    # that request 1 gave back; request 3 (host block 0) gets the next one; pairs are reported
    # by ascending pool block
    assert seen_in[:3] == [(1, 0), (0, 1), (2, 3)]
    assert s.totals["swap_in"] == s.totals["swap_out"] and s.totals["recomputed"] == 0


def test_swap_without_host_space_falls_back_to_recomputation():
    s = ref(mode=SWAP, num_cpu_blocks=0)
    for rid in (1, 2, 3):
        s.add_request(rid, 2, 6)
    s.step()
    o = s.step()
    assert o["preempted"] == [3] and o["swap_out"] == [] and s.waiting[0].computed == 0


def test_requests_that_can_never_run_are_refused():
    s = ref()
    with pytest.raises(ValueError):
        s.add_request(1, 9, 1)         # 5 blocks at full length > pool of 4
    with pytest.raises(ValueError):
        s.add_request(1, 65, 1)        # prompt above the token budget
    s.add_request(1, 2, 2)
    with pytest.raises(KeyError):
        s.add_request(1, 2, 2)


def test_hand_worked_trace_recomputation_larger_than_the_budget_runs_alone():
    """Without chunking a prefill is atomic.  A victim whose prompt + generated - 1 tokens exceed
    the budget of a whole iteration must still come back (it sits at the head of the queue and
    would otherwise block it for ever): it is prefilled as the only prefill of an iteration."""
    s = ref(max_num_batched_tokens=2)  # 4 blocks of 2 tokens, recompute mode, budget = one prompt
    s.add_request(1, 2, 6)
    s.add_request(2, 2, 5)
    o = s.step()                       # request 1 uses the whole budget; request 2 waits for the next iteration
    assert o["prefill"] == [(1, 2)] and o["head_blocked"] and o["free_blocks"] == 3
    o = s.step()                       # 1 grows into block 1; 2 is prefilled into block 2
    assert o["prefill"] == [(2, 2)] and o["decode"] == [(1, 3, [0, 1])] and o["free_blocks"] == 1
    o = s.step()                       # 2 grows into block 3: the pool is full
    assert o["decode"] == [(1, 4, [0, 1]), (2, 3, [2, 3])] and o["free_blocks"] == 0
    o = s.step()                       # 1 needs a third block: the last scheduled request (2) is evicted
    assert o["preempted"] == [2] and o["decode"] == [(1, 5, [0, 1, 2])] and o["free_blocks"] == 1
    o = s.step()                       # 2 has 2 output tokens: 2 + 2 - 1 = 3 tokens = 2 blocks, only 1 free
    assert o["head_blocked"] and o["prefill"] == [] and o["decode"] == [(1, 6, [0, 1, 2])]
    s.add_request(3, 2, 2)             # a newcomer queues behind the victim
    o = s.step()                       # 1 takes the last block and ends with its sixth token
    assert o["decode"] == [(1, 7, [0, 1, 2, 3])] and o["finished"] == [1] and o["free_blocks"] == 4
    o = s.step()                       # 3 tokens > budget 2: admitted alone; 3 would fit the pool but waits
    assert o["prefill"] == [(2, 3)] and o["head_blocked"] and o["free_blocks"] == 2
    assert [r.rid for r in s.waiting] == [3] and s.totals["recomputed"] == 3
    o = s.step()                       # 2 decodes where it stopped (context 4); 3 is prefilled
    assert o["decode"] == [(2, 4, [0, 1])] and o["prefill"] == [(3, 2)]
    for _ in range(3):
        o = s.step()
    assert s.totals["finished"] == 3 and not s.running and not s.waiting
    assert s.totals["decoded"] == 5 + 4 + 1


def test_a_request_that_could_not_return_beside_the_watermark_is_refused():
    """Evicted at full length a request needs all its blocks plus the watermark to be admitted
    again; if the pool cannot give that, it would block the head of the queue for ever."""
    kw = dict(num_gpu_blocks=8, block_size=16, max_num_batched_tokens=128, watermark_blocks=2)
    s = ref(**kw)
    with pytest.raises(ValueError):
        s.add_request(1, 120, 1)       # 8 blocks + 2 > 8
    with pytest.raises(ValueError):
        s.add_request(1, 90, 8)        # 97 tokens at full length: 7 blocks + 2 > 8
    s.add_request(1, 96, 1)            # 6 blocks + 2 = 8: runs at once
    o = s.step()
    assert o["prefill"] == [(1, 96)] and o["finished"] == [1] and not o["head_blocked"]
    L = sched.Scheduler(mode=RECOMPUTE, num_cpu_blocks=0, max_num_seqs=8, max_blocks_per_seq=8, **kw)
    with pytest.raises(binding.PkvError):
        L.add_request(1, 120, 1)
    with pytest.raises(binding.PkvError):
        L.add_request(1, 90, 8)
    L.add_request(1, 96, 1)
    assert L.step().num_finished == 1


@pytest.mark.parametrize("mode,budget,chunked", [(RECOMPUTE, 256, False), (SWAP, 256, False), (RECOMPUTE, 64, True)])
def test_liveness_an_idle_engine_always_admits_the_head(mode, budget, chunked):
    """Whatever the load did before: when nothing runs and the whole pool is free, the request
    at the head of the queue is admitted in that iteration, and every request finishes."""
    total = 48
    s = ref(num_gpu_blocks=total, num_cpu_blocks=8, block_size=16, max_num_seqs=12, max_num_batched_tokens=budget,
            max_blocks_per_seq=40, watermark_blocks=2, mode=mode, chunked=chunked)
    stream = W.poisson_request_stream(21, 300, 0.3, prompt_median=100, out_median=150, max_prompt=256, max_new=380)
    submitted, oversized, steps = 0, 0, 0
    while steps < len(stream) or ((s.running or s.waiting) and steps < 60000):
        arrivals = stream[steps] if steps < len(stream) else []
        steps += 1
        for rid, p, n in arrivals:
            s.add_request(rid, p, n)
            submitted += 1
        idle = not s.running and len(s.free_gpu) == total and bool(s.waiting)
        o = s.step()
        if idle:
            assert o["prefill"] or o["swap_in"], "idle engine left the head of the queue waiting"
        if not chunked:
            oversized += sum(1 for _, t in o["prefill"] if t > budget)
    assert s.totals["finished"] == submitted and not s.running and not s.waiting
    assert s.totals["preemptions"] > 0
    if mode == RECOMPUTE and not chunked:
        assert oversized > 0           # the load did produce recomputations beyond the budget


# ---- properties the paper states, over seeded loads ------------------------------------------
@pytest.mark.parametrize("mode", [SWAP, RECOMPUTE])
@pytest.mark.parametrize("seed", [31, 32, 33])
def test_paper_properties_persistent_blocks_victim_first_and_recompute_length(mode, seed):
    """Sec. 5.1.1: a running request keeps its blocks until it finishes, so between finishes and
    preemptions the number of free blocks never rises.  Sec. 5.1.2: the victim goes to the front
    of the waiting queue, so no request that has never run is admitted while a victim waits; a
    recomputed request re-processes its prompt and all previously generated tokens (all but the
    newest, whose K/V the next decode step writes)."""
    s = ref(num_gpu_blocks=64, num_cpu_blocks=24, block_size=16, max_num_seqs=16, max_num_batched_tokens=2048,
            max_blocks_per_seq=40, mode=mode)
    stream = W.poisson_request_stream(seed, 400, 0.25, prompt_median=96, out_median=120, max_prompt=256, max_new=300)
    prompts, decoded, ran_before, victims_waiting = {}, {}, set(), set()
    free_before, steps = 64, 0
    while steps < len(stream) or ((s.running or s.waiting) and steps < 60000):
        arrivals = stream[steps] if steps < len(stream) else []
        steps += 1
        for rid, p, n in arrivals:
            s.add_request(rid, p, n)
            prompts[rid] = p
        o = s.step()
        if not o["finished"] and not o["preempted"]:
            assert o["free_blocks"] <= free_before
        free_before = o["free_blocks"]
        for rid, tokens in o["prefill"]:
            if rid in ran_before:      # a recomputation
                assert tokens == prompts[rid] + (1 + decoded.get(rid, 0)) - 1
            victims_waiting.discard(rid)
        back = {r.rid for r in s.running}
        victims_waiting -= back
        newcomers = [rid for rid, _ in o["prefill"] if rid not in ran_before]
        if newcomers:
            assert not victims_waiting, "a newcomer was admitted while a victim was waiting"
        ran_before |= {rid for rid, _ in o["prefill"]}
        for rid, _, _ in o["decode"]:
            decoded[rid] = decoded.get(rid, 0) + 1
        victims_waiting |= set(o["preempted"])
    assert s.totals["preemptions"] > 0 and s.totals["finished"] == len(prompts)


# ---- chunked prefill (the paper's section "Effects of Chunked Prefill") ---------------------------
def test_chunked_hand_worked_trace_long_prompt_in_chunks_beside_a_decoding_request():
    s = ref(num_gpu_blocks=8, block_size=4, max_num_seqs=4, max_num_batched_tokens=8, chunked=True)
    s.add_request(1, 3, 10)
    o = s.step()                       # whole prompt in one chunk: block 0
    assert o["prefill"] == [(1, 3, 3)] and o["free_blocks"] == 7
    s.add_request(2, 20, 3)            # 2.5 budgets long: impossible without chunking
    o = s.step()                       # the decode token of request 1 costs 1 of the 8: chunk of 7 -> blocks 1, 2
    assert o["decode"] == [(1, 4, [0])] and o["prefill"] == [(2, 7, 7)] and o["free_blocks"] == 5
    o = s.step()                       # request 1 grows into block 3; next 7 tokens -> 14 cached, blocks 4, 5
    assert o["decode"] == [(1, 5, [0, 3])] and o["prefill"] == [(2, 7, 14)] and o["free_blocks"] == 2
    o = s.step()                       # the last 6 tokens: 20 cached, block 6; this chunk yields the first token
    assert o["decode"] == [(1, 6, [0, 3])] and o["prefill"] == [(2, 6, 20)] and o["free_blocks"] == 1
    o = s.step()                       # now both decode; request 2 starts a new block at 20 = 5 * 4 tokens
    assert o["decode"] == [(1, 7, [0, 3]), (2, 21, [1, 2, 4, 5, 6, 7])] and o["prefill"] == [] and o["free_blocks"] == 0
    # request 1 decoded in every iteration (no compute-bound stall behind the long prompt), and
    # the cache use rose chunk by chunk: 7, 5, 2, 1, 0 blocks free
    assert s.totals["decoded"] == 5 and s.totals["preemptions"] == 0


def test_chunked_running_chunks_are_reported_before_admissions_of_the_same_iteration():
    s = ref(num_gpu_blocks=8, block_size=4, max_num_seqs=4, max_num_batched_tokens=8, chunked=True)
    s.add_request(1, 10, 5)
    o = s.step()
    assert o["prefill"] == [(1, 8, 8)] and o["free_blocks"] == 6
    s.add_request(2, 3, 5)
    o = s.step()                       # the last 2 tokens of request 1 (block 2), then request 2 whole (block 3)
    assert o["prefill"] == [(1, 2, 10), (2, 3, 3)] and o["decode"] == [] and o["free_blocks"] == 4
    o = s.step()
    assert o["decode"] == [(1, 11, [0, 1, 2]), (2, 4, [3])]


def test_chunked_without_chunking_the_long_prompt_is_refused():
    s = ref(num_gpu_blocks=8, block_size=4, max_num_seqs=4, max_num_batched_tokens=8)
    with pytest.raises(ValueError):
        s.add_request(2, 20, 3)
    with pytest.raises(ValueError):    # the budget must pay one decode token per running request
        ref(max_num_seqs=8, max_num_batched_tokens=4, chunked=True)


def test_chunked_partial_prefill_is_the_lifo_victim_and_starts_over_under_recompute():
    s = ref(num_gpu_blocks=4, block_size=2, max_num_seqs=4, max_num_batched_tokens=4, chunked=True)
    s.add_request(1, 2, 6)
    s.add_request(2, 6, 2)
    o = s.step()                       # request 1 whole (block 0), request 2 gets the 2 tokens left: block 1
    assert o["prefill"] == [(1, 2, 2), (2, 2, 2)] and o["free_blocks"] == 2
    s.add_request(3, 2, 2)             # waits: the budget of this iteration is used up by then
    o = s.step()                       # request 1 takes block 2; the chunk of 3 needs 2 blocks, 1 is free:
    assert o["preempted"] == [2] and o["prefill"] == []          # the last scheduled request goes: itself
    assert o["decode"] == [(1, 3, [0, 2])] and o["free_blocks"] == 2 and s.waiting[0].computed == 0
    assert [r.rid for r in s.waiting] == [2, 3]                  # ... to the front of the queue
    o = s.step()                       # it starts over: 3 tokens (budget 4 - 1 decode) into blocks 3, 1
    assert o["prefill"] == [(2, 3, 3)] and o["decode"] == [(1, 4, [0, 2])] and o["free_blocks"] == 0
    o = s.step()                       # request 1 needs a third block: victim is request 2 again
    assert o["preempted"] == [2] and o["decode"] == [(1, 5, [0, 2, 3])] and o["free_blocks"] == 1
    assert s.totals["recomputed"] == 0                           # it never produced a token


def test_chunked_swap_keeps_the_progress_of_a_partial_prefill():
    s = ref(num_gpu_blocks=4, num_cpu_blocks=4, block_size=2, max_num_seqs=4, max_num_batched_tokens=4,
            chunked=True, mode=SWAP)
    s.add_request(1, 2, 4)
    s.add_request(2, 6, 1)
    s.step()                           # request 1: block 0; request 2: 2 of 6 tokens, block 1
    o = s.step()                       # request 2 cannot get the 2 blocks of its next chunk: swapped out
    assert o["preempted"] == [2] and o["swap_out"] == [(1, 0)] and s.waiting[0].computed == 2
    o = s.step()                       # back at once (1 block), into pool block 3; no chunk in this iteration
    assert o["swap_in"] == [(0, 3)] and o["prefill"] == [] and o["decode"] == [(1, 4, [0, 2])]
    o = s.step()                       # request 1 takes the last block, request 2 is squeezed out again;
    assert o["preempted"] == [2] and o["swap_out"] == [(3, 1)]   # request 1 ends with its fourth token
    assert o["finished"] == [1] and o["free_blocks"] == 4
    o = s.step()
    assert o["swap_in"] == [(1, 3)] and o["prefill"] == []
    o = s.step()                       # the remaining 4 tokens in one chunk; max_new = 1: done
    assert o["prefill"] == [(2, 4, 6)] and o["finished"] == [2]
    assert s.totals["recomputed"] == 0 and s.totals["swap_in"] == s.totals["swap_out"] == 2


@pytest.mark.parametrize("mode", [SWAP, RECOMPUTE])
def test_chunked_invariants_under_overload(mode):
    total, budget = 64, 96
    s = ref(num_gpu_blocks=total, num_cpu_blocks=48, block_size=16, max_num_seqs=16,
            max_num_batched_tokens=budget, max_blocks_per_seq=32, mode=mode, chunked=True)
    stream = W.poisson_request_stream(6, 400, 0.25, prompt_median=96, out_median=96, max_prompt=256, max_new=200)
    submitted = sum(len(a) for a in stream)
    prompts = {rid: p for a in stream for rid, p, _ in a}
    prefilled = {}

    def check(o):
        owned = [b for r in s.running for b in r.blocks]
        assert len(owned) == len(set(owned)) and sorted(owned + s.free_gpu) == list(range(total))
        assert len(o["decode"]) + sum(t for _, t, _ in o["prefill"]) <= budget      # one budget for both
        for r in s.running:
            assert len(r.blocks) == -(-r.computed // 16)
            assert r.prefilling == (r.computed < r.target) or not r.prefilling
        for rid, tok, ctx in o["prefill"]:
            assert 0 < tok <= ctx
            prefilled[rid] = prefilled.get(rid, 0) + tok
        assert not (o["preempted"] and o["swap_in"])

    drive(s, stream, 4000, check)
    assert s.totals["finished"] == submitted and not s.running and not s.waiting
    assert s.totals["preemptions"] > 0
    assert s.totals["decoded"] == sum(n - 1 for a in stream for _, _, n in a)
    if mode == SWAP:                   # with host space for every victim no token is prefilled twice
        assert s.totals["recomputed"] == 0 or s.totals["swap_out"] > 0
    assert all(prefilled[rid] >= p for rid, p in prompts.items())


def drive(s, stream, extra_steps, on_step):
    for arrivals in stream:
        for rid, p, n in arrivals:
            s.add_request(rid, p, n)
        on_step(s.step())
    for _ in range(extra_steps):
        on_step(s.step())


@pytest.mark.parametrize("mode", [SWAP, RECOMPUTE])
def test_invariants_under_overload(mode):
    total = 64
    s = ref(num_gpu_blocks=total, num_cpu_blocks=48, block_size=16, max_num_seqs=16,
            max_num_batched_tokens=2048, max_blocks_per_seq=32, mode=mode)
    stream = W.poisson_request_stream(5, 400, 0.25, prompt_median=96, out_median=96, max_prompt=256, max_new=200)
    submitted = sum(len(a) for a in stream)
    order_admitted, first_seen = [], set()

    def check(o):
        owned = [b for r in s.running for b in r.blocks]
        assert len(owned) == len(set(owned))                          # no block has two owners
        assert sorted(owned + s.free_gpu) == list(range(total))       # none lost, none invented
        host = [c for r in s.waiting for c in r.cpu_blocks]
        assert sorted(host + s.free_cpu) == list(range(48))
        for r in s.running:
            assert len(r.blocks) == -(-r.computed // 16) and r.computed == r.prompt + r.generated - 1
        for rid, ctx, blocks in o["decode"]:
            assert len(blocks) == -(-ctx // 16)
        assert not (o["preempted"] and (o["prefill"] or o["swap_in"]))
        for rid, _ in o["prefill"]:
            if rid not in first_seen:
                first_seen.add(rid)
                order_admitted.append(rid)

    drive(s, stream, 3000, check)
    assert order_admitted == sorted(order_admitted)                   # first admissions in arrival order
    assert s.totals["finished"] == submitted and not s.running and not s.waiting
    assert s.totals["preemptions"] > 0 and s.totals["blocked"] > 0    # the load did saturate the pool
    assert s.totals["decoded"] == sum(n - 1 for a in stream for _, _, n in a)   # every token exactly once
    if mode == SWAP:
        assert s.totals["swap_in"] == s.totals["swap_out"] > 0


# ---- the C++ library against the reference -------------------------------------------------
def test_header_and_library_agree_on_the_exported_names():
    src = open(os.path.join(ROOT, "include", "pkv_sched.h")).read()
    names = sorted(set(re.findall(r"\b(pkv_sched_[a-z_]+)\s*\(", src)))
    assert names == sorted(sched.SCHED_EXPORTS)
    L = binding.lib()
    for n in names:
        assert hasattr(L, n), n


def test_create_rejects_bad_configurations_and_getters_check_capacity():
    L = sched._lib()
    assert not L.pkv_sched_create(None)
    bad = sched.SchedConfig(0, 0, 16, 4, 64, 8, 0, 0, 0)
    assert not L.pkv_sched_create(ctypes.byref(bad))
    bad = sched.SchedConfig(8, 0, 16, 4, 64, 8, 0, 2, 0)
    assert not L.pkv_sched_create(ctypes.byref(bad))
    bad = sched.SchedConfig(8, 0, 16, 4, 64, 8, 0, 0, 2)            # chunked_prefill is 0 or 1
    assert not L.pkv_sched_create(ctypes.byref(bad))
    bad = sched.SchedConfig(8, 0, 16, 8, 4, 8, 0, 0, 1)             # budget below the decode tokens
    assert not L.pkv_sched_create(ctypes.byref(bad))
    s = sched.Scheduler(num_gpu_blocks=4, num_cpu_blocks=4, block_size=2, max_num_seqs=8,
                        max_num_batched_tokens=64, max_blocks_per_seq=8, mode=sched.RECOMPUTE)
    with pytest.raises(binding.PkvError):
        s.add_request(1, 9, 1)
    s.add_request(1, 2, 5)
    with pytest.raises(binding.PkvError):
        s.add_request(1, 2, 5)
    s.step(); s.step()
    assert L.pkv_sched_decode_batch(s._h, None, None, None, 0) == -2
    assert L.pkv_sched_decode_batch(s._h, None, None, None, 1) == 1
    assert L.pkv_sched_step(None, None) == 1
    with pytest.raises(binding.PkvError):
        s.request_blocks(12345)


@pytest.mark.parametrize("mode,seed,cpu_blocks,chunked,budget", [
    (SWAP, 11, 64, False, 1024), (RECOMPUTE, 12, 0, False, 1024), (SWAP, 13, 6, False, 1024),
    (SWAP, 14, 64, True, 128), (RECOMPUTE, 15, 0, True, 96), (SWAP, 16, 6, True, 64),
    (RECOMPUTE, 17, 0, False, 400), (SWAP, 18, 6, False, 400)])   # recomputations beyond the budget
def test_library_reproduces_the_reference_trace_exactly(mode, seed, cpu_blocks, chunked, budget):
    kw = dict(num_gpu_blocks=96, num_cpu_blocks=cpu_blocks, block_size=16, max_num_seqs=24,
              max_num_batched_tokens=budget, max_blocks_per_seq=40, watermark_blocks=1, chunked=chunked)
    r = RefScheduler(mode=mode, **kw)
    s = sched.Scheduler(mode=mode, **kw)
    stream = W.poisson_request_stream(seed, 300, 0.3, prompt_median=120, out_median=100, max_prompt=400, max_new=200)
    stream += [[] for _ in range(2500)]
    oversized = 0
    for arrivals in stream:
        for rid, p, n in arrivals:
            r.add_request(rid, p, n)
            s.add_request(rid, p, n)
        o, info = r.step(), s.step()
        ids, lens, tabs = s.decode_batch()
        assert [d[0] for d in o["decode"]] == ids.tolist() and [d[1] for d in o["decode"]] == lens.tolist()
        for row, (_, _, blocks) in zip(tabs, o["decode"]):
            assert row[:len(blocks)].tolist() == blocks and np.all(row[len(blocks):] == -1)
        assert [tuple(p) for p in s.swap_out().tolist()] == o["swap_out"]
        assert [tuple(p) for p in s.swap_in().tolist()] == o["swap_in"]
        pid, ptok = s.prefills()
        if chunked:
            assert list(zip(pid.tolist(), ptok.tolist(), s.prefill_contexts().tolist())) == o["prefill"]
        else:
            assert list(zip(pid.tolist(), ptok.tolist())) == o["prefill"]
            assert s.prefill_contexts().tolist() == ptok.tolist()
            oversized += sum(1 for t in ptok.tolist() if t > budget)
        for q in r.running:
            assert s.request_blocks(q.rid).tolist() == q.blocks
        for q in r.waiting[:3]:
            assert s.request_blocks(q.rid).size == 0
        assert s.finished().tolist() == o["finished"]
        assert (info.free_blocks, info.running, info.waiting, info.swapped, info.head_blocked, info.num_preempted) == \
               (o["free_blocks"], o["running"], o["waiting"], o["swapped"], int(o["head_blocked"]), len(o["preempted"]))
    assert s.totals() == r.totals and r.totals["preemptions"] > 0 and r.totals["finished"] > 0
    if budget == 400 and mode == RECOMPUTE:
        assert oversized > 0           # the trace covers recomputations beyond the budget
