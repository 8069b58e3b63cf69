"""ctypes binding of the scheduler / block-manager model (pkv_sched.h).  Marshalling only:
every decision is taken in the C++ library."""
from __future__ import annotations

import ctypes

import numpy as np

from . import binding

SWAP, RECOMPUTE = 0, 1

SCHED_EXPORTS = [
    "pkv_sched_create", "pkv_sched_destroy", "pkv_sched_add_request", "pkv_sched_step",
    "pkv_sched_decode_batch", "pkv_sched_swap_out", "pkv_sched_swap_in", "pkv_sched_prefills",
    "pkv_sched_finished", "pkv_sched_request_blocks", "pkv_sched_totals", "pkv_sched_prefill_contexts",
]

TOTALS = ("steps", "preemptions", "swap_out", "swap_in", "recomputed", "finished", "blocked", "decoded")


class SchedConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "num_gpu_blocks", "num_cpu_blocks", "block_size", "max_num_seqs", "max_num_batched_tokens",
        "max_blocks_per_seq", "watermark_blocks", "preemption_mode", "chunked_prefill")]


class StepInfo(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "num_decode", "num_prefill", "num_prefill_tokens", "num_preempted", "num_swap_out_blocks",
        "num_swap_in_blocks", "num_finished", "free_blocks", "running", "waiting", "swapped",
        "head_blocked")]


_ready = False


def _lib():
    global _ready
    L = binding.lib()
    if not _ready:
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.pkv_sched_create.restype = vp
        L.pkv_sched_create.argtypes = [ctypes.POINTER(SchedConfig)]
        L.pkv_sched_destroy.restype = None
        L.pkv_sched_destroy.argtypes = [vp]
        L.pkv_sched_add_request.restype = i32
        L.pkv_sched_add_request.argtypes = [vp, i64, i32, i32]
        L.pkv_sched_step.restype = i32
        L.pkv_sched_step.argtypes = [vp, ctypes.POINTER(StepInfo)]
        L.pkv_sched_decode_batch.restype = i32
        L.pkv_sched_decode_batch.argtypes = [vp, vp, vp, vp, i32]
        for name in ("pkv_sched_swap_out", "pkv_sched_swap_in", "pkv_sched_finished", "pkv_sched_prefill_contexts"):
            getattr(L, name).restype = i32
            getattr(L, name).argtypes = [vp, vp, i32]
        L.pkv_sched_prefills.restype = i32
        L.pkv_sched_prefills.argtypes = [vp, vp, vp, i32]
        L.pkv_sched_request_blocks.restype = i32
        L.pkv_sched_request_blocks.argtypes = [vp, i64, vp, i32]
        L.pkv_sched_totals.restype = i32
        L.pkv_sched_totals.argtypes = [vp, vp]
        _ready = True
    return L


class Scheduler:
    """One scheduler instance.  `step()` runs an engine iteration and returns its StepInfo; the
    arrays of that iteration are read with decode_batch(), swap_out(), swap_in(), ..."""

    def __init__(self, *, num_gpu_blocks, num_cpu_blocks, block_size, max_num_seqs,
                 max_num_batched_tokens, max_blocks_per_seq, watermark_blocks=0, mode=SWAP, chunked=False):
        self.cfg = SchedConfig(num_gpu_blocks, num_cpu_blocks, block_size, max_num_seqs,
                               max_num_batched_tokens, max_blocks_per_seq, watermark_blocks, mode,
                               1 if chunked else 0)
        self._h = _lib().pkv_sched_create(ctypes.byref(self.cfg))
        if not self._h:
            raise ValueError("invalid scheduler configuration")

    def close(self):
        if self._h:
            _lib().pkv_sched_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def add_request(self, rid: int, prompt_len: int, max_new_tokens: int):
        st = _lib().pkv_sched_add_request(self._h, rid, prompt_len, max_new_tokens)
        if st != binding.PKV_OK:
            raise binding.PkvError(st, "pkv_sched_add_request")

    def step(self) -> StepInfo:
        info = StepInfo()
        st = _lib().pkv_sched_step(self._h, ctypes.byref(info))
        if st != binding.PKV_OK:
            raise binding.PkvError(st, "pkv_sched_step")
        self._info = info
        return info

    def decode_batch(self):
        """(request ids int64 [B], context_lens int32 [B], block_tables int32 [B, max_blocks])."""
        n = self._info.num_decode
        ids = np.empty(n, np.int64)
        lens = np.empty(n, np.int32)
        tabs = np.empty((n, self.cfg.max_blocks_per_seq), np.int32)
        got = _lib().pkv_sched_decode_batch(self._h, ids.ctypes.data, lens.ctypes.data, tabs.ctypes.data, n)
        assert got == n, got
        return ids, lens, tabs

    def _pairs(self, fn, n):
        m = np.empty((n, 2), np.int32)
        got = fn(self._h, m.ctypes.data, n)
        assert got == n, got
        return m

    def swap_out(self):
        """[n, 2] int32 (pool block, host block) pairs of the last iteration."""
        return self._pairs(_lib().pkv_sched_swap_out, self._info.num_swap_out_blocks)

    def swap_in(self):
        """[n, 2] int32 (host block, pool block) pairs of the last iteration."""
        return self._pairs(_lib().pkv_sched_swap_in, self._info.num_swap_in_blocks)

    def prefills(self):
        n = self._info.num_prefill
        ids, tok = np.empty(n, np.int64), np.empty(n, np.int32)
        got = _lib().pkv_sched_prefills(self._h, ids.ctypes.data, tok.ctypes.data, n)
        assert got == n, got
        return ids, tok

    def prefill_contexts(self):
        """Cached tokens of each prefill record's request after this iteration (int32 array)."""
        n = self._info.num_prefill
        ctx = np.empty(n, np.int32)
        got = _lib().pkv_sched_prefill_contexts(self._h, ctx.ctypes.data, n)
        assert got == n, got
        return ctx

    def finished(self):
        n = self._info.num_finished
        ids = np.empty(n, np.int64)
        got = _lib().pkv_sched_finished(self._h, ids.ctypes.data, n)
        assert got == n, got
        return ids

    def request_blocks(self, rid: int):
        """Pool blocks of a live request in logical order (int32 array)."""
        b = np.empty(self.cfg.max_blocks_per_seq, np.int32)
        n = _lib().pkv_sched_request_blocks(self._h, rid, b.ctypes.data, b.size)
        if n < 0:
            raise binding.PkvError(-n, "pkv_sched_request_blocks")
        return b[:n].copy()

    def totals(self) -> dict:
        t = np.zeros(8, np.int64)
        st = _lib().pkv_sched_totals(self._h, t.ctypes.data)
        assert st == binding.PKV_OK
        return dict(zip(TOTALS, (int(x) for x in t)))
