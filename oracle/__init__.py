"""fp64 CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product path (the HIP library and its binding) never does.
The arithmetic lives in ``pkv_oracle.c`` (plain C, fp64, straight from the
definition); this file only compiles it with gcc and marshals numpy arrays.

bfloat16 tensors are passed as ``numpy.uint16`` arrays holding the raw bits.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pkv_oracle.c")
_LIB = os.path.join(_HERE, "libpkv_oracle.so")
_lock = threading.Lock()
_lib = None

F32, BF16, F8E4M3 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile pkv_oracle.c into libpkv_oracle.so next to it (gcc, OpenMP)."""
    with _lock:
        stale = (not os.path.exists(_LIB)
                 or os.path.getmtime(_LIB) < os.path.getmtime(_SRC))
        if force or stale:
            tmp = _LIB + f".tmp{os.getpid()}"
            subprocess.check_call(
                ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                 "-ffp-contract=off", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
            os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32, i64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
        lib.orc_paged_decode_attention.restype = ctypes.c_int
        lib.orc_paged_decode_attention.argtypes = (
            [i32] * 8 + [i64] * 6 + [vp] * 5 + [ctypes.c_float, vp, vp, i32])
        lib.orc_paged_decode_attention_kv.restype = ctypes.c_int
        lib.orc_paged_decode_attention_kv.argtypes = (
            [i32] * 9 + [ctypes.c_float] * 2 + [i64] * 6 + [vp] * 5 + [ctypes.c_float, vp, vp, i32])
        lib.orc_kv_block_swap.restype = ctypes.c_int
        lib.orc_kv_block_swap.argtypes = [i32, i64, i64, i64, i32, i32, vp, vp, vp, i32]
        lib.orc_kv_append.restype = ctypes.c_int
        lib.orc_kv_append.argtypes = [i32] * 7 + [i64] * 6 + [vp] * 6
        lib.orc_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.uint8:
        return F8E4M3
    raise TypeError(f"oracle takes float32, uint16 (bf16 bits) or uint8 (e4m3 codes), got {a.dtype}")


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def paged_decode_attention(q, k_pool, v_pool, block_tables, context_lens, scale,
                           *, block_size, k_strides=None, v_strides=None,
                           return_weights=False, k_scale=1.0, v_scale=1.0):
    """out[i,h,:] = softmax_t(scale * q[i,h] . K_t) @ V over the paged pool.

    The pools may be 8-bit (numpy.uint8 holding OCP E4M3 codes) beside a bfloat16 q; K and V are
    then k_scale / v_scale times the stored values.

    q [B,Hq,D]; k_pool/v_pool [num_blocks,Hkv,bs,D] C-contiguous unless
    element strides (block, head, token) are given, in which case the pools may
    be any 1-D/N-D contiguous buffers and ``Hkv`` is taken from ``k_pool.shape[1]``.
    Returns float64 [B,Hq,D] (and the weights [B,Hq,max_ctx] when asked).
    """
    lib = _load()
    q = np.ascontiguousarray(q)
    k_pool = np.ascontiguousarray(k_pool)
    v_pool = np.ascontiguousarray(v_pool)
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    cl = np.ascontiguousarray(context_lens, dtype=np.int32)
    code = _dtype_code(q)
    kv_code = _dtype_code(k_pool)
    if _dtype_code(v_pool) != kv_code or (kv_code != code and (kv_code, code) != (F8E4M3, BF16)):
        raise TypeError("q, k_pool, v_pool must share one dtype, or be bf16 with 8-bit pools")
    B, Hq, D = q.shape
    nblk, Hkv = k_pool.shape[0], k_pool.shape[1]
    if k_strides is None:
        assert k_pool.shape == (nblk, Hkv, block_size, D), k_pool.shape
        k_strides = (Hkv * block_size * D, block_size * D, D)
    if v_strides is None:
        assert v_pool.shape == (nblk, Hkv, block_size, D), v_pool.shape
        v_strides = (Hkv * block_size * D, block_size * D, D)
    assert bt.ndim == 2 and bt.shape[0] == B and cl.shape == (B,)
    out = np.empty((B, Hq, D), dtype=np.float64)
    max_ctx = int(cl.max()) if (return_weights and B > 0) else 0
    w = np.zeros((B, Hq, max_ctx), dtype=np.float64) if return_weights else None
    rc = lib.orc_paged_decode_attention_kv(
        B, Hq, Hkv, D, block_size, nblk, bt.shape[1], code, kv_code,
        float(np.float32(k_scale)), float(np.float32(v_scale)),
        *[int(x) for x in k_strides], *[int(x) for x in v_strides],
        _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(bt), _ptr(cl),
        float(np.float32(scale)), _ptr(out), _ptr(w) if w is not None else None,
        max_ctx)
    if rc != 0:
        raise IndexError(f"oracle: index outside pool/table (code {rc})")
    return (out, w) if return_weights else out


def kv_block_swap(src, dst, mapping, *, num_planes, block_bytes,
                  src_plane_stride=None, dst_plane_stride=None,
                  src_num_blocks=None, dst_num_blocks=None):
    """Bytewise block copy src -> dst (uint8 views, dst modified in place)."""
    lib = _load()
    s8 = src.reshape(-1).view(np.uint8)
    d8 = dst.reshape(-1).view(np.uint8)
    assert s8.flags.c_contiguous and d8.flags.c_contiguous and d8.flags.writeable
    mp = np.ascontiguousarray(mapping, dtype=np.int32).reshape(-1, 2)
    if src_plane_stride is None:
        src_plane_stride = s8.size // num_planes
    if dst_plane_stride is None:
        dst_plane_stride = d8.size // num_planes
    if src_num_blocks is None:
        src_num_blocks = src_plane_stride // block_bytes
    if dst_num_blocks is None:
        dst_num_blocks = dst_plane_stride // block_bytes
    assert (num_planes - 1) * src_plane_stride + src_num_blocks * block_bytes <= s8.size
    assert (num_planes - 1) * dst_plane_stride + dst_num_blocks * block_bytes <= d8.size
    rc = lib.orc_kv_block_swap(num_planes, block_bytes, src_plane_stride,
                               dst_plane_stride, src_num_blocks, dst_num_blocks,
                               _ptr(s8), _ptr(d8), _ptr(mp), mp.shape[0])
    if rc != 0:
        raise IndexError("oracle: mapping entry outside its plane")
    return dst


def kv_append(k_pool, v_pool, k_new, v_new, block_tables, context_lens, *, block_size,
              k_strides=None, v_strides=None):
    """Write row k_new[i], v_new[i] ([B,Hkv,D]) at token position context_lens[i]-1 of
    every sequence (pools modified in place; same layout rules as the attention oracle)."""
    lib = _load()
    assert k_pool.flags.c_contiguous and v_pool.flags.c_contiguous
    assert k_pool.flags.writeable and v_pool.flags.writeable
    k_new = np.ascontiguousarray(k_new)
    v_new = np.ascontiguousarray(v_new)
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    cl = np.ascontiguousarray(context_lens, dtype=np.int32)
    code = _dtype_code(k_pool)
    if {_dtype_code(v_pool), _dtype_code(k_new), _dtype_code(v_new)} != {code}:
        raise TypeError("pools and new rows must share one dtype")
    B, Hkv, D = k_new.shape
    nblk = k_pool.shape[0]
    if k_strides is None:
        assert k_pool.shape == (nblk, Hkv, block_size, D), k_pool.shape
        k_strides = (Hkv * block_size * D, block_size * D, D)
    if v_strides is None:
        assert v_pool.shape == (nblk, Hkv, block_size, D), v_pool.shape
        v_strides = (Hkv * block_size * D, block_size * D, D)
    assert bt.ndim == 2 and bt.shape[0] == B and cl.shape == (B,)
    rc = lib.orc_kv_append(B, Hkv, D, block_size, nblk, bt.shape[1], k_pool.itemsize,
                           *[int(x) for x in k_strides], *[int(x) for x in v_strides],
                           _ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool), _ptr(bt), _ptr(cl))
    if rc != 0:
        raise IndexError(f"oracle: append outside pool/table (code {rc})")
    return k_pool, v_pool


def kv_append_chunk(k_pool, v_pool, k_new, v_new, block_tables, context_lens, query_lens, *, block_size):
    """The K/V rows of a prefill chunk join the cache (Sec. 2.2 "KV-Cache"; Sec. 2.1 prefill):
    k_new, v_new are packed [total, Hkv, D] in sequence order; row j of sequence i's
    query_lens[i] rows goes to token position context_lens[i] - query_lens[i] + j (the chunk is the
    tail of the context, as in paged_prefill_attention; query_lens above the context are clipped).
    Pools [blocks, Hkv, block_size, D], modified in place.  Plain loops."""
    first = 0
    for i, (n, q) in enumerate(zip(context_lens.tolist(), query_lens.tolist())):
        ql = min(q, n)
        for j in range(ql):
            pos = n - ql + j
            blk = int(block_tables[i, pos // block_size])
            if not 0 <= blk < k_pool.shape[0]:
                raise IndexError("oracle: chunk row outside the pool")
            k_pool[blk, :, pos % block_size, :] = k_new[first + j]
            v_pool[blk, :, pos % block_size, :] = v_new[first + j]
        first += q
    return k_pool, v_pool


def paged_prefill_attention(q, k_pool, v_pool, block_tables, context_lens, query_lens, scale,
                            *, block_size, k_strides=None, v_strides=None, k_scale=1.0, v_scale=1.0):
    """Causal attention of the last query_lens[i] tokens of every sequence over the paged cache
    (the prefill / re-prefill of the recompute recovery path, arXiv 2602.07878 Sec. 2.1 and
    Sec. 5.1.2: a token attends to itself and to everything before it).

    q is packed [sum(query_lens), Hq, D] in sequence order; context_lens[i] counts all cached
    tokens of sequence i INCLUDING those query_lens[i] tokens, whose K/V are already in the pool.
    Query token j of sequence i sits at position context_lens[i] - query_lens[i] + j and sees
    positions 0..that, which is exactly the decode definition with that many tokens: the
    function is written as one decode-oracle row per query token.  Returns float64 [sum, Hq, D].

    A query length above the context length is clipped, by the rule the library's header gives for
    this call and for kv_append_chunk: only the first min(query_lens[i], context_lens[i]) rows of
    sequence i exist (row j at position j then); the surplus rows have no definition and come back
    as NaN.
    """
    cl = np.ascontiguousarray(context_lens, dtype=np.int64)
    ql = np.ascontiguousarray(query_lens, dtype=np.int64)
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    assert cl.shape == ql.shape and np.all(ql >= 0) and np.all(cl >= 0)
    q = np.ascontiguousarray(q)
    assert q.shape[0] == int(ql.sum())
    live = np.minimum(ql, cl)                                          # rows of a sequence that exist
    rows_seq = np.repeat(np.arange(len(ql)), ql)                       # sequence of every query row
    first = np.cumsum(ql) - ql                                         # first packed row of a sequence
    j = np.arange(int(ql.sum())) - first[rows_seq]                     # index inside its sequence
    ctx = (cl[rows_seq] - live[rows_seq] + j + 1).astype(np.int32)     # tokens that row may see
    out = np.full(q.shape, np.nan, np.float64)
    keep = j < live[rows_seq]
    if keep.any():
        out[keep] = paged_decode_attention(q[keep], k_pool, v_pool, bt[rows_seq[keep]], ctx[keep], scale,
                                           block_size=block_size, k_strides=k_strides, v_strides=v_strides,
                                           k_scale=k_scale, v_scale=v_scale)
    return out
