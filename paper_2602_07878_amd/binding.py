"""Thin ctypes binding of libpkv.so: argument marshalling only.

Every step of the hot path runs in the HIP kernels of the library; PyTorch is
used for device memory and streams.  If the library has not been built this
module raises -- there is no fallback implementation.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpkv.so")

PKV_F32, PKV_BF16, PKV_F8_E4M3 = 0, 1, 2
PKV_OK = 0
PKV_ERR_HIP = 7
FLAG_VECTOR_ALU = 1

EXPORTS = [
    "pkv_version", "pkv_init", "pkv_static_scratch_bytes", "paged_decode_attention_static", "pkv_status_string", "pkv_last_hip_error_string", "pkv_attn_partition_tokens", "pkv_attn_workspace_bytes",
    "pkv_attn_plan_bytes", "pkv_attn_plan", "paged_decode_attention_planned",
    "paged_decode_attention_planned_timed", "paged_decode_attention_planned_append",
    "paged_decode_attention", "paged_decode_attention_timed", "paged_prefill_attention", "paged_prefill_attention_ws",
    "pkv_prefill_workspace_bytes", "kv_append", "kv_append_chunk", "kv_block_swap",
    "kv_swap_out_host", "kv_swap_in_host",
    "pkv_validate_tables_host",
    "pkv_validate_mapping_host", "pkv_validate_tables", "pkv_validate_mapping", "pkv_validate_chunks_host",
    "pkv_validate_chunks",
    "pkv_probe_copy", "pkv_probe_read",
]


class AttnDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "num_q_heads", "num_kv_heads", "head_dim", "block_size", "num_pool_blocks",
        "max_blocks_per_seq", "max_context_len", "partition_tokens", "kv_dtype", "out_dtype",
        "flags")] + [(n, ctypes.c_int64) for n in (
            "k_stride_block", "k_stride_head", "k_stride_token",
            "v_stride_block", "v_stride_head", "v_stride_token")] + [
        ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float)]


class SwapDesc(ctypes.Structure):
    _fields_ = [("num_planes", ctypes.c_int32), ("src_num_blocks", ctypes.c_int32),
                ("dst_num_blocks", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("block_bytes", ctypes.c_int64), ("src_plane_stride_bytes", ctypes.c_int64),
                ("dst_plane_stride_bytes", ctypes.c_int64)]


class PkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib = None


def lib() -> ctypes.CDLL:
    """Open libpkv.so (once).  A missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -m paper_2602_07878_amd.build`")
        # The callers' tensors and streams come from PyTorch, which ships its own copy of the
        # HIP runtime: load it first, so that the library binds to that same runtime instead
        # of bringing a second one into the process (whose streams would be foreign to it).
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.pkv_version.restype = i32
        L.pkv_version.argtypes = []
        L.pkv_init.restype = i32
        L.pkv_init.argtypes = []
        L.pkv_static_scratch_bytes.restype = sz
        L.pkv_static_scratch_bytes.argtypes = []
        L.paged_decode_attention_static.restype = i32
        L.paged_decode_attention_static.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp,
                                                    ctypes.c_float, vp, vp]
        L.pkv_status_string.restype = ctypes.c_char_p
        L.pkv_status_string.argtypes = [i32]
        L.pkv_last_hip_error_string.restype = ctypes.c_char_p
        L.pkv_last_hip_error_string.argtypes = []
        L.pkv_attn_partition_tokens.restype = i32
        L.pkv_attn_partition_tokens.argtypes = [ctypes.POINTER(AttnDesc)]
        L.pkv_attn_workspace_bytes.restype = sz
        L.pkv_attn_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc)]
        L.paged_decode_attention.restype = i32
        L.paged_decode_attention.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp,
                                             ctypes.c_float, vp, vp, sz, vp]
        L.paged_decode_attention_timed.restype = i32
        L.paged_decode_attention_timed.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp,
                                                   ctypes.c_float, vp, vp, sz, vp, vp, vp]
        L.pkv_attn_plan_bytes.restype = sz
        L.pkv_attn_plan_bytes.argtypes = [ctypes.POINTER(AttnDesc)]
        L.pkv_attn_plan.restype = i32
        L.pkv_attn_plan.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, sz, vp]
        L.paged_decode_attention_planned.restype = i32
        L.paged_decode_attention_planned.argtypes = [ctypes.POINTER(AttnDesc), vp, sz, vp, vp, vp, vp, vp,
                                                     ctypes.c_float, vp, vp, sz, vp]
        L.paged_decode_attention_planned_append.restype = i32
        L.paged_decode_attention_planned_append.argtypes = [ctypes.POINTER(AttnDesc), vp, sz, vp, vp, vp, vp, vp, vp, vp,
                                                            ctypes.c_float, vp, vp, sz, vp]
        L.paged_decode_attention_planned_timed.restype = i32
        L.paged_decode_attention_planned_timed.argtypes = [ctypes.POINTER(AttnDesc), vp, sz, vp, vp, vp, vp, vp,
                                                           ctypes.c_float, vp, vp, sz, vp, vp, vp]
        L.paged_prefill_attention.restype = i32
        L.paged_prefill_attention.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, i32,
                                              ctypes.c_float, vp, vp]
        L.paged_prefill_attention_ws.restype = i32
        L.paged_prefill_attention_ws.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, i32, ctypes.c_int64,
                                                 ctypes.c_float, vp, vp, ctypes.c_size_t, vp]
        L.pkv_prefill_workspace_bytes.restype = ctypes.c_size_t
        L.pkv_prefill_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_int64, i32]
        L.kv_append.restype = i32
        L.kv_append.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp]
        L.kv_append_chunk.restype = i32
        L.kv_append_chunk.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int64, vp]
        for name in ("kv_swap_out_host", "kv_swap_in_host"):
            getattr(L, name).restype = i32
            getattr(L, name).argtypes = [ctypes.POINTER(SwapDesc), vp, vp, vp, i32, vp, sz, vp]
        L.kv_block_swap.restype = i32
        L.kv_block_swap.argtypes = [ctypes.POINTER(SwapDesc), vp, vp, vp, i32, vp]
        L.pkv_validate_tables_host.restype = i32
        L.pkv_validate_tables_host.argtypes = [ctypes.POINTER(AttnDesc), vp, vp]
        L.pkv_validate_mapping_host.restype = i32
        L.pkv_validate_mapping_host.argtypes = [ctypes.POINTER(SwapDesc), vp, i32]
        L.pkv_validate_tables.restype = i32
        L.pkv_validate_tables.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp]
        L.pkv_validate_mapping.restype = i32
        L.pkv_validate_mapping.argtypes = [ctypes.POINTER(SwapDesc), vp, i32, vp]
        L.pkv_probe_copy.restype = i32
        L.pkv_probe_copy.argtypes = [vp, vp, sz, vp]
        L.pkv_probe_read.restype = i32
        L.pkv_probe_read.argtypes = [vp, vp, sz, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().pkv_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != PKV_OK:
        if status == PKV_ERR_HIP:
            where += " (" + lib().pkv_last_hip_error_string().decode() + ")"
        raise PkvError(status, where)


def _stream_ptr(stream) -> Optional[int]:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _torch_dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return PKV_F32
    if t.dtype == torch.bfloat16:
        return PKV_BF16
    if t.dtype in (torch.uint8, torch.float8_e4m3fn):   # 8-bit pools: E4M3 codes
        return PKV_F8_E4M3
    raise TypeError(f"unsupported dtype {t.dtype}")


def attn_desc_for(q, k_pool, v_pool, block_tables, *, max_context_len: int,
                  partition_tokens: int = 0, out_dtype=None, flags: int = 0,
                  k_scale: float = 1.0, v_scale: float = 1.0) -> AttnDesc:
    """Descriptor for torch tensors: q [B,Hq,D]; pools [blocks,Hkv,bs,D] (any strides with a
    unit-stride last dim); block_tables [B,max_blocks].  8-bit pools (uint8 or float8_e4m3fn
    tensors of E4M3 codes) go with a bfloat16 q and the factors k_scale, v_scale."""
    import torch
    B, Hq, D = q.shape
    nblk, Hkv, bs, Dk = k_pool.shape
    assert Dk == D and v_pool.shape == k_pool.shape
    assert k_pool.stride(3) == 1 and v_pool.stride(3) == 1 and q.is_contiguous()
    code = _torch_dtype_code(k_pool)
    assert _torch_dtype_code(v_pool) == code
    assert _torch_dtype_code(q) == (PKV_BF16 if code == PKV_F8_E4M3 else code)
    d = AttnDesc()
    d.batch, d.num_q_heads, d.num_kv_heads, d.head_dim = B, Hq, Hkv, D
    d.block_size, d.num_pool_blocks = bs, nblk
    d.max_blocks_per_seq = block_tables.shape[1]
    d.max_context_len = int(max_context_len)
    d.partition_tokens = int(partition_tokens)
    d.kv_dtype = code
    d.out_dtype = PKV_F32 if out_dtype in (None, torch.float32) else PKV_BF16
    d.flags = int(flags)
    d.k_stride_block, d.k_stride_head, d.k_stride_token = (k_pool.stride(i) for i in range(3))
    d.v_stride_block, d.v_stride_head, d.v_stride_token = (v_pool.stride(i) for i in range(3))
    d.k_scale, d.v_scale = float(k_scale), float(v_scale)
    return d


def attn_workspace_bytes(desc: AttnDesc) -> int:
    return int(lib().pkv_attn_workspace_bytes(ctypes.byref(desc)))


def new_workspace(nbytes: int, device, *, stream=None):
    """Allocate a workspace tensor of `nbytes` bytes (contents need no initialisation)."""
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def paged_decode_attention(q, k_pool, v_pool, block_tables, context_lens, scale, out, *,
                           max_context_len: int, partition_tokens: int = 0, workspace=None,
                           desc: Optional[AttnDesc] = None, stream=None, flags: int = 0,
                           kernel_events=None, k_scale: float = 1.0, v_scale: float = 1.0):
    """out[i,h,:] = softmax_t(scale * q[i,h] . K_t) V_t over the paged pool (device tensors).
    Returns the workspace tensor used (reusable by the caller)."""
    import torch
    L = lib()
    if desc is None:
        desc = attn_desc_for(q, k_pool, v_pool, block_tables, max_context_len=max_context_len,
                             partition_tokens=partition_tokens, out_dtype=out.dtype, flags=flags,
                             k_scale=k_scale, v_scale=v_scale)
    assert block_tables.dtype == torch.int32 and context_lens.dtype == torch.int32
    assert block_tables.is_contiguous() and context_lens.is_contiguous() and out.is_contiguous()
    need = int(L.pkv_attn_workspace_bytes(ctypes.byref(desc)))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = new_workspace(need, q.device, stream=stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    args = (ctypes.byref(desc), q.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr(),
            block_tables.data_ptr(), context_lens.data_ptr(), float(scale), out.data_ptr(),
            ws_ptr, ws_bytes, _stream_ptr(stream))
    if kernel_events is None:
        st = L.paged_decode_attention(*args)
    else:   # two torch.cuda.Event(enable_timing=True) that have been recorded once (so they exist)
        st = L.paged_decode_attention_timed(*args, ctypes.c_void_p(kernel_events[0].cuda_event),
                                            ctypes.c_void_p(kernel_events[1].cuda_event))
    _check(st, "paged_decode_attention")
    return workspace


def attn_plan(desc: AttnDesc, block_tables, context_lens, plan=None, *, stream=None):
    """Write the per-step plan for `desc`, `block_tables` and `context_lens` (device tensors) into
    `plan` (a uint8 device tensor; allocated here when None or too small).  Returns the plan tensor."""
    import torch
    L = lib()
    need = int(L.pkv_attn_plan_bytes(ctypes.byref(desc)))
    if plan is None or plan.numel() * plan.element_size() < need:
        plan = torch.empty(max(need, 256), dtype=torch.uint8, device=block_tables.device)
    _check(L.pkv_attn_plan(ctypes.byref(desc), block_tables.data_ptr(), context_lens.data_ptr(), plan.data_ptr(),
                           plan.numel() * plan.element_size(), _stream_ptr(stream)), "pkv_attn_plan")
    return plan


def paged_decode_attention_planned(desc: AttnDesc, plan, q, k_pool, v_pool, block_tables, context_lens, scale, out, *,
                                   workspace=None, stream=None, kernel_events=None, k_new=None, v_new=None):
    """paged_decode_attention with a plan from attn_plan (same desc, tables and lengths); with
    k_new / v_new the new token's rows are appended to the pools in the same call.
    Returns the workspace tensor used."""
    L = lib()
    need = int(L.pkv_attn_workspace_bytes(ctypes.byref(desc)))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = new_workspace(need, q.device, stream=stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    args = (ctypes.byref(desc), plan.data_ptr(), plan.numel() * plan.element_size(), q.data_ptr(), k_pool.data_ptr(),
            v_pool.data_ptr(), block_tables.data_ptr(), context_lens.data_ptr(), float(scale), out.data_ptr(),
            ws_ptr, ws_bytes, _stream_ptr(stream))
    if k_new is not None:
        assert kernel_events is None
        st = L.paged_decode_attention_planned_append(*args[:4], k_new.data_ptr(), v_new.data_ptr(), *args[4:])
    elif kernel_events is None:
        st = L.paged_decode_attention_planned(*args)
    else:
        st = L.paged_decode_attention_planned_timed(*args, ctypes.c_void_p(kernel_events[0].cuda_event),
                                                    ctypes.c_void_p(kernel_events[1].cuda_event))
    _check(st, "paged_decode_attention_planned")
    return workspace


def init():
    """Once-per-device set-up of the library for the current device (optional: the first call of
    an entry point does its own)."""
    _check(lib().pkv_init(), "pkv_init")


def paged_decode_attention_static(q, k_pool, v_pool, block_tables, context_lens, scale, out, *,
                                  max_context_len: int, partition_tokens: int = 0,
                                  desc: Optional[AttnDesc] = None, stream=None, flags: int = 0):
    """paged_decode_attention with the library's static device scratch instead of a workspace:
    no tensor is allocated here or in the library."""
    if desc is None:
        desc = attn_desc_for(q, k_pool, v_pool, block_tables, max_context_len=max_context_len,
                             partition_tokens=partition_tokens, out_dtype=out.dtype, flags=flags)
    st = lib().paged_decode_attention_static(
        ctypes.byref(desc), q.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr(), block_tables.data_ptr(),
        context_lens.data_ptr(), float(scale), out.data_ptr(), _stream_ptr(stream))
    _check(st, "paged_decode_attention_static")


def swap_desc(num_planes: int, block_bytes: int, src_num_blocks: int, dst_num_blocks: int,
              src_plane_stride_bytes: Optional[int] = None,
              dst_plane_stride_bytes: Optional[int] = None) -> SwapDesc:
    d = SwapDesc()
    d.num_planes, d.src_num_blocks, d.dst_num_blocks, d.reserved = (
        num_planes, src_num_blocks, dst_num_blocks, 0)
    d.block_bytes = block_bytes
    d.src_plane_stride_bytes = (src_num_blocks * block_bytes if src_plane_stride_bytes is None
                                else src_plane_stride_bytes)
    d.dst_plane_stride_bytes = (dst_num_blocks * block_bytes if dst_plane_stride_bytes is None
                                else dst_plane_stride_bytes)
    return d


def prefill_workspace_bytes(desc: AttnDesc, total_query_tokens: int, max_query_len: int) -> int:
    """Bytes of device workspace with which paged_prefill_attention splits the walks (0: it will
    not), plus, for 8-bit pools, the bf16 copy of the sequences' blocks that the call walks."""
    return int(lib().pkv_prefill_workspace_bytes(ctypes.byref(desc), int(total_query_tokens), int(max_query_len)))


def paged_prefill_attention(desc: AttnDesc, q, k_pool, v_pool, block_tables, context_lens, query_lens,
                            cu_query_lens, max_query_len: int, scale: float, out, *, stream=None, workspace=None):
    """Causal attention of the last query_lens[i] tokens of every sequence (q, out packed
    [total, Hq, D]; all tensors on the device).  workspace: a device byte tensor of at least
    prefill_workspace_bytes(desc, q.shape[0], max_query_len) bytes lets few, long walks be split."""
    assert q.is_contiguous() and out.is_contiguous() and out.shape == q.shape
    if workspace is None:
        st = lib().paged_prefill_attention(ctypes.byref(desc), q.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr(),
                                           block_tables.data_ptr(), context_lens.data_ptr(), query_lens.data_ptr(),
                                           cu_query_lens.data_ptr(), int(max_query_len), float(scale),
                                           out.data_ptr(), _stream_ptr(stream))
    else:
        st = lib().paged_prefill_attention_ws(ctypes.byref(desc), q.data_ptr(), k_pool.data_ptr(), v_pool.data_ptr(),
                                              block_tables.data_ptr(), context_lens.data_ptr(), query_lens.data_ptr(),
                                              cu_query_lens.data_ptr(), int(max_query_len), int(q.shape[0]), float(scale),
                                              out.data_ptr(), workspace.data_ptr(),
                                              workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    _check(st, "paged_prefill_attention")


def kv_append(desc: AttnDesc, k_new, v_new, k_pool, v_pool, block_tables, context_lens, *, stream=None):
    """Write rows k_new[i], v_new[i] ([B,Hkv,D], device) at token position context_lens[i]-1."""
    assert k_new.is_contiguous() and v_new.is_contiguous()
    st = lib().kv_append(ctypes.byref(desc), k_new.data_ptr(), v_new.data_ptr(), k_pool.data_ptr(),
                         v_pool.data_ptr(), block_tables.data_ptr(), context_lens.data_ptr(),
                         _stream_ptr(stream))
    _check(st, "kv_append")


def kv_append_chunk(desc: AttnDesc, k_new, v_new, k_pool, v_pool, block_tables, context_lens, query_lens,
                    cu_query_lens, *, stream=None):
    """Write the rows of a prefill chunk (k_new, v_new packed [total, Hkv, D], device) to the tail
    positions context_lens[i] - query_lens[i] .. context_lens[i] - 1 of their sequences."""
    assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.shape == v_new.shape
    st = lib().kv_append_chunk(ctypes.byref(desc), k_new.data_ptr(), v_new.data_ptr(), k_pool.data_ptr(),
                               v_pool.data_ptr(), block_tables.data_ptr(), context_lens.data_ptr(),
                               query_lens.data_ptr(), cu_query_lens.data_ptr(), int(k_new.shape[0]),
                               _stream_ptr(stream))
    _check(st, "kv_append_chunk")


def kv_block_swap(desc: SwapDesc, src_pool, dst, block_mapping, *, stream=None):
    """Copy (plane, block) chunks src_pool -> dst per block_mapping [n,2] int32 (device)."""
    import torch
    assert block_mapping.dtype == torch.int32 and block_mapping.is_contiguous()
    n_pairs = block_mapping.numel() // 2
    st = lib().kv_block_swap(ctypes.byref(desc), src_pool.data_ptr(), dst.data_ptr(),
                             block_mapping.data_ptr(), n_pairs, _stream_ptr(stream))
    _check(st, "kv_block_swap")


def kv_swap_out_host(desc: SwapDesc, src_pool, host_dst, block_mapping, staging=None, *, stream=None):
    """Pool blocks block_mapping[:,0] (device) -> slots 0..n-1 of the pinned host tensor host_dst,
    in pieces through the device tensor `staging`, or (staging None) written by the kernel itself."""
    assert host_dst.is_pinned() and block_mapping.is_contiguous()
    st = lib().kv_swap_out_host(ctypes.byref(desc), src_pool.data_ptr(), host_dst.data_ptr(),
                                block_mapping.data_ptr(), block_mapping.numel() // 2,
                                staging.data_ptr() if staging is not None else None,
                                staging.numel() * staging.element_size() if staging is not None else 0,
                                _stream_ptr(stream))
    _check(st, "kv_swap_out_host")


def kv_swap_in_host(desc: SwapDesc, host_src, dst_pool, block_mapping, staging=None, *, stream=None):
    """Slots 0..n-1 of the pinned host tensor host_src -> pool blocks block_mapping[:,1] (device)."""
    assert host_src.is_pinned() and block_mapping.is_contiguous()
    st = lib().kv_swap_in_host(ctypes.byref(desc), host_src.data_ptr(), dst_pool.data_ptr(),
                               block_mapping.data_ptr(), block_mapping.numel() // 2,
                               staging.data_ptr() if staging is not None else None,
                               staging.numel() * staging.element_size() if staging is not None else 0,
                               _stream_ptr(stream))
    _check(st, "kv_swap_in_host")


def validate_chunks(desc: AttnDesc, context_lens, query_lens, cu_query_lens, max_query_len: int,
                    total_query_tokens: int, *, stream=None) -> int:
    """Status of the range check of the chunk arrays (device tensors; copies them and waits)."""
    L = lib()
    L.pkv_validate_chunks.restype = ctypes.c_int32
    L.pkv_validate_chunks.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p]
    return int(L.pkv_validate_chunks(ctypes.byref(desc), context_lens.data_ptr(), query_lens.data_ptr(),
                                     cu_query_lens.data_ptr(), int(max_query_len), int(total_query_tokens),
                                     _stream_ptr(stream)))


def validate_tables(desc: AttnDesc, block_tables, context_lens, *, stream=None) -> int:
    return int(lib().pkv_validate_tables(ctypes.byref(desc), block_tables.data_ptr(),
                                         context_lens.data_ptr(), _stream_ptr(stream)))


def validate_mapping(desc: SwapDesc, block_mapping, *, stream=None) -> int:
    return int(lib().pkv_validate_mapping(ctypes.byref(desc), block_mapping.data_ptr(),
                                          block_mapping.numel() // 2, _stream_ptr(stream)))


def probe_copy(src, dst, nbytes: int, *, stream=None):
    _check(lib().pkv_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream_ptr(stream)),
           "pkv_probe_copy")


def probe_read(src, sink, nbytes: int, *, stream=None):
    _check(lib().pkv_probe_read(src.data_ptr(), sink.data_ptr(), nbytes, _stream_ptr(stream)),
           "pkv_probe_read")
