#!/usr/bin/env python3
"""Benchmark of the paged-KV decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one paged_decode_attention layer-call (block-table walk, K/V
streaming, scores, softmax, accumulate, split-K merge) over the batch of the
Llama-3-8B-shaped configuration (batch 64, 32/8 heads, D 128, bf16, contexts
uniform in [128, 4096]); consecutive steps cycle over distinct per-layer KV
pools, as the layers of one decode iteration do, so every step streams data that
is not in any cache.  The preemption-swap legs (gather to staging, scatter to
fresh blocks) of the Squeeze configuration are timed in the same run and
reported under "swap".  One JSON line is printed on stdout.
"""
from __future__ import annotations

import argparse
import numpy as np
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
STREAM_KERNEL = "attn_stream_flat_bf16_d128<4>"   # the kernel that streams K and V for the timed workload
PLAN_EVERY = 32   # layer calls that share one plan: the decoder layers of the 8B model (Sec. 4.2)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def upload_attn(w, layers, torch):
    import numpy as np
    dev = "cuda:0"
    def conv(a):     # uint16 = bf16 bits, uint8 = E4M3 codes, else float32
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)
    k0, v0 = conv(w.k_pool), conv(w.v_pool)
    # every layer gets its own allocation (same values: only addresses matter for timing)
    ks = [k0] + [k0.clone() for _ in range(layers - 1)]
    vs = [v0] + [v0.clone() for _ in range(layers - 1)]
    return dict(q=conv(w.q), ks=ks, vs=vs,
                bt=torch.from_numpy(w.block_tables).to(dev),
                cl=torch.from_numpy(w.context_lens).to(dev))


def time_attention(w, d, steps, warmup, torch, binding, kernel_events=False, planned=False):
    """Returns (out, ms per call, wall ms per call, sorted ms of every launch of the K/V-streaming kernel).
    With kernel_events, every call also records an event right before and right after that
    kernel (paged_decode_attention_timed), on the stream the kernels run on.  planned: the calls
    go through paged_decode_attention_planned, and every PLAN_EVERY-th call is preceded by
    pkv_attn_plan, inside the timed region (a decode step plans once and calls once per layer)."""
    out = torch.empty(w.B, w.Hq, w.D, dtype=torch.float32, device="cuda:0")
    desc = binding.attn_desc_for(d["q"], d["ks"][0], d["vs"][0], d["bt"],
                                 max_context_len=w.max_context_len,
                                 partition_tokens=w.partition_tokens)
    ws = binding.new_workspace(binding.attn_workspace_bytes(desc), "cuda:0")
    L = len(d["ks"])

    evs = None
    if kernel_events:
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(steps)]
        for a, b in evs:       # an event handle exists only once it has been recorded
            a.record()
            b.record()

    plan = binding.attn_plan(desc, d["bt"], d["cl"]) if planned else None

    def step(i, ke=None):
        if planned:
            if i % PLAN_EVERY == 0:
                binding.attn_plan(desc, d["bt"], d["cl"], plan)
            binding.paged_decode_attention_planned(desc, plan, d["q"], d["ks"][i % L], d["vs"][i % L], d["bt"],
                                                   d["cl"], w.scale, out, workspace=ws, kernel_events=ke)
        else:
            binding.paged_decode_attention(d["q"], d["ks"][i % L], d["vs"][i % L], d["bt"], d["cl"],
                                           w.scale, out, max_context_len=w.max_context_len,
                                           workspace=ws, desc=desc, kernel_events=ke)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        step(i, evs[i] if evs else None)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = e0.elapsed_time(e1)
    kern = sorted(a.elapsed_time(b) for a, b in evs) if evs else None
    return out, ev_ms / steps, wall_ms / steps, kern


def source_fingerprint():
    """Hash of what defines the dominant kernel: its source file and, of the shared header, the
    constants and the parameter block it is launched with (the part up to the end of AttnParams;
    the prototypes of other files further down do not touch the kernel).  Counter-derived figures
    under profiles/ are quoted only while this is unchanged."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2602_07878_amd", "csrc")
    h = hashlib.sha256()
    for name in ("attn_stream_flat.hip", "attn_stream_common.h", "attn_stream_mfma.hip"):   # (the last holds the merge)
        h.update(open(os.path.join(csrc, name), "rb").read())
    head = open(os.path.join(csrc, "pkv_internal.h")).read()
    end = head.index("};", head.index("struct AttnParams {")) + 2
    h.update(head[:end].encode())
    return h.hexdigest()[:16]


def recorded_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (its
    `key = value` header lines), or None if that summary is missing or was taken from other
    sources than the ones now in the tree."""
    path = os.path.join(ROOT, "profiles", "attn_stream_cfg2_hbm_traffic.txt")
    rec = {}
    try:
        for line in open(path):
            if line.startswith("# ") and " = " in line:
                k, v = line[2:].split(" = ", 1)
                rec[k.strip()] = v.strip()
        if (rec.get("source_fingerprint") == source_fingerprint() and rec.get("workload") == workload
                and rec.get("kernel") == kernel):
            return float(rec["hbm_bytes_per_launch"])
    except (OSError, ValueError, KeyError):
        pass
    return None


def time_append(w, d, torch, binding, reps=200):
    """The new token's K/V rows of every sequence written into the pools (the step right before
    attention in a decode iteration): time of the append alone and of append + attention."""
    desc = binding.attn_desc_for(d["q"], d["ks"][0], d["vs"][0], d["bt"], max_context_len=w.max_context_len,
                                 partition_tokens=w.partition_tokens)
    ws = binding.new_workspace(binding.attn_workspace_bytes(desc), "cuda:0")
    out = torch.empty(w.B, w.Hq, w.D, dtype=torch.float32, device="cuda:0")
    kn = torch.randn(w.B, w.Hkv, w.D, device="cuda:0").to(d["ks"][0].dtype)
    vn = torch.randn(w.B, w.Hkv, w.D, device="cuda:0").to(d["ks"][0].dtype)
    L = len(d["ks"])

    def run(with_attention):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(reps):
            binding.kv_append(desc, kn, vn, d["ks"][i % L], d["vs"][i % L], d["bt"], d["cl"])
            if with_attention:
                binding.paged_decode_attention(d["q"], d["ks"][i % L], d["vs"][i % L], d["bt"], d["cl"],
                                               w.scale, out, max_context_len=w.max_context_len,
                                               workspace=ws, desc=desc)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3
    plan = binding.attn_plan(desc, d["bt"], d["cl"])

    def run_planned(fused):
        # the planned call with the append as a launch of its own in front of it, or inside it
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(reps):
            if i % PLAN_EVERY == 0:
                binding.attn_plan(desc, d["bt"], d["cl"], plan)
            if not fused:
                binding.kv_append(desc, kn, vn, d["ks"][i % L], d["vs"][i % L], d["bt"], d["cl"])
            binding.paged_decode_attention_planned(desc, plan, d["q"], d["ks"][i % L], d["vs"][i % L], d["bt"], d["cl"],
                                                   w.scale, out, workspace=ws, k_new=kn if fused else None,
                                                   v_new=vn if fused else None)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3
    run(True)
    run_planned(True)
    return {"append_us": run(False), "append_plus_attention_us": run(True),
            "append_plus_planned_attention_us": run_planned(False),
            "planned_attention_that_appends_us": run_planned(True),
            "bytes_written": 2 * w.B * w.Hkv * w.D * 2}


def time_swap(sw, reps, torch, binding, oracle_check=True):
    """Gather the victims' blocks to contiguous staging, then scatter to fresh blocks."""
    g = torch.Generator(device="cuda:0")
    g.manual_seed(sw.seed)
    pool = torch.randint(-2**31, 2**31 - 1, (sw.pool_bytes // 4,), dtype=torch.int32,
                         device="cuda:0", generator=g)
    pool_before = {}
    if oracle_check:
        pv = pool.view(sw.num_planes, -1)
        pool_before = {p: pv[p].cpu().numpy().view(np.uint8).copy() for p in (0, sw.num_planes - 1)}
    staging = torch.zeros(sw.staging_bytes // 4, dtype=torch.int32, device="cuda:0")
    gm = torch.from_numpy(sw.gather_mapping).cuda()
    # the order of the pairs is free: listing them by ascending destination block makes the
    # pool writes sequential, which this part rewards (scatter 5.5 -> 5.8 TB/s of traffic);
    # the gather already writes its staging slots in order
    smap = sw.scatter_mapping[np.argsort(sw.scatter_mapping[:, 1], kind="stable")]
    sm = torch.from_numpy(np.ascontiguousarray(smap)).cuda()
    dg = binding.swap_desc(sw.num_planes, sw.block_bytes, sw.num_pool_blocks, sw.n_blocks)
    ds = binding.swap_desc(sw.num_planes, sw.block_bytes, sw.n_blocks, sw.num_pool_blocks)
    res = {}
    for name, fn in (("gather", lambda: binding.kv_block_swap(dg, pool, staging, gm)),
                     ("scatter", lambda: binding.kv_block_swap(ds, staging, pool, sm))):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        res[name] = {"ms": ms, "payload_GBps": sw.payload_bytes / ms / 1e6,
                     "traffic_GBps": 2 * sw.payload_bytes / ms / 1e6,
                     "frac_hbm_peak": 2 * sw.payload_bytes / ms / 1e6 / HBM_PEAK_GBS}
    # (1) on the device, no oracle involved: after the scatter the victims' new blocks hold what
    #     staging holds, on three planes; (2) against the oracle (memcpy per pair on the host): the
    #     gathered staging plane and the scattered pool plane of the first and the last plane,
    #     byte for byte, from the pool bytes as they were before the scatter
    v = pool.view(sw.num_planes, sw.num_pool_blocks, sw.block_bytes // 4)
    s = staging.view(sw.num_planes, sw.n_blocks, sw.block_bytes // 4)
    idx = torch.from_numpy(sw.new_blocks).long().cuda()
    ok = all(bool(torch.equal(v[p][idx], s[p])) for p in (0, sw.num_planes // 2, sw.num_planes - 1))
    res["device_self_check_new_blocks_equal_staging_3_planes"] = ok
    if oracle_check:
        import oracle
        planes_ok = []
        cpu_s = 0.0
        for p in (0, sw.num_planes - 1):
            before = pool_before[p]                                  # host copy taken before any swap
            st_ref = np.zeros(sw.n_blocks * sw.block_bytes, np.uint8)
            t = time.perf_counter()
            oracle.kv_block_swap(before, st_ref, sw.gather_mapping, num_planes=1, block_bytes=sw.block_bytes)
            cpu_s += time.perf_counter() - t
            pool_ref = before.copy()
            oracle.kv_block_swap(st_ref, pool_ref, smap, num_planes=1, block_bytes=sw.block_bytes)
            planes_ok.append(bool(np.array_equal(s[p].cpu().numpy().view(np.uint8).reshape(-1), st_ref)) and
                             bool(np.array_equal(v[p].cpu().numpy().view(np.uint8).reshape(-1), pool_ref)))
        res["bit_exact_vs_oracle_first_and_last_plane"] = all(planes_ok)
        # the oracle's memcpy per block on this host's cores, for scale (two planes of the gather)
        res["cpu_oracle_gather"] = {"payload_GBps": 2 * sw.n_blocks * sw.block_bytes / cpu_s / 1e9,
                                    "cores": oracle.num_threads(), "sample": "two of the planes"}
    res["payload_GB"] = sw.payload_bytes / 1e9
    res["victims"] = int(sw.victim_lens.size)
    res["blocks"] = sw.n_blocks
    del pool, staging
    torch.cuda.empty_cache()
    return res


def time_swap_host(sw, torch, binding, staging_mib=256, reps=2, decode_batch=None):
    """The same victims' blocks out to pinned host memory and back in (PCIe-bound), in pieces
    through a device staging buffer."""
    g = torch.Generator(device="cuda:0")
    g.manual_seed(sw.seed)
    pool = torch.randint(-2**31, 2**31 - 1, (sw.pool_bytes // 4,), dtype=torch.int32, device="cuda:0", generator=g)
    host = torch.empty(sw.staging_bytes, dtype=torch.uint8).pin_memory()
    staging = torch.empty(staging_mib << 20, dtype=torch.uint8, device="cuda:0")
    gm = torch.from_numpy(sw.gather_mapping).cuda()
    sm = torch.from_numpy(sw.scatter_mapping).cuda()
    d_out = binding.swap_desc(sw.num_planes, sw.block_bytes, sw.num_pool_blocks, sw.n_blocks)
    d_in = binding.swap_desc(sw.num_planes, sw.block_bytes, sw.n_blocks, sw.num_pool_blocks)
    res = {}
    # both forms once for the bytes: the host slots of the first and the last plane against the
    # pool blocks they came from, and the pool's new blocks against the host slots afterwards
    P, NB, nb_, bb = sw.num_planes, sw.num_pool_blocks, sw.n_blocks, sw.block_bytes
    pv, hv = pool.view(torch.uint8).view(P, NB, bb), host.view(P, nb_, bb)
    src_i, new_i = (torch.from_numpy(a).long().cuda() for a in (sw.src_blocks, sw.new_blocks))
    checks = {}
    for form, st in (("staged", staging), ("unstaged", None)):
        host.zero_()
        binding.kv_swap_out_host(d_out, pool, host, gm, st)
        torch.cuda.synchronize()
        ok = all(bool(torch.equal(hv[p], pv[p][src_i].cpu())) for p in (0, P - 1))
        binding.kv_swap_in_host(d_in, host, pool, sm, st)
        torch.cuda.synchronize()
        ok = ok and all(bool(torch.equal(pv[p][new_i].cpu(), hv[p])) for p in (0, P - 1))
        checks[form] = ok
    res["bit_exact_first_and_last_plane_pool_vs_host"] = checks
    for name, fn in (("out", lambda: binding.kv_swap_out_host(d_out, pool, host, gm, staging)),
                     ("in", lambda: binding.kv_swap_in_host(d_in, host, pool, sm, staging)),
                     # without a staging buffer: the copy kernel reads and writes the host memory itself
                     ("out_unstaged", lambda: binding.kv_swap_out_host(d_out, pool, host, gm)),
                     ("in_unstaged", lambda: binding.kv_swap_in_host(d_in, host, pool, sm))):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / reps * 1e3
        res[name] = {"ms": ms, "payload_GBps": sw.payload_bytes / ms / 1e6}
    res["payload_GB"] = sw.payload_bytes / 1e9
    res["staging_MiB"] = staging_mib
    # what this box's PCIe link gives a plain pinned copy, for comparison (the boxes differ)
    n = min(1 << 30, host.numel(), pool.numel() * 4)
    dev_bytes = pool.view(torch.uint8)[:n]
    plain = {}
    for name, fn in (("d2h", lambda: host[:n].copy_(dev_bytes, non_blocking=True)),
                     ("h2d", lambda: dev_bytes.copy_(host[:n], non_blocking=True))):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        plain[name] = n * reps / (time.perf_counter() - t0) / 1e9
    res["plain_pinned_copy_GBps"] = plain
    # The paper's setting: the other requests keep decoding while a victim's blocks leave.  Decode
    # calls of the benchmark batch on one stream, alone and while each form of the swap-out runs
    # on another stream.
    if decode_batch is not None:
        w, d = decode_batch
        out = torch.empty(w.B, w.Hq, w.D, dtype=torch.float32, device="cuda:0")
        desc = binding.attn_desc_for(d["q"], d["ks"][0], d["vs"][0], d["bt"], max_context_len=w.max_context_len)
        ws = binding.new_workspace(binding.attn_workspace_bytes(desc), "cuda:0")
        plan = binding.attn_plan(desc, d["bt"], d["cl"])
        L = len(d["ks"])
        s_swap, s_dec = torch.cuda.Stream(), torch.cuda.Stream()
        calls = 800                      # about as long as the swap-out

        def decode(n):
            for i in range(n):
                if i % PLAN_EVERY == 0:
                    binding.attn_plan(desc, d["bt"], d["cl"], plan, stream=s_dec)
                binding.paged_decode_attention_planned(desc, plan, d["q"], d["ks"][i % L], d["vs"][i % L], d["bt"],
                                                       d["cl"], w.scale, out, workspace=ws, stream=s_dec)
        ov = {}
        for mode in ("alone", "staged", "unstaged"):
            torch.cuda.synchronize()
            a0, a1, b0, b1 = (torch.cuda.Event(enable_timing=True) for _ in range(4))
            decode(PLAN_EVERY)           # the decode stream is busy when the swap arrives
            b0.record(s_dec)
            if mode != "alone":
                a0.record(s_swap)
                binding.kv_swap_out_host(d_out, pool, host, gm, staging if mode == "staged" else None, stream=s_swap)
                a1.record(s_swap)
            decode(calls)
            b1.record(s_dec)
            torch.cuda.synchronize()
            ov[mode] = {"decode_us_per_call": b0.elapsed_time(b1) / calls * 1e3}
            if mode != "alone":
                ov[mode]["swap_out_GBps"] = sw.payload_bytes / a0.elapsed_time(a1) / 1e6
        res["decode_calls_while_swapping_out"] = ov
        del out, ws, plan
    del pool, host, staging
    torch.cuda.empty_cache()
    return res


MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X published dense bf16 matrix-core rate


def time_prefill(torch, binding, B=16, n=4096, Hq=32, Hkv=8, reps=5, oracle_rows=256, f8=False):
    """Re-prefill of B preempted requests of n tokens each (the recompute recovery path): causal
    attention of all n tokens over the paged cache, 8B-shaped heads.  Flops counted: 4*D per
    (query, visible key) pair and query head, i.e. the causal half only.  f8: the pools hold E4M3
    codes (the call then walks a bf16 copy it makes in its workspace)."""
    D, bs = 128, 16
    nblk = B * ((n + bs - 1) // bs)
    g = torch.Generator(device="cuda:0")
    g.manual_seed(1006)
    kp = torch.randn(nblk, Hkv, bs, D, device="cuda:0", generator=g).bfloat16()
    vp = torch.randn(nblk, Hkv, bs, D, device="cuda:0", generator=g).bfloat16()
    if f8:
        kp, vp = (t.to(torch.float8_e4m3fn).view(torch.uint8) for t in (kp, vp))
    bt = torch.randperm(nblk, device="cuda:0", generator=g).int().view(B, -1)
    cl = torch.full((B,), n, dtype=torch.int32, device="cuda:0")
    cu = torch.arange(0, (B + 1) * n, n, dtype=torch.int32, device="cuda:0")
    q = torch.randn(B * n, Hq, D, device="cuda:0", generator=g).bfloat16()
    out = torch.empty(B * n, Hq, D, device="cuda:0")
    desc = binding.attn_desc_for(q, kp, vp, bt, max_context_len=n)
    desc.batch = B
    need = binding.prefill_workspace_bytes(desc, B * n, n)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0") if need else None
    f = lambda: binding.paged_prefill_attention(desc, q, kp, vp, bt, cl, cl, cu, n, D ** -0.5, out, workspace=ws)
    f()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        f()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    flops = 4.0 * D * (n * (n + 1) // 2) * Hq * B
    res = {"workload": f"causal re-prefill, {B} sequences x {n} tokens, {Hq}/{Hkv} heads, "
                       f"{'bf16 q over 8-bit (E4M3) pools' if f8 else 'bf16'}", "ms": ms, "workspace_MiB": need >> 20,
           "tflops": flops / ms / 1e9, "bound": "mfma", "peak_tflops": MFMA_BF16_PEAK_TFLOPS,
           "frac": flops / ms / 1e9 / MFMA_BF16_PEAK_TFLOPS}
    if oracle_rows:
        rows = np.unique(np.concatenate([np.random.default_rng(1).integers(0, B * n, oracle_rows),
                                         np.arange(B) * n, np.arange(B) * n + n - 1]))
        res.update(prefill_error(torch, q, kp, vp, bt, np.full(B, n), np.full(B, n), out, rows, D ** -0.5))
    return res


def prefill_error(torch, q, kp, vp, bt, ctx_lens, q_lens, out, rows, scale):
    """Max abs error of the sampled packed output rows (all heads) against the fp64 oracle: a query
    token is one decode-oracle row over the positions it may see."""
    import oracle
    bits = lambda t: (t.contiguous().cpu().numpy() if t.dtype == torch.uint8      # E4M3 codes as they are
                      else t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16))
    cu = np.concatenate([[0], np.cumsum(q_lens)])
    seq = np.searchsorted(cu, rows, side="right") - 1
    ctx = (np.asarray(ctx_lens)[seq] - np.asarray(q_lens)[seq] + (rows - cu[seq]) + 1).astype(np.int32)
    ridx = torch.from_numpy(rows).cuda()
    ref = oracle.paged_decode_attention(bits(q[ridx]), bits(kp), bits(vp), bt.cpu().numpy()[seq], ctx,
                                        float(np.float32(scale)), block_size=kp.shape[2])
    err = float(np.abs(out[ridx].double().cpu().numpy() - ref).max())
    return {"max_abs_err_vs_oracle": err, "oracle_rows_checked": int(rows.size)}


def time_prefill_chunk(torch, binding, n=8192, chunk=512, Hq=32, Hkv=8, reps=20, oracle_check=True):
    """One chunk of a chunked prefill: the last `chunk` tokens of one sequence of n cached tokens
    (the paper's example budget is 512 tokens per iteration), with and without the workspace
    that lets the library split the walk."""
    D, bs = 128, 16
    nblk = (n + bs - 1) // bs
    g = torch.Generator(device="cuda:0")
    g.manual_seed(1008)
    kp = torch.randn(nblk, Hkv, bs, D, device="cuda:0", generator=g).bfloat16()
    vp = torch.randn(nblk, Hkv, bs, D, device="cuda:0", generator=g).bfloat16()
    bt = torch.randperm(nblk, device="cuda:0", generator=g).int().view(1, -1)
    cl = torch.full((1,), n, dtype=torch.int32, device="cuda:0")
    ql = torch.full((1,), chunk, dtype=torch.int32, device="cuda:0")
    cu = torch.tensor([0, chunk], dtype=torch.int32, device="cuda:0")
    q = torch.randn(chunk, Hq, D, device="cuda:0", generator=g).bfloat16()
    out = torch.empty(chunk, Hq, D, device="cuda:0")
    desc = binding.attn_desc_for(q, kp, vp, bt, max_context_len=n)
    desc.batch = 1
    need = binding.prefill_workspace_bytes(desc, chunk, chunk)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda:0")
    res = {"workload": f"one {chunk}-token chunk over a context of {n} tokens, {Hq}/{Hkv} heads, bf16",
           "workspace_MiB": need / 2**20}
    flops = 4.0 * D * (chunk * (n - chunk) + chunk * (chunk + 1) // 2) * Hq
    for name, w in (("unsplit", None), ("split", ws if need else None)):
        f = lambda: binding.paged_prefill_attention(desc, q, kp, vp, bt, cl, ql, cu, chunk, D ** -0.5, out, workspace=w)
        f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        res[name] = {"us": us, "tflops": flops / us / 1e6}
        if oracle_check:   # every row of the chunk
            res[name].update(prefill_error(torch, q, kp, vp, bt, np.array([n]), np.array([chunk]), out,
                                           np.arange(chunk), D ** -0.5))
    return res


def time_model_sweep(torch, binding, B=64, Hq=32, Hkv=8, seed=1009, tables=16, reps=3):
    """The execution-time model of the paper's Sec. 4.2, T_exec ~ N_ctx * d * sizeof(T) / BW_HBM:
    decode attention of a fixed batch of B sequences (8B-shaped heads, bf16) while their contexts
    grow from about 13 K to 262 K cached tokens in total; a straight line is fitted to time against
    KV bytes.  Every call reads other physical blocks of a 4 GiB pool (a fresh random table), so
    nothing is re-read from a cache."""
    import numpy as np
    from paper_2602_07878_amd import workloads as W
    D, bs = 128, 16
    nblk = (4 << 30) // (2 * Hkv * bs * D * 2)                      # K and V pools of 2 GiB each
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    kp = torch.randn(nblk, Hkv, bs, D, device="cuda:0", generator=g).bfloat16()
    vp = torch.randn(nblk, Hkv, bs, D, device="cuda:0", generator=g).bfloat16()
    q = torch.randn(B, Hq, D, device="cuda:0", generator=g).bfloat16()
    out = torch.empty(B, Hq, D, device="cuda:0")
    base = W.lens_uniform(seed, B, 128, 4096).astype(np.int64)     # the cfg2 length mix, scaled
    pts = []
    for frac in (0.1, 0.2, 0.3, 0.4, 0.5, 0.65, 0.8, 1.0, 1.25, 1.5, 2.0):
        lens = np.maximum(16, (base * frac).astype(np.int64)).astype(np.int32)
        nb = (lens + bs - 1) // bs
        maxb = int(nb.max())
        tabs = []
        for _ in range(tables):
            perm = torch.randperm(nblk, device="cuda:0", generator=g)[:int(nb.sum())].int().cpu().numpy()
            t = np.full((B, maxb), -1, np.int32)
            pos = 0
            for i in range(B):
                t[i, :nb[i]] = perm[pos:pos + nb[i]]
                pos += int(nb[i])
            tabs.append(torch.from_numpy(t).cuda())
        cl = torch.from_numpy(lens).cuda()
        desc = binding.attn_desc_for(q, kp, vp, tabs[0], max_context_len=int(lens.max()))
        ws = binding.new_workspace(binding.attn_workspace_bytes(desc), "cuda:0")
        # one plan per table, written ahead of the timed calls: in a decode step a plan serves
        # the calls of all layers, here every call has a table of its own
        plans = [binding.attn_plan(desc, t, cl) for t in tabs]
        fs = (lambda i: binding.paged_decode_attention_planned(desc, plans[i % tables], q, kp, vp, tabs[i % tables], cl,
                                                               D ** -0.5, out, workspace=ws),
              lambda i: binding.paged_decode_attention(q, kp, vp, tabs[i % tables], cl, D ** -0.5, out,
                                                       max_context_len=int(lens.max()), workspace=ws, desc=desc))
        us = []
        for f in fs:
            for i in range(tables):
                f(i)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(tables * reps):
                f(i)
            e1.record()
            torch.cuda.synchronize()
            us.append(e0.elapsed_time(e1) / (tables * reps) * 1e3)
        pts.append((int(lens.sum()), us[0], us[1]))
        del plans
    x = np.array([p[0] * 2 * Hkv * D * 2 for p in pts], np.float64)   # KV bytes per call

    def fit(col):
        y = np.array([p[col] for p in pts], np.float64)
        slope, icpt = np.polyfit(x, y, 1)
        r2 = 1.0 - float(((y - (slope * x + icpt)) ** 2).sum() / ((y - y.mean()) ** 2).sum())
        return {"points_tokens_us": [[p[0], round(p[col], 2)] for p in pts],
                "marginal_bandwidth_GBps": float(1e-3 / slope), "intercept_us": float(icpt), "r_squared": float(r2)}
    del kp, vp
    torch.cuda.empty_cache()
    res = {"model": "T_exec = a + N_ctx * bytes_per_token / BW (Sec. 4.2)", "batch": B,
           "calls": "paged_decode_attention_planned, the plans written ahead of the timed calls"}
    res.update(fit(1))
    res["without_plan"] = fit(2)
    return res


def serve_loop(torch, binding, steps, mode="recompute", seed=1007, chunked=False, swap_area="device"):
    """The scheduler model driving the GPU calls for `steps` engine iterations under a benign
    Poisson load that saturates the pool (the Fill state, with preemptions): per iteration the
    swaps, the prefills (new and recomputed requests: their K/V rows into the cache, then their
    attention), the KV append and the decode attention of one layer, 8B-shaped heads.  K/V contents are random; only shapes and tables matter here.
    chunked: prefills proceed in chunks under a 512-token budget per iteration (the example the
    paper's section on chunked prefill gives) instead of whole within 8192 tokens.
    swap_area: the scheduler's host blocks in a device buffer (the gather/scatter alone) or in
    page-locked host memory (the swap as the paper has it: over PCIe)."""
    import numpy as np
    from paper_2602_07878_amd import sched, workloads as W
    Hq, Hkv, D, bs = 32, 8, 128, 16
    n_gpu, n_cpu, max_blocks = 12288, 12288, 384
    s = sched.Scheduler(num_gpu_blocks=n_gpu, num_cpu_blocks=n_cpu, block_size=bs, max_num_seqs=256,
                        max_num_batched_tokens=512 if chunked else 8192, max_blocks_per_seq=max_blocks,
                        watermark_blocks=n_gpu // 100, mode=sched.SWAP if mode == "swap" else sched.RECOMPUTE,
                        chunked=chunked)
    stream = W.poisson_request_stream(seed, steps, 0.45, prompt_median=700, prompt_sigma=0.9, out_median=400,
                                      out_sigma=0.7, max_prompt=4096, max_new=1500)
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    kp = torch.randn(n_gpu, Hkv, bs, D, device="cuda:0", generator=g).bfloat16()
    vp = torch.randn(n_gpu, Hkv, bs, D, device="cuda:0", generator=g).bfloat16()
    if swap_area == "pinned host":
        sk, sv = (torch.empty(n_cpu, Hkv, bs, D, dtype=torch.bfloat16).pin_memory() for _ in range(2))
    else:
        sk, sv = (torch.empty(n_cpu, Hkv, bs, D, device="cuda:0", dtype=torch.bfloat16) for _ in range(2))
    bb = Hkv * bs * D * 2
    d_out, d_in = binding.swap_desc(1, bb, n_gpu, n_cpu), binding.swap_desc(1, bb, n_cpu, n_gpu)
    q_all = torch.randn(8192, Hq, D, device="cuda:0", generator=g).bfloat16()
    kn, vn = torch.randn(256, Hkv, D, device="cuda:0", generator=g).bfloat16(), \
        torch.randn(256, Hkv, D, device="cuda:0", generator=g).bfloat16()
    out = torch.empty(8192, Hq, D, device="cuda:0")
    kc_all = torch.randn(8192, Hkv, D, device="cuda:0", generator=g).bfloat16()     # the chunks' new K/V rows
    vc_all = torch.randn(8192, Hkv, D, device="cuda:0", generator=g).bfloat16()
    pf_ws = torch.empty(8192 * Hq * 16 * (D + 2) * 4, dtype=torch.uint8, device="cuda:0")   # most the split prefill asks for
    scale = D ** -0.5
    rec = []
    occ = []
    for arrivals in stream:
        for rid, pl, nn in arrivals:
            s.add_request(rid, pl, nn)
        info = s.step()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if info.num_swap_out_blocks:
            m = torch.from_numpy(s.swap_out()).cuda()
            binding.kv_block_swap(d_out, kp, sk, m)
            binding.kv_block_swap(d_out, vp, sv, m)
        if info.num_swap_in_blocks:
            m = torch.from_numpy(s.swap_in()).cuda()
            binding.kv_block_swap(d_in, sk, kp, m)
            binding.kv_block_swap(d_in, sv, vp, m)
        pf_tokens = 0
        if info.num_prefill:
            pid, ptok = s.prefills()
            pctx = s.prefill_contexts()
            rows = [(rid, t, c) for rid, t, c in zip(pid.tolist(), ptok.tolist(), pctx.tolist())]
            tabs = np.full((len(rows), max_blocks), -1, np.int32)
            keep = []
            for i, (rid, t, c) in enumerate(rows):
                try:
                    b = s.request_blocks(rid)
                except binding.PkvError:
                    continue                      # finished within its prefill
                tabs[i, :b.size] = b
                keep.append(i)
            if keep:
                tabs = tabs[keep]
                lens = np.array([rows[i][1] for i in keep], np.int32)      # query tokens (the chunk)
                ctxs = np.array([rows[i][2] for i in keep], np.int32)      # cached tokens after it
                pf_tokens = int(lens.sum())
                cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
                qv = q_all[:pf_tokens]
                desc = binding.attn_desc_for(qv, kp, vp, torch.from_numpy(tabs).cuda(), max_context_len=int(ctxs.max()))
                desc.batch = len(keep)
                d_tabs, d_ctx, d_len, d_cu = (torch.from_numpy(a).cuda() for a in (tabs, ctxs, lens, cu))
                binding.kv_append_chunk(desc, kc_all[:pf_tokens], vc_all[:pf_tokens], kp, vp, d_tabs, d_ctx, d_len, d_cu)
                need = binding.prefill_workspace_bytes(desc, pf_tokens, int(lens.max()))   # > 0: few long walks, split them
                binding.paged_prefill_attention(desc, qv, kp, vp, d_tabs, d_ctx, d_len, d_cu, int(lens.max()), scale,
                                                out[:pf_tokens], workspace=pf_ws[:need] if need else None)
        kv_tokens = 0
        if info.num_decode:
            ids, lens, tabs = s.decode_batch()
            B = len(ids)
            kv_tokens = int(lens.sum())
            bt, cl = torch.from_numpy(tabs).cuda(), torch.from_numpy(lens).cuda()
            desc = binding.attn_desc_for(q_all[:B], kp, vp, bt, max_context_len=int(lens.max()))
            binding.kv_append(desc, kn[:B], vn[:B], kp, vp, bt, cl)
            binding.paged_decode_attention(q_all[:B], kp, vp, bt, cl, scale, out[:B], max_context_len=int(lens.max()),
                                           desc=desc)
        e1.record()
        rec.append((e0, e1, info.num_decode, kv_tokens, pf_tokens, info.num_preempted,
                    info.num_swap_out_blocks + info.num_swap_in_blocks))
        occ.append(1.0 - info.free_blocks / n_gpu)
    torch.cuda.synchronize()
    us = np.array([a.elapsed_time(b) * 1e3 for a, b, *_ in rec])
    dec = np.array([r[2] for r in rec]); kvt = np.array([r[3] for r in rec]); pft = np.array([r[4] for r in rec])
    pre = np.array([r[5] for r in rec])
    steady = np.arange(len(rec)) >= len(rec) // 4          # after the pool has filled
    quiet = steady & (pft == 0) & (pre == 0) & (dec > 0)     # iterations that only decode
    t = s.totals()
    q = lambda a, f: float(np.percentile(a, f)) if a.size else None
    swp = np.array([r[6] for r in rec])
    swapping = steady & (swp > 0)
    return {"iterations": len(rec), "mode": mode, "swap_area": swap_area if mode == "swap" else None,
            "iteration_us_with_swaps_p50_p90": [q(us[swapping], 50), q(us[swapping], 90)] if swapping.any() else None,
            "blocks_per_swapping_iteration_mean": float(swp[swapping].mean()) if swapping.any() else None,
            "chunked_prefill_budget": 512 if chunked else None,
            "finished": t["finished"], "preemptions": t["preemptions"],
            "head_blocked_iterations": t["blocked"], "recomputed_tokens": t["recomputed"],
            "swapped_blocks": t["swap_out"] + t["swap_in"],
            "pool_occupancy_min_max_after_fill": [float(np.min(np.array(occ)[steady])), float(np.max(np.array(occ)[steady]))],
            "decode_batch_mean": float(dec[steady].mean()), "kv_tokens_per_iteration_mean": float(kvt[steady].mean()),
            "iteration_us_decode_only_p50_p90": [q(us[quiet], 50), q(us[quiet], 90)],
            "iteration_us_with_prefill_or_preemption_p50_p90": [q(us[steady & ~quiet & (dec > 0)], 50),
                                                                q(us[steady & ~quiet & (dec > 0)], 90)],
            "decode_only_kv_GBps_mean": float((kvt[quiet] * 4096 / us[quiet] / 1e3).mean()) if quiet.any() else None,
            "note": "one layer; an iteration's GPU time includes the Python-side launches of this script"}


def probe_ceilings(torch, binding, nbytes=4 << 30, reps=5):
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").random_(0, 255)
    b = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    sink = torch.empty(1 << 16, dtype=torch.uint8, device="cuda:0")
    out = {}
    for name, fn, traffic in (("read", lambda: binding.probe_read(a, sink, nbytes), nbytes),
                              ("copy", lambda: binding.probe_copy(a, b, nbytes), 2 * nbytes)):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        out[name + "_GBps"] = traffic / (e0.elapsed_time(e1) / reps) / 1e6
    del a, b
    torch.cuda.empty_cache()
    return out


def cpu_baseline(w, reps=3):
    """The fp64 oracle, untouched, timed on this host's cores on the same workload."""
    import oracle
    best = None
    for _ in range(reps):
        t = time.perf_counter()
        ref = oracle.paged_decode_attention(w.q, w.k_pool, w.v_pool, w.block_tables,
                                            w.context_lens, w.scale, block_size=w.block_size)
        dt = time.perf_counter() - t
        best = dt if best is None else min(best, dt)
    res = {"value": w.kv_bytes / best / 1e9, "unit": "KV GB/s", "cores": oracle.num_threads(),
           "kind": "oracle", "seconds": best,
           "sample": f"the full {w.name} workload (all {w.B} sequences, {w.Hq} heads), "
                     f"best of {reps} runs"}
    try:                                    # the same on one thread, once
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1, user_api="openmp"):
            if oracle.num_threads() == 1:
                t = time.perf_counter()
                oracle.paged_decode_attention(w.q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, w.scale,
                                              block_size=w.block_size)
                dt = time.perf_counter() - t
                res["one_thread"] = {"value": w.kv_bytes / dt / 1e9, "unit": "KV GB/s", "seconds": dt}
    except ImportError:
        pass
    return ref, res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--layers", type=int, default=16, help="distinct KV layer pools cycled over")
    ap.add_argument("--no-swap", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-overlap", action="store_true",
                    help="skip the decode calls timed while a swap-out runs (keeps a kernel trace's rows apart)")
    ap.add_argument("--no-extra", action="store_true", help="skip the Fill and long-context configurations")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the fit of the paper's linear execution-time model to a sweep of the cached context")
    ap.add_argument("--serve", type=int, default=0, metavar="ITERATIONS",
                    help="also run the scheduler-driven serving loop for this many engine iterations")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only; --gpus must be 1 (the kernels need no "
              "collective: every GPU of a tensor-parallel group would run them on its own KV heads)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_07878_amd import binding, workloads as W
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()   # fail loudly if the HIP library is missing

    t = time.time()
    w = W.config2_llama8b()
    log(f"[bench] generated {w.name}: T={w.total_tokens} tokens, KV bytes/call={w.kv_bytes/1e6:.1f} MB "
        f"({time.time()-t:.1f}s)")
    d = upload_attn(w, args.layers, torch)
    # pass 1 (the timed region behind `value`): K plain calls.  Pass 2: K calls that also record
    # an event before and after every launch of the streaming kernel; the two extra stream
    # markers per call cost a few microseconds, which is why `value` does not come from it.
    # the calls without a plan first (every call works the tables out for itself; a kernel of its own)
    out_u, ms_u, _, _ = time_attention(w, d, args.steps, args.warmup, torch, binding)
    _, _, _, kern_u = time_attention(w, d, args.steps, 4, torch, binding, kernel_events=True)
    # The headline: the calls bring a per-step plan (Sec. 4.2: the layer calls of a step share tables
    # and lengths), written once per PLAN_EVERY calls, at least once, inside the timed region.
    out, ms, wall_ms, _ = time_attention(w, d, args.steps, args.warmup, torch, binding, planned=True)
    _, ms_ev, _, kern = time_attention(w, d, args.steps, 4, torch, binding, kernel_events=True, planned=True)
    kern_ms = sum(kern) / len(kern)
    pct = lambda q: kern[min(len(kern) - 1, int(q * len(kern)))] * 1e3
    gbps = w.kv_bytes / ms / 1e6
    kern_gbps = w.kv_bytes / kern_ms / 1e6
    log(f"[bench] attention: {ms*1e3:.1f} us/call, {gbps:.0f} KV GB/s = {gbps/HBM_PEAK_GBS:.1%} of HBM peak; "
        f"streaming kernel alone {kern_ms*1e3:.1f} us = {kern_gbps:.0f} GB/s")

    result = {
        "metric": "decode-attention KV GB/s", "value": gbps, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.B, "q_heads": w.Hq, "kv_heads": w.Hkv,
                   "head_dim": w.D, "block_size": w.block_size, "context_tokens": w.total_tokens,
                   "kv_bytes_per_call": w.kv_bytes, "layer_pools_cycled": args.layers,
                   "partition_tokens": w.partition_tokens,    # 0: split chosen by the library
                   "plan": f"pkv_attn_plan once per {PLAN_EVERY} calls, inside the timed region"},
        "frac_hbm_peak": gbps / HBM_PEAK_GBS,
        "decode_tokens_per_s": w.B / (ms * 1e-3),
        "kv_tokens_per_s": w.total_tokens / (ms * 1e-3),
        "wall_ms_per_step": wall_ms,
        "roofline": {"bound": "hbm", "achieved": kern_gbps, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": kern_gbps / HBM_PEAK_GBS, "traffic": recorded_traffic(w.name, STREAM_KERNEL),
                     "traffic_source": "recorded: profiles/attn_stream_cfg2_hbm_traffic.txt (rocprofv3 --pmc, "
                                       "null when the kernel's sources have changed since)",
                     "kernel": STREAM_KERNEL, "us_per_launch": kern_ms * 1e3,
                     "us_per_launch_p10_p50_p90": [pct(0.1), pct(0.5), pct(0.9)],
                     "algorithmic_bytes_per_launch": w.kv_bytes,
                     "timed_region": f"second pass of {args.steps} steps with an event before and after "
                                     f"each launch ({ms_ev * 1e3:.1f} us per call in that pass)"},
    }
    ku = sum(kern_u) / len(kern_u)
    result["without_plan"] = {"ms": ms_u, "kv_GBps": w.kv_bytes / ms_u / 1e6, "frac_hbm_peak": w.kv_bytes / ms_u / 1e6 / HBM_PEAK_GBS,
                              "kernel": "attn_stream_mfma_d128<4>", "kernel_us": ku * 1e3,
                              "kernel_GBps": w.kv_bytes / ku / 1e6, "kernel_frac": w.kv_bytes / ku / 1e6 / HBM_PEAK_GBS,
                              "max_abs_diff_to_planned": float((out - out_u).abs().max())}
    log(f"[bench] without a plan: {result['without_plan']}")
    result["kv_append"] = time_append(w, d, torch, binding)
    log(f"[bench] append ahead of attention: {result['kv_append']}")
    result["ceilings"] = probe_ceilings(torch, binding)
    result["prefill"] = time_prefill(torch, binding)
    log(f"[bench] prefill: {result['prefill']}")
    result["prefill_kv_f8e4m3"] = time_prefill(torch, binding, f8=True)
    log(f"[bench] prefill over 8-bit pools: {result['prefill_kv_f8e4m3']}")
    result["prefill_chunk"] = time_prefill_chunk(torch, binding)
    log(f"[bench] prefill chunk: {result['prefill_chunk']}")
    log(f"[bench] ceilings: {result['ceilings']}")

    if not args.no_cpu:
        ref, cb = cpu_baseline(w)
        err = float(np.abs(out.cpu().numpy().astype(np.float64) - ref).max())
        result["cpu_baseline"] = cb
        result["max_abs_err_vs_oracle"] = err
        log(f"[bench] oracle: {cb['seconds']:.2f}s on {cb['cores']} threads = {cb['value']:.2f} KV GB/s; "
            f"GPU max abs err {err:.2e}")
    del d
    torch.cuda.empty_cache()

    if not args.no_swap:
        swh = W.config4_squeeze(victims=16)
        w2 = W.config2_llama8b()
        result["swap_host_leg"] = time_swap_host(
            swh, torch, binding, decode_batch=None if args.no_overlap else (w2, upload_attn(w2, 8, torch)))
        log(f"[bench] swap host leg {swh.name} ({int(swh.victim_lens.size)} victims): {result['swap_host_leg']}")
        swap = {}
        for sw in (W.config4_squeeze(), W.config4_evict_all_256(), W.config4_squeeze_f8()):
            swap[sw.name] = time_swap(sw, 5, torch, binding)
            log(f"[bench] swap {sw.name}: {swap[sw.name]}")
        result["swap"] = swap

    # every kernel family against the roofline that bounds it (the headline one is `roofline`)
    rl = {"paged_prefill_attention": {"bound": "mfma", "achieved": result["prefill"]["tflops"],
                                      "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                      "frac": result["prefill"]["frac"], "workload": result["prefill"]["workload"],
                                      "max_abs_err_vs_oracle": result["prefill"].get("max_abs_err_vs_oracle")}}
    for name, sres in result.get("swap", {}).items():
        for leg in ("gather", "scatter"):
            rl[f"kv_block_swap_{leg}_{name}"] = {"bound": "hbm", "achieved": sres[leg]["traffic_GBps"],
                                                 "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                                 "frac": sres[leg]["frac_hbm_peak"],
                                                 "algorithmic_bytes": 2 * int(sres["payload_GB"] * 1e9)}
    result["other_rooflines"] = rl

    if not args.no_extra:
        # The headline batch with an 8-bit (E4M3) KV cache: the same tokens, half the bytes.
        t = time.time()
        w8 = W.config2_llama8b_f8()
        d8 = upload_attn(w8, args.layers, torch)
        out8u, ms8u, _, k8us = time_attention(w8, d8, 128, 32, torch, binding, kernel_events=True)
        out8, ms8, _, k8s = time_attention(w8, d8, 128, 32, torch, binding, kernel_events=True, planned=True)
        k8, k8u = sum(k8s) / len(k8s), sum(k8us) / len(k8us)
        g8 = w8.kv_bytes / ms8 / 1e6
        f8 = {"ms": ms8, "kv_GBps": g8, "frac_hbm_peak": g8 / HBM_PEAK_GBS, "kernel_ms": k8,
              "context_tokens": w8.total_tokens, "kv_bytes_per_call": w8.kv_bytes, "bytes_per_token": 2 * w8.Hkv * w8.D,
              "kv_tokens_per_s": w8.total_tokens / (ms8 * 1e-3),
              "plan": f"pkv_attn_plan once per {PLAN_EVERY} calls, inside the timed region",
              "without_plan": {"ms": ms8u, "kernel_ms": k8u, "same_bits": bool((out8 == out8u).all())}}
        if not args.no_cpu:
            import oracle
            ref8 = oracle.paged_decode_attention(w8.q, w8.k_pool, w8.v_pool, w8.block_tables, w8.context_lens,
                                                 w8.scale, block_size=w8.block_size)
            f8["max_abs_err_vs_oracle"] = float(np.abs(out8.cpu().numpy().astype(np.float64) - ref8).max())
        rl[f"paged_decode_attention_{w8.name}"] = {
            "bound": "hbm", "achieved": w8.kv_bytes / k8 / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": w8.kv_bytes / k8 / 1e6 / HBM_PEAK_GBS, "us_per_launch": k8 * 1e3, "per_call_GBps": g8,
            "per_call_frac": g8 / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": w8.kv_bytes,
            "max_abs_err_vs_oracle": f8.get("max_abs_err_vs_oracle")}
        result["kv_f8e4m3"] = f8
        log(f"[bench] {w8.name}: {f8} (setup {time.time()-t:.0f}s)")
        del d8
        torch.cuda.empty_cache()

        # The other decode configurations, each through the same call, with its own kernel time
        # (events attached to the streaming kernel's dispatch) and its error against the oracle on
        # the full workload: the Fill-state mix, and the long-context batch as configured
        # (512-token partials) and with the library's own split.
        extra = {}
        for mk, layers in ((W.config3_fill, 4), (W.config5_long70b, 2)):
            t = time.time()
            wx = mk()
            dx = upload_attn(wx, layers, torch)
            refx = None
            if not args.no_cpu:
                import oracle
                refx = oracle.paged_decode_attention(wx.q, wx.k_pool, wx.v_pool, wx.block_tables, wx.context_lens,
                                                     wx.scale, block_size=wx.block_size)
            for pt in sorted({wx.partition_tokens, 0}, reverse=True):
                wx.partition_tokens = pt
                outx, msx, _, kxs = time_attention(wx, dx, 40, 8, torch, binding, kernel_events=True)
                kx = sum(kxs) / len(kxs)
                g = wx.kv_bytes / msx / 1e6
                key = wx.name + (f"_partition{pt}" if pt else "")
                extra[key] = {"ms": msx, "kv_GBps": g, "frac_hbm_peak": g / HBM_PEAK_GBS,
                              "kernel_ms": kx, "context_tokens": wx.total_tokens,
                              "partition_tokens": pt, "kv_bytes_per_call": wx.kv_bytes}
                if refx is not None:
                    extra[key]["max_abs_err_vs_oracle"] = float(np.abs(outx.cpu().numpy().astype(np.float64) - refx).max())
                outp, msp, _, kps = time_attention(wx, dx, 40, 8, torch, binding, kernel_events=True, planned=True)
                extra[key]["with_plan"] = {"ms": msp, "kernel_ms": sum(kps) / len(kps),
                                           "frac_hbm_peak": wx.kv_bytes / msp / 1e6 / HBM_PEAK_GBS,
                                           "max_abs_diff_to_unplanned": float((outp - outx).abs().max())}
                rl[f"paged_decode_attention_{key}"] = {
                    "bound": "hbm", "achieved": wx.kv_bytes / kx / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": wx.kv_bytes / kx / 1e6 / HBM_PEAK_GBS, "us_per_launch": kx * 1e3,
                    "per_call_GBps": g, "per_call_frac": g / HBM_PEAK_GBS,
                    "algorithmic_bytes_per_launch": wx.kv_bytes,
                    "max_abs_err_vs_oracle": extra[key].get("max_abs_err_vs_oracle")}
                log(f"[bench] {key}: {extra[key]} (setup {time.time()-t:.0f}s)")
            del dx
            torch.cuda.empty_cache()
        result["other_configs"] = extra

    if not args.no_sweep:
        # Sec. 4.2: time linear in the KV bytes streamed; the fit is an acceptance item (R^2 >= 0.98)
        result["time_model"] = time_model_sweep(torch, binding)
        result["time_model"]["r_squared_at_least_0.98"] = result["time_model"]["r_squared"] >= 0.98
        log(f"[bench] time model: {result['time_model']}")
    if args.serve > 0:
        result["serving_loop"] = {m: serve_loop(torch, binding, args.serve, mode=m) for m in ("recompute", "swap")}
        result["serving_loop"]["swap_to_pinned_host"] = serve_loop(torch, binding, args.serve, mode="swap",
                                                                   swap_area="pinned host")
        result["serving_loop"]["recompute_chunked_prefill"] = serve_loop(torch, binding, args.serve, mode="recompute",
                                                                         chunked=True)
        log(f"[bench] serving loop: {result['serving_loop']}")

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
