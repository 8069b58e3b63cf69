"""The scheduler model driving the GPU calls over time (Sec. 5.1 dynamics -> the data movement
of Sec. 2.2, 4.2 and 5.1.2): every engine iteration moves preempted requests' blocks out to a
swap area and returning ones back with kv_block_swap, appends the new tokens' K/V with
kv_append and runs paged_decode_attention on the scheduler's block tables.  The same sequence
is replayed on numpy pools with the oracle: pools must agree bit for bit after every swap, and
attention within tolerance."""
import numpy as np
import pytest

from paper_2602_07878_amd import workloads as W

pytestmark = pytest.mark.gpu

HKV, HQ, D, BS = 2, 8, 128, 16


def rows_of(rid, n):
    """All K and V rows request `rid` will ever cache (stand-in for what a model computes)."""
    rng = np.random.default_rng([7, rid])
    k = W.f32_to_bf16_bits(rng.standard_normal((n, HKV, D)).astype(np.float32))
    v = W.f32_to_bf16_bits(rng.standard_normal((n, HKV, D)).astype(np.float32))
    return k, v


@pytest.mark.parametrize("mode,chunked,swap_area", [("swap", False, "device"), ("recompute", False, "device"),
                                                    ("swap", True, "device"), ("recompute", True, "device"),
                                                    ("swap", False, "pinned host")])
def test_scheduler_driven_decode_with_preemption(mode, chunked, swap_area):
    """With chunked=True prompts are prefilled in chunks under a 64-token budget, and the chunks'
    causal attention over the paged cache (paged_prefill_attention on the scheduler's tables,
    query_lens = chunk, context_lens = tokens cached after it) is checked against the oracle.
    swap_area: where the scheduler's host blocks live: a device buffer standing in for host
    memory, or page-locked host memory that kv_block_swap reads and writes over the link."""
    import oracle
    import torch
    from paper_2602_07878_amd import binding, sched
    n_gpu, n_cpu = 80, 64
    s = sched.Scheduler(num_gpu_blocks=n_gpu, num_cpu_blocks=n_cpu, block_size=BS, max_num_seqs=16,
                        max_num_batched_tokens=64 if chunked else 1024, max_blocks_per_seq=24,
                        mode=sched.SWAP if mode == "swap" else sched.RECOMPUTE, chunked=chunked)
    stream = W.poisson_request_stream(31, 120, 0.35, prompt_median=100, out_median=90, max_prompt=250, max_new=130)
    stream += [[] for _ in range(1500 if chunked else 500)]      # (a 64-token budget drains the queue more slowly)
    rows = {}
    up = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    # pools [blocks][Hkv][bs][D] as bf16 bits (NaN wherever nothing was written yet); the swap
    # area has the same block shape (a device buffer stands in for host memory)
    hk = np.full((n_gpu, HKV, BS, D), 0x7FC0, np.uint16)
    hv = hk.copy()
    sk, sv = np.zeros((n_cpu, HKV, BS, D), np.uint16), np.zeros((n_cpu, HKV, BS, D), np.uint16)
    dk, dv, dsk, dsv = up(hk), up(hv), up(sk), up(sv)
    if swap_area == "pinned host":
        dsk, dsv = (torch.from_numpy(a.view(np.int16).copy()).pin_memory().view(torch.bfloat16) for a in (sk, sv))
    block_bytes = HKV * BS * D * 2
    out_desc = binding.swap_desc(1, block_bytes, n_gpu, n_cpu)
    in_desc = binding.swap_desc(1, block_bytes, n_cpu, n_gpu)
    scale = float(D) ** -0.5
    checked = swaps = prefill_checked = later_chunks = split_used = 0
    rng = np.random.default_rng(99)
    for it, arrivals in enumerate(stream):
        for rid, p, n in arrivals:
            s.add_request(rid, p, n)
            rows[rid] = rows_of(rid, p + n)
        info = s.step()
        # 1. swaps: victims leave before anything is written into the blocks they gave up
        for count, getter, desc, src, dst, hsrc, hdst in (
                (info.num_swap_out_blocks, s.swap_out, out_desc, (dk, dv), (dsk, dsv), (hk, hv), (sk, sv)),
                (info.num_swap_in_blocks, s.swap_in, in_desc, (dsk, dsv), (dk, dv), (sk, sv), (hk, hv))):
            if count:
                m = getter()
                dm = torch.from_numpy(m).cuda()
                for a, b, ha, hb in zip(src, dst, hsrc, hdst):
                    binding.kv_block_swap(desc, a, b, dm)
                    oracle.kv_block_swap(ha, hb, m, num_planes=1, block_bytes=block_bytes)
                swaps += 1
        # 2. prefills (new and recomputed requests): the model's rows land in the request's blocks
        pid, ptok = s.prefills()
        pctx = s.prefill_contexts()
        chunk_rows = []                                     # (block table row, chunk tokens, cached tokens after)
        new_k, new_v = [], []
        for rid, tokens, ctx in zip(pid.tolist(), ptok.tolist(), pctx.tolist()):
            assert chunked or ctx == tokens
            try:
                blocks = s.request_blocks(rid)
            except binding.PkvError:
                continue                                    # finished within its prefill
            tok = np.arange(ctx - tokens, ctx)              # the chunk's positions
            k_all, v_all = rows[rid]
            new_k.append(k_all[tok]); new_v.append(v_all[tok])
            row = np.full(24, -1, np.int32)
            row[:blocks.size] = blocks
            chunk_rows.append((row, tokens, ctx))
            later_chunks += ctx > tokens
        if chunk_rows:                                      # the chunks' K/V rows join the cache: kv_append_chunk
            tabs_c = np.stack([r for r, _, _ in chunk_rows])
            ql_c = np.array([t for _, t, _ in chunk_rows], np.int32)
            cl_c = np.array([c for _, _, c in chunk_rows], np.int32)
            kn_c, vn_c = np.concatenate(new_k), np.concatenate(new_v)
            oracle.kv_append_chunk(hk, hv, kn_c, vn_c, tabs_c, cl_c, ql_c, block_size=BS)
            d_bt = torch.from_numpy(tabs_c).cuda()
            dkn, dvn = up(kn_c), up(vn_c)
            desc_c = binding.attn_desc_for(torch.empty(1, HQ, D, dtype=torch.bfloat16, device="cuda"), dk, dv, d_bt,
                                           max_context_len=int(cl_c.max()))
            desc_c.batch = len(chunk_rows)
            cu_c = torch.from_numpy(np.concatenate([[0], np.cumsum(ql_c)]).astype(np.int32)).cuda()
            binding.kv_append_chunk(desc_c, dkn, dvn, dk, dv, d_bt, torch.from_numpy(cl_c).cuda(),
                                    torch.from_numpy(ql_c).cuda(), cu_c)
        if chunked and chunk_rows and (it % 5 == 0 or any(c > t for _, t, c in chunk_rows)) and prefill_checked < 60:
            tabs = np.stack([r for r, _, _ in chunk_rows])
            ql = np.array([t for _, t, _ in chunk_rows], np.int32)
            cl = np.array([c for _, _, c in chunk_rows], np.int32)
            q = W.f32_to_bf16_bits(rng.standard_normal((int(ql.sum()), HQ, D)).astype(np.float32))
            ref = oracle.paged_prefill_attention(q, hk, hv, tabs, cl, ql, scale, block_size=BS)
            dq, bt = up(q), torch.from_numpy(tabs).cuda()
            cu = torch.from_numpy(np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)).cuda()
            out = torch.empty(int(ql.sum()), HQ, D, dtype=torch.float32, device="cuda")
            desc = binding.attn_desc_for(dq, dk, dv, bt, max_context_len=int(cl.max()))
            desc.batch = len(chunk_rows)
            need = binding.prefill_workspace_bytes(desc, int(ql.sum()), int(ql.max()))      # few chunks: split walks
            ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
            split_used += need > 0
            binding.paged_prefill_attention(desc, dq, dk, dv, bt, torch.from_numpy(cl).cuda(),
                                            torch.from_numpy(ql).cuda(), cu, int(ql.max()), scale, out, workspace=ws)
            torch.cuda.synchronize()
            got = out.cpu().numpy().astype(np.float64)
            assert np.all(np.isfinite(got)) and np.abs(got - ref).max() <= 2e-3, (it, mode, "chunk")
            prefill_checked += 1
        # 3. decode: append the new tokens' rows, then attention over the grown contexts
        if info.num_decode:
            ids, lens, tabs = s.decode_batch()
            kn = np.stack([rows[r][0][c - 1] for r, c in zip(ids.tolist(), lens.tolist())])
            vn = np.stack([rows[r][1][c - 1] for r, c in zip(ids.tolist(), lens.tolist())])
            bt, cl = torch.from_numpy(tabs).cuda(), torch.from_numpy(lens).cuda()
            q = W.f32_to_bf16_bits(rng.standard_normal((info.num_decode, HQ, D)).astype(np.float32))
            dq = up(q)
            desc = binding.attn_desc_for(dq, dk, dv, bt, max_context_len=int(lens.max()))
            binding.kv_append(desc, up(kn), up(vn), dk, dv, bt, cl)
            oracle.kv_append(hk, hv, kn, vn, tabs, lens, block_size=BS)
            if it % 9 == 0 or info.num_swap_in_blocks or info.num_preempted:
                out = torch.empty(info.num_decode, HQ, D, dtype=torch.float32, device="cuda")
                binding.paged_decode_attention(dq, dk, dv, bt, cl, scale, out, max_context_len=int(lens.max()))
                ref = oracle.paged_decode_attention(q, hk, hv, tabs, lens, scale, block_size=BS)
                torch.cuda.synchronize()
                got = out.cpu().numpy().astype(np.float64)
                assert np.all(np.isfinite(got)) and np.abs(got - ref).max() <= 2e-3, (it, mode)
                checked += 1
        if info.num_swap_out_blocks or info.num_swap_in_blocks or it % 50 == 0:
            torch.cuda.synchronize()
            assert np.array_equal(bits(dk), hk) and np.array_equal(bits(dv), hv), it
            assert np.array_equal(bits(dsk), sk) and np.array_equal(bits(dsv), sv), it
    t = s.totals()
    print(mode, "chunked" if chunked else "whole prefills", t, "attention checks", checked,
          "chunk attention checks", prefill_checked, "of which with split walks", split_used,
          "later chunks", later_chunks, flush=True)
    assert t["finished"] == sum(len(a) for a in stream) and t["preemptions"] > 0 and checked > 20
    if chunked:
        assert prefill_checked > 20 and later_chunks > 20
    if mode == "swap":
        assert swaps > 0 and t["swap_in"] == t["swap_out"] > 0
    else:
        assert t["recomputed"] > 0
