"""A decode step (kv_append, then paged_decode_attention: stream kernel + merge) and a prefill
chunk with split walks captured into a HIP graph and replayed: the calls enqueue kernels only
(no allocation, no synchronisation, no memset), so a launch-bound serving loop can replay them.
The graph is replayed several times with the program's own eager work and synchronisations in
between, the inputs changed in place before each replay, and every replay is checked against
the eager result of the same inputs and against the oracle."""
import numpy as np
import pytest

from paper_2602_07878_amd import workloads as W
from helpers import to_device

pytestmark = pytest.mark.gpu


def up(a):
    import torch
    return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)


def test_decode_step_and_split_prefill_replayed_from_a_graph():
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    w = W.make_attn_workload("graph", 91, dtype="bf16", Hq=32, Hkv=8, D=128, block_size=16,
                             context_lens=list(W.lens_uniform(91, 24, 40, 3000)), pool_factor=1.2)
    dev = to_device(w)
    q, kp, vp, bt, cl = dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"], dev["context_lens"]
    kn = torch.zeros(w.B, w.Hkv, w.D, dtype=torch.bfloat16, device="cuda")
    vn = torch.zeros_like(kn)
    out_g = torch.zeros(w.B, w.Hq, w.D, dtype=torch.float32, device="cuda")
    out_e = torch.zeros_like(out_g)
    desc = binding.attn_desc_for(q, kp, vp, bt, max_context_len=w.max_context_len)
    ws = binding.new_workspace(binding.attn_workspace_bytes(desc), "cuda")
    # the chunk: the last 200 tokens of sequence 0 alone (few workgroups, so the walks are split)
    n0 = int(w.context_lens[0])
    w1 = W.make_attn_workload("graph_chunk", 92, dtype="bf16", Hq=32, Hkv=8, D=128, block_size=16,
                              context_lens=[2600], pool_factor=1.1)
    d1 = to_device(w1)
    cq = torch.zeros(200, 32, 128, dtype=torch.bfloat16, device="cuda")
    cout_g = torch.zeros(200, 32, 128, dtype=torch.float32, device="cuda")
    cout_e = torch.zeros_like(cout_g)
    ql = torch.tensor([200], dtype=torch.int32, device="cuda")
    cu = torch.tensor([0, 200], dtype=torch.int32, device="cuda")
    desc1 = binding.attn_desc_for(cq, d1["k_pool"], d1["v_pool"], d1["block_tables"], max_context_len=2600)
    desc1.batch = 1
    need = binding.prefill_workspace_bytes(desc1, 200, 200)
    assert need > 0
    pws = torch.empty(need, dtype=torch.uint8, device="cuda")

    def step(out, cout):
        binding.kv_append(desc, kn, vn, kp, vp, bt, cl)
        binding.paged_decode_attention(q, kp, vp, bt, cl, w.scale, out, max_context_len=w.max_context_len,
                                       workspace=ws, desc=desc)
        binding.paged_prefill_attention(desc1, cq, d1["k_pool"], d1["v_pool"], d1["block_tables"], d1["context_lens"],
                                        ql, cu, 200, w1.scale, cout, workspace=pws)

    step(out_e, cout_e)                                   # warm-up: kernel attributes are set on first use
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(out_g, cout_g)
    rng = np.random.default_rng(93)
    hk, hv = w.k_pool, w.v_pool
    for replay in range(4):
        # new inputs in place: queries, the rows to append, the chunk's queries
        qn = W.f32_to_bf16_bits(rng.standard_normal((w.B, w.Hq, w.D)).astype(np.float32))
        knn = W.f32_to_bf16_bits(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
        vnn = W.f32_to_bf16_bits(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
        cqn = W.f32_to_bf16_bits(rng.standard_normal((200, 32, 128)).astype(np.float32))
        q.copy_(up(qn)); kn.copy_(up(knn)); vn.copy_(up(vnn)); cq.copy_(up(cqn))
        out_g.fill_(-7.0); cout_g.fill_(-7.0)
        g.replay()
        torch.cuda.synchronize()
        step(out_e, cout_e)                               # eager work of the same inputs between the replays
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e) and torch.equal(cout_g, cout_e), replay     # same kernels, same split: bit-equal
        oracle.kv_append(hk, hv, knn, vnn, w.block_tables, w.context_lens, block_size=16)
        ref = oracle.paged_decode_attention(qn, hk, hv, w.block_tables, w.context_lens, w.scale, block_size=16)
        assert np.abs(out_g.cpu().numpy().astype(np.float64) - ref).max() <= 2e-3, replay
        cref = oracle.paged_prefill_attention(cqn, w1.k_pool, w1.v_pool, w1.block_tables, w1.context_lens,
                                              np.array([200], np.int32), w1.scale, block_size=16)
        assert np.abs(cout_g.cpu().numpy().astype(np.float64) - cref).max() <= 2e-3, replay


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f8"])
def test_planned_decode_step_replayed_from_a_graph(dtype, fused):
    """One decode step as a serving loop would capture it: pkv_attn_plan, then for each of three
    layers kv_append and paged_decode_attention_planned on that layer's pools (fused: the append
    inside the attention call).  Between replays
    the context lengths grow by a token (in place, as a scheduler does), so every replay builds
    another plan; each is checked against the eager calls and against the oracle."""
    import oracle
    import torch
    from paper_2602_07878_amd import binding
    layers = 3
    lens = [int(x) for x in W.lens_uniform(95, 20, 30, 2500)]
    import copy
    base = W.make_attn_workload("graph_planned", 96, dtype=dtype, Hq=32, Hkv=8, D=128, block_size=16,
                                context_lens=[n + 8 for n in lens], pool_factor=1.2)
    base.context_lens = np.asarray(lens, np.int32).copy()        # the contexts start 8 tokens short of their blocks
    ws_ = [base]
    for l in range(1, layers):         # other layers: the same tables, other contents (dims rotated, K and V exchanged)
        w = copy.deepcopy(base)
        w.k_pool = np.roll(base.v_pool if l % 2 else base.k_pool, 5 * l, axis=-1).copy()
        w.v_pool = np.roll(base.k_pool if l % 2 else base.v_pool, 3 * l, axis=-1).copy()
        w.q = np.roll(base.q, l, axis=1).copy()
        ws_.append(w)
    devs = [to_device(w) for w in ws_]
    bt, cl = devs[0]["block_tables"], devs[0]["context_lens"]
    w0 = ws_[0]
    desc = binding.attn_desc_for(devs[0]["q"], devs[0]["k_pool"], devs[0]["v_pool"], bt,
                                 max_context_len=max(lens) + 8)
    plan = torch.zeros(binding.lib().pkv_attn_plan_bytes(desc), dtype=torch.uint8, device="cuda")
    wsp = binding.new_workspace(binding.attn_workspace_bytes(desc), "cuda")
    kdt = devs[0]["k_pool"].dtype
    kn = [torch.zeros(w0.B, w0.Hkv, w0.D, dtype=kdt, device="cuda") for _ in range(layers)]
    vn = [torch.zeros_like(kn[0]) for _ in range(layers)]
    outs_g = [torch.zeros(w0.B, w0.Hq, w0.D, device="cuda") for _ in range(layers)]
    outs_e = [torch.zeros_like(outs_g[0]) for _ in range(layers)]

    def step(outs):
        binding.attn_plan(desc, bt, cl, plan)
        for l in range(layers):
            d = devs[l]
            if not fused:
                binding.kv_append(desc, kn[l], vn[l], d["k_pool"], d["v_pool"], bt, cl)
            binding.paged_decode_attention_planned(desc, plan, d["q"], d["k_pool"], d["v_pool"], bt, cl, w0.scale,
                                                   outs[l], workspace=wsp, k_new=kn[l] if fused else None,
                                                   v_new=vn[l] if fused else None)

    cl += 1
    step(outs_e)                                          # warm-up
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(outs_g)
    rng = np.random.default_rng(97)
    host_len = np.asarray(lens, np.int32) + 1
    for l in range(layers):                               # the oracle's pools follow the warm-up append (rows of zeros)
        z = np.zeros((w0.B, w0.Hkv, w0.D), ws_[l].k_pool.dtype)
        oracle.kv_append(ws_[l].k_pool, ws_[l].v_pool, z, z, w0.block_tables, host_len, block_size=16)
    for replay in range(4):
        cl += 1
        host_len += 1
        rows = []
        for l in range(layers):
            if dtype == "bf16":
                a = W.f32_to_bf16_bits(rng.standard_normal((w0.B, w0.Hkv, w0.D)).astype(np.float32))
                b = W.f32_to_bf16_bits(rng.standard_normal((w0.B, w0.Hkv, w0.D)).astype(np.float32))
                kn[l].copy_(up(a)); vn[l].copy_(up(b))
            else:
                a = W.f32_to_f8e4m3_bits(rng.standard_normal((w0.B, w0.Hkv, w0.D)).astype(np.float32))
                b = W.f32_to_f8e4m3_bits(rng.standard_normal((w0.B, w0.Hkv, w0.D)).astype(np.float32))
                kn[l].copy_(torch.from_numpy(a).cuda()); vn[l].copy_(torch.from_numpy(b).cuda())
            rows.append((a, b))
            outs_g[l].fill_(-7.0)
        g.replay()
        torch.cuda.synchronize()
        step(outs_e)                                      # the same step eagerly (the append rewrites the same rows)
        torch.cuda.synchronize()
        for l in range(layers):
            assert torch.equal(outs_g[l], outs_e[l]), (replay, l)
            oracle.kv_append(ws_[l].k_pool, ws_[l].v_pool, rows[l][0], rows[l][1], w0.block_tables, host_len,
                             block_size=16)
            ref = oracle.paged_decode_attention(ws_[l].q, ws_[l].k_pool, ws_[l].v_pool, w0.block_tables, host_len,
                                                w0.scale, block_size=16)
            assert np.abs(outs_g[l].cpu().numpy().astype(np.float64) - ref).max() <= 2e-3, (replay, l)
