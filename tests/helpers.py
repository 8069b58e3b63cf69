"""Test-side glue: move a host workload to the GPU, call the HIP path through
the C ABI binding, bring results back.  No arithmetic of the method here."""
import numpy as np


def to_device(w, device="cuda:0"):
    import torch
    def conv(a):     # uint16 = bf16 bits, uint8 = E4M3 codes (passed as they are), else float32
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
        return torch.from_numpy(a).to(device)
    return dict(q=conv(w.q), k_pool=conv(w.k_pool), v_pool=conv(w.v_pool),
                block_tables=torch.from_numpy(w.block_tables).to(device),
                context_lens=torch.from_numpy(w.context_lens).to(device))


def run_hip(w, dev=None, *, partition_tokens=None, out_dtype=None, max_context_len=None,
            canary=True, flags=0, planned=False, calls=1):
    """Returns float64 numpy [B,Hq,D] from the HIP library (and checks canaries round `out`).
    planned: through pkv_attn_plan + paged_decode_attention_planned, `calls` calls on one plan."""
    import torch
    from paper_2602_07878_amd import binding
    dev = dev or to_device(w)
    odt = out_dtype or torch.float32
    n = w.B * w.Hq * w.D
    pad = 64
    buf = torch.full((n + 2 * pad,), 12345.0, dtype=odt, device=dev["q"].device)
    out = buf[pad:pad + n].view(w.B, w.Hq, w.D)
    pt = w.partition_tokens if partition_tokens is None else partition_tokens
    mcl = w.max_context_len if max_context_len is None else max_context_len
    if planned:
        desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"], max_context_len=mcl,
                                     partition_tokens=pt, out_dtype=odt, flags=flags, k_scale=w.k_scale,
                                     v_scale=w.v_scale)
        plan = binding.attn_plan(desc, dev["block_tables"], dev["context_lens"])
        ws = None
        for _ in range(calls):
            ws = binding.paged_decode_attention_planned(desc, plan, dev["q"], dev["k_pool"], dev["v_pool"],
                                                        dev["block_tables"], dev["context_lens"], w.scale, out,
                                                        workspace=ws)
    else:
        binding.paged_decode_attention(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                       dev["context_lens"], w.scale, out, max_context_len=mcl,
                                       partition_tokens=pt, flags=flags, k_scale=w.k_scale, v_scale=w.v_scale)
    torch.cuda.synchronize()
    if canary:
        assert torch.all(buf[:pad] == 12345.0) and torch.all(buf[pad + n:] == 12345.0)
    return out.float().cpu().numpy().astype(np.float64)


def run_oracle(w):
    import oracle
    return oracle.paged_decode_attention(w.q, w.k_pool, w.v_pool, w.block_tables,
                                         w.context_lens, w.scale, block_size=w.block_size,
                                         k_scale=w.k_scale, v_scale=w.v_scale)
