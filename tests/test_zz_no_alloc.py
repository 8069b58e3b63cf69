"""paged_decode_attention_static (the entry point for callers that cannot allocate) against
paged_decode_attention with a caller workspace: same kernels, so the outputs must agree bit for
bit, and both within the bf16 tolerance of the oracle; two calls in a row, the second with a
smaller input, so that the second call meets the first call's leftovers in the shared array."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_07878_amd import binding, workloads as W
from helpers import run_hip, run_oracle, to_device

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-3   # max abs error, bf16 inputs with fp32 accumulation


def run_static(w, dev, partition_tokens=0):
    n = w.B * w.Hq * w.D
    pad = 64
    buf = torch.full((n + 2 * pad,), 12345.0, dtype=torch.float32, device=dev["q"].device)
    out = buf[pad:pad + n].view(w.B, w.Hq, w.D)
    binding.paged_decode_attention_static(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                          dev["context_lens"], w.scale, out,
                                          max_context_len=w.max_context_len,
                                          partition_tokens=partition_tokens)
    torch.cuda.synchronize()
    assert torch.all(buf[:pad] == 12345.0) and torch.all(buf[pad + n:] == 12345.0)
    return out.cpu().numpy().astype(np.float64)


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    binding.init()
    assert binding.lib().pkv_static_scratch_bytes() == 16 << 20
    # first a batch whose partials fill a good part of the array, then a smaller one with other
    # lengths: its partials land on slots the first call used
    big = W.config2_llama8b(B=24, seed=2101)
    small = W.config2_llama8b(B=5, seed=2102)
    for w in (big, small):
        print(f"static scratch case {w.name} B={w.B}", flush=True)
        dev = to_device(w)
        got = run_static(w, dev)
        want = run_hip(w, dev, partition_tokens=0)
        assert np.array_equal(got, want)
        assert np.isfinite(got).all()
        assert np.abs(got - run_oracle(w)).max() <= TOL_BF16


def test_static_scratch_with_capped_partials_and_fp32_path():
    # a caller-set cap (many partials per pair: the other merge kernel), then the fp32 / vector-ALU
    # kernels whose partials use another layout of the same array
    w = W.config2_llama8b(B=6, seed=2103)
    dev = to_device(w)
    got = run_static(w, dev, partition_tokens=128)
    assert np.array_equal(got, run_hip(w, dev, partition_tokens=128))
    assert np.abs(got - run_oracle(w)).max() <= TOL_BF16
    t = W.config1_tiny()
    devt = to_device(t)
    gt = run_static(t, devt, partition_tokens=64)
    assert np.array_equal(gt, run_hip(t, devt, partition_tokens=64))
    assert np.abs(gt - run_oracle(t)).max() <= 1e-5


def test_static_scratch_rejects_sizes_beyond_the_array():
    # long contexts with a small cap need more partial slots than 16 MiB hold: refused on the host
    w = W.config2_llama8b(B=4, seed=2104)
    dev = to_device(w)
    desc = binding.attn_desc_for(dev["q"], dev["k_pool"], dev["v_pool"], dev["block_tables"],
                                 max_context_len=1 << 20, partition_tokens=64)
    desc.max_blocks_per_seq = (1 << 20) // 16   # never dereferenced: the call must not launch
    assert binding.attn_workspace_bytes(desc) > (16 << 20)
    out = torch.zeros((w.B, w.Hq, w.D), dtype=torch.float32, device="cuda:0")
    st = binding.lib().paged_decode_attention_static(
        ctypes.byref(desc), dev["q"].data_ptr(), dev["k_pool"].data_ptr(), dev["v_pool"].data_ptr(),
        dev["block_tables"].data_ptr(), dev["context_lens"].data_ptr(), float(w.scale), out.data_ptr(), None)
    assert binding.status_string(st) == "PKV_ERR_WORKSPACE"
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
