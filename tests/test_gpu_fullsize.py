"""Parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (same descriptors, same workspace handling), against the fp64 oracle."""
import time

import numpy as np
import pytest

import oracle
from paper_2602_07878_amd import workloads as W
from helpers import run_hip, run_oracle, to_device

pytestmark = pytest.mark.gpu


def full_check(w, tol=2e-3, **kw):
    t0 = time.time()
    dev = to_device(w)
    got = run_hip(w, dev, **kw)
    t1 = time.time()
    ref = run_oracle(w)
    t2 = time.time()
    assert np.all(np.isfinite(got))
    err = float(np.abs(got - ref).max())
    print(f"{w.name}: T={w.total_tokens} gpu+upload {t1-t0:.1f}s oracle {t2-t1:.1f}s max_abs_err {err:.3e}",
          flush=True)
    assert err <= tol, err
    return got, dev


def test_config2_full():
    w = W.config2_llama8b()
    got, dev = full_check(w)
    again = run_hip(w, dev)
    assert np.array_equal(got, again)                 # bit-reproducible launch to launch
    vec = run_hip(w, dev, flags=1)                    # the vector-ALU kernel on the same inputs
    assert np.abs(vec - got).max() <= 2e-3
    ref = run_oracle(w)
    planned = run_hip(w, dev, planned=True, calls=2)  # with a per-step plan, as bench.py times it
    assert np.abs(planned - ref).max() <= 2e-3
    assert np.array_equal(planned, run_hip(w, dev, planned=True))


def test_config2_with_8_bit_pools_full():
    """The 8B-shaped batch with an E4M3 KV cache (half the bytes per cached token), as bench.py times it."""
    w = W.config2_llama8b_f8()
    got, dev = full_check(w)
    again = run_hip(w, dev)
    assert np.array_equal(got, again)
    vec = run_hip(w, dev, flags=1)
    assert np.abs(vec - got).max() <= 2e-3
    assert np.array_equal(got, run_hip(w, dev, planned=True))     # same kernel code with a plan: same bits


def test_config3_fill_state_full():
    w = W.config3_fill()
    assert w.notes["occupancy"] >= 0.949
    got, dev = full_check(w)
    assert np.abs(run_hip(w, dev, planned=True) - got).max() <= 1e-5


def test_config5_long_context_full_as_configured_and_auto_split():
    w = W.config5_long70b()
    assert w.partition_tokens == 512
    got, dev = full_check(w)                          # 512-token partials, as configured
    auto = run_hip(w, dev, partition_tokens=0)        # library-chosen split
    assert np.abs(auto - got).max() <= 2e-3
    assert np.abs(run_hip(w, dev, planned=True) - got).max() <= 1e-5


@pytest.mark.parametrize("make", [W.config4_squeeze, W.config4_squeeze_f8], ids=["bf16_32KiB_blocks", "e4m3_16KiB_blocks"])
def test_config4_swap_full_size_round_trip(make):
    import torch
    from paper_2602_07878_amd import binding
    sw = make()
    P, bb, NB, n = sw.num_planes, sw.block_bytes, sw.num_pool_blocks, sw.n_blocks
    t0 = time.time()
    pool = W.random_bytes(sw.pool_bytes, 1004)
    d_pool = torch.from_numpy(pool).cuda()
    d_st = torch.full((sw.staging_bytes,), 0xAB, dtype=torch.uint8, device="cuda:0")
    gm, sm = torch.from_numpy(sw.gather_mapping).cuda(), torch.from_numpy(sw.scatter_mapping).cuda()
    dg = binding.swap_desc(P, bb, NB, n)
    ds = binding.swap_desc(P, bb, n, NB)
    assert binding.validate_mapping(dg, gm) == 0 and binding.validate_mapping(ds, sm) == 0
    binding.kv_block_swap(dg, d_pool, d_st, gm)
    torch.cuda.synchronize()
    t1 = time.time()
    # gather: every byte of the staging buffer against the oracle's memcpy
    ref_st = np.full(sw.staging_bytes, 0xAB, np.uint8)
    oracle.kv_block_swap(pool, ref_st, sw.gather_mapping, num_planes=P, block_bytes=bb)
    got_st = d_st.cpu().numpy()
    assert np.array_equal(got_st, ref_st)
    t2 = time.time()
    # scatter into a poisoned pool: sampled planes compared bytewise, untouched blocks included
    d_pool.fill_(0xCD)
    binding.kv_block_swap(ds, d_st, d_pool, sm)
    torch.cuda.synchronize()
    plane_bytes = NB * bb
    for p in (0, 17, 40, P - 1):
        ref_plane = np.full(plane_bytes, 0xCD, np.uint8)
        oracle.kv_block_swap(ref_st[p * n * bb:(p + 1) * n * bb], ref_plane, sw.scatter_mapping,
                             num_planes=1, block_bytes=bb)
        got_plane = d_pool[p * plane_bytes:(p + 1) * plane_bytes].cpu().numpy()
        assert np.array_equal(got_plane, ref_plane)
        # round trip: the victims' blocks are where the new mapping says, bit for bit
        a = got_plane.reshape(NB, bb)[sw.new_blocks]
        b = pool[p * plane_bytes:(p + 1) * plane_bytes].reshape(NB, bb)[sw.src_blocks]
        assert np.array_equal(a, b)
    print(f"swap {sw.name}: payload {sw.payload_bytes/1e9:.1f} GB setup+gather {t1-t0:.1f}s "
          f"gather check {t2-t1:.1f}s scatter check {time.time()-t2:.1f}s", flush=True)
