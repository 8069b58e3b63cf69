"""Stored vectors under tests/golden/ (written by tests/golden/write_vectors.py from the oracle
alone; the paper prints no worked numeric example to store instead): the oracle must still
produce them, and the HIP path must agree with them."""
import importlib.util
import os
import zlib

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
spec = importlib.util.spec_from_file_location("write_vectors", os.path.join(HERE, "golden", "write_vectors.py"))
gold = importlib.util.module_from_spec(spec)
spec.loader.exec_module(gold)


def stored_decode():
    rows = [l for l in open(os.path.join(HERE, "golden", "decode_small.txt")) if not l.startswith("#")]
    return np.array([[float.fromhex(x) for x in l.split()] for l in rows]).reshape(3, 2, 128)


def stored_swap():
    kv = dict(l.split() for l in open(os.path.join(HERE, "golden", "swap_small.txt")) if not l.startswith("#"))
    return int(kv["pairs"]), int(kv["staging_bytes"]), int(kv["crc32"], 16), bytes.fromhex(kv["first_32_bytes"])


def test_oracle_still_produces_the_stored_vectors():
    _, out = gold.decode_case()
    assert np.array_equal(out, stored_decode())            # same arithmetic, same order: bit for bit
    sw, _, staging = gold.swap_case()
    pairs, nbytes, crc, head = stored_swap()
    assert (sw.n_blocks, staging.size) == (pairs, nbytes)
    assert zlib.crc32(staging.tobytes()) == crc and staging[:32].tobytes() == head


@pytest.mark.gpu
def test_hip_path_agrees_with_the_stored_vectors():
    import torch
    from helpers import run_hip
    from paper_2602_07878_amd import binding
    w, _ = gold.decode_case()
    got = run_hip(w)
    assert np.abs(got - stored_decode()).max() <= 2e-3      # bf16 inputs, fp32 accumulation
    sw, pool, _ = gold.swap_case()
    pairs, nbytes, crc, head = stored_swap()
    d_pool = torch.from_numpy(pool).cuda()
    d_st = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    desc = binding.swap_desc(sw.num_planes, sw.block_bytes, sw.num_pool_blocks, sw.n_blocks)
    binding.kv_block_swap(desc, d_pool, d_st, torch.from_numpy(sw.gather_mapping).cuda())
    torch.cuda.synchronize()
    st = d_st.cpu().numpy()
    assert zlib.crc32(st.tobytes()) == crc and st[:32].tobytes() == head
