"""Writes the stored vectors of this folder.  Calls only oracle/ and the seeded input generators.

The paper (arXiv 2602.07878) prints no worked numeric example of the operations built here, so
there is no published value to store.  What is stored instead are outputs of the fp64 oracle on
small seeded cases: they pin the oracle against silent drift (tests/test_golden.py recomputes
them) and give the GPU tests a reference that does not depend on the oracle being rebuilt.  The
oracle itself is pinned to mathematics in tests/test_oracle_pins.py.

    python tests/golden/write_vectors.py        # rewrites decode_small.txt and swap_small.txt
"""
import os
import sys
import zlib

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2602_07878_amd import workloads as W  # noqa: E402

DECODE = dict(name="golden_decode", seed=4242, dtype="bf16", Hq=2, Hkv=1, D=128, block_size=16,
              context_lens=(1, 17, 40))
SWAP = dict(name="golden_swap", seed=4343, victim_lens=(33, 5, 70), num_planes=3, block_bytes=256)


def decode_case():
    w = W.make_attn_workload(DECODE["name"], DECODE["seed"], **{k: v for k, v in DECODE.items() if k not in ("name", "seed")})
    out = oracle.paged_decode_attention(w.q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, w.scale,
                                        block_size=w.block_size)
    return w, out


def swap_case():
    sw = W.make_swap_workload(SWAP["name"], SWAP["seed"], victim_lens=SWAP["victim_lens"], num_planes=SWAP["num_planes"],
                              block_bytes=SWAP["block_bytes"])
    pool = W.random_bytes(sw.pool_bytes, SWAP["seed"] + 1)
    staging = np.zeros(sw.num_planes * sw.n_blocks * sw.block_bytes, np.uint8)
    oracle.kv_block_swap(pool, staging, sw.gather_mapping, num_planes=sw.num_planes, block_bytes=sw.block_bytes)
    return sw, pool, staging


def main():
    w, out = decode_case()
    with open(os.path.join(HERE, "decode_small.txt"), "w") as f:
        f.write("# fp64 oracle output of paged decode attention (Sec. 2.2 / 4.2 of arXiv 2602.07878), written by write_vectors.py\n")
        f.write(f"# case: {DECODE}\n# shape: {out.shape} (sequence, query head, dim), one row per line, C hexadecimal floats\n")
        for row in out.reshape(-1, out.shape[-1]):
            f.write(" ".join(float(x).hex() for x in row) + "\n")
    sw, pool, staging = swap_case()
    with open(os.path.join(HERE, "swap_small.txt"), "w") as f:
        f.write("# oracle result of the KV-block gather of the swap path (Sec. 5.1.2), written by write_vectors.py\n")
        f.write(f"# case: {SWAP}; pool bytes seeded with {SWAP['seed'] + 1}\n")
        f.write(f"pairs {sw.n_blocks}\nstaging_bytes {staging.size}\ncrc32 {zlib.crc32(staging.tobytes()):08x}\n")
        f.write("first_32_bytes " + staging[:32].tobytes().hex() + "\n")


if __name__ == "__main__":
    main()
