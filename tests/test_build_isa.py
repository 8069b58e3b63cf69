"""What the kernels rely on in the compiled code, checked on the ISA that hipcc emits for gfx950
(no GPU needed): the two attention kernels must not spill (a spill reload waits on the same
counter as the direct-to-LDS fetches in flight and stalls the pipeline on them), and the
cache-policy hints must survive optimisation (the compiler once merged a nontemporal and a plain
store of two branches into one plain store)."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_07878_amd", "csrc")
HIPCC = "/opt/rocm/bin/hipcc"


def isa_of(src):
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only",
               "-o", out, os.path.join(CSRC, src)]
        subprocess.run(cmd, check=True, capture_output=True)
        return open(out).read()


def kernel_metadata(isa):
    """{kernel symbol: {key: int}} from the amdhsa.kernels metadata."""
    meta = {}
    for block in isa.split("  - .agpr_count:")[1:]:
        name = re.search(r"\.name:\s+(\S+)", block).group(1)
        meta[name] = {k: int(v) for k, v in re.findall(r"\.(vgpr_spill_count|sgpr_spill_count|private_segment_fixed_size|vgpr_count):\s+(\d+)", block)}
    return meta


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
@pytest.mark.parametrize("src,kernel,max_vgprs", [("attn_prefill_mfma.hip", "attn_prefill_mfma_d128", 256),
                                                  ("attn_stream_mfma.hip", "attn_stream_mfma_d128", 256)])
def test_attention_kernels_do_not_spill(src, kernel, max_vgprs):
    meta = kernel_metadata(isa_of(src))
    hot = {n: m for n, m in meta.items() if kernel in n}
    assert hot, list(meta)
    for n, m in hot.items():
        # (scalar registers may overflow into lanes of a vector register: that touches no memory)
        assert m["vgpr_spill_count"] == 0 and m["private_segment_fixed_size"] == 0, (n, m)
        assert m["vgpr_count"] <= max_vgprs, (n, m)          # two wavefronts per SIMD


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_cache_policy_hints_survive():
    stream = isa_of("attn_stream_mfma.hip")
    lds_loads = re.findall(r"global_load_lds_dwordx4[^\n]*", stream)
    assert lds_loads and all(" nt" in l for l in lds_loads)              # K/V are read once: streamed past L2
    stores = re.findall(r"global_store_dwordx4[^\n]*", stream)
    assert any(" nt" in l for l in stores) and any(" nt" not in l for l in stores)   # both kinds of partial store
    swap = isa_of("swap.hip")
    loads = re.findall(r"global_load_dwordx4[^\n]*", swap)
    assert loads and all(" nt" in l for l in loads)
