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
                                                  ("attn_stream_mfma.hip", "attn_stream_mfma_d128", 256),
                                                  ("attn_stream_flat.hip", "attn_stream_flat_", 256)])
def test_attention_kernels_do_not_spill(src, kernel, max_vgprs):
    meta = kernel_metadata(isa_of(src))
    hot = {n: m for n, m in meta.items() if kernel in n}
    assert hot, list(meta)
    for n, m in hot.items():
        # (scalar registers may overflow into lanes of a vector register: that touches no memory)
        assert m["vgpr_spill_count"] == 0 and m["private_segment_fixed_size"] == 0, (n, m)
        assert m["vgpr_count"] <= max_vgprs, (n, m)          # two wavefronts per SIMD


def registers_named(line):
    """Vector register numbers an instruction line names (v7, v[8:11])."""
    regs = set()
    for m in re.finditer(r"\bv(\d+)\b", line):
        regs.add(int(m.group(1)))
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", line):
        regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    return regs


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_registers_that_wait_for_data_in_flight_are_left_alone():
    """The flat streaming kernels leave loads in flight across several tiles, into registers the
    compiler must not touch (it may move a value it manages at any join of control flow, and a
    register moved while its load is in flight takes the old contents along): v174 and up in the
    8-bit kernels (v170 and up in those that take a plan), v234 and up in the bf16 kernels.  Only the kernels' own statements (between
    the compiler's inline-assembly markers) may name them, and the loads that stay in flight must
    target exactly them."""
    isa = isa_of("attn_stream_flat.hip")
    bodies = re.findall(r"^(_ZN\S*attn_stream_flat_(f8_planned|f8|bf16)_d128\S*):[^\n]*\n(.*?)s_endpgm", isa, re.S | re.M)
    assert len(bodies) == 12
    for name, kind, body in bodies:
        first = {"f8": 174, "f8_planned": 170, "bf16": 234}[kind]
        in_asm = False
        for line in body.splitlines():
            if "#ASMSTART" in line:
                in_asm = True
            elif "#ASMEND" in line:
                in_asm = False
            text = line.split(";")[0]
            high = {r for r in registers_named(text) if r >= first}
            if not in_asm:
                assert not high, (name, line)
            elif re.search(r"global_load_dwordx4 v\[\d+:\d+\], v\d+, s\[", text):
                dest = re.search(r"global_load_dwordx4 (v\[\d+:\d+\]),", text).group(1)
                assert min(registers_named(dest)) >= first, (name, line)     # tile bytes
            elif re.search(r"global_load_dwordx4 v\[\d+:\d+\], v\[\d+:\d+\], off", text):
                dest = min(registers_named(re.search(r"global_load_dwordx4 (v\[\d+:\d+\]),", text).group(1)))
                assert dest >= first or "s_waitcnt vmcnt(0)" in body[body.index(line):body.index(line) + 400], (name, line)


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_cache_policy_hints_survive():
    flat = isa_of("attn_stream_flat.hip")
    # tiles are streamed past L2; a plan's descriptors are not (every layer call reads them again)
    lds_loads = re.findall(r"global_load_lds_dwordx4[^\n]*", flat)
    assert sum(" nt" in l for l in lds_loads) >= 4 * 16 and any(" nt" not in l for l in lds_loads)
    raw_loads = re.findall(r"global_load_dwordx4 v\[(?:1[7-9]\d|2[0-3]\d):\d+\], v\d+, s\[[^\n]*", flat)   # into v170..v239
    assert len(raw_loads) >= 8 * 32 and all(" nt" in l for l in raw_loads)
    stream = isa_of("attn_stream_mfma.hip")
    lds_loads = re.findall(r"global_load_lds_dwordx4[^\n]*", stream)
    assert lds_loads and all(" nt" in l for l in lds_loads)              # K/V are read once: streamed past L2
    stores = re.findall(r"global_store_dwordx4[^\n]*", stream)
    assert any(" nt" in l for l in stores) and any(" nt" not in l for l in stores)   # both kinds of partial store
    swap = isa_of("swap.hip")
    loads = re.findall(r"global_load_dwordx4[^\n]*", swap)
    assert loads and all(" nt" in l for l in loads)
