"""Host-sanitizer leg (CPU only): the C oracle, the scheduler model and the library's host-side
checks rebuilt with AddressSanitizer + UndefinedBehaviorSanitizer on the host code and run as
stand-alone programs (tests/sanitize/*), on buffers of exactly the stated sizes.  Their results
must equal those of the regular builds (oracle library, scheduler reference, regular libpkv), and
the sanitizers must stay silent.  The sanitizer runtime is linked into each program, nothing is
preloaded."""
import ctypes
import glob
import os
import subprocess

import numpy as np
import pytest

import oracle
from oracle.sched_ref import RefScheduler, SWAP, RECOMPUTE
from paper_2602_07878_amd import binding, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
FLAGS = ["-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:exitcode=97", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, env=ENV, **kw)
    assert r.returncode == 0, (cmd, r.returncode, r.stderr.decode()[-3000:])
    assert b"runtime error" not in r.stderr and b"AddressSanitizer" not in r.stderr, r.stderr.decode()[-3000:]
    return r.stdout


@pytest.fixture(scope="module")
def oracle_exe(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_driver")
    subprocess.check_call(["gcc", "-std=c11", "-ffp-contract=off", "-Wall", "-Wextra", "-static-libasan"] + FLAGS +
                          [os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "pkv_oracle.c"),
                           "-o", exe, "-lm"])
    return exe


def write_case(path, header, arrays):
    h = np.zeros(24, np.int64)
    h[:len(header)] = header
    with open(path, "wb") as f:
        f.write(h.tobytes())
        for a in arrays:
            b = np.ascontiguousarray(a).tobytes()
            f.write(np.int64(len(b)).tobytes())
            f.write(b)


def read_arrays(path):
    out, raw, pos = [], open(path, "rb").read(), 0
    while pos < len(raw):
        n = int(np.frombuffer(raw, np.int64, 1, pos)[0])
        out.append(raw[pos + 8:pos + 8 + n])
        pos += 8 + n
    return out


@pytest.mark.parametrize("name", ["tiny_f32", "ragged_bf16_gqa", "token_major"])
def test_oracle_attention_under_sanitizers(oracle_exe, tmp_path, name):
    if name == "tiny_f32":
        w = W.config1_tiny()
    elif name == "ragged_bf16_gqa":
        w = W.make_attn_workload(name, 71, dtype="bf16", Hq=8, Hkv=2, D=128, block_size=16,
                                 context_lens=[1, 15, 16, 17, 0, 300, 33], pool_factor=1.0)
    else:
        w = W.make_attn_workload(name, 72, dtype="bf16", Hq=4, Hkv=4, D=64, block_size=32,
                                 context_lens=[64, 5, 97], pool_factor=1.0)
    nblk, Hkv, bs, D = w.k_pool.shape
    ks = (Hkv * bs * D, bs * D, D)
    kp, vp = w.k_pool, w.v_pool
    if name == "token_major":          # same values stored [blocks][bs][Hkv][D]
        kp = np.ascontiguousarray(w.k_pool.transpose(0, 2, 1, 3))
        vp = np.ascontiguousarray(w.v_pool.transpose(0, 2, 1, 3))
        ks = (bs * Hkv * D, D, Hkv * D)
    scale_bits = int(np.float32(w.scale).view(np.uint32))
    header = [0, w.B, w.Hq, Hkv, D, bs, nblk, w.block_tables.shape[1], 1 if w.dtype == "bf16" else 0,
              *ks, *ks, scale_bits]
    write_case(tmp_path / "c.bin", header, [w.q, kp, vp, w.block_tables, w.context_lens])
    run([oracle_exe, str(tmp_path / "c.bin"), str(tmp_path / "r.bin")])
    got, rc = read_arrays(tmp_path / "r.bin")
    assert np.frombuffer(rc, np.int64)[0] == 0
    ref = oracle.paged_decode_attention(w.q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, w.scale,
                                        block_size=bs)
    # same arithmetic, same order: bit-equal (both builds keep fp contraction off)
    assert np.array_equal(np.frombuffer(got, np.float64).reshape(ref.shape), ref)


def test_oracle_swap_and_append_under_sanitizers(oracle_exe, tmp_path):
    sw = W.make_swap_workload("san", 5, victim_lens=(100, 40, 17), num_planes=3, block_bytes=256)
    pool = W.random_bytes(sw.pool_bytes, 6)
    st = np.zeros(sw.staging_bytes, np.uint8)
    write_case(tmp_path / "s.bin", [1, 3, 256, sw.num_pool_blocks * 256, sw.n_blocks * 256, sw.num_pool_blocks,
                                    sw.n_blocks, sw.n_blocks], [pool, st, sw.gather_mapping])
    run([oracle_exe, str(tmp_path / "s.bin"), str(tmp_path / "sr.bin")])
    got, rc = read_arrays(tmp_path / "sr.bin")
    ref = st.copy()
    oracle.kv_block_swap(pool, ref, sw.gather_mapping, num_planes=3, block_bytes=256)
    assert np.frombuffer(rc, np.int64)[0] == 0 and np.array_equal(np.frombuffer(got, np.uint8), ref)
    # a mapping entry outside its plane is reported, nothing past the buffers is touched
    bad = sw.gather_mapping.copy()
    bad[-1, 0] = sw.num_pool_blocks
    write_case(tmp_path / "s2.bin", [1, 3, 256, sw.num_pool_blocks * 256, sw.n_blocks * 256, sw.num_pool_blocks,
                                     sw.n_blocks, sw.n_blocks], [pool, st, bad])
    run([oracle_exe, str(tmp_path / "s2.bin"), str(tmp_path / "sr2.bin")])
    assert np.frombuffer(read_arrays(tmp_path / "sr2.bin")[1], np.int64)[0] != 0

    w = W.make_attn_workload("san_append", 73, dtype="bf16", Hq=4, Hkv=2, D=64, block_size=16,
                             context_lens=[1, 16, 17, 0, 48], pool_factor=1.0)
    rng = np.random.default_rng(9)
    kn = W.f32_to_bf16_bits(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
    vn = W.f32_to_bf16_bits(rng.standard_normal((w.B, w.Hkv, w.D)).astype(np.float32))
    nblk, Hkv, bs, D = w.k_pool.shape
    ks = (Hkv * bs * D, bs * D, D)
    write_case(tmp_path / "a.bin", [2, w.B, Hkv, D, bs, nblk, w.block_tables.shape[1], 2, *ks, *ks],
               [kn, vn, w.k_pool, w.v_pool, w.block_tables, w.context_lens])
    run([oracle_exe, str(tmp_path / "a.bin"), str(tmp_path / "ar.bin")])
    gk, gv, rc = read_arrays(tmp_path / "ar.bin")
    rk, rv = w.k_pool.copy(), w.v_pool.copy()
    oracle.kv_append(rk, rv, kn, vn, w.block_tables, w.context_lens, block_size=bs)
    assert np.frombuffer(rc, np.int64)[0] == 0
    assert np.array_equal(np.frombuffer(gk, np.uint16), rk.reshape(-1))
    assert np.array_equal(np.frombuffer(gv, np.uint16), rv.reshape(-1))


def ref_line(o, chunked):
    dec = " ".join(f"{rid}:{n}:{','.join(map(str, blocks))}" for rid, n, blocks in o["decode"])
    so = " ".join(f"{a}>{b}" for a, b in o["swap_out"])
    si = " ".join(f"{a}>{b}" for a, b in o["swap_in"])
    pf = " ".join(f"{p[0]}:{p[1]}:{p[2] if chunked else p[1]}" for p in o["prefill"])
    fin = " ".join(str(r) for r in o["finished"])
    join = lambda tag, body: tag + (" " + body if body else "")
    return " ".join([join("D", dec), join("O", so), join("I", si), join("P", pf), join("F", fin),
                     f"S {o['free_blocks']} {o['running']} {o['waiting']} {o['swapped']} "
                     f"{int(o['head_blocked'])} {len(o['preempted'])}"])


@pytest.mark.parametrize("mode,chunked,budget,cpu", [(SWAP, 0, 1024, 6), (RECOMPUTE, 0, 300, 0), (SWAP, 1, 64, 64),
                                                     (RECOMPUTE, 1, 96, 0)])
def test_scheduler_model_under_sanitizers(tmp_path, mode, chunked, budget, cpu):
    exe = str(tmp_path / "sched_driver")
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-static-libasan"] + FLAGS +
                          ["-I", os.path.join(ROOT, "include"), os.path.join(SAN, "sched_driver.cpp"),
                           os.path.join(ROOT, "paper_2602_07878_amd", "csrc", "sched.cpp"), "-o", exe])
    kw = dict(num_gpu_blocks=64, num_cpu_blocks=cpu, block_size=16, max_num_seqs=12, max_num_batched_tokens=budget,
              max_blocks_per_seq=40, watermark_blocks=1)
    stream = W.poisson_request_stream(40 + budget, 250, 0.3, prompt_median=110, out_median=100, max_prompt=300,
                                      max_new=200)
    stream += [[(10**6, 5000, 5), (10**6 + 1, 10, 0)]]      # refused: cannot ever fit / no output
    stream += [[] for _ in range(1500)]
    with open(tmp_path / "in.txt", "w") as f:
        f.write(f"{kw['num_gpu_blocks']} {cpu} 16 12 {budget} 40 1 {mode} {chunked} {len(stream)}\n")
        for arrivals in stream:
            f.write(" ".join([str(len(arrivals))] + [f"{a} {b} {c}" for a, b, c in arrivals]) + "\n")
    got = run([exe, str(tmp_path / "in.txt")]).decode().splitlines()
    r = RefScheduler(mode=mode, chunked=bool(chunked), **kw)
    for it, arrivals in enumerate(stream):
        marks = []
        for rid, p, n in arrivals:
            try:
                r.add_request(rid, p, n)
                marks.append("A0")
            except ValueError:
                marks.append("A2")
        line = " ".join(marks + [ref_line(r.step(), chunked)])
        assert got[it] == line, (it, got[it], line)
    assert got[len(stream)] == "T " + " ".join(str(v) for v in r.totals.values())
    assert r.totals["preemptions"] > 0


def test_library_host_checks_under_sanitizers(tmp_path):
    """api.hip's validators and pre-launch checks in a build whose host code is instrumented."""
    exe = str(tmp_path / "abi_driver")
    csrc = os.path.join(ROOT, "paper_2602_07878_amd", "csrc")
    srcs = sorted(glob.glob(os.path.join(csrc, "*.hip")) + glob.glob(os.path.join(csrc, "*.cpp")))
    cmd = ["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-static-libsan",
           "-I", os.path.join(ROOT, "include"), "-I", csrc, os.path.join(SAN, "abi_driver.cpp")] + srcs + ["-o", exe]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-3000:]
    got = run([exe]).decode().split()
    L = binding.lib()
    want = ["0", "6", "6", "6", "1", "2",        # tables
            "0", "6", "6", "6", "0", "4",        # mappings
            "0", "6", "6", "6",                  # chunk arrays
            "5", "1", "4", "5", "PKV_ERR_INDEX"]
    assert got == want, got
    assert L.pkv_status_string(6).decode() == "PKV_ERR_INDEX"
