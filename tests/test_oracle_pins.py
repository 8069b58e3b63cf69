"""Pins of the fp64 CPU oracle against facts that do not come from the oracle:
closed forms, invariants, a library routine, exact-rational brute force.
The paper (arXiv 2602.07878) prints no worked attention example, so there is
no golden value to quote; every pin below is mathematics or a library special
case.  Each is chosen so that a plausible slip in the oracle (wrong GQA map,
wrong slot index, missing scale, max not subtracted, K/V swapped, transposed
table) fails at least one of them."""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2602_07878_amd import workloads as W


def f32(x):
    return np.asarray(x, dtype=np.float32)


def gather_rows(pool, table_row, n, g, bs):
    """Test-local gather (not the oracle's): rows of logical tokens 0..n-1."""
    rows = []
    for t in range(n):
        rows.append(pool[table_row[t // bs], g, t % bs])
    return np.stack(rows) if rows else np.zeros((0, pool.shape[-1]), pool.dtype)


def as_f64(a):
    return W.bf16_bits_to_f32(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)


def small(seed, dtype="f32", Hq=4, Hkv=2, D=8, bs=4, lens=(1, 5, 9, 16), **kw):
    return W.make_attn_workload("t", seed, dtype=dtype, Hq=Hq, Hkv=Hkv, D=D, block_size=bs,
                                context_lens=lens, **kw)


def run(w, **kw):
    return oracle.paged_decode_attention(w.q, w.k_pool, w.v_pool, w.block_tables,
                                         w.context_lens, w.scale, block_size=w.block_size, **kw)


# P1 ------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_token_context_returns_that_v_row(dtype):
    w = small(1, dtype=dtype, Hq=6, Hkv=3, lens=(1, 1, 1))
    out = run(w)
    G = w.Hq // w.Hkv
    for i in range(w.B):
        for h in range(w.Hq):
            v0 = as_f64(w.v_pool[w.block_tables[i, 0], h // G, 0])
            assert np.array_equal(out[i, h], v0)


# P2 ------------------------------------------------------------------------
@pytest.mark.parametrize("how", ["same_keys", "zero_q", "zero_scale"])
def test_uniform_scores_give_mean_of_v(how):
    w = small(2, lens=(3, 7, 13, 16), poison=True)
    if how == "same_keys":
        row = f32(np.linspace(-1, 1, w.D))
        finite = ~np.isnan(w.k_pool)
        w.k_pool[finite] = np.broadcast_to(row, w.k_pool.shape)[finite]
    elif how == "zero_q":
        w.q[:] = 0
    else:
        w.scale = 0.0
    out = run(w)
    G = w.Hq // w.Hkv
    for i in range(w.B):
        n = int(w.context_lens[i])
        for h in range(w.Hq):
            v = gather_rows(w.v_pool, w.block_tables[i], n, h // G, w.block_size).astype(np.float64)
            np.testing.assert_allclose(out[i, h], v.mean(axis=0), rtol=0, atol=1e-14)


# P3 ------------------------------------------------------------------------
def test_physical_block_placement_is_irrelevant_bitwise():
    w = small(3, Hq=4, Hkv=2, lens=(2, 6, 11, 16), pool_factor=1.5)
    base = run(w)
    rng = np.random.default_rng(33)
    perm = rng.permutation(w.num_pool_blocks)          # old block b moves to perm[b]
    k2 = np.empty_like(w.k_pool)
    v2 = np.empty_like(w.v_pool)
    k2[perm] = w.k_pool
    v2[perm] = w.v_pool
    bt2 = np.where(w.block_tables >= 0, perm[np.maximum(w.block_tables, 0)], -1).astype(np.int32)
    out2 = oracle.paged_decode_attention(w.q, k2, v2, bt2, w.context_lens, w.scale,
                                         block_size=w.block_size)
    assert np.array_equal(base, out2)


# P4 ------------------------------------------------------------------------
def test_logical_token_order_is_irrelevant():
    bs, D, n = 4, 8, 14
    w = small(4, Hq=2, Hkv=1, D=D, bs=bs, lens=(n,), num_pool_blocks=4, poison=False)
    w.block_tables[0, :4] = [0, 1, 2, 3]
    base = run(w)
    rng = np.random.default_rng(5)
    p = rng.permutation(n)
    k2, v2 = w.k_pool.copy(), w.v_pool.copy()
    kflat = w.k_pool.transpose(1, 0, 2, 3).reshape(1, 16, D)
    vflat = w.v_pool.transpose(1, 0, 2, 3).reshape(1, 16, D)
    kf2, vf2 = kflat.copy(), vflat.copy()
    kf2[0, :n] = kflat[0, p]
    vf2[0, :n] = vflat[0, p]
    k2 = kf2.reshape(1, 4, bs, D).transpose(1, 0, 2, 3).copy()
    v2 = vf2.reshape(1, 4, bs, D).transpose(1, 0, 2, 3).copy()
    out2 = oracle.paged_decode_attention(w.q, k2, v2, w.block_tables, w.context_lens, w.scale,
                                         block_size=bs)
    np.testing.assert_allclose(out2, base, rtol=0, atol=1e-13)
    assert not np.array_equal(k2, w.k_pool)


# P5 ------------------------------------------------------------------------
def test_weights_sum_to_one_and_output_in_convex_hull():
    w = small(5, dtype="bf16", Hq=8, Hkv=2, D=16, bs=16, lens=(17, 64, 100, 256))
    out, wts = run(w, return_weights=True)
    G = w.Hq // w.Hkv
    for i in range(w.B):
        n = int(w.context_lens[i])
        s = wts[i, :, :n].sum(axis=1)
        np.testing.assert_allclose(s, 1.0, rtol=0, atol=1e-15 * n)
        assert np.all(wts[i, :, :n] >= 0) and np.all(wts[i, :, n:] == 0)
        for h in range(w.Hq):
            v = as_f64(gather_rows(w.v_pool, w.block_tables[i], n, h // G, w.block_size))
            assert np.all(out[i, h] <= v.max(axis=0) + 1e-12)
            assert np.all(out[i, h] >= v.min(axis=0) - 1e-12)


# P6 ------------------------------------------------------------------------
def test_adding_a_constant_vector_to_all_keys_changes_nothing():
    # exact in fp32 inputs: keys and shift are small integers / 8
    rng = np.random.default_rng(6)
    w = small(6, Hq=2, Hkv=2, D=8, bs=4, lens=(9, 16), poison=False)
    w.k_pool[:] = rng.integers(-16, 17, size=w.k_pool.shape).astype(np.float32) / 8
    w.q[:] = rng.integers(-8, 9, size=w.q.shape).astype(np.float32) / 4
    w.scale = 0.5
    base = run(w)
    c = f32(rng.integers(200, 400, size=w.D))           # shifts scores by up to ~1e4:
    w.k_pool += c                                       # naive exp() without max would overflow
    shifted = run(w)
    assert np.all(np.isfinite(shifted))
    np.testing.assert_allclose(shifted, base, rtol=0, atol=1e-12)


# P7 ------------------------------------------------------------------------
@pytest.mark.parametrize("target", [0, 6, 12])
def test_one_hot_limit(target):
    # the planted score is ~1e3: any position whose score escaped the max
    # subtraction (first, middle, last) would overflow exp()
    w = small(7, Hq=2, Hkv=1, D=8, bs=4, lens=(13,), poison=False)
    blk, slot = w.block_tables[0, target // 4], target % 4
    qh = w.q[0, 0].astype(np.float64)
    w.q[0, 1] = w.q[0, 0]
    beta = 400.0
    w.k_pool[blk, 0, slot] = f32(beta * qh / np.linalg.norm(qh))
    w.scale = 1.0
    out = run(w)
    # gap between the planted score and any other is > beta*|q| - |q|*max|k| >> 50
    v = w.v_pool[blk, 0, slot].astype(np.float64)
    np.testing.assert_allclose(out[0, 0], v, rtol=0, atol=13 * math.exp(-50) + 1e-15)
    np.testing.assert_allclose(out[0, 1], v, rtol=0, atol=13 * math.exp(-50) + 1e-15)


# P8 ------------------------------------------------------------------------
def test_gqa_equals_mha_on_replicated_kv_heads():
    w = small(8, dtype="bf16", Hq=8, Hkv=2, D=16, bs=4, lens=(3, 10, 16, 7))
    G = 4
    out = run(w)
    k_rep = np.repeat(w.k_pool, G, axis=1)
    v_rep = np.repeat(w.v_pool, G, axis=1)
    out_mha = oracle.paged_decode_attention(w.q, k_rep, v_rep, w.block_tables, w.context_lens,
                                            w.scale, block_size=w.block_size)
    assert np.array_equal(out, out_mha)
    # identical queries inside a group -> identical rows; across groups -> different
    w.q[:, 1] = w.q[:, 0]
    w.q[:, 4] = w.q[:, 0]
    out2 = run(w)
    assert np.array_equal(out2[:, 0], out2[:, 1])
    assert not np.array_equal(out2[:, 0], out2[:, 4])


# P9 ------------------------------------------------------------------------
def test_split_merge_algebra_reproduces_unsplit_result():
    """(m, l, O) of disjoint token ranges merged by log-sum-exp equal the whole."""
    bs, D = 4, 8
    n = 29
    w = small(9, Hq=2, Hkv=1, D=D, bs=bs, lens=(n,), poison=False)
    whole = run(w)[0]
    cuts = [0, 4, 12, 20, 29]             # block-aligned partitions
    parts = []
    for a, b in zip(cuts[:-1], cuts[1:]):
        # a sub-context is expressed with a shifted table and its own length
        bt = w.block_tables[:, a // bs:(b + bs - 1) // bs].copy()
        out_p, wts = oracle.paged_decode_attention(
            w.q, w.k_pool, w.v_pool, bt, np.array([b - a], np.int32), w.scale,
            block_size=bs, return_weights=True)
        # recover (m, l) of the part from the test's own score computation
        for_h = []
        for h in range(2):
            k = gather_rows(w.k_pool, bt[0], b - a, 0, bs).astype(np.float64)
            s = float(np.float32(w.scale)) * (k @ w.q[0, h].astype(np.float64))
            m = s.max()
            l = np.exp(s - m).sum()
            for_h.append((m, l, out_p[0, h] * l))
        parts.append(for_h)
    for h in range(2):
        M = max(p[h][0] for p in parts)
        L = sum(p[h][1] * math.exp(p[h][0] - M) for p in parts)
        O = sum(p[h][2] * math.exp(p[h][0] - M) for p in parts)
        np.testing.assert_allclose(O / L, whole[h], rtol=0, atol=1e-13)


# P10 -----------------------------------------------------------------------
@pytest.mark.parametrize("dtype,Hq,Hkv,D,bs", [("f32", 8, 8, 64, 16), ("bf16", 8, 2, 32, 16),
                                                ("bf16", 16, 2, 128, 16)])
def test_matches_library_sdpa_in_fp64(dtype, Hq, Hkv, D, bs):
    import torch
    import torch.nn.functional as F
    w = W.make_attn_workload("t", 10, dtype=dtype, Hq=Hq, Hkv=Hkv, D=D, block_size=bs,
                             context_lens=(17, 64, 100, 256), num_pool_blocks=64)
    out = run(w)
    G = Hq // Hkv
    for i in range(w.B):
        n = int(w.context_lens[i])
        k = np.stack([as_f64(gather_rows(w.k_pool, w.block_tables[i], n, g, bs)) for g in range(Hkv)])
        v = np.stack([as_f64(gather_rows(w.v_pool, w.block_tables[i], n, g, bs)) for g in range(Hkv)])
        kt = torch.from_numpy(k).repeat_interleave(G, dim=0)[None]       # [1,Hq,n,D]
        vt = torch.from_numpy(v).repeat_interleave(G, dim=0)[None]
        qt = torch.from_numpy(as_f64(w.q[i]))[None, :, None, :]          # [1,Hq,1,D]
        ref = F.scaled_dot_product_attention(qt, kt, vt, attn_mask=None, dropout_p=0.0,
                                             is_causal=False, scale=float(np.float32(w.scale)))
        np.testing.assert_allclose(out[i], ref[0, :, 0].numpy(), rtol=0, atol=1e-12)


# P11 -----------------------------------------------------------------------
def test_brute_force_exact_rationals_tiny():
    """Scores chosen as exact multiples of ln 2 so that exp() is an exact power
    of two and the whole softmax can be written with Fractions."""
    bs, D = 2, 4
    lens = (5, 3)
    w = small(11, Hq=2, Hkv=1, D=D, bs=bs, lens=lens, poison=True)
    rng = np.random.default_rng(11)
    # q = e_0 * 1 (head 0), e_1 * 2 (head 1); K integer entries; scale = ln2 rounded to fp32
    w.q[:] = 0
    w.q[:, 0, 0] = 1.0
    w.q[:, 1, 1] = 2.0
    finite = ~np.isnan(w.k_pool)
    w.k_pool[finite] = rng.integers(-3, 4, size=int(finite.sum())).astype(np.float32)
    fv = ~np.isnan(w.v_pool)
    w.v_pool[fv] = rng.integers(-8, 9, size=int(fv.sum())).astype(np.float32) / 4
    w.scale = float(np.float32(math.log(2.0)))
    out = run(w)
    ln2_err = abs(float(np.float32(math.log(2.0))) - math.log(2.0))
    for i, n in enumerate(lens):
        for h in range(2):
            ks = gather_rows(w.k_pool, w.block_tables[i], n, 0, bs)
            vs = gather_rows(w.v_pool, w.block_tables[i], n, 0, bs)
            e = [int(ks[t, 0]) if h == 0 else 2 * int(ks[t, 1]) for t in range(n)]
            wt = [Fraction(2) ** x for x in e]
            Z = sum(wt)
            for d in range(D):
                exact = sum(wt[t] * Fraction(float(vs[t, d])) for t in range(n)) / Z
                # scale is ln 2 rounded to fp32, so every weight 2^e (|e| <= 6) is off by
                # a relative 6*ln2_err at most; |v| <= 2 and numerator and Z both move
                assert abs(out[i, h, d] - float(exact)) <= 2 * 2 * 6 * ln2_err + 1e-15


def test_brute_force_python_loops_tiny():
    """The definition typed out with Python floats and math.exp on random inputs."""
    bs, D = 2, 3
    lens = (4, 1, 5)
    w = small(111, dtype="bf16", Hq=4, Hkv=2, D=D, bs=bs, lens=lens, poison=True)
    out = run(w)
    kf, vf, qf = (W.bf16_bits_to_f32(a) for a in (w.k_pool, w.v_pool, w.q))
    sc = float(np.float32(w.scale))
    for i, n in enumerate(lens):
        for h in range(4):
            g = h // 2
            scores = []
            for t in range(n):
                blk, slot = int(w.block_tables[i, t // bs]), t % bs
                scores.append(sc * sum(float(qf[i, h, d]) * float(kf[blk, g, slot, d])
                                       for d in range(D)))
            mx = max(scores)
            ex = [math.exp(x - mx) for x in scores]
            z = sum(ex)
            for d in range(D):
                ref = 0.0
                for t in range(n):
                    blk, slot = int(w.block_tables[i, t // bs]), t % bs
                    ref += ex[t] / z * float(vf[blk, g, slot, d])
                assert abs(out[i, h, d] - ref) <= 1e-14


# P12 -----------------------------------------------------------------------
def test_nan_poison_outside_defined_reads_is_never_seen():
    lens = (1, 5, 9, 16, 0, 7)
    w_clean = small(12, dtype="bf16", Hq=4, Hkv=2, lens=lens, pool_factor=2.0, poison=False)
    w_pois = small(12, dtype="bf16", Hq=4, Hkv=2, lens=lens, pool_factor=2.0, poison=True)
    assert np.any(W.bf16_bits_to_f32(w_pois.k_pool) != W.bf16_bits_to_f32(w_pois.k_pool))  # has NaN
    a, b = run(w_clean), run(w_pois)
    assert np.all(np.isfinite(b))
    assert np.array_equal(a, b)
    assert np.all(b[4] == 0.0)          # empty context -> zero row


def test_bad_table_entry_is_reported():
    w = small(13, lens=(5,))
    w.block_tables[0, 1] = w.num_pool_blocks
    with pytest.raises(IndexError):
        run(w)


# Tiny config of the benchmark list: value-independent sanity at its real shape
def test_config1_shapes_and_transposed_operand_slip():
    w = W.config1_tiny()
    out = run(w)
    assert out.shape == (4, 8, 64) and np.all(np.isfinite(out))
    # swapping K and V pools must change the answer (guards a K/V mix-up)
    out_sw = oracle.paged_decode_attention(w.q, w.v_pool, w.k_pool, w.block_tables,
                                           w.context_lens, w.scale, block_size=16)
    assert np.abs(out - out_sw).max() > 1e-3


# Swap oracle ----------------------------------------------------------------
def _pool(planes, nblk, bb, seed):
    return W.random_bytes(planes * nblk * bb, seed).copy()


def test_swap_identity_mapping_is_memcpy():
    planes, nblk, bb = 3, 7, 64
    src = _pool(planes, nblk, bb, 1)
    dst = np.zeros_like(src)
    m = np.stack([np.arange(nblk), np.arange(nblk)], 1)
    oracle.kv_block_swap(src, dst, m, num_planes=planes, block_bytes=bb)
    assert np.array_equal(src, dst)


def test_swap_permutation_then_inverse_is_identity_and_direction_is_src_to_dst():
    planes, nblk, bb = 2, 9, 32
    src = _pool(planes, nblk, bb, 2)
    rng = np.random.default_rng(2)
    p = rng.permutation(nblk)
    mid = np.zeros_like(src)
    oracle.kv_block_swap(src, mid, np.stack([np.arange(nblk), p], 1), num_planes=planes, block_bytes=bb)
    s3 = src.reshape(planes, nblk, bb)
    m3 = mid.reshape(planes, nblk, bb)
    for j in range(nblk):                      # block j of src landed in block p[j] of dst
        assert np.array_equal(m3[:, p[j]], s3[:, j])
    back = np.zeros_like(src)
    oracle.kv_block_swap(mid, back, np.stack([p, np.arange(nblk)], 1), num_planes=planes, block_bytes=bb)
    assert np.array_equal(back, src)


def test_swap_round_trip_with_strides_and_untouched_bytes():
    sw = W.make_swap_workload("t", 5, victim_lens=(5, 33, 16, 70), num_planes=4, block_bytes=48,
                              block_size=16, pool_factor=1.5)
    n, P, bb, NB = sw.n_blocks, sw.num_planes, sw.block_bytes, sw.num_pool_blocks
    pad = 16
    pstride = NB * bb + pad                      # plane stride larger than the plane
    pool = W.random_bytes(P * pstride + 8 - (P * pstride) % 8, 6)[:P * pstride].copy()
    staging = np.full(P * n * bb, 0xAB, np.uint8)
    oracle.kv_block_swap(pool, staging, sw.gather_mapping, num_planes=P, block_bytes=bb,
                         src_plane_stride=pstride, src_num_blocks=NB)
    pool2 = np.full_like(pool, 0xCD)
    oracle.kv_block_swap(staging, pool2, sw.scatter_mapping, num_planes=P, block_bytes=bb,
                         dst_plane_stride=pstride, dst_num_blocks=NB)
    touched = np.zeros(pool.size, bool)
    for p in range(P):
        for j in range(n):
            s = p * pstride + int(sw.src_blocks[j]) * bb
            d = p * pstride + int(sw.new_blocks[j]) * bb
            assert np.array_equal(pool2[d:d + bb], pool[s:s + bb])
            assert np.array_equal(staging[(p * n + j) * bb:(p * n + j + 1) * bb], pool[s:s + bb])
            touched[d:d + bb] = True
    assert np.all(pool2[~touched] == 0xCD)


def test_swap_rejects_out_of_range_pair():
    src = np.zeros(64, np.uint8)
    dst = np.zeros(64, np.uint8)
    with pytest.raises(IndexError):
        oracle.kv_block_swap(src, dst, [[0, 4]], num_planes=1, block_bytes=16)


# Append oracle (Sec. 2.2: the new token's K/V rows join the cache) -----------------
def _new_rows(w, seed):
    rng = np.random.default_rng(seed)
    shape = (w.B, w.Hkv, w.D)
    k = rng.standard_normal(shape).astype(np.float32)
    v = rng.standard_normal(shape).astype(np.float32)
    if w.k_pool.dtype == np.uint16:
        return W.f32_to_bf16_bits(k), W.f32_to_bf16_bits(v)
    return k, v


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_append_writes_exactly_the_last_token_rows(dtype):
    lens = (1, 5, 8, 16, 0, 7)            # last slot of a block, first slot, empty sequence
    w = small(21, dtype=dtype, Hq=4, Hkv=2, lens=lens, pool_factor=2.0)
    kn, vn = _new_rows(w, 5)
    k0, v0 = w.k_pool.copy(), w.v_pool.copy()
    oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=w.block_size)
    # expected image built here with the test's own index arithmetic
    ke, ve = k0.copy(), v0.copy()
    for i, n in enumerate(lens):
        if n == 0:
            continue
        blk, slot = w.block_tables[i, (n - 1) // w.block_size], (n - 1) % w.block_size
        ke[blk, :, slot, :] = kn[i]
        ve[blk, :, slot, :] = vn[i]
    assert np.array_equal(w.k_pool.view(np.uint8), ke.view(np.uint8))   # bytewise: NaN poison stays put
    assert np.array_equal(w.v_pool.view(np.uint8), ve.view(np.uint8))
    assert not np.array_equal(ke.view(np.uint8), k0.view(np.uint8))


def test_append_then_attention_equals_attention_over_the_longer_contiguous_history():
    # grow every sequence by one token with append, then compare with softmax attention
    # written out here over explicitly concatenated K/V (no paging at all)
    lens0 = (3, 4, 7, 12)
    w = small(22, dtype="f32", Hq=4, Hkv=2, D=8, bs=4, lens=tuple(n + 1 for n in lens0), pool_factor=1.5)
    kn, vn = _new_rows(w, 6)
    hist_k = [[gather_rows(w.k_pool, w.block_tables[i], lens0[i], g, 4) for g in range(2)] for i in range(4)]
    hist_v = [[gather_rows(w.v_pool, w.block_tables[i], lens0[i], g, 4) for g in range(2)] for i in range(4)]
    oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=4)
    out = run(w)
    for i in range(4):
        for h in range(4):
            g = h // 2
            K = np.concatenate([hist_k[i][g], kn[i, g][None]]).astype(np.float64)
            V = np.concatenate([hist_v[i][g], vn[i, g][None]]).astype(np.float64)
            s = float(np.float32(w.scale)) * (K @ w.q[i, h].astype(np.float64))
            p = np.exp(s - s.max())
            assert np.abs(out[i, h] - (p / p.sum()) @ V).max() < 1e-12


def test_append_respects_strided_token_major_layout_and_reports_bad_table():
    w = small(23, dtype="bf16", Hq=4, Hkv=2, D=8, bs=4, lens=(6, 9), pool_factor=1.5)
    kn, vn = _new_rows(w, 7)
    # token-major copy of the pools: [block][slot][head][D]
    kt = np.ascontiguousarray(w.k_pool.transpose(0, 2, 1, 3))
    vt = np.ascontiguousarray(w.v_pool.transpose(0, 2, 1, 3))
    st = (4 * 2 * 8, 8, 2 * 8)            # block, head, token strides in elements
    oracle.kv_append(kt, vt, kn, vn, w.block_tables, w.context_lens, block_size=4, k_strides=st, v_strides=st)
    oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=4)
    assert np.array_equal(kt.transpose(0, 2, 1, 3), w.k_pool)
    assert np.array_equal(vt.transpose(0, 2, 1, 3), w.v_pool)
    # K head-major and V token-major in one call (their strides are independent)
    w2 = small(23, dtype="bf16", Hq=4, Hkv=2, D=8, bs=4, lens=(6, 9), pool_factor=1.5)
    vt2 = np.ascontiguousarray(w2.v_pool.transpose(0, 2, 1, 3))
    oracle.kv_append(w2.k_pool, vt2, kn, vn, w2.block_tables, w2.context_lens, block_size=4,
                     k_strides=(2 * 4 * 8, 4 * 8, 8), v_strides=st)
    assert np.array_equal(w2.k_pool, w.k_pool) and np.array_equal(vt2.transpose(0, 2, 1, 3), w.v_pool)
    w.block_tables[1, 2] = -1
    with pytest.raises(IndexError):
        oracle.kv_append(w.k_pool, w.v_pool, kn, vn, w.block_tables, w.context_lens, block_size=4)


# Prefill oracle (causal attention of a chunk over the paged cache) ---------------------------
def _contiguous(w, i, g):
    n = int(w.context_lens[i])
    return (as_f64(gather_rows(w.k_pool, w.block_tables[i], n, g, w.block_size)),
            as_f64(gather_rows(w.v_pool, w.block_tables[i], n, g, w.block_size)))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prefill_of_whole_sequences_matches_library_causal_sdpa(dtype):
    import torch
    lens = (1, 5, 9, 16)
    w = small(31, dtype=dtype, Hq=4, Hkv=2, D=8, bs=4, lens=lens)
    rng = np.random.default_rng(3)
    q = rng.standard_normal((sum(lens), 4, 8)).astype(np.float32)
    if dtype == "bf16":
        q = W.f32_to_bf16_bits(q)
    out = oracle.paged_prefill_attention(q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, lens,
                                         w.scale, block_size=4)
    row = 0
    for i, n in enumerate(lens):
        qi = torch.from_numpy(as_f64(q[row:row + n])).permute(1, 0, 2)              # [Hq, n, D]
        K = torch.stack([torch.from_numpy(_contiguous(w, i, h // 2)[0]) for h in range(4)])
        V = torch.stack([torch.from_numpy(_contiguous(w, i, h // 2)[1]) for h in range(4)])
        ref = torch.nn.functional.scaled_dot_product_attention(qi, K, V, is_causal=True,
                                                               scale=float(np.float32(w.scale)))
        assert np.abs(out[row:row + n] - ref.permute(1, 0, 2).numpy()).max() < 1e-12
        row += n


def test_prefill_chunk_is_the_tail_of_the_full_causal_result_and_one_token_is_decode():
    lens = (7, 12, 16)
    w = small(32, dtype="f32", Hq=4, Hkv=2, D=8, bs=4, lens=lens)
    rng = np.random.default_rng(4)
    q_full = rng.standard_normal((sum(lens), 4, 8)).astype(np.float32)
    full = oracle.paged_prefill_attention(q_full, w.k_pool, w.v_pool, w.block_tables, w.context_lens,
                                          lens, w.scale, block_size=4)
    chunk = (3, 12, 1)                  # a tail, the whole sequence, a single token
    starts = np.cumsum(lens) - np.array(lens)
    q_chunk = np.concatenate([q_full[s + n - c:s + n] for s, n, c in zip(starts, lens, chunk)])
    part = oracle.paged_prefill_attention(q_chunk, w.k_pool, w.v_pool, w.block_tables, w.context_lens,
                                          chunk, w.scale, block_size=4)
    want = np.concatenate([full[s + n - c:s + n] for s, n, c in zip(starts, lens, chunk)])
    assert np.array_equal(part, want)
    # the last token of every sequence sees everything: the decode result
    q_last = np.stack([q_full[s + n - 1] for s, n in zip(starts, lens)])
    dec = oracle.paged_decode_attention(q_last, w.k_pool, w.v_pool, w.block_tables, w.context_lens,
                                        w.scale, block_size=4)
    assert np.array_equal(np.stack([full[s + n - 1] for s, n in zip(starts, lens)]), dec)
    # the first token of a sequence sees only itself
    for i, s in enumerate(starts):
        for h in range(4):
            assert np.array_equal(full[s, h], _contiguous(w, i, h // 2)[1][0])


def test_prefill_query_length_above_the_context_is_clipped_like_the_chunk_append():
    """The library's rule for a query length above the context length (the same one kv_append_chunk
    follows): only the first min(query, context) rows of the sequence exist, row j at position j,
    so they equal the whole-sequence result; the surplus rows have no value (NaN)."""
    lens = (7, 12, 0, 5)
    over = (9, 12, 2, 30)
    w = small(33, dtype="f32", Hq=4, Hkv=2, D=8, bs=4, lens=lens)
    rng = np.random.default_rng(6)
    q_over = rng.standard_normal((sum(over), 4, 8)).astype(np.float32)
    got = oracle.paged_prefill_attention(q_over, w.k_pool, w.v_pool, w.block_tables, w.context_lens,
                                         over, w.scale, block_size=4)
    first = np.cumsum(over) - np.array(over)
    q_exact = np.concatenate([q_over[f:f + n] for f, n in zip(first, lens)])
    whole = oracle.paged_prefill_attention(q_exact, w.k_pool, w.v_pool, w.block_tables, w.context_lens,
                                           lens, w.scale, block_size=4)
    row = 0
    for f, n, o in zip(first, lens, over):
        assert np.array_equal(got[f:f + n], whole[row:row + n])
        assert np.isnan(got[f + n:f + o]).all()
        row += n
    # the rows the chunk append writes for the same lengths are exactly the rows that exist
    kp, vp = w.k_pool.copy(), w.v_pool.copy()
    kn = rng.standard_normal((sum(over), 2, 8)).astype(np.float32)
    oracle.kv_append_chunk(kp, vp, kn, kn, w.block_tables, w.context_lens, np.array(over), block_size=4)
    for i, (f, n) in enumerate(zip(first, lens)):
        for j in range(n):
            assert np.array_equal(kp[w.block_tables[i, j // 4], :, j % 4], kn[f + j])


# ---- chunk append --------------------------------------------------------------------------------
def test_chunk_append_equals_token_by_token_append_and_touches_nothing_else():
    """The chunk routine (Python loops) against the single-token routine (C) applied once per
    token with a growing context, and against positions worked out here."""
    w = W.make_attn_workload("chunk", 31, dtype="bf16", Hq=4, Hkv=2, D=16, block_size=4,
                             context_lens=(9, 4, 17, 6), pool_factor=1.5)
    ql = np.array([5, 4, 0, 9], np.int32)                 # a tail, a whole prompt, nothing, more than the context (clipped to 6)
    rng = np.random.default_rng(32)
    total = int(ql.sum())
    kn = rng.integers(0, 2**16, (total, 2, 16)).astype(np.uint16)
    vn = rng.integers(0, 2**16, (total, 2, 16)).astype(np.uint16)
    k1, v1 = w.k_pool.copy(), w.v_pool.copy()
    oracle.kv_append_chunk(k1, v1, kn, vn, w.block_tables, w.context_lens, ql, block_size=4)
    # token by token with the C routine: sequence i alone, context growing from n - ql + 1 to n
    k2, v2 = w.k_pool.copy(), w.v_pool.copy()
    first = 0
    for i, (n, q) in enumerate(zip(w.context_lens.tolist(), ql.tolist())):
        use = min(q, n)
        for j in range(use):
            cl = np.zeros(w.B, np.int32)
            cl[i] = n - use + j + 1
            rows_k = np.zeros((w.B, 2, 16), np.uint16); rows_v = np.zeros((w.B, 2, 16), np.uint16)
            rows_k[i], rows_v[i] = kn[first + j], vn[first + j]
            oracle.kv_append(k2, v2, rows_k, rows_v, w.block_tables, cl, block_size=4)
        first += q
    assert np.array_equal(k1, k2) and np.array_equal(v1, v2)
    # positions by hand for sequence 0: the last 5 of 9 tokens are positions 4..8 = blocks 1, 1, 1, 1, 2
    for j, pos in enumerate(range(4, 9)):
        assert np.array_equal(k1[w.block_tables[0, pos // 4], :, pos % 4], kn[j])
    assert int(np.any(k1 != w.k_pool, axis=(1, 3)).sum()) <= 5 + 4 + 6   # at most one (block, slot) per written token


# ---- 8-bit (OCP E4M3) pools -------------------------------------------------------------------------
def torch_f8_to_f64(codes):
    """Library decode of E4M3 codes, independent of the oracle's."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(codes, np.uint8)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def test_f8_all_256_codes_decode_as_the_format_defines():
    """Every code through the oracle's V path (a 1-token context returns the V row: its 128 dims hold
    codes 0..127, those of a second sequence 128..255) against a library conversion, and a few
    codes against the values the format definition fixes."""
    D = 128
    k_pool = np.zeros((2, 1, 16, D), np.uint8)
    v_pool = np.zeros((2, 1, 16, D), np.uint8)
    v_pool[0, 0, 0] = np.arange(128)
    v_pool[1, 0, 0] = np.arange(128, 256)
    q = np.zeros((2, 1, D), np.uint16)
    out = oracle.paged_decode_attention(q, k_pool, v_pool, np.array([[0], [1]], np.int32), np.array([1, 1], np.int32),
                                        1.0, block_size=16)
    got = out.reshape(256)
    ref = torch_f8_to_f64(np.arange(256))
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and np.isnan(ref[0x7F]) and np.isnan(ref[0xFF])
    ok = ~np.isnan(ref)
    assert ok.sum() == 254 and np.array_equal(got[ok], ref[ok])
    assert got[0x80] == 0.0                  # the sign of -0.0 (code 0x80) does not survive the weighted sum
    fixed = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x39: 1.125, 0x40: 2.0,
             0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0, 0x78: 256.0, 0x77: 240.0}
    for code, value in fixed.items():
        assert got[code] == value, (hex(code), got[code], value)


def test_f8_keys_decode_in_the_score_path():
    """q = unit vector along dim 3 and scale 1: the score of token t is its key's dim-3 value, so the
    log of a weight ratio is a difference of decoded key values."""
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], np.uint8)
    codes = codes[np.abs(torch_f8_to_f64(codes)) <= 32]          # keep exp() far from overflow
    n, D = len(codes), 8
    nb = (n + 15) // 16
    k_pool = np.zeros((nb, 1, 16, D), np.uint8)
    k_pool.reshape(nb * 16, D)[:n, 3] = codes
    v_pool = np.zeros_like(k_pool)
    q = np.zeros((1, 1, D), np.uint16)
    q[0, 0, 3] = 0x3F80                                          # bf16 1.0
    _, w = oracle.paged_decode_attention(q, k_pool, v_pool, np.arange(nb, dtype=np.int32)[None], np.array([n], np.int32),
                                         1.0, block_size=16, return_weights=True)
    vals = torch_f8_to_f64(codes)
    np.testing.assert_allclose(np.log(w[0, 0, :n] / w[0, 0, 0]), vals - vals[0], rtol=0, atol=1e-9)


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 2, 32), (16, 2, 128)])
def test_f8_pools_match_library_sdpa_on_dequantised_tensors(Hq, Hkv, D):
    import torch
    import torch.nn.functional as F
    ks, vs = 0.75, 1.5
    w = W.make_attn_workload("t8", 12, dtype="f8", Hq=Hq, Hkv=Hkv, D=D, block_size=16,
                             context_lens=(17, 64, 100, 256), num_pool_blocks=64)
    assert w.k_pool.dtype == np.uint8 and w.q.dtype == np.uint16
    out = run(w, k_scale=ks, v_scale=vs)
    G = Hq // Hkv
    for i in range(w.B):
        n = int(w.context_lens[i])
        k = np.stack([torch_f8_to_f64(gather_rows(w.k_pool, w.block_tables[i], n, g, 16)) for g in range(Hkv)]) * ks
        v = np.stack([torch_f8_to_f64(gather_rows(w.v_pool, w.block_tables[i], n, g, 16)) for g in range(Hkv)]) * vs
        kt = torch.from_numpy(k).repeat_interleave(G, dim=0)[None]
        vt = torch.from_numpy(v).repeat_interleave(G, dim=0)[None]
        qt = torch.from_numpy(as_f64(w.q[i]))[None, :, None, :]
        ref = F.scaled_dot_product_attention(qt, kt, vt, attn_mask=None, dropout_p=0.0, is_causal=False,
                                             scale=float(np.float32(w.scale)))
        np.testing.assert_allclose(out[i], ref[0, :, 0].numpy(), rtol=0, atol=1e-12)


def test_f8_scales_equal_prescaled_wider_pools_and_poison_is_not_read():
    """k_scale and v_scale are plain factors on the stored values: the same call on bf16 pools that
    hold scale * value (powers of two: exact in bf16) gives the same result bit for bit; NaN codes
    in free blocks and dead tail slots are never read."""
    w = W.make_attn_workload("t8s", 13, dtype="f8", Hq=4, Hkv=2, D=16, block_size=16,
                             context_lens=(5, 33, 16, 0), pool_factor=1.5, poison=True)
    assert (w.k_pool == 0x7F).any()
    got = run(w, k_scale=0.25, v_scale=4.0)
    assert np.isfinite(got).all() and np.all(got[3] == 0.0)
    kb = W.f32_to_bf16_bits((torch_f8_to_f64(w.k_pool) * 0.25).astype(np.float32))
    vb = W.f32_to_bf16_bits((torch_f8_to_f64(w.v_pool) * 4.0).astype(np.float32))
    wide = oracle.paged_decode_attention(w.q, kb, vb, w.block_tables, w.context_lens, w.scale, block_size=16)
    assert np.array_equal(got, wide)


def test_f8_prefill_is_the_prefill_of_prescaled_wider_pools():
    """The prefill oracle over 8-bit pools hands the pools' scales on to its decode rows: a chunk
    over a cached prefix equals, bit for bit, the same chunk over bf16 pools that hold
    scale * value (powers of two: exact in bf16); with the scales left out it does not."""
    w = W.make_attn_workload("t8p", 17, dtype="f8", Hq=4, Hkv=2, D=16, block_size=16,
                             context_lens=(40, 7, 33), pool_factor=1.5, poison=True)
    ql = np.array([9, 7, 1], np.int32)
    q = W.f32_to_bf16_bits(np.random.default_rng(18).standard_normal((int(ql.sum()), 4, 16)).astype(np.float32))
    got = oracle.paged_prefill_attention(q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, ql, w.scale,
                                         block_size=16, k_scale=0.5, v_scale=8.0)
    kb = W.f32_to_bf16_bits((torch_f8_to_f64(w.k_pool) * 0.5).astype(np.float32))
    vb = W.f32_to_bf16_bits((torch_f8_to_f64(w.v_pool) * 8.0).astype(np.float32))
    wide = oracle.paged_prefill_attention(q, kb, vb, w.block_tables, w.context_lens, ql, w.scale, block_size=16)
    assert np.isfinite(got).all() and np.array_equal(got, wide)
    plain = oracle.paged_prefill_attention(q, w.k_pool, w.v_pool, w.block_tables, w.context_lens, ql, w.scale,
                                           block_size=16)
    assert np.abs(plain - got).max() > 0.1


def test_f8_generator_rounds_to_nearest_even_and_saturates():
    """The input generator's float32 -> E4M3 rounding against the library conversion (in range), and
    its closed-form corner cases."""
    import torch
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(100000) * rng.choice([1e-3, 0.01, 0.1, 1, 10, 100], 100000)).astype(np.float32)
    x = x[np.abs(x) <= 448]
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(W.f32_to_f8e4m3_bits(x), ref)
    corner = np.array([0.0, -0.0, 2.0 ** -10, 1.5 * 2.0 ** -10, 2.5 * 2.0 ** -9, 3.5 * 2.0 ** -9, 1.0625, 1.1875, 448.0,
                       1e9, -1e9, np.nan], np.float32)
    want = np.array([0x00, 0x80, 0x00, 0x01, 0x02, 0x04, 0x38, 0x3A, 0x7E, 0x7E, 0xFE, 0x7F], np.uint8)
    assert np.array_equal(W.f32_to_f8e4m3_bits(corner), want)
