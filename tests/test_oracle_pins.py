"""Pins of the CPU oracle against things other than itself: brute force on un-paged KV,
torch's float64 SDPA, closed forms, invariants and reductions (CPU only)."""
import math
import os

import numpy as np
import pytest

from paper_2508_15919_amd import synth
from paper_2508_15919_amd.synth import DECODE, PREFILL, StepBatch, bf16_bits_to_f64, f32_to_bf16_bits
from tests import brute

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def small_mixed(seed=3, Hq=4, Hkv=2, D=64):
    return synth.make_batch(Hq, Hkv, D, [DECODE, PREFILL, DECODE, PREFILL, DECODE],
                            [1, 19, 1, 33, 1], [1, 19, 50, 70, 16], seed)


def manual_batch(Hq, Hkv, D, kind, q_len, ctx_len, q_f32, k_f32, v_f32, pages=None):
    """Step over explicit per-request K/V (float32 [c, Hkv, D]) placed token by token."""
    R = len(kind)
    npg = [(c + 15) // 16 for c in ctx_len]
    total = sum(npg)
    if pages is None:
        pages = list(range(total))[::-1]
    pool = np.full((total + 2, Hkv, 2, 16 * D), synth.BF16_NAN, dtype=np.uint16)
    indptr = np.zeros(R + 1, np.int32)
    indptr[1:] = np.cumsum(npg)
    for r in range(R):
        kb, vb = f32_to_bf16_bits(k_f32[r]), f32_to_bf16_bits(v_f32[r])
        for t in range(ctx_len[r]):
            pg = pages[indptr[r] + t // 16]
            for g in range(Hkv):
                pool[pg, g, 0].reshape(D // 16, 16, 16)[:, t % 16, :] = kb[t, g].reshape(D // 16, 16)
                pool[pg, g, 1].reshape(D, 16)[:, t % 16] = vb[t, g]
    q = f32_to_bf16_bits(np.concatenate(q_f32, axis=0))
    return StepBatch(Hq, Hkv, D, total + 2, np.array(kind, np.int32), np.array(q_len, np.int32),
                     np.array(ctx_len, np.int32), indptr, np.array(pages, np.int32), q, pool)


def test_brute_force_on_unpaged_kv(oracle):
    for seed, (Hq, Hkv, D) in enumerate([(4, 2, 64), (8, 1, 128), (6, 6, 32), (32, 8, 128), (3, 1, 16)]):
        b = small_mixed(seed, Hq, Hkv, D)
        got = oracle.attention_batch(b)
        ref = brute.dense_attention(b)
        assert np.abs(got - ref).max() <= 1e-12


def test_config1_matches_brute_force(oracle):
    b = synth.config(1)
    assert list(b.ctx_len) == [37, 64, 129, 32] and list(b.q_len) == [1, 1, 1, 32]
    assert int(b.bt_indptr[-1]) == 3 + 4 + 9 + 2
    assert np.abs(oracle.attention_batch(b) - brute.dense_attention(b)).max() <= 1e-12


def test_torch_sdpa_float64(oracle):
    torch = pytest.importorskip("torch")
    b = small_mixed(11)
    got = oracle.attention_batch(b)
    G = b.num_q_heads // b.num_kv_heads
    qi = b.q_indptr()
    for r in range(b.num_requests):
        k, v = brute.unpage(b, r)
        c, ql = int(b.ctx_len[r]), int(b.q_len[r])
        q = torch.from_numpy(bf16_bits_to_f64(b.q[qi[r]:qi[r + 1]])).permute(1, 0, 2)      # [Hq, ql, D]
        kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(G, dim=0)
        vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(G, dim=0)
        pos = (c - ql) + torch.arange(ql)
        allowed = torch.arange(c)[None, :] <= pos[:, None]
        o = torch.nn.functional.scaled_dot_product_attention(q, kt, vt, attn_mask=allowed)
        assert np.abs(o.permute(1, 0, 2).numpy() - got[qi[r]:qi[r + 1]]).max() <= 1e-12


def test_golden_two_key_logistic(oracle):
    want = {}
    with open(os.path.join(GOLD, "two_key_logistic.txt")) as f:
        for line in f:
            if line.startswith("out"):
                k, v = line.split()
                want[k] = float(v)
    D = 16                       # the two coordinates of the example, zero padded to one 16-dimension block
    e0, e1 = np.zeros(D, np.float32), np.zeros(D, np.float32)
    e0[0], e1[1] = 1.0, 1.0
    q = [e0.reshape(1, 1, D)]
    k = [np.stack([np.zeros(D, np.float32), e0]).reshape(2, 1, D)]
    v = [np.stack([e0, e1]).reshape(2, 1, D)]
    b = manual_batch(1, 1, D, [DECODE], [1], [2], q, k, v)
    got = oracle.attention_batch(b, scale=1.0)
    assert abs(got[0, 0, 0] - want["out0"]) < 1e-15 and abs(got[0, 0, 1] - want["out1"]) < 1e-15
    assert np.all(got[0, 0, 2:] == 0.0)
    assert abs(want["out1"] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15


def test_single_token_context_returns_v_exactly(oracle):
    b = synth.make_batch(4, 2, 64, [DECODE, PREFILL], [1, 1], [1, 1], 5)
    got = oracle.attention_batch(b)
    for r in range(2):
        _, v = brute.unpage(b, r)
        for h in range(4):
            assert np.array_equal(got[r, h], v[0, h // 2])


def test_page_permutation_invariance_is_bit_exact(oracle):
    b = small_mixed(21)
    a = oracle.attention_batch(b)
    for s in (1, 2):
        p = synth.permute_pages(b, s)
        assert not np.array_equal(p.bt_pages, b.bt_pages)
        assert np.array_equal(oracle.attention_batch(p), a)


def test_uniform_keys_give_mean_of_values(oracle):
    rng = np.random.default_rng(0)
    Hq, Hkv, D, c, ql = 4, 2, 16, 45, 7
    krow = rng.standard_normal((1, Hkv, D)).astype(np.float32)
    k = [np.repeat(krow, c, axis=0)]
    v = [rng.standard_normal((c, Hkv, D)).astype(np.float32)]
    q = [rng.standard_normal((ql, Hq, D)).astype(np.float32)]
    b = manual_batch(Hq, Hkv, D, [PREFILL], [ql], [c], q, k, v)
    got = oracle.attention_batch(b)
    vv = bf16_bits_to_f64(f32_to_bf16_bits(v[0]))
    for i in range(ql):
        n = c - ql + i + 1
        for h in range(Hq):
            assert np.abs(got[i, h] - vv[:n, h // 2].mean(axis=0)).max() < 1e-13


def test_constant_values_pass_through(oracle):
    rng = np.random.default_rng(1)
    Hq, Hkv, D, c = 2, 1, 32, 70
    vrow = rng.standard_normal((1, Hkv, D)).astype(np.float32)
    b = manual_batch(Hq, Hkv, D, [DECODE], [1], [c], [rng.standard_normal((1, Hq, D)).astype(np.float32)],
                     [rng.standard_normal((c, Hkv, D)).astype(np.float32)], [np.repeat(vrow, c, axis=0)])
    got = oracle.attention_batch(b)
    want = bf16_bits_to_f64(f32_to_bf16_bits(vrow))[0, 0]
    assert np.abs(got[0] - want[None]).max() < 1e-14


def test_dominant_key_selects_its_value(oracle):
    rng = np.random.default_rng(2)
    Hq, Hkv, D, c, j = 1, 1, 16, 40, 23
    k = np.zeros((c, 1, D), np.float32)
    k[j, 0, 0] = 64.0
    q = np.zeros((1, 1, D), np.float32)
    q[0, 0, 0] = 16.0                        # s_j = 1024/4 = 256, all others 0
    v = rng.standard_normal((c, 1, D)).astype(np.float32)
    b = manual_batch(Hq, Hkv, D, [DECODE], [1], [c], [q], [k], [v])
    got = oracle.attention_batch(b)
    assert np.abs(got[0, 0] - bf16_bits_to_f64(f32_to_bf16_bits(v))[j, 0]).max() < 1e-20


def test_softmax_shift_invariance(oracle):
    # q = e0; adding a constant to coordinate 0 of every key shifts every score equally.
    rng = np.random.default_rng(3)
    Hq, Hkv, D, c = 1, 1, 16, 33
    q = np.zeros((1, 1, D), np.float32)
    q[0, 0, 0] = 1.0
    k = (rng.integers(-8, 9, (c, 1, D)) / 4.0).astype(np.float32)       # exactly bf16-representable
    v = rng.standard_normal((c, 1, D)).astype(np.float32)
    k2 = k.copy()
    k2[:, 0, 0] += 4.0
    a = oracle.attention_batch(manual_batch(Hq, Hkv, D, [DECODE], [1], [c], [q], [k], [v]))
    b = oracle.attention_batch(manual_batch(Hq, Hkv, D, [DECODE], [1], [c], [q], [k2], [v]))
    assert np.abs(a - b).max() < 1e-14


def _shared_prefix_pair(seed, Hq=4, Hkv=2, D=64):
    """One 64-token prompt; returns its K/V/Q so that several steps can view the same cache."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((64, Hq, D)).astype(np.float32),
            rng.standard_normal((64, Hkv, D)).astype(np.float32),
            rng.standard_normal((64, Hkv, D)).astype(np.float32))


def test_chunk_split_invariance(oracle):
    Hq, Hkv, D = 4, 2, 64
    q, k, v = _shared_prefix_pair(4)
    whole = oracle.attention_batch(manual_batch(Hq, Hkv, D, [PREFILL], [64], [64], [q], [k], [v]))
    first = oracle.attention_batch(manual_batch(Hq, Hkv, D, [PREFILL], [32], [32], [q[:32]], [k[:32]], [v[:32]]))
    second = oracle.attention_batch(manual_batch(Hq, Hkv, D, [PREFILL], [32], [64], [q[32:]], [k], [v]))
    assert np.array_equal(whole[:32], first) and np.array_equal(whole[32:], second)


def test_prefill_row_equals_decode_over_same_pages(oracle):
    Hq, Hkv, D = 4, 2, 64
    q, k, v = _shared_prefix_pair(5)
    whole = oracle.attention_batch(manual_batch(Hq, Hkv, D, [PREFILL], [64], [64], [q], [k], [v]))
    for i in (0, 15, 16, 40, 63):
        dec = oracle.attention_batch(manual_batch(Hq, Hkv, D, [DECODE], [1], [i + 1], [q[i:i + 1]],
                                                  [k[:i + 1]], [v[:i + 1]]))
        assert np.array_equal(dec[0], whole[i])
    # decode == prefill with a one-token chunk
    a = oracle.attention_batch(manual_batch(Hq, Hkv, D, [DECODE], [1], [64], [q[63:]], [k], [v]))
    b = oracle.attention_batch(manual_batch(Hq, Hkv, D, [PREFILL], [1], [64], [q[63:]], [k], [v]))
    assert np.array_equal(a, b)


def test_duplicate_q_heads_in_a_group_agree_and_groups_differ(oracle):
    b = small_mixed(31, Hq=8, Hkv=2, D=64)
    b.q[:, 1] = b.q[:, 0]          # same group (heads 0..3 -> kv 0)
    b.q[:, 4] = b.q[:, 0]          # other group (heads 4..7 -> kv 1)
    got = oracle.attention_batch(b)
    assert np.array_equal(got[:, 0], got[:, 1])
    assert not np.allclose(got[:, 0], got[:, 4])


def test_poisoned_extra_pages_and_tails_change_nothing(oracle):
    kinds, ql, cl = [DECODE, PREFILL, DECODE], [1, 20, 1], [37, 50, 129]
    a = synth.make_batch(4, 2, 64, kinds, ql, cl, 9, poison=False)
    b = synth.make_batch(4, 2, 64, kinds, ql, cl, 9, poison=True, extra_pages_per_request=2)
    ra, rb = oracle.attention_batch(a), oracle.attention_batch(b)
    assert np.isfinite(rb).all() and np.abs(ra - brute.dense_attention(a)).max() < 1e-12
    assert np.abs(rb - brute.dense_attention(b)).max() < 1e-12


def test_shared_prefix_pages(oracle):
    b = synth.make_batch(4, 2, 64, [DECODE, DECODE], [1, 1], [48, 48], 13)
    b.bt_pages[b.bt_indptr[1]: b.bt_indptr[1] + 2] = b.bt_pages[0:2]     # first 32 tokens shared
    got = oracle.attention_batch(b)
    assert np.abs(got - brute.dense_attention(b)).max() < 1e-12


def test_rows_entry_point_matches_full(oracle):
    b = small_mixed(17)
    full = oracle.attention_batch(b)
    qi = b.q_indptr()
    req = [1, 1, 3, 3, 4, 0]
    row = [0, 18, 5, 32, 0, 0]
    head = [0, 3, 2, 1, 3, 2]
    got = oracle.attention_rows_batch(b, req, row, head)
    for k in range(len(req)):
        assert np.array_equal(got[k], full[qi[req[k]] + row[k], head[k]])


def test_gather_is_a_bit_copy(oracle):
    b = small_mixed(19)
    for r in range(b.num_requests):
        k, v = oracle.gather_kv(b.num_kv_heads, b.head_dim, b.num_pages, b.ctx_len, b.bt_indptr, b.bt_pages,
                                b.pool, r)
        bk, bv = brute.unpage(b, r)
        assert np.array_equal(bf16_bits_to_f64(k), bk) and np.array_equal(bf16_bits_to_f64(v), bv)


def test_gather_recovers_tokens_written_one_by_one(oracle):
    rng = np.random.default_rng(8)
    Hkv, D, c = 2, 64, 41
    k = rng.standard_normal((c, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((c, Hkv, D)).astype(np.float32)
    b = manual_batch(4, Hkv, D, [DECODE], [1], [c], [np.zeros((1, 4, D), np.float32)], [k], [v])
    gk, gv = oracle.gather_kv(Hkv, D, b.num_pages, b.ctx_len, b.bt_indptr, b.bt_pages, b.pool, 0)
    assert np.array_equal(gk, f32_to_bf16_bits(k)) and np.array_equal(gv, f32_to_bf16_bits(v))


def test_append_writes_exactly_the_chunk_tokens(oracle):
    # pinned by the independent numpy un-paging: after the append the chunk's tokens read back as the
    # new K/V, and every other element of the pool is untouched
    b = small_mixed(23, Hq=8, Hkv=2, D=64)
    rng = np.random.default_rng(4)
    T = b.total_q
    k_new = f32_to_bf16_bits(rng.standard_normal((T, 2, 64)).astype(np.float32))
    v_new = f32_to_bf16_bits(rng.standard_normal((T, 2, 64)).astype(np.float32))
    before = b.pool.copy()
    oracle.append_kv(2, 64, b.num_pages, b.q_len, b.ctx_len, b.bt_indptr, b.bt_pages, k_new, v_new, b.pool)
    qi = b.q_indptr()
    touched = np.zeros(b.pool.shape, bool)
    for r in range(b.num_requests):
        c, ql = int(b.ctx_len[r]), int(b.q_len[r])
        k, v = brute.unpage(b, r)
        assert np.array_equal(k[c - ql:], bf16_bits_to_f64(k_new[qi[r]:qi[r + 1]]))
        assert np.array_equal(v[c - ql:], bf16_bits_to_f64(v_new[qi[r]:qi[r + 1]]))
        for t in range(c - ql, c):
            pg = b.bt_pages[b.bt_indptr[r] + t // 16]
            touched[pg, :, 0].reshape(2, 4, 16, 16)[:, :, t % 16, :] = True
            touched[pg, :, 1].reshape(2, 64, 16)[:, :, t % 16] = True
    assert np.array_equal(b.pool[~touched], before[~touched])
    assert touched.sum() == 2 * T * 2 * 64


def test_copy_pages_moves_whole_pages_and_nothing_else(oracle):
    # pinned by numpy's fancy indexing, and end to end: a request un-paged through the destination
    # pool and its new block table reads exactly what it read through the source pool
    b = small_mixed(29, Hq=8, Hkv=2, D=64)
    rng = np.random.default_rng(8)
    r = 1
    src_ids = b.bt_pages[b.bt_indptr[r]:b.bt_indptr[r + 1]].copy()
    dst = f32_to_bf16_bits(rng.standard_normal((40,) + b.pool.shape[1:]).astype(np.float32))
    before = dst.copy()
    dst_ids = rng.permutation(40)[:len(src_ids)].astype(np.int32)
    oracle.copy_pages(2, 64, src_ids, dst_ids, b.pool, dst)
    want = before.copy()
    want[dst_ids] = b.pool[src_ids]
    assert np.array_equal(dst, want)
    k0, v0 = brute.unpage(b, r)
    import copy
    b2 = copy.copy(b)
    b2.pool, b2.num_pages = dst, 40
    b2.bt_pages = b.bt_pages.copy()
    b2.bt_pages[b.bt_indptr[r]:b.bt_indptr[r + 1]] = dst_ids
    k1, v1 = brute.unpage(b2, r)
    assert np.array_equal(k0, k1) and np.array_equal(v0, v1)
    with pytest.raises(ValueError):
        oracle.copy_pages(2, 64, [0], [40], b.pool, dst)


def test_split_merge_identity_in_fp64():
    # (m, l, acc) partials over any partition of the keys merge to the one-pass result.
    rng = np.random.default_rng(6)
    n, D = 300, 8
    s = rng.standard_normal(n) * 3
    v = rng.standard_normal((n, D))
    w = np.exp(s - s.max())
    ref = (w[:, None] * v).sum(0) / w.sum()
    cuts = np.sort(rng.choice(np.arange(1, n), 6, replace=False))
    parts = np.split(np.arange(n), cuts)
    ms = [s[p].max() for p in parts]
    ls = [np.exp(s[p] - m).sum() for p, m in zip(parts, ms)]
    accs = [(np.exp(s[p] - m)[:, None] * v[p]).sum(0) for p, m in zip(parts, ms)]
    mstar = max(ms)
    ell = sum(l * math.exp(m - mstar) for l, m in zip(ls, ms))
    o = sum(a * math.exp(m - mstar) for a, m in zip(accs, ms)) / ell
    assert np.abs(o - ref).max() < 1e-12


def test_oracle_rejects_bad_inputs(oracle):
    b = small_mixed(2)
    bad = synth.permute_pages(b, 1)
    bad.bt_pages[0] = b.num_pages
    with pytest.raises(ValueError):
        oracle.attention_batch(bad)
    bad = synth.permute_pages(b, 1)
    bad.ctx_len[1] = 5                   # < q_len
    with pytest.raises(ValueError):
        oracle.attention_batch(bad)


def test_bf16_rounding_helper_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.140625, 1e-3], np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    got = synth.bf16_bits_to_f32(f32_to_bf16_bits(x))
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == np.float32(1.015625) and got[3] == -2.5
    torch = pytest.importorskip("torch")
    r = np.random.default_rng(0).standard_normal(4096).astype(np.float32)
    want = torch.from_numpy(r).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(synth.bf16_bits_to_f32(f32_to_bf16_bits(r)), want)
