"""Pins of the fp64 CPU oracle: closed forms, invariants, library routines and brute force.

Each check takes the oracle through its public Python functions only, and compares it with
something that is not the oracle: a closed form worked out by hand, numpy/scipy library
routines, or a pure-Python ``math.fsum`` evaluation.  They are plain functions so that the
mutant test can run the same checks against deliberately broken builds of the oracle.
"""
import math

import numpy as np
from scipy.special import logsumexp, softmax

import oracle
from workloads import bf16_to_f32, f32_to_bf16, normal_bf16

D = 128
SCALE = float(np.float32(1.0 / math.sqrt(D)))


def f64(bits):
    return bf16_to_f32(bits).astype(np.float64)


def rnd(seed, stream, *shape):
    return normal_bf16(seed, stream, int(np.prod(shape))).reshape(shape)


def small_ints(seed, stream, lo, hi, *shape):
    """bf16 bit patterns of integers in [lo, hi]: exactly representable, sums stay exact."""
    z = f64(rnd(seed, stream, *shape))
    v = np.clip(np.rint(z * (hi - lo) / 4.0), lo, hi)
    return f32_to_bf16(v.astype(np.float32))


# 1 ---------------------------------------------------------------------------------------
def check_single_key():
    """kv_len = 1: the softmax has one term, so out is that V row and lse is its score."""
    Hq, Hkv = 8, 2
    q, k, v = rnd(11, 0, 1, 1, Hq, D), rnd(11, 1, 1, Hkv, D), rnd(11, 2, 1, Hkv, D)
    out, lse = oracle.attn(q, [k], [v], [1], SCALE)
    for h in range(Hq):
        g = h // (Hq // Hkv)
        np.testing.assert_array_equal(out[0, 0, h], f64(v[0, g]))
        s0 = SCALE * float(np.dot(f64(q[0, 0, h]), f64(k[0, g])))
        assert abs(lse[0, 0, h] - s0) < 1e-12 * max(1.0, abs(s0))


# 2 ---------------------------------------------------------------------------------------
def check_identical_keys():
    """All keys equal: uniform weights, out = mean of the V rows, lse = s + ln L."""
    Hq, Hkv, L = 4, 2, 37
    q, k1, v = rnd(12, 0, 1, 1, Hq, D), rnd(12, 1, 1, Hkv, D), rnd(12, 2, L, Hkv, D)
    k = np.repeat(k1, L, axis=0)
    out, lse = oracle.attn(q, [k], [v], [L], SCALE)
    for h in range(Hq):
        g = h // 2
        np.testing.assert_allclose(out[0, 0, h], f64(v[:, g]).mean(axis=0), rtol=0, atol=1e-12)
        s = SCALE * float(np.dot(f64(q[0, 0, h]), f64(k1[0, g])))
        assert abs(lse[0, 0, h] - (s + math.log(L))) < 1e-12


# 3 ---------------------------------------------------------------------------------------
def check_weights_sum_to_one():
    """The normalised weights of a row are positive, one per visible key, and sum to 1."""
    Hq, Hkv, T, L = 4, 2, 3, 50
    q, k, v = rnd(13, 0, 1, T, Hq, D), rnd(13, 1, L, Hkv, D), rnd(13, 2, L, Hkv, D)
    for t in range(T):
        for h in range(Hq):
            w = oracle.attn_weights(q, [k], [v], [L], SCALE, 0, t, h)
            assert w.shape == (L - T + t + 1,)
            assert np.all(w > 0)
            assert abs(math.fsum(w) - 1.0) < 1e-13


# 4 ---------------------------------------------------------------------------------------
def check_zero_query():
    """q = 0: every score is 0, so out = mean(V) and lse = ln L."""
    Hq, Hkv, L = 4, 4, 23
    q = np.zeros((1, 1, Hq, D), dtype=np.uint16)
    k, v = rnd(14, 1, L, Hkv, D), rnd(14, 2, L, Hkv, D)
    out, lse = oracle.attn(q, [k], [v], [L], SCALE)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, 0, h], f64(v[:, h]).mean(axis=0), rtol=0, atol=1e-13)
        assert abs(lse[0, 0, h] - math.log(L)) < 1e-13


# 5 ---------------------------------------------------------------------------------------
def check_dominant_key():
    """One key aligned with q and scaled up: its weight tends to 1 and out to its V row.

    The max must be subtracted before exp, or exp(score) overflows (score ~ 3e4 here).
    """
    Hq, Hkv, L, jstar = 2, 1, 40, 17
    q, k, v = rnd(15, 0, 1, 1, Hq, D), rnd(15, 1, L, Hkv, D), rnd(15, 2, L, Hkv, D)
    k = k.copy()
    k[jstar, 0] = f32_to_bf16(bf16_to_f32(q[0, 0, 0]) * np.float32(2048.0))   # exact: power of two
    out, lse = oracle.attn(q, [k], [v], [L], SCALE)
    s = SCALE * (f64(k[:, 0]) @ f64(q[0, 0, 0]))
    gap = s[jstar] - np.max(np.delete(s, jstar))
    assert gap > 700.0                                   # exp(-gap) underflows to exactly 0
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))
    np.testing.assert_array_equal(out[0, 0, 0], f64(v[jstar, 0]))
    assert abs(lse[0, 0, 0] - s[jstar]) < 1e-9 * abs(s[jstar])


# 6 ---------------------------------------------------------------------------------------
def check_key_shift():
    """Adding one vector u to every key adds c = scale*q.u to every score: out unchanged, lse += c."""
    Hq, Hkv, L = 4, 2, 29
    q = small_ints(16, 0, -3, 3, 1, 1, Hq, D)
    k = small_ints(16, 1, -4, 4, L, Hkv, D)
    u = small_ints(16, 3, -3, 3, 1, Hkv, D)
    v = rnd(16, 2, L, Hkv, D)
    scale = 1.0 / 64.0                                    # keeps the scores O(1) for integer inputs
    k2 = f32_to_bf16((bf16_to_f32(k) + bf16_to_f32(u)).astype(np.float32))
    np.testing.assert_array_equal(f64(k2), f64(k) + f64(u))          # the shifted keys are exact in bf16
    out1, lse1 = oracle.attn(q, [k], [v], [L], scale)
    out2, lse2 = oracle.attn(q, [k2], [v], [L], scale)
    np.testing.assert_allclose(out2, out1, rtol=0, atol=1e-13)
    for h in range(Hq):
        c = scale * float(np.dot(f64(q[0, 0, h]), f64(u[0, h // 2])))
        assert abs((lse2[0, 0, h] - lse1[0, 0, h]) - c) < 1e-12
    assert np.max(np.abs(lse2 - lse1)) > 0.05            # the shift is not vacuous


# 7 ---------------------------------------------------------------------------------------
def check_causal_equals_sequential():
    """A block of T new tokens with the in-block causal mask equals T single-token calls whose
    kv_len grows by one each: token t sees the prefix and new tokens 0..t."""
    B, T, Hq, Hkv = 2, 4, 4, 2
    lens = [21, 9]
    q = rnd(17, 0, B, T, Hq, D)
    ks = [rnd(17, 1 + 2 * b, lens[b], Hkv, D) for b in range(B)]
    vs = [rnd(17, 2 + 2 * b, lens[b], Hkv, D) for b in range(B)]
    out, lse = oracle.attn(q, ks, vs, lens, SCALE)
    for t in range(T):
        lens_t = [L - T + t + 1 for L in lens]
        o1, l1 = oracle.attn(q[:, t:t + 1], ks, vs, lens_t, SCALE)
        np.testing.assert_allclose(out[:, t], o1[:, 0], rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[:, t], l1[:, 0], rtol=0, atol=1e-13)
    # and the mask matters: the last token's row differs from the first token's
    assert np.max(np.abs(lse[:, 0] - lse[:, T - 1])) > 1e-3


# 8 ---------------------------------------------------------------------------------------
def check_merge_closed_forms():
    """The aggregation formula against hand-worked cases and scipy's logsumexp."""
    rng_o = f64(rnd(18, 0, 3, 5, D))
    # one part: identity
    o, l = oracle.merge(rng_o[:1], np.array([[0.3, -1.0, 2.0, 0.0, 5.0]]))
    np.testing.assert_array_equal(o, rng_o[0])
    np.testing.assert_array_equal(l, [0.3, -1.0, 2.0, 0.0, 5.0])
    # two parts of equal lse: plain average, lse + ln 2
    ls = np.array([[1.5] * 5, [1.5] * 5])
    o, l = oracle.merge(rng_o[:2], ls)
    np.testing.assert_allclose(o, 0.5 * (rng_o[0] + rng_o[1]), rtol=0, atol=1e-15)
    np.testing.assert_allclose(l, 1.5 + math.log(2.0), rtol=0, atol=1e-15)
    # weights ratio e^1 : 1 for a lse gap of 1
    ls = np.array([[1.0] * 5, [0.0] * 5])
    o, l = oracle.merge(rng_o[:2], ls)
    w0 = math.e / (math.e + 1.0)
    np.testing.assert_allclose(o, w0 * rng_o[0] + (1 - w0) * rng_o[1], rtol=0, atol=1e-15)
    # an empty part (lse = -inf) is ignored, whatever its out holds
    ls = np.array([[0.7] * 5, [-np.inf] * 5, [0.2] * 5])
    parts = rng_o.copy()
    parts[1] = np.nan
    o, l = oracle.merge(parts, ls)
    o2, l2 = oracle.merge(rng_o[[0, 2]], ls[[0, 2]])
    np.testing.assert_array_equal(o, o2)
    np.testing.assert_array_equal(l, l2)
    # general: scipy logsumexp / softmax over the part axis, including huge offsets (no overflow)
    ls = f64(rnd(18, 1, 3, 5)) * 3.0 + 1000.0
    o, l = oracle.merge(rng_o, ls)
    np.testing.assert_allclose(l, logsumexp(ls, axis=0), rtol=0, atol=1e-12)
    w = softmax(ls, axis=0)
    np.testing.assert_allclose(o, np.einsum("sr,srd->rd", w, rng_o), rtol=0, atol=1e-11)   # ulp(1000) ~ 1e-13


def check_split_merge_identity():
    """Attention over [0, L) equals the aggregation of attention over any partition of [0, L)."""
    Hq, Hkv, L = 8, 2, 97
    q, k, v = rnd(19, 0, 1, 1, Hq, D), rnd(19, 1, L, Hkv, D), rnd(19, 2, L, Hkv, D)
    full_o, full_l = oracle.attn(q, [k], [v], [L], SCALE)
    for cuts in ([0, 40, 97], [0, 1, 2, 96, 97], [0, 33, 66, 97]):
        po, pl = [], []
        for a, b in zip(cuts[:-1], cuts[1:]):
            o, l = oracle.attn(q, [k[a:b]], [v[a:b]], [b - a], SCALE)
            po.append(o)
            pl.append(l)
        mo, ml = oracle.merge(np.stack(po), np.stack(pl))
        np.testing.assert_allclose(mo, full_o, rtol=0, atol=1e-13)
        np.testing.assert_allclose(ml, full_l, rtol=0, atol=1e-13)


# 9 ---------------------------------------------------------------------------------------
def check_gqa_equals_mha_on_duplicated_heads():
    """Query head h reads KV head h // G: duplicating each KV head G times and running with
    n_kv_heads = n_q_heads (plain multi-head attention) gives the same rows."""
    B, T, Hq, Hkv = 2, 2, 10, 2
    G = Hq // Hkv
    lens = [13, 30]
    q = rnd(20, 0, B, T, Hq, D)
    ks = [rnd(20, 1 + 2 * b, lens[b], Hkv, D) for b in range(B)]
    vs = [rnd(20, 2 + 2 * b, lens[b], Hkv, D) for b in range(B)]
    o1, l1 = oracle.attn(q, ks, vs, lens, SCALE)
    o2, l2 = oracle.attn(q, [np.repeat(k, G, axis=1) for k in ks], [np.repeat(v, G, axis=1) for v in vs],
                         lens, SCALE)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)
    # heads of different groups do differ
    assert np.max(np.abs(l1[..., 0] - l1[..., G])) > 1e-3


# 10 --------------------------------------------------------------------------------------
def brute_force_row(qrow, K, V, scale):
    """softmax(scale * K q) V for one row in pure Python, with exactly rounded sums."""
    L, Dh, Dv = len(K), len(qrow), len(V[0])
    s = [scale * math.fsum(qrow[d] * K[j][d] for d in range(Dh)) for j in range(L)]
    m = max(s)
    e = [math.exp(x - m) for x in s]
    Z = math.fsum(e)
    out = [math.fsum(e[j] * V[j][d] for j in range(L)) / Z for d in range(Dv)]
    return out, m + math.log(Z)


def check_brute_force_tiny():
    """Pure-Python evaluation of the definition on tiny ragged inputs (GQA, T > 1, D = 4..128)."""
    for (B, T, Hq, Hkv, Dh, lens, seed) in [(2, 1, 4, 2, 4, [3, 8], 30), (2, 3, 6, 3, 16, [5, 3], 31),
                                            (1, 2, 2, 1, 128, [7], 32), (3, 1, 3, 3, 8, [1, 2, 6], 33)]:
        scale = float(np.float32(1.0 / math.sqrt(Dh)))
        q = rnd(seed, 0, B, T, Hq, Dh)
        # K/V buffers longer than kv_len: rows past kv_len must not be read into the result
        ks = [rnd(seed, 1 + 2 * b, lens[b] + 2, Hkv, Dh) for b in range(B)]
        vs = [rnd(seed, 2 + 2 * b, lens[b] + 2, Hkv, Dh) for b in range(B)]
        out, lse = oracle.attn(q, ks, vs, lens, scale)
        G = Hq // Hkv
        for b in range(B):
            Kf, Vf = f64(ks[b]), f64(vs[b])
            for t in range(T):
                Lv = lens[b] - T + t + 1
                for h in range(Hq):
                    g = h // G
                    o, l = brute_force_row(list(f64(q[b, t, h])), Kf[:Lv, g].tolist(), Vf[:Lv, g].tolist(), scale)
                    np.testing.assert_allclose(out[b, t, h], o, rtol=0, atol=1e-14)
                    assert abs(lse[b, t, h] - l) < 1e-14 * max(1.0, abs(l))


# 11 --------------------------------------------------------------------------------------
def check_joint_permutation():
    """Permuting (k_j, v_j) pairs together leaves out and lse unchanged (single new token)."""
    Hq, Hkv, L = 4, 2, 61
    q, k, v = rnd(21, 0, 1, 1, Hq, D), rnd(21, 1, L, Hkv, D), rnd(21, 2, L, Hkv, D)
    perm = np.argsort(f64(rnd(21, 5, L)), kind="stable")
    assert not np.array_equal(perm, np.arange(L))
    o1, l1 = oracle.attn(q, [k], [v], [L], SCALE)
    o2, l2 = oracle.attn(q, [k[perm]], [v[perm]], [L], SCALE)
    np.testing.assert_allclose(o2, o1, rtol=0, atol=1e-13)
    np.testing.assert_allclose(l2, l1, rtol=0, atol=1e-13)
    # permuting V alone does change the result
    o3, _ = oracle.attn(q, [k], [v[perm]], [L], SCALE)
    assert np.max(np.abs(o3 - o1)) > 1e-3


# 12 --------------------------------------------------------------------------------------
def check_against_scipy():
    """numpy matmul + scipy softmax / logsumexp on a ragged GQA batch spanning hundreds of keys."""
    B, T, Hq, Hkv = 3, 2, 8, 2
    G = Hq // Hkv
    lens = [300, 17, 129]
    q = rnd(22, 0, B, T, Hq, D)
    ks = [rnd(22, 1 + 2 * b, lens[b], Hkv, D) for b in range(B)]
    vs = [rnd(22, 2 + 2 * b, lens[b], Hkv, D) for b in range(B)]
    out, lse = oracle.attn(q, ks, vs, lens, SCALE)
    for b in range(B):
        Kf, Vf = f64(ks[b]), f64(vs[b])
        for t in range(T):
            Lv = lens[b] - T + t + 1
            for h in range(Hq):
                s = SCALE * (Kf[:Lv, h // G] @ f64(q[b, t, h]))
                np.testing.assert_allclose(out[b, t, h], softmax(s) @ Vf[:Lv, h // G], rtol=0, atol=1e-13)
                assert abs(lse[b, t, h] - logsumexp(s)) < 1e-12
                w = oracle.attn_weights(q, ks, vs, lens, SCALE, b, t, h)
                np.testing.assert_allclose(w, softmax(s), rtol=0, atol=1e-15)


# 13 --------------------------------------------------------------------------------------
def check_rejects_bad_arguments():
    q, k, v = rnd(23, 0, 1, 2, 4, D), rnd(23, 1, 5, 2, D), rnd(23, 2, 5, 2, D)
    for bad in (lambda: oracle.attn(q, [k], [v], [1], SCALE),               # kv_len < q_len
                lambda: oracle.attn(q[:, :, :3], [k], [v], [5], SCALE)):    # 3 heads over 2 KV heads
        try:
            bad()
        except ValueError:
            continue
        raise AssertionError("oracle accepted an argument its definition does not cover")


# 14 --------------------------------------------------------------------------------------
def check_page_identity():
    """Address -> (page, offset) of section 4.3, against divmod and hand-worked values."""
    page = 2 << 20
    start = 0x7F0000000000
    assert oracle.page_of(start, start, page) == (0, 0)
    assert oracle.page_of(start + page - 1, start, page) == (0, page - 1)
    assert oracle.page_of(start + page, start, page) == (1, 0)
    assert oracle.page_of(start + 5 * page + 2048 * 3 + 16, start, page) == (5, 6160)
    for off in (1, 4097, 123456789, (1 << 27) - 1):
        assert oracle.page_of(start + off, start, page) == divmod(off, page)


# 15 --------------------------------------------------------------------------------------
def check_write_kvcache():
    """Appending q_len new rows at rows [kv_len - q_len, kv_len): numpy slice assignment says the
    same, rows outside the window and other sequences' buffers keep their bytes."""
    B, T, Hkv = 3, 2, 2
    lens = [5, 2, 9]
    ks = [rnd(24, 1 + 2 * b, lens[b] + 3, Hkv, D) for b in range(B)]
    vs = [rnd(24, 2 + 2 * b, lens[b] + 3, Hkv, D) for b in range(B)]
    k_new, v_new = rnd(24, 50, B, T, Hkv, D), rnd(24, 51, B, T, Hkv, D)
    want_k, want_v = [k.copy() for k in ks], [v.copy() for v in vs]
    for b in range(B):
        want_k[b][lens[b] - T:lens[b]] = k_new[b]
        want_v[b][lens[b] - T:lens[b]] = v_new[b]
    oracle.write_kvcache(k_new, v_new, ks, vs, lens)
    for b in range(B):
        np.testing.assert_array_equal(ks[b], want_k[b])
        np.testing.assert_array_equal(vs[b], want_v[b])
    try:
        oracle.write_kvcache(k_new, v_new, ks, vs, [5, 1, 9])      # kv_len < q_len
    except ValueError:
        return
    raise AssertionError("oracle accepted kv_len < q_len for write_kvcache")


# 16 --------------------------------------------------------------------------------------
def check_mla_reduces_to_attention_with_one_shared_kv_head():
    """Latent-KV attention is attention with one KV head whose K is the cached row and whose V is the
    row's first d_v columns: the (separately written) oracle_mla must agree with the pinned
    oracle_attn when d_v = d_qk, and its d_v < d_qk result must be the leading columns of that."""
    B, T, H, Dq, Dv = 2, 2, 6, 128, 64
    lens = [19, 40]
    q = rnd(25, 0, B, T, H, Dq)
    cs = [rnd(25, 1 + b, lens[b] + 2, Dq) for b in range(B)]
    scale = 0.11
    full_o, full_l = oracle.mla(q, cs, lens, Dq, scale)
    ref_o, ref_l = oracle.attn(q, [c[:, None, :] for c in cs], [c[:, None, :] for c in cs], lens, scale)
    np.testing.assert_allclose(full_o, ref_o, rtol=0, atol=1e-13)
    np.testing.assert_allclose(full_l, ref_l, rtol=0, atol=1e-13)
    part_o, part_l = oracle.mla(q, cs, lens, Dv, scale)
    np.testing.assert_array_equal(part_o, full_o[..., :Dv])
    np.testing.assert_array_equal(part_l, full_l)
    # heads differ, and the trailing key columns (the rope part) do matter
    assert np.max(np.abs(full_l[..., 0] - full_l[..., 1])) > 1e-3
    cs2 = [c.copy() for c in cs]
    for c in cs2:
        c[:, Dv:] = 0
    assert np.max(np.abs(oracle.mla(q, cs2, lens, Dv, scale)[1] - part_l)) > 1e-3


def check_mla_brute_force():
    """oracle_mla against the pure-Python fsum evaluation and scipy, MLA-like odd sizes (d_qk = 72, d_v = 64)."""
    B, T, H, Dq, Dv = 2, 3, 4, 72, 64
    lens = [7, 4]
    q = rnd(26, 0, B, T, H, Dq)
    cs = [rnd(26, 1 + b, lens[b] + 1, Dq) for b in range(B)]
    scale = float(np.float32(1.0 / math.sqrt(Dq)))
    out, lse = oracle.mla(q, cs, lens, Dv, scale)
    for b in range(B):
        C = f64(cs[b])
        for t in range(T):
            Lv = lens[b] - T + t + 1
            for h in range(H):
                o, l = brute_force_row(list(f64(q[b, t, h])), C[:Lv].tolist(), C[:Lv, :Dv].tolist(), scale)
                np.testing.assert_allclose(out[b, t, h], o, rtol=0, atol=1e-14)
                assert abs(lse[b, t, h] - l) < 1e-14 * max(1.0, abs(l))
                s_ = scale * (C[:Lv] @ f64(q[b, t, h]))
                np.testing.assert_allclose(out[b, t, h], softmax(s_) @ C[:Lv, :Dv], rtol=0, atol=1e-13)


ALL_CHECKS = [check_single_key, check_identical_keys, check_weights_sum_to_one, check_zero_query,
              check_dominant_key, check_key_shift, check_causal_equals_sequential, check_merge_closed_forms,
              check_split_merge_identity, check_gqa_equals_mha_on_duplicated_heads, check_brute_force_tiny,
              check_joint_permutation, check_against_scipy, check_rejects_bad_arguments, check_page_identity, check_write_kvcache,
              check_mla_reduces_to_attention_with_one_shared_kv_head, check_mla_brute_force]
