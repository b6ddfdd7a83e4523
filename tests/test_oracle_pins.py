"""Pins for the CPU oracle: closed forms, invariants, brute force, library special
cases and the sizes the paper prints.  No GPU, no HIP library.  Every pin runs on
both forms of the oracle (numpy and plain C)."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import c_oracle, decode_attention as np_oracle

IMPLS = {"numpy": np_oracle, "c": c_oracle}


@pytest.fixture(params=sorted(IMPLS))
def impl(request):
    return IMPLS[request.param]


def rng(seed):
    return np.random.default_rng(seed)


def f16(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float16))


def one_head(impl, q, K, V, scale, L=None):
    """Single sequence, single head through the batch entry point."""
    L = K.shape[0] if L is None else L
    out, lse = impl.decode(f16(q)[None, None], f16(K)[None, None], f16(V)[None, None],
                           np.array([L], np.int32), scale)
    return out[0, 0], lse[0, 0]


# ---------------------------------------------------------------- fp16 widening
def test_c_half_widening_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([c_oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------- brute force
def brute_force(q, K, V, scale):
    """Second way: exact rational dot products, math.exp, explicit weights."""
    L, D = K.shape
    sc = Fraction(float(np.float32(scale)))
    s = [float(sc * sum(Fraction(float(q[d])) * Fraction(float(K[t, d])) for d in range(D)))
         for t in range(L)]
    e = [math.exp(x - max(s)) for x in s]
    Z = math.fsum(e)
    out = [math.fsum(e[t] / Z * float(V[t, d]) for t in range(L)) for d in range(V.shape[1])]
    return np.array(out), max(s) + math.log(Z)


@pytest.mark.parametrize("L,D,seed", [(1, 1, 0), (2, 3, 1), (5, 4, 2), (4, 2, 3), (3, 4, 4)])
def test_brute_force_tiny(impl, L, D, seed):
    r = rng(seed)
    q, K, V = f16(r.normal(size=D)), f16(r.normal(size=(L, D))), f16(r.normal(size=(L, D)))
    scale = 1.0 / math.sqrt(D)
    out, lse = one_head(impl, q, K, V, scale)
    want, want_lse = brute_force(q, K, V, scale)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-14)
    assert abs(lse - want_lse) < 1e-13


def test_brute_force_batch_heads(impl):
    """B = 2, Hq = 2 (one KV head each): indexing of batch and head."""
    r = rng(11)
    B, H, D = 2, 2, 4
    Ls = [5, 3]
    q = f16(r.normal(size=(B, H, D)))
    K = f16(r.normal(size=(B, H, 5, D)))
    V = f16(r.normal(size=(B, H, 5, D)))
    out, lse = impl.decode(q, K, V, np.array(Ls, np.int32), 0.5)
    for b in range(B):
        for h in range(H):
            want, wl = brute_force(q[b, h], K[b, h, :Ls[b]], V[b, h, :Ls[b]], 0.5)
            np.testing.assert_allclose(out[b, h], want, rtol=0, atol=1e-14)
            assert abs(lse[b, h] - wl) < 1e-13


# ---------------------------------------------------------------- library special cases
@pytest.mark.parametrize("L,D", [(257, 64), (1000, 128)])
def test_matches_stock_softmax_matmul(impl, L, D):
    r = rng(5)
    q, K, V = f16(r.normal(size=D)), f16(r.normal(size=(L, D))), f16(r.normal(size=(L, D)))
    scale = np.float32(1.0 / math.sqrt(D))
    out, lse = one_head(impl, q, K, V, scale)
    s = float(scale) * np.einsum("td,d->t", K.astype(np.float64), q.astype(np.float64))
    want = scipy.special.softmax(s) @ V.astype(np.float64)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-13)
    assert abs(lse - scipy.special.logsumexp(s)) < 1e-12


def test_matches_torch_sdpa_fp64(impl):
    r = rng(6)
    B, H, L, D = 2, 3, 77, 64
    q = f16(r.normal(size=(B, H, D)))
    K = f16(r.normal(size=(B, H, L + 9, D)))
    V = f16(r.normal(size=(B, H, L + 9, D)))
    scale = 1.0 / math.sqrt(D)
    out, _ = impl.decode(q, K, V, np.full(B, L, np.int32), scale)
    tq = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    tk = torch.from_numpy(K[:, :, :L].astype(np.float64))
    tv = torch.from_numpy(V[:, :, :L].astype(np.float64))
    want = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, scale=float(np.float32(scale)))[:, :, 0, :].numpy()
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- closed forms
def test_identical_keys_give_mean_of_v(impl):
    r = rng(7)
    L, D = 37, 16
    q = f16(r.normal(size=D))
    K = np.repeat(f16(r.normal(size=(1, D))), L, axis=0)
    V = f16(r.normal(size=(L, D)))
    out, lse = one_head(impl, q, K, V, 0.25)
    np.testing.assert_allclose(out, V.astype(np.float64).mean(axis=0), rtol=0, atol=1e-14)
    s0 = 0.25 * float(K[0].astype(np.float64) @ q.astype(np.float64))
    assert abs(lse - (s0 + math.log(L))) < 1e-13


def test_zero_scale_gives_mean_of_v(impl):
    r = rng(8)
    L, D = 20, 8
    q, K, V = f16(r.normal(size=D)), f16(r.normal(size=(L, D))), f16(r.normal(size=(L, D)))
    out, lse = one_head(impl, q, K, V, 0.0)
    np.testing.assert_allclose(out, V.astype(np.float64).mean(axis=0), rtol=0, atol=1e-14)
    assert abs(lse - math.log(L)) < 1e-14


def test_dominant_score_selects_its_row(impl):
    r = rng(9)
    L, D, j = 50, 32, 17
    K = f16(r.normal(size=(L, D)))
    V = f16(r.normal(size=(L, D)))
    q = f16(4.0 * K[j].astype(np.float64))
    s = K.astype(np.float64) @ q.astype(np.float64)
    gap = s[j] - np.delete(s, j).max()
    assert gap > 30
    out, _ = one_head(impl, q, K, V, 1.0)
    bound = (L - 1) * math.exp(-gap) * 2 * np.abs(V).max()
    np.testing.assert_allclose(out, V[j].astype(np.float64), rtol=0, atol=bound + 1e-15)


def test_constant_v_and_weights_sum_to_one(impl):
    r = rng(10)
    L, D = 333, 8
    q, K = f16(r.normal(size=D)), f16(r.normal(size=(L, D)))
    out, _ = one_head(impl, q, K, np.ones((L, D)), 0.7)
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=1e-14)


def test_numpy_weights_sum_to_one_and_are_positive():
    r = rng(12)
    q, K, V = f16(r.normal(size=16)), f16(r.normal(size=(99, 16))), f16(r.normal(size=(99, 16)))
    _, _, w = np_oracle.attend_one(q, K, V, 0.3)
    assert abs(w.sum() - 1.0) < 1e-15 and (w > 0).all()


def test_single_position_returns_v0_exactly(impl):
    r = rng(13)
    D = 128
    q, K, V = f16(r.normal(size=D)), f16(r.normal(size=(4, D))), f16(r.normal(size=(4, D)))
    out, lse = one_head(impl, q, K, V, 0.1, L=1)
    assert np.array_equal(out, V[0].astype(np.float64))
    want = float(np.float32(0.1)) * float(K[0].astype(np.float64) @ q.astype(np.float64))
    assert abs(lse - want) < 1e-14


# ---------------------------------------------------------------- invariants
def test_permutation_of_positions(impl):
    r = rng(14)
    L, D = 64, 32
    q, K, V = f16(r.normal(size=D)), f16(r.normal(size=(L, D))), f16(r.normal(size=(L, D)))
    p = r.permutation(L)
    a, la = one_head(impl, q, K, V, 0.2)
    b, lb = one_head(impl, q, K[p], V[p], 0.2)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)
    assert abs(la - lb) < 1e-13


def test_rows_behind_the_length_are_ignored_bitwise(impl):
    r = rng(15)
    L, cap, D = 21, 40, 16
    q, K, V = f16(r.normal(size=D)), f16(r.normal(size=(cap, D))), f16(r.normal(size=(cap, D)))
    a, la = one_head(impl, q, K, V, 0.3, L=L)
    K2, V2 = K.copy(), V.copy()
    K2[L:], V2[L:] = np.nan, np.inf
    b, lb = one_head(impl, q, K2, V2, 0.3, L=L)
    assert np.array_equal(a, b) and la == lb
    c, _ = one_head(impl, q, K[:L], V[:L], 0.3)
    assert np.array_equal(a, c)


def test_linear_in_v(impl):
    r = rng(16)
    L, D = 30, 8
    q, K = f16(r.normal(size=D)), f16(r.normal(size=(L, D)))
    V1 = r.integers(-8, 9, size=(L, D)).astype(np.float64)
    V2 = r.integers(-8, 9, size=(L, D)).astype(np.float64)
    o1, _ = one_head(impl, q, K, V1, 0.4)
    o2, _ = one_head(impl, q, K, V2, 0.4)
    o12, _ = one_head(impl, q, K, V1 + V2, 0.4)
    o3, _ = one_head(impl, q, K, 4.0 * V1, 0.4)
    np.testing.assert_allclose(o12, o1 + o2, rtol=0, atol=1e-13)
    np.testing.assert_allclose(o3, 4.0 * o1, rtol=0, atol=1e-13)


def test_key_shift_orthogonal_to_query(impl):
    """Adding to every key a vector u with q.u = c shifts all scores by the same
    amount: the output stays, the lse moves by scale * c.  Small integers keep
    every fp16 value and dot product exact."""
    r = rng(17)
    L, D = 25, 8
    q = r.integers(-3, 4, size=D).astype(np.float64)
    q[0] = 1.0
    K = r.integers(-4, 5, size=(L, D)).astype(np.float64)
    V = f16(r.normal(size=(L, D)))
    u = r.integers(-3, 4, size=D).astype(np.float64)
    c = 5.0
    u[0] += c - q @ u          # now q.u = c exactly (q[0] = 1)
    assert q @ u == c
    a, la = one_head(impl, q, K, V, 0.125)
    b, lb = one_head(impl, q, K + u, V, 0.125)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)
    assert abs((lb - la) - 0.125 * c) < 1e-13


def test_heads_are_independent(impl):
    r = rng(18)
    B, H, L, D = 2, 3, 19, 8
    q, K, V = f16(r.normal(size=(B, H, D))), f16(r.normal(size=(B, H, L, D))), \
        f16(r.normal(size=(B, H, L, D)))
    lens = np.array([L, L - 4], np.int32)
    a, _ = impl.decode(q, K, V, lens, 0.3)
    q2, K2, V2 = q.copy(), K.copy(), V.copy()
    q2[:, 1], K2[:, 1], V2[:, 1] = 1.0, 2.0, 3.0
    b, _ = impl.decode(q2, K2, V2, lens, 0.3)
    assert np.array_equal(a[:, [0, 2]], b[:, [0, 2]])


# ---------------------------------------------------------------- segment identity (merge)
@pytest.mark.parametrize("cuts", [(0, 9, 40), (0, 1, 39, 40), (0, 13, 13, 27, 40), (0, 40)])
def test_segments_merge_to_whole(impl, cuts):
    r = rng(19)
    L, D = 40, 16
    q, K, V = f16(r.normal(size=D)), f16(3 * r.normal(size=(L, D))), f16(r.normal(size=(L, D)))
    whole, lse = one_head(impl, q, K, V, 0.35)
    outs, lses = [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        if a == b:
            outs.append(np.zeros(D))
            lses.append(-np.inf)
        else:
            o, l = one_head(impl, q, K[a:b], V[a:b], 0.35)
            outs.append(o)
            lses.append(l)
    merged, mlse = np_oracle.merge_segments(outs, lses)
    np.testing.assert_allclose(merged, whole, rtol=0, atol=1e-14)
    assert abs(mlse - lse) < 1e-13


def test_merge_all_empty():
    out, lse = np_oracle.merge_segments(np.zeros((3, 4)), np.full(3, -np.inf))
    assert np.array_equal(out, np.zeros(4)) and lse == -np.inf


# ---------------------------------------------------------------- grouped queries, paging
def test_grouped_queries_equal_replicated_kv(impl):
    r = rng(20)
    B, Hkv, G, L, D = 2, 2, 4, 23, 16
    q = f16(r.normal(size=(B, Hkv * G, D)))
    K, V = f16(r.normal(size=(B, Hkv, L, D))), f16(r.normal(size=(B, Hkv, L, D)))
    lens = np.array([L, 7], np.int32)
    a, la = impl.decode(q, K, V, lens, 0.25)
    Kr, Vr = np.repeat(K, G, axis=1), np.repeat(V, G, axis=1)
    b, lb = impl.decode(q, f16(Kr), f16(Vr), lens, 0.25)
    assert np.array_equal(a, b) and np.array_equal(la, lb)
    # the head of group g of KV head hk is hk*G + g: changing KV head 1 moves heads 4..7 only
    K2 = K.copy()
    K2[:, 1] += 1
    c, _ = impl.decode(q, K2, V, lens, 0.25)
    assert np.array_equal(a[:, :G], c[:, :G]) and not np.array_equal(a[:, G:], c[:, G:])


def make_paged(r, B, Hkv, D, lens, ps):
    max_pages = (max(lens) + ps - 1) // ps
    need = [(L + ps - 1) // ps for L in lens]
    P = sum(need) + 2
    kp, vp = f16(r.normal(size=(P, Hkv, ps, D))), f16(r.normal(size=(P, Hkv, ps, D)))
    perm = r.permutation(P).astype(np.int32)
    table = np.full((B, max_pages), -1, np.int32)
    at = 0
    for b in range(B):
        table[b, :need[b]] = perm[at:at + need[b]]
        at += need[b]
    return kp, vp, table


def test_paged_equals_gathered_contiguous(impl):
    r = rng(21)
    B, Hkv, G, D, ps = 3, 2, 2, 8, 4
    lens = [9, 4, 14]
    kp, vp, table = make_paged(r, B, Hkv, D, lens, ps)
    cap = table.shape[1] * ps
    Kc, Vc = np.zeros((B, Hkv, cap, D), np.float16), np.zeros((B, Hkv, cap, D), np.float16)
    for b in range(B):
        for t in range(lens[b]):
            Kc[b, :, t] = kp[table[b, t // ps], :, t % ps]
            Vc[b, :, t] = vp[table[b, t // ps], :, t % ps]
    q = f16(r.normal(size=(B, Hkv * G, D)))
    a, la = impl.decode(q, kp, vp, np.array(lens, np.int32), 0.3, page_table=table)
    b_, lb = impl.decode(q, Kc, Vc, np.array(lens, np.int32), 0.3)
    assert np.array_equal(a, b_) and np.array_equal(la, lb)


def test_empty_sequence(impl):
    r = rng(22)
    q, K, V = f16(r.normal(size=(2, 1, 4))), f16(r.normal(size=(2, 1, 6, 4))), \
        f16(r.normal(size=(2, 1, 6, 4)))
    out, lse = impl.decode(q, K, V, np.array([0, 6], np.int32), 0.5)
    assert np.array_equal(out[0], np.zeros((1, 4))) and lse[0, 0] == -np.inf
    assert np.isfinite(out[1]).all() and np.isfinite(lse[1, 0])


def test_length_is_cut_off_at_capacity(impl):
    r = rng(23)
    q, K, V = f16(r.normal(size=(1, 1, 4))), f16(r.normal(size=(1, 1, 6, 4))), \
        f16(r.normal(size=(1, 1, 6, 4)))
    a, _ = impl.decode(q, K, V, np.array([6], np.int32), 0.5)
    b, _ = impl.decode(q, K, V, np.array([60], np.int32), 0.5)
    assert np.array_equal(a, b)


# ---------------------------------------------------------------- append
def bits(a):
    return a.view(np.uint16)


def test_append_contiguous_bit_exact(impl):
    r = rng(24)
    B, Hkv, cap, D = 3, 2, 10, 8
    K = r.integers(0, 65536, size=(B, Hkv, cap, D)).astype(np.uint16).view(np.float16)
    V = r.integers(0, 65536, size=(B, Hkv, cap, D)).astype(np.uint16).view(np.float16)
    kn = r.integers(0, 65536, size=(B, Hkv, D)).astype(np.uint16).view(np.float16)  # NaN payloads too
    vn = r.integers(0, 65536, size=(B, Hkv, D)).astype(np.uint16).view(np.float16)
    lens = np.array([1, 10, 6], np.int32)
    K0, V0 = K.copy(), V.copy()
    impl.kv_append(K, V, kn, vn, lens)
    changed = np.zeros((B, Hkv, cap, D), bool)
    for b in range(B):
        t = lens[b] - 1
        assert np.array_equal(bits(K[b, :, t]), bits(kn[b]))
        assert np.array_equal(bits(V[b, :, t]), bits(vn[b]))
        changed[b, :, t] = True
    assert np.array_equal(bits(K)[~changed], bits(K0)[~changed])
    assert np.array_equal(bits(V)[~changed], bits(V0)[~changed])


def test_append_out_of_range_is_a_no_op(impl):
    r = rng(25)
    K, V = f16(r.normal(size=(3, 1, 4, 2))), f16(r.normal(size=(3, 1, 4, 2)))
    K0, V0 = K.copy(), V.copy()
    impl.kv_append(K, V, f16(np.ones((3, 1, 2))), f16(np.ones((3, 1, 2))),
                   np.array([0, 5, -3], np.int32))
    assert np.array_equal(bits(K), bits(K0)) and np.array_equal(bits(V), bits(V0))


def test_append_paged_lands_behind_the_page_table(impl):
    r = rng(26)
    B, Hkv, D, ps = 3, 2, 4, 4
    lens = [9, 4, 13]
    kp, vp, table = make_paged(r, B, Hkv, D, lens, ps)
    kn, vn = f16(r.normal(size=(B, Hkv, D))), f16(r.normal(size=(B, Hkv, D)))
    k0, v0 = kp.copy(), vp.copy()
    impl.kv_append(kp, vp, kn, vn, np.array(lens, np.int32), page_table=table)
    changed = np.zeros(kp.shape, bool)
    for b in range(B):
        t = lens[b] - 1
        page = table[b, t // ps]
        assert np.array_equal(bits(kp[page, :, t % ps]), bits(kn[b]))
        assert np.array_equal(bits(vp[page, :, t % ps]), bits(vn[b]))
        changed[page, :, t % ps] = True
    assert np.array_equal(bits(kp)[~changed], bits(k0)[~changed])
    assert np.array_equal(bits(vp)[~changed], bits(v0)[~changed])


def test_bulk_write_equals_one_append_per_row():
    """kv_write is by definition kv_append applied row by row (checked against the
    plain-C append too), for both layouts, with runs that start anywhere, overrun
    the capacity or are empty."""
    r = rng(40)
    B, Hkv, D, N, ps = 3, 2, 8, 7, 4
    k_src = r.integers(0, 65536, size=(B, Hkv, N, D)).astype(np.uint16).view(np.float16)
    v_src = r.integers(0, 65536, size=(B, Hkv, N, D)).astype(np.uint16).view(np.float16)
    start, count = np.array([0, 5, 9], np.int32), np.array([7, 0, 6], np.int32)
    for paged in (False, True):
        if paged:
            K, V, table = make_paged(r, B, Hkv, D, [12, 12, 12], ps)
        else:
            K, V, table = f16(r.normal(size=(B, Hkv, 12, D))), f16(r.normal(size=(B, Hkv, 12, D))), None
        for appender in (np_oracle.kv_append, c_oracle.kv_append):
            Ka, Va, Kb, Vb = K.copy(), V.copy(), K.copy(), V.copy()
            np_oracle.kv_write(Ka, Va, k_src, v_src, start, count, table)
            for i in range(N):
                lens = np.where(i < count, start + i + 1, 0).astype(np.int32)   # 0: skipped
                appender(Kb, Vb, np.ascontiguousarray(k_src[:, :, i]), np.ascontiguousarray(v_src[:, :, i]),
                         lens, table)
            assert np.array_equal(bits(Ka), bits(Kb)) and np.array_equal(bits(Va), bits(Vb))
            assert not np.array_equal(bits(Ka), bits(K))
            # sequence 1 (count 0) untouched; sequence 2 wrote rows 9..11 only (capacity 12)
            if not paged:
                assert np.array_equal(bits(Ka[1]), bits(K[1]))
                assert np.array_equal(bits(Ka[2, :, :9]), bits(K[2, :, :9]))
                assert np.array_equal(bits(Ka[2, :, 9:12]), bits(k_src[2, :, :3]))


def test_append_then_decode_sees_the_new_token(impl):
    """A new key far along q dominates: the output becomes the new v."""
    r = rng(27)
    D, cap = 16, 12
    q = f16(r.normal(size=(1, 1, D)))
    K, V = f16(0.1 * r.normal(size=(1, 1, cap, D))), f16(r.normal(size=(1, 1, cap, D)))
    kn = f16(40.0 * q / np.linalg.norm(q.astype(np.float64)))
    vn = f16(r.normal(size=(1, 1, D)))
    lens = np.array([8], np.int32)
    impl.kv_append(K, V, kn.reshape(1, 1, D), vn, lens)
    out, _ = impl.decode(q, K, V, lens, 1.0)
    np.testing.assert_allclose(out[0, 0], vn[0, 0].astype(np.float64), rtol=0, atol=1e-9)


# ---------------------------------------------------------------- the two forms agree
def test_numpy_and_c_forms_agree():
    r = rng(28)
    B, Hkv, G, L, D = 2, 2, 2, 300, 128
    q = f16(r.normal(size=(B, Hkv * G, D)))
    K, V = f16(r.normal(size=(B, Hkv, L, D))), f16(r.normal(size=(B, Hkv, L, D)))
    lens = np.array([L, 123], np.int32)
    a, la = np_oracle.decode(q, K, V, lens, 0.0884)
    b, lb = c_oracle.decode(q, K, V, lens, 0.0884, nthreads=2)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)
    np.testing.assert_allclose(la, lb, rtol=0, atol=1e-12)


def test_c_pair_sampling_leaves_other_rows_alone():
    r = rng(29)
    q, K, V = f16(r.normal(size=(2, 4, 8))), f16(r.normal(size=(2, 4, 5, 8))), \
        f16(r.normal(size=(2, 4, 5, 8)))
    full, _ = c_oracle.decode(q, K, V, np.array([5, 5], np.int32), 0.3)
    part, _ = c_oracle.decode(q, K, V, np.array([5, 5], np.int32), 0.3, pair_stride=3, pair_offset=1)
    flat_full, flat_part = full.reshape(8, 8), part.reshape(8, 8)
    for p in range(8):
        if p % 3 == 1:
            assert np.array_equal(flat_part[p], flat_full[p])
        else:
            assert np.isnan(flat_part[p]).all()


# ---------------------------------------------------------------- sizes the paper prints
def golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_sizes.txt")
    rows = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, value, tol, _ = [x.strip() for x in line.split("|")]
        rows[name] = (float(value), float(tol))
    return rows


def test_kv_sizes_printed_in_the_paper():
    g = golden()
    layers, hidden = 40, 5120
    v, tol = g["kv_bytes_13b_b128_s2048"]
    got = np_oracle.kv_cache_bytes(128, 2048, layers, hidden)
    assert got == 2 * 2 * 128 * 2048 * layers * hidden
    assert abs(got - v) / v <= tol
    v, tol = g["kv_bytes_13b_b32_s4096"]
    got = np_oracle.kv_cache_bytes(32, 4096, layers, hidden)
    assert abs(got - v) / v <= tol
    v, tol = g["kv_over_weights_13b"]
    assert abs(got / (13e9 * 2) - v) / v <= tol


def test_group_and_traffic_arithmetic():
    g = golden()
    # one decode step of one (sequence, head) reads 2*L rows of D fp16
    assert np_oracle.decode_kv_read_bytes([1], 1, 128) == 2 * g["row_bytes"][0]
    assert np_oracle.decode_kv_read_bytes([16], 1, 128) == 2 * g["group_bytes"][0]
    s = 4096
    vectors_moved = 4                       # q, k, v in; out back
    cache_vectors = np_oracle.decode_kv_read_bytes([s], 1, 128) // 256
    assert cache_vectors / vectors_moved == g["pcie_ratio_s4096"][0]
    # the 13B-shaped 4K config: 16 x 40 heads x 4096 positions
    assert np_oracle.decode_kv_read_bytes([4096] * 16, 40, 128) == 1_342_177_280
