"""Pins for the SparF (Algorithm 1) oracle: special cases that reduce to the dense
definition, a brute-force second implementation, invariants of the selection
and of the output, and planted mistakes.  No GPU."""
import math

import numpy as np
import pytest

from oracle import decode_attention as dense
from oracle import sparf_attention as sparf


def rng(seed):
    return np.random.default_rng(seed)


def f16(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float16))


def draw(seed, S=60, D=16):
    r = rng(seed)
    return f16(r.normal(size=D)), f16(r.normal(size=(S, D))), f16(r.normal(size=(S, D)))


# ---------------------------------------------------------------- reduces to the dense definition
@pytest.mark.parametrize("r,l", [(1, 0), (4, 3), (16, 60), (7, 1)])
def test_selecting_every_row_gives_dense_attention(r, l):
    q, K, V = draw(1)
    res = sparf.sparf_one(q, K, V, 0.25, r=r, k=60, l=l)
    want, _, _ = dense.attend_one(q, K, V, 0.25)
    np.testing.assert_allclose(res["out"], want, rtol=0, atol=1e-13)
    assert abs(res["kept_mass"] - 1.0) < 1e-13 and len(res["kept_rows"]) == 60


def test_all_components_give_exact_scores_and_exact_top_k():
    q, K, V = draw(2, S=80, D=8)
    res = sparf.sparf_one(q, K, V, 0.3, r=8, k=10, l=0)
    _, _, w = dense.attend_one(q, K, V, 0.3)
    np.testing.assert_allclose(res["approx_weights"], w, rtol=0, atol=1e-14)
    assert set(res["kept_rows"]) == set(np.argsort(-w)[:10])
    assert abs(res["kept_mass"] - np.sort(w)[-10:].sum()) < 1e-14


# ---------------------------------------------------------------- brute force, written a second way
def brute(q, K, V, scale, r, k, l):
    S, D = K.shape
    qf = [float(x) for x in q]
    sc = float(np.float32(scale))
    dims = sorted(sorted(range(D), key=lambda d: (-abs(qf[d]), d))[:r])
    rho = sum(abs(qf[d]) for d in dims) / sum(abs(x) for x in qf)
    lg = [sum(qf[d] * float(K[t, d]) for d in dims) * sc / math.sqrt(rho) for t in range(S)]
    mx = max(lg)
    e = [math.exp(x - mx) for x in lg]
    z = sum(e)
    shat = [x / z for x in e]
    boosted = [shat[t] + (1.0 if t >= S - l else 0.0) for t in range(S)]
    rows = sorted(sorted(range(S), key=lambda t: (-boosted[t], t))[:k])
    alpha = sum(shat[t] for t in rows)
    full = [sc * sum(qf[d] * float(K[t, d]) for d in range(D)) for t in rows]
    mx = max(full)
    e = [math.exp(x - mx) for x in full]
    z = sum(e)
    vbar = [sum(float(V[t, d]) for t in range(S)) / S for d in range(D)]
    out = [alpha * sum(e[i] / z * float(V[t, d]) for i, t in enumerate(rows)) + (1 - alpha) * vbar[d]
           for d in range(D)]
    return np.array(out), rows, alpha, dims


@pytest.mark.parametrize("S,D,r,k,l,seed", [(7, 4, 2, 3, 1, 0), (12, 6, 3, 5, 2, 1), (9, 5, 5, 4, 0, 2),
                                            (10, 4, 1, 10, 3, 3), (6, 3, 2, 1, 1, 4)])
def test_brute_force_tiny(S, D, r, k, l, seed):
    q, K, V = draw(seed + 10, S, D)
    res = sparf.sparf_one(q, K, V, 0.5, r, k, l)
    out, rows, alpha, dims = brute(q, K, V, 0.5, r, k, l)
    assert list(res["kept_dims"]) == dims and list(res["kept_rows"]) == rows
    assert abs(res["kept_mass"] - alpha) < 1e-14
    np.testing.assert_allclose(res["out"], out, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- temperature of the approximate softmax
def test_temperature_with_equal_magnitudes_is_sqrt_r():
    """|q| constant: the r kept components carry r/D of the 1-norm, so the
    temperature sqrt(d_h * r/D) equals sqrt(r), the usual one for an r-dim dot."""
    r_ = rng(5)
    D, S, r = 16, 40, 4
    q = f16(r_.choice([-1.0, 1.0], size=D) * 0.5)
    K, V = f16(r_.normal(size=(S, D))), f16(r_.normal(size=(S, D)))
    res = sparf.sparf_one(q, K, V, 1.0 / math.sqrt(D), r, 5, 0)
    dims = res["kept_dims"]
    assert list(dims) == [0, 1, 2, 3]                      # ties towards the lower index
    lg = K[:, dims].astype(np.float64) @ q[dims].astype(np.float64) / math.sqrt(r)
    np.testing.assert_allclose(res["approx_weights"], sparf.softmax(lg), rtol=0, atol=1e-7)


def test_components_are_chosen_by_magnitude_not_sign():
    q = f16([0.1, -5.0, 0.2, 3.0, -0.3, 0.05])
    K, V = f16(rng(6).normal(size=(9, 6))), f16(rng(7).normal(size=(9, 6)))
    assert list(sparf.sparf_one(q, K, V, 0.4, 2, 3, 0)["kept_dims"]) == [1, 3]


# ---------------------------------------------------------------- selection and kept mass
@pytest.mark.parametrize("l", [0, 1, 5, 8])
def test_most_recent_rows_are_always_selected(l):
    q, K, V = draw(8, S=50, D=8)
    K[-8:] = f16(-4.0 * q)                                   # make the recent rows the weakest
    res = sparf.sparf_one(q, K, V, 0.5, r=4, k=8, l=l)
    assert set(range(50 - l, 50)) <= set(res["kept_rows"]) and len(res["kept_rows"]) == 8
    if l == 0:
        assert not set(range(42, 50)) & set(res["kept_rows"])


def test_alpha_is_the_selected_mass_and_grows_with_k():
    q, K, V = draw(9, S=64, D=16)
    prev = 0.0
    for k in [1, 4, 16, 40, 64]:
        res = sparf.sparf_one(q, K, V, 0.3, r=6, k=k, l=1)
        assert 0.0 < res["kept_mass"] <= 1.0 + 1e-15
        assert res["kept_mass"] > prev - 1e-15
        assert abs(res["kept_mass"] - res["approx_weights"][res["kept_rows"]].sum()) < 1e-15
        prev = res["kept_mass"]
    assert abs(prev - 1.0) < 1e-13


def test_two_step_page_load_recovers_exactly_the_selection():
    """The algorithm's second page-wise load: fetching whole n-row pages that hold a selected row and then
    filtering inside the page yields the selected rows and nothing else."""
    q, K, V = draw(10, S=100, D=8)
    res = sparf.sparf_one(q, K, V, 0.5, r=3, k=12, l=2)
    for n in (4, 16):
        pages = sparf.pages_touched(res["kept_rows"], n)
        fetched = np.concatenate([np.arange(p * n, min((p + 1) * n, 100)) for p in pages])
        keep = np.zeros(100, bool)
        keep[res["kept_rows"]] = True
        assert list(fetched[keep[fetched]]) == list(res["kept_rows"])
        assert len(pages) <= 12 and len(fetched) >= 12


# ---------------------------------------------------------------- output: the blend
def test_constant_v_passes_through():
    q, K, _ = draw(11)
    V = np.full((60, 16), 0.75, np.float16)
    for r, k, l in [(2, 5, 1), (16, 1, 0), (1, 30, 30)]:
        np.testing.assert_allclose(sparf.sparf_one(q, K, V, 0.2, r, k, l)["out"], 0.75, atol=1e-14)


def test_output_is_a_convex_combination():
    q, K, V = draw(12, S=70, D=8)
    res = sparf.sparf_one(q, K, V, 0.6, r=3, k=9, l=2)
    V64 = V.astype(np.float64)
    assert (res["out"] <= V64.max(axis=0) + 1e-12).all() and (res["out"] >= V64.min(axis=0) - 1e-12).all()
    # and exactly alpha * (attention over the selected rows alone) + (1 - alpha) * mean of V
    sub, _, _ = dense.attend_one(q, K[res["kept_rows"]], V[res["kept_rows"]], 0.6)
    want = res["kept_mass"] * sub + (1 - res["kept_mass"]) * V64.mean(axis=0)
    np.testing.assert_allclose(res["out"], want, rtol=0, atol=1e-13)


def test_dominant_key_is_found_through_the_kept_components():
    r_ = rng(13)
    D, S = 32, 200
    q = f16(r_.normal(size=D))
    K, V = f16(0.3 * r_.normal(size=(S, D))), f16(r_.normal(size=(S, D)))
    K[77] = f16(6.0 * q)
    res = sparf.sparf_one(q, K, V, 1.0, r=8, k=4, l=1)
    assert 77 in res["kept_rows"] and res["kept_mass"] > 1 - 1e-6
    np.testing.assert_allclose(res["out"], V[77].astype(np.float64), rtol=0, atol=1e-4)


def test_helpers_on_their_own():
    """The pieces sparf_one is made of, each against a value worked out by hand."""
    # magnitudes 5, 4, 3, 3: the tie between components 2 and 3 goes to the lower index
    assert list(sparf.kept_components(np.array([3.0, -5.0, 3.0, 4.0, 0.5]), 3)) == [0, 1, 3]
    # all components kept: plain softmax of scale * K q (the temperature correction is 1)
    K = np.array([[1.0, 0.0], [0.0, 2.0], [1.0, 1.0]])
    q = np.array([2.0, -1.0])
    logits, w = sparf.approximate_weights(q, K, np.array([0, 1]), 0.5)
    np.testing.assert_allclose(logits, [1.0, -1.0, 0.5], atol=1e-15)
    np.testing.assert_allclose(w, np.exp([1.0, -1.0, 0.5]) / np.exp([1.0, -1.0, 0.5]).sum(), atol=1e-15)
    # one of two components kept, |q_kept|_1 / |q|_1 = 2/3: logits = scale * sqrt(3/2) * K[:, 0] * q[0]
    logits, _ = sparf.approximate_weights(q, K, np.array([0]), 0.5)
    np.testing.assert_allclose(logits, 0.5 * math.sqrt(1.5) * np.array([2.0, 0.0, 2.0]), atol=1e-15)
    # three of five positions kept, the most recent two forced in: the best of the other three joins them
    assert list(sparf.kept_positions(np.array([0.1, 0.5, 0.3, 0.05, 0.05]), 3, 2)) == [1, 3, 4]
    assert list(sparf.kept_positions(np.array([0.1, 0.5, 0.3, 0.05, 0.05]), 2, 0)) == [1, 2]
    # kept mass 0.8, attention over the two kept rows with equal scores = their mean
    V = np.array([[1.0, 1.0], [3.0, 5.0], [9.0, 9.0]])
    out, mass, exact = sparf.blend(np.zeros(2), K, V, 1.0, np.array([0.5, 0.3, 0.2]), [0, 1], np.array([10.0, 20.0]))
    assert mass == 0.8 and list(exact) == [0.5, 0.5]
    np.testing.assert_allclose(out, 0.8 * np.array([2.0, 3.0]) + 0.2 * np.array([10.0, 20.0]), atol=1e-15)


def test_finish_from_selection_matches_the_full_run():
    q, K, V = draw(14)
    res = sparf.sparf_one(q, K, V, 0.25, 5, 9, 2)
    out, alpha = sparf.finish_from_selection(q, K, V, 0.25, res["approx_weights"], res["kept_rows"], res["mean_v"])
    assert np.array_equal(out, res["out"]) and alpha == res["kept_mass"]


def test_batch_form_and_group_mapping():
    r_ = rng(15)
    B, Hkv, G, cap, D = 2, 2, 3, 40, 8
    q = f16(r_.normal(size=(B, Hkv * G, D)))
    K, V = f16(r_.normal(size=(B, Hkv, cap, D))), f16(r_.normal(size=(B, Hkv, cap, D)))
    lens = np.array([33, 0], np.int32)
    out, alpha, sel = sparf.decode(q, K, V, lens, 0.4, 3, 6, 1)
    assert np.array_equal(out[1], np.zeros((Hkv * G, D))) and (alpha[1] == 0).all()
    for h in range(Hkv * G):
        one = sparf.sparf_one(q[0, h], K[0, h // G, :33], V[0, h // G, :33], 0.4, 3, 6, 1)
        assert np.array_equal(out[0, h], one["out"]) and list(sel[0][h]) == list(one["kept_rows"])


def test_one_eighth_of_the_dense_bytes():
    """r = d_h/8 components and k = S/16 rows read one eighth of what dense reads
    (the compression ratio the paper evaluates, Sec. VI-B)."""
    S, D = 4096, 128
    assert sparf.bytes_moved(S, D, r=16, k=256) * 8 == dense.decode_kv_read_bytes([S], 1, D)


# ---------------------------------------------------------------- planted mistakes
def mutant(name):
    def run(q, K, V, scale, r, k, l):
        q64, K64, V64 = (np.asarray(x, np.float64) for x in (q, K, V))
        S, D = K64.shape
        sc = float(np.float32(scale))
        dims = sparf.argtopk(q64 if name == "signed_topr" else np.abs(q64), r)
        rho = np.abs(q64[dims]).sum() / np.abs(q64).sum()
        temp = 1.0 if name == "no_temperature" else 1.0 / math.sqrt(rho)
        s_hat = sparf.softmax(K64[:, dims] @ q64[dims] * sc * temp)
        m = np.zeros(S)
        if name != "l_unused":
            m[S - min(l, k):] = 1.0
        if name == "oldest_not_recent":
            m = m[::-1].copy()
        rows = sparf.argtopk(s_hat + m, k)
        alpha = 1.0 if name == "alpha_one" else s_hat[rows].sum()
        s = sparf.softmax(sc * (K64[rows] @ q64))
        vbar = np.zeros(D) if name == "no_vbar" else V64.mean(axis=0)
        if name == "vbar_of_selected":
            vbar = V64[rows].mean(axis=0)
        return alpha * (s @ V64[rows]) + (1 - alpha) * vbar, rows, alpha
    return run


@pytest.mark.parametrize("name", ["signed_topr", "no_temperature", "l_unused", "oldest_not_recent",
                                  "alpha_one", "no_vbar", "vbar_of_selected"])
def test_planted_mistakes_differ_from_the_oracle(name):
    """Each mutant of the algorithm disagrees with the oracle on at least one of the
    pinned situations above (so the pins would catch it in the oracle)."""
    run = mutant(name)
    caught = False
    for seed, (S, D, r, k, l) in enumerate([(12, 6, 3, 5, 2), (50, 8, 4, 8, 5), (60, 16, 6, 9, 1)]):
        q, K, V = draw(seed + 10, S, D)
        if seed == 1:
            K[-8:] = f16(-4.0 * q)
        want_out, want_rows, want_alpha, _ = brute(q, K, V, 0.5, r, k, l)
        out, rows, alpha = run(q, K, V, 0.5, r, k, l)
        if list(rows) != want_rows or abs(alpha - want_alpha) > 1e-9 or np.abs(out - want_out).max() > 1e-9:
            caught = True
    assert caught
