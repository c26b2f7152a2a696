"""Pins of the CPU oracle against things other than itself: hand-worked fixtures, closed forms,
invariants, NumPy library routines and exact-rational brute force on tiny inputs.  CPU only."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle


# ----------------------------------------------------------------------------- helpers (NumPy only)
def dense_importance(q, k, scale):
    """Library-routine form of Sec. 3.2: dense masked softmax, column sums, head mean (fp64)."""
    q = q.astype(np.float64)
    k = k.astype(np.float64)
    B, L, H, N, D = q.shape
    Hkv = k.shape[2]
    kk = np.repeat(k, H // Hkv, axis=2)  # GQA == MHA with every KV head repeated
    s = np.einsum("blhmd,blhnd->blhmn", q, kk) * scale.astype(np.float64)[None, :, None, None, None]
    mask = np.tril(np.ones((N, N), dtype=bool))
    s = np.where(mask, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    a = e / e.sum(axis=-1, keepdims=True)
    return a.sum(axis=-2).mean(axis=2)


def rng_qk(seed, B, L, H, Hkv, N, D):
    r = np.random.default_rng(seed)
    q = r.standard_normal((B, L, H, N, D)).astype(np.float32)
    k = r.standard_normal((B, L, Hkv, N, D)).astype(np.float32)
    sc = r.uniform(0.1, 1.0, L).astype(np.float32)
    return q, k, sc


# ----------------------------------------------------------------------------- stage 1: importance
def test_importance_hand_worked_fixture(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "importance_two_tokens.json")))
    sub = lambda x: np.array(json.loads(json.dumps(x).replace('"ln2"', repr(g["ln2"]))
                                        .replace('"ln3"', repr(g["ln3"]))), dtype=np.float32)
    c = g["case_one_head"]
    imp = oracle.importance(sub(c["q"])[None, None, None], sub(c["k"])[None, None, None],
                            np.ones(1, np.float32))
    np.testing.assert_allclose(imp[0, 0], c["importance"], rtol=1e-6)
    c = g["case_two_heads"]
    imp = oracle.importance(sub(c["q"])[None, None], sub(c["k"])[None, None], np.ones(1, np.float32))
    np.testing.assert_allclose(imp[0, 0], c["importance"], rtol=1e-6)


def test_importance_zero_logits_is_harmonic_tail():
    # scale = 0 (or q = 0) makes every causal row uniform: a[m][n] = 1/(m+1), so
    # I[n] = sum_{m>=n} 1/(m+1) = H_N - H_n (harmonic numbers, 0-based n).
    N = 37
    q, k, sc = rng_qk(1, 1, 2, 3, 3, N, 8)
    Hn = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, N + 1))])
    want = Hn[N] - Hn[:N]
    imp = oracle.importance(q, k, np.zeros(2, np.float32))
    np.testing.assert_allclose(imp[0, 0], want, rtol=1e-6)
    imp = oracle.importance(np.zeros_like(q), k, sc)
    np.testing.assert_allclose(imp[0, 1], want, rtol=1e-6)


def test_importance_invariants():
    q, k, sc = rng_qk(2, 2, 3, 4, 4, 50, 16)
    imp = oracle.importance(q, k, sc)
    N = 50
    np.testing.assert_allclose(imp.sum(-1), N, rtol=1e-5)  # every softmax row sums to one
    assert (imp[..., 0] >= 1.0 - 1e-6).all()  # row 0 attends only to position 0
    assert (imp[..., N - 1] <= 1.0 + 1e-6).all()  # only the last row can see the last key
    assert (imp > 0).all()


def test_importance_one_hot_limit():
    # a huge logit on key 0 for every query: all rows m >= 1 put ~all mass on column 0
    N, D = 12, 4
    q = np.ones((1, 1, 1, N, D), np.float32)
    k = np.zeros((1, 1, 1, N, D), np.float32)
    k[..., 0, :] = 50.0
    imp = oracle.importance(q, k, np.ones(1, np.float32))[0, 0]
    assert abs(imp[0] - N) < 1e-6 and np.all(imp[1:] < 1e-6)


@pytest.mark.parametrize("H,Hkv", [(4, 4), (4, 2), (6, 1)])
def test_importance_matches_dense_numpy(H, Hkv):
    q, k, sc = rng_qk(3 + H + Hkv, 2, 2, H, Hkv, 33, 8)
    imp, lse = oracle.importance(q, k, sc, want_lse=True)
    np.testing.assert_allclose(imp, dense_importance(q, k, sc), rtol=2e-6)
    # lse of the last row against a direct evaluation
    kk = np.repeat(k, H // Hkv, axis=2).astype(np.float64)
    s_last = np.einsum("blhd,blhnd->blhn", q[:, :, :, -1].astype(np.float64), kk) * sc[None, :, None, None]
    np.testing.assert_allclose(lse[..., -1], np.log(np.exp(s_last).sum(-1)), rtol=1e-9)


def test_importance_gqa_equals_repeated_mha():
    q, k, sc = rng_qk(9, 1, 2, 4, 2, 20, 8)
    a = oracle.importance(q, k, sc)
    b = oracle.importance(q, np.repeat(k, 2, axis=2), sc)
    np.testing.assert_array_equal(a, b)


def test_importance_is_not_transposed():
    # key 0 huge for the LAST query only: column 0 gains one unit from row N-1, nothing else moves
    N, D = 6, 2
    q = np.zeros((1, 1, 1, N, D), np.float32)
    q[..., N - 1, :] = 10.0
    k = np.zeros((1, 1, 1, N, D), np.float32)
    k[..., 0, :] = 10.0
    imp = oracle.importance(q, k, np.ones(1, np.float32))[0, 0]
    Hn = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, N + 1))])
    base = (Hn[N] - Hn[:N]) - 1.0 / N  # rows 0..N-2 uniform
    want = base.copy()
    want[0] += 1.0
    np.testing.assert_allclose(imp, want, atol=1e-6)


# ----------------------------------------------------------------------------- stage 2: sort + prefix
def test_sort_matches_stable_argsort_with_ties():
    r = np.random.default_rng(5)
    for N in (1, 2, 7, 8, 64, 333):
        imp = (r.integers(0, 5, N) / 4.0).astype(np.float32)  # many ties
        st, order, cum, prefix = oracle.sort_prefix_layer(imp)
        assert st == 0 or imp.sum() == 0
        if st == 0:
            np.testing.assert_array_equal(order, np.argsort(-imp, kind="stable"))


def test_sort_negative_zero_is_zero():
    imp = np.array([0.0, -0.0, 1.0, -0.0, 0.0], np.float32)
    st, order, cum, prefix = oracle.sort_prefix_layer(imp)
    assert st == 0
    np.testing.assert_array_equal(order, [2, 0, 1, 3, 4])


def test_prefix_exact_integer_cumsum():
    r = np.random.default_rng(6)
    N = 500
    imp = r.random(N).astype(np.float32) * 3
    st, order, cum, prefix = oracle.sort_prefix_layer(imp)
    assert st == 0
    # weights are floor(imp * 2^36) exactly (Python ints, any summation order)
    w = [int(math.floor(float(imp[i]) * 2.0 ** 36)) for i in order]
    tot = 0
    for j in range(N):
        tot += w[j]
        assert int(cum[j]) == tot
    assert sum(reversed(w)) == int(cum[-1])
    assert np.all(np.diff(cum.astype(np.int64)) >= 0)
    assert prefix[-1] == np.float32(1.0)
    ref = np.cumsum(np.sort(imp.astype(np.float64))[::-1]) / imp.astype(np.float64).sum()
    assert np.max(np.abs(prefix - ref)) <= N * 2.0 ** -36 + 2.0 ** -23


def test_prefix_weights_round_down_for_tiny_importance():
    """Importance below 2^-13 has a fractional part after the scaling by 2^36 (an fp32 value v has
    v*2^36 integral only from 2^-13 upwards), so these weights tell floor from round-to-nearest
    and from ceil: expected sums are exact Python integers."""
    vals = [3 * 2.0 ** -38, 2.0 ** -37, 1.0, 5 * 2.0 ** -38, 7 * 2.0 ** -39, 2.0 ** -36 + 2.0 ** -37]
    imp = np.array(vals, np.float32)
    assert [float(x) for x in imp] == vals  # all exactly representable
    st, order, cum, prefix = oracle.sort_prefix_layer(imp)
    assert st == 0
    exact = [Fraction(v) * 2 ** 36 for v in vals]              # 3/4, 1/2, 2^36, 5/4, 7/8, 3/2
    assert [e.denominator for e in exact] == [4, 2, 1, 4, 8, 2]
    w_floor = {i: e.numerator // e.denominator for i, e in enumerate(exact)}
    assert [w_floor[i] for i in range(6)] == [0, 0, 2 ** 36, 1, 0, 1]
    np.testing.assert_array_equal(order, [2, 5, 3, 4, 0, 1])   # 2^36, 3/2, 5/4, 7/8, 3/4, 1/2
    want, tot = [], 0
    for i in order:
        tot += w_floor[int(i)]
        want.append(tot)
    assert [int(c) for c in cum] == want == [2 ** 36, 2 ** 36 + 1, 2 ** 36 + 2, 2 ** 36 + 2, 2 ** 36 + 2, 2 ** 36 + 2]
    # a layer made only of such values: floor gives 0, 0, 1 -> sum 1 (rounding would give 3)
    st, order, cum, prefix = oracle.sort_prefix_layer(np.array([3 * 2.0 ** -38, 2.0 ** -37, 2.0 ** -36], np.float32))
    assert st == 0 and [int(c) for c in cum] == [1, 1, 1] and order.tolist() == [2, 0, 1]


def test_status_bits():
    assert oracle.sort_prefix_layer(np.array([1, np.nan, 2], np.float32))[0] & oracle.NONFINITE
    assert oracle.sort_prefix_layer(np.array([1, np.inf, 2], np.float32))[0] & oracle.NONFINITE
    assert oracle.sort_prefix_layer(np.array([1, -1e-3, 2], np.float32))[0] & oracle.NEGATIVE
    assert oracle.sort_prefix_layer(np.zeros(4, np.float32))[0] == oracle.ZERO_LAYER
    assert oracle.sort_prefix_layer(np.full(4, 1e-12, np.float32))[0] == oracle.ZERO_LAYER
    assert oracle.sort_prefix_layer(np.full(4, 2.0 ** 17, np.float32))[0] & oracle.RANGE
    sel = oracle.select(np.array([[[1, 2, 3], [0, 0, 0]], [[1, 2, 3], [3, 2, 1]]], np.float32), 4)
    assert sel["status"].tolist() == [oracle.ZERO_LAYER, 0]
    assert sel["lengths"][0].tolist() == [0, 0] and sel["lengths"][1].sum() == 4


# ----------------------------------------------------------------------------- stage 3: search
def test_algorithm1_hand_trace(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "algo1_hand_trace.json")))
    imp = np.array(g["importance"], np.float32)[None]
    for c in g["cases"]:
        sel = oracle.select(imp, c["budget_tokens"], c["tol_tokens"], c["max_iters"], bool(c["fixup"]))
        assert sel["order"][0].tolist() == g["order"], c
        np.testing.assert_array_equal(sel["prefix"][0], np.array(g["prefix"], np.float32))
        assert sel["lengths"][0].tolist() == c["lengths"], c
        assert sel["p"][0] == c["p"], c
        assert sel["iters"][0] == c["iters"], c
        assert sel["raw_total"][0] == c["raw_total"], c
        assert sel["status"][0] == 0


def exact_layer_len(cum_l, p: Fraction):
    """min{k >= 1 : C_k / T >= p} in exact rational arithmetic; p >= 1 -> N."""
    N = len(cum_l)
    if p >= 1:
        return N
    T = int(cum_l[-1])
    for k in range(1, N + 1):
        if Fraction(int(cum_l[k - 1]), T) >= p:
            return k
    return N


def exact_algorithm1(cum, budget, tol, max_iters):
    """Algorithm 1 in exact rational arithmetic (dyadic p is exact)."""
    L, N = cum.shape
    p1, p2 = Fraction(0), Fraction(1)
    p, K, lens, it_done = None, None, None, 0
    for it in range(1, max_iters + 1):
        p = (p1 + p2) / 2
        lens = [exact_layer_len(cum[l], p) for l in range(L)]
        K = sum(lens)
        it_done = it
        d = K - budget
        if abs(d) <= tol:
            break
        if d < 0:
            p1 = p
        else:
            p2 = p
    return lens, p, it_done, K


@pytest.mark.parametrize("seed", range(6))
def test_search_matches_exact_rational_bisection(seed):
    # small dyadic importances: every product p*T is exact in fp64 for <= 20 iterations, so the
    # fp64 comparison of the oracle and the rational one must agree bit for bit
    r = np.random.default_rng(100 + seed)
    L, N = int(r.integers(1, 6)), int(r.integers(2, 24))
    imp = (r.integers(0, 64, (1, L, N)) / 16.0).astype(np.float32)
    imp[:, :, 0] += 1.0
    for budget in sorted(set(int(x) for x in r.integers(L + 1, L * N, 5))):
        for tol in (0, 2):
            sel = oracle.select(imp, budget, tol, 20, fixup=False)
            lens, p, it, K = exact_algorithm1(sel["cum"][0], budget, tol, 20)
            assert sel["lengths"][0].tolist() == lens
            assert Fraction(float(sel["p"][0])) == p
            assert sel["iters"][0] == it and sel["raw_total"][0] == K


def test_total_is_monotone_in_p_and_hits_every_breakpoint():
    r = np.random.default_rng(7)
    L, N = 3, 9
    imp = (r.integers(1, 32, (L, N)) / 8.0).astype(np.float32)
    cum = np.stack([oracle.sort_prefix_layer(imp[l])[2] for l in range(L)])
    # evaluate K(p) through a 1-iteration "search" at chosen p by exploiting the bracket:
    # K(p) for any p equals the exact rational count; check monotonicity over all breakpoints
    pts = sorted({Fraction(int(c), int(cum[l, -1])) for l in range(L) for c in cum[l]})
    mids = [(a + b) / 2 for a, b in zip([Fraction(0)] + pts[:-1], pts)]
    Ks = [sum(exact_layer_len(cum[l], p) for l in range(L)) for p in sorted(pts + mids)]
    assert Ks == sorted(Ks) and Ks[0] == L and Ks[-1] == L * N
    # every reachable total is found exactly by the oracle's bisection (delta == 0)
    for K in sorted(set(Ks)):
        if L < K < L * N:
            lens, p, it, raw = oracle.search(cum, K, 0, 64, fixup=False)
            assert raw == K and lens.sum() == K
            assert sum(exact_layer_len(cum[l], Fraction(p)) for l in range(L)) == K


def test_geometric_importance_closed_form():
    # I_n ~ rho^n gives P^k = (1-rho^k)/(1-rho^N), hence k(p) = ceil(ln(1-p(1-rho^N))/ln rho).
    N, rhos = 200, [0.90, 0.95, 0.98]
    imp = np.stack([rho ** np.arange(N) for rho in rhos])
    imp = (imp / imp.sum(-1, keepdims=True) * N).astype(np.float32)[None]
    for steps in (1, 2, 3, 4, 5):
        sel = oracle.select(imp, budget_tokens=3 * N - 1, max_iters=steps, fixup=False)
        p = sel["p"][0]
        for l, rho in enumerate(rhos):
            x = math.log(1 - p * (1 - rho ** N)) / math.log(rho)
            if abs(x - round(x)) > 1e-3:  # away from a breakpoint of the rounded weights
                assert sel["lengths"][0, l] == math.ceil(x)


def test_identical_layers_get_identical_ratios():
    # the uniform configuration R_l = r is recovered when all layers share one distribution
    r = np.random.default_rng(8)
    N, L = 64, 5
    row = r.random(N).astype(np.float32) + 0.01
    imp = np.tile(row, (1, L, 1))
    sel = oracle.select(imp, budget_tokens=L * 16, fixup=True)
    assert sel["lengths"][0].tolist() == [16] * L
    sel = oracle.select(imp, budget_tokens=L * 16 + 2, fixup=True)  # unreachable: all layers jump together
    assert sel["lengths"][0].sum() == L * 16 + 2
    assert sel["lengths"][0].max() - sel["lengths"][0].min() <= 1


@pytest.mark.parametrize("seed", range(4))
def test_search_postconditions_and_fixup(seed):
    r = np.random.default_rng(200 + seed)
    B, L, N = 2, 6, 97
    imp = np.exp(r.standard_normal((B, L, N)) * r.uniform(0.5, 3, (B, L, 1))).astype(np.float32)
    for budget in (L + 1, L * N // 5, L * N // 2, L * N - 1):
        for tol in (0, 9):
            raw = oracle.select(imp, budget, tol, 64, fixup=False)
            fix = oracle.select(imp, budget, tol, 64, fixup=True)
            for b in range(B):
                hit = abs(raw["raw_total"][b] - budget) <= tol
                assert hit or raw["iters"][b] == 64 or raw["iters"][b] >= 50  # tolerance, cap or stall
                assert raw["lengths"][b].sum() == raw["raw_total"][b]
                assert fix["lengths"][b].sum() == budget
                assert fix["lengths"][b].min() >= 1 and fix["lengths"][b].max() <= N
                if raw["raw_total"][b] == budget:
                    np.testing.assert_array_equal(raw["lengths"][b], fix["lengths"][b])
                # brute-force the rescale rule
                K = int(raw["raw_total"][b])
                if K != budget:
                    num = [int(k) * budget for k in raw["lengths"][b]]
                    base = [min(max(x // K, 1), N) for x in num]
                    rem = [x % K for x in num]
                    d = budget - sum(base)
                    idx = sorted(range(L), key=(lambda l: (-rem[l], l)) if d > 0 else (lambda l: (rem[l], l)))
                    i = 0
                    while d != 0:
                        l = idx[i % L]
                        if d > 0 and base[l] < N:
                            base[l] += 1
                            d -= 1
                        elif d < 0 and base[l] > 1:
                            base[l] -= 1
                            d += 1
                        i += 1
                    assert fix["lengths"][b].tolist() == base


def test_iteration_counts_in_the_papers_range():
    # Sanity only (Tab. "Robustness to delta": 7.8 .. 11.5 average steps at r = 50% for thresholds
    # 0.0125 .. 0.1 in ratio-sum units): a threshold of floor(delta*N) tokens stops in ~4..14 steps.
    from pkv_workloads import synthetic_importance
    imp = synthetic_importance(8, 32, 680, seed=1).numpy()
    for thr in (0.0125, 0.1):
        sel = oracle.select(imp, budget_tokens=32 * 680 // 2, tol_tokens=int(thr * 680), fixup=True)
        assert 3 <= sel["iters"].mean() <= 16


# ----------------------------------------------------------------------------- stage 4: compaction + decode
def make_cache_case(seed, B=2, L=3, Hkv=2, N=19, D=8, cap=3, frac=0.4):
    r = np.random.default_rng(seed)
    k = r.standard_normal((B, L, Hkv, N, D)).astype(np.float32)
    v = r.standard_normal((B, L, Hkv, N, D)).astype(np.float32)
    imp = r.random((B, L, N)).astype(np.float32) + 0.01
    sel = oracle.select(imp, max(L + 1, int(frac * L * N)))
    cache = oracle.compact(k, v, sel["order"], sel["lengths"], cap)
    return k, v, sel, cache


def test_compaction_is_fancy_indexing():
    k, v, sel, cache = make_cache_case(11)
    B, L = sel["lengths"].shape
    off = 0
    for b in range(B):
        for l in range(L):
            n = sel["lengths"][b, l]
            assert cache["seg_off"][b, l] == off and cache["caps"][b, l] == n + 3
            off += n + 3
            kp = oracle.segment(cache, "kept_pos", b, l)[:n]
            assert np.all(np.diff(kp) > 0)
            assert set(kp.tolist()) == set(sel["order"][b, l, :n].tolist())
            np.testing.assert_array_equal(oracle.segment(cache, "kc", b, l)[:, :n], k[b, l][:, kp])
            np.testing.assert_array_equal(oracle.segment(cache, "vc", b, l)[:, :n], v[b, l][:, kp])
            assert np.isnan(oracle.segment(cache, "kc", b, l)[:, n:]).all()
    np.testing.assert_array_equal(cache["lens"], sel["lengths"])


def test_compaction_full_budget_is_identity():
    k, v, sel, cache = make_cache_case(12, frac=1.0, cap=0)
    assert (sel["lengths"] == k.shape[3]).all() and (sel["p"] == 1.0).all()
    np.testing.assert_array_equal(cache["kc"].reshape(k.shape), k)
    np.testing.assert_array_equal(cache["vc"].reshape(v.shape), v)


def dense_attention(q, K, V, scale):
    """q [H,D], K/V [H,n,D] fp64 -> softmax(scale q K^T) V, the textbook definition."""
    s = np.einsum("hd,hnd->hn", q, K) * scale
    s -= s.max(-1, keepdims=True)
    e = np.exp(s)
    return np.einsum("hn,hnd->hd", e / e.sum(-1, keepdims=True), V)


def test_decode_matches_dense_attention_over_kept_set_with_append():
    k, v, sel, cache = make_cache_case(13, Hkv=2, cap=2)
    B, L, Hkv, N, D = k.shape
    H = 4
    r = np.random.default_rng(14)
    sc = r.uniform(0.1, 1, L).astype(np.float32)
    keptK = {(b, l): k[b, l][:, np.sort(sel["order"][b, l, :sel["lengths"][b, l]])].astype(np.float64)
             for b in range(B) for l in range(L)}
    keptV = {(b, l): v[b, l][:, np.sort(sel["order"][b, l, :sel["lengths"][b, l]])].astype(np.float64)
             for b in range(B) for l in range(L)}
    for step in range(2):
        q = r.standard_normal((B, L, H, D)).astype(np.float32)
        kn = r.standard_normal((B, L, Hkv, D)).astype(np.float32)
        vn = r.standard_normal((B, L, Hkv, D)).astype(np.float32)
        out = oracle.decode_attn(cache, q, kn, vn, sc)
        for b in range(B):
            for l in range(L):
                keptK[b, l] = np.concatenate([keptK[b, l], kn[b, l][:, None].astype(np.float64)], 1)
                keptV[b, l] = np.concatenate([keptV[b, l], vn[b, l][:, None].astype(np.float64)], 1)
                want = dense_attention(q[b, l].astype(np.float64), np.repeat(keptK[b, l], 2, 0),
                                       np.repeat(keptV[b, l], 2, 0), float(sc[l]))
                np.testing.assert_allclose(out[b, l], want, rtol=1e-5, atol=1e-6)
        assert (cache["lens"] == sel["lengths"] + step + 1).all()
    with pytest.raises(ValueError):
        oracle.decode_attn(cache, q, kn, vn, sc)  # capacity of 2 is used up


def test_decode_full_budget_reproduces_full_cache_attention():
    k, v, sel, cache = make_cache_case(15, frac=1.0, cap=0)
    B, L, Hkv, N, D = k.shape
    r = np.random.default_rng(16)
    q = r.standard_normal((B, L, Hkv, D)).astype(np.float32)
    sc = r.uniform(0.1, 1, L).astype(np.float32)
    out = oracle.decode_attn(cache, q, None, None, sc)
    for b in range(B):
        for l in range(L):
            want = dense_attention(q[b, l].astype(np.float64), k[b, l].astype(np.float64),
                                   v[b, l].astype(np.float64), float(sc[l]))
            np.testing.assert_allclose(out[b, l], want, rtol=1e-5, atol=1e-6)


def test_decode_special_cases():
    k, v, sel, cache = make_cache_case(17, cap=1)
    B, L, Hkv, N, D = k.shape
    r = np.random.default_rng(18)
    q = r.standard_normal((B, L, Hkv, D)).astype(np.float32)
    # scale = 0: uniform weights -> mean of the kept V rows
    out = oracle.decode_attn(cache, q, None, None, np.zeros(L, np.float32))
    for b in range(B):
        for l in range(L):
            n = cache["lens"][b, l]
            np.testing.assert_allclose(out[b, l], oracle.segment(cache, "vc", b, l)[:, :n].mean(1), rtol=1e-5, atol=1e-6)
    # permuting the cache slots does not change the output
    sc = np.full(L, 0.3, np.float32)
    a = oracle.decode_attn(cache, q, None, None, sc)
    for b in range(B):
        for l in range(L):
            n = cache["lens"][b, l]
            perm = r.permutation(n)
            for nm in ("kc", "vc"):
                seg = oracle.segment(cache, nm, b, l)
                seg[:, :n] = seg[:, perm]
    np.testing.assert_allclose(oracle.decode_attn(cache, q, None, None, sc), a, rtol=1e-6, atol=1e-7)
    # a single slot returns its value row; layer range limits the work; bf16 rounding of the output
    one = oracle.compact(k, v, sel["order"], np.ones((B, L), np.int32), 0)
    o = oracle.decode_attn(one, q, None, None, sc, l0=1, l1=2)
    assert np.isnan(o[:, 0]).all() and np.isnan(o[:, 2]).all()
    for b in range(B):
        np.testing.assert_allclose(o[b, 1], oracle.segment(one, "vc", b, 1)[:, 0], rtol=1e-6)
    ob = oracle.decode_attn(cache, q, None, None, sc, out_bf16=True)
    import torch
    np.testing.assert_array_equal(ob, torch.from_numpy(oracle.decode_attn(cache, q, None, None, sc))
                                  .to(torch.bfloat16).float().numpy())


def test_bf16_output_rounds_ties_to_even():
    """A cache of one slot returns its value row exactly (softmax weight 1), so the bf16 rounding of
    the output is seen in isolation: values half way between two bf16 numbers go to the one with the
    even mantissa, whichever side that is, for both signs; non-ties go to the nearest."""
    vals = np.array([1 + 2.0 ** -8,        # tie between 1 and 1+2^-7 -> 1 (even)
                     1 + 3 * 2.0 ** -8,    # tie between 1+2^-7 and 1+2^-6 -> 1+2^-6 (even)
                     -(1 + 2.0 ** -8), -(1 + 3 * 2.0 ** -8),
                     1 + 2.0 ** -8 + 2.0 ** -20,   # just above the tie -> up
                     1 + 3 * 2.0 ** -8 - 2.0 ** -20,  # just below the tie -> down
                     2.0 ** -10 * (1 + 5 * 2.0 ** -8),  # tie at another exponent: 1+2^-6 (even) vs 1+3*2^-7
                     0.0], np.float32)
    want = np.array([1.0, 1 + 2.0 ** -6, -1.0, -(1 + 2.0 ** -6), 1 + 2.0 ** -7, 1 + 2.0 ** -7,
                     2.0 ** -10 * (1 + 2.0 ** -6), 0.0], np.float32)
    D = vals.size
    k = np.ones((1, 1, 1, 1, D), np.float32)
    v = vals.reshape(1, 1, 1, 1, D).copy()
    cache = oracle.compact(k, v, np.zeros((1, 1, 1), np.int32), np.ones((1, 1), np.int32), 0)
    q = np.full((1, 1, 1, D), 0.25, np.float32)
    exact = oracle.decode_attn(cache, q, None, None, np.ones(1, np.float32))
    np.testing.assert_array_equal(exact.reshape(-1), vals)
    got = oracle.decode_attn(cache, q, None, None, np.ones(1, np.float32), out_bf16=True)
    np.testing.assert_array_equal(got.reshape(-1), want)


def test_empty_cache_segment_gives_zero_output():
    k, v, sel, _ = make_cache_case(19)
    B, L = sel["lengths"].shape
    cache = oracle.compact(k, v, sel["order"], np.zeros((B, L), np.int32), 1)
    q = np.ones((B, L, 2, 8), np.float32)
    out = oracle.decode_attn(cache, q, None, None, np.ones(L, np.float32))
    assert (out == 0).all()


def test_importance_row_restriction_keeps_tail_columns_exact():
    q, k, sc = rng_qk(31, 1, 2, 3, 3, 40, 8)
    full = oracle.importance(q, k, sc)
    tail = oracle.importance(q, k, sc, m_lo=25)
    np.testing.assert_array_equal(tail[..., 25:], full[..., 25:])
    assert np.isnan(tail[..., :25]).all()


# ----------------------------------------------------------------------------- offline configuration
def test_offline_config_hand_example_and_invariants():
    # two samples, three layers: totals (6, 3, 3) of 12; budget 8 of L*N = 3*10:
    # 6*8/12 = 4 r0, 3*8/12 = 2 r0, 2 r0 -> exactly (4, 2, 2)
    sl = np.array([[4, 1, 2], [2, 2, 1]], np.int32)
    assert oracle.offline_config(sl, 10, 8).tolist() == [4, 2, 2]
    # budget 10: 6*10/12 = 5 r0, 3*10/12 = 2 r6, 2 r6 -> one token missing, tie on the remainder -> lower layer
    assert oracle.offline_config(sl, 10, 10).tolist() == [5, 3, 2]
    # a single sample that already meets the budget is returned unchanged
    one = np.array([[3, 5, 2]], np.int32)
    assert oracle.offline_config(one, 10, 10).tolist() == [3, 5, 2]
    # clamps
    assert oracle.offline_config(sl, 10, 3).tolist() == [1, 1, 1]
    assert oracle.offline_config(sl, 10, 30).tolist() == [10, 10, 10]
    assert oracle.offline_config(np.zeros((2, 3), np.int32), 10, 8).tolist() == [0, 0, 0]
    r = np.random.default_rng(3)
    for _ in range(20):
        S, L, N = int(r.integers(1, 6)), int(r.integers(2, 9)), int(r.integers(4, 50))
        sl = r.integers(1, N + 1, (S, L)).astype(np.int32)
        budget = int(r.integers(L + 1, L * N))
        out = oracle.offline_config(sl, N, budget)
        assert out.sum() == budget and out.min() >= 1 and out.max() <= N
        # repeating the sample set does not change the configuration (ratios are averaged)
        np.testing.assert_array_equal(oracle.offline_config(np.tile(sl, (3, 1)), N, budget), out)


def test_rank_is_select_without_the_search():
    imp = np.random.default_rng(4).random((2, 3, 17)).astype(np.float32)
    a, b = oracle.rank(imp), oracle.select(imp, 20)
    for k in ("order", "cum", "prefix", "status"):
        np.testing.assert_array_equal(a[k], b[k])


# ------------------------------------------------------ decode-time pruning at a fixed distance
def run_evict(seed, lengths, N, d, T, Hkv=2, H=4, D=8, extra=None):
    """Build a cache with the given per-layer lengths (B = 1) and run T pruning decode steps.
    Returns per-step outputs and the inputs, plus the state after each step."""
    r = np.random.default_rng(seed)
    lengths = np.asarray(lengths, np.int32)[None]
    L = lengths.shape[1]
    k = r.standard_normal((1, L, Hkv, N, D)).astype(np.float32)
    v = r.standard_normal((1, L, Hkv, N, D)).astype(np.float32)
    order = np.stack([r.permutation(N) for _ in range(L)])[None].astype(np.int32)
    cap = d + 1 + (T if extra is None else extra)
    cache = oracle.compact(k, v, order, lengths, cap)
    sc = r.uniform(0.1, 1, L).astype(np.float32)
    q = r.standard_normal((T, 1, L, H, D)).astype(np.float32)
    kn = r.standard_normal((T, 1, L, Hkv, D)).astype(np.float32)
    vn = r.standard_normal((T, 1, L, Hkv, D)).astype(np.float32)
    outs, states = [], []
    for t in range(1, T + 1):
        outs.append(oracle.decode_attn_evict(cache, lengths, q[t - 1], kn[t - 1], vn[t - 1], sc, N, t, d))
        states.append([(int(cache["lens"][0, l]), oracle.segment(cache, "kept_pos", 0, l).copy())
                       for l in range(L)])
    return dict(k=k, v=v, order=order, lengths=lengths, sc=sc, q=q, kn=kn, vn=vn, outs=outs, states=states,
                cache=cache)


def test_evict_hand_trace(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "evict_hand_trace.json")))
    N, d, T = g["N"], g["d"], len(g["target"])
    x = run_evict(31, [g["base_len"]], N, d, T)
    for t in range(1, T + 1):
        perm, kp = x["states"][t - 1][0]
        assert perm == g["permanent_after_step"][t - 1]
        live = sorted(int(p) - N + 1 for p in kp if p >= N)
        assert live == g["live_decode_tokens_after_step"][t - 1]
        assert perm + min(t, d) == max(g["target"][t - 1], g["base_len"] + min(t, d))


@pytest.mark.parametrize("seed,N,d,T", [(1, 16, 1, 40), (2, 16, 3, 60), (3, 33, 8, 120), (4, 7, 2, 50)])
def test_evict_cache_size_closed_form_and_set_invariants(seed, N, d, T):
    """Because the target grows by at most one entry per step, the rule has a closed form: the cache holds
    max(target(t), k_l + min(t, d)) entries after step t.  Besides: the d newest tokens are always live,
    kept prompt entries never leave, a pruned token never returns, survivors keep their decision order,
    and every live slot holds the K/V rows of the position it is labelled with."""
    r = np.random.default_rng(seed)
    L = 5
    lengths = np.concatenate([[0, 1, N], r.integers(1, N + 1, L - 3)])
    x = run_evict(seed + 100, lengths, N, d, T)
    from fractions import Fraction
    for l in range(L):
        kl = int(lengths[l])
        prev_live = None
        for t in range(1, T + 1):
            perm, kp = x["states"][t - 1][l]
            tgt = max(1, int(Fraction(kl * (N + t), N) + Fraction(1, 2)))     # round half up, exactly
            live = [int(p) for p in kp if p >= 0]
            assert len(live) == len(set(live)) == perm + min(t, d) == max(tgt, kl + min(t, d))
            assert set(range(N + t - min(t, d), N + t)) <= set(live)            # the d newest
            assert set(np.sort(x["order"][0, l, :kl]).tolist()) == {p for p in live if p < N}
            assert list(kp[:kl]) == sorted(kp[:kl]) and list(kp[kl:perm]) == sorted(kp[kl:perm])
            if prev_live is not None:
                gone = prev_live - set(live)
                assert len(gone) <= 1 and all(p == N + t - d - 1 for p in gone)  # only the decided token
                assert set(live) - prev_live <= {N + t - 1} | set()              # only the new token enters
            prev_live = set(live)
            if t == T:
                K = oracle.segment(x["cache"], "kc", 0, l)
                V = oracle.segment(x["cache"], "vc", 0, l)
                for slot, p in enumerate(kp):
                    if p < 0:
                        continue
                    wk = x["k"][0, l, :, p] if p < N else x["kn"][p - N, 0, l]
                    wv = x["v"][0, l, :, p] if p < N else x["vn"][p - N, 0, l]
                    np.testing.assert_array_equal(K[:, slot], wk)
                    np.testing.assert_array_equal(V[:, slot], wv)


def test_evict_distance_beyond_horizon_is_plain_append():
    """d >= T: nothing is ever decided, so every step equals the append-only decode step."""
    for N, T, d in ((12, 5, 9), (12, 5, 20)):       # also a distance longer than the prompt
        x = run_evict(41, [3, 7, 12], N, d, T)
        cache = oracle.compact(x["k"], x["v"], x["order"], x["lengths"], T)
        for t in range(T):
            want = oracle.decode_attn(cache, x["q"][t], x["kn"][t], x["vn"][t], x["sc"])
            np.testing.assert_array_equal(x["outs"][t], want)


def attention_over_positions(x, l, t, positions):
    """Dense softmax attention of step t's query over an explicit list of sequence positions."""
    N = x["k"].shape[3]
    K = np.stack([x["k"][0, l, :, p] if p < N else x["kn"][p - N, 0, l] for p in positions], 1)
    V = np.stack([x["v"][0, l, :, p] if p < N else x["vn"][p - N, 0, l] for p in positions], 1)
    H = x["q"].shape[3]
    rep = H // K.shape[0]
    return dense_attention(x["q"][t - 1, 0, l].astype(np.float64), np.repeat(K, rep, 0).astype(np.float64),
                           np.repeat(V, rep, 0).astype(np.float64), float(x["sc"][l]))


def test_evict_full_ratio_keeps_everything_and_tiny_ratio_is_a_sliding_window():
    """R_l = 1: every decided token survives -> full-cache attention over prompt + all decode tokens.
    One kept prompt entry of a long prompt: the target stays at 1, every decided token is pruned ->
    attention over that entry plus a sliding window of the d newest tokens."""
    N, d, T = 40, 3, 12
    x = run_evict(51, [N, 1], N, d, T)
    sink = int(x["order"][0, 1, 0])
    for t in range(1, T + 1):
        full = attention_over_positions(x, 0, t, list(range(N + t)))
        np.testing.assert_allclose(x["outs"][t - 1][0, 0], full, rtol=1e-5, atol=1e-6)
        window = [sink] + list(range(N + t - min(t, d), N + t))
        np.testing.assert_allclose(x["outs"][t - 1][0, 1], attention_over_positions(x, 1, t, window),
                                   rtol=1e-5, atol=1e-6)


def test_evict_general_case_attends_to_exactly_the_live_set():
    N, d, T = 24, 4, 40
    x = run_evict(61, [6, 13, 20], N, d, T)
    for l in range(3):
        for t in (1, 4, 5, 17, 40):
            _, kp = x["states"][t - 1][l]
            live = [int(p) for p in kp if p >= 0]
            np.testing.assert_allclose(x["outs"][t - 1][0, l], attention_over_positions(x, l, t, live),
                                       rtol=1e-5, atol=1e-6)


def test_evict_refuses_bad_capacity_or_distance():
    with pytest.raises(ValueError):
        run_evict(71, [3], 8, 0, 2)                 # distance 0 would decide the token being stored
    with pytest.raises(ValueError):
        run_evict(72, [8], 8, 2, 6, extra=1)        # survivors do not fit in front of the ring
    x = run_evict(73, [3], 8, 2, 6, extra=0)        # R small enough that nothing survives in 6 steps
    assert x["states"][-1][0][0] == 3


# --------------------------------------------------------------- Gini diagnostic and cache merging
def test_gini_matches_mean_absolute_difference_and_closed_forms():
    """G = sum_ij |x_i - x_j| / (2 N sum x) relates to the Lorenz-curve (trapezoid) form by the factor the
    discrete curve carries: G_lorenz = G_mad exactly for the same weights; flat -> 0, one-hot -> (N-1)/N,
    geometric weights have a closed form."""
    from fractions import Fraction
    r = np.random.default_rng(5)
    imp = (r.random((2, 3, 37)) ** 3).astype(np.float32) + 1e-3
    imp[0, 0] = 1.0                       # flat
    imp[0, 1] = 0.0; imp[0, 1, 11] = 2.0  # one-hot
    sel = oracle.rank(imp)
    got = oracle.gini(sel["cum"])
    N = imp.shape[-1]
    for b in range(2):
        for l in range(3):
            w = [int(np.floor(np.float64(x) * 2.0 ** 36)) for x in imp[b, l]]
            tot = sum(w)
            mad = Fraction(sum(abs(a - c) for a in w for c in w), 2 * N * tot)
            assert abs(got[b, l] - float(mad)) < 1e-12
    assert got[0, 0] == 0.0
    assert abs(got[0, 1] - (N - 1) / N) < 1e-15
    # weights 2^-i (exact in fp32 and in the fixed point): sum_k C_k and T in closed form
    n = 20
    geo = (2.0 ** -np.arange(n)).astype(np.float32)[None, None]
    g = oracle.gini(oracle.rank(geo)["cum"])[0, 0]
    T = 2 - 2.0 ** (1 - n)
    S = sum(2 - 2.0 ** (1 - k) for k in range(1, n + 1))
    assert abs(g - (2 * S / T - n - 1) / n) < 1e-14
    # a more concentrated layer has the larger coefficient and, under one shared p, the shorter prefix
    conc = np.stack([np.sort(r.random(64).astype(np.float32) ** 8 + 1e-4)[::-1],
                     np.sort(r.random(64).astype(np.float32) + 0.5)[::-1]])[None]
    s2 = oracle.select(conc, 40)
    g2 = oracle.gini(s2["cum"])[0]
    assert g2[0] > g2[1] and s2["lengths"][0, 0] < s2["lengths"][0, 1]


def test_merge_position_is_nearest_kept_average():
    """Brute force in NumPy: match = argmax of -|m - n| over the kept positions (first maximum = lower
    position on a tie), merged vector = mean of the group; the groups partition all positions, so the
    count-weighted sum of the merged vectors equals the sum of all vectors; a full budget changes nothing."""
    k, v, sel, cache = make_cache_case(91, B=2, L=3, Hkv=2, N=23, D=8, cap=2, frac=0.3)
    before = {n: cache[n].copy() for n in ("kc", "vc")}
    oracle.merge_position(cache, k, v)
    B, L, Hkv, N, D = k.shape
    for b in range(B):
        for l in range(L):
            n = int(sel["lengths"][b, l])
            kp = oracle.segment(cache, "kept_pos", b, l)[:n]
            c = -np.abs(np.arange(N)[:, None] - kp[None, :])
            match = c.argmax(1)                                   # first maximum
            counts = np.bincount(match, minlength=n)
            assert counts.sum() == N and (counts >= 1).all() and (match[kp] == np.arange(n)).all()
            for name, src in (("kc", k), ("vc", v)):
                seg = oracle.segment(cache, name, b, l)
                for j in range(n):
                    want = src[b, l][:, match == j].astype(np.float64).mean(1)
                    np.testing.assert_allclose(seg[:, j], want, rtol=1e-6, atol=1e-7)
                mass = (seg[:, :n].astype(np.float64) * counts[None, :, None]).sum(1)
                np.testing.assert_allclose(mass, src[b, l].astype(np.float64).sum(1), rtol=1e-5, atol=1e-5)
                assert np.isnan(seg[:, n:]).all()                  # the decode slots stay untouched
    # tie: position 2 between kept 1 and 3 goes to 1
    k1 = np.arange(5, dtype=np.float32).reshape(1, 1, 1, 5, 1)
    order = np.array([[[1, 3, 0, 2, 4]]], np.int32)
    c1 = oracle.compact(k1, k1, order, np.array([[2]], np.int32), 0)
    oracle.merge_position(c1, k1, k1)
    np.testing.assert_array_equal(oracle.segment(c1, "kc", 0, 0)[0, :, 0], [1.0, 3.5])   # {0,1,2} and {3,4}
    # full budget: every group is a single position
    kf, vf, self_, cf = make_cache_case(92, frac=1.0, cap=0)
    ref = cf["kc"].copy()
    oracle.merge_position(cf, kf, vf)
    np.testing.assert_array_equal(cf["kc"], ref)
    # bf16 storage: merged vectors are representable in bfloat16
    kb, vb, selb, cb = make_cache_case(93, frac=0.4)
    oracle.merge_position(cb, kb, vb, storage_bf16=True)
    kc = cb["kc"][~np.isnan(cb["kc"])]
    assert ((kc.view(np.uint32) & 0xffff) == 0).all()


def test_merge_feature_is_cosine_argmax_average():
    """Brute force in NumPy (normalised rows, one matrix product, first maximum); keys and values are matched
    on their own; the groups partition all positions (mass conservation); cosine is scale-free."""
    k, v, sel, cache = make_cache_case(94, B=2, L=2, Hkv=2, N=29, D=8, cap=2, frac=0.3)
    r = np.random.default_rng(95)
    k *= r.uniform(0.1, 30.0, k.shape[:-1] + (1,)).astype(np.float32)       # norms all over the place
    cache = oracle.compact(k, v, sel["order"], sel["lengths"], 2)
    mk, mv = oracle.merge_feature(cache, k, v)
    mk2, best = oracle.feature_match(cache, k)
    np.testing.assert_array_equal(mk, mk2)
    np.testing.assert_allclose(oracle.match_cosine(cache, k, mk), best, rtol=0, atol=0)
    B, L, Hkv, N, D = k.shape
    assert not np.array_equal(mk, mv)
    for b in range(B):
        for l in range(L):
            n = int(sel["lengths"][b, l])
            kp = oracle.segment(cache, "kept_pos", b, l)[:n]
            pruned = np.setdiff1d(np.arange(N), kp)
            for name, src, match in (("kc", k, mk), ("vc", v, mv)):
                seg = oracle.segment(cache, name, b, l)
                for h in range(Hkv):
                    x = src[b, l, h].astype(np.float64)
                    xn = x / np.linalg.norm(x, axis=1, keepdims=True)
                    cos = xn[pruned] @ xn[kp].T
                    want = cos.argmax(1)
                    got = match[b, l, h]
                    assert (got[kp] == -1).all()
                    np.testing.assert_array_equal(got[pruned], want)
                    np.testing.assert_allclose(best[b, l, h][pruned], cos.max(1), rtol=1e-12) if name == "kc" else None
                    counts = 1 + np.bincount(want, minlength=n)
                    for j in range(n):
                        mean = (x[kp[j]] + x[pruned[want == j]].sum(0)) / counts[j]
                        np.testing.assert_allclose(seg[h, j], mean, rtol=1e-6, atol=1e-6)
                    mass = (seg[h, :n].astype(np.float64) * counts[:, None]).sum(0)
                    np.testing.assert_allclose(mass, x.sum(0), rtol=1e-5, atol=1e-4)
                    assert np.isnan(seg[h, n:]).all()


def test_merge_feature_special_cases():
    """(a) Vectors on a circle whose angle grows (slightly convexly) with the position: the most similar
    retained vector is the nearest in position, the lower one half way, whatever the lengths of the vectors --
    the result is that of positional merging.  (b) A pruned vector that is a positive multiple of a retained one
    goes to it, with cosine 1.  (c) A zero vector has cosine 0 with everything; among all-zero vectors it goes to slot 0
    (first maximum); a vector opposite to every retained one still goes to the least bad.  (d) Full budget: nothing
    changes.  (e) bf16 storage gives bf16-representable averages."""
    N, n_l = 41, 2
    r = np.random.default_rng(96)
    theta = 0.02 * np.arange(N) ** 1.001
    rad = r.uniform(0.2, 5.0, N)
    x = np.zeros((1, n_l, 1, N, 2), np.float32)
    x[0, :, 0, :, 0] = (rad * np.cos(theta))[None]
    x[0, :, 0, :, 1] = (rad * np.sin(theta))[None]
    imp = r.random((1, n_l, N)).astype(np.float32) + 0.01
    sel = oracle.select(imp, 14)
    c_feat = oracle.compact(x, x, sel["order"], sel["lengths"], 0)
    c_pos = oracle.compact(x, x, sel["order"], sel["lengths"], 0)
    oracle.merge_feature(c_feat, x, x)
    oracle.merge_position(c_pos, x, x)
    np.testing.assert_allclose(c_feat["kc"], c_pos["kc"], rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(c_feat["vc"], c_pos["vc"], rtol=1e-6, atol=1e-7)
    # (b), (c)
    k = r.standard_normal((1, 1, 1, 6, 4)).astype(np.float32)
    k[0, 0, 0, 4] = 2.5 * k[0, 0, 0, 1]
    k[0, 0, 0, 5] = 0.0
    order = np.array([[[0, 1, 2, 3, 4, 5]]], np.int32)
    cache = oracle.compact(k, k, order, np.array([[3]], np.int32), 0)
    match, best = oracle.feature_match(cache, k)
    assert match[0, 0, 0].tolist()[:3] == [-1, -1, -1] and match[0, 0, 0, 4] == 1
    assert abs(best[0, 0, 0, 4] - 1.0) < 1e-12 and best[0, 0, 0, 5] == 0.0
    kz = np.zeros((1, 1, 1, 4, 4), np.float32)
    cz = oracle.compact(kz, kz, np.array([[[2, 1, 0, 3]]], np.int32), np.array([[2]], np.int32), 0)
    mz, bz = oracle.feature_match(cz, kz)
    assert mz[0, 0, 0].tolist() == [0, -1, -1, 0] and (bz[0, 0, 0, [0, 3]] == 0).all()
    # an opposite vector (cosine -1) still goes to the better of the bad choices
    ko = np.array([[[[[1, 0], [0, 1], [-1, -0.1]]]]], np.float32)
    co = oracle.compact(ko, ko, np.array([[[0, 1, 2]]], np.int32), np.array([[2]], np.int32), 0)
    mo, bo = oracle.feature_match(co, ko)
    assert mo[0, 0, 0, 2] == 1 and bo[0, 0, 0, 2] < 0
    # (d)
    kf, vf, self_, cf = make_cache_case(97, frac=1.0, cap=0)
    ref = {n: cf[n].copy() for n in ("kc", "vc")}
    mk, mv = oracle.merge_feature(cf, kf, vf)
    assert (mk == -1).all() and (mv == -1).all()
    np.testing.assert_array_equal(cf["kc"], ref["kc"])
    np.testing.assert_array_equal(cf["vc"], ref["vc"])
    # bf16 storage
    kb, vb, selb, cb = make_cache_case(98, frac=0.4)
    oracle.merge_feature(cb, kb, vb, storage_bf16=True)
    kc = cb["kc"][~np.isnan(cb["kc"])]
    assert ((kc.view(np.uint32) & 0xffff) == 0).all()


# ------------------------------------------------------------------ causal prefill attention
def test_prefill_attention_matches_dense_numpy_and_ties_to_importance():
    """Dense masked softmax in NumPy (incl. GQA and per-layer scale); constant V gives that constant; with
    V = identity the output rows are the attention probabilities, whose column sums, averaged over the
    heads, are the importance of Sec. 3.2; lse agrees with the importance oracle's; row 0 returns v_0."""
    q, k, sc = rng_qk(71, 2, 2, 4, 2, 13, 8)
    r = np.random.default_rng(72)
    v = r.standard_normal(k.shape).astype(np.float32)
    out, lse = oracle.prefill_attn(q, k, v, sc)
    B, L, H, N, D = q.shape
    kk, vv = np.repeat(k, 2, axis=2).astype(np.float64), np.repeat(v, 2, axis=2).astype(np.float64)
    s = np.einsum("blhmd,blhnd->blhmn", q.astype(np.float64), kk) * sc.astype(np.float64)[None, :, None, None, None]
    s = np.where(np.tril(np.ones((N, N), dtype=bool)), s, -np.inf)
    mx = s.max(-1, keepdims=True)
    e = np.exp(s - mx)
    a = e / e.sum(-1, keepdims=True)
    np.testing.assert_allclose(out, np.einsum("blhmn,blhnd->blhmd", a, vv), rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(lse, (mx + np.log(e.sum(-1, keepdims=True)))[..., 0], rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(out[..., 0, :], np.repeat(v, 2, axis=2)[..., 0, :])       # row 0 sees only key 0
    _, lse_imp = oracle.importance(q, k, sc, want_lse=True)
    np.testing.assert_allclose(lse, lse_imp, rtol=1e-13, atol=1e-13)
    const, _ = oracle.prefill_attn(q, k, np.full_like(v, 0.75), sc)
    np.testing.assert_allclose(const, 0.75, rtol=1e-6)
    # V = identity (D = N): out[m, n] = a[m][n]
    q2, k2, sc2 = rng_qk(73, 1, 2, 2, 2, 8, 8)
    eye = np.broadcast_to(np.eye(8, dtype=np.float32), (1, 2, 2, 8, 8)).copy()
    probs, _ = oracle.prefill_attn(q2, k2, eye, sc2)
    assert (np.triu(probs[0, 0, 0], 1) == 0).all()                                          # causal
    np.testing.assert_allclose(probs.sum(-2).mean(2), oracle.importance(q2, k2, sc2), rtol=1e-6)
