"""GPU parity: every stage of the HIP path, called through the C-ABI binding, against the CPU oracle
on the same seeded inputs.  Bars: indices / lengths / integers bit-exact; importance within 1e-3
relative; decode attention output within 2e-2 absolute."""
import numpy as np
import pytest
import torch

import oracle
import paper_2412_03409_amd as P
from pkv_workloads import CONFIGS, make_decode, make_prefill, synthetic_importance

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

from tolerances import (DECODE_ATOL as OUT_ATOL, IMPORTANCE_RTOL as IMP_RTOL, LSE_ATOL, LSE_RTOL, MERGE_ATOL,
                        MERGE_RTOL_BF16, MERGE_RTOL_F32)


def np32(t):
    return t.detach().float().cpu().numpy()


def rand_qk(seed, B, L, H, Hkv, N, D, dtype, smax=3.0, sinks=True):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((B, L, H, N, D), generator=g).to(dtype)
    k = torch.randn((B, L, Hkv, N, D), generator=g)
    if sinks:
        k[:, :, :, 0] *= 4.0
        k[:, :, :, N // 3] *= 4.0
    k = k.to(dtype)
    scale = ((torch.rand(L, generator=g) * (smax - 0.5) + 0.5) / D ** 0.5).float()
    return q, k, scale


def check_importance(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert np.isfinite(got).all(), "non-finite importance"
    err = np.abs(got - want) / np.maximum(np.abs(want), 1e-30)
    bad = (err > IMP_RTOL) & (np.abs(got - want) > 1e-9)
    assert not bad.any(), f"max rel err {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"


# --------------------------------------------------------------------------------------- importance
@pytest.mark.parametrize("B,L,H,Hkv,N,D,dtype", [
    (1, 4, 2, 2, 128, 64, torch.float32),      # the Tiny shape
    (2, 2, 4, 2, 77, 128, torch.float32),      # fp32, GQA, ragged
    (1, 2, 4, 4, 200, 128, torch.bfloat16),    # several 128-row tiles + ragged tail
    (2, 3, 8, 2, 333, 64, torch.bfloat16),     # GQA, D = 64
    (1, 1, 2, 2, 1, 128, torch.bfloat16),      # a single position
    (1, 2, 2, 1, 31, 128, torch.bfloat16),     # less than one MFMA tile
    (1, 1, 3, 3, 680, 128, torch.bfloat16),    # the LLaVA prompt length
    (1, 1, 2, 2, 704, 128, torch.bfloat16),    # 11 tile pairs: the last wavefront only copies (spread start)
    (1, 2, 2, 1, 736, 64, torch.bfloat16),     # 12 pairs: every wavefront of the one workgroup has tiles
    (1, 1, 2, 2, 768, 128, torch.bfloat16),    # 24 tiles, still one workgroup per head
    (1, 1, 2, 2, 770, 128, torch.bfloat16),    # 25 tiles: two workgroups per head
    (1, 1, 2, 2, 1100, 128, torch.bfloat16),   # beyond 1024
    (1, 1, 2, 1, 2300, 128, torch.bfloat16),   # long prompt: the software-pipelined stages below the diagonal
    (1, 1, 1, 1, 2100, 64, torch.bfloat16),    # ... with D = 64
])
def test_importance_matches_oracle(B, L, H, Hkv, N, D, dtype):
    q, k, scale = rand_qk(N + D + H, B, L, H, Hkv, N, D, dtype)
    want, lse = oracle.importance(np32(q), np32(k), scale.numpy(), want_lse=True)
    got = P.prefixkv_importance(q.to(DEV), k.to(DEV), scale.to(DEV))
    check_importance(np32(got), want)
    np.testing.assert_allclose(np32(got).sum(-1), N, rtol=1e-4)
    # caller-supplied lse (from its own prefill attention) skips the first pass
    got2 = P.prefixkv_importance(q.to(DEV), k.to(DEV), scale.to(DEV),
                                 lse=torch.from_numpy(lse.astype(np.float32)).to(DEV))
    check_importance(np32(got2), want)


def test_importance_and_prefill_random_shapes():
    """Seeded random shapes (prompt lengths around every tile, block and stage boundary, both head dimensions,
    grouped heads, negative scales): importance in one and two passes, and for bf16 the prefill attention."""
    r = np.random.default_rng(79)
    for case in range(18):
        B, L = int(r.integers(1, 3)), int(r.integers(1, 4))
        Hkv = int(r.choice([1, 2, 3]))
        grp = int(r.choice([1, 1, 2, 4]))
        D = int(r.choice([64, 128]))
        dtype = torch.float32 if case % 6 == 5 else torch.bfloat16
        N = int(r.choice([2, 17, 32, 33, 64, 127, 128, 129, 255, 256, 257, 384, 511, 513, 640, 769, 1025]))
        if dtype == torch.float32 and N > 300:
            N = 129
        q, k, scale = rand_qk(3000 + case, B, L, Hkv * grp, Hkv, N, D, dtype)
        if case % 4 == 3:
            scale = -scale
        want, lse = oracle.importance(np32(q), np32(k), scale.numpy(), want_lse=True)
        got = P.prefixkv_importance(q.to(DEV), k.to(DEV), scale.to(DEV))
        check_importance(np32(got), want)
        got2 = P.prefixkv_importance(q.to(DEV), k.to(DEV), scale.to(DEV),
                                     lse=torch.from_numpy(lse.astype(np.float32)).to(DEV))
        check_importance(np32(got2), want)
        if dtype == torch.bfloat16:
            g = torch.Generator().manual_seed(4000 + case)
            v = torch.randn(k.shape, generator=g).to(torch.bfloat16)
            out, lse_g = P.prefixkv_prefill_attn(q.to(DEV), k.to(DEV), v.to(DEV), scale.to(DEV))
            want_out, want_lse = oracle.prefill_attn(np32(q), np32(k), np32(v), scale.numpy(), out_bf16=True)
            torch.cuda.synchronize()
            assert np.abs(np32(out) - want_out).max() <= OUT_ATOL, case
            np.testing.assert_allclose(lse_g.cpu().numpy(), want_lse, rtol=LSE_RTOL, atol=LSE_ATOL)


def test_importance_strided_inputs_and_determinism():
    B, L, H, N, D = 1, 2, 4, 150, 128
    q, k, scale = rand_qk(5, B, L, H, H, N, D, torch.bfloat16)
    # a fused [B,L,H,N,2D] buffer holding q and k side by side: row stride 2D
    qk = torch.cat([q, k], dim=-1).to(DEV)
    qv, kv = qk[..., :D], qk[..., D:]
    a = P.prefixkv_importance(qv, kv, scale.to(DEV))
    b = P.prefixkv_importance(q.to(DEV), k.to(DEV), scale.to(DEV))
    assert torch.equal(a, b)
    check_importance(np32(a), oracle.importance(np32(q), np32(k), scale.numpy()))


def test_importance_tiny_config_full():
    w = CONFIGS["tiny"]
    x = make_prefill(w)
    want = oracle.importance(np32(x["q"]), np32(x["k"]), x["scale"].numpy())
    got = P.prefixkv_importance(x["q"].to(DEV), x["k"].to(DEV), x["scale"].to(DEV))
    check_importance(np32(got), want)


# --------------------------------------------------------------------------------------- select
def check_select(imp, budget, tol=0, max_iters=64, fixup=True):
    want = oracle.select(imp.numpy(), budget, tol, max_iters, fixup)
    got = P.prefixkv_select(imp.to(DEV), budget, tol, max_iters, fixup)
    torch.cuda.synchronize()
    st = got.status.cpu().numpy()
    np.testing.assert_array_equal(st, want["status"])
    np.testing.assert_array_equal(got.lengths.cpu().numpy(), want["lengths"])
    np.testing.assert_array_equal(got.iters.cpu().numpy(), want["iters"])
    np.testing.assert_array_equal(got.raw_total.cpu().numpy(), want["raw_total"])
    np.testing.assert_array_equal(got.p.cpu().numpy(), want["p"])
    ok = st == 0
    np.testing.assert_array_equal(got.order.cpu().numpy()[ok], want["order"][ok])
    np.testing.assert_array_equal(got.cum.cpu().numpy().view(np.uint64)[ok], want["cum"][ok])
    np.testing.assert_array_equal(got.prefix.cpu().numpy()[ok], want["prefix"][ok])
    return want


@pytest.mark.parametrize("B,L,N", [(1, 1, 1), (1, 3, 5), (2, 4, 128), (3, 32, 680), (2, 40, 680),
                                   (1, 64, 64), (2, 8, 8192), (1, 5, 1025), (2, 7, 2049),
                                   (1, 2, 33), (2, 3, 34), (1, 33, 100), (1, 6, 1100),   # probe / window boundaries
                                   (1, 64, 680), (1, 2, 4096)])                           # two layers per lane group; 4 keys per lane
@pytest.mark.parametrize("ties", [False, True])
def test_select_bit_exact(B, L, N, ties):
    imp = synthetic_importance(B, L, N, seed=B * 1000 + L * 10 + N, ties=ties)
    total = L * N
    for budget in sorted({1, L, L + 1, max(L + 1, total // 10), max(L + 1, total // 5), max(L + 1, total // 2),
                          total - 1, total, total + 5}):
        if budget >= 1:
            check_select(imp, budget)
    check_select(imp, max(L + 1, total // 5), tol=max(1, N // 20))
    check_select(imp, max(L + 1, total // 5), max_iters=7)
    check_select(imp, max(L + 1, total // 5), max_iters=8)      # the last step the tabulated ratios serve
    check_select(imp, max(L + 1, total // 5), max_iters=9, fixup=False)
    check_select(imp, max(L + 1, total // 2), tol=3, fixup=False)


def test_select_random_shapes():
    """Seeded random shapes, budgets, tolerances and iteration limits: everything stage 2+3 returns is bit-exact."""
    r = np.random.default_rng(2024)
    for case in range(80):
        B, L = int(r.integers(1, 4)), int(r.integers(1, 65))
        N = int(r.choice([1, 2, 7, 31, 32, 33, 34, 35, 63, 64, 65, 100, 257, 680, 1023, 1024, 1025, 1089, 1090, 1200, 3000]))
        imp = synthetic_importance(B, L, N, seed=1000 + case, ties=bool(case % 3 == 0))
        if case % 7 == 0 and N > 4:
            imp[:, :, N // 2:] = 0.0                     # long runs of zero weight: flat cumulative sums
        total = L * N
        budget = int(r.integers(1, total + 3))
        tol = int(r.choice([0, 0, 1, 5, max(1, N // 10)]))
        max_iters = int(r.choice([1, 2, 3, 8, 64]))
        check_select(imp, budget, tol=tol, max_iters=max_iters, fixup=bool(case % 2))


def test_select_identical_layers_need_the_rescale():
    # all layers jump together, so most totals are unreachable: exercises stall + largest remainder
    row = synthetic_importance(1, 1, 96, seed=3)[0, 0]
    imp = row.repeat(2, 6, 1).contiguous()
    for budget in (7, 100, 101, 333, 575):
        want = check_select(imp, budget)
        assert (want["lengths"].sum(-1) == budget).all()


def test_select_status_words():
    imp = synthetic_importance(6, 3, 50, seed=4)
    imp[1, 2, 7] = float("nan")
    imp[2, 0, 0] = float("inf")
    imp[3, 1, 3] = -0.25
    imp[4, 1, :] = 0.0
    imp[5, 2, 9] = -0.0           # allowed
    want = check_select(imp, 40)
    assert want["status"].tolist() == [0, 1, 1, 2, 4, 0]
    big = synthetic_importance(1, 2, 16, seed=5)
    big[0, 1, :] = 2.0 ** 16
    want = check_select(big, 9)
    assert want["status"][0] == 8


def test_select_on_device_importance_of_tiny_config():
    w = CONFIGS["tiny"]
    x = make_prefill(w)
    imp = P.prefixkv_importance(x["q"].to(DEV), x["k"].to(DEV), x["scale"].to(DEV)).cpu()
    want = check_select(imp, w.budget_tokens())   # both sides consume the SAME importance tensor
    assert want["lengths"].sum() == w.budget_tokens()


# ------------------------------------------------------------------- offline estimation (Sec. 3.3)
@pytest.mark.parametrize("B,L,N,ties", [(1, 1, 1, False), (2, 4, 128, True), (3, 32, 680, False),
                                        (2, 8, 8192, False), (1, 5, 1025, True)])
def test_rank_bit_exact(B, L, N, ties):
    imp = synthetic_importance(B, L, N, seed=77 + B + L + N, ties=ties)
    got = P.prefixkv_rank(imp.to(DEV))
    want = oracle.rank(imp.numpy())
    np.testing.assert_array_equal(got.status.cpu().numpy(), want["status"])
    np.testing.assert_array_equal(got.order.cpu().numpy(), want["order"])
    np.testing.assert_array_equal(got.cum.cpu().numpy().view(np.uint64), want["cum"])
    np.testing.assert_array_equal(got.prefix.cpu().numpy(), want["prefix"])
    assert P.prefixkv_rank(imp.to(DEV), want_prefix=False).prefix is None


def test_rank_status_words():
    imp = synthetic_importance(5, 3, 50, seed=4)
    imp[1, 2, 7] = float("nan")
    imp[2, 1, 3] = -0.25
    imp[3, 1, :] = 0.0
    imp[4, 0, 3] = float("inf")
    imp[4, 2, 5] = -1.0
    got = P.prefixkv_rank(imp.to(DEV)).status.cpu().numpy()
    want = oracle.rank(imp.numpy())["status"]
    np.testing.assert_array_equal(got, want)
    assert want.tolist() == [0, 1, 2, 4, 3]


@pytest.mark.parametrize("S,L,N", [(1, 1, 1), (1, 4, 128), (10, 32, 680), (7, 40, 680), (3, 64, 8192),
                                   (100, 5, 33)])
def test_offline_config_bit_exact(S, L, N):
    rng = np.random.default_rng(S * 100 + L + N)
    total = L * N
    for budget in sorted({1, L, L + 1, max(L + 1, total // 10), max(L + 1, total // 5), total - 1, total,
                          total + 3}):
        if budget < 1:
            continue
        for kind in ("select", "random", "skewed", "zeros"):
            if kind == "select":       # what the search really produces on S samples
                imp = synthetic_importance(S, L, N, seed=S + L + N + budget % 97)
                sl = oracle.select(imp.numpy(), min(budget, total))["lengths"]
            elif kind == "random":
                sl = rng.integers(0, N + 1, size=(S, L)).astype(np.int32)
            elif kind == "skewed":     # one layer takes almost everything: clamps and the cyclic walk
                sl = np.ones((S, L), np.int32)
                sl[:, L // 2] = N
            else:
                sl = np.zeros((S, L), np.int32)
            got = P.prefixkv_offline_config(torch.from_numpy(sl).to(DEV), N, budget, B_out=3).cpu().numpy()
            want = oracle.offline_config(sl, N, budget)
            np.testing.assert_array_equal(got, np.broadcast_to(want, (3, L)), err_msg=f"{kind} budget {budget}")


def test_offline_pipeline_on_tiny_config():
    """Calibrate on some sequences, deploy the shared configuration on others (Sec. 3.3, last
    paragraph): rank each deployed sequence, compact with the shared lengths, decode."""
    w = CONFIGS["tiny"]
    x = make_prefill(w)
    Bk = w.budget_tokens()
    q, k, v, scale = (x[n].to(DEV) for n in ("q", "k", "v", "scale"))
    imp = P.prefixkv_importance(q, k, scale)
    cal = P.prefixkv_select(imp[:1].contiguous(), Bk)
    shared = P.prefixkv_offline_config(cal.lengths, w.N, Bk, B_out=w.B)
    rk = P.prefixkv_rank(imp)
    steps = 3
    tokens = P.prefixkv_cache_tokens_upper_bound(w.B, Bk, w.L, steps)
    cache = P.prefixkv_compact(k, v, rk.order, shared, steps, tokens)
    # oracle on the same importance tensor
    impn = imp.cpu().numpy()
    osel = oracle.select(impn[:1], Bk)
    oshared = oracle.offline_config(osel["lengths"], w.N, Bk)
    np.testing.assert_array_equal(shared.cpu().numpy(), np.broadcast_to(oshared, (w.B, w.L)))
    assert oshared.sum() == Bk
    orank = oracle.rank(impn)
    olen = np.broadcast_to(oshared, (w.B, w.L)).copy()
    ocache = oracle.compact(np32(x["k"]), np32(x["v"]), orank["order"], olen, steps)
    dec = make_decode(w, steps=steps)
    sc = x["scale"].numpy()
    for t in range(steps):
        out = P.prefixkv_decode_attn(cache, dec["q"][t].to(DEV), dec["k"][t].to(DEV), dec["v"][t].to(DEV),
                                     scale, w.N)
        ref = oracle.decode_attn(ocache, np32(dec["q"][t]), np32(dec["k"][t]), np32(dec["v"][t]), sc,
                                 out_bf16=(w.dtype == "bf16"))
        assert np.abs(np32(out) - ref).max() <= OUT_ATOL
    np.testing.assert_array_equal(cache.lens.cpu().numpy(), olen + steps)


# --------------------------------------------------------------------------------------- compaction
def run_compact(k, v, sel, cap, budget):
    B, L = sel["lengths"].shape
    tokens = P.prefixkv_cache_tokens_upper_bound(B, budget, L, cap)
    got = P.prefixkv_compact(k.to(DEV), v.to(DEV), torch.from_numpy(sel["order"]).to(DEV),
                             torch.from_numpy(sel["lengths"]).to(DEV), cap, tokens)
    want = oracle.compact(np32(k), np32(v), sel["order"], sel["lengths"], cap)
    return got, want


def check_cache(got, want, dtype):
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.seg_off.cpu().numpy(), want["seg_off"])
    np.testing.assert_array_equal(got.caps.cpu().numpy(), want["caps"])
    np.testing.assert_array_equal(got.lens.cpu().numpy(), want["lens"])
    B, L = want["lens"].shape
    Hkv, D = want["Hkv"], want["D"]
    kc, vc, kp = np32(got.kc), np32(got.vc), got.kept_pos.cpu().numpy()
    for b in range(B):
        for l in range(L):
            n, off, cap = want["lens"][b, l], int(want["seg_off"][b, l]), int(want["caps"][b, l])
            wkp = oracle.segment(want, "kept_pos", b, l)[:n]
            nk = int((wkp >= 0).sum())          # slots appended during decode carry no prompt position
            np.testing.assert_array_equal(kp[off:off + nk], wkp[:nk])
            gk = kc[off * Hkv * D:(off + cap) * Hkv * D].reshape(Hkv, cap, D)[:, :n]
            gv = vc[off * Hkv * D:(off + cap) * Hkv * D].reshape(Hkv, cap, D)[:, :n]
            np.testing.assert_array_equal(gk, oracle.segment(want, "kc", b, l)[:, :n])
            np.testing.assert_array_equal(gv, oracle.segment(want, "vc", b, l)[:, :n])


@pytest.mark.parametrize("B,L,Hkv,N,D,frac", [
    (1, 2, 2, 128, 64, 0.5),
    (2, 3, 4, 333, 128, 0.2),
    (2, 2, 2, 70, 64, 0.33),
    (1, 2, 2, 100, 128, 1.0),          # full budget: nothing to merge
    (1, 2, 2, 97, 128, 0.03),          # one or two retained vectors take everything
    (1, 2, 1, 2100, 128, 0.15),        # several position blocks and LDS stages, ragged tails
    (1, 1, 2, 8192, 64, 0.1),
])
def test_merge_feature_matches_oracle(B, L, Hkv, N, D, frac):
    """Feature-similarity merging (Sec. 4.3, cosine metric).  The assignment is an argmax decided in the
    kernel's fp32: it must be as good as the oracle's within the rounding of that arithmetic, identical on the
    planted exact ties (duplicate retained vectors: the lowest position wins; zero vectors: slot 0), and the
    averages must be the oracle's for the assignment the kernel took."""
    g = torch.Generator().manual_seed(N + D + 7)
    k = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    v = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    k *= (0.05 + 20.0 * torch.rand((B, L, Hkv, N, 1), generator=g)).to(torch.bfloat16)   # norms all over the place
    imp = synthetic_importance(B, L, N, seed=N + 9)
    budget = max(L + 1, int(frac * L * N))
    sel = oracle.select(imp.numpy(), budget)
    planted = []
    for b in range(B):
        for l in range(L):
            n = int(sel["lengths"][b, l])
            kept = np.sort(sel["order"][b, l, :n])
            pruned = np.setdiff1d(np.arange(N), kept)
            if n >= 4 and len(pruned) >= 3:
                k[b, l, :, kept[n - 2]] = k[b, l, :, kept[1]]           # duplicate retained vectors
                k[b, l, :, pruned[0]] = 2.0 * k[b, l, :, kept[1]]       # parallel to both: exact tie
                v[b, l, :, pruned[1]] = 0.0                             # zero vector
                v[b, l, :, kept[2]] = 0.0                               # zero retained vector
                planted.append((b, l, pruned[0], 1, pruned[1]))
    got, want = run_compact(k, v, sel, 2, budget)
    match = P.prefixkv_merge_feature(got, k.to(DEV), v.to(DEV))
    torch.cuda.synchronize()
    gm = match.cpu().numpy()
    for plane, name, src in ((0, "kc", np32(k)), (1, "vc", np32(v))):
        wm, best = oracle.feature_match(want, src)
        np.testing.assert_array_equal(gm[plane] == -1, wm == -1)
        assert (gm[plane] >= -1).all()
        for b in range(B):
            for l in range(L):
                assert (gm[plane, b, l] < max(1, int(sel["lengths"][b, l]))).all()
        cos = oracle.match_cosine(want, src, gm[plane])
        assert (cos >= best - 5e-6).all(), float((best - cos).max())
        assert (gm[plane] != wm).mean() < 1e-3            # near ties are rare
        oracle.merge_by_match(want, name, src, gm[plane], storage_bf16=True)
    for b, l, m_dup, slot_dup, m_zero in planted:
        assert (gm[0, b, l, :, m_dup] == slot_dup).all()
        assert (gm[1, b, l, :, m_zero] == 0).all()
    np.testing.assert_array_equal(got.lens.cpu().numpy(), want["lens"])
    kc, vc = np32(got.kc), np32(got.vc)
    for b in range(B):
        for l in range(L):
            off, cap, n = int(want["seg_off"][b, l]), int(want["caps"][b, l]), int(want["lens"][b, l])
            gk = kc[off * Hkv * D:(off + cap) * Hkv * D].reshape(Hkv, cap, D)[:, :n]
            gv = vc[off * Hkv * D:(off + cap) * Hkv * D].reshape(Hkv, cap, D)[:, :n]
            # fp32 sums on the GPU, fp64 in the oracle: equal up to one unit in the last place of bf16
            # (and up to the rounding of an fp32 sum where the terms cancel)
            np.testing.assert_allclose(gk, oracle.segment(want, "kc", b, l)[:, :n], rtol=MERGE_RTOL_BF16, atol=MERGE_ATOL)
            np.testing.assert_allclose(gv, oracle.segment(want, "vc", b, l)[:, :n], rtol=MERGE_RTOL_BF16, atol=MERGE_ATOL)
    if frac == 1.0:
        assert (gm == -1).all()


@pytest.mark.parametrize("B,L,Hkv,N,D,dtype,frac", [
    (1, 4, 2, 128, 64, torch.float32, 0.5),
    (2, 3, 4, 333, 128, torch.bfloat16, 0.2),
    (2, 2, 2, 70, 64, torch.bfloat16, 0.33),
    (1, 2, 2, 100, 128, torch.float32, 1.0),
    (1, 3, 1, 8192, 128, torch.bfloat16, 0.1),
    (1, 2, 2, 1500, 64, torch.bfloat16, 0.9),      # more kept rows than one round of 17 chunks: workgroups walk on
    (2, 1, 3, 1024, 128, torch.float32, 1.0),      # a whole copy of a power-of-two prompt
])
def test_compact_bit_exact(B, L, Hkv, N, D, dtype, frac):
    g = torch.Generator().manual_seed(N + D)
    k = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
    v = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
    imp = synthetic_importance(B, L, N, seed=N)
    budget = max(L + 1, int(frac * L * N))
    sel = oracle.select(imp.numpy(), budget)
    got, want = run_compact(k, v, sel, 5, budget)
    check_cache(got, want, dtype)


def test_compact_and_merge_random_shapes():
    """Seeded random shapes for the gather and for both merging variants."""
    r = np.random.default_rng(80)
    for case in range(16):
        B, L = int(r.integers(1, 3)), int(r.integers(1, 5))
        Hkv = int(r.choice([1, 2, 5]))
        D = int(r.choice([64, 128]))
        dtype = torch.float32 if case % 4 == 3 else torch.bfloat16
        N = int(r.choice([3, 50, 64, 65, 200, 700, 1500]))
        frac = float(r.choice([0.05, 0.3, 0.7, 1.0]))
        g = torch.Generator().manual_seed(5000 + case)
        k = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
        v = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
        imp = synthetic_importance(B, L, N, seed=5000 + case)
        budget = max(L + 1, int(frac * L * N))
        sel = oracle.select(imp.numpy(), budget)
        cap = int(r.integers(0, 7))
        got, want = run_compact(k, v, sel, cap, budget)
        check_cache(got, want, dtype)
        bf = dtype == torch.bfloat16
        rtol = MERGE_RTOL_BF16 if bf else MERGE_RTOL_F32

        def compare():
            torch.cuda.synchronize()
            kc, vc = np32(got.kc), np32(got.vc)
            for b in range(B):
                for l in range(L):
                    off, cp, n = int(want["seg_off"][b, l]), int(want["caps"][b, l]), int(want["lens"][b, l])
                    gk = kc[off * Hkv * D:(off + cp) * Hkv * D].reshape(Hkv, cp, D)[:, :n]
                    gv = vc[off * Hkv * D:(off + cp) * Hkv * D].reshape(Hkv, cp, D)[:, :n]
                    np.testing.assert_allclose(gk, oracle.segment(want, "kc", b, l)[:, :n], rtol=rtol, atol=MERGE_ATOL)
                    np.testing.assert_allclose(gv, oracle.segment(want, "vc", b, l)[:, :n], rtol=rtol, atol=MERGE_ATOL)

        if case % 2 == 0 or not bf:
            P.prefixkv_merge_position(got, k.to(DEV), v.to(DEV))
            oracle.merge_position(want, np32(k), np32(v), storage_bf16=bf)
            compare()
        else:
            match = P.prefixkv_merge_feature(got, k.to(DEV), v.to(DEV)).cpu().numpy()
            for plane, nm, src in ((0, "kc", np32(k)), (1, "vc", np32(v))):
                wm, best = oracle.feature_match(want, src)
                np.testing.assert_array_equal(match[plane] == -1, wm == -1)
                assert (oracle.match_cosine(want, src, match[plane]) >= best - 5e-6).all()
                oracle.merge_by_match(want, nm, src, match[plane], storage_bf16=True)
            compare()


def test_compact_with_empty_segments():
    B, L, Hkv, N, D = 2, 3, 2, 40, 64
    g = torch.Generator().manual_seed(1)
    k = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    v = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    imp = synthetic_importance(B, L, N, seed=9)
    imp[1, 1, 3] = float("nan")            # sequence 1 is rejected: all its lengths are 0
    sel = oracle.select(imp.numpy(), 30)
    assert sel["lengths"][1].sum() == 0
    got, want = run_compact(k, v, sel, 2, 30)
    check_cache(got, want, torch.bfloat16)


# ------------------------------------------------- Gini diagnostic and position merging (Sec. 4.3)
@pytest.mark.parametrize("B,L,N", [(1, 1, 1), (2, 4, 128), (3, 32, 680), (1, 3, 8192)])
def test_gini_matches_oracle(B, L, N):
    imp = synthetic_importance(B, L, N, seed=31 + N)
    if N > 1:
        imp[0, 0] = 1.0                               # flat layer
        imp[0, L - 1] = 0.0; imp[0, L - 1, N // 2] = 3.0   # everything on one position
    rk = P.prefixkv_rank(imp.to(DEV))
    got = P.prefixkv_gini(rk.cum).cpu().numpy()
    want = oracle.gini(oracle.rank(imp.numpy())["cum"])
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-15)
    if N > 1 and L > 1:
        assert got[0, 0] == 0.0 and abs(got[0, L - 1] - (N - 1) / N) < 1e-14


@pytest.mark.parametrize("B,L,Hkv,N,D,dtype,frac", [
    (1, 4, 2, 128, 64, torch.float32, 0.5),
    (2, 3, 4, 333, 128, torch.bfloat16, 0.2),
    (2, 2, 2, 70, 64, torch.bfloat16, 0.33),
    (1, 2, 2, 100, 128, torch.float32, 1.0),          # full budget: nothing to merge
    (1, 2, 2, 97, 128, torch.bfloat16, 0.03),         # one or two kept positions take everything
    (1, 3, 1, 8192, 128, torch.bfloat16, 0.1),
])
def test_merge_position_matches_oracle(B, L, Hkv, N, D, dtype, frac):
    g = torch.Generator().manual_seed(N + D + 1)
    k = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
    v = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
    imp = synthetic_importance(B, L, N, seed=N + 5)
    budget = max(L + 1, int(frac * L * N))
    sel = oracle.select(imp.numpy(), budget)
    got, want = run_compact(k, v, sel, 3, budget)
    P.prefixkv_merge_position(got, k.to(DEV), v.to(DEV))
    bf = dtype == torch.bfloat16
    oracle.merge_position(want, np32(k), np32(v), storage_bf16=bf)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.lens.cpu().numpy(), want["lens"])
    kc, vc = np32(got.kc), np32(got.vc)
    # fp32 sums on the GPU, fp64 in the oracle: equal up to one unit in the last place of the storage dtype
    rtol = MERGE_RTOL_BF16 if bf else MERGE_RTOL_F32
    for b in range(B):
        for l in range(L):
            off, cap, n = int(want["seg_off"][b, l]), int(want["caps"][b, l]), int(want["lens"][b, l])
            gk = kc[off * Hkv * D:(off + cap) * Hkv * D].reshape(Hkv, cap, D)[:, :n]
            gv = vc[off * Hkv * D:(off + cap) * Hkv * D].reshape(Hkv, cap, D)[:, :n]
            np.testing.assert_allclose(gk, oracle.segment(want, "kc", b, l)[:, :n], rtol=rtol, atol=MERGE_ATOL)
            np.testing.assert_allclose(gv, oracle.segment(want, "vc", b, l)[:, :n], rtol=rtol, atol=MERGE_ATOL)
    if frac == 1.0:   # every group is one position: bit-identical to the plain gather
        plain, pw = run_compact(k, v, sel, 3, budget)
        check_cache(got, pw, dtype)


# --------------------------------------------------------------------------------------- decode
def run_decode_case(B, L, H, Hkv, N, D, dtype, frac, steps, seed, layer_range=None, zero_seq=False):
    g = torch.Generator().manual_seed(seed)
    k = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
    v = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
    scale = ((torch.rand(L, generator=g) * 2.5 + 0.5) / D ** 0.5).float()
    imp = synthetic_importance(B, L, N, seed=seed)
    if zero_seq:
        imp[0, 0, 0] = float("nan")
    budget = max(L + 1, int(frac * L * N))
    sel = oracle.select(imp.numpy(), budget)
    got, want = run_compact(k, v, sel, steps, budget)
    l0, l1 = layer_range or (0, L)
    bf = dtype == torch.bfloat16
    for t in range(steps + 1):
        q = torch.randn((B, L, H, D), generator=g).to(dtype)
        kn = torch.randn((B, L, Hkv, D), generator=g).to(dtype)
        vn = torch.randn((B, L, Hkv, D), generator=g).to(dtype)
        append = t < steps       # the last step attends without appending
        o = P.prefixkv_decode_attn(got, q.to(DEV), kn.to(DEV) if append else None,
                                   vn.to(DEV) if append else None, scale.to(DEV), N, l0, l1)
        ref = oracle.decode_attn(want, np32(q), np32(kn) if append else None, np32(vn) if append else None,
                                 scale.numpy(), l0, l1, out_bf16=bf)
        torch.cuda.synchronize()
        err = np.abs(np32(o)[:, l0:l1] - ref[:, l0:l1])
        assert err.max() <= OUT_ATOL, f"step {t}: max abs err {err.max():.3e}"
        np.testing.assert_array_equal(got.lens.cpu().numpy(), want["lens"])
    check_cache(got, want, dtype)   # appended rows landed in the right slots, bit for bit


@pytest.mark.parametrize("B,L,H,Hkv,N,D,dtype,frac,steps", [
    (1, 4, 2, 2, 128, 64, torch.float32, 0.5, 8),       # the Tiny shape
    (2, 3, 4, 4, 300, 128, torch.bfloat16, 0.3, 3),     # MHA, several chunks per segment
    (2, 2, 8, 2, 500, 128, torch.bfloat16, 0.5, 2),     # GQA group of 4
    (1, 2, 16, 2, 260, 64, torch.bfloat16, 0.6, 2),     # GQA group of 8, D = 64
    (1, 2, 6, 2, 150, 128, torch.bfloat16, 0.4, 2),     # group of 3: falls back to 1 head per unit
    (1, 2, 4, 2, 90, 128, torch.float32, 0.9, 2),       # fp32 rows of 512 B (two sub-blocks per chunk)
    (1, 2, 2, 2, 63, 128, torch.bfloat16, 1.0, 2),      # 63 -> 64 -> 65 slots: crosses a chunk edge
    (1, 2, 4, 4, 1500, 128, torch.bfloat16, 0.7, 2),    # N > 1024: long segments on the two-wavefront shape
    (1, 2, 8, 2, 4200, 128, torch.bfloat16, 0.8, 2),    # N > 4096, GQA: split segments
    (1, 1, 2, 2, 5000, 64, torch.float32, 0.9, 1),      # long fp32 segment: 8-wavefront launch shape
    (1, 2, 4, 2, 3000, 128, torch.bfloat16, 0.9, 2),    # grouped (2 heads per KV head), segments split in 3 pieces
    (1, 2, 16, 2, 2500, 64, torch.bfloat16, 0.95, 2),   # grouped (8 heads), D = 64, split segments
    (2, 3, 8, 2, 1100, 128, torch.bfloat16, 0.95, 3),   # the appended row crosses a piece boundary (1024)
    (1, 1, 8, 1, 8192, 128, torch.bfloat16, 1.0, 1),    # grouped (8 heads), one segment of 8 pieces
    # 512 to 1024 (sequence, layer, head) units: the largest launches that are resident at once
    (2, 9, 32, 32, 70, 64, torch.bfloat16, 0.3, 3),
    (3, 6, 32, 32, 200, 128, torch.bfloat16, 0.5, 2),
    (1, 18, 32, 32, 50, 64, torch.float32, 0.4, 2),
    (1, 5, 120, 120, 40, 64, torch.bfloat16, 1.0, 2),   # many heads, full budget
])
def test_decode_matches_oracle(B, L, H, Hkv, N, D, dtype, frac, steps):
    run_decode_case(B, L, H, Hkv, N, D, dtype, frac, steps, seed=N + H)


def test_decode_random_shapes():
    """Seeded random shapes over every launch path: one head per workgroup, fp32 head groups, the grouped-query
    kernel with and without split segments, layer ranges, one to three steps."""
    r = np.random.default_rng(77)
    for case in range(36):
        B, L = int(r.integers(1, 4)), int(r.integers(1, 6))
        Hkv = int(r.choice([1, 2, 4]))
        grp = int(r.choice([1, 1, 2, 3, 4, 8]))
        D = int(r.choice([64, 128]))
        dtype = torch.float32 if case % 5 == 4 else torch.bfloat16
        N = int(r.choice([1, 5, 63, 64, 65, 130, 300, 700, 1100, 2300]))
        if dtype == torch.float32 and N > 700:
            N = 700
        frac = float(r.choice([0.05, 0.2, 0.5, 0.9, 1.0]))
        steps = int(r.integers(1, 4))
        l0 = int(r.integers(0, L))
        l1 = int(r.integers(l0 + 1, L + 1))
        run_decode_case(B, L, Hkv * grp, Hkv, N, D, dtype, frac, steps, seed=500 + case,
                        layer_range=(l0, l1) if case % 2 else None)


# ------------------------------------------------ decode with pruning at a fixed distance (Sec. 3.1)
def run_evict_case(B, L, H, Hkv, N, D, dtype, frac, d, steps, seed, extra=None, zero_seq=False):
    g = torch.Generator().manual_seed(seed)
    k = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
    v = torch.randn((B, L, Hkv, N, D), generator=g).to(dtype)
    scale = ((torch.rand(L, generator=g) * 2.5 + 0.5) / D ** 0.5).float()
    imp = synthetic_importance(B, L, N, seed=seed)
    if zero_seq:
        imp[0, 0, 0] = float("nan")
    budget = max(L + 1, int(frac * L * N))
    sel = oracle.select(imp.numpy(), budget)
    cap = d + 1 + (steps if extra is None else extra)
    got, want = run_compact(k, v, sel, cap, budget)
    base = torch.from_numpy(sel["lengths"]).to(DEV)
    bf = dtype == torch.bfloat16
    esz = 2 if bf else 4
    for t in range(1, steps + 1):
        q = torch.randn((B, L, H, D), generator=g).to(dtype)
        kn = torch.randn((B, L, Hkv, D), generator=g).to(dtype)
        vn = torch.randn((B, L, Hkv, D), generator=g).to(dtype)
        o = P.prefixkv_decode_attn_evict(got, base, q.to(DEV), kn.to(DEV), vn.to(DEV), scale.to(DEV), N, t, d)
        ref = oracle.decode_attn_evict(want, sel["lengths"], np32(q), np32(kn), np32(vn), scale.numpy(), N, t, d,
                                       out_bf16=bf)
        torch.cuda.synchronize()
        err = np.abs(np32(o) - ref)
        assert err.max() <= OUT_ATOL, f"step {t}: max abs err {err.max():.3e}"
        np.testing.assert_array_equal(got.lens.cpu().numpy(), want["lens"], err_msg=f"step {t}")
    # every live slot (permanent entries and ring) holds the same position and the same bytes
    kc, vc, kp = np32(got.kc), np32(got.vc), got.kept_pos.cpu().numpy()
    nring = min(steps, d + 1)
    for b in range(B):
        for l in range(L):
            off, cp, perm = int(want["seg_off"][b, l]), int(want["caps"][b, l]), int(want["lens"][b, l])
            slots = list(range(perm)) + list(range(cp - d - 1, cp - d - 1 + nring))
            wkp = oracle.segment(want, "kept_pos", b, l)
            np.testing.assert_array_equal(kp[off:off + cp][slots], wkp[slots])
            live = [s_ for s_ in slots if wkp[s_] >= 0]
            gk = kc[off * Hkv * D:(off + cp) * Hkv * D].reshape(Hkv, cp, D)
            gv = vc[off * Hkv * D:(off + cp) * Hkv * D].reshape(Hkv, cp, D)
            np.testing.assert_array_equal(gk[:, live], oracle.segment(want, "kc", b, l)[:, live])
            np.testing.assert_array_equal(gv[:, live], oracle.segment(want, "vc", b, l)[:, live])
    return sel, want


@pytest.mark.parametrize("B,L,H,Hkv,N,D,dtype,frac,d,steps", [
    (1, 4, 2, 2, 128, 64, torch.float32, 0.5, 1, 12),     # the Tiny shape, decide from step 2 on
    (1, 4, 2, 2, 128, 64, torch.float32, 0.5, 4, 24),
    (2, 3, 4, 4, 300, 128, torch.bfloat16, 0.3, 3, 30),   # survivors and pruned tokens alternate
    (2, 2, 8, 2, 500, 128, torch.bfloat16, 0.5, 7, 20),   # GQA group of 4
    (1, 2, 16, 2, 260, 64, torch.bfloat16, 0.6, 2, 9),    # GQA group of 8, D = 64
    (1, 2, 6, 2, 150, 128, torch.bfloat16, 0.4, 5, 16),   # group of 3: three workgroups share a kv head
    (1, 2, 2, 2, 63, 128, torch.bfloat16, 1.0, 2, 8),     # ratio 1: every decided token survives
    (1, 2, 2, 2, 60, 128, torch.bfloat16, 0.5, 70, 80),   # ring longer than a chunk
    (1, 2, 4, 4, 1500, 128, torch.bfloat16, 0.7, 6, 10),  # 4-wavefront launch shape
    (1, 2, 8, 2, 4200, 128, torch.bfloat16, 0.8, 3, 6),   # 8-wavefront launch shape, GQA
    (1, 3, 2, 2, 64, 64, torch.float32, 0.06, 63, 70),    # one kept entry per layer: sliding window
    (1, 2, 8, 2, 1500, 128, torch.bfloat16, 0.6, 700, 12),  # grouped: the ring rows straddle a piece boundary
    (1, 2, 4, 2, 2100, 128, torch.bfloat16, 0.95, 3, 8),    # grouped, split permanent region, survivors
    (1, 2, 16, 2, 300, 64, torch.bfloat16, 0.5, 40, 60),    # grouped (8 heads), D = 64, ring longer than the kept part
])
def test_decode_evict_matches_oracle(B, L, H, Hkv, N, D, dtype, frac, d, steps):
    run_evict_case(B, L, H, Hkv, N, D, dtype, frac, d, steps, seed=N + H + d)


def test_decode_evict_random_shapes():
    """Seeded random shapes, distances and step counts for decode with pruning (all launch paths)."""
    r = np.random.default_rng(78)
    for case in range(20):
        B, L = int(r.integers(1, 3)), int(r.integers(1, 5))
        Hkv = int(r.choice([1, 2, 4]))
        grp = int(r.choice([1, 1, 2, 4, 8]))
        D = int(r.choice([64, 128]))
        dtype = torch.float32 if case % 6 == 5 else torch.bfloat16
        N = int(r.choice([5, 40, 64, 130, 300, 1100]))
        if dtype == torch.float32 and N > 300:
            N = 300
        frac = float(r.choice([0.1, 0.3, 0.6, 1.0]))
        d = int(r.choice([1, 2, 3, 5, 9, 40]))
        steps = int(r.integers(1, 13))
        run_evict_case(B, L, Hkv * grp, Hkv, N, D, dtype, frac, d, steps, seed=900 + case)


def test_decode_evict_rejected_sequence_and_size_law():
    B, L, N, d, steps = 2, 3, 96, 3, 40
    sel, want = run_evict_case(B, L, 4, 2, N, 128, torch.bfloat16, 0.25, d, steps, seed=5, zero_seq=True)
    assert sel["lengths"][0].sum() == 0                    # rejected: only the ring is ever cached
    for b in range(B):
        for l in range(L):
            kl = int(sel["lengths"][b, l])
            target = max(1, (2 * kl * (N + steps) + N) // (2 * N))
            assert int(want["lens"][b, l]) + d == max(target, kl + d)


def test_decode_evict_without_position_tracking_and_capacity_guard():
    """kept_pos = NULL is allowed; a segment whose capacity cannot hold the ring is left alone and
    outputs zeros (device-side guard; the oracle refuses such a call, so there is no reference)."""
    B, L, H, Hkv, N, D, d = 1, 2, 2, 2, 50, 64, 4
    g = torch.Generator().manual_seed(3)
    k = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    v = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    sel = oracle.select(synthetic_importance(B, L, N, seed=8).numpy(), 40)
    scale = torch.full((L,), 0.1)
    q = torch.randn((B, L, H, D), generator=g).to(torch.bfloat16)
    kn = torch.randn((B, L, Hkv, D), generator=g).to(torch.bfloat16)
    base = torch.from_numpy(sel["lengths"]).to(DEV)
    got, want = run_compact(k, v, sel, d + 1, 40)
    before = got.kept_pos.clone()
    o = P.prefixkv_decode_attn_evict(got, base, q.to(DEV), kn.to(DEV), kn.to(DEV), scale.to(DEV), N, 1, d,
                                     track_positions=False)
    ref = oracle.decode_attn_evict(want, sel["lengths"], np32(q), np32(kn), np32(kn), scale.numpy(), N, 1, d,
                                   out_bf16=True)
    assert np.abs(np32(o) - ref).max() <= OUT_ATOL
    assert torch.equal(before, got.kept_pos)
    small, _ = run_compact(k, v, sel, d, 40)               # one slot short of a ring
    kc0, lens0 = small.kc.clone(), small.lens.clone()
    o = P.prefixkv_decode_attn_evict(small, base, q.to(DEV), kn.to(DEV), kn.to(DEV), scale.to(DEV), N, 1, d)
    torch.cuda.synchronize()
    assert (o == 0).all() and torch.equal(kc0, small.kc) and torch.equal(lens0, small.lens)


def test_decode_layer_range_and_rejected_sequence():
    run_decode_case(2, 4, 4, 4, 100, 128, torch.bfloat16, 0.3, 2, seed=7, layer_range=(1, 3))
    run_decode_case(2, 4, 8, 2, 1300, 128, torch.bfloat16, 0.9, 2, seed=9, layer_range=(1, 3))   # grouped, split
    run_decode_case(2, 3, 4, 2, 100, 128, torch.bfloat16, 0.3, 2, seed=8, zero_seq=True)
    run_decode_case(2, 12, 32, 32, 60, 64, torch.bfloat16, 0.4, 2, seed=10, layer_range=(2, 11))   # many units, layer range
    run_decode_case(2, 10, 32, 32, 60, 64, torch.bfloat16, 0.4, 2, seed=11, zero_seq=True)         # many units, one empty sequence


def test_full_budget_reproduces_full_cache_attention():
    # budget of 100%: the compressed path must equal plain attention over the whole prefill cache
    B, L, H, N, D = 1, 2, 4, 150, 128
    g = torch.Generator().manual_seed(21)
    k = torch.randn((B, L, H, N, D), generator=g).to(torch.bfloat16)
    v = torch.randn((B, L, H, N, D), generator=g).to(torch.bfloat16)
    q = torch.randn((B, L, H, D), generator=g).to(torch.bfloat16)
    scale = torch.full((L,), 1.0 / D ** 0.5)
    imp = synthetic_importance(B, L, N, seed=2).to(DEV)
    sel = P.prefixkv_select(imp, L * N)
    tokens = P.prefixkv_cache_tokens_upper_bound(B, L * N, L, 0)
    cache = P.prefixkv_compact(k.to(DEV), v.to(DEV), sel.order, sel.lengths, 0, tokens)
    o = P.prefixkv_decode_attn(cache, q.to(DEV), None, None, scale.to(DEV), N)
    s = torch.einsum("blhd,blhnd->blhn", q.double(), k.double()) * scale.double()[None, :, None, None]
    ref = torch.einsum("blhn,blhnd->blhd", torch.softmax(s, -1), v.double())
    assert (o.cpu().double() - ref).abs().max() <= OUT_ATOL
    assert torch.equal(cache.kc.view(k.shape).cpu(), k)


# --------------------------------------------------------------------------------------- end to end
def test_tiny_config_end_to_end():
    w = CONFIGS["tiny"]
    x, dec = make_prefill(w), make_decode(w)
    imp = P.prefixkv_importance(x["q"].to(DEV), x["k"].to(DEV), x["scale"].to(DEV))
    sel = P.prefixkv_select(imp, w.budget_tokens())
    tokens = P.prefixkv_cache_tokens_upper_bound(w.B, w.budget_tokens(), w.L, w.decode_steps)
    cache = P.prefixkv_compact(x["k"].to(DEV), x["v"].to(DEV), sel.order, sel.lengths, w.decode_steps, tokens)
    o_sel = oracle.select(imp.cpu().numpy(), w.budget_tokens())      # same importance tensor on both sides
    np.testing.assert_array_equal(sel.lengths.cpu().numpy(), o_sel["lengths"])
    np.testing.assert_array_equal(sel.order.cpu().numpy(), o_sel["order"])
    assert int(sel.lengths.sum()) == w.budget_tokens()
    o_cache = oracle.compact(np32(x["k"]), np32(x["v"]), o_sel["order"], o_sel["lengths"], w.decode_steps)
    for t in range(w.decode_steps):
        o = P.prefixkv_decode_attn(cache, dec["q"][t].to(DEV), dec["k"][t].to(DEV), dec["v"][t].to(DEV),
                                   x["scale"].to(DEV), w.N)
        ref = oracle.decode_attn(o_cache, np32(dec["q"][t]), np32(dec["k"][t]), np32(dec["v"][t]),
                                 x["scale"].numpy())
        assert np.abs(np32(o) - ref).max() <= OUT_ATOL
    check_cache(cache, o_cache, torch.float32)


@pytest.mark.parametrize("variant", ["tiny", "gqa_split", "gqa_pruning"])
def test_decode_loop_graph_replays_match_eager(variant):
    # the decode loop captured as one HIP graph: several replays, with eager work and synchronisations
    # between them, must each reproduce the eager outputs and the final cache bit for bit.  The grouped-query
    # variants run the planning kernel + work-list kernel pair, with segments long enough to be split.
    from paper_2412_03409_amd.pipeline import HotPath
    ev = None
    if variant == "tiny":
        w = CONFIGS["tiny"].with_(decode_steps=6)
    else:
        w = CONFIGS["gqa_long"].with_(B=1, L=3, N=2600, decode_steps=5, budget=0.7)
        ev = 2 if variant == "gqa_pruning" else None
    x, dec = make_prefill(w), make_decode(w)
    hp = HotPath(x["q"].to(DEV), x["k"].to(DEV), x["v"].to(DEV), x["scale"].to(DEV), w.budget_tokens(), w.decode_steps,
                 evict_distance=ev)
    dq, dk, dv = dec["q"].to(DEV), dec["k"].to(DEV), dec["v"].to(DEV)
    hp.run_importance(); hp.run_select(); hp.run_compact()
    hp.run_decode_loop(dq, dk, dv)
    torch.cuda.synchronize()
    want_out, want_kc, want_lens = hp.out.clone(), hp.cache.kc.clone(), hp.cache.lens.clone()
    hp.capture_decode_loop(dq, dk, dv)
    for rep in range(4):
        hp.out.zero_()
        hp.run_importance(); hp.run_select(); hp.run_compact()      # eager work between replays
        torch.cuda.synchronize()
        hp.replay_decode_loop()
        torch.cuda.synchronize()
        assert torch.equal(hp.out, want_out), f"replay {rep}"
        assert torch.equal(hp.cache.lens, want_lens), f"replay {rep}"
        # compare occupied slots only (the rest of the buffer is never written)
        assert torch.equal(torch.nan_to_num(hp.cache.kc), torch.nan_to_num(want_kc)), f"replay {rep}"


# ------------------------------------------- prefill attention that hands lse to the importance stage
@pytest.mark.parametrize("B,L,H,Hkv,N,D", [
    (1, 1, 1, 1, 1, 64), (1, 1, 2, 2, 16, 128), (1, 2, 2, 2, 33, 64), (2, 2, 4, 2, 130, 128),
    (1, 2, 4, 4, 257, 128), (1, 1, 8, 2, 680, 128), (1, 1, 2, 1, 1100, 64),
])
def test_prefill_attention_matches_oracle_and_feeds_importance(B, L, H, Hkv, N, D):
    g = torch.Generator().manual_seed(N * 7 + D)
    q = torch.randn((B, L, H, N, D), generator=g).to(torch.bfloat16)
    k = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    v = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    scale = ((torch.rand(L, generator=g) * 2.5 + 0.5) / D ** 0.5).float()
    out, lse = P.prefixkv_prefill_attn(q.to(DEV), k.to(DEV), v.to(DEV), scale.to(DEV))
    want_out, want_lse = oracle.prefill_attn(np32(q), np32(k), np32(v), scale.numpy(), out_bf16=True)
    torch.cuda.synchronize()
    assert np.isfinite(np32(out)).all()
    assert np.abs(np32(out) - want_out).max() <= OUT_ATOL
    np.testing.assert_allclose(lse.cpu().numpy(), want_lse, rtol=LSE_RTOL, atol=LSE_ATOL)
    # the importance stage with this lse (one pass) meets the same bar as with its own (two passes)
    imp1 = P.prefixkv_importance(q.to(DEV), k.to(DEV), scale.to(DEV), lse=lse)
    check_importance(imp1.cpu().numpy(), oracle.importance(np32(q), np32(k), scale.numpy()))


def test_prefill_attention_negative_scale_and_sinks():
    """A negative logit scale (moved into the queries by the kernel) and large sink keys that make the
    running maximum jump late in the row."""
    B, L, H, Hkv, N, D = 1, 2, 2, 2, 200, 128
    g = torch.Generator().manual_seed(12)
    q = torch.randn((B, L, H, N, D), generator=g).to(torch.bfloat16)
    k = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    v = torch.randn((B, L, Hkv, N, D), generator=g).to(torch.bfloat16)
    k[..., 150, :] *= 4
    k[..., 0, :] *= 3
    scale = torch.tensor([-0.11, 0.2])
    out, lse = P.prefixkv_prefill_attn(q.to(DEV), k.to(DEV), v.to(DEV), scale.to(DEV))
    want_out, want_lse = oracle.prefill_attn(np32(q), np32(k), np32(v), scale.numpy(), out_bf16=True)
    assert np.abs(np32(out) - want_out).max() <= OUT_ATOL
    np.testing.assert_allclose(lse.cpu().numpy(), want_lse, rtol=LSE_RTOL, atol=LSE_ATOL)


def test_prefill_attention_strided_inputs_and_refusals():
    B, L, H, N, D = 1, 2, 2, 70, 128
    g = torch.Generator().manual_seed(4)
    big = torch.randn((3, B, L, H, N, D), generator=g).to(torch.bfloat16).to(DEV)   # q, k, v interleaved: strided views
    q, k, v = big[0], big[1], big[2]
    scale = torch.full((L,), 0.1, device=DEV)
    out, lse = P.prefixkv_prefill_attn(q, k, v, scale)
    ref, ref_lse = P.prefixkv_prefill_attn(q.contiguous(), k.contiguous(), v.contiguous(), scale)
    assert torch.equal(out, ref) and torch.equal(lse, ref_lse)
    with pytest.raises(P.PrefixKVError):
        P.prefixkv_prefill_attn(q.float(), k.float(), v.float(), scale)            # bf16 storage only
