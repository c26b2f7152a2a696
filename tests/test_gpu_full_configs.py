"""GPU parity at the full sizes of the five workload configurations, through the same pre-allocated
pipeline and launch configuration the benchmark times (HIP graph for the decode loop).

The whole batch runs on the GPU; the oracle checks everything for the small configs and a sampled
sequence (for the long-context config also sampled layers and the tail columns of the importance)
for the large ones, plus properties that hold at any size.  Inputs are generated on the device from
seeded generators; the sampled slices are copied back for the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2412_03409_amd as P
from paper_2412_03409_amd.pipeline import HotPath
from pkv_workloads import CONFIGS, make_decode, make_prefill

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
from tolerances import (DECODE_ATOL as OUT_ATOL, IMPORTANCE_RTOL as IMP_RTOL, LSE_ATOL, LSE_RTOL, MERGE_ATOL,
                        MERGE_RTOL_BF16)


def f32(t):
    return t.detach().float().cpu().numpy()


def check_importance(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - want)
    bad = (err > IMP_RTOL * np.abs(want)) & (err > 1e-9)
    assert not bad.any(), f"max rel err {(err / np.maximum(np.abs(want), 1e-30)).max():.3e}"


def run_config(name, budget, sample_b, steps, imp_layers=None, imp_tail=None):
    w = CONFIGS[name]
    Bk = w.budget_tokens(budget)
    x = make_prefill(w, device=DEV)
    dec = make_decode(w, steps=steps, device=DEV)
    hp = HotPath(x["q"], x["k"], x["v"], x["scale"], Bk, steps)
    hp.run_importance(); hp.run_select(); hp.run_compact()
    torch.cuda.synchronize()
    scale = x["scale"].cpu().numpy()
    imp = hp.importance.cpu().numpy()

    # ---- properties that hold at any size, over the whole batch
    np.testing.assert_allclose(imp.sum(-1), w.N, rtol=2e-4)        # every causal softmax row sums to one
    assert (imp[..., 0] >= 1 - 1e-3).all() and (imp[..., -1] <= 1 + 1e-3).all() and (imp >= 0).all()
    assert (hp.sel.status.cpu().numpy() == 0).all()
    lengths = hp.sel.lengths.cpu().numpy()
    assert (lengths.sum(1) == Bk).all() and lengths.min() >= 1 and lengths.max() <= w.N
    order = hp.sel.order.cpu().numpy()
    assert (np.sort(order, axis=-1) == np.arange(w.N)).all()       # every row is a permutation
    cum = hp.sel.cum.cpu().numpy().view(np.uint64)
    assert (np.diff(cum.astype(np.int64), axis=-1) >= 0).all()

    # ---- importance against the oracle on the sampled sequence
    b = sample_b
    layers = list(range(w.L)) if imp_layers is None else imp_layers
    m_lo = 0 if imp_tail is None else w.N - imp_tail
    for l0 in ([None] if imp_layers is None else layers):
        sl = slice(None) if l0 is None else slice(l0, l0 + 1)
        want = oracle.importance(f32(x["q"][b:b + 1, sl]), f32(x["k"][b:b + 1, sl]), scale[sl], m_lo=m_lo)
        check_importance(imp[b:b + 1, sl, m_lo:], want[..., m_lo:])

    # ---- selection: both sides consume the GPU's importance tensor; everything is bit-exact
    want = oracle.select(imp, Bk)
    np.testing.assert_array_equal(order, want["order"])
    np.testing.assert_array_equal(cum, want["cum"])
    np.testing.assert_array_equal(hp.sel.prefix.cpu().numpy(), want["prefix"])
    np.testing.assert_array_equal(lengths, want["lengths"])
    np.testing.assert_array_equal(hp.sel.p.cpu().numpy(), want["p"])
    np.testing.assert_array_equal(hp.sel.iters.cpu().numpy(), want["iters"])
    np.testing.assert_array_equal(hp.sel.raw_total.cpu().numpy(), want["raw_total"])

    # ---- ragged layout over the whole batch, then compaction + decode of the sampled sequence
    caps = hp.cache.caps.cpu().numpy()
    seg_off = hp.cache.seg_off.cpu().numpy()
    np.testing.assert_array_equal(caps, lengths + steps)
    np.testing.assert_array_equal(seg_off.ravel(), np.concatenate([[0], np.cumsum(caps.ravel())[:-1]]))
    np.testing.assert_array_equal(hp.cache.lens.cpu().numpy(), lengths)
    ocache = oracle.compact(f32(x["k"][b:b + 1]), f32(x["v"][b:b + 1]), want["order"][b:b + 1],
                            want["lengths"][b:b + 1], steps)

    def compare_cache():
        Hkv, D = w.Hkv, w.D
        lo, hi = int(seg_off[b, 0]), int(seg_off[b, -1] + caps[b, -1])
        kc = f32(hp.cache.kc[lo * Hkv * D:hi * Hkv * D])
        vc = f32(hp.cache.vc[lo * Hkv * D:hi * Hkv * D])
        kp = hp.cache.kept_pos[lo:hi].cpu().numpy()
        for l in range(w.L):
            n, cap, off = int(ocache["lens"][0, l]), int(caps[b, l]), int(seg_off[b, l]) - lo
            gk = kc[off * Hkv * D:(off + cap) * Hkv * D].reshape(Hkv, cap, D)[:, :n]
            gv = vc[off * Hkv * D:(off + cap) * Hkv * D].reshape(Hkv, cap, D)[:, :n]
            np.testing.assert_array_equal(gk, oracle.segment(ocache, "kc", 0, l)[:, :n])
            np.testing.assert_array_equal(gv, oracle.segment(ocache, "vc", 0, l)[:, :n])
            nk = int(lengths[b, l])
            np.testing.assert_array_equal(kp[off:off + nk], oracle.segment(ocache, "kept_pos", 0, l)[:nk])

    compare_cache()
    # the decode loop exactly as the benchmark runs it: one HIP graph of `steps` launches
    dq, dk, dv = dec["q"], dec["k"], dec["v"]
    hp.capture_decode_loop(dq, dk, dv)
    hp.run_compact()
    hp.replay_decode_loop()
    torch.cuda.synchronize()
    bf = w.dtype == "bf16"
    for t in range(steps):
        ref = oracle.decode_attn(ocache, f32(dq[t, b:b + 1]), f32(dk[t, b:b + 1]), f32(dv[t, b:b + 1]), scale,
                                 out_bf16=bf)
        err = np.abs(f32(hp.out[t, b:b + 1]) - ref).max()
        assert err <= OUT_ATOL, f"decode step {t}: max abs err {err:.3e}"
    np.testing.assert_array_equal(hp.cache.lens.cpu().numpy(), lengths + steps)
    compare_cache()       # appended rows landed in the right slots, bit for bit
    assert torch.isfinite(hp.out.float()).all()


def test_tiny_full():
    run_config("tiny", 0.5, 0, steps=8)


def test_llava7b_b1_full():
    run_config("llava7b_b1", 0.2, 0, steps=4)


@pytest.mark.parametrize("budget", [0.1, 0.2, 0.5])
def test_llava7b_b16_sampled_sequence(budget):
    run_config("llava7b_b16", budget, sample_b=11, steps=2)


def test_llava13b_b8_sampled_sequence():
    run_config("llava13b_b8", 0.2, sample_b=5, steps=2)


@pytest.mark.timeout(400)
def test_gqa_long_sampled_sequence_and_tail_columns():
    run_config("gqa_long", 0.1, sample_b=2, steps=2, imp_layers=[0, 19], imp_tail=160)


@pytest.mark.timeout(600)
def test_gqa_long_every_column_of_the_sharpest_layer():
    """All 8192 columns of one (sequence, layer) at the long-context size against the oracle: the early
    columns accumulate over thousands of query rows and hold the sink keys.  The layer with the
    largest logit scale is taken (its sink columns dominate), and one with the smallest."""
    w = CONFIGS["gqa_long"]
    x = make_prefill(w, device=DEV)
    imp = P.prefixkv_importance(x["q"], x["k"], x["scale"])
    torch.cuda.synchronize()
    scale = x["scale"].cpu().numpy()
    b = 1
    for l in (int(np.argmax(scale)), int(np.argmin(scale))):
        print(f"gqa_long importance, all columns: sequence {b}, layer {l}, scale {scale[l]:.4f}", flush=True)
        want = oracle.importance(f32(x["q"][b:b + 1, l:l + 1]), f32(x["k"][b:b + 1, l:l + 1]), scale[l:l + 1])
        got = imp[b:b + 1, l:l + 1].cpu().numpy()
        assert got.shape == want.shape == (1, 1, w.N)
        check_importance(got, want)
        top = np.argsort(-want[0, 0])[:8]
        print("  largest columns", top.tolist(), "importance", np.round(want[0, 0, top], 2).tolist(), flush=True)


def run_config_pruning(name, budget, sample_b, steps, d):
    """The same pipeline with the decode loop pruning at distance d (one HIP graph of `steps` launches);
    the sampled sequence is checked against the oracle step by step, the whole batch against the closed
    form of the cache size."""
    w = CONFIGS[name]
    Bk = w.budget_tokens(budget)
    x = make_prefill(w, device=DEV)
    dec = make_decode(w, steps=steps, device=DEV)
    hp = HotPath(x["q"], x["k"], x["v"], x["scale"], Bk, steps, evict_distance=d)
    hp.run_importance(); hp.run_select(); hp.run_compact()
    torch.cuda.synchronize()
    scale = x["scale"].cpu().numpy()
    lengths = hp.sel.lengths.cpu().numpy()
    b = sample_b
    want = oracle.select(hp.importance[b:b + 1].cpu().numpy(), Bk)
    np.testing.assert_array_equal(lengths[b:b + 1], want["lengths"])
    ocache = oracle.compact(f32(x["k"][b:b + 1]), f32(x["v"][b:b + 1]), want["order"], want["lengths"],
                            hp.decode_capacity)
    dq, dk, dv = dec["q"], dec["k"], dec["v"]
    hp.capture_decode_loop(dq, dk, dv)
    hp.run_compact()
    hp.replay_decode_loop()
    torch.cuda.synchronize()
    bf = w.dtype == "bf16"
    for t in range(steps):
        ref = oracle.decode_attn_evict(ocache, want["lengths"], f32(dq[t, b:b + 1]), f32(dk[t, b:b + 1]),
                                       f32(dv[t, b:b + 1]), scale, w.N, t + 1, d, out_bf16=bf)
        err = np.abs(f32(hp.out[t, b:b + 1]) - ref).max()
        assert err <= OUT_ATOL, f"decode step {t + 1}: max abs err {err:.3e}"
    perm = hp.cache.lens.cpu().numpy()
    np.testing.assert_array_equal(perm[b:b + 1], ocache["lens"])
    k64 = lengths.astype(np.int64)
    target = np.maximum(1, (2 * k64 * (w.N + steps) + w.N) // (2 * w.N))
    np.testing.assert_array_equal(perm + min(steps, d), np.maximum(target, k64 + min(steps, d)))
    # labels of the sampled sequence's slots: permanent entries and ring
    seg_off, caps = hp.cache.seg_off.cpu().numpy(), hp.cache.caps.cpu().numpy()
    kp = hp.cache.kept_pos.cpu().numpy()
    for l in range(w.L):
        off, cp, pm = int(seg_off[b, l]), int(caps[b, l]), int(perm[b, l])
        slots = list(range(pm)) + list(range(cp - d - 1, cp - d - 1 + min(steps, d + 1)))
        np.testing.assert_array_equal(kp[off:off + cp][slots], oracle.segment(ocache, "kept_pos", 0, l)[slots])
    assert torch.isfinite(hp.out.float()).all()


def test_tiny_pruning_decode():
    run_config_pruning("tiny", 0.5, 0, steps=24, d=4)


def test_llava7b_b1_pruning_decode():
    run_config_pruning("llava7b_b1", 0.2, 0, steps=40, d=8)


def test_llava7b_b16_pruning_decode_sampled_sequence():
    run_config_pruning("llava7b_b16", 0.2, sample_b=7, steps=12, d=5)


@pytest.mark.parametrize("name,layers", [("llava7b_b1", [0, 17, 31]), ("gqa_long", [5])])
def test_prefill_attention_feeds_one_pass_importance_at_full_size(name, layers):
    """Prefill attention at the benchmark shapes: output and lse of sampled layers against the oracle (for the
    long prompt only the rows of the last block are cheap enough for the CPU, so the check there is the
    one-pass importance of the tail columns), and the importance computed from that lse against the
    two-pass importance of the library itself."""
    w = CONFIGS[name]
    if name == "gqa_long":
        w = w.with_(B=1, L=8)
    x = make_prefill(w, device=DEV)
    out, lse = P.prefixkv_prefill_attn(x["q"], x["k"], x["v"], x["scale"])
    imp1 = P.prefixkv_importance(x["q"], x["k"], x["scale"], lse=lse)
    imp2 = P.prefixkv_importance(x["q"], x["k"], x["scale"])
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    check_importance(imp1.cpu().numpy(), imp2.cpu().numpy())
    scale = x["scale"].cpu().numpy()
    for l in layers:
        sl = slice(l, l + 1)
        if name == "llava7b_b1":
            want_out, want_lse = oracle.prefill_attn(f32(x["q"][:1, sl]), f32(x["k"][:1, sl]), f32(x["v"][:1, sl]),
                                                     scale[sl], out_bf16=True)
            assert np.abs(f32(out[:1, sl]) - want_out).max() <= OUT_ATOL
            np.testing.assert_allclose(lse[:1, sl].cpu().numpy(), want_lse, rtol=LSE_RTOL, atol=LSE_ATOL)
        else:
            m_lo = w.N - 96
            want = oracle.importance(f32(x["q"][:1, sl]), f32(x["k"][:1, sl]), scale[sl], m_lo=m_lo)
            check_importance(imp1[:1, sl, m_lo:].cpu().numpy(), want[..., m_lo:])


@pytest.mark.parametrize("name,layers", [("llava7b_b1", [0, 13, 31]), ("llava13b_b8", [7])])
def test_merging_at_full_size(name, layers):
    """Positional and feature merging at benchmark shapes, whole batch on the GPU; sampled layers of sequence 0
    against the oracle.  Properties over everything: the assignment planes mark exactly the kept positions with
    -1 and name slots below the layer's length elsewhere."""
    w = CONFIGS[name]
    Bk = w.budget_tokens(w.budget)
    x = make_prefill(w, device=DEV)
    hp = HotPath(x["q"], x["k"], x["v"], x["scale"], Bk, 2)
    hp.run_importance(); hp.run_select(); hp.run_compact()
    match = P.prefixkv_merge_feature(hp.cache, x["k"], x["v"])
    torch.cuda.synchronize()
    lens = hp.cache.lens.cpu().numpy()
    gm = match.cpu().numpy()
    assert ((gm == -1).sum(-1) == lens[None, :, :, None]).all()
    assert (gm < lens[None, :, :, None, None]).all() and (gm >= -1).all()
    kc_feat, vc_feat = hp.cache.kc.clone(), hp.cache.vc.clone()
    hp.run_compact()
    P.prefixkv_merge_position(hp.cache, x["k"], x["v"])
    torch.cuda.synchronize()
    sel_order, sel_len = hp.sel.order[:1].cpu().numpy(), hp.sel.lengths[:1].cpu().numpy()
    seg_off, caps = hp.cache.seg_off.cpu().numpy(), hp.cache.caps.cpu().numpy()
    Hkv, D = w.Hkv, w.D
    for l in layers:
        sl = slice(l, l + 1)
        k1, v1 = f32(x["k"][:1, sl]), f32(x["v"][:1, sl])
        n = int(sel_len[0, l])
        off, cap = int(seg_off[0, l]), int(caps[0, l])
        seg = lambda t: f32(t[off * Hkv * D:(off + cap) * Hkv * D]).reshape(Hkv, cap, D)[:, :n]
        # feature merging: the kernel's choice is as good as the oracle's; averages for that choice
        want = oracle.compact(k1, v1, sel_order[:, sl], sel_len[:, sl], 2)
        for plane, nm, src, got in ((0, "kc", k1, kc_feat), (1, "vc", v1, vc_feat)):
            wm, best = oracle.feature_match(want, src)
            g = gm[plane, :1, sl]
            np.testing.assert_array_equal(g == -1, wm == -1)
            assert (oracle.match_cosine(want, src, g) >= best - 5e-6).all()
            assert (g != wm).mean() < 1e-3
            oracle.merge_by_match(want, nm, src, g, storage_bf16=True)
            np.testing.assert_allclose(seg(got), oracle.segment(want, nm, 0, 0)[:, :n], rtol=MERGE_RTOL_BF16, atol=MERGE_ATOL)
        # positional merging
        want = oracle.compact(k1, v1, sel_order[:, sl], sel_len[:, sl], 2)
        oracle.merge_position(want, k1, v1, storage_bf16=True)
        np.testing.assert_allclose(seg(hp.cache.kc), oracle.segment(want, "kc", 0, 0)[:, :n], rtol=MERGE_RTOL_BF16, atol=MERGE_ATOL)
        np.testing.assert_allclose(seg(hp.cache.vc), oracle.segment(want, "vc", 0, 0)[:, :n], rtol=MERGE_RTOL_BF16, atol=MERGE_ATOL)
