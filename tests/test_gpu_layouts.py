"""GPU parity of the *_strided entry points: Q / K / V and the caches in head-major and padded layouts.

The oracle knows one layout (token-major).  Each test lays the same values out differently on the device,
hands the strides to the library, brings the results back to token-major and applies the same checks as the
tests of the plain entry points.  Padding elements are filled with a marker that must survive every call."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import FILTER_BUDGET, FILTER_THRESHOLD
from parity import check_decode, check_prefill

pytestmark = pytest.mark.gpu

MARK = 0x7FC1        # a NaN bit pattern: reading a padding element as data would poison the scores


def relayout(t, kind):
    """A [.., T, H, d] device tensor -> a view of the same logical shape over other storage.
    Returns (view, storage)."""
    import torch
    if kind == "dense":
        return t, t
    if kind == "head_major":                                   # storage [.., H, T, d]
        s = t.transpose(-3, -2).contiguous()
        return s.transpose(-3, -2), s
    if kind == "padded":                                       # storage [.., T, H + 1, d + 8]: row and slice padding
        shape = list(t.shape)
        shape[-2] += 1
        shape[-1] += 8
        s = torch.full(shape, 0, dtype=torch.int16, device=t.device)
        s.fill_(int(MARK))
        s = s.view(torch.bfloat16)
        view = s[..., : t.shape[-2], : t.shape[-1]]
        view.copy_(t)
        return view, s
    raise ValueError(kind)


def padding_intact(view, storage, kind):
    import torch
    if kind != "padded":
        return True
    s = storage.view(torch.int16)
    H, d = view.shape[-2], view.shape[-1]
    return bool((s[..., H:, :] == np.int16(MARK)).all()) and bool((s[..., :, d:] == np.int16(MARK)).all())


def prefill_strided(t, Mv, budget, mode, vis_valid, txt_len, is_key, gamma, alpha, Rcap, scale, kinds):
    import torch
    import paper_2411_10803_amd as md
    from paper_2411_10803_amd import harness
    kq, kkv, kout = kinds
    B, N, H, d = t["q_txt"].shape
    Cdim = t["hidden"].shape[2]
    q, _ = relayout(harness.to_dev(t["q_txt"], True), kq)
    k, ks = relayout(harness.to_dev(t["k"], True), kkv)
    v, vs = relayout(harness.to_dev(t["v"], True), kkv)
    dev = q.device
    ko, kos = relayout(torch.zeros((B, Rcap + N, H, d), dtype=torch.bfloat16, device=dev), kout)
    vo, vos = relayout(torch.zeros((B, Rcap + N, H, d), dtype=torch.bfloat16, device=dev), kout)
    out = {
        "hidden_out": torch.zeros((B, Rcap + N, Cdim), dtype=torch.bfloat16, device=dev), "k_out": ko, "v_out": vo,
        "kept_index": torch.full((B, Rcap), -1, dtype=torch.int32, device=dev),
        "kept_count": torch.zeros((B,), dtype=torch.int32, device=dev),
        "out_len": torch.zeros((B,), dtype=torch.int32, device=dev),
        "out_protect": torch.zeros((B, Rcap + N), dtype=torch.uint8, device=dev),
        "out_ids": torch.full((B, Rcap + N), -1, dtype=torch.int32, device=dev),
        "score_global": torch.zeros((B, Mv), dtype=torch.float32, device=dev),
        "score_indiv": torch.zeros((B, Mv), dtype=torch.float32, device=dev),
    }
    md.mustdrop_prefill_filter_strided(q, k, v, harness.to_dev(t["hidden"], True), harness.to_dev(vis_valid),
                                       harness.to_dev(txt_len), harness.to_dev(is_key), Mv, scale, mode, budget, gamma,
                                       alpha, out, Rcap=Rcap)
    torch.cuda.synchronize()
    assert padding_intact(ko, kos, kout) and padding_intact(vo, vos, kout)
    assert padding_intact(k, ks, kkv) and padding_intact(v, vs, kkv)
    out["k_out"], out["v_out"] = ko.contiguous(), vo.contiguous()
    return harness.outputs_to_host(out)


@pytest.mark.parametrize("kinds", [("head_major", "head_major", "head_major"), ("padded", "padded", "dense"),
                                   ("dense", "head_major", "padded"), ("dense", "dense", "dense")])
def test_prefill_filter_in_other_layouts(kinds):
    cfg = wl.tiny(wl.CONFIGS[2], B=3, Hg=9, Wg=13, N=45, H=6, d=64, C=264)
    Mv = cfg.M
    t = wl.prefill_inputs(cfg)
    rng = np.random.default_rng(5)
    vis_valid = (rng.random((cfg.B, Mv)) > 0.25).astype(np.uint8)
    txt_len = np.array([45, 20, 3], dtype=np.int32)
    is_key = wl.random_key_mask(cfg, 6, valid=vis_valid)
    scale, gamma, alpha = 1.0 / np.sqrt(cfg.d), 1.0 / Mv, 2.0 / (Mv + cfg.N)
    for mode, budget, Rcap in ((FILTER_BUDGET, 30, 30), (FILTER_THRESHOLD, 0, Mv)):
        g = prefill_strided(t, Mv, budget, mode, vis_valid, txt_len, is_key, gamma, alpha, Rcap, scale, kinds)
        o = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], vis_valid, txt_len, is_key, Mv, scale, mode,
                                  budget, gamma, alpha, Rcap)
        check_prefill(g, o, t, Mv, vis_valid, is_key, mode, budget, gamma, alpha, Rcap)


def test_prefill_filter_head_major_at_the_benchmark_head_shape():
    """32 heads of 128 on a batch slice of the LLaVA-1.5 workload, K / V / outputs head-major."""
    cfg = wl.CONFIGS[2]
    t = wl.prefill_inputs(cfg, samples=[0, 7])
    is_key = wl.random_key_mask(cfg, cfg.key_budget)[[0, 7]]
    scale, gamma, alpha = 1.0 / np.sqrt(cfg.d), 1.0 / cfg.M, 2.0 / (cfg.M + cfg.N)
    g = prefill_strided(t, cfg.M, 192, FILTER_BUDGET, None, None, is_key, gamma, alpha, 192, scale,
                        ("head_major", "head_major", "head_major"))
    o = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], None, None, is_key, cfg.M, scale, FILTER_BUDGET,
                              192, gamma, alpha, 192)
    check_prefill(g, o, t, cfg.M, None, is_key, FILTER_BUDGET, 192, gamma, alpha, 192)
    assert np.all(g["kept_count"] == 192)


def test_dense_layouts_take_the_plain_path_bit_for_bit():
    import torch
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[2], B=2, Hg=8, Wg=8, N=32, H=4, d=128, C=512)
    t = wl.prefill_inputs(cfg)
    scale, gamma, alpha = 1.0 / np.sqrt(cfg.d), 1.0 / cfg.M, 2.0 / (cfg.M + cfg.N)
    a = prefill_strided(t, cfg.M, 20, FILTER_BUDGET, None, None, None, gamma, alpha, 20, scale, ("dense",) * 3)
    b = harness.prefill_on_gpu(t, cfg.M, None, None, None, scale, FILTER_BUDGET, 20, gamma, alpha, 20)
    for name in b:
        assert np.array_equal(a[name], b[name]), name


def initial_state(t):
    B, Lcap = t["protect"].shape
    return {"k": t["k_cache"].copy(), "v": t["v_cache"].copy(), "acc": np.zeros((B, Lcap), np.float32),
            "ids": np.tile(np.arange(Lcap, dtype=np.int32), (B, 1)), "protect": t["protect"].copy(),
            "len": t["len0"].copy()}


@pytest.mark.parametrize("kind,H,d", [("head_major", 32, 128), ("padded", 32, 128), ("head_major", 5, 64)])
def test_decode_loop_on_other_cache_layouts(kind, H, d):
    """Append + evict steps on a head-major / padded cache, every step from the oracle's state."""
    import torch
    import paper_2411_10803_amd as md
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[5], B=2, L0=300, steps=4, decode_budget=96, n_protect=20, H=H, d=d)
    t = wl.decode_inputs(cfg)
    s = initial_state(t)
    scale = 1 / np.sqrt(cfg.d)
    B, Lcap = s["ids"].shape
    for step in range(cfg.steps):
        dv = harness.decode_state_to_dev(s)
        kc, kcs = relayout(dv["k"], kind)
        vc, vcs = relayout(dv["v"], kind)
        if step > 0:
            md.mustdrop_decode_append_strided(harness.to_dev(t["k_new"][step], True), harness.to_dev(t["v_new"][step], True),
                                              kc, vc, dv["acc"], dv["ids"], dv["protect"], dv["len"], cfg.L0 + step)
            for b in range(cfg.B):
                n = s["len"][b]
                s["k"][b, n], s["v"][b, n] = t["k_new"][step][b], t["v_new"][step][b]
                s["acc"][b, n], s["ids"][b, n], s["protect"][b, n] = 0.0, cfg.L0 + step, 1
                s["len"][b] = n + 1
            assert np.array_equal(harness.to_host(kc.contiguous()), s["k"])
            assert np.array_equal(harness.to_host(vc.contiguous()), s["v"])
            assert np.array_equal(harness.to_host(dv["len"]), s["len"])
        ev = torch.full((B, Lcap), -1, dtype=torch.int32, device="cuda")
        evc = torch.zeros((B,), dtype=torch.int32, device="cuda")
        md.mustdrop_decode_evict_strided(harness.to_dev(t["q_steps"][step], True), kc, vc, dv["acc"], dv["ids"],
                                         dv["protect"], dv["len"], scale, 1.0, cfg.decode_budget, ev, evc)
        torch.cuda.synchronize()
        assert padding_intact(kc, kcs, kind) and padding_intact(vc, vcs, kind)
        dv["k"], dv["v"] = kc.contiguous(), vc.contiguous()
        g = harness.decode_state_to_host(dv, ev, evc)
        o = {k: v.copy() for k, v in s.items()}
        acc_pre = o["acc"].astype(np.float64)
        r = oracle.decode_evict(t["q_steps"][step], o["k"], o["v"], o["acc"], o["ids"], o["protect"], o["len"], scale,
                                1.0, cfg.decode_budget)
        o["acc_all"] = (acc_pre + r["a_t"]).astype(np.float32)
        o["evicted_ids"], o["evicted_count"] = r["evicted_ids"], r["evicted_count"]
        check_decode(g, o, s, cfg.decode_budget)
        assert np.all(g["len"] == cfg.decode_budget)
        s = {k: o[k] for k in ("k", "v", "acc", "ids", "protect", "len")}


@pytest.mark.parametrize("kind", ["head_major", "padded", "dense"])
def test_static_policy_on_other_cache_layouts(kind):
    """mustdrop_decode_keep_strided over three layers: bytes and indices only, bit for bit."""
    import torch
    import paper_2411_10803_amd as md
    from paper_2411_10803_amd import harness
    n_layers, B, Lcap, H, d = 3, 2, 333, 6, 64
    rng = np.random.default_rng(17)
    k = rng.integers(0, 1 << 16, size=(n_layers, B, Lcap, H, d), dtype=np.uint16) & np.uint16(0xBFFF)
    v = rng.integers(0, 1 << 16, size=(n_layers, B, Lcap, H, d), dtype=np.uint16) & np.uint16(0xBFFF)
    acc = rng.random((B, Lcap)).astype(np.float32)
    ids = np.stack([rng.permutation(4 * Lcap)[:Lcap] for _ in range(B)]).astype(np.int32)
    protect = (rng.random((B, Lcap)) < 0.3).astype(np.uint8)
    lens = np.array([Lcap, 200], dtype=np.int32)
    keep = (rng.random((B, Lcap)) < 0.4).astype(np.uint8)
    ko, vo, ao, io, po, lo = k.copy(), v.copy(), acc.copy(), ids.copy(), protect.copy(), lens.copy()
    o = oracle.decode_keep(ko, vo, keep, ao, io, po, lo)
    kd, kds = relayout(harness.to_dev(k, True), kind)
    vd, vds = relayout(harness.to_dev(v, True), kind)
    ad, idd, pd, ld = (harness.to_dev(a) for a in (acc, ids, protect, lens))
    ev = torch.full((B, Lcap), -1, dtype=torch.int32, device="cuda")
    evc = torch.zeros((B,), dtype=torch.int32, device="cuda")
    md.mustdrop_decode_keep_strided(kd, vd, harness.to_dev(keep), ad, idd, pd, ld, ev, evc)
    torch.cuda.synchronize()
    assert padding_intact(kd, kds, kind) and padding_intact(vd, vds, kind)
    assert np.array_equal(harness.to_host(ld), lo)
    kg, vg = harness.to_host(kd.contiguous()), harness.to_host(vd.contiguous())
    for b in range(B):
        n, ne = int(lo[b]), int(o["evicted_count"][b])
        for l in range(n_layers):
            assert np.array_equal(kg[l, b, :n], ko[l, b, :n]) and np.array_equal(vg[l, b, :n], vo[l, b, :n])
            assert np.array_equal(kg[l, b, lens[b]:], k[l, b, lens[b]:])
        assert np.array_equal(harness.to_host(idd)[b, :n], io[b, :n])
        assert np.array_equal(harness.to_host(pd)[b, :n], po[b, :n])
        assert np.array_equal(harness.to_host(ad)[b, :n], ao[b, :n])
        assert np.array_equal(harness.to_host(ev)[b, :ne], o["evicted_ids"][b, :ne])
