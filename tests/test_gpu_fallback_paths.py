"""GPU parity on shapes that take the general (not register-resident / not streaming) kernels:
more than 8192 tokens or cache entries per sample, head counts and head sizes outside the fast set."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import FILTER_BUDGET
from parity import check_decode, check_encode, check_prefill

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T,Hg,Wg", [(4, 48, 48), (3, 55, 53)])      # the second: windows clipped in every direction
def test_encode_more_than_8192_tokens_per_sample(T, Hg, Wg):
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[4], B=2, T=T, Hg=Hg, Wg=Wg, D=64, Hc=2, dc=32, kt=2, kh=2, kw=2, key_budget=40)
    assert cfg.M > 8192
    e = wl.encode_inputs(cfg)
    args = (cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, 0.9, cfg.key_budget)
    g = harness.encode_on_gpu(e["x"], cfg.x_dtype, e["q_cls"], e["k_cls"], cfg.x_dtype, None, None, *args)
    o = oracle.encode_merge(e["x"], cfg.x_dtype, e["q_cls"], e["k_cls"], cfg.x_dtype, None, None, *args)
    s = check_encode(g, o, e["x"], cfg.x_dtype, None, *args)
    assert s["merged_rows_checked"] + s["copied_rows_checked"] > 1000


@pytest.mark.parametrize("T,Hg,Wg,Hc", [(2, 64, 64, 4), (1, 75, 80, 8), (1, 75, 80, 2)])
def test_encode_between_4608_and_8192_tokens_per_sample(T, Hg, Wg, Hc):
    # the register-resident decision kernel at eight tokens per thread, where its dynamic LDS exceeds 64 KiB
    # (8192 and 6000 tokens); with a head count that is not a multiple of 4 the general kernel takes over
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[4], B=2, T=T, Hg=Hg, Wg=Wg, D=64, Hc=Hc, dc=64 // Hc, kt=1 if T == 1 else 2, kh=2, kw=2, key_budget=70)
    assert 4608 < cfg.M <= 8192
    e = wl.encode_inputs(cfg)
    rng = np.random.default_rng(5)
    valid = (rng.random((cfg.B, cfg.M)) > 0.1).astype(np.uint8)
    for v in (None, valid):
        args = (cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, 0.9, cfg.key_budget)
        g = harness.encode_on_gpu(e["x"], cfg.x_dtype, e["q_cls"], e["k_cls"], cfg.x_dtype, None, v, *args)
        o = oracle.encode_merge(e["x"], cfg.x_dtype, e["q_cls"], e["k_cls"], cfg.x_dtype, None, v, *args)
        s = check_encode(g, o, e["x"], cfg.x_dtype, v, *args)
        assert s["merged_rows_checked"] + s["copied_rows_checked"] > 1000


def test_prefill_more_than_8192_vision_tokens():
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[2], B=1, T=1, Hg=92, Wg=92, N=20, H=2, d=64, C=64)
    Mv = cfg.M
    assert Mv > 8192
    t = wl.prefill_inputs(cfg)
    is_key = wl.random_key_mask(cfg, 50)
    scale, gamma, alpha = 1 / 8.0, 1.0 / Mv, 2.0 / cfg.L
    for R in (300, 1000):
        g = harness.prefill_on_gpu(t, Mv, None, None, is_key, scale, FILTER_BUDGET, R, gamma, alpha, R)
        o = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], None, None, is_key, Mv, scale,
                                  FILTER_BUDGET, R, gamma, alpha, R)
        check_prefill(g, o, t, Mv, None, is_key, FILTER_BUDGET, R, gamma, alpha, R)
        assert g["kept_count"][0] == R


@pytest.mark.parametrize("H,d,L0", [(2, 64, 300), (32, 64, 500), (8, 256, 200), (1, 128, 9000), (32, 128, 9000),
                                    (5, 64, 700), (40, 128, 600), (28, 128, 1300)])
def test_decode_general_kernels(H, d, L0):
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[5], B=2, L0=L0, steps=1, decode_budget=L0 // 3, n_protect=L0 // 10, H=H, d=d)
    t = wl.decode_inputs(cfg)
    B, Lcap = cfg.B, t["Lcap"]
    s0 = {"k": t["k_cache"], "v": t["v_cache"], "acc": np.zeros((B, Lcap), np.float32),
          "ids": np.tile(np.arange(Lcap, dtype=np.int32), (B, 1)), "protect": t["protect"].copy(), "len": t["len0"].copy()}
    scale = 1.0 / np.sqrt(d)
    dv = harness.decode_state_to_dev(s0)
    ev, evc = harness.decode_on_gpu(harness.to_dev(t["q_steps"][0], True), dv, scale, 1.0, cfg.decode_budget)
    g = harness.decode_state_to_host(dv, ev, evc)
    o = {k_: v_.copy() for k_, v_ in s0.items()}
    r = oracle.decode_evict(t["q_steps"][0], o["k"], o["v"], o["acc"], o["ids"], o["protect"], o["len"], scale, 1.0,
                            cfg.decode_budget)
    o["acc_all"] = r["a_t"].astype(np.float32)
    o["evicted_ids"], o["evicted_count"] = r["evicted_ids"], r["evicted_count"]
    check_decode(g, o, s0, cfg.decode_budget)
    assert np.all(g["len"] == cfg.decode_budget)


@pytest.mark.parametrize("Hg,Wg", [(50, 54), (70, 80)])          # 2700 and 5600 vision tokens: 3 and 6 tokens per thread
def test_prefill_selection_forms_between_the_powers_of_two(Hg, Wg):
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[2], B=2, T=1, Hg=Hg, Wg=Wg, N=20, H=2, d=64, C=64)
    Mv = cfg.M
    t = wl.prefill_inputs(cfg)
    is_key = wl.random_key_mask(cfg, 40)
    rng = np.random.default_rng(11)
    vis = (rng.random((cfg.B, Mv)) > 0.15).astype(np.uint8)
    scale, gamma, alpha = 1 / 8.0, 1.0 / Mv, 2.0 / cfg.L
    R = 400
    g = harness.prefill_on_gpu(t, Mv, vis, None, is_key, scale, FILTER_BUDGET, R, gamma, alpha, R)
    o = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], vis, None, is_key, Mv, scale,
                              FILTER_BUDGET, R, gamma, alpha, R)
    check_prefill(g, o, t, Mv, vis, is_key, FILTER_BUDGET, R, gamma, alpha, R)
    assert np.all(g["kept_count"] == R)


@pytest.mark.parametrize("L0", [2500, 5600])                     # streaming kernels with 3 and 6 entries per thread
def test_decode_selection_forms_between_the_powers_of_two(L0):
    test_decode_general_kernels(4, 128, L0)
