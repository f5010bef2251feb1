"""The input generators: determinism, shapes, and the closed form that ties the random field to the
window similarity the oracle computes (checks generator and cosine code together)."""
import numpy as np
import pytest

import oracle
import workloads as wl


def test_configs_have_the_benchmark_shapes():
    c = wl.CONFIGS
    assert (c[1].B, c[1].M, c[1].N, c[1].x_dtype, c[1].budgets) == (1, 576, 32, wl.F32, (192,))
    assert (c[2].B, c[2].M, c[2].N, c[2].budgets) == (16, 576, 64, (192, 128, 64))
    assert (c[3].B, c[3].M, c[3].N, c[3].key_budget, c[3].budgets) == (8, 2880, 128, 128, (320,))
    assert (c[4].B, c[4].M, (c[4].kt, c[4].kh, c[4].kw), c[4].budgets) == (4, 4608, (2, 2, 2), (512,))
    assert (c[5].B, c[5].L0, c[5].steps, c[5].decode_budget) == (64, 4096, 256, 1024)
    for i in (1, 2, 3, 4, 5):
        assert (c[i].H, c[i].d, c[i].C, c[i].D) == (32, 128, 4096, 1024)


def test_generators_are_seeded_and_subsets_match_the_full_batch():
    cfg = wl.tiny(wl.CONFIGS[2], B=3, Hg=6, Wg=6, D=32, Hc=4, dc=8, N=4, H=2, d=8, C=16)
    a, b = wl.encode_inputs(cfg), wl.encode_inputs(cfg)
    assert np.array_equal(a["x"], b["x"]) and np.array_equal(a["k_cls"], b["k_cls"])
    sub = wl.encode_inputs(cfg, samples=[2])
    assert np.array_equal(sub["x"][0], a["x"][2])
    p, ps = wl.prefill_inputs(cfg), wl.prefill_inputs(cfg, samples=[1])
    assert np.array_equal(ps["k"][0], p["k"][1]) and p["k"].shape == (3, 40, 2, 8)
    assert np.array_equal(a["k_cls"][:, 1:].reshape(3, 36, 32), a["x"])     # synthetic keys = the features


@pytest.mark.parametrize("ell,expect", [(1.0, 0.715), (2.0, 0.911), (4.0, 0.970)])
def test_field_correlation_closed_form(ell, expect):
    # white noise smoothed by a Gaussian of std ell has autocorrelation exp(-r^2 / (4 ell^2)); with
    # N(0, sigma_n^2) noise on top, E cos(x_p, x_q) ~ rho(r) / (1 + sigma_n^2).  A 2x2 window has four
    # pairs at r = 1 and two at r = sqrt(2).
    cfg = wl.tiny(wl.CONFIGS[1], ell=(ell, ell))
    e = wl.encode_inputs(cfg)
    rho = lambda r2: np.exp(-r2 / (4 * ell * ell)) / (1 + cfg.sigma_n ** 2)
    closed = (4 * rho(1.0) + 2 * rho(2.0)) / 6
    assert closed == pytest.approx(expect, abs=2e-3)
    o = oracle.encode_merge(e["x"], cfg.x_dtype, None, None, cfg.x_dtype, None, None,
                            1, 24, 24, 1, 2, 2, 2.0, 0)
    assert o["window_sim"].mean() == pytest.approx(closed, abs=5e-3)
    assert o["window_sim"].std() < 3.0 / np.sqrt(cfg.D)                      # concentration ~ 1/sqrt(D)


def test_video_and_tile_fields_are_redundant_across_frames():
    cfg = wl.tiny(wl.CONFIGS[4], B=1, D=256, Hc=4, dc=64)
    x, _, _ = wl.vision_features(cfg)
    f = x[0].reshape(8, 576, 256)
    cos = (f[0] * f[1]).sum(-1) / np.linalg.norm(f[0], axis=-1) / np.linalg.norm(f[1], axis=-1)
    assert cos.mean() > 0.99                                                 # drift sigma = 0.05 per frame
    cfg = wl.tiny(wl.CONFIGS[3], B=1, D=256, Hc=4, dc=64)
    x, _, _ = wl.vision_features(cfg)
    f = x[0].reshape(5, 576, 256)
    cos = (f[0] * f[3]).sum(-1) / np.linalg.norm(f[0], axis=-1) / np.linalg.norm(f[3], axis=-1)
    assert 0.35 < cos.mean() < 0.65                                          # half the variance is shared


def test_decode_inputs_plant_heavy_hitters():
    cfg = wl.tiny(wl.CONFIGS[5], B=2, L0=256, steps=3, H=2, d=128, n_protect=8)
    t = wl.decode_inputs(cfg)
    assert t["k_cache"].shape == (2, 259, 2, 128) and t["q_steps"].shape == (3, 2, 2, 128)
    k = wl.bf16_bits_to_f32(t["k_cache"]).astype(np.float64)
    q = wl.bf16_bits_to_f32(t["q_steps"]).astype(np.float64)
    lg = np.einsum("bhc,bjhc->bhj", q[0], k[:, :256]) / np.sqrt(128)
    for b in range(2):
        hv = t["heavy"][b] == 1
        gap = lg[b][:, hv].mean() - lg[b][:, ~hv].mean()
        assert 2.5 < gap < 3.5                                               # about +3 sigma of unit logits
        assert t["protect"][b].sum() == 8
    assert np.all(np.isfinite(wl.bf16_bits_to_f32(t["v_cache"])))
