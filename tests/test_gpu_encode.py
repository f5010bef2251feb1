"""GPU parity: mustdrop_encode_merge (HIP, through the C ABI) against the CPU oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from parity import check_encode

pytestmark = pytest.mark.gpu


def both(x, x_dtype, q, k, qk_dtype, mass, valid, T, Hg, Wg, kt, kh, kw, tau, key_budget):
    from paper_2411_10803_amd import harness
    g = harness.encode_on_gpu(x, x_dtype, q, k, qk_dtype, mass, valid, T, Hg, Wg, kt, kh, kw, tau, key_budget)
    o = oracle.encode_merge(x, x_dtype, q, k, qk_dtype, mass, valid, T, Hg, Wg, kt, kh, kw, tau, key_budget)
    return g, o


def run_cfg(cfg, tau=None, valid=None, mass=None, key_budget=None, samples=None):
    e = wl.encode_inputs(cfg, samples)
    kb = cfg.key_budget if key_budget is None else key_budget
    tau = cfg.tau if tau is None else tau
    q, k = (e["q_cls"], e["k_cls"]) if kb > 0 else (None, None)
    g, o = both(e["x"], cfg.x_dtype, q, k, cfg.x_dtype, mass, valid, cfg.T, cfg.Hg, cfg.Wg,
                cfg.kt, cfg.kh, cfg.kw, tau, kb)
    s = check_encode(g, o, e["x"], cfg.x_dtype, valid, cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, tau, kb)
    return g, o, s


def median_tau(cfg):
    e = wl.encode_inputs(cfg)
    o = oracle.encode_merge(e["x"], cfg.x_dtype, None, None, cfg.x_dtype, None, None, cfg.T, cfg.Hg, cfg.Wg,
                            cfg.kt, cfg.kh, cfg.kw, 2.0, 0)
    return float(np.median(o["window_sim"]))


def test_config1_single_image_fp32():
    cfg = wl.CONFIGS[1]
    g, o, s = run_cfg(cfg)
    assert g["out_count"][0] == o["out_count"][0]
    # mixed decisions: threshold at the median similarity
    run_cfg(cfg, tau=median_tau(cfg))


def test_config2_batch16_bf16():
    cfg = wl.CONFIGS[2]
    g, o, s = run_cfg(cfg)
    assert np.array_equal(g["out_count"], o["out_count"]) or s["ambiguous_windows"] > 0
    run_cfg(cfg, tau=median_tau(cfg))


def test_config3_tiles_and_config4_video_windows():
    run_cfg(wl.tiny(wl.CONFIGS[3], B=2))
    cfg4 = wl.tiny(wl.CONFIGS[4], B=2)
    run_cfg(cfg4)
    run_cfg(cfg4, tau=median_tau(cfg4))


def test_ragged_padding_masses_and_small_shapes():
    # odd sizes: several tiles plus a ragged tail in every kernel, padding, non-unit masses
    cfg = wl.tiny(wl.CONFIGS[2], B=3, T=2, Hg=6, Wg=10, D=200, Hc=25, dc=8, kt=2, kh=3, kw=2, key_budget=7)
    rng = np.random.default_rng(5)
    valid = (rng.random((cfg.B, cfg.M)) > 0.2).astype(np.uint8)
    mass = rng.integers(1, 6, size=(cfg.B, cfg.M)).astype(np.float32)
    tau = median_tau(cfg)
    g, o, s = run_cfg(cfg, tau=tau, valid=valid, mass=mass)
    assert (g["out_count"] < valid.sum(1)).any()
    # garbage in the padding slots changes nothing
    e = wl.encode_inputs(cfg)
    x2, k2 = e["x"].copy(), e["k_cls"].copy()
    bad = valid == 0
    x2[bad] = 0x7FC0
    k2[:, 1:][bad] = 0x7F80
    from paper_2411_10803_amd import harness
    g2 = harness.encode_on_gpu(x2, cfg.x_dtype, e["q_cls"], k2, cfg.x_dtype, mass, valid, cfg.T, cfg.Hg, cfg.Wg,
                               cfg.kt, cfg.kh, cfg.kw, tau, cfg.key_budget)
    for name in ("out_count", "out_index", "out_mass", "out_is_key", "key_index"):
        assert np.array_equal(g[name], g2[name]), name
    for b in range(cfg.B):
        n = g["out_count"][b]
        assert np.array_equal(g["out_x"][b, :n], g2["out_x"][b, :n])


@pytest.mark.parametrize("kt,kh,kw", [(1, 1, 1), (1, 1, 2), (1, 2, 2), (2, 2, 2), (1, 3, 3), (1, 4, 4), (2, 2, 4)])
def test_window_shapes(kt, kh, kw):
    cfg = wl.tiny(wl.CONFIGS[4], B=2, T=4, Hg=12, Wg=12, D=256, Hc=4, dc=64, kt=kt, kh=kh, kw=kw, key_budget=9,
                  x_dtype=wl.F32)
    tau = median_tau(cfg) if kt * kh * kw > 1 else 0.5
    g, o, s = run_cfg(cfg, tau=tau)
    if kt * kh * kw == 1:
        assert np.all(g["out_count"] == cfg.M)


@pytest.mark.parametrize("T,Hg,Wg,kt,kh,kw,bf16", [
    (1, 27, 27, 1, 2, 2, True),      # a 27 x 27 patch grid under 2 x 2 windows: clipped last row and column
    (3, 7, 10, 2, 2, 4, False),      # clipped in all three directions
    (1, 5, 3, 1, 3, 4, False),       # window wider than the grid
    (5, 6, 6, 2, 2, 2, True),        # odd number of frames under frame pairs
    (1, 40, 33, 1, 2, 2, True),      # more than 1024 tokens: two rounds per thread in the decision kernel
])
def test_grids_the_window_does_not_divide(T, Hg, Wg, kt, kh, kw, bf16):
    cfg = wl.tiny(wl.CONFIGS[4], B=3, T=T, Hg=Hg, Wg=Wg, D=128, Hc=2, dc=64, kt=kt, kh=kh, kw=kw, key_budget=5,
                  x_dtype=wl.BF16 if bf16 else wl.F32)
    tau = median_tau(cfg)
    rng = np.random.default_rng(T * 100 + Hg)
    run_cfg(cfg, tau=tau)
    valid = (rng.random((cfg.B, cfg.M)) > 0.2).astype(np.uint8)
    mass = rng.integers(1, 5, size=(cfg.B, cfg.M)).astype(np.float32)
    run_cfg(cfg, tau=tau, valid=valid, mass=mass)
    run_cfg(cfg, tau=tau, valid=valid, mass=mass, key_budget=0)
    # every window merges: one survivor per window (all of them hold at least one token)
    g, o, s = run_cfg(cfg, tau=-2.0, key_budget=0)
    W = -(-T // kt) * -(-Hg // kh) * -(-Wg // kw)
    assert (g["out_count"] == W).all() and g["window_sim"].shape == (cfg.B, W)
    assert np.allclose(g["out_mass"][:, :W].sum(1), cfg.M)


def test_special_cases_and_key_budget_edges():
    from paper_2411_10803_amd import harness
    # constant image: everything merges; orthogonal tokens: nothing does
    D = 64
    row = np.linspace(0.5, 2.0, D, dtype=np.float32)
    x = np.broadcast_to(row, (2, 64, D)).copy()
    g = harness.encode_on_gpu(x, wl.F32, None, None, wl.F32, None, None, 1, 8, 8, 1, 2, 2, 0.999, 0)
    assert np.all(g["out_count"] == 16) and np.all(g["out_mass"][:, :16] == 4)
    assert np.array_equal(g["out_x"][:, :16], np.broadcast_to(row, (2, 16, D)))
    x = np.zeros((1, 64, D), dtype=np.float32)
    x[0, np.arange(64), np.arange(64)] = 2.0
    g = harness.encode_on_gpu(x, wl.F32, None, None, wl.F32, None, None, 1, 8, 8, 1, 2, 2, 1e-6, 0)
    assert g["out_count"][0] == 64 and np.array_equal(g["out_x"], x)
    # key budget = M (every token is a key -> nothing merges) and more keys asked than valid tokens
    cfg = wl.tiny(wl.CONFIGS[2], B=2, Hg=8, Wg=8, D=64, Hc=2, dc=32)
    g, o, _ = run_cfg(cfg, tau=-1.0, key_budget=cfg.M)
    assert np.all(g["out_count"] == cfg.M)
    valid = np.zeros((cfg.B, cfg.M), dtype=np.uint8)
    valid[:, :5] = 1
    g, o, _ = run_cfg(cfg, tau=-1.0, key_budget=9, valid=valid)
    assert np.array_equal(g["key_index"], o["key_index"]) and g["key_index"][0].tolist() == [0, 1, 2, 3, 4, -1, -1, -1, -1]
    # exact ties in a_cls: lower index wins (zero query -> uniform attention)
    e = wl.encode_inputs(cfg)
    q0 = np.zeros_like(e["q_cls"])
    g = harness.encode_on_gpu(e["x"], cfg.x_dtype, q0, e["k_cls"], cfg.x_dtype, None, None, 1, 8, 8, 1, 2, 2, 2.0, 6)
    assert g["key_index"].tolist() == [[0, 1, 2, 3, 4, 5]] * 2


def test_determinism():
    cfg = wl.CONFIGS[2]
    e = wl.encode_inputs(cfg, samples=[0, 1, 2, 3])
    from paper_2411_10803_amd import harness
    runs = [harness.encode_on_gpu(e["x"], cfg.x_dtype, e["q_cls"], e["k_cls"], cfg.x_dtype, None, None,
                                  1, 24, 24, 1, 2, 2, 0.9, 32) for _ in range(3)]
    for r in runs[1:]:
        for name in ("out_x", "out_index", "out_mass", "out_count", "key_index", "a_cls", "window_sim"):
            assert np.array_equal(runs[0][name], r[name]), name


@pytest.mark.parametrize("shape", ["cfg2_slice", "ragged_small", "long_general"])
def test_adaptive_key_threshold(shape):
    """Eq. 7 as printed: keys = {a_cls > mean + lambda * std}, several lambdas, with and without padding."""
    from paper_2411_10803_amd import harness
    if shape == "cfg2_slice":
        cfg, samples = wl.CONFIGS[2], [0, 5, 11]
    elif shape == "ragged_small":
        cfg, samples = wl.tiny(wl.CONFIGS[2], B=3, T=2, Hg=6, Wg=10, D=200, Hc=25, dc=8, kt=2, kh=3, kw=2), None
    else:                                            # more than 8192 tokens per sample: the general kernels
        cfg, samples = wl.tiny(wl.CONFIGS[2], B=1, T=1, Hg=96, Wg=96, D=64, Hc=4, dc=16), None
    e = wl.encode_inputs(cfg, samples)
    B = e["x"].shape[0]
    rng = np.random.default_rng(9)
    tau = median_tau(cfg) if samples is None else cfg.tau
    for lam, masked, cap in ((0.0, False, cfg.M), (1.0, True, cfg.M), (2.5, False, 4), (-0.5, True, 7), (50.0, False, 0)):
        valid = (rng.random((B, cfg.M)) > 0.2).astype(np.uint8) if masked else None
        g = harness.encode_adaptive_on_gpu(e["x"], cfg.x_dtype, e["q_cls"], e["k_cls"], cfg.x_dtype, None, valid,
                                           cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, tau, lam, cap)
        o = oracle.encode_merge_adaptive(e["x"], cfg.x_dtype, e["q_cls"], e["k_cls"], cfg.x_dtype, None, valid,
                                         cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, tau, lam, cap)
        check_encode(g, o, e["x"], cfg.x_dtype, valid, cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, tau, cap,
                     key_lambda=lam)
        if lam == 50.0:
            assert np.all(g["key_count"] == 0)
