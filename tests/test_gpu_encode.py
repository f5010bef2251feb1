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


def clear_tau(sims, q=0.5):
    """A threshold near the q-quantile of the oracle's window similarities that no similarity comes closer to
    than twice the margin: every merge decision is then decisive."""
    v = np.sort(np.asarray(sims, dtype=np.float64).ravel())
    i0 = int(q * (v.size - 1))
    for step in range(v.size):
        for i in (i0 + step, i0 - step):
            if 0 <= i < v.size - 1 and v[i + 1] - v[i] > 4e-3:
                return float(np.float32(0.5 * (v[i] + v[i + 1])))
    raise AssertionError("no gap between the window similarities")


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


@pytest.mark.parametrize("Hg,Wg", [(1, 3), (3, 5), (7, 9)])
def test_adaptive_rule_is_strict_at_an_exact_tie(Hg, Wg):
    """Eq. 7 prints '>'.  One head, a zero CLS query, M = 2^k - 1 tokens: every a_cls is exactly 1/(M+1),
    so mu == a_cls in fp32 as in fp64 and the key set must be empty for any lambda (the oracle's pin, here
    through the fp32 kernels)."""
    from paper_2411_10803_amd import harness
    M, D = Hg * Wg, 16
    rng = np.random.default_rng(M)
    x = rng.standard_normal((2, M, D)).astype(np.float32)
    k = np.ascontiguousarray(rng.standard_normal((2, 1 + M, 1, D)).astype(np.float32))
    q = np.zeros((2, 1, D), dtype=np.float32)
    for lam in (-1.0, 0.0, 2.0):
        g = harness.encode_adaptive_on_gpu(x, wl.F32, q, k, wl.F32, None, None, 1, Hg, Wg, 1, 1, 1, 2.0, lam, M)
        o = oracle.encode_merge_adaptive(x, wl.F32, q, k, wl.F32, None, None, 1, Hg, Wg, 1, 1, 1, 2.0, lam, M)
        assert np.all(o["key_count"] == 0)
        assert np.all(g["a_cls"] == np.float32(1.0 / (M + 1)))
        assert np.all(g["key_count"] == 0) and np.all(g["key_index"] == -1) and g["out_is_key"].sum() == 0
        assert np.array_equal(g["out_count"], o["out_count"])


def _second_call_inputs(o1, cls_row, Hc, dc):
    B, M, D = o1["out_x"].shape
    k2 = np.concatenate([cls_row.reshape(B, 1, D), o1["out_x"]], axis=1).reshape(B, 1 + M, Hc, dc)
    return o1["out_x"], np.ascontiguousarray(k2), o1["out_mass"], o1["out_valid"]


@pytest.mark.parametrize("which", ["small_f32", "cfg2_bf16"])
def test_paper_order_merge_then_keys_as_a_chain(which):
    """Sec. 3.3 in the paper's order, each side running its own chain: a merging call without keys, then a
    key-selection call (1x1x1 windows) on that call's out_x / out_valid / out_mass as a 1 x 1 x M grid."""
    from paper_2411_10803_amd import harness
    if which == "small_f32":
        cfg = wl.tiny(wl.CONFIGS[2], B=3, Hg=10, Wg=14, D=128, Hc=8, dc=16, x_dtype=wl.F32, key_budget=9)
    else:
        cfg = wl.tiny(wl.CONFIGS[2], B=4)
    e = wl.encode_inputs(cfg)
    dt, M = cfg.x_dtype, cfg.M
    tau = clear_tau(oracle.encode_merge(e["x"], dt, None, None, dt, None, None, cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh,
                                        cfg.kw, 2.0, 0)["window_sim"], 0.5 if which == "small_f32" else 0.3)
    a1 = (cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, tau, 0)
    g1, o1 = both(e["x"], dt, None, None, dt, None, None, *a1)
    s1 = check_encode(g1, o1, e["x"], dt, None, *a1)
    assert s1["ambiguous_windows"] == 0 and np.array_equal(g1["out_count"], o1["out_count"])
    assert o1["out_count"].sum() < cfg.B * M and o1["out_count"].min() > cfg.key_budget
    a2 = (1, 1, M, 1, 1, 1, 5.0, cfg.key_budget)
    gx, gk, gm, gv = _second_call_inputs(g1, e["q_cls"], cfg.Hc, cfg.dc)
    ox, ok, om, ov = _second_call_inputs(o1, e["q_cls"], cfg.Hc, cfg.dc)
    g2 = harness.encode_on_gpu(gx, dt, e["q_cls"], gk, dt, gm, gv, *a2)
    o2 = oracle.encode_merge(ox, dt, e["q_cls"], ok, dt, om, ov, *a2)
    check_encode(g2, o2, gx, dt, gv, *a2)
    for b in range(cfg.B):
        n = int(g1["out_count"][b])
        assert g2["out_count"][b] == n
        assert np.array_equal(g2["out_x"][b, :n], g1["out_x"][b, :n])       # nothing merges: rows pass through
        assert np.array_equal(g2["out_mass"][b, :n], g1["out_mass"][b, :n])
        assert g2["out_mass"][b, :n].sum() == M                            # mass conserved over both calls
        keys = g2["key_index"][b]
        assert np.all(keys >= 0) and np.all(keys < n) and g2["out_is_key"][b, :n].sum() == cfg.key_budget


def test_hierarchical_remerge_with_carried_masses():
    """A second merging call on the survivors of the first (laid out as a 1 x 1 x M row, windows of four,
    masses carried): each side runs its own chain; mass and the mass-weighted feature sum are conserved."""
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[2], B=3, Hg=12, Wg=12, D=256, Hc=4, dc=64, x_dtype=wl.F32)
    e = wl.encode_inputs(cfg)
    dt, M = cfg.x_dtype, cfg.M
    a1 = (1, cfg.Hg, cfg.Wg, 1, 2, 2, clear_tau(oracle.encode_merge(e["x"], dt, None, None, dt, None, None, 1, cfg.Hg,
                                                                    cfg.Wg, 1, 2, 2, 2.0, 0)["window_sim"]), 0)
    g1, o1 = both(e["x"], dt, None, None, dt, None, None, *a1)
    s1 = check_encode(g1, o1, e["x"], dt, None, *a1)
    assert s1["ambiguous_windows"] == 0 and o1["out_count"].sum() < cfg.B * M
    sims2 = oracle.encode_merge(o1["out_x"], dt, None, None, dt, o1["out_mass"], o1["out_valid"],
                                1, 1, M, 1, 1, 4, 2.0, 0)["window_sim"]
    live = np.concatenate([sims2[b, : int(o1["out_count"][b]) // 4] for b in range(cfg.B)])
    a2 = (1, 1, M, 1, 1, 4, clear_tau(live), 0)
    g2 = harness.encode_on_gpu(g1["out_x"], dt, None, None, dt, g1["out_mass"], g1["out_valid"], *a2)
    o2 = oracle.encode_merge(o1["out_x"], dt, None, None, dt, o1["out_mass"], o1["out_valid"], *a2)
    s2 = check_encode(g2, o2, g1["out_x"], dt, g1["out_valid"], *a2)
    assert s2["merged_rows_checked"] > 10
    assert g2["out_count"].sum() < g1["out_count"].sum() and g2["out_mass"].max() > 4.0
    tot = e["x"].astype(np.float64).sum(1)
    for b in range(cfg.B):
        n2 = int(g2["out_count"][b])
        assert g2["out_mass"][b, :n2].sum() == M
        lhs = (g2["out_mass"][b, :n2, None].astype(np.float64) * g2["out_x"][b, :n2]).sum(0)
        assert np.allclose(lhs, tot[b], rtol=1e-4, atol=1e-3)
