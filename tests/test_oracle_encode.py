"""Pins for the stage-1 oracle (Sec. 3.3: Local Spatial Merging, Eq. 5; Key Retaining, Eq. 6-7).

The paper prints no worked example, so the oracle is pinned by closed forms,
invariants, library routines and pure-Python brute force on tiny grids."""
from fractions import Fraction
from itertools import combinations

import numpy as np
import pytest

import oracle
import workloads as wl
from workloads import BF16, F32


def run(x, T, Hg, Wg, kt=1, kh=2, kw=2, tau=0.5, key_budget=0, q=None, k=None, mass=None, valid=None,
        dtype=F32, qk_dtype=None):
    return oracle.encode_merge(x, dtype, q, k, dtype if qk_dtype is None else qk_dtype, mass, valid,
                               T, Hg, Wg, kt, kh, kw, tau, key_budget)


def rand_tokens(rng, B, M, D):
    return rng.standard_normal((B, M, D)).astype(np.float32)


# ---------------------------------------------------------------- special cases
def test_constant_image_merges_every_window():
    # all tokens equal -> every pairwise cosine is 1 -> every window merges (tau < 1)
    T, Hg, Wg, D = 2, 4, 6, 16
    row = np.linspace(0.5, 2.0, D, dtype=np.float32)
    x = np.broadcast_to(row, (1, T * Hg * Wg, D)).copy()
    for (kt, kh, kw) in [(1, 2, 2), (2, 2, 2), (1, 2, 3)]:
        o = run(x, T, Hg, Wg, kt, kh, kw, tau=0.999)
        ws = kt * kh * kw
        n = T * Hg * Wg // ws
        assert o["out_count"][0] == n
        assert np.allclose(o["window_sim"], 1.0, atol=1e-12)
        assert np.all(o["out_mass"][0, :n] == ws)
        assert np.array_equal(o["out_x"][0, :n], np.broadcast_to(row, (n, D)))
        # representative sits at the lowest member index (top-left, earliest frame)
        exp_idx = sorted(((wt * kt) * Hg + wy * kh) * Wg + wx * kw
                         for wt in range(T // kt) for wy in range(Hg // kh) for wx in range(Wg // kw))
        assert o["out_index"][0, :n].tolist() == exp_idx


def test_orthogonal_tokens_merge_nothing():
    Hg = Wg = 4
    x = np.eye(16, dtype=np.float32)[None] * 3.0
    o = run(x, 1, Hg, Wg, tau=1e-9)
    assert o["out_count"][0] == 16
    assert np.array_equal(o["out_x"], x)
    assert np.array_equal(o["out_index"][0], np.arange(16))
    assert np.all(o["window_sim"] == 0.0)
    assert np.all(o["out_mass"] == 1.0)


def test_pair_count_and_mean_over_unordered_pairs():
    # window = {a, a, b, b} with a orthogonal to b: 2 of the C(4,2)=6 pairs have cosine 1 -> S = 1/3
    a = np.array([1, 0, 0, 0], dtype=np.float32)
    b = np.array([0, 2, 0, 0], dtype=np.float32)
    x = np.stack([a, a, b, b])[None]          # grid 2x2
    o = run(x, 1, 2, 2, tau=0.9)
    assert o["window_sim"][0, 0] == pytest.approx(1.0 / 3.0, abs=1e-15)
    # 2x2x2 window {a x4, b x4}: 2*C(4,2)=12 of the C(8,2)=28 pairs are 1
    x8 = np.stack([a, a, b, b, a, b, a, b])[None]
    o = run(x8, 2, 2, 2, kt=2, tau=0.9)
    assert o["window_sim"][0, 0] == pytest.approx(12.0 / 28.0, abs=1e-15)
    # strict ">" in Eq. 5: S == tau does not merge
    c = np.array([1, 0], dtype=np.float32)
    x2 = np.stack([c, c, c, c])[None]
    assert run(x2, 1, 2, 2, tau=1.0)["out_count"][0] == 4
    assert run(x2, 1, 2, 2, tau=np.nextafter(np.float32(1), np.float32(0)))["out_count"][0] == 1


def test_zero_norm_token_has_cosine_zero():
    x = np.zeros((1, 4, 4), dtype=np.float32)
    x[0, 0] = [1, 0, 0, 0]
    x[0, 1] = [1, 0, 0, 0]
    o = run(x, 1, 2, 2, tau=0.0)
    assert o["window_sim"][0, 0] == pytest.approx(1.0 / 6.0)


# ---------------------------------------------------------------- library pin
def test_window_sim_matches_sklearn_cosine():
    from sklearn.metrics.pairwise import cosine_similarity
    rng = np.random.default_rng(3)
    T, Hg, Wg, D = 2, 4, 4, 32
    base = rng.standard_normal((1, 1, D))
    x = (base + 0.7 * rng.standard_normal((1, T * Hg * Wg, D))).astype(np.float32)
    for (kt, kh, kw) in [(1, 2, 2), (2, 2, 2), (1, 4, 2)]:
        o = run(x, T, Hg, Wg, kt, kh, kw, tau=2.0)
        w = 0
        for wt in range(T // kt):
            for wy in range(Hg // kh):
                for wx in range(Wg // kw):
                    mem = [((wt * kt + dt) * Hg + wy * kh + dy) * Wg + wx * kw + dx
                           for dt in range(kt) for dy in range(kh) for dx in range(kw)]
                    cs = cosine_similarity(x[0, mem].astype(np.float64))
                    iu = np.triu_indices(len(mem), 1)
                    assert o["window_sim"][0, w] == pytest.approx(cs[iu].mean(), abs=1e-12)
                    w += 1


# ---------------------------------------------------------------- brute force
def brute_encode(x, T, Hg, Wg, kt, kh, kw, tau, keys, mass, valid):
    """Pure-Python enumeration of windows, pairs and merges for one sample (float64 lists)."""
    M, D = len(x), len(x[0])
    merged_into = {}
    for wt in range(-(-T // kt)):
        for wy in range(-(-Hg // kh)):
            for wx in range(-(-Wg // kw)):
                mem = [((wt * kt + dt) * Hg + wy * kh + dy) * Wg + wx * kw + dx
                       for dt in range(kt) for dy in range(kh) for dx in range(kw)
                       if wt * kt + dt < T and wy * kh + dy < Hg and wx * kw + dx < Wg]      # border windows are clipped
                mem = [m for m in mem if valid[m]]
                if len(mem) < 2 or any(m in keys for m in mem):
                    continue
                tot = 0.0
                pairs = list(combinations(mem, 2))
                for (m, n) in pairs:
                    dot = sum(float(x[m][c]) * float(x[n][c]) for c in range(D))
                    nm = sum(float(x[m][c]) ** 2 for c in range(D)) ** 0.5
                    nn = sum(float(x[n][c]) ** 2 for c in range(D)) ** 0.5
                    tot += dot / (nm * nn) if nm > 0 and nn > 0 else 0.0
                if tot / len(pairs) > tau:
                    merged_into[min(mem)] = mem
    absorbed = {m for mem in merged_into.values() for m in mem}
    rows = []
    for t in range(M):
        if not valid[t]:
            continue
        if t in merged_into:
            mem = merged_into[t]
            ms = sum(mass[m] for m in mem)
            rows.append((t, ms, [sum(mass[m] * float(x[m][c]) for m in mem) / ms for c in range(D)], 0))
        elif t not in absorbed:
            rows.append((t, mass[t], [float(v) for v in x[t]], int(t in keys)))
    return rows


@pytest.mark.parametrize("T,Hg,Wg,kt", [(1, 6, 6, 1), (2, 4, 6, 2), (1, 5, 7, 1), (3, 3, 5, 2)])
def test_brute_force_tiny_grids(T, Hg, Wg, kt):
    rng = np.random.default_rng(11 + T)
    M, D = T * Hg * Wg, 8
    base = rng.standard_normal((1, 1, D))
    x = (base + 0.6 * rng.standard_normal((2, M, D))).astype(np.float32)
    mass = rng.integers(1, 4, size=(2, M)).astype(np.float32)
    valid = (rng.random((2, M)) > 0.15).astype(np.uint8)
    k = rng.standard_normal((2, 1 + M, 2, 4)).astype(np.float32)
    q = rng.standard_normal((2, 2, 4)).astype(np.float32)
    sims = np.sort(run(x, T, Hg, Wg, kt, 2, 2, tau=2.0, valid=valid)["window_sim"].ravel())
    tau = float(0.5 * (sims[len(sims) // 2 - 1] + sims[len(sims) // 2]))   # mid-gap: no near-tie
    n_merged_total = 0
    o = run(x, T, Hg, Wg, kt, 2, 2, tau=tau, key_budget=3, q=q, k=k, mass=mass, valid=valid)
    for b in range(2):
        keys = set(int(i) for i in o["key_index"][b] if i >= 0)
        rows = brute_encode(x[b].tolist(), T, Hg, Wg, kt, 2, 2, tau, keys, mass[b].tolist(), valid[b].tolist())
        n = o["out_count"][b]
        assert n == len(rows)
        n_merged_total += int(valid[b].sum()) - n
        for s, (idx, ms, feat, isk) in enumerate(rows):
            assert o["out_index"][b, s] == idx
            assert o["out_mass"][b, s] == pytest.approx(ms)
            assert o["out_is_key"][b, s] == isk
            assert np.allclose(o["out_x"][b, s], feat, rtol=1e-6, atol=1e-7)
        assert o["out_valid"][b].tolist() == [1] * n + [0] * (M - n)
    assert n_merged_total > 0          # the case does merge something
    assert (o["window_sim"] <= tau).any()  # ... and leaves something unmerged


def test_grid_the_window_does_not_divide_equals_the_padded_grid():
    """A grid that the window does not divide behaves like the next larger grid that it does divide, with
    the added cells marked as padding (clipped border windows hold fewer tokens)."""
    rng = np.random.default_rng(23)
    T, Hg, Wg, kt, kh, kw, D = 3, 5, 7, 2, 2, 3, 16
    Tp, Hp, Wp = 4, 6, 9
    M, Mp = T * Hg * Wg, Tp * Hp * Wp
    base = rng.standard_normal((1, 1, D))
    x = (base + 0.5 * rng.standard_normal((2, M, D))).astype(np.float32)
    mass = rng.integers(1, 4, size=(2, M)).astype(np.float32)
    valid = (rng.random((2, M)) > 0.1).astype(np.uint8)
    # the same tokens placed in the padded grid; pad cells hold garbage and are invalid
    pos = np.array([((t * Hp) + y) * Wp + xx for t in range(T) for y in range(Hg) for xx in range(Wg)])
    xp = np.full((2, Mp, D), np.nan, np.float32)
    mp = np.full((2, Mp), 7.0, np.float32)
    vp = np.zeros((2, Mp), np.uint8)
    xp[:, pos], mp[:, pos], vp[:, pos] = x, mass, valid
    k = rng.standard_normal((2, 1 + M, 2, 8)).astype(np.float32)
    q = rng.standard_normal((2, 2, 8)).astype(np.float32)
    kp = np.full((2, 1 + Mp, 2, 8), np.nan, np.float32)
    kp[:, 0], kp[:, 1 + pos] = k[:, 0], k[:, 1:]
    sims = np.sort(run(x, T, Hg, Wg, kt, kh, kw, tau=2.0, valid=valid)["window_sim"].ravel())
    tau = float(0.5 * (sims[len(sims) // 2 - 1] + sims[len(sims) // 2]))
    a = run(x, T, Hg, Wg, kt, kh, kw, tau=tau, key_budget=4, q=q, k=k, mass=mass, valid=valid)
    b = run(xp, Tp, Hp, Wp, kt, kh, kw, tau=tau, key_budget=4, q=q, k=kp, mass=mp, valid=vp)
    assert a["window_sim"].shape == b["window_sim"].shape == (2, 2 * 3 * 3)
    assert np.array_equal(a["window_sim"], b["window_sim"])
    assert np.array_equal(a["out_count"], b["out_count"]) and (a["out_count"] < valid.sum(1)).all()
    for s in range(2):
        n = a["out_count"][s]
        assert np.array_equal(pos[a["out_index"][s, :n]], b["out_index"][s, :n])
        assert np.array_equal(pos[a["key_index"][s]], b["key_index"][s])
        for name in ("out_mass", "out_is_key", "out_x"):
            assert np.array_equal(a[name][s, :n], b[name][s, :n]), name


def test_window_wider_than_the_grid_is_one_clipped_window():
    # 1 x 3 x 3 grid under a 1 x 4 x 4 window: a single window of nine tokens, 36 pairs
    rng = np.random.default_rng(29)
    from sklearn.metrics.pairwise import cosine_similarity
    x = rng.standard_normal((1, 9, 12)).astype(np.float32)
    o = run(x, 1, 3, 3, 1, 4, 4, tau=-2.0)
    assert o["window_sim"].shape == (1, 1) and o["out_count"][0] == 1 and o["out_mass"][0, 0] == 9.0
    cs = cosine_similarity(x[0].astype(np.float64))
    assert o["window_sim"][0, 0] == pytest.approx(cs[np.triu_indices(9, 1)].mean(), abs=1e-12)
    assert np.allclose(o["out_x"][0, 0], x[0].astype(np.float64).mean(0), rtol=1e-6)


# ---------------------------------------------------------------- invariants
def smooth_case(B=2, Hg=8, Wg=8, T=2, D=64, seed=5):
    cfg = wl.tiny(wl.CONFIGS[2], B=B, Hg=Hg, Wg=Wg, T=T, D=D, Hc=4, dc=D // 4, x_dtype=F32,
                  field_kind="video", key_budget=5)
    return cfg, wl.encode_inputs(cfg)


def test_mass_and_weighted_sum_are_conserved():
    cfg, e = smooth_case()
    rng = np.random.default_rng(0)
    mass = rng.integers(1, 5, size=(cfg.B, cfg.M)).astype(np.float32)
    tau = float(np.median(run(e["x"], cfg.T, cfg.Hg, cfg.Wg, 2, 2, 2, tau=2.0)["window_sim"]))
    o = run(e["x"], cfg.T, cfg.Hg, cfg.Wg, 2, 2, 2, tau=tau, mass=mass)
    for b in range(cfg.B):
        n = o["out_count"][b]
        assert o["out_mass"][b, :n].sum() == pytest.approx(mass[b].sum(), rel=1e-12)
        lhs = (o["out_mass"][b, :n, None].astype(np.float64) * o["out_x"][b, :n]).sum(0)
        rhs = (mass[b][:, None].astype(np.float64) * e["x"][b]).sum(0)
        assert np.allclose(lhs, rhs, rtol=1e-5, atol=1e-4)
        assert np.all(np.diff(o["out_index"][b, :n]) > 0)
    assert cfg.B * cfg.M // 8 < o["out_count"].sum() < cfg.B * cfg.M   # some windows merged, some not


def test_merged_set_monotone_in_tau_and_scale_invariant():
    cfg, e = smooth_case()
    sims = run(e["x"], cfg.T, cfg.Hg, cfg.Wg, tau=2.0)["window_sim"]
    prev = None
    for tau in np.quantile(sims, [0.1, 0.4, 0.7, 0.95]):
        o = run(e["x"], cfg.T, cfg.Hg, cfg.Wg, tau=float(tau))
        merged = o["window_sim"] > np.float32(tau).astype(np.float64)
        assert np.array_equal(cfg.M - 3 * merged.sum(1), o["out_count"])
        if prev is not None:
            assert np.all(merged <= prev)       # raising tau never adds a merged window
        prev = merged
    tau = float(np.median(sims))
    o1 = run(e["x"], cfg.T, cfg.Hg, cfg.Wg, tau=tau)
    x4 = e["x"].copy()
    x4[:, ::3] *= 4.0                            # scaling a token by c > 0 changes no decision
    o2 = run(x4, cfg.T, cfg.Hg, cfg.Wg, tau=tau)
    assert np.array_equal(o1["out_index"], o2["out_index"])
    assert np.allclose(o1["window_sim"], o2["window_sim"], atol=1e-12)


def test_member_permutation_inside_window():
    rng = np.random.default_rng(9)
    base = rng.standard_normal(16)
    x = (base + 0.2 * rng.standard_normal((1, 4, 16))).astype(np.float32)
    mass = np.array([[1, 2, 3, 4]], dtype=np.float32)
    o1 = run(x, 1, 2, 2, tau=0.1, mass=mass)
    perm = [2, 0, 3, 1]
    o2 = run(x[:, perm].copy(), 1, 2, 2, tau=0.1, mass=mass[:, perm].copy())
    assert o1["out_count"][0] == o2["out_count"][0] == 1
    assert o1["window_sim"][0, 0] == pytest.approx(o2["window_sim"][0, 0], abs=1e-14)
    assert np.allclose(o1["out_x"][0, 0], o2["out_x"][0, 0], rtol=1e-6)
    assert o1["out_mass"][0, 0] == 10.0


def test_key_tokens_survive_bit_for_bit():
    cfg, e = smooth_case()
    mass = np.random.default_rng(1).integers(1, 5, size=(cfg.B, cfg.M)).astype(np.float32)
    o = run(e["x"], cfg.T, cfg.Hg, cfg.Wg, 2, 2, 2, tau=-1.0, key_budget=cfg.key_budget,
            q=e["q_cls"], k=e["k_cls"], mass=mass)
    for b in range(cfg.B):
        n = o["out_count"][b]
        # tau = -1 merges every window that holds no key token
        n_key_windows = len({_window_of(int(j), cfg, 2, 2, 2) for j in o["key_index"][b]})
        W = cfg.M // 8
        assert n == (W - n_key_windows) + 8 * n_key_windows
        idx = o["out_index"][b, :n].tolist()
        for j in o["key_index"][b]:
            s = idx.index(int(j))
            assert o["out_is_key"][b, s] == 1
            assert o["out_mass"][b, s] == mass[b, j]
            assert np.array_equal(o["out_x"][b, s], e["x"][b, j])
        assert o["out_is_key"][b, :n].sum() == cfg.key_budget
        assert np.all(np.diff(o["key_index"][b]) > 0)


def _window_of(tok, cfg, kt, kh, kw):
    x = tok % cfg.Wg
    y = (tok // cfg.Wg) % cfg.Hg
    t = tok // (cfg.Wg * cfg.Hg)
    return (t // kt, y // kh, x // kw)


def test_cls_scores_single_head_reduce_to_argsort_of_logits():
    rng = np.random.default_rng(21)
    B, M, D = 2, 30, 12
    q = rng.standard_normal((B, 1, D)).astype(np.float32)
    k = rng.standard_normal((B, 1 + M, 1, D)).astype(np.float32)
    k[0, 5] = k[0, 9]                      # an exact tie -> lower index wins
    x = rand_tokens(rng, B, M, D)
    o = run(x, 1, 5, 6, 1, 1, 1, tau=2.0, key_budget=7, q=q, k=k)
    for b in range(B):
        logit = (k[b, :, 0].astype(np.float64) @ q[b, 0].astype(np.float64)) / np.sqrt(D)
        top = np.sort(np.argsort(-logit[1:], kind="stable")[:7])
        assert o["key_index"][b].tolist() == top.tolist()
        p = np.exp(logit - logit.max())
        p /= p.sum()
        assert np.allclose(o["a_cls"][b], p[1:], rtol=1e-12, atol=0)
        # softmax runs over the CLS key too: patch probabilities sum to 1 - p_cls
        assert o["a_cls"][b].sum() == pytest.approx(1.0 - p[0], rel=1e-12)


def test_cls_scores_multi_head_match_numpy_einsum():
    cfg, e = smooth_case()
    o = run(e["x"], cfg.T, cfg.Hg, cfg.Wg, tau=2.0, key_budget=cfg.key_budget, q=e["q_cls"], k=e["k_cls"])
    q = e["q_cls"].astype(np.float64)
    k = e["k_cls"].astype(np.float64)
    lg = np.einsum("bhc,bjhc->bhj", q, k) / np.sqrt(cfg.dc)
    p = np.exp(lg - lg.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    a = p.mean(1)[:, 1:]
    assert np.allclose(o["a_cls"], a, rtol=1e-12, atol=0)
    for b in range(cfg.B):
        assert o["key_index"][b].tolist() == np.sort(np.argsort(-a[b], kind="stable")[:cfg.key_budget]).tolist()


def test_padding_content_and_position_do_not_matter():
    cfg, e = smooth_case()
    rng = np.random.default_rng(4)
    valid = (rng.random((cfg.B, cfg.M)) > 0.2).astype(np.uint8)
    args = dict(kt=2, kh=2, kw=2, tau=0.3, key_budget=4, q=e["q_cls"])
    o1 = run(e["x"], cfg.T, cfg.Hg, cfg.Wg, k=e["k_cls"], valid=valid, **args)
    x2 = e["x"].copy()
    k2 = e["k_cls"].copy()
    bad = valid == 0
    junk = np.array([np.nan, np.inf, -np.inf, 1e30], dtype=np.float32)
    x2[bad] = junk[rng.integers(0, 4, size=(int(bad.sum()), cfg.D))]
    k2[:, 1:][bad] = np.nan
    o2 = run(x2, cfg.T, cfg.Hg, cfg.Wg, k=k2, valid=valid, **args)
    for name in ("out_count", "out_index", "out_mass", "out_is_key", "key_index"):
        assert np.array_equal(o1[name], o2[name]), name
    for b in range(cfg.B):
        n = o1["out_count"][b]
        assert np.array_equal(o1["out_x"][b, :n], o2["out_x"][b, :n])
        assert n <= valid[b].sum()
    # shuffling what sits in the padding slots (valid tokens keep their cells) changes nothing
    x3 = x2.copy()
    for b in range(cfg.B):
        slots = np.flatnonzero(bad[b])
        x3[b, slots] = x2[b, rng.permutation(slots)]
    o3 = run(x3, cfg.T, cfg.Hg, cfg.Wg, k=k2, valid=valid, **args)
    assert np.array_equal(o1["out_index"], o3["out_index"])


def test_window_with_fewer_than_two_valid_members_is_left_alone():
    x = np.ones((1, 4, 4), dtype=np.float32)
    valid = np.array([[1, 0, 0, 0]], dtype=np.uint8)
    o = run(x, 1, 2, 2, tau=-1.0, valid=valid)
    assert o["out_count"][0] == 1 and o["out_index"][0, 0] == 0 and o["out_mass"][0, 0] == 1.0
    valid = np.array([[0, 1, 0, 1]], dtype=np.uint8)
    o = run(x, 1, 2, 2, tau=0.5, valid=valid)
    assert o["out_count"][0] == 1 and o["out_index"][0, 0] == 1 and o["out_mass"][0, 0] == 2.0


def chain_second_call_inputs(o1, cls_row, Hc, dc):
    """Inputs of the key-selection call on an already merged sequence: the survivors of the first call as
    a 1 x 1 x M grid (slots beyond out_count are padding), their masses, and keys made the way the
    synthetic workload makes them (row 0 = the CLS row, then the token rows, viewed as Hc x dc)."""
    B, M, D = o1["out_x"].shape
    k2 = np.concatenate([cls_row.reshape(B, 1, D), o1["out_x"]], axis=1).reshape(B, 1 + M, Hc, dc)
    return o1["out_x"], np.ascontiguousarray(k2), o1["out_mass"], o1["out_valid"]


def test_two_call_form_matches_paper_order():
    """Sec. 3.3 in the paper's order: merge at the first layer (a call without keys), then Key Retaining
    at a deep layer on the MERGED sequence (a call with 1x1x1 windows on the first call's outputs)."""
    cfg, e = smooth_case(T=1)
    budget = 4
    o1 = run(e["x"], 1, cfg.Hg, cfg.Wg, tau=0.2)
    assert np.all(o1["out_count"] < cfg.M) and np.all(o1["out_count"] > budget)
    x2, k2, mass2, valid2 = chain_second_call_inputs(o1, e["q_cls"], cfg.Hc, cfg.dc)
    o2 = run(x2, 1, 1, cfg.M, 1, 1, 1, tau=5.0, key_budget=budget, q=e["q_cls"], k=k2, mass=mass2, valid=valid2)
    q = wl.to_f64(e["q_cls"], F32)
    for b in range(cfg.B):
        n = int(o1["out_count"][b])
        # 1x1x1 windows never merge: the second call passes the merged sequence through unchanged
        assert o2["out_count"][b] == n
        assert np.array_equal(o2["out_x"][b, :n], o1["out_x"][b, :n])
        assert np.array_equal(o2["out_mass"][b, :n], o1["out_mass"][b, :n])
        assert np.array_equal(o2["out_index"][b, :n], np.arange(n))
        # token mass is conserved across both calls: every patch is still represented exactly once
        assert o2["out_mass"][b, :n].sum() == cfg.M
        lhs = (o2["out_mass"][b, :n, None].astype(np.float64) * o2["out_x"][b, :n]).sum(0)
        assert np.allclose(lhs, e["x"][b].astype(np.float64).sum(0), rtol=1e-5, atol=1e-4)
        # the keys are survivors (never a padding slot), and they are the top scores of the merged
        # sequence: recomputed here with numpy on the first call's rows
        keys = o2["key_index"][b]
        assert np.all(keys >= 0) and np.all(keys < n) and o2["out_is_key"][b, :n].sum() == budget
        rows = wl.to_f64(o1["out_x"][b, :n], F32).reshape(n, cfg.Hc, cfg.dc)
        kk = np.concatenate([q[b][None], rows], axis=0)
        logits = np.einsum("hc,jhc->hj", q[b], kk) / np.sqrt(cfg.dc)
        p = np.exp(logits - logits.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        a = p[:, 1:].mean(axis=0)
        assert sorted(np.argsort(-a, kind="stable")[:budget].tolist()) == keys.tolist()
    # the one-call form scores the unmerged grid instead: a different computation (other softmax support)
    o3 = run(e["x"], 1, cfg.Hg, cfg.Wg, tau=0.2, key_budget=budget, q=e["q_cls"], k=e["k_cls"])
    assert not np.allclose(o3["a_cls"][0, :8], o2["a_cls"][0, :8], rtol=1e-3)


def test_hierarchical_remerge_conserves_mass_and_matches_brute_force():
    """Merging an already merged sequence again (the caller lays the survivors out on a new grid and
    hands over their masses): the total mass and the mass-weighted feature sum survive both calls, and the
    second call's rows are the brute-force mass-weighted means of the first call's rows."""
    cfg, e = smooth_case(B=2, Hg=8, Wg=8, T=1)
    M = cfg.M
    sims = run(e["x"], 1, cfg.Hg, cfg.Wg, tau=2.0)["window_sim"]
    o1 = run(e["x"], 1, cfg.Hg, cfg.Wg, tau=float(np.quantile(sims, 0.4)))
    assert np.all(o1["out_count"] < M) and np.all(o1["out_count"] >= M // 4) and o1["out_count"].max() > M // 4
    # second level: the survivors, in order, as a 1 x 1 x M row cut into windows of four; padding at the tail
    x2, mass2, valid2 = o1["out_x"], o1["out_mass"], o1["out_valid"]
    s2 = run(x2, 1, 1, M, 1, 1, 4, tau=2.0, mass=mass2, valid=valid2)["window_sim"]
    tau2 = float(np.median(s2[0, : int(o1["out_count"][0]) // 4]))
    o2 = run(x2, 1, 1, M, 1, 1, 4, tau=tau2, mass=mass2, valid=valid2)
    total_x = e["x"].astype(np.float64).sum(1)
    assert o2["out_count"].sum() < o1["out_count"].sum() and o2["out_mass"].max() > 4.0    # some merges of merges
    for b in range(cfg.B):
        n1, n2 = int(o1["out_count"][b]), int(o2["out_count"][b])
        assert n2 <= n1
        assert o1["out_mass"][b, :n1].sum() == M and o2["out_mass"][b, :n2].sum() == M
        lhs = (o2["out_mass"][b, :n2, None].astype(np.float64) * o2["out_x"][b, :n2]).sum(0)
        assert np.allclose(lhs, total_x[b], rtol=1e-5, atol=1e-4)
        # brute force over the second level's windows
        xs = x2[b].astype(np.float64)
        want_idx, want_mass, want_rows = [], [], []
        for w0 in range(0, M, 4):
            mem = [j for j in range(w0, min(w0 + 4, M)) if valid2[b, j]]
            if not mem:
                continue
            cs = []
            for m, q in combinations(mem, 2):
                den = np.linalg.norm(xs[m]) * np.linalg.norm(xs[q])
                cs.append(xs[m] @ xs[q] / den if den > 0 else 0.0)
            if len(mem) >= 2 and np.mean(cs) > np.float64(np.float32(tau2)):
                mm = mass2[b, mem].astype(np.float64)
                want_idx.append(mem[0]); want_mass.append(mm.sum())
                want_rows.append((mm[:, None] * xs[mem]).sum(0) / mm.sum())
            else:
                for j in mem:
                    want_idx.append(j); want_mass.append(float(mass2[b, j])); want_rows.append(xs[j])
        assert o2["out_index"][b, :n2].tolist() == want_idx
        assert np.allclose(o2["out_mass"][b, :n2], want_mass, rtol=0, atol=0)
        assert np.allclose(o2["out_x"][b, :n2], np.asarray(want_rows), rtol=1e-6, atol=1e-7)


# ---------------------------------------------------------------- storage rounding
def test_bf16_store_is_one_rounding_to_nearest_even():
    rng = np.random.default_rng(2)
    n = 400
    a = wl.f32_to_bf16_bits((rng.standard_normal(n) * 3).astype(np.float32))
    b = wl.f32_to_bf16_bits((wl.bf16_bits_to_f32(a) * (1 + 0.01 * rng.standard_normal(n))).astype(np.float32))
    # n windows of 1x1x2 over a grid 1 x 1 x 2n, D = 8 (same value in every channel)
    x = np.empty((1, 2 * n, 8), dtype=np.uint16)
    x[0, 0::2] = a[:, None]
    x[0, 1::2] = b[:, None]
    mass = np.ones((1, 2 * n), dtype=np.float32)
    mass[0, 1::2] = 2.0
    o = oracle.encode_merge(x, BF16, None, None, BF16, mass, None, 1, 1, 2 * n, 1, 1, 2, -2.0, 0)
    assert o["out_count"][0] == n
    got = wl.bf16_bits_to_f32(o["out_x"][0, :n, 0])
    fa = wl.bf16_bits_to_f32(a)
    fb = wl.bf16_bits_to_f32(b)
    for i in range(n):
        exact = (Fraction(float(fa[i])) + 2 * Fraction(float(fb[i]))) / 3
        g = Fraction(float(got[i]))
        bits = int(o["out_x"][0, i, 0])
        lo = Fraction(float(wl.bf16_bits_to_f32(np.array([bits - 1], dtype=np.uint16))[0]))
        hi = Fraction(float(wl.bf16_bits_to_f32(np.array([bits + 1], dtype=np.uint16))[0]))
        # nearest: no neighbour is strictly closer; on a tie the stored mantissa is even
        assert abs(g - exact) <= abs(lo - exact) and abs(g - exact) <= abs(hi - exact)
        if abs(g - exact) == abs(lo - exact) or abs(g - exact) == abs(hi - exact):
            assert bits % 2 == 0


def test_generator_bf16_rounding_matches_torch():
    import torch
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(10000) * 10.0 ** rng.integers(-6, 6, 10000)).astype(np.float32)
    ours = wl.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)


# ------------------------------------------------------------------ Eq. 7 as printed: O = {a_cls > mu}
def _adaptive_case():
    cfg = wl.tiny(wl.CONFIGS[2], B=3, Hg=8, Wg=10, D=64, Hc=4, dc=16)
    e = wl.encode_inputs(cfg)
    rng = np.random.default_rng(21)
    valid = (rng.random((cfg.B, cfg.M)) > 0.2).astype(np.uint8)
    return cfg, e, valid


def _adaptive(cfg, e, valid, lam, cap=None, tau=2.0):
    return oracle.encode_merge_adaptive(e["x"], cfg.x_dtype, e["q_cls"], e["k_cls"], cfg.x_dtype, None, valid,
                                        cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, tau, lam,
                                        cfg.M if cap is None else cap)


def test_adaptive_key_set_is_the_threshold_rule_on_an_independent_a_cls():
    """O = {a_cls > mean + lambda * std}: the scores recomputed with numpy (einsum + softmax over the 1+M keys,
    head mean), the threshold applied in numpy."""
    cfg, e, valid = _adaptive_case()
    lam = 0.7
    o = _adaptive(cfg, e, valid, lam)
    q = wl.to_f64(e["q_cls"], cfg.x_dtype)
    k = wl.to_f64(e["k_cls"], cfg.x_dtype)
    for b in range(cfg.B):
        vb = valid[b].astype(bool)
        logits = np.einsum("hc,jhc->hj", q[b], k[b]) / np.sqrt(cfg.dc)
        logits[:, 1:][:, ~vb] = -np.inf
        p = np.exp(logits - logits.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        a = p[:, 1:].mean(axis=0)
        mu = a[vb].mean() + np.float64(np.float32(lam)) * a[vb].std()
        want = np.flatnonzero(vb & (a > mu))
        assert o["key_count"][b] == want.size and 0 < want.size < vb.sum()
        assert o["key_index"][b, :want.size].tolist() == want.tolist()
        assert np.all(o["key_index"][b, want.size:] == -1)


def test_adaptive_threshold_uses_the_population_standard_deviation():
    """On eight tokens the population and the sample standard deviation differ by 7 %: a lambda is searched for
    which the two thresholds separate a token, and the oracle must side with the population form."""
    cfg = wl.tiny(wl.CONFIGS[2], B=1, Hg=2, Wg=4, D=32, Hc=2, dc=16)
    e = wl.encode_inputs(cfg)
    base = _adaptive(cfg, e, None, 0.0)
    a = base["a_cls"][0]
    found = None
    for lam in np.linspace(0.05, 2.5, 400):
        l32 = np.float64(np.float32(lam))
        pop = set(np.flatnonzero(a > a.mean() + l32 * a.std()).tolist())
        smp = set(np.flatnonzero(a > a.mean() + l32 * a.std(ddof=1)).tolist())
        if pop != smp:
            found = (float(lam), pop)
            break
    assert found is not None
    o = _adaptive(cfg, e, None, found[0])
    assert set(o["key_index"][0, :o["key_count"][0]].tolist()) == found[1]


def test_adaptive_key_set_limits_monotonicity_and_the_budget_form():
    cfg, e, valid = _adaptive_case()
    tau = 0.5                                        # low enough for many windows to merge when no key blocks them
    none = _adaptive(cfg, e, valid, 1e6, tau=tau)    # threshold above every score: no keys
    base = oracle.encode_merge(e["x"], cfg.x_dtype, None, None, cfg.x_dtype, None, valid, cfg.T, cfg.Hg, cfg.Wg,
                               cfg.kt, cfg.kh, cfg.kw, tau, 0)
    assert np.all(none["key_count"] == 0)
    for name in ("out_count", "out_index", "out_mass", "out_is_key", "out_x"):
        assert np.array_equal(none[name], base[name]), name
    every = _adaptive(cfg, e, valid, -1e6, tau=tau)  # threshold below every score: every valid token is a key
    assert np.array_equal(every["key_count"], valid.sum(1))
    assert np.array_equal(every["out_count"], valid.sum(1))          # a window with a key never merges
    prev = None
    for lam in (-1.0, 0.0, 0.5, 1.0, 2.0):
        o = _adaptive(cfg, e, valid, lam, tau=tau)
        keys = [set(o["key_index"][b, :o["key_count"][b]].tolist()) for b in range(cfg.B)]
        if prev is not None:
            assert all(keys[b] <= prev[b] for b in range(cfg.B))     # a higher threshold keeps a subset
        prev = keys
        # with |O| = n the printed rule and the budget form (top-n) name the same set, and all else follows
        for b in range(cfg.B):
            n = int(o["key_count"][b])
            eb = {kk: vv[b:b + 1] for kk, vv in e.items() if kk != "ell"}
            ob = oracle.encode_merge(eb["x"], cfg.x_dtype, eb["q_cls"], eb["k_cls"], cfg.x_dtype, None, valid[b:b + 1],
                                     cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, tau, n) if n > 0 else None
            if ob is not None:
                assert ob["key_index"][0].tolist() == o["key_index"][b, :n].tolist()
                assert ob["out_count"][0] == o["out_count"][b]
                assert np.array_equal(ob["out_index"][0], o["out_index"][b])


def test_adaptive_key_index_capacity():
    cfg, e, valid = _adaptive_case()
    full = _adaptive(cfg, e, valid, 0.0)
    cap = 3
    o = _adaptive(cfg, e, valid, 0.0, cap=cap)
    assert np.array_equal(o["key_count"], full["key_count"]) and np.all(full["key_count"] > cap)
    assert np.array_equal(o["key_index"], full["key_index"][:, :cap])
    assert np.array_equal(o["out_index"], full["out_index"])         # the capacity limits the list, not the set


@pytest.mark.parametrize("Hg,Wg", [(1, 3), (3, 5), (7, 9)])
def test_adaptive_rule_is_strict_at_an_exact_tie(Hg, Wg):
    """Eq. 7 prints a strict '>'.  One head, a zero CLS query and M = 2^k - 1 tokens make every logit 0,
    so every a_cls is exactly 1/(M+1) (a power of two): the mean is exact, the standard deviation is 0
    and mu == a_cls for any lambda.  Strict '>' selects nothing; '>=' would select every token."""
    M, D = Hg * Wg, 16
    assert (M + 1) & M == 0
    rng = np.random.default_rng(M)
    x = rng.standard_normal((2, M, D)).astype(np.float32)
    k = np.ascontiguousarray(rng.standard_normal((2, 1 + M, 1, D)).astype(np.float32))
    q = np.zeros((2, 1, D), dtype=np.float32)
    for lam in (-1.0, 0.0, 2.0):
        o = oracle.encode_merge_adaptive(x, F32, q, k, F32, None, None, 1, Hg, Wg, 1, 1, 1, 2.0, lam, M)
        assert np.all(o["a_cls"] == 1.0 / (M + 1))
        assert np.all(o["key_count"] == 0) and np.all(o["key_index"] == -1) and o["out_is_key"].sum() == 0
    # the same tie among the valid tokens of a padded grid (15 valid of 20 slots)
    if M == 15:
        valid = np.ones((2, 20), dtype=np.uint8)
        valid[:, [1, 6, 7, 13, 19]] = 0
        x20 = rng.standard_normal((2, 20, D)).astype(np.float32)
        k20 = np.ascontiguousarray(rng.standard_normal((2, 21, 1, D)).astype(np.float32))
        o = oracle.encode_merge_adaptive(x20, F32, q, k20, F32, None, valid, 1, 4, 5, 1, 1, 1, 2.0, 0.0, 20)
        assert np.all(o["a_cls"][valid.astype(bool)] == 1.0 / 16) and np.all(o["key_count"] == 0)
    # one token lifted by a hair is the only one above the threshold: the rule is not vacuous here
    q1 = np.zeros((2, 1, D), dtype=np.float32)
    q1[:, 0, 0] = 1.0
    k1 = np.zeros((2, 1 + M, 1, D), dtype=np.float32)
    k1[:, 2, 0, 0] = 0.25
    o = oracle.encode_merge_adaptive(x, F32, q1, k1, F32, None, None, 1, Hg, Wg, 1, 1, 1, 2.0, 0.0, M)
    assert np.all(o["key_count"] == 1) and np.all(o["key_index"][:, 0] == 1)
