"""Pins for the stage-2 oracle (Sec. 3.4: global filter Eq. 8-9, individual filter Eq. 10, token drop)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import FILTER_BUDGET, FILTER_THRESHOLD


def make(B=2, Mv=40, N=6, H=3, d=8, C=16, seed=0, qscale=1.0):
    rng = np.random.default_rng(seed)
    L = Mv + N
    f = lambda *s: wl.f32_to_bf16_bits(rng.standard_normal(s).astype(np.float32))
    q = wl.f32_to_bf16_bits((qscale * rng.standard_normal((B, N, H, d))).astype(np.float32))
    return dict(q=q, k=f(B, L, H, d), v=f(B, L, H, d), hidden=f(B, L, C), Mv=Mv, N=N, H=H, d=d, C=C, B=B)


def run(t, mode=FILTER_BUDGET, budget=10, gamma=None, alpha=None, vis_valid=None, txt_len=None, is_key=None,
        Rcap=None, scale=None):
    Mv, N = t["Mv"], t["N"]
    gamma = 1.0 / Mv if gamma is None else gamma
    alpha = 2.0 / (Mv + N) if alpha is None else alpha
    scale = 1.0 / np.sqrt(t["d"]) if scale is None else scale
    return oracle.prefill_filter(t["q"], t["k"], t["v"], t["hidden"], vis_valid, txt_len, is_key, Mv,
                                 scale, mode, budget, gamma, alpha, Rcap)


def numpy_scores(t, scale, vis_valid=None, txt_len=None):
    """Independent fp64 einsum + softmax (not the oracle's loops)."""
    scale = float(np.float32(scale))               # the C ABI carries the scale as a float
    q = wl.to_f64(t["q"], wl.BF16)
    k = wl.to_f64(t["k"], wl.BF16)
    B, N, Mv = t["B"], t["N"], t["Mv"]
    lg = scale * np.einsum("bihc,bjhc->bhij", q, k)              # [B,H,N,L]
    mask = np.ones((B, 1, N, Mv + N), dtype=bool)
    mask[:, :, :, Mv:] = np.tril(np.ones((N, N), dtype=bool))[None, None]
    if vis_valid is not None:
        mask[:, :, :, :Mv] &= vis_valid.astype(bool)[:, None, None, :]
    lg = np.where(mask, lg, -np.inf)
    p = np.exp(lg - lg.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    a = p.mean(1)[:, :, :Mv]                                     # head mean, vision columns
    if txt_len is not None:
        rows = np.arange(N)[None, :, None] < txt_len[:, None, None]
        a = np.where(rows, a, 0.0)
    return a.sum(1), a.max(1), p.mean(1)


def test_scores_match_independent_numpy_and_selection_matches_stable_argsort():
    t = make(seed=1)
    is_key = np.zeros((t["B"], t["Mv"]), dtype=np.uint8)
    is_key[:, [3, 17, 30]] = 1
    gamma, alpha, R = 1.0 / 40, 2.0 / 46, 12
    o = run(t, budget=R, is_key=is_key, gamma=gamma, alpha=alpha)
    V, I, _ = numpy_scores(t, 1 / np.sqrt(t["d"]))
    assert np.allclose(o["score_global"], V, rtol=1e-12, atol=0)
    assert np.allclose(o["score_indiv"], I, rtol=1e-12, atol=0)
    for b in range(t["B"]):
        G = V[b].sum()
        s = np.maximum(V[b] / (np.float64(np.float32(gamma)) * G), I[b] / np.float64(np.float32(alpha)))
        s[is_key[b] == 1] = np.inf
        kept = np.sort(np.argsort(-s, kind="stable")[:R])
        assert o["kept_index"][b].tolist() == kept.tolist()
        assert o["kept_count"][b] == R and o["out_len"][b] == R + t["N"]


def test_softmax_rows_sum_to_one_so_G_is_bounded_by_text_length():
    t = make(seed=2)
    txt_len = np.array([6, 4], dtype=np.int32)
    o = run(t, txt_len=txt_len)
    V, I, pm = numpy_scores(t, 1 / np.sqrt(t["d"]), txt_len=txt_len)
    # every text row's probabilities over vision + visible text columns sum to 1, also after the head mean
    assert np.allclose(pm.sum(-1), 1.0, atol=1e-12)
    G = o["score_global"].sum(1)
    assert np.all(G < txt_len) and np.all(G > 0)
    assert np.allclose(o["score_global"], V, rtol=1e-12, atol=0)
    assert np.all(o["score_indiv"] <= o["score_global"] + 1e-15)


def test_zero_queries_give_harmonic_numbers_and_lowest_index_tie_break():
    t = make(seed=3)
    t["q"][:] = 0
    Mv, N = t["Mv"], t["N"]
    is_key = np.zeros((t["B"], Mv), dtype=np.uint8)
    is_key[:, [20, 33]] = 1
    o = run(t, budget=7, is_key=is_key)
    # text row i sees Mv + i + 1 keys with equal weight
    Vexp = sum(1.0 / (Mv + i + 1) for i in range(N))
    assert np.allclose(o["score_global"], Vexp, rtol=1e-13, atol=0)
    assert np.allclose(o["score_indiv"], 1.0 / (Mv + 1), rtol=1e-13, atol=0)
    for b in range(t["B"]):
        assert o["kept_index"][b].tolist() == [0, 1, 2, 3, 4, 20, 33]


def test_threshold_mode_special_cases():
    t = make(seed=4)
    Mv = t["Mv"]
    is_key = np.zeros((t["B"], Mv), dtype=np.uint8)
    is_key[:, [1, 2]] = 1
    o = run(t, mode=FILTER_THRESHOLD, gamma=-1.0, alpha=0.5, is_key=is_key)
    assert np.all(o["kept_count"] == Mv)                        # gamma < 0: nothing is in D
    o = run(t, mode=FILTER_THRESHOLD, gamma=0.5, alpha=0.0, is_key=is_key)
    assert np.all(o["kept_count"] == Mv)                        # alpha <= 0: the individual test never fires
    o = run(t, mode=FILTER_THRESHOLD, gamma=1.0, alpha=np.inf, is_key=is_key)
    assert np.all(o["kept_count"] == 2)                         # everything but the keys is dropped
    assert np.all(o["kept_index"][:, :2] == [1, 2])
    # |D| is dynamic: count follows the rule, not a budget
    V, I, _ = numpy_scores(t, 1 / np.sqrt(t["d"]))
    gamma, alpha = np.float32(1.0 / Mv), np.float32(0.06)
    o = run(t, mode=FILTER_THRESHOLD, gamma=gamma, alpha=alpha, is_key=is_key)
    for b in range(t["B"]):
        drop = (V[b] <= np.float64(gamma) * V[b].sum()) & (I[b] < np.float64(alpha)) & (is_key[b] == 0)
        assert o["kept_count"][b] == Mv - drop.sum()
        assert o["kept_index"][b, :o["kept_count"][b]].tolist() == np.flatnonzero(~drop).tolist()


def test_budget_edges_and_bitwise_copy():
    t = make(seed=5)
    Mv, N, B = t["Mv"], t["N"], t["B"]
    o = run(t, budget=Mv)
    assert np.array_equal(o["k_out"], t["k"]) and np.array_equal(o["v_out"], t["v"])
    assert np.array_equal(o["hidden_out"], t["hidden"])
    is_key = wl.random_key_mask(wl.tiny(wl.CONFIGS[2], B=B, Hg=5, Wg=8), 6)
    o = run(t, budget=6, is_key=is_key)
    for b in range(B):
        assert o["kept_index"][b].tolist() == np.flatnonzero(is_key[b]).tolist()
    for R in (7, 13, 25):
        o = run(t, budget=R, is_key=is_key)
        assert np.all(o["kept_count"] == R)
        for b in range(B):
            kept = o["kept_index"][b]
            assert np.all(np.diff(kept) > 0)
            assert set(np.flatnonzero(is_key[b])) <= set(kept.tolist())
            rows = np.concatenate([kept, Mv + np.arange(N)])
            assert np.array_equal(o["k_out"][b], t["k"][b, rows])
            assert np.array_equal(o["v_out"][b], t["v"][b, rows])
            assert np.array_equal(o["hidden_out"][b], t["hidden"][b, rows])
            assert o["out_protect"][b].tolist() == [int(is_key[b, j]) for j in kept] + [1] * N
    # more keys than budget: keys win, the true count is reported, storage stops at Rcap
    o = run(t, budget=4, is_key=is_key)
    assert np.all(o["kept_count"] == 6)
    for b in range(B):
        assert o["kept_index"][b].tolist() == np.flatnonzero(is_key[b])[:4].tolist()


def test_planted_token_is_rescued_by_individual_attention():
    # one text query aligned with one vision key whose global score is low: global-only drops it, dual keeps it
    t = make(B=1, Mv=48, N=8, H=2, d=16, seed=6, qscale=0.3)
    k = wl.bf16_bits_to_f32(t["k"]).copy()
    q = wl.bf16_bits_to_f32(t["q"]).copy()
    jstar, istar = 11, 5
    k[0, jstar] = -0.25 * q[0].mean(0)         # mildly anti-aligned with the average query ...
    q[0, istar] = 6.0 * k[0, jstar] / np.linalg.norm(k[0, jstar])   # ... but one text token points straight at it
    t["k"], t["q"] = wl.f32_to_bf16_bits(k), wl.f32_to_bf16_bits(q)
    V, I, _ = numpy_scores(t, 1 / np.sqrt(t["d"]))
    gamma = np.float32(1.0 / 48)
    alpha = np.float32(0.5 * I[0, jstar])
    if not V[0, jstar] <= np.float64(gamma) * V[0].sum():
        pytest.skip("construction did not put the planted token in D")
    glob = run(t, mode=FILTER_THRESHOLD, gamma=gamma, alpha=np.inf)
    dual = run(t, mode=FILTER_THRESHOLD, gamma=gamma, alpha=alpha)
    kg = set(glob["kept_index"][0, :glob["kept_count"][0]].tolist())
    kd = set(dual["kept_index"][0, :dual["kept_count"][0]].tolist())
    assert jstar not in kg and jstar in kd
    assert kg <= kd                              # the individual test only ever rescues tokens


def test_single_text_token_makes_dual_equal_global():
    t = make(N=1, seed=7)
    o = run(t, mode=FILTER_THRESHOLD, gamma=1.0 / 40, alpha=0.02)
    assert np.allclose(o["score_global"], o["score_indiv"], rtol=1e-15, atol=0)
    for b in range(t["B"]):
        V = o["score_global"][b]
        thr_g = np.float64(np.float32(1.0 / 40)) * V.sum()
        drop = (V <= thr_g) & (V < np.float64(np.float32(0.02)))
        assert o["kept_count"][b] == t["Mv"] - drop.sum()


def test_padding_content_and_position_do_not_matter():
    t = make(seed=8)
    rng = np.random.default_rng(0)
    B, Mv, N = t["B"], t["Mv"], t["N"]
    vis_valid = (rng.random((B, Mv)) > 0.25).astype(np.uint8)
    txt_len = np.array([N, N - 2], dtype=np.int32)
    o1 = run(t, budget=9, vis_valid=vis_valid, txt_len=txt_len)
    V, I, _ = numpy_scores(t, 1 / np.sqrt(t["d"]), vis_valid=vis_valid, txt_len=txt_len)
    assert np.allclose(o1["score_global"], np.where(vis_valid == 1, V, 0), rtol=1e-12, atol=0)
    t2 = {k_: (v_.copy() if isinstance(v_, np.ndarray) else v_) for k_, v_ in t.items()}
    bad = vis_valid == 0
    t2["k"][:, :Mv][bad] = 0x7FC0                # NaN in padded vision slots
    t2["v"][:, :Mv][bad] = 0x7F80
    t2["hidden"][:, :Mv][bad] = 0xFFFF
    t2["k"][1, Mv + N - 2:] = 0x7FC0             # NaN in padded text rows
    t2["q"][1, N - 2:] = 0x7FC0
    o2 = run(t2, budget=9, vis_valid=vis_valid, txt_len=txt_len)
    for name in ("kept_index", "kept_count", "out_len", "score_global", "score_indiv"):
        assert np.array_equal(o1[name], o2[name]), name
    for b in range(B):
        n = o1["out_len"][b]
        assert n == 9 + txt_len[b]
        assert np.array_equal(o1["k_out"][b, :n], o2["k_out"][b, :n])
        assert not (set(o1["kept_index"][b].tolist()) & set(np.flatnonzero(bad[b]).tolist()))


def test_budget_rule_equals_threshold_rule_with_jointly_scaled_thresholds():
    # keeping the top-R by s = max(V/(gamma G), I/alpha) is the paper's rule with (gamma, alpha) scaled by a common c
    t = make(seed=9)
    R = 15
    gamma, alpha = np.float32(1 / 40), np.float32(0.05)
    ob = run(t, budget=R, gamma=gamma, alpha=alpha)
    V, I, _ = numpy_scores(t, 1 / np.sqrt(t["d"]))
    for b in range(t["B"]):
        s = np.sort(np.maximum(V[b] / (np.float64(gamma) * V[b].sum()), I[b] / np.float64(alpha)))[::-1]
        c = 0.5 * (s[R - 1] + s[R])
        ot = run(t, mode=FILTER_THRESHOLD, gamma=np.float32(gamma * c), alpha=np.float32(alpha * c))
        if abs(s[R - 1] - s[R]) > 1e-4 * c:
            assert ot["kept_index"][b, :ot["kept_count"][b]].tolist() == ob["kept_index"][b].tolist()


def test_boundary_cases_of_eq9_and_eq10():
    # Eq. 9 uses "<=": two vision tokens with identical score V and gamma = 1/2 give V == gamma*G -> both in D
    t = make(B=1, Mv=2, N=1, seed=10)
    t["q"][:] = 0
    o = run(t, mode=FILTER_THRESHOLD, gamma=0.5, alpha=np.inf)
    assert o["kept_count"][0] == 0 and o["out_len"][0] == 1
    # Eq. 10 uses "<": I_j == alpha is not "truly unimportant".  Mv = 3, N = 1, Q = 0 -> every a_ij = 1/4
    t = make(B=1, Mv=3, N=1, seed=10)
    t["q"][:] = 0
    o = run(t, mode=FILTER_THRESHOLD, gamma=1.0, alpha=0.25)
    assert o["kept_count"][0] == 3
    o = run(t, mode=FILTER_THRESHOLD, gamma=1.0, alpha=np.nextafter(np.float32(0.25), np.float32(1)))
    assert o["kept_count"][0] == 0


def test_chained_calls_keep_the_key_set_and_shrink_to_the_budgets():
    """Sec. 3.3 / 3.4: tokens of the key set are retained by every later filtering step.  Three chained
    oracle calls (budgets 48 -> 20 -> 9) on a small sample: every call keeps exactly its budget, rows are
    bitwise copies, and the keys of the first call are still present at the end."""
    cfg = wl.tiny(wl.CONFIGS[2], B=2, Hg=8, Wg=8, N=8, H=2, d=64, C=64)
    t = wl.prefill_inputs(cfg)
    key = wl.random_key_mask(cfg, 6)
    keys0 = [set(np.flatnonzero(key[b]).tolist()) for b in range(cfg.B)]
    scale = 1.0 / np.sqrt(cfg.d)
    Mv, vis = cfg.M, None
    orig = np.tile(np.arange(cfg.M), (cfg.B, 1))
    for layer, R in enumerate((48, 20, 9)):
        q = t["q_txt"] if layer == 0 else wl.layer_text_queries(cfg, layer)
        o = oracle.prefill_filter(q, t["k"], t["v"], t["hidden"], vis, None, key, Mv, scale, FILTER_BUDGET, R,
                                  1.0 / Mv, 2.0 / (Mv + cfg.N), R)
        assert np.all(o["kept_count"] == R)
        for b in range(cfg.B):
            rows = np.concatenate([o["kept_index"][b], Mv + np.arange(cfg.N)])
            assert np.array_equal(o["k_out"][b], t["k"][b, rows])
            assert np.array_equal(o["hidden_out"][b], t["hidden"][b, rows])
        orig = np.take_along_axis(orig, o["kept_index"], axis=1)
        t = {"q_txt": q, "k": o["k_out"], "v": o["v_out"], "hidden": o["hidden_out"]}
        key, vis, Mv = o["out_protect"][:, :R].copy(), None, R
    for b in range(cfg.B):
        assert keys0[b] <= set(orig[b].tolist())


def test_row_normalisers_match_numpy_logsumexp():
    """The row normalisers the oracle reports (what an attention kernel leaves behind, Sec. 3.4) against a
    numpy log-sum-exp over the visible keys; rows beyond txt_len report 0."""
    t = make(B=3, Mv=37, N=9, H=4, d=16, seed=11)
    rng = np.random.default_rng(5)
    vis_valid = (rng.random((t["B"], t["Mv"])) > 0.25).astype(np.uint8)
    txt_len = np.array([9, 4, 0], dtype=np.int32)
    scale = 0.31
    o = run(t, budget=10, vis_valid=vis_valid, txt_len=txt_len, scale=scale)
    q, k = wl.to_f64(t["q"], wl.BF16), wl.to_f64(t["k"], wl.BF16)
    lg = float(np.float32(scale)) * np.einsum("bihc,bjhc->bhij", q, k)
    Mv, N = t["Mv"], t["N"]
    mask = np.ones((t["B"], 1, N, Mv + N), dtype=bool)
    mask[:, :, :, Mv:] = np.tril(np.ones((N, N), dtype=bool))[None, None]
    mask[:, :, :, :Mv] &= vis_valid.astype(bool)[:, None, None, :]
    lg = np.where(mask, lg, -np.inf)
    mx = lg.max(-1)
    lse = mx + np.log(np.exp(lg - mx[..., None]).sum(-1))            # [B,H,N]
    for b in range(t["B"]):
        tl = int(txt_len[b])
        assert np.allclose(o["row_lse"][b, :, :tl], lse[b, :, :tl], rtol=1e-13, atol=1e-13)
        assert np.all(o["row_lse"][b, :, tl:] == 0.0)
    # they are exactly what turns a logit into the probability the scores are made of
    b, h, i = 0, 2, 5
    p = np.exp(lg[b, h, i, :Mv] - o["row_lse"][b, h, i])
    assert np.isclose(p.sum() + np.exp(lg[b, h, i, Mv:] - o["row_lse"][b, h, i]).sum(), 1.0, rtol=1e-12)
