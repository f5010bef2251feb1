"""GPU parity: mustdrop_prefill_filter (HIP, through the C ABI) against the CPU oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import FILTER_BUDGET, FILTER_THRESHOLD
from parity import check_prefill

pytestmark = pytest.mark.gpu


def run(t, Mv, budget, mode=FILTER_BUDGET, vis_valid=None, txt_len=None, is_key=None, gamma=None, alpha=None,
        Rcap=None, scale=None, d=128):
    from paper_2411_10803_amd import harness
    N = t["q_txt"].shape[1]
    gamma = 1.0 / Mv if gamma is None else gamma
    alpha = 2.0 / (Mv + N) if alpha is None else alpha
    scale = 1.0 / np.sqrt(t["q_txt"].shape[3]) if scale is None else scale
    if Rcap is None:
        Rcap = budget if mode == FILTER_BUDGET else Mv
    g = harness.prefill_on_gpu(t, Mv, vis_valid, txt_len, is_key, scale, mode, budget, gamma, alpha, Rcap)
    o = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], vis_valid, txt_len, is_key, Mv, scale, mode,
                              budget, gamma, alpha, Rcap)
    s = check_prefill(g, o, t, Mv, vis_valid, is_key, mode, budget, gamma, alpha, Rcap)
    return g, o, s


def test_config1_single_sample():
    cfg = wl.CONFIGS[1]
    t = wl.prefill_inputs(cfg)
    is_key = wl.random_key_mask(cfg, cfg.key_budget)
    g, o, s = run(t, cfg.M, 192, is_key=is_key)
    assert g["kept_count"][0] == 192


def test_config2_three_budgets_on_a_batch_slice():
    cfg = wl.CONFIGS[2]
    t = wl.prefill_inputs(cfg, samples=[0, 1, 2, 15])
    is_key = wl.random_key_mask(cfg, cfg.key_budget)[[0, 1, 2, 15]]
    for R in cfg.budgets:
        g, o, s = run(t, cfg.M, R, is_key=is_key)
        assert np.all(g["kept_count"] == R)


def test_config3_long_sequence_128_text_rows():
    cfg = wl.CONFIGS[3]
    t = wl.prefill_inputs(cfg, samples=[0])
    is_key = wl.random_key_mask(cfg, cfg.key_budget)[[0]]
    g, o, s = run(t, cfg.M, 320, is_key=is_key)
    assert g["kept_count"][0] == 320


def test_ragged_padding_and_odd_shapes():
    # Mv and N not multiples of the 32-wide tiles, padded vision slots and padded text tail, NaN in padding
    cfg = wl.tiny(wl.CONFIGS[2], B=3, Hg=7, Wg=11, N=45, H=6, d=64, C=264)
    Mv = cfg.M
    t = wl.prefill_inputs(cfg)
    rng = np.random.default_rng(3)
    vis_valid = (rng.random((cfg.B, Mv)) > 0.3).astype(np.uint8)
    txt_len = np.array([45, 17, 1], dtype=np.int32)
    is_key = wl.random_key_mask(cfg, 5, valid=vis_valid)
    bad = vis_valid == 0
    t["k"][:, :Mv][bad] = 0x7FC0
    t["v"][:, :Mv][bad] = 0x7F80
    t["hidden"][:, :Mv][bad] = 0xFFFF
    for b in range(cfg.B):
        t["k"][b, Mv + txt_len[b]:] = 0x7FC0
        t["q_txt"][b, txt_len[b]:] = 0x7FC0
    for R in (5, 20, 40):
        run(t, Mv, R, vis_valid=vis_valid, txt_len=txt_len, is_key=is_key)
    g, o, s = run(t, Mv, 0, mode=FILTER_THRESHOLD, vis_valid=vis_valid, txt_len=txt_len, is_key=is_key,
                  gamma=1.0 / Mv, alpha=1.5 / Mv)
    assert len(set(g["kept_count"].tolist())) > 1          # dynamic |D|
    # budget >= number of valid tokens: everything valid is kept
    g, o, s = run(t, Mv, Mv, vis_valid=vis_valid, txt_len=txt_len, is_key=is_key)
    assert np.array_equal(g["kept_count"], vis_valid.sum(1))


def test_padding_tails_of_different_lengths_are_skipped_not_scored():
    # After the vision-encoder stage the valid slots of a sample are a prefix and the rest is padding: the
    # sweeps stop at the last valid slot.  Samples whose last valid slot falls on and off the 32-key and
    # 128-key boundaries, holes before it, one sample with no valid slot at all, NaN in every invalid row.
    # Two shapes: 128 text rows with several key chunks, and d = 64 with a vision length off the tile grid.
    for cfg, lasts in ((wl.tiny(wl.CONFIGS[3], B=6, T=2, H=8, C=256), (1151, 640, 127, 333, 31, None)),
                       (wl.tiny(wl.CONFIGS[2], B=5, Hg=9, Wg=13, N=45, H=6, d=64, C=264), (116, 95, 64, 0, None))):
        Mv = cfg.M
        t = wl.prefill_inputs(cfg)
        rng = np.random.default_rng(17)
        vis_valid = np.zeros((cfg.B, Mv), np.uint8)
        for b, last in enumerate(lasts):
            if last is None:
                continue
            vis_valid[b, :last + 1] = rng.random(last + 1) > (0.0 if b == 0 else 0.25)   # sample 0: a plain prefix
            vis_valid[b, last] = 1
        bad = vis_valid == 0
        t["k"][:, :Mv][bad] = 0x7FC0
        t["v"][:, :Mv][bad] = 0x7F80
        t["hidden"][:, :Mv][bad] = 0xFFFF
        is_key = wl.random_key_mask(cfg, 6, valid=vis_valid)
        for R in (8, 48):
            g, o, s = run(t, Mv, R, vis_valid=vis_valid, is_key=is_key)
            assert np.array_equal(g["kept_count"], np.minimum(np.maximum(R, is_key.sum(1)), vis_valid.sum(1)))
            assert np.all(g["score_global"][bad] == 0) and np.all(g["score_indiv"][bad] == 0)
        g, o, s = run(t, Mv, 0, mode=FILTER_THRESHOLD, vis_valid=vis_valid, is_key=is_key, gamma=1.0 / Mv, alpha=1.5 / Mv)
        assert g["kept_count"][len(lasts) - 1] == 0
        # the same mask and the caller's row normalisers: one sweep, same selection
        from paper_2411_10803_amd import harness
        scale = 1.0 / np.sqrt(cfg.d)
        o = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], vis_valid, None, is_key, Mv, scale, FILTER_BUDGET,
                                  48, 1.0 / Mv, 2.0 / cfg.L, 48)
        g2 = harness.prefill_on_gpu(t, Mv, vis_valid, None, is_key, scale, FILTER_BUDGET, 48, 1.0 / Mv, 2.0 / cfg.L, 48,
                                    row_lse=o["row_lse"].astype(np.float32))
        check_prefill(g2, o, t, Mv, vis_valid, is_key, FILTER_BUDGET, 48, 1.0 / Mv, 2.0 / cfg.L, 48)


def test_long_prompts_more_than_128_text_rows():
    # the column scores of a long prompt come from several launches (128 text rows each) that are merged
    cfg = wl.tiny(wl.CONFIGS[2], B=2, Hg=9, Wg=13, N=300, H=4, d=128, C=64)
    t = wl.prefill_inputs(cfg)
    txt_len = np.array([300, 131], dtype=np.int32)
    is_key = wl.random_key_mask(cfg, 7)
    for R in (20, 60):
        run(t, cfg.M, R, txt_len=txt_len, is_key=is_key)
    run(t, cfg.M, 0, mode=FILTER_THRESHOLD, txt_len=txt_len, is_key=is_key, gamma=1.0 / cfg.M, alpha=1.5 / cfg.M)
    cfg = wl.tiny(wl.CONFIGS[2], B=1, Hg=6, Wg=6, N=1024, H=2, d=64, C=64)
    run(wl.prefill_inputs(cfg), cfg.M, 12)


def test_threshold_mode_and_special_cases():
    cfg = wl.tiny(wl.CONFIGS[2], B=2, Hg=8, Wg=12, N=32, H=4, d=128, C=512)
    Mv = cfg.M
    t = wl.prefill_inputs(cfg)
    is_key = wl.random_key_mask(cfg, 4)
    g, _, _ = run(t, Mv, 0, mode=FILTER_THRESHOLD, gamma=-1.0, alpha=0.5, is_key=is_key)
    assert np.all(g["kept_count"] == Mv)
    g, _, _ = run(t, Mv, 0, mode=FILTER_THRESHOLD, gamma=1.0, alpha=np.inf, is_key=is_key)
    assert np.all(g["kept_count"] == 4)
    run(t, Mv, 0, mode=FILTER_THRESHOLD, gamma=1.0 / Mv, alpha=2.0 / Mv, is_key=is_key)
    # more keys than budget: true count reported, storage stops at Rcap
    g, o, _ = run(t, Mv, 2, is_key=is_key)
    assert np.all(g["kept_count"] == 4) and np.all(g["out_len"] == 2 + 32)
    # zero queries: every score ties -> lowest indices win, harmonic-number closed form
    t0 = dict(t)
    t0["q_txt"] = np.zeros_like(t["q_txt"])
    g, o, _ = run(t0, Mv, 10)
    assert g["kept_index"].tolist() == [list(range(10))] * 2
    H_ = sum(1.0 / (Mv + i + 1) for i in range(32))
    assert np.allclose(g["score_global"], H_, rtol=1e-5) and np.allclose(g["score_indiv"], 1.0 / (Mv + 1), rtol=1e-5)
    # literal N(0,1)/sqrt(d) inputs: near-uniform softmax, graded on counts and invariants
    tl = wl.prefill_inputs(cfg, literal_scale=True)
    g, o, s = run(tl, Mv, 24, is_key=is_key)
    assert np.all(g["kept_count"] == 24)


def test_determinism():
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[2], B=2)
    t = wl.prefill_inputs(cfg)
    runs = [harness.prefill_on_gpu(t, cfg.M, None, None, None, 1 / np.sqrt(128), FILTER_BUDGET, 128,
                                   1.0 / cfg.M, 2.0 / cfg.L) for _ in range(3)]
    for r in runs[1:]:
        for name in ("kept_index", "score_global", "score_indiv", "k_out", "hidden_out"):
            assert np.array_equal(runs[0][name], r[name]), name


@pytest.mark.parametrize("which", ["cfg2_slice", "cfg3_one", "ragged_d64", "long_prompt"])
def test_row_lse_input_skips_the_first_sweep_and_gives_the_same_answer(which):
    """Sec. 3.4: the text-to-vision scores are a by-product of the layer's attention.  With the attention's row
    normalisers handed over (here: the oracle's, rounded to fp32) the library reads K once; V, I and the selection
    must still match the plain oracle result, and the results with and without the normalisers must agree."""
    from paper_2411_10803_amd import harness
    rng = np.random.default_rng(17)
    vis_valid = txt_len = None
    if which == "cfg2_slice":
        cfg, samples, R = wl.CONFIGS[2], [0, 3, 9, 15], 128
    elif which == "cfg3_one":
        cfg, samples, R = wl.CONFIGS[3], [2], 320
    elif which == "ragged_d64":
        cfg, samples, R = wl.tiny(wl.CONFIGS[2], B=3, Hg=7, Wg=11, N=45, H=6, d=64, C=264), None, 20
        vis_valid = (rng.random((cfg.B, cfg.M)) > 0.3).astype(np.uint8)
        txt_len = np.array([45, 17, 1], dtype=np.int32)
    else:
        cfg, samples, R = wl.tiny(wl.CONFIGS[2], B=2, Hg=9, Wg=13, N=200, H=4, d=128, C=256), None, 40
        txt_len = np.array([200, 131], dtype=np.int32)
    t = wl.prefill_inputs(cfg, samples)
    B = t["k"].shape[0]
    is_key = wl.random_key_mask(cfg, 8)[:B]
    if vis_valid is not None:
        is_key &= vis_valid
    Mv, N = cfg.M, cfg.N
    scale, gamma, alpha = 1.0 / np.sqrt(cfg.d), 1.0 / Mv, 2.0 / (Mv + N)
    o = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], vis_valid, txt_len, is_key, Mv, scale,
                              FILTER_BUDGET, R, gamma, alpha, R)
    lse = o["row_lse"].astype(np.float32)
    if txt_len is not None:                       # entries of rows beyond txt_len are ignored: poison them
        for b in range(B):
            lse[b, :, int(txt_len[b]):] = np.nan
    g0 = harness.prefill_on_gpu(t, Mv, vis_valid, txt_len, is_key, scale, FILTER_BUDGET, R, gamma, alpha, R)
    g1 = harness.prefill_on_gpu(t, Mv, vis_valid, txt_len, is_key, scale, FILTER_BUDGET, R, gamma, alpha, R, row_lse=lse)
    check_prefill(g0, o, t, Mv, vis_valid, is_key, FILTER_BUDGET, R, gamma, alpha, R)
    s1 = check_prefill(g1, o, t, Mv, vis_valid, is_key, FILTER_BUDGET, R, gamma, alpha, R)
    assert s1["max_V_rel"] < 1e-4 and s1["max_I_rel"] < 1e-4
    ok = np.ones((B, Mv), bool) if vis_valid is None else vis_valid.astype(bool)
    assert np.allclose(g1["score_global"][ok], g0["score_global"][ok], rtol=1e-5, atol=0)
    assert np.allclose(g1["score_indiv"][ok], g0["score_indiv"][ok], rtol=1e-5, atol=0)
    assert np.array_equal(g1["kept_count"], g0["kept_count"])
    # threshold mode through the same path
    gth = harness.prefill_on_gpu(t, Mv, vis_valid, txt_len, is_key, scale, FILTER_THRESHOLD, 0, gamma, alpha, Mv, row_lse=lse)
    oth = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], vis_valid, txt_len, is_key, Mv, scale,
                                FILTER_THRESHOLD, 0, gamma, alpha, Mv)
    check_prefill(gth, oth, t, Mv, vis_valid, is_key, FILTER_THRESHOLD, 0, gamma, alpha, Mv)
