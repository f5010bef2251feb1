"""GPU parity at the benchmark's full sizes and launch configurations (all five workloads).

The GPU runs the full batch and the oracle checks every sample of it, element by element; the prefill
stage is fed from the encode stage's own validity mask and key set, as the benchmark chains them."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import FILTER_BUDGET
from parity import check_decode, check_encode, check_prefill

pytestmark = pytest.mark.gpu

BENCH_TAU = wl.CONFIGS[2].bench_tau


def encode_both(cfg, tau, samples=None):
    from paper_2411_10803_amd import harness
    e = wl.encode_inputs(cfg)
    args = (cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, tau, cfg.key_budget)
    g = harness.encode_on_gpu(e["x"], cfg.x_dtype, e["q_cls"], e["k_cls"], cfg.x_dtype, None, None, *args)
    idx = list(range(cfg.B)) if samples is None else samples
    sub = lambda a: np.ascontiguousarray(a[idx])
    o = oracle.encode_merge(sub(e["x"]), cfg.x_dtype, sub(e["q_cls"]), sub(e["k_cls"]), cfg.x_dtype, None, None, *args)
    gs = {k: (v[idx] if isinstance(v, np.ndarray) and v.shape[:1] == (cfg.B,) else v) for k, v in g.items()}
    s = check_encode(gs, o, sub(e["x"]), cfg.x_dtype, None, *args)
    return e, g, s


def prefill_both(cfg, t, vis_valid, is_key, budget, samples=None):
    from paper_2411_10803_amd import harness
    scale, gamma, alpha = 1.0 / np.sqrt(cfg.d), 1.0 / cfg.M, 2.0 / cfg.L
    g = harness.prefill_on_gpu(t, cfg.M, vis_valid, None, is_key, scale, FILTER_BUDGET, budget, gamma, alpha, budget)
    idx = list(range(cfg.B)) if samples is None else samples
    sub = lambda a: None if a is None else np.ascontiguousarray(a[idx])
    ts = {k: sub(v) for k, v in t.items()}
    o = oracle.prefill_filter(ts["q_txt"], ts["k"], ts["v"], ts["hidden"], sub(vis_valid), None, sub(is_key), cfg.M,
                              scale, FILTER_BUDGET, budget, gamma, alpha, budget)
    gs = {k: v[idx] for k, v in g.items()}
    s = check_prefill(gs, o, ts, cfg.M, sub(vis_valid), sub(is_key), FILTER_BUDGET, budget, gamma, alpha, budget)
    # properties on the whole batch: count = min(budget, valid tokens), keys kept, rows are exact copies
    for b in range(cfg.B):
        nv = cfg.M if vis_valid is None else int(vis_valid[b].sum())
        assert g["kept_count"][b] == min(budget, nv)
        n = int(g["kept_count"][b])
        kept = g["kept_index"][b, :n]
        assert np.all(np.diff(kept) > 0)
        if is_key is not None:
            keys = np.flatnonzero(is_key[b] & (1 if vis_valid is None else vis_valid[b]))
            assert set(keys.tolist()) <= set(kept.tolist())
        rows = np.concatenate([kept, cfg.M + np.arange(cfg.N)])
        assert np.array_equal(g["k_out"][b, :rows.size], t["k"][b, rows])
        assert np.array_equal(g["hidden_out"][b, :rows.size], t["hidden"][b, rows])
        assert np.array_equal(g["out_ids"][b, :rows.size], rows)
    return g, s


def test_config2_full_batch_chained_three_budgets():
    cfg = wl.CONFIGS[2]
    e, g1, s1 = encode_both(cfg, BENCH_TAU)
    assert s1["merged_rows_checked"] > 100 and s1["copied_rows_checked"] > 1000   # both kinds of rows were compared
    assert 300 < g1["out_count"].mean() < 576                  # partial merging, near the paper's average of 440
    t = wl.prefill_inputs(cfg)
    for R in cfg.budgets:
        prefill_both(cfg, t, g1["out_valid"], g1["out_is_key"], R)
    # nominal shape as well: all 576 slots valid, seeded key set
    prefill_both(cfg, t, None, wl.random_key_mask(cfg, cfg.key_budget), 192, samples=[0, 7, 15])


def test_config1_full():
    cfg = wl.CONFIGS[1]
    e, g1, s1 = encode_both(cfg, cfg.bench_tau)
    assert s1["merged_rows_checked"] > 10 and 192 < g1["out_count"][0] < cfg.M
    t = wl.prefill_inputs(cfg)
    prefill_both(cfg, t, g1["out_valid"], g1["out_is_key"], 192)


def test_config3_full_batch():
    cfg = wl.CONFIGS[3]
    e, g1, s1 = encode_both(cfg, cfg.bench_tau)
    assert s1["merged_rows_checked"] > 100 and np.all(g1["out_count"] > 320) and np.all(g1["out_count"] < cfg.M)
    t = wl.prefill_inputs(cfg)
    prefill_both(cfg, t, g1["out_valid"], g1["out_is_key"], 320)          # chained, every sample
    prefill_both(cfg, t, None, wl.random_key_mask(cfg, cfg.key_budget), 320, samples=[5])   # nominal shape


def test_config4_full_batch_video_windows():
    cfg = wl.CONFIGS[4]
    e, g1, s1 = encode_both(cfg, cfg.bench_tau)
    assert s1["merged_rows_checked"] > 100 and np.all(g1["out_count"] > 512) and np.all(g1["out_count"] < cfg.M)
    t = wl.prefill_inputs(cfg)
    prefill_both(cfg, t, g1["out_valid"], g1["out_is_key"], 512)          # chained, every sample
    prefill_both(cfg, t, None, wl.random_key_mask(cfg, cfg.key_budget), 512, samples=[3])   # nominal shape


def test_config5_decode_full_size():
    import torch
    import paper_2411_10803_amd as md
    from paper_2411_10803_amd import harness
    cfg = wl.CONFIGS[5]
    steps = cfg.steps                                # all 256 steps of the workload
    t = wl.decode_inputs(cfg, steps=steps, Lcap=cfg.L0 + cfg.steps)
    B, Lcap = cfg.B, t["Lcap"]
    scale = 1.0 / np.sqrt(cfg.d)
    s0 = {"k": t["k_cache"], "v": t["v_cache"], "acc": np.zeros((B, Lcap), np.float32),
          "ids": np.tile(np.arange(Lcap, dtype=np.int32), (B, 1)), "protect": t["protect"].copy(), "len": t["len0"].copy()}
    d = harness.decode_state_to_dev(s0)
    ws = md.decode_workspace(B, Lcap, cfg.H)
    qs, kn, vn = (harness.to_dev(t[n], True) for n in ("q_steps", "k_new", "v_new"))
    # step 1 (4096 -> 1024) on the full batch against the oracle on every sample
    ev, evc = harness.decode_on_gpu(qs[0], d, scale, 1.0, cfg.decode_budget, ws)
    g = harness.decode_state_to_host(d, ev, evc)
    o = {k: v.copy() for k, v in s0.items()}
    r = oracle.decode_evict(t["q_steps"][0], o["k"], o["v"], o["acc"], o["ids"], o["protect"], o["len"], scale, 1.0,
                            cfg.decode_budget)
    o["acc_all"] = r["a_t"].astype(np.float32)
    o["evicted_ids"], o["evicted_count"] = r["evicted_ids"], r["evicted_count"]
    summ = check_decode(g, o, s0, cfg.decode_budget)
    assert np.all(g["len"] == cfg.decode_budget)
    for b in range(B):
        assert set(np.flatnonzero(t["heavy"][b]).tolist()) <= set(g["ids"][b, :cfg.decode_budget].tolist())
    # free-running loops on both sides, each on its own state: append + evict for every further step.  The
    # oracle's loop never sees a GPU value.  A step is decisive for a sample when the two smallest running
    # scores among its unprotected entries are more than the margin apart: there the evicted id must be the
    # oracle's.  At a near-tie the two sides may evict different entries; their states then differ and the
    # sample leaves the comparison.  A sample that never parted must end in the oracle's state (slot-by-slot
    # ids, scores within tolerance, rows bit-identical).
    from parity import MARGIN, RTOL
    gpu_evicted = []
    for s in range(1, steps):
        md.mustdrop_decode_append(kn[s], vn[s], d["k"], d["v"], d["acc"], d["ids"], d["protect"], d["len"], cfg.L0 + s)
        ev, evc = harness.decode_on_gpu(qs[s], d, scale, 1.0, cfg.decode_budget, ws)
        gpu_evicted.append((ev[:, 0].clone(), evc.clone()))
    torch.cuda.synchronize()
    from concurrent.futures import ThreadPoolExecutor
    pool = ThreadPoolExecutor(8)
    decisive = np.ones(B, dtype=bool)
    n_compared = 0
    for s in range(1, steps):
        for b in range(B):
            n = int(o["len"][b])
            o["k"][b, n], o["v"][b, n] = t["k_new"][s][b], t["v_new"][s][b]
            o["acc"][b, n], o["ids"][b, n], o["protect"][b, n] = 0.0, cfg.L0 + s, 1
            o["len"][b] = n + 1
        acc_pre, prot_pre, len_pre = o["acc"].copy(), o["protect"].copy(), o["len"].copy()
        # the oracle (single-threaded C) on slices of the batch side by side: samples are independent, the slices
        # are views of the one state, the library call releases the interpreter lock
        def oracle_slice(lo):
            sl = slice(lo, lo + 8)
            return oracle.decode_evict(t["q_steps"][s][sl], o["k"][sl], o["v"][sl], o["acc"][sl], o["ids"][sl], o["protect"][sl],
                                       o["len"][sl], scale, 1.0, cfg.decode_budget)
        parts = list(pool.map(oracle_slice, range(0, B, 8)))
        r = {k: np.concatenate([q[k] for q in parts], axis=0) for k in ("a_t", "evicted_ids", "evicted_count")}
        ge, gc = (x.cpu().numpy() for x in gpu_evicted[s - 1])
        assert np.all(r["evicted_count"] == 1) and np.all(gc == 1)
        for b in range(B):
            n = int(len_pre[b])
            upd = (acc_pre[b, :n].astype(np.float64) + r["a_t"][b, :n]).astype(np.float32)
            low = np.sort(upd[prot_pre[b, :n] == 0])[:2].astype(np.float64)
            if not decisive[b]:
                continue                                 # the two loops parted at an earlier near-tie
            near_tie = abs(low[1] - low[0]) <= MARGIN * abs(0.5 * (low[0] + low[1]))
            if ge[b] != r["evicted_ids"][b, 0]:
                assert near_tie, f"step {s}, sample {b}: evicted id differs at a decisive step"
                decisive[b] = False                      # a legitimate difference: the states differ from here on
            else:
                n_compared += 1
    print(f"decode loop: {int(decisive.sum())} of {B} samples never met a near-tie; {n_compared} evictions compared")
    assert decisive.sum() >= B - 4 and n_compared >= (B - 4) * (steps - 1)
    g = harness.decode_state_to_host(d)
    assert np.all(g["len"] == cfg.decode_budget)
    for b in range(B):
        ids = g["ids"][b, :cfg.decode_budget]
        assert len(set(ids.tolist())) == ids.size                           # ids stay unique
        prot_ids = set(np.flatnonzero(t["protect"][b]).tolist()) | set(range(cfg.L0 + 1, cfg.L0 + steps))
        assert prot_ids <= set(ids.tolist())                                # protected entries never leave
        old, slots = ids[ids < cfg.L0], np.flatnonzero(ids < cfg.L0)
        assert np.array_equal(g["k"][b, slots], t["k_cache"][b, old])       # rows still paired with their ids
        assert np.array_equal(g["v"][b, slots], t["v_cache"][b, old])
        if decisive[b]:
            nb = cfg.decode_budget
            assert np.array_equal(g["ids"][b, :nb], o["ids"][b, :nb])
            assert np.array_equal(g["protect"][b, :nb], o["protect"][b, :nb])
            assert np.array_equal(g["k"][b, :nb], o["k"][b, :nb]) and np.array_equal(g["v"][b, :nb], o["v"][b, :nb])
            rel = np.abs(g["acc"][b, :nb].astype(np.float64) - o["acc"][b, :nb]) / np.maximum(np.abs(o["acc"][b, :nb]), 1e-300)
            assert rel.max() <= RTOL
