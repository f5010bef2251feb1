"""GPU parity: mustdrop_decode_evict / mustdrop_decode_append (HIP, through the C ABI) against the CPU oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from parity import check_decode

pytestmark = pytest.mark.gpu


def initial_state(t):
    B, Lcap = t["protect"].shape
    return {"k": t["k_cache"].copy(), "v": t["v_cache"].copy(), "acc": np.zeros((B, Lcap), np.float32),
            "ids": np.tile(np.arange(Lcap, dtype=np.int32), (B, 1)), "protect": t["protect"].copy(),
            "len": t["len0"].copy()}


def oracle_step(s, q, scale, decay, budget):
    """Oracle step on a copy of host state `s`; also returns the updated scores in pre-compaction order."""
    o = {k: v.copy() for k, v in s.items()}
    acc_pre = o["acc"].astype(np.float64)
    r = oracle.decode_evict(q, o["k"], o["v"], o["acc"], o["ids"], o["protect"], o["len"], scale, decay, budget)
    o["acc_all"] = (float(np.float32(decay)) * acc_pre + r["a_t"]).astype(np.float32)
    o["evicted_ids"], o["evicted_count"] = r["evicted_ids"], r["evicted_count"]
    return o


def gpu_step(s, q, scale, decay, budget):
    from paper_2411_10803_amd import harness
    d = harness.decode_state_to_dev(s)
    ev, evc = harness.decode_on_gpu(harness.to_dev(q, True), d, scale, decay, budget)
    return harness.decode_state_to_host(d, ev, evc)


def test_first_step_evicts_to_budget_and_matches_oracle():
    cfg = wl.tiny(wl.CONFIGS[5], B=3, L0=1500, steps=2, decode_budget=400, n_protect=50)
    t = wl.decode_inputs(cfg)
    s = initial_state(t)
    scale = 1 / np.sqrt(cfg.d)
    g = gpu_step(s, t["q_steps"][0], scale, 1.0, cfg.decode_budget)
    o = oracle_step(s, t["q_steps"][0], scale, 1.0, cfg.decode_budget)
    summ = check_decode(g, o, s, cfg.decode_budget)
    assert np.all(g["len"] == 400)
    for b in range(cfg.B):
        heavy = set(np.flatnonzero(t["heavy"][b]).tolist())
        assert heavy <= set(g["ids"][b, :400].tolist())        # planted heavy hitters survive


def test_teacher_forced_decode_loop_with_append():
    # every step starts from the oracle's state, so each step is compared from identical inputs
    from paper_2411_10803_amd import harness
    import paper_2411_10803_amd as md
    cfg = wl.tiny(wl.CONFIGS[5], B=2, L0=300, steps=6, decode_budget=96, n_protect=20, H=8)
    t = wl.decode_inputs(cfg)
    s = initial_state(t)
    scale = 1 / np.sqrt(cfg.d)
    for step in range(cfg.steps):
        if step > 0:
            # append on the GPU, and the same by hand on the host state
            d = harness.decode_state_to_dev(s)
            md.mustdrop_decode_append(harness.to_dev(t["k_new"][step], True), harness.to_dev(t["v_new"][step], True),
                                      d["k"], d["v"], d["acc"], d["ids"], d["protect"], d["len"], cfg.L0 + step)
            ga = harness.decode_state_to_host(d)
            for b in range(cfg.B):
                n = s["len"][b]
                s["k"][b, n], s["v"][b, n] = t["k_new"][step][b], t["v_new"][step][b]
                s["acc"][b, n], s["ids"][b, n], s["protect"][b, n] = 0.0, cfg.L0 + step, 1
                s["len"][b] = n + 1
            for name in ("k", "v", "acc", "ids", "protect", "len"):
                assert np.array_equal(ga[name], s[name]), f"append: {name}"
        g = gpu_step(s, t["q_steps"][step], scale, 1.0, cfg.decode_budget)
        o = oracle_step(s, t["q_steps"][step], scale, 1.0, cfg.decode_budget)
        check_decode(g, o, s, cfg.decode_budget)
        assert np.all(g["len"] == cfg.decode_budget)
        s = {k: o[k] for k in ("k", "v", "acc", "ids", "protect", "len")}


def test_special_cases():
    cfg = wl.tiny(wl.CONFIGS[5], B=2, L0=200, steps=1, decode_budget=64, n_protect=30, H=4, d=64)
    t = wl.decode_inputs(cfg)
    scale = 1 / np.sqrt(cfg.d)
    q = t["q_steps"][0]
    # static policy of the paper: budget = number of protected entries -> survivors = protected set
    s = initial_state(t)
    g = gpu_step(s, q, scale, 1.0, 30)
    o = oracle_step(s, q, scale, 1.0, 30)
    check_decode(g, o, s, 30)
    for b in range(cfg.B):
        assert set(g["ids"][b, :30].tolist()) == set(np.flatnonzero(t["protect"][b]).tolist())
    # nothing to evict: only the scores change; cumulative score sums to the step count
    s = initial_state(t)
    g = gpu_step(s, q, scale, 1.0, 1000)
    assert np.array_equal(g["k"], s["k"]) and np.array_equal(g["ids"], s["ids"]) and np.all(g["len"] == 200)
    assert np.allclose(g["acc"][:, :200].sum(1), 1.0, rtol=1e-4)
    assert np.all(g["evicted_count"] == 0)
    g2 = gpu_step(g, q, scale, 0.5, 1000)
    assert np.allclose(g2["acc"][:, :200], 1.5 * g["acc"][:, :200], rtol=1e-5)
    # more protected entries than budget: exactly the protected stay
    g = gpu_step(s, q, scale, 1.0, 5)
    assert np.all(g["len"] == 30)
    # all scores tie (zero query): lower ids win, whatever slot they sit in
    s = initial_state(t)
    s["protect"][:] = 0
    s["ids"][:, :200] = np.arange(199, -1, -1, dtype=np.int32)
    g = gpu_step(s, np.zeros_like(q), scale, 1.0, 50)
    o = oracle_step(s, np.zeros_like(q), scale, 1.0, 50)
    assert np.array_equal(g["ids"][:, :50], o["ids"][:, :50])
    assert set(g["ids"][0, :50].tolist()) == set(range(50))
    # ragged lengths, an empty sample, a full cache
    s = initial_state(t)
    s["len"][:] = [0, 137]
    g = gpu_step(s, q, scale, 1.0, 64)
    o = oracle_step(s, q, scale, 1.0, 64)
    check_decode(g, o, s, 64)
    assert g["len"].tolist() == o["len"].tolist()


def test_determinism():
    cfg = wl.tiny(wl.CONFIGS[5], B=2, L0=1024, steps=1, decode_budget=256, n_protect=32)
    t = wl.decode_inputs(cfg)
    s = initial_state(t)
    runs = [gpu_step(s, t["q_steps"][0], 1 / np.sqrt(128), 1.0, 256) for _ in range(3)]
    for r in runs[1:]:
        for name in ("k", "v", "acc", "ids", "protect", "len", "evicted_ids"):
            assert np.array_equal(runs[0][name], r[name]), name


@pytest.mark.parametrize("n_layers,B,Lcap,H,d,seed", [(4, 3, 700, 32, 128, 1), (2, 2, 2500, 5, 64, 2), (1, 1, 9, 1, 8, 3)])
def test_static_policy_over_layers(n_layers, B, Lcap, H, d, seed):
    """Sec. 3.5 as printed: keep the flagged entries in the caches of all layers (no scoring).  Integer and
    byte work only: everything must match the oracle bit for bit."""
    import torch
    import paper_2411_10803_amd as md
    from paper_2411_10803_amd import harness
    rng = np.random.default_rng(seed)
    k = rng.integers(0, 1 << 16, size=(n_layers, B, Lcap, H, d), dtype=np.uint16) & np.uint16(0xBFFF)
    v = rng.integers(0, 1 << 16, size=(n_layers, B, Lcap, H, d), dtype=np.uint16) & np.uint16(0xBFFF)
    acc = rng.random((B, Lcap)).astype(np.float32)
    ids = np.stack([rng.permutation(4 * Lcap)[:Lcap] for _ in range(B)]).astype(np.int32)
    protect = (rng.random((B, Lcap)) < 0.3).astype(np.uint8)
    lens = rng.integers(0, Lcap + 1, size=B).astype(np.int32)
    lens[0] = Lcap
    keep = (rng.random((B, Lcap)) < rng.random((B, 1))).astype(np.uint8)
    for with_acc in (True, False):
        ko, vo, ao, io, po, lo = k.copy(), v.copy(), acc.copy(), ids.copy(), protect.copy(), lens.copy()
        o = oracle.decode_keep(ko, vo, keep, ao if with_acc else None, io, po, lo)
        kd, vd = harness.to_dev(k, True), harness.to_dev(v, True)
        ad, idd, pd, ld = (harness.to_dev(a) for a in (acc, ids, protect, lens))
        ev = torch.full((B, Lcap), -1, dtype=torch.int32, device="cuda")
        evc = torch.zeros((B,), dtype=torch.int32, device="cuda")
        md.mustdrop_decode_keep(kd, vd, harness.to_dev(keep), ad if with_acc else None, idd, pd, ld, ev, evc)
        torch.cuda.synchronize()
        assert np.array_equal(harness.to_host(ld), lo)
        assert np.array_equal(harness.to_host(evc), o["evicted_count"])
        kg, vg = harness.to_host(kd), harness.to_host(vd)
        for b in range(B):
            n, ne = int(lo[b]), int(o["evicted_count"][b])
            for l in range(n_layers):
                assert np.array_equal(kg[l, b, :n], ko[l, b, :n]) and np.array_equal(vg[l, b, :n], vo[l, b, :n])
                assert np.array_equal(kg[l, b, lens[b]:], k[l, b, lens[b]:])          # beyond the old length: untouched
            assert np.array_equal(harness.to_host(idd)[b, :n], io[b, :n])
            assert np.array_equal(harness.to_host(pd)[b, :n], po[b, :n])
            if with_acc:
                assert np.array_equal(harness.to_host(ad)[b, :n], ao[b, :n])
            assert np.array_equal(harness.to_host(ev)[b, :ne], o["evicted_ids"][b, :ne])
