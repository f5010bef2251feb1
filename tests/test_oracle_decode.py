"""Pins for the stage-3 oracle (Sec. 3.5: output-aware cache policy; decode attention of Eq. 4)."""
from itertools import combinations

import numpy as np
import pytest

import oracle
import workloads as wl


def state(B=2, L=24, Lcap=32, H=2, d=8, seed=0, n_protect=4):
    rng = np.random.default_rng(seed)
    f = lambda *s: wl.f32_to_bf16_bits(rng.standard_normal(s).astype(np.float32))
    k = f(B, Lcap, H, d)
    v = f(B, Lcap, H, d)
    protect = np.zeros((B, Lcap), dtype=np.uint8)
    for b in range(B):
        protect[b, rng.choice(L, n_protect, replace=False)] = 1
    return dict(q=f(B, H, d), k=k, v=v, acc=np.zeros((B, Lcap), np.float32),
                ids=np.tile(np.arange(Lcap, dtype=np.int32), (B, 1)), protect=protect,
                len=np.full(B, L, np.int32), H=H, d=d, B=B, L=L, Lcap=Lcap)


def step(s, budget, decay=1.0, scale=None):
    scale = 1 / np.sqrt(s["d"]) if scale is None else scale
    return oracle.decode_evict(s["q"], s["k"], s["v"], s["acc"], s["ids"], s["protect"], s["len"], scale, decay, budget)


def numpy_probs(s, scale):
    scale = float(np.float32(scale))               # the C ABI carries the scale as a float
    q = wl.to_f64(s["q"], wl.BF16)
    k = wl.to_f64(s["k"], wl.BF16)
    out = np.zeros((s["B"], s["Lcap"]))
    for b in range(s["B"]):
        n = s["len"][b]
        lg = scale * np.einsum("hc,jhc->hj", q[b], k[b, :n])
        p = np.exp(lg - lg.max(-1, keepdims=True))
        p /= p.sum(-1, keepdims=True)
        out[b, :n] = p.mean(0)
    return out


def test_probabilities_match_numpy_and_sum_to_one():
    s = state(seed=1)
    ref = numpy_probs(s, 1 / np.sqrt(s["d"]))
    o = step(s, budget=100)
    assert np.allclose(o["a_t"], ref, rtol=1e-12, atol=0)
    assert np.allclose(o["a_t"].sum(1), 1.0, atol=1e-12)
    assert np.array_equal(s["len"], [24, 24]) and np.all(o["evicted_count"] == 0)
    assert np.allclose(s["acc"], ref, rtol=1e-6)
    # cumulative score: with decay 1 and no eviction the total equals the number of steps
    for _ in range(3):
        step(s, budget=100)
    assert np.allclose(s["acc"].sum(1), 4.0, rtol=1e-5)
    s2 = state(seed=1)
    s2["acc"][:] = 5.0
    step(s2, budget=100, decay=0.0)               # decay 0: instantaneous score
    assert np.allclose(s2["acc"][:, :24], ref[:, :24], rtol=1e-6)
    assert np.all(s2["acc"][:, 24:] == 5.0)       # slots beyond len are not touched
    s3 = state(seed=1)
    s3["acc"][:] = 2.0
    step(s3, budget=100, decay=0.5)
    assert np.allclose(s3["acc"][:, :24], 1.0 + ref[:, :24], rtol=1e-6)


def test_static_policy_keeps_exactly_the_protected_set():
    # protect = S_few and budget = |S_few|: the survivors are S_few whatever the scores say
    s = state(seed=2, n_protect=7)
    want = [set(s["ids"][b, np.flatnonzero(s["protect"][b, :24])].tolist()) for b in range(2)]
    o = step(s, budget=7)
    for b in range(2):
        assert s["len"][b] == 7
        assert set(s["ids"][b, :7].tolist()) == want[b]
        assert np.all(s["protect"][b, :7] == 1)
        assert o["evicted_count"][b] == 17
    # more protected entries than budget: exactly the protected are kept
    s = state(seed=2, n_protect=7)
    step(s, budget=3)
    assert np.all(s["len"] == 7)


def test_hole_filling_layout_and_row_pairing():
    s = state(seed=3, B=3, L=30, Lcap=30, n_protect=5)
    k0, v0, ids0, p0 = s["k"].copy(), s["v"].copy(), s["ids"].copy(), s["protect"].copy()
    budget = 12
    o = step(s, budget=budget)
    acc_after_update = numpy_probs(dict(s, k=k0, len=np.full(3, 30)), 1 / np.sqrt(s["d"]))
    for b in range(3):
        n = s["len"][b]
        assert n == budget
        unprot = np.flatnonzero(p0[b] == 0)
        order = unprot[np.argsort(-acc_after_update[b, unprot].astype(np.float32), kind="stable")]
        keep = set(np.flatnonzero(p0[b]).tolist()) | set(order[:budget - 5].tolist())
        assert set(s["ids"][b, :n].tolist()) == keep
        # survivors already below new_len do not move; movers fill holes in ascending order
        holes = [j for j in range(n) if j not in keep]
        movers = [j for j in range(n, 30) if j in keep]
        assert len(holes) == len(movers)
        expect = np.arange(n)
        expect[holes] = movers
        assert s["ids"][b, :n].tolist() == expect.tolist()
        # every row stays bit-identical and paired with its id / protect flag
        for slot in range(n):
            src = s["ids"][b, slot]
            assert np.array_equal(s["k"][b, slot], k0[b, src])
            assert np.array_equal(s["v"][b, slot], v0[b, src])
            assert s["protect"][b, slot] == p0[b, src]
            assert s["acc"][b, slot] == pytest.approx(acc_after_update[b, src], rel=1e-6)
        ev = o["evicted_ids"][b, :o["evicted_count"][b]]
        assert ev.tolist() == sorted(set(range(30)) - keep)


def test_top_by_score_is_the_subset_with_the_largest_retained_mass():
    s = state(seed=4, B=1, L=12, Lcap=12, H=2, d=4, n_protect=2)
    p0 = s["protect"].copy()
    a = numpy_probs(s, 1 / np.sqrt(s["d"]))[0].astype(np.float32)
    step(s, budget=6)
    unprot = np.flatnonzero(p0[0] == 0).tolist()
    best = max(combinations(unprot, 4), key=lambda c: sum(float(a[j]) for j in c))
    assert set(s["ids"][0, :6].tolist()) == set(best) | set(np.flatnonzero(p0[0]).tolist())


def test_ties_break_towards_lower_id():
    s = state(seed=5, B=1, L=10, Lcap=10, n_protect=0)
    s["q"][:] = 0                                  # uniform attention: every entry ties
    s["ids"][0] = np.array([9, 8, 7, 6, 5, 4, 3, 2, 1, 0], dtype=np.int32)
    step(s, budget=4)
    assert s["len"][0] == 4
    assert set(s["ids"][0, :4].tolist()) == {0, 1, 2, 3}
    # ids 9..6 sat in slots 0..3 and were evicted; survivors (slots 6..9) fill them in ascending slot order
    assert s["ids"][0, :4].tolist() == [3, 2, 1, 0]


def test_planted_heavy_hitters_survive_the_first_step():
    cfg = wl.tiny(wl.CONFIGS[5], B=2, L0=512, steps=1, decode_budget=128, n_protect=16, H=4, d=128)
    t = wl.decode_inputs(cfg)
    acc = np.zeros((2, t["Lcap"]), np.float32)
    ids = np.tile(np.arange(t["Lcap"], dtype=np.int32), (2, 1))
    length = t["len0"].copy()
    oracle.decode_evict(t["q_steps"][0], t["k_cache"], t["v_cache"], acc, ids, t["protect"], length,
                        1 / np.sqrt(cfg.d), 1.0, cfg.decode_budget)
    for b in range(2):
        heavy = set(np.flatnonzero(t["heavy"][b]).tolist())
        assert 10 < len(heavy) < cfg.decode_budget - 16
        assert heavy <= set(ids[b, :length[b]].tolist())
        assert length[b] == cfg.decode_budget


def test_length_rule():
    for budget, n_protect, L in [(10, 3, 24), (24, 3, 24), (30, 3, 24), (2, 5, 24)]:
        s = state(seed=6, L=L, n_protect=n_protect)
        step(s, budget=budget)
        assert np.all(s["len"] == min(L, max(budget, n_protect)))


def _random_state(rng, n_layers, B, Lcap, H, d, lens):
    k = rng.integers(0, 1 << 16, size=(n_layers, B, Lcap, H, d), dtype=np.uint16) & np.uint16(0xBFFF)
    v = rng.integers(0, 1 << 16, size=(n_layers, B, Lcap, H, d), dtype=np.uint16) & np.uint16(0xBFFF)
    acc = rng.random((B, Lcap)).astype(np.float32)
    ids = np.stack([rng.permutation(10 * Lcap)[:Lcap] for _ in range(B)]).astype(np.int32)
    protect = (rng.random((B, Lcap)) < 0.3).astype(np.uint8)
    return k, v, acc, ids, protect, np.array(lens, dtype=np.int32)


def test_static_policy_over_layers_brute_force_and_invariants():
    """Sec. 3.5 as printed: only the flagged entries stay, in every layer's cache.  Checked against a direct
    Python construction of the hole-filling layout and against the invariants that define it."""
    rng = np.random.default_rng(11)
    n_layers, B, Lcap, H, d = 3, 4, 23, 2, 8
    k, v, acc, ids, protect, lens = _random_state(rng, n_layers, B, Lcap, H, d, [23, 17, 1, 0])
    keep = (rng.random((B, Lcap)) < 0.4).astype(np.uint8)
    keep[2, 0] = 0                                   # a sample that loses everything
    k0, v0, acc0, ids0, prot0 = k.copy(), v.copy(), acc.copy(), ids.copy(), protect.copy()
    out = oracle.decode_keep(k, v, keep, acc, ids, protect, lens)
    for b, n in enumerate([23, 17, 1, 0]):
        kept = [j for j in range(n) if keep[b, j]]
        dropped = [j for j in range(n) if not keep[b, j]]
        new_len = len(kept)
        assert lens[b] == new_len
        # slot -> source: kept entries below new_len stay; holes take the kept entries beyond, both ascending
        holes = [j for j in dropped if j < new_len]
        movers = [j for j in kept if j >= new_len]
        assert len(holes) == len(movers)
        src = list(range(new_len))
        for h_, m_ in zip(holes, movers):
            src[h_] = m_
        assert sorted(src) == kept                   # the live set is exactly the kept set
        for l in range(n_layers):
            assert np.array_equal(k[l, b, :new_len], k0[l, b, src])
            assert np.array_equal(v[l, b, :new_len], v0[l, b, src])
            assert np.array_equal(k[l, b, n:], k0[l, b, n:])             # beyond the old length: untouched
        assert np.array_equal(ids[b, :new_len], ids0[b, src])
        assert np.array_equal(protect[b, :new_len], prot0[b, src])
        assert np.array_equal(acc[b, :new_len], acc0[b, src])
        assert out["evicted_count"][b] == len(dropped)
        assert out["evicted_ids"][b, :len(dropped)].tolist() == ids0[b, dropped].tolist()


def test_static_policy_equals_the_per_step_policy_with_the_kept_set_protected():
    """The printed policy is the special case of the scored one in which the kept set is the protected set
    and the budget is its size: both oracle functions must then leave the same cache (one layer)."""
    rng = np.random.default_rng(12)
    B, Lcap, H, d = 3, 40, 2, 16
    k, v, acc, ids, _, lens = _random_state(rng, 1, B, Lcap, H, d, [40, 33, 12])
    keep = (rng.random((B, Lcap)) < 0.5).astype(np.uint8)
    q = wl.f32_to_bf16_bits(rng.standard_normal((B, H, d)).astype(np.float32))
    budget = 3                                       # below every sample's kept count: only the protected stay
    assert min(int(keep[b, :lens[b]].sum()) for b in range(B)) >= budget
    s1 = {"k": k[0].copy(), "v": v[0].copy(), "acc": acc.copy(), "ids": ids.copy(), "protect": keep.copy(), "len": lens.copy()}
    oracle.decode_evict(q, s1["k"], s1["v"], s1["acc"], s1["ids"], s1["protect"], s1["len"], 0.25, 1.0, budget)
    k2, v2, ids2, prot2, len2 = k.copy(), v.copy(), ids.copy(), keep.copy(), lens.copy()
    oracle.decode_keep(k2, v2, keep, None, ids2, prot2, len2)
    assert np.array_equal(s1["len"], len2)
    for b in range(B):
        n = len2[b]
        assert np.array_equal(s1["k"][b, :n], k2[0, b, :n]) and np.array_equal(s1["v"][b, :n], v2[0, b, :n])
        assert np.array_equal(s1["ids"][b, :n], ids2[b, :n])
        assert np.all(prot2[b, :n] == 1)
