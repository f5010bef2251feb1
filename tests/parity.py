"""GPU-vs-oracle comparison rules shared by the GPU tests, the smoke check and the benchmark.

Bar (from the benchmark spec): selected / merged indices bit-exact wherever the score margin
exceeds 1e-3; scores and merged features within 1e-2 relative error; copied rows bit-exact.
Margins: merge |S - tau| > 1e-3 (cosine units); top-k: token j is decisive iff
|s_j - s_cut| > 1e-3 * |s_cut| with s_cut the midpoint of the oracle's k-th and (k+1)-th scores.
Decisive items must match exactly; the others may differ but counts must still match.

Every function takes numpy arrays (GPU results already copied to the host) and raises
AssertionError with a description; it returns a small summary dict.
"""
from __future__ import annotations

import numpy as np

import workloads as wl

MARGIN = 1e-3
RTOL = 1e-2


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.maximum(np.abs(ref), 1e-300)
    return np.abs(got - ref) / den


def _topk_decisive(scores, k):
    """Boolean mask of decisive candidates for a top-k cut over `scores` (1-D, candidates only)."""
    n = scores.size
    if k <= 0 or k >= n:
        return np.ones(n, dtype=bool)
    s = np.sort(scores)[::-1]
    cut = 0.5 * (s[k - 1] + s[k])
    return np.abs(scores - cut) > MARGIN * abs(cut)


def _f64(a, dtype):
    return wl.to_f64(a, dtype)


# ------------------------------------------------------------------------------------------ stage 1
def check_encode(g, o, x, x_dtype, valid, T, Hg, Wg, kt, kh, kw, tau, key_budget, key_lambda=None):
    """g: GPU outputs, o: oracle outputs (dicts of numpy arrays).  key_lambda given: the key set is the
    printed form of Eq. 7 (a_cls > mean + key_lambda * std), key_budget then being the capacity of
    key_index; a token is decisive iff |a_cls - mu| > 1e-3 * |mu|."""
    B, M, D = x.shape
    ws = kt * kh * kw
    nwx, nwy = -(-Wg // kw), -(-Hg // kh)          # border windows are clipped to the grid
    tau64 = float(np.float32(tau))
    summary = {"ambiguous_windows": 0, "ambiguous_keys": 0, "max_sim_err": 0.0, "max_acls_rel": 0.0,
               "max_feat_rel": 0.0, "merged_rows_checked": 0, "copied_rows_checked": 0}

    def window_of(tok):
        xx, yy, tt = tok % Wg, (tok // Wg) % Hg, tok // (Wg * Hg)
        return ((tt // kt) * nwy + yy // kh) * nwx + xx // kw

    sim_err = np.abs(g["window_sim"].astype(np.float64) - o["window_sim"])
    assert sim_err.max() <= RTOL, f"window similarity off by {sim_err.max()}"
    summary["max_sim_err"] = float(sim_err.max())

    for b in range(B):
        vb = np.ones(M, bool) if valid is None else valid[b].astype(bool)
        amb_tok = np.zeros(M, bool)
        if key_lambda is not None and vb.any():
            ra = rel_err(g["a_cls"][b][vb], o["a_cls"][b][vb])
            assert ra.max() <= RTOL, f"a_cls relative error {ra.max()}"
            summary["max_acls_rel"] = max(summary["max_acls_rel"], float(ra.max()))
            cand = np.flatnonzero(vb)
            a = o["a_cls"][b][cand]
            mu = a.mean() + float(np.float32(key_lambda)) * a.std()
            dec = np.abs(a - mu) > MARGIN * abs(mu)
            ng_k, no_k = int(g["key_count"][b]), int(o["key_count"][b])
            if dec.all():
                assert ng_k == no_k, f"key count {ng_k} != {no_k}"
                assert np.array_equal(g["key_index"][b], o["key_index"][b]), "key_index differs"
            stored = g["key_index"][b][:min(ng_k, key_budget)]
            assert np.all(np.diff(stored) > 0) and np.all(g["key_index"][b][min(ng_k, key_budget):] == -1)
            # membership of the decisive tokens: from out_is_key of the survivors (a key token always survives)
            gkeys = set(int(t) for t, kf in zip(g["out_index"][b, :g["out_count"][b]], g["out_is_key"][b]) if kf)
            okeys = set(int(t) for t, kf in zip(o["out_index"][b, :o["out_count"][b]], o["out_is_key"][b]) if kf)
            assert len(gkeys) == ng_k and len(okeys) == no_k
            for j, d in zip(cand, dec):
                if d:
                    assert (int(j) in gkeys) == (int(j) in okeys), f"sample {b}: decisive key token {j} differs"
                else:
                    amb_tok[j] = True
            summary["ambiguous_keys"] += int((~dec).sum())
        elif key_budget > 0:
            ra = rel_err(g["a_cls"][b][vb], o["a_cls"][b][vb])
            assert ra.max() <= RTOL, f"a_cls relative error {ra.max()}"
            summary["max_acls_rel"] = max(summary["max_acls_rel"], float(ra.max()))
            cand = np.flatnonzero(vb)
            dec = _topk_decisive(o["a_cls"][b][cand], key_budget)
            gk = set(int(i) for i in g["key_index"][b] if i >= 0)
            ok = set(int(i) for i in o["key_index"][b] if i >= 0)
            assert len(gk) == len(ok), f"key count {len(gk)} != {len(ok)}"
            assert list(g["key_index"][b][:len(gk)]) == sorted(gk), "key_index not ascending"
            for j, d in zip(cand, dec):
                if d:
                    assert (j in gk) == (j in ok), f"sample {b}: decisive key token {j} differs"
                else:
                    amb_tok[j] = True
            summary["ambiguous_keys"] += int((~dec).sum())
        # ambiguous windows: similarity inside the margin band, or holding a non-decisive key candidate
        W = -(-T // kt) * nwy * nwx
        amb_w = np.abs(o["window_sim"][b] - tau64) <= MARGIN
        for j in np.flatnonzero(amb_tok):
            amb_w[window_of(int(j))] = True
        summary["ambiguous_windows"] += int(amb_w.sum())

        ng, no = int(g["out_count"][b]), int(o["out_count"][b])
        gi, oi = g["out_index"][b, :ng], o["out_index"][b, :no]
        assert np.all(np.diff(gi) > 0), "out_index not strictly ascending"
        if g.get("out_valid") is not None:
            assert g["out_valid"][b].tolist() == [1] * ng + [0] * (M - ng)
        gpos = {int(t): s for s, t in enumerate(gi)}
        opos = {int(t): s for s, t in enumerate(oi)}
        if not amb_w.any():
            assert ng == no and np.array_equal(gi, oi), f"sample {b}: survivor lists differ"
        for tok in range(M):
            if not vb[tok] or amb_w[window_of(tok)]:
                continue
            assert (tok in gpos) == (tok in opos), f"sample {b}: token {tok} survives on one side only"
            if tok not in gpos:
                continue
            sg, so = gpos[tok], opos[tok]
            assert g["out_is_key"][b, sg] == o["out_is_key"][b, so]
            assert abs(g["out_mass"][b, sg] - o["out_mass"][b, so]) <= 1e-5 * abs(o["out_mass"][b, so])
            grow, orow = g["out_x"][b, sg], o["out_x"][b, so]
            gf, of = _f64(grow, x_dtype), _f64(orow, x_dtype)
            if np.array_equal(orow.view(np.uint8), x[b, tok].view(np.uint8)):
                # unmerged token: bit-identical copy
                assert np.array_equal(grow.view(np.uint8), x[b, tok].view(np.uint8)), \
                    f"sample {b}: copied row of token {tok} is not bit-identical"
                summary["copied_rows_checked"] += 1
            else:
                rms = np.sqrt(np.mean(of * of))
                row_rel = np.linalg.norm(gf - of) / max(np.linalg.norm(of), 1e-300)
                assert row_rel <= RTOL, f"merged row {tok}: relative error {row_rel}"
                assert np.max(np.abs(gf - of)) <= RTOL * rms, f"merged row {tok}: element error"
                summary["max_feat_rel"] = max(summary["max_feat_rel"], float(row_rel))
                summary["merged_rows_checked"] += 1
    return summary


# ------------------------------------------------------------------------------------------ stage 2
def check_prefill(g, o, t, Mv, vis_valid, is_key, mode, budget, gamma, alpha, Rcap):
    """t: inputs (k, v, hidden as uint16 arrays)."""
    B = t["k"].shape[0]
    N = t["q_txt"].shape[1]
    summary = {"ambiguous": 0, "max_V_rel": 0.0, "max_I_rel": 0.0}
    g32, a32 = float(np.float32(gamma)), float(np.float32(alpha))
    for b in range(B):
        vb = np.ones(Mv, bool) if vis_valid is None else vis_valid[b].astype(bool)
        kb = np.zeros(Mv, bool) if is_key is None else (is_key[b].astype(bool) & vb)
        Vo, Io = o["score_global"][b], o["score_indiv"][b]
        rv = rel_err(g["score_global"][b][vb], Vo[vb])
        ri = rel_err(g["score_indiv"][b][vb], Io[vb])
        assert np.all(g["score_global"][b][~vb] == 0) and np.all(g["score_indiv"][b][~vb] == 0)
        if vb.any():                                  # (a sample may have no valid vision token at all)
            assert rv.max() <= RTOL and ri.max() <= RTOL, f"sample {b}: score error V {rv.max()} I {ri.max()}"
            summary["max_V_rel"] = max(summary["max_V_rel"], float(rv.max()))
            summary["max_I_rel"] = max(summary["max_I_rel"], float(ri.max()))
        G = Vo[vb].sum()
        cand = np.flatnonzero(vb & ~kb)
        if mode == 0:
            s = np.maximum(Vo[cand] / (g32 * G) if G > 0 else np.zeros(cand.size), Io[cand] / a32)
            dec = _topk_decisive(s, budget - int(kb.sum()))
        else:
            # drop iff V <= gamma*G and I < alpha: a token is decisive when its fate cannot change inside the
            # margin band -- clearly above either threshold (kept whatever the other score does), or clearly
            # below both (dropped)
            tv, ta = g32 * G, a32
            v_hi, v_lo = Vo[cand] > tv + MARGIN * abs(tv), Vo[cand] < tv - MARGIN * abs(tv)
            i_hi, i_lo = Io[cand] > ta + MARGIN * abs(ta), Io[cand] < ta - MARGIN * abs(ta)
            dec = v_hi | i_hi | (v_lo & i_lo)
        summary["ambiguous"] += int((~dec).sum())
        cg, co = int(g["kept_count"][b]), int(o["kept_count"][b])
        if mode == 0 or dec.all():
            assert cg == co, f"sample {b}: kept_count {cg} != {co}"
        ng = min(cg, Rcap)
        gi = g["kept_index"][b, :ng]
        oi = o["kept_index"][b, :min(co, Rcap)]
        assert np.all(np.diff(gi) > 0), "kept_index not ascending"
        gs, os_ = set(gi.tolist()), set(oi.tolist())
        if cg <= Rcap and co <= Rcap:
            assert set(np.flatnonzero(kb).tolist()) <= gs, "a key token was dropped"
            for j, d in zip(cand, dec):
                if d:
                    assert (int(j) in gs) == (int(j) in os_), f"sample {b}: decisive token {j} differs"
        # rows: bit-identical copies of the rows the GPU says it kept, then the text rows
        tl = int(g["out_len"][b]) - ng
        assert tl == int(o["out_len"][b]) - min(co, Rcap)
        rows = np.concatenate([gi, Mv + np.arange(tl)]).astype(np.int64)
        n = rows.size
        assert np.array_equal(g["k_out"][b, :n], t["k"][b, rows]), f"sample {b}: K rows differ"
        assert np.array_equal(g["v_out"][b, :n], t["v"][b, rows]), f"sample {b}: V rows differ"
        assert np.array_equal(g["hidden_out"][b, :n], t["hidden"][b, rows]), f"sample {b}: hidden rows differ"
        kflag = [int(kb[j]) for j in gi] + [1] * tl
        assert g["out_protect"][b, :n].tolist() == kflag
        if dec.all():
            assert np.array_equal(gi, oi)
    return summary


# ------------------------------------------------------------------------------------------ stage 3
def check_decode(g, o, pre, budget):
    """g / o: state after the step (dicts with k, v, acc, ids, protect, len, evicted_ids, evicted_count);
    pre: state before the step (k, v, ids, protect, len) for row-identity checks."""
    B, Lcap = pre["ids"].shape
    summary = {"ambiguous": 0, "max_acc_rel": 0.0}
    for b in range(B):
        n0 = int(pre["len"][b])
        ng, no = int(g["len"][b]), int(o["len"][b])
        assert ng == no, f"sample {b}: len {ng} != {no}"
        src_of = {int(i): s for s, i in enumerate(pre["ids"][b, :n0])}
        acc_o = {int(i): float(a) for i, a in zip(o["ids"][b, :no], o["acc"][b, :no])}
        # the oracle's post-update scores of ALL entries are needed for the margin: survivors from its
        # state, evicted ones are at most the cut by construction -> derive the cut from survivors/evicted
        gid, oid = g["ids"][b, :ng], o["ids"][b, :no]
        assert len(set(gid.tolist())) == ng, "duplicate ids after compaction"
        prot0 = {int(i) for i, p in zip(pre["ids"][b, :n0], pre["protect"][b, :n0]) if p}
        assert prot0 <= set(gid.tolist()), "a protected entry was evicted"
        if "acc_all" in o:                       # oracle's updated scores in pre-compaction slot order
            acc_all = o["acc_all"][b, :n0].astype(np.float64)
            unprot = np.array([s for s in range(n0) if not pre["protect"][b, s]], dtype=np.int64)
            extra = max(min(budget - len(prot0), unprot.size), 0) if n0 > budget else unprot.size
            dec = _topk_decisive(acc_all[unprot], extra)
            summary["ambiguous"] += int((~dec).sum())
            gs, os_ = set(gid.tolist()), set(oid.tolist())
            for s, d in zip(unprot, dec):
                if d:
                    i = int(pre["ids"][b, s])
                    assert (i in gs) == (i in os_), f"sample {b}: decisive entry id {i} differs"
            all_dec = bool(dec.all())
        else:
            all_dec = set(gid.tolist()) == set(oid.tolist())
        # every surviving row is bit-identical to its source row and stays paired with id / protect
        for slot in range(ng):
            i = int(gid[slot])
            s = src_of[i]
            assert np.array_equal(g["k"][b, slot], pre["k"][b, s]), f"sample {b}: K row of id {i} changed"
            assert np.array_equal(g["v"][b, slot], pre["v"][b, s]), f"sample {b}: V row of id {i} changed"
            assert g["protect"][b, slot] == pre["protect"][b, s]
            if i in acc_o:
                r = abs(float(g["acc"][b, slot]) - acc_o[i]) / max(abs(acc_o[i]), 1e-300)
                assert r <= RTOL, f"sample {b}: acc of id {i} off by {r}"
                summary["max_acc_rel"] = max(summary["max_acc_rel"], r)
        if all_dec:
            assert np.array_equal(gid, oid), f"sample {b}: slot layout differs from hole filling"
            if g.get("evicted_count") is not None:
                ne = int(g["evicted_count"][b])
                assert ne == int(o["evicted_count"][b])
                assert np.array_equal(g["evicted_ids"][b, :ne], o["evicted_ids"][b, :ne])
        else:
            # layout must still be a valid hole filling of the GPU's own keep set
            keep = set(gid.tolist())
            kept_slots = [s for s in range(n0) if int(pre["ids"][b, s]) in keep]
            holes = [s for s in range(ng) if int(pre["ids"][b, s]) not in keep]
            movers = [s for s in kept_slots if s >= ng]
            expect = pre["ids"][b, :ng].copy()
            expect[holes] = pre["ids"][b, movers]
            assert np.array_equal(gid, expect), f"sample {b}: layout is not hole filling"
    return summary
