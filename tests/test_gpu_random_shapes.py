"""GPU parity on randomly drawn shapes and options: every stage, HIP (through the C ABI) against the
oracle, with the comparison rules of parity.py.  Shapes cover ragged tiles, odd head counts, both
dtypes of the vision features, padding masks, masses, key sets, both filter modes, long prompts and
caches longer than one selection round."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import FILTER_BUDGET, FILTER_THRESHOLD
from parity import check_decode, check_encode, check_prefill
from test_gpu_decode import gpu_step, initial_state, oracle_step
from test_gpu_encode import both

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed,n_iter,big", [(101, 10, 1), (102, 10, 1), (103, 6, 3)])
def test_random_shapes(seed, n_iter, big):
    from paper_2411_10803_amd import harness
    rng = np.random.default_rng(seed)
    for it in range(n_iter):
        # ---- encode
        kt, kh, kw = [(1,1,1),(1,1,2),(1,2,2),(2,2,2),(1,3,3),(1,4,4),(2,2,4),(1,2,1)][rng.integers(8)]
        T, Hg, Wg = int(kt * rng.integers(1, 4)), int(kh * rng.integers(1, big * 9)), int(kw * rng.integers(1, big * 9))
        if rng.random() < 0.4:                           # a grid that the window does not divide
            T, Hg, Wg = T + int(rng.integers(0, kt)), Hg + int(rng.integers(0, kh)), Wg + int(rng.integers(0, kw))
        dc = [8, 16, 32, 64][rng.integers(4)]; Hc = int(rng.integers(1, 17)); D = Hc * dc
        bf = bool(rng.integers(2))
        B = int(rng.integers(1, 5))
        M = T * Hg * Wg
        cfg = wl.tiny(wl.CONFIGS[2], B=B, T=T, Hg=Hg, Wg=Wg, D=D, Hc=Hc, dc=dc, kt=kt, kh=kh, kw=kw,
                      x_dtype=wl.BF16 if bf else wl.F32, key_budget=int(rng.integers(0, M + 1)))
        e = wl.encode_inputs(cfg)
        valid = (rng.random((B, M)) > 0.15).astype(np.uint8) if rng.integers(2) else None
        mass = rng.integers(1, 5, size=(B, M)).astype(np.float32) if rng.integers(2) else None
        o0 = oracle.encode_merge(e["x"], cfg.x_dtype, None, None, cfg.x_dtype, None, valid, T, Hg, Wg, kt, kh, kw, 2.0, 0)
        tau = float(np.median(o0["window_sim"]))
        kb = cfg.key_budget
        q, k = (e["q_cls"], e["k_cls"]) if kb > 0 else (None, None)
        print(f"[{seed}:{it}] encode B={B} grid={T}x{Hg}x{Wg} win={kt}x{kh}x{kw} D={D} Hc={Hc} bf16={bf} kb={kb} valid={valid is not None} mass={mass is not None}", flush=True)
        g, o = both(e["x"], cfg.x_dtype, q, k, cfg.x_dtype, mass, valid, T, Hg, Wg, kt, kh, kw, tau, kb)
        check_encode(g, o, e["x"], cfg.x_dtype, valid, T, Hg, Wg, kt, kh, kw, tau, kb)
        # ---- prefill
        Hg2, Wg2 = int(rng.integers(1, 20 * big)), int(rng.integers(1, 20 * big))
        N = int(rng.integers(1, 129)) if rng.integers(4) else int(rng.integers(129, 500)); H = int(rng.integers(1, 9)); d = [64, 128][rng.integers(2)]; C = 8 * int(rng.integers(1, 40))
        B = int(rng.integers(1, 4))
        cfg = wl.tiny(wl.CONFIGS[2], B=B, T=1, Hg=Hg2, Wg=Wg2, N=N, H=H, d=d, C=C)
        Mv = cfg.M
        t = wl.prefill_inputs(cfg)
        vis = (rng.random((B, Mv)) > 0.25).astype(np.uint8) if rng.integers(2) else None
        txt_len = rng.integers(1, N + 1, size=B).astype(np.int32) if rng.integers(2) else None
        is_key = wl.random_key_mask(cfg, int(rng.integers(0, max(Mv // 4, 1) + 1)), valid=vis) if rng.integers(2) else None
        mode = FILTER_BUDGET if rng.integers(3) else FILTER_THRESHOLD
        R = int(rng.integers(0, Mv + 1))
        Rcap = max(R, 1) if mode == FILTER_BUDGET else Mv
        if is_key is not None and mode == FILTER_BUDGET:
            Rcap = max(Rcap, int(is_key.sum(1).max()), 1)
        gamma, alpha = 1.0 / Mv, (2.0 if mode == FILTER_BUDGET else 1.2) / (Mv + N)
        scale = 1.0 / np.sqrt(d)
        print(f"[{seed}:{it}] prefill B={B} Mv={Mv} N={N} H={H} d={d} C={C} mode={mode} R={R} Rcap={Rcap} vis={vis is not None} txt={txt_len is not None} key={is_key is not None}", flush=True)
        g = harness.prefill_on_gpu(t, Mv, vis, txt_len, is_key, scale, mode, R, gamma, alpha, Rcap)
        o = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], vis, txt_len, is_key, Mv, scale, mode, R, gamma, alpha, Rcap)
        check_prefill(g, o, t, Mv, vis, is_key, mode, R, gamma, alpha, Rcap)
        # ---- decode
        H = [4, 8, 16, 32, 5, 40, 12][rng.integers(7)]; d = [64, 128][rng.integers(2)]
        L0 = int(rng.integers(2, 1500 * big * big)); budget = int(rng.integers(1, L0 + 50)); B = int(rng.integers(1, 4))
        cfg = wl.tiny(wl.CONFIGS[5], B=B, L0=L0, steps=2, decode_budget=budget, n_protect=int(rng.integers(0, min(L0, budget) + 1)), H=H, d=d)
        t = wl.decode_inputs(cfg)
        s = initial_state(t)
        print(f"[{seed}:{it}] decode B={B} L0={L0} budget={budget} H={H} d={d} nprot={cfg.n_protect}", flush=True)
        g = gpu_step(s, t["q_steps"][0], 1 / np.sqrt(d), 0.7, budget)
        o = oracle_step(s, t["q_steps"][0], 1 / np.sqrt(d), 0.7, budget)
        check_decode(g, o, s, budget)
