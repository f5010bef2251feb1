"""GPU parity: progressive prefill (Sec. 3.4: the filter is applied again in later layers).

Three chained calls of mustdrop_prefill_filter with budgets 192 -> 128 -> 64: each call works on the
compacted hidden / K / V rows of the previous one, with that call's protect flags as key set.  The HIP
chain and the oracle chain each run from their own outputs; they are compared call by call."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import FILTER_BUDGET
from parity import check_prefill

pytestmark = pytest.mark.gpu


def chain(run_call, cfg, t0, is_key0, budgets, samples):
    """run_call(t, Mv, vis_valid, is_key, R) -> outputs (host arrays).  Returns the per-call (inputs, outputs)."""
    t, Mv, vis, key = t0, cfg.M, None, is_key0
    calls = []
    for layer, R in enumerate(budgets):
        q = t0["q_txt"] if layer == 0 else wl.layer_text_queries(cfg, layer, samples)
        tin = {"q_txt": q, "k": t["k"], "v": t["v"], "hidden": t["hidden"]}
        out = run_call(tin, Mv, vis, key, R)
        calls.append((tin, Mv, vis, key, R, out))
        kept = np.minimum(out["kept_count"], R)
        vis = (np.arange(R)[None, :] < kept[:, None]).astype(np.uint8)
        key = out["out_protect"][:, :R].copy()
        t = {"k": out["k_out"], "v": out["v_out"], "hidden": out["hidden_out"]}
        Mv = R
    return calls


@pytest.mark.parametrize("budgets", [(192, 128, 64), (100, 37, 36)])
def test_three_chained_calls(budgets):
    from paper_2411_10803_amd import harness
    samples = [0, 7]
    cfg = wl.CONFIGS[2]
    t0 = wl.prefill_inputs(cfg, samples=samples)
    is_key0 = wl.random_key_mask(cfg, cfg.key_budget)[samples]
    N, d = cfg.N, cfg.d
    scale = 1.0 / np.sqrt(d)

    def params(Mv):
        return 1.0 / Mv, 2.0 / (Mv + N)

    def gpu_call(t, Mv, vis, key, R):
        g, a = params(Mv)
        return harness.prefill_on_gpu(t, Mv, vis, None, key, scale, FILTER_BUDGET, R, g, a, R)

    def ref_call(t, Mv, vis, key, R):
        g, a = params(Mv)
        return oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], vis, None, key, Mv, scale, FILTER_BUDGET,
                                     R, g, a, R)

    gc = chain(gpu_call, cfg, t0, is_key0, budgets, samples)
    oc = chain(ref_call, cfg, t0, is_key0, budgets, samples)
    for layer, ((tg, Mv, vis, key, R, g), (to, _, viso, keyo, _, o)) in enumerate(zip(gc, oc)):
        # the two chains see identical inputs as long as every earlier call kept the same rows
        for name in ("q_txt", "k", "v", "hidden"):
            assert np.array_equal(tg[name], to[name]), f"call {layer}: the chains' {name} inputs differ"
        assert (vis is None and viso is None) or np.array_equal(vis, viso)
        assert np.array_equal(key, keyo)
        gm, al = params(Mv)
        check_prefill(g, o, tg, Mv, vis, key, FILTER_BUDGET, R, gm, al, R)
        assert np.array_equal(g["kept_index"], o["kept_index"]), f"call {layer}: kept sets differ"
        assert np.all(g["kept_count"] == R)
        # key tokens of the first call survive every later call (Sec. 3.3: the key set is never dropped)
    first_keys = [set(np.flatnonzero(is_key0[b]).tolist()) for b in range(len(samples))]
    ids = gc[0][5]["out_ids"]
    for layer in range(1, len(budgets)):
        kept = gc[layer][5]["kept_index"]
        ids = np.take_along_axis(ids, np.maximum(kept, 0), axis=1)       # original positions of the survivors
    for b in range(len(samples)):
        assert first_keys[b] <= set(ids[b].tolist())
