"""The entry points allocate nothing, never synchronise and keep every count on the device, so a
caller can record them into a HIP graph.  The graph is replayed several times with eager work and
synchronisations in between and with new contents in the same input buffers; every replay must give
exactly what an eager call gives on those contents."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def _eq(a, b, names):
    import torch
    for n in names:
        assert torch.equal(a[n], b[n]), f"replay differs from the eager call in {n}"


def test_prefill_filter_in_a_graph():
    import torch
    import paper_2411_10803_amd as md
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[2], B=4)
    base = wl.prefill_inputs(cfg)
    variants = [{k: np.roll(v, i, axis=0) for k, v in base.items()} for i in (1, 2, 3)]   # new contents per replay
    dev = {k: harness.to_dev(v, True) for k, v in base.items()}
    is_key = harness.to_dev(wl.random_key_mask(cfg, cfg.key_budget))
    R, Mv, N = 192, cfg.M, cfg.N
    scale, gamma, alpha = 1.0 / float(np.sqrt(cfg.d)), 1.0 / Mv, 2.0 / (Mv + N)

    def call(out, ws):
        return md.mustdrop_prefill_filter(dev["q_txt"], dev["k"], dev["v"], dev["hidden"], None, None, is_key, Mv, scale,
                                          md.FILTER_BUDGET, R, gamma, alpha, Rcap=R, out=out, workspace=ws)

    out_g = call(None, None)                         # eager warm-up: allocates the outputs and the workspace
    out_e = call(None, None)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(out_g, out_g["workspace"])
    names = ["hidden_out", "k_out", "v_out", "kept_index", "kept_count", "out_len", "out_protect", "out_ids",
             "score_global", "score_indiv"]
    for rep, var in enumerate(variants):
        for k, v in var.items():
            dev[k].copy_(harness.to_dev(v, True))
        for n in names:                              # stale results must not pass for fresh ones
            out_g[n].zero_()
        torch.cuda.synchronize()
        graph.replay()
        call(out_e, out_e["workspace"])              # eager, same stream order, separate buffers
        torch.cuda.synchronize()
        _eq(out_g, out_e, names)
        assert int(out_g["kept_count"].min()) == R


def test_decode_steps_in_a_graph():
    import torch
    import paper_2411_10803_amd as md
    from paper_2411_10803_amd import harness
    cfg = wl.tiny(wl.CONFIGS[5], B=4, L0=300, steps=4, decode_budget=256, n_protect=16)
    t = wl.decode_inputs(cfg)
    Lcap = t["Lcap"]
    B, H, d = cfg.B, cfg.H, cfg.d
    qs, kn, vn = (harness.to_dev(t[n], True) for n in ("q_steps", "k_new", "v_new"))

    def fresh():
        return {"k": harness.to_dev(t["k_cache"], True), "v": harness.to_dev(t["v_cache"], True),
                "acc": torch.zeros((B, Lcap), dtype=torch.float32, device="cuda"),
                "ids": torch.arange(Lcap, dtype=torch.int32, device="cuda").repeat(B, 1).contiguous(),
                "protect": harness.to_dev(t["protect"]).clone(),
                "len": torch.full((B,), cfg.L0, dtype=torch.int32, device="cuda")}

    sg, se = fresh(), fresh()
    q_buf, kn_buf, vn_buf = qs[0].clone(), kn[0].clone(), vn[0].clone()
    ws_g, ws_e = md.decode_workspace(B, Lcap, H), md.decode_workspace(B, Lcap, H)
    scale = 1.0 / float(np.sqrt(d))

    def step(s, q, kx, vx, ws, new_id):
        md.mustdrop_decode_append(kx, vx, s["k"], s["v"], s["acc"], s["ids"], s["protect"], s["len"], new_id, 1)
        md.mustdrop_decode_evict(q, s["k"], s["v"], s["acc"], s["ids"], s["protect"], s["len"], scale, 1.0,
                                 cfg.decode_budget, workspace=ws)

    # eager warm-up on scratch states, then one append + evict step recorded on the graph's state
    step(fresh(), q_buf, kn_buf, vn_buf, ws_g, 10_000)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(sg, q_buf, kn_buf, vn_buf, ws_g, 10_000)
    # the capture itself executes nothing: sg is still the initial state
    for s in range(1, cfg.steps):
        q_buf.copy_(qs[s]); kn_buf.copy_(kn[s]); vn_buf.copy_(vn[s])
        torch.cuda.synchronize()
        graph.replay()
        step(se, qs[s], kn[s], vn[s], ws_e, 10_000)
        torch.cuda.synchronize()
        n = int(se["len"][0])
        assert torch.equal(sg["len"], se["len"]) and n == cfg.decode_budget
        for name in ("k", "v", "acc", "ids", "protect"):
            assert torch.equal(sg[name][:, :n], se[name][:, :n]), f"step {s}: {name} differs"
