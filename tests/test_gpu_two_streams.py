"""Calls that do not share a workspace may overlap in time: two three-stage chains on different inputs, issued to
two HIP streams so that their kernels interleave on the device, must give exactly what each chain gives when it
runs alone.  (Every stage is deterministic, so "exactly" means bit for bit.)"""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


class _Chain:
    """encode_merge -> prefill_filter -> decode_evict on one batch, with its own outputs, state and workspaces."""

    def __init__(self, cfg, shift):
        import torch
        import paper_2411_10803_amd as md
        from paper_2411_10803_amd import harness
        self.md, self.cfg = md, cfg
        roll = lambda a: np.ascontiguousarray(np.roll(a, shift, axis=0))      # the second chain sees other data
        e, p = wl.encode_inputs(cfg), wl.prefill_inputs(cfg)
        self.x, self.q_cls, self.k_cls = (harness.to_dev(roll(e[n]), True) for n in ("x", "q_cls", "k_cls"))
        self.q_txt, self.k, self.v, self.hidden = (harness.to_dev(roll(p[n]), True) for n in ("q_txt", "k", "v", "hidden"))
        rng = np.random.default_rng([cfg.seed, 77, shift])
        self.q_dec = harness.to_dev(wl.f32_to_bf16_bits(rng.standard_normal((cfg.B, cfg.H, cfg.d)).astype(np.float32)), True)
        self.R = cfg.budgets[0]
        self.enc, self.pre = None, None
        self.acc = torch.zeros((cfg.B, self.R + cfg.N), dtype=torch.float32, device="cuda")
        self.dec_ws = md.decode_workspace(cfg.B, self.R + cfg.N, cfg.H)

    def step(self):
        md, c = self.md, self.cfg
        self.enc = md.mustdrop_encode_merge(self.x, self.q_cls, self.k_cls, None, None, c.T, c.Hg, c.Wg, c.kt, c.kh, c.kw,
                                            0.955, c.key_budget, out=self.enc, workspace=(self.enc or {}).get("workspace"))
        self.pre = md.mustdrop_prefill_filter(self.q_txt, self.k, self.v, self.hidden, self.enc["out_valid"], None,
                                              self.enc["out_is_key"], c.M, 1.0 / float(np.sqrt(c.d)), md.FILTER_BUDGET,
                                              self.R, 1.0 / c.M, 2.0 / (c.M + c.N), Rcap=self.R, out=self.pre,
                                              workspace=(self.pre or {}).get("workspace"))
        o = self.pre
        md.mustdrop_decode_evict(self.q_dec, o["k_out"], o["v_out"], self.acc, o["out_ids"], o["out_protect"], o["out_len"],
                                 1.0 / float(np.sqrt(c.d)), 0.0, self.R * 2 // 3 + c.N, workspace=self.dec_ws)

    def snapshot(self):
        names_e = ("out_x", "out_index", "out_mass", "out_is_key", "out_valid", "out_count", "key_index")
        names_p = ("hidden_out", "k_out", "v_out", "kept_index", "kept_count", "out_len", "out_protect", "out_ids")
        snap = {"enc." + n: self.enc[n].clone() for n in names_e}
        snap.update({"pre." + n: self.pre[n].clone() for n in names_p})
        snap["acc"] = self.acc.clone()
        return snap


@pytest.mark.parametrize("number", [2, 3])
def test_two_chains_on_two_streams_match_the_chains_run_alone(number):
    import torch
    cfg = wl.tiny(wl.CONFIGS[number], B=4)
    chains = [_Chain(cfg, 0), _Chain(cfg, 1)]
    def clear(ch):                                    # stale results must not pass for fresh ones; the parts of the
        for d in (ch.enc, ch.pre):                    # outputs that a call leaves untouched read zero in every run
            for n, t in d.items():
                if n != "workspace" and t is not None:
                    t.zero_()
        ch.acc.zero_()

    alone = []
    for ch in chains:                                 # each chain alone, on the default stream
        ch.step()                                     # (the first call allocates the outputs and workspaces)
        clear(ch)
        ch.step()
        torch.cuda.synchronize()
        alone.append(ch.snapshot())
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    main = torch.cuda.current_stream()
    for rep in range(6):
        for ch in chains:
            clear(ch)
        for st in streams:
            st.wait_stream(main)
        for ch, st in zip(chains if rep % 2 == 0 else chains[::-1], streams):
            with torch.cuda.stream(st):
                ch.step()
        for st in streams:
            main.wait_stream(st)
        torch.cuda.synchronize()
        for ch, ref in zip(chains, alone):
            got = ch.snapshot()
            for n in ref:
                assert torch.equal(got[n], ref[n]), f"chain result differs in {n} when another chain runs beside it (round {rep})"
