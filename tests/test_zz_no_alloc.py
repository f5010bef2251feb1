"""GPU check of mustdrop_encode_merge_noalloc (the entry point on the library's static scratch buffer,
for callers that cannot allocate): its outputs against mustdrop_encode_merge's, on two calls in a row, the
second on a smaller input, so that what the first call left in the shared buffer must not matter."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

NAMES = ("out_index", "out_mass", "out_is_key", "out_valid", "out_count", "key_index", "a_cls", "window_sim")


def fresh_outputs(torch, x, key_budget, W):
    B, M, _ = x.shape
    z = lambda shape, dt, fill=0: torch.full(shape, fill, dtype=dt, device="cuda")
    return {"out_x": torch.zeros_like(x), "out_index": z((B, M), torch.int32, -1), "out_mass": z((B, M), torch.float32),
            "out_is_key": z((B, M), torch.uint8), "out_valid": z((B, M), torch.uint8), "out_count": z((B,), torch.int32),
            "key_index": z((B, max(key_budget, 1)), torch.int32, -1), "a_cls": z((B, M), torch.float32),
            "window_sim": z((B, W), torch.float32)}


def run_pair(cfg, tau, valid=None):
    import torch
    import paper_2411_10803_amd as md
    from paper_2411_10803_amd import harness
    e = wl.encode_inputs(cfg)
    bf = cfg.x_dtype == wl.BF16
    x, q, k = (harness.to_dev(e[n], bf) for n in ("x", "q_cls", "k_cls"))
    vd = harness.to_dev(valid)
    W = -(-cfg.T // cfg.kt) * -(-cfg.Hg // cfg.kh) * -(-cfg.Wg // cfg.kw)
    args = (cfg.T, cfg.Hg, cfg.Wg, cfg.kt, cfg.kh, cfg.kw, tau, cfg.key_budget)
    ref = md.mustdrop_encode_merge(x, q, k, None, vd, *args, out=fresh_outputs(torch, x, cfg.key_budget, W))
    got = md.mustdrop_encode_merge_noalloc(x, q, k, None, vd, *args, out=fresh_outputs(torch, x, cfg.key_budget, W))
    torch.cuda.synchronize()
    r, g = harness.outputs_to_host(ref), harness.outputs_to_host(got)
    # the two entry points run the same kernels in the same order: integer outputs and scores are bit-identical
    for name in NAMES:
        assert np.array_equal(r[name], g[name]), name
    for b in range(cfg.B):
        n = int(r["out_count"][b])
        assert np.array_equal(r["out_x"][b, :n], g["out_x"][b, :n])
    assert r["out_count"].sum() > 0
    return r


def test_noalloc_matches_the_workspace_entry_point_twice_the_second_call_smaller():
    big = wl.CONFIGS[2]                                          # 16 x 576 tokens, bf16, 32 keys
    r1 = run_pair(big, 0.955)
    assert np.all(r1["out_count"] < big.M) or np.any(r1["out_count"] < big.M)
    small = wl.tiny(wl.CONFIGS[2], B=3, Hg=10, Wg=14, D=128, Hc=8, dc=16, x_dtype=wl.F32, key_budget=5)
    valid = (np.random.default_rng(3).random((small.B, small.M)) > 0.15).astype(np.uint8)
    run_pair(small, 0.5, valid)


def test_noalloc_rejects_a_shape_beyond_its_buffer():
    import torch
    import paper_2411_10803_amd as md
    x = torch.zeros((200, 4608, 8), dtype=torch.float32, device="cuda")
    out = fresh_outputs(torch, x, 0, 64)
    with pytest.raises(md.MustDropError) as err:
        md.mustdrop_encode_merge_noalloc(x, None, None, None, None, 8, 24, 24, 1, 2, 2, 0.9, 0, out=out)
    assert err.value.code == 5
