"""Figures the paper prints, against the geometry and the budget rule this build uses.

Table 3 prints the KV-cache memory that goes with 576 / 440 / 64 / 45 vision tokens; those numbers fix
the size of one cached token (32 layers, K and V, 32 heads x 128, 16 bits), which is the row size the
prefill compaction and the decode stage move.  Table 1 prints the retained-token settings that the
benchmark workloads take as budgets."""
import os

import numpy as np

import oracle
import workloads as wl
from oracle import FILTER_BUDGET

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
LLAVA_7B_LAYERS = 32


def rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


def test_table3_kv_cache_memory_fixes_the_bytes_per_cached_token():
    cfg = wl.CONFIGS[2]
    per_layer = 2 * cfg.H * cfg.d * 2                      # K row + V row of one token, bf16
    assert per_layer == 16 * 1024                          # what decode_move / prefill_compact copy per token
    per_token_mb = per_layer * LLAVA_7B_LAYERS / 1e6
    table = rows("table3_kv_cache.txt")
    base_tokens = int(table[0][1])
    assert base_tokens == cfg.M == 576
    for stage, tokens, mb, red in table:
        tokens, mb = int(tokens), float(mb)
        assert abs(tokens * per_token_mb - mb) <= 0.003 * mb + 0.05, (stage, tokens * per_token_mb, mb)
        if red != "-":
            assert abs(100.0 * (1 - tokens / base_tokens) - float(red)) <= 0.06, stage


def test_table1_budgets_are_the_benchmark_budgets_and_the_budget_rule_keeps_exactly_that_many():
    table = rows("table1_budgets.txt")
    for model, full, kept, red in table:
        assert abs(100.0 * (1 - int(kept) / int(full)) - float(red)) <= 0.06
    assert [int(r[2]) for r in table if r[0] == "llava-1.5-7b"] == list(wl.CONFIGS[2].budgets)
    assert int(table[3][1]) == wl.CONFIGS[3].M and int(table[3][2]) == wl.CONFIGS[3].budgets[0]
    # the budget form of Eq. 9-10 on the 576-token grid (small heads to stay fast): exactly R vision tokens stay
    cfg = wl.tiny(wl.CONFIGS[2], B=1, N=8, H=1, d=64, C=8)
    t = wl.prefill_inputs(cfg)
    for R in cfg.budgets:
        o = oracle.prefill_filter(t["q_txt"], t["k"], t["v"], t["hidden"], None, None, None, cfg.M,
                                  1.0 / np.sqrt(cfg.d), FILTER_BUDGET, R, 1.0 / cfg.M, 2.0 / cfg.L, R)
        assert int(o["kept_count"][0]) == R and int(o["out_len"][0]) == R + cfg.N
