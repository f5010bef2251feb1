"""CPU oracle for the MustDrop token-reduction path -- TEST INFRASTRUCTURE ONLY.

``mustdrop_ref.c`` is the oracle; this file only compiles it with gcc and
marshals numpy arrays into it.  Nothing here is imported by the product
package; only the tests, the smoke check and the benchmark's cpu_baseline leg
may use it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mustdrop_ref.c")
_LIB = os.path.join(_HERE, "libmustdrop_ref.so")

F32, BF16 = 0, 1
FILTER_BUDGET, FILTER_THRESHOLD = 0, 1

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle (plain C, no HIP, -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_LIB)
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"], "oracle inputs must be contiguous"
    return a.ctypes.data_as(C.c_void_p)


def _stored_dtype(code: int):
    return np.uint16 if code == BF16 else np.float32


def encode_merge(x, x_dtype, q_cls, k_cls, qk_dtype, mass_in, valid,
                 T, Hg, Wg, kt, kh, kw, tau, key_budget) -> Dict[str, np.ndarray]:
    """Sec. 3.3 (Eq. 5-7).  x [B, M, D]; q_cls [B, Hc, dc]; k_cls [B, 1+M, Hc, dc]."""
    B, M, D = x.shape
    assert M == T * Hg * Wg
    if key_budget > 0:
        Hc, dc = q_cls.shape[1], q_cls.shape[2]
    else:
        Hc, dc = 1, D
    W = -(-T // kt) * -(-Hg // kh) * -(-Wg // kw)        # border windows are clipped to the grid
    out = {
        "out_x": np.zeros((B, M, D), dtype=_stored_dtype(x_dtype)),
        "out_index": np.full((B, M), -1, dtype=np.int32),
        "out_mass": np.zeros((B, M), dtype=np.float32),
        "out_is_key": np.zeros((B, M), dtype=np.uint8),
        "out_valid": np.zeros((B, M), dtype=np.uint8),
        "out_count": np.zeros((B,), dtype=np.int32),
        "key_index": np.full((B, max(key_budget, 1)), -1, dtype=np.int32),
        "a_cls": np.zeros((B, M), dtype=np.float64),
        "window_sim": np.zeros((B, W), dtype=np.float64),
    }
    rc = lib().mustdrop_encode_merge_ref(
        _p(x), C.c_int(x_dtype), _p(q_cls), _p(k_cls), C.c_int(qk_dtype), _p(mass_in), _p(valid),
        C.c_int(B), C.c_int(T), C.c_int(Hg), C.c_int(Wg), C.c_int(D), C.c_int(Hc), C.c_int(dc),
        C.c_int(kt), C.c_int(kh), C.c_int(kw), C.c_float(tau), C.c_int(key_budget),
        _p(out["out_x"]), _p(out["out_index"]), _p(out["out_mass"]), _p(out["out_is_key"]),
        _p(out["out_valid"]), _p(out["out_count"]), _p(out["key_index"]),
        _p(out["a_cls"]), _p(out["window_sim"]))
    if rc != 0:
        raise ValueError(f"mustdrop_encode_merge_ref: error {rc}")
    if key_budget == 0:
        out["key_index"] = np.zeros((B, 0), dtype=np.int32)
    return out


def encode_merge_adaptive(x, x_dtype, q_cls, k_cls, qk_dtype, mass_in, valid,
                          T, Hg, Wg, kt, kh, kw, tau, key_lambda, key_cap) -> Dict[str, np.ndarray]:
    """Sec. 3.3 with Eq. 7 as printed: O = {a_cls > mu}, mu = mean + key_lambda * std of a_cls over the valid
    tokens.  key_index holds the first key_cap keys (ascending), key_count the size of O."""
    B, M, D = x.shape
    assert M == T * Hg * Wg
    Hc, dc = q_cls.shape[1], q_cls.shape[2]
    W = -(-T // kt) * -(-Hg // kh) * -(-Wg // kw)        # border windows are clipped to the grid
    out = {
        "out_x": np.zeros((B, M, D), dtype=_stored_dtype(x_dtype)),
        "out_index": np.full((B, M), -1, dtype=np.int32),
        "out_mass": np.zeros((B, M), dtype=np.float32),
        "out_is_key": np.zeros((B, M), dtype=np.uint8),
        "out_valid": np.zeros((B, M), dtype=np.uint8),
        "out_count": np.zeros((B,), dtype=np.int32),
        "key_index": np.full((B, max(key_cap, 1)), -1, dtype=np.int32),
        "key_count": np.zeros((B,), dtype=np.int32),
        "a_cls": np.zeros((B, M), dtype=np.float64),
        "window_sim": np.zeros((B, W), dtype=np.float64),
    }
    rc = lib().mustdrop_encode_merge_adaptive_ref(
        _p(x), C.c_int(x_dtype), _p(q_cls), _p(k_cls), C.c_int(qk_dtype), _p(mass_in), _p(valid),
        C.c_int(B), C.c_int(T), C.c_int(Hg), C.c_int(Wg), C.c_int(D), C.c_int(Hc), C.c_int(dc),
        C.c_int(kt), C.c_int(kh), C.c_int(kw), C.c_float(tau), C.c_float(key_lambda), C.c_int(key_cap),
        _p(out["out_x"]), _p(out["out_index"]), _p(out["out_mass"]), _p(out["out_is_key"]),
        _p(out["out_valid"]), _p(out["out_count"]), _p(out["key_index"]), _p(out["key_count"]),
        _p(out["a_cls"]), _p(out["window_sim"]))
    if rc != 0:
        raise ValueError(f"mustdrop_encode_merge_adaptive_ref: error {rc}")
    if key_cap == 0:
        out["key_index"] = np.zeros((B, 0), dtype=np.int32)
    return out


def prefill_filter(q_txt, k, v, hidden, vis_valid, txt_len, is_key, Mv, softmax_scale, mode, budget,
                   gamma, alpha, Rcap=None) -> Dict[str, np.ndarray]:
    """Sec. 3.4 (Eq. 8-10) + token drop.  q_txt [B,N,H,d]; k, v [B,L,H,d]; hidden [B,L,C] (bf16 bits)."""
    B, N, H, d = q_txt.shape
    L = k.shape[1]
    assert L == Mv + N
    Cdim = hidden.shape[2]
    if Rcap is None:
        Rcap = budget if mode == FILTER_BUDGET else Mv
    out = {
        "hidden_out": np.zeros((B, Rcap + N, Cdim), dtype=np.uint16),
        "k_out": np.zeros((B, Rcap + N, H, d), dtype=np.uint16),
        "v_out": np.zeros((B, Rcap + N, H, d), dtype=np.uint16),
        "kept_index": np.full((B, Rcap), -1, dtype=np.int32),
        "kept_count": np.zeros((B,), dtype=np.int32),
        "out_len": np.zeros((B,), dtype=np.int32),
        "out_protect": np.zeros((B, Rcap + N), dtype=np.uint8),
        "out_ids": np.full((B, Rcap + N), -1, dtype=np.int32),
        "score_global": np.zeros((B, Mv), dtype=np.float64),
        "score_indiv": np.zeros((B, Mv), dtype=np.float64),
        "row_lse": np.zeros((B, H, N), dtype=np.float64),
    }
    rc = lib().mustdrop_prefill_filter_ref(
        _p(q_txt), _p(k), _p(v), _p(hidden), _p(vis_valid), _p(txt_len), _p(is_key),
        C.c_int(B), C.c_int(Mv), C.c_int(N), C.c_int(H), C.c_int(d), C.c_int(Cdim),
        C.c_float(softmax_scale), C.c_int(mode), C.c_int(budget), C.c_float(gamma), C.c_float(alpha),
        C.c_int(Rcap),
        _p(out["hidden_out"]), _p(out["k_out"]), _p(out["v_out"]),
        _p(out["kept_index"]), _p(out["kept_count"]), _p(out["out_len"]), _p(out["out_protect"]), _p(out["out_ids"]),
        _p(out["score_global"]), _p(out["score_indiv"]), _p(out["row_lse"]))
    if rc != 0:
        raise ValueError(f"mustdrop_prefill_filter_ref: error {rc}")
    return out


def decode_evict(q, k_cache, v_cache, acc, ids, protect, length, softmax_scale, decay, budget):
    """Sec. 3.5, one decode step.  State arrays are updated IN PLACE.
    q [B,H,d]; k_cache, v_cache [B,Lcap,H,d] (bf16 bits); acc f32, ids i32, protect u8 [B,Lcap]; length i32 [B]."""
    B, Lcap, H, d = k_cache.shape
    out = {
        "evicted_ids": np.full((B, Lcap), -1, dtype=np.int32),
        "evicted_count": np.zeros((B,), dtype=np.int32),
        "a_t": np.zeros((B, Lcap), dtype=np.float64),
    }
    rc = lib().mustdrop_decode_evict_ref(
        _p(q), _p(k_cache), _p(v_cache), _p(acc), _p(ids), _p(protect), _p(length),
        C.c_int(B), C.c_int(Lcap), C.c_int(H), C.c_int(d),
        C.c_float(softmax_scale), C.c_float(decay), C.c_int(budget),
        _p(out["evicted_ids"]), _p(out["evicted_count"]), _p(out["a_t"]))
    if rc != 0:
        raise ValueError(f"mustdrop_decode_evict_ref: error {rc}")
    return out


def decode_keep(k_caches, v_caches, keep, acc, ids, protect, length):
    """Sec. 3.5, the static policy: only the entries flagged in ``keep`` stay in the caches of all layers.
    State arrays are updated IN PLACE.  k_caches, v_caches [n_layers,B,Lcap,H,d] (bf16 bits); keep u8, ids i32,
    protect u8 [B,Lcap]; acc f32 [B,Lcap] or None; length i32 [B]."""
    n_layers, B, Lcap, H, d = k_caches.shape
    out = {
        "evicted_ids": np.full((B, Lcap), -1, dtype=np.int32),
        "evicted_count": np.zeros((B,), dtype=np.int32),
    }
    rc = lib().mustdrop_decode_keep_ref(
        _p(k_caches), _p(v_caches), _p(keep), _p(acc), _p(ids), _p(protect), _p(length),
        C.c_int(n_layers), C.c_int(B), C.c_int(Lcap), C.c_int(H), C.c_int(d),
        _p(out["evicted_ids"]), _p(out["evicted_count"]))
    if rc != 0:
        raise ValueError(f"mustdrop_decode_keep_ref: error {rc}")
    return out
