"""ctypes binding of libmustdrop.so: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

F32, BF16 = 0, 1
FILTER_BUDGET, FILTER_THRESHOLD = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
# MUSTDROP_LIBRARY selects another build of the same ABI (e.g. one compiled with different tile parameters)
_LIB_PATH = os.environ.get("MUSTDROP_LIBRARY") or os.path.join(_HERE, "libmustdrop.so")
_lib = None

EXPORTS = [
    "mustdrop_last_error", "mustdrop_version",
    "mustdrop_encode_merge_workspace_bytes", "mustdrop_encode_merge", "mustdrop_encode_merge_adaptive",
    "mustdrop_encode_merge_noalloc",
    "mustdrop_prefill_filter_workspace_bytes", "mustdrop_prefill_filter",
    "mustdrop_decode_evict_workspace_bytes", "mustdrop_decode_evict", "mustdrop_decode_append", "mustdrop_decode_keep",
    "mustdrop_prefill_filter_strided", "mustdrop_decode_evict_strided", "mustdrop_decode_append_strided",
    "mustdrop_decode_keep_strided",
    "mustdrop_profile_start", "mustdrop_profile_stop",
]


class KvLayout(C.Structure):
    """md_kv_layout: element strides of the batch, token and head axes."""
    _fields_ = [("batch", C.c_int64), ("token", C.c_int64), ("head", C.c_int64)]


class MustDropError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"mustdrop error {code}: {message}")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def library() -> C.CDLL:
    """Loads the HIP library built in-tree (python -m paper_2411_10803_amd.build).  No fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2411_10803_amd.build` "
                              "(there is no CPU fallback)")
        lib = C.CDLL(_LIB_PATH)
        lib.mustdrop_last_error.restype = C.c_char_p
        lib.mustdrop_version.restype = C.c_int
        for n in ("mustdrop_encode_merge_workspace_bytes", "mustdrop_prefill_filter_workspace_bytes",
                  "mustdrop_decode_evict_workspace_bytes"):
            getattr(lib, n).restype = C.c_size_t
        for n in ("mustdrop_encode_merge", "mustdrop_encode_merge_adaptive", "mustdrop_encode_merge_noalloc", "mustdrop_prefill_filter", "mustdrop_decode_evict", "mustdrop_decode_append",
                  "mustdrop_decode_keep", "mustdrop_prefill_filter_strided", "mustdrop_decode_evict_strided",
                  "mustdrop_decode_append_strided", "mustdrop_decode_keep_strided"):
            getattr(lib, n).restype = C.c_int
        _lib = lib
    return _lib


def _check(rc: int):
    if rc != 0:
        raise MustDropError(rc, library().mustdrop_last_error().decode())


def _ptr(t) -> C.c_void_p:
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return C.c_void_p(0)
    if isinstance(t, int):
        return C.c_void_p(t)
    assert t.is_contiguous(), "tensors handed to the C ABI must be contiguous"
    return C.c_void_p(t.data_ptr())


def _view_ptr(t) -> C.c_void_p:
    """Device pointer of a [.., tokens, H, d] view whose last axis is contiguous (any other strides)."""
    assert t.stride(-1) == 1, "the head dimension must be contiguous"
    return C.c_void_p(t.data_ptr())


def _layout(t):
    """md_kv_layout of a [B, tokens, H, d] view (the last three axes of a [layers, B, tokens, H, d] one)."""
    st = t.stride()
    return KvLayout(st[-4], st[-3], st[-2])


def _stream(stream=None) -> C.c_void_p:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _workspace(nbytes: int, device):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def encode_workspace(B, T, Hg, Wg, Hc, kt, kh, kw, device="cuda"):
    n = library().mustdrop_encode_merge_workspace_bytes(B, T, Hg, Wg, Hc, kt, kh, kw)
    return _workspace(n, device)


def prefill_workspace(B, Mv, N, H, Rcap, device="cuda"):
    n = library().mustdrop_prefill_filter_workspace_bytes(B, Mv, N, H, Rcap)
    return _workspace(n, device)


def decode_workspace(B, Lcap, H, device="cuda"):
    n = library().mustdrop_decode_evict_workspace_bytes(B, Lcap, H)
    return _workspace(n, device)


def mustdrop_encode_merge(x, q_cls, k_cls, mass_in, valid, T, Hg, Wg, kt, kh, kw, tau, key_budget,
                          out: Optional[Dict] = None, workspace=None, stream=None, want_scores=True) -> Dict:
    """Sec. 3.3.  x [B, M, D] (f32 / bf16); q_cls [B, Hc, dc]; k_cls [B, 1+M, Hc, dc]; returns the output tensors."""
    import torch
    B, M, D = x.shape
    dev = x.device
    if key_budget > 0:
        Hc, dc = q_cls.shape[1], q_cls.shape[2]
        qk_dtype = _dtype_code(q_cls)
    else:
        Hc, dc, qk_dtype = 1, D, _dtype_code(x)
    W = -(-T // kt) * -(-Hg // kh) * -(-Wg // kw)          # border windows are clipped to the grid
    if out is None:
        out = {
            "out_x": torch.zeros_like(x),
            "out_index": torch.full((B, M), -1, dtype=torch.int32, device=dev),
            "out_mass": torch.zeros((B, M), dtype=torch.float32, device=dev),
            "out_is_key": torch.zeros((B, M), dtype=torch.uint8, device=dev),
            "out_valid": torch.zeros((B, M), dtype=torch.uint8, device=dev),
            "out_count": torch.zeros((B,), dtype=torch.int32, device=dev),
            "key_index": torch.full((B, max(key_budget, 1)), -1, dtype=torch.int32, device=dev),
            "a_cls": torch.zeros((B, M), dtype=torch.float32, device=dev) if want_scores else None,
            "window_sim": torch.zeros((B, max(W, 1)), dtype=torch.float32, device=dev) if want_scores else None,
        }
    if workspace is None:
        workspace = encode_workspace(B, T, Hg, Wg, Hc, kt, kh, kw, dev)
    out["workspace"] = workspace
    _check(library().mustdrop_encode_merge(
        _ptr(x), C.c_int(_dtype_code(x)), _ptr(q_cls), _ptr(k_cls), C.c_int(qk_dtype), _ptr(mass_in), _ptr(valid),
        C.c_int(B), C.c_int(T), C.c_int(Hg), C.c_int(Wg), C.c_int(D), C.c_int(Hc), C.c_int(dc),
        C.c_int(kt), C.c_int(kh), C.c_int(kw), C.c_float(tau), C.c_int(key_budget),
        _ptr(out["out_x"]), _ptr(out["out_index"]), _ptr(out["out_mass"]), _ptr(out["out_is_key"]),
        _ptr(out["out_valid"]), _ptr(out["out_count"]), _ptr(out["key_index"]),
        _ptr(out.get("a_cls")), _ptr(out.get("window_sim")),
        _ptr(workspace), C.c_size_t(workspace.numel()), _stream(stream)))
    return out


def mustdrop_encode_merge_noalloc(x, q_cls, k_cls, mass_in, valid, T, Hg, Wg, kt, kh, kw, tau, key_budget, out: Dict,
                                  stream=None) -> Dict:
    """mustdrop_encode_merge on the library's static scratch buffer (no workspace argument; the call allocates
    nothing, so `out` must hold every output tensor; "a_cls" and "window_sim" may be None)."""
    B, M, D = x.shape
    if key_budget > 0:
        Hc, dc = q_cls.shape[1], q_cls.shape[2]
        qk_dtype = _dtype_code(q_cls)
    else:
        Hc, dc, qk_dtype = 1, D, _dtype_code(x)
    _check(library().mustdrop_encode_merge_noalloc(
        _ptr(x), C.c_int(_dtype_code(x)), _ptr(q_cls), _ptr(k_cls), C.c_int(qk_dtype), _ptr(mass_in), _ptr(valid),
        C.c_int(B), C.c_int(T), C.c_int(Hg), C.c_int(Wg), C.c_int(D), C.c_int(Hc), C.c_int(dc),
        C.c_int(kt), C.c_int(kh), C.c_int(kw), C.c_float(tau), C.c_int(key_budget),
        _ptr(out["out_x"]), _ptr(out["out_index"]), _ptr(out["out_mass"]), _ptr(out["out_is_key"]),
        _ptr(out["out_valid"]), _ptr(out["out_count"]), _ptr(out["key_index"]),
        _ptr(out.get("a_cls")), _ptr(out.get("window_sim")), _stream(stream)))
    return out


def mustdrop_encode_merge_adaptive(x, q_cls, k_cls, mass_in, valid, T, Hg, Wg, kt, kh, kw, tau, key_lambda, key_cap,
                                   out: Optional[Dict] = None, workspace=None, stream=None, want_scores=True) -> Dict:
    """Sec. 3.3 with Eq. 7 as printed: keys = {a_cls > mean + key_lambda * std}; key_index holds the first key_cap
    of them, key_count their number."""
    import torch
    B, M, D = x.shape
    dev = x.device
    Hc, dc = q_cls.shape[1], q_cls.shape[2]
    W = -(-T // kt) * -(-Hg // kh) * -(-Wg // kw)          # border windows are clipped to the grid
    if out is None:
        out = {
            "out_x": torch.zeros_like(x),
            "out_index": torch.full((B, M), -1, dtype=torch.int32, device=dev),
            "out_mass": torch.zeros((B, M), dtype=torch.float32, device=dev),
            "out_is_key": torch.zeros((B, M), dtype=torch.uint8, device=dev),
            "out_valid": torch.zeros((B, M), dtype=torch.uint8, device=dev),
            "out_count": torch.zeros((B,), dtype=torch.int32, device=dev),
            "key_index": torch.full((B, max(key_cap, 1)), -1, dtype=torch.int32, device=dev),
            "key_count": torch.zeros((B,), dtype=torch.int32, device=dev),
            "a_cls": torch.zeros((B, M), dtype=torch.float32, device=dev) if want_scores else None,
            "window_sim": torch.zeros((B, max(W, 1)), dtype=torch.float32, device=dev) if want_scores else None,
        }
    if workspace is None:
        workspace = encode_workspace(B, T, Hg, Wg, Hc, kt, kh, kw, dev)
    out["workspace"] = workspace
    _check(library().mustdrop_encode_merge_adaptive(
        _ptr(x), C.c_int(_dtype_code(x)), _ptr(q_cls), _ptr(k_cls), C.c_int(_dtype_code(q_cls)), _ptr(mass_in), _ptr(valid),
        C.c_int(B), C.c_int(T), C.c_int(Hg), C.c_int(Wg), C.c_int(D), C.c_int(Hc), C.c_int(dc),
        C.c_int(kt), C.c_int(kh), C.c_int(kw), C.c_float(tau), C.c_float(key_lambda), C.c_int(key_cap),
        _ptr(out["out_x"]), _ptr(out["out_index"]), _ptr(out["out_mass"]), _ptr(out["out_is_key"]),
        _ptr(out["out_valid"]), _ptr(out["out_count"]), _ptr(out["key_index"]), _ptr(out["key_count"]),
        _ptr(out.get("a_cls")), _ptr(out.get("window_sim")),
        _ptr(workspace), C.c_size_t(workspace.numel()), _stream(stream)))
    return out


def mustdrop_prefill_filter(q_txt, k, v, hidden, vis_valid, txt_len, is_key, Mv, softmax_scale, mode, budget,
                            gamma, alpha, Rcap=None, out: Optional[Dict] = None, workspace=None, stream=None,
                            want_scores=True, row_lse=None) -> Dict:
    """Sec. 3.4.  q_txt [B,N,H,d]; k, v [B,L,H,d]; hidden [B,L,C] (bf16); row_lse [B,H,N] f32 or None."""
    import torch
    B, N, H, d = q_txt.shape
    Cdim = hidden.shape[2]
    dev = q_txt.device
    if Rcap is None:
        Rcap = budget if mode == FILTER_BUDGET else Mv
    if out is None:
        out = {
            "hidden_out": torch.zeros((B, Rcap + N, Cdim), dtype=hidden.dtype, device=dev),
            "k_out": torch.zeros((B, Rcap + N, H, d), dtype=k.dtype, device=dev),
            "v_out": torch.zeros((B, Rcap + N, H, d), dtype=v.dtype, device=dev),
            "kept_index": torch.full((B, Rcap), -1, dtype=torch.int32, device=dev),
            "kept_count": torch.zeros((B,), dtype=torch.int32, device=dev),
            "out_len": torch.zeros((B,), dtype=torch.int32, device=dev),
            "out_protect": torch.zeros((B, Rcap + N), dtype=torch.uint8, device=dev),
            "out_ids": torch.full((B, Rcap + N), -1, dtype=torch.int32, device=dev),
            "score_global": torch.zeros((B, Mv), dtype=torch.float32, device=dev) if want_scores else None,
            "score_indiv": torch.zeros((B, Mv), dtype=torch.float32, device=dev) if want_scores else None,
        }
    if workspace is None:
        workspace = prefill_workspace(B, Mv, N, H, Rcap, dev)
    out["workspace"] = workspace
    _check(library().mustdrop_prefill_filter(
        _ptr(q_txt), _ptr(k), _ptr(v), _ptr(hidden), _ptr(vis_valid), _ptr(txt_len), _ptr(is_key), _ptr(row_lse),
        C.c_int(B), C.c_int(Mv), C.c_int(N), C.c_int(H), C.c_int(d), C.c_int(Cdim),
        C.c_float(softmax_scale), C.c_int(mode), C.c_int(budget), C.c_float(gamma), C.c_float(alpha),
        C.c_int(Rcap),
        _ptr(out["hidden_out"]), _ptr(out["k_out"]), _ptr(out["v_out"]),
        _ptr(out["kept_index"]), _ptr(out["kept_count"]), _ptr(out.get("out_len")), _ptr(out.get("out_protect")), _ptr(out.get("out_ids")),
        _ptr(out.get("score_global")), _ptr(out.get("score_indiv")),
        _ptr(workspace), C.c_size_t(workspace.numel()), _stream(stream)))
    return out


def mustdrop_decode_evict(q, k_cache, v_cache, acc, ids, protect, length, softmax_scale, decay, budget,
                          evicted_ids=None, evicted_count=None, workspace=None, stream=None):
    """Sec. 3.5, one decode step; the cache state is updated in place.  Returns the workspace used."""
    B, Lcap, H, d = k_cache.shape
    if workspace is None:
        workspace = decode_workspace(B, Lcap, H, k_cache.device)
    _check(library().mustdrop_decode_evict(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(acc), _ptr(ids), _ptr(protect), _ptr(length),
        C.c_int(B), C.c_int(Lcap), C.c_int(H), C.c_int(d),
        C.c_float(softmax_scale), C.c_float(decay), C.c_int(budget),
        _ptr(evicted_ids), _ptr(evicted_count),
        _ptr(workspace), C.c_size_t(workspace.numel()), _stream(stream)))
    return workspace


def mustdrop_decode_append(k_new, v_new, k_cache, v_cache, acc, ids, protect, length, new_id, protect_new=1,
                           stream=None):
    """Eq. 3: appends one entry per sample at slot len[b] (device-side, asynchronous)."""
    B, Lcap, H, d = k_cache.shape
    _check(library().mustdrop_decode_append(
        _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(acc), _ptr(ids), _ptr(protect), _ptr(length),
        C.c_int(B), C.c_int(Lcap), C.c_int(H), C.c_int(d), C.c_int(int(new_id)), C.c_int(int(protect_new)),
        _stream(stream)))


def mustdrop_decode_keep(k_caches, v_caches, keep, acc, ids, protect, length, evicted_ids=None, evicted_count=None,
                         workspace=None, stream=None):
    """Sec. 3.5, the static policy: only the entries flagged in ``keep`` stay, in the caches of all layers
    (k_caches, v_caches [n_layers,B,Lcap,H,d]); the state is updated in place.  Returns the workspace used."""
    n_layers, B, Lcap, H, d = k_caches.shape
    if workspace is None:
        workspace = decode_workspace(B, Lcap, H, k_caches.device)
    _check(library().mustdrop_decode_keep(
        _ptr(k_caches), _ptr(v_caches), _ptr(keep), _ptr(acc), _ptr(ids), _ptr(protect), _ptr(length),
        C.c_int(n_layers), C.c_int(B), C.c_int(Lcap), C.c_int(H), C.c_int(d),
        _ptr(evicted_ids), _ptr(evicted_count),
        _ptr(workspace), C.c_size_t(workspace.numel()), _stream(stream)))
    return workspace


def mustdrop_prefill_filter_strided(q_txt, k, v, hidden, vis_valid, txt_len, is_key, Mv, softmax_scale, mode, budget,
                                    gamma, alpha, out: Dict, Rcap=None, workspace=None, stream=None, row_lse=None) -> Dict:
    """Sec. 3.4 on Q / K / V in any layout: q_txt, k, v and out["k_out"], out["v_out"] are [B, tokens, H, d] VIEWS
    (e.g. a permuted head-major tensor); their strides are handed over as md_kv_layout.  k and v share one
    layout, k_out and v_out another.  `out` must hold every output tensor (see mustdrop_prefill_filter)."""
    B, N, H, d = q_txt.shape
    Cdim = hidden.shape[2]
    if Rcap is None:
        Rcap = budget if mode == FILTER_BUDGET else Mv
    assert k.stride() == v.stride() and out["k_out"].stride() == out["v_out"].stride()
    assert tuple(out["k_out"].shape) == (B, Rcap + N, H, d)
    if workspace is None:
        workspace = prefill_workspace(B, Mv, N, H, Rcap, q_txt.device)
    out["workspace"] = workspace
    lq, lkv, lo = _layout(q_txt), _layout(k), _layout(out["k_out"])
    _check(library().mustdrop_prefill_filter_strided(
        _view_ptr(q_txt), _view_ptr(k), _view_ptr(v), _ptr(hidden), _ptr(vis_valid), _ptr(txt_len), _ptr(is_key), _ptr(row_lse),
        C.c_int(B), C.c_int(Mv), C.c_int(N), C.c_int(H), C.c_int(d), C.c_int(Cdim),
        C.c_float(softmax_scale), C.c_int(mode), C.c_int(budget), C.c_float(gamma), C.c_float(alpha),
        C.c_int(Rcap),
        _ptr(out["hidden_out"]), _view_ptr(out["k_out"]), _view_ptr(out["v_out"]),
        _ptr(out["kept_index"]), _ptr(out["kept_count"]), _ptr(out.get("out_len")), _ptr(out.get("out_protect")), _ptr(out.get("out_ids")),
        _ptr(out.get("score_global")), _ptr(out.get("score_indiv")),
        C.byref(lq), C.byref(lkv), C.byref(lo),
        _ptr(workspace), C.c_size_t(workspace.numel()), _stream(stream)))
    return out


def mustdrop_decode_evict_strided(q, k_cache, v_cache, acc, ids, protect, length, softmax_scale, decay, budget,
                                  evicted_ids=None, evicted_count=None, workspace=None, stream=None):
    """Sec. 3.5, one decode step on caches given as [B, Lcap, H, d] views of any layout."""
    B, Lcap, H, d = k_cache.shape
    assert k_cache.stride() == v_cache.stride()
    if workspace is None:
        workspace = decode_workspace(B, Lcap, H, k_cache.device)
    lay = _layout(k_cache)
    _check(library().mustdrop_decode_evict_strided(
        _ptr(q), _view_ptr(k_cache), _view_ptr(v_cache), _ptr(acc), _ptr(ids), _ptr(protect), _ptr(length),
        C.c_int(B), C.c_int(Lcap), C.c_int(H), C.c_int(d),
        C.c_float(softmax_scale), C.c_float(decay), C.c_int(budget),
        _ptr(evicted_ids), _ptr(evicted_count), C.byref(lay),
        _ptr(workspace), C.c_size_t(workspace.numel()), _stream(stream)))
    return workspace


def mustdrop_decode_append_strided(k_new, v_new, k_cache, v_cache, acc, ids, protect, length, new_id, protect_new=1,
                                   stream=None):
    """Eq. 3 on caches given as [B, Lcap, H, d] views of any layout."""
    B, Lcap, H, d = k_cache.shape
    assert k_cache.stride() == v_cache.stride()
    lay = _layout(k_cache)
    _check(library().mustdrop_decode_append_strided(
        _ptr(k_new), _ptr(v_new), _view_ptr(k_cache), _view_ptr(v_cache), _ptr(acc), _ptr(ids), _ptr(protect),
        _ptr(length), C.c_int(B), C.c_int(Lcap), C.c_int(H), C.c_int(d), C.c_int(int(new_id)),
        C.c_int(int(protect_new)), C.byref(lay), _stream(stream)))


def mustdrop_decode_keep_strided(k_caches, v_caches, keep, acc, ids, protect, length, evicted_ids=None,
                                 evicted_count=None, workspace=None, stream=None):
    """Sec. 3.5, the static policy on caches given as [n_layers, B, Lcap, H, d] views of any layout."""
    n_layers, B, Lcap, H, d = k_caches.shape
    assert k_caches.stride() == v_caches.stride()
    if workspace is None:
        workspace = decode_workspace(B, Lcap, H, k_caches.device)
    lay = _layout(k_caches)
    _check(library().mustdrop_decode_keep_strided(
        _view_ptr(k_caches), _view_ptr(v_caches), _ptr(keep), _ptr(acc), _ptr(ids), _ptr(protect), _ptr(length),
        C.c_int(n_layers), C.c_int(B), C.c_int(Lcap), C.c_int(H), C.c_int(d),
        _ptr(evicted_ids), _ptr(evicted_count), C.byref(lay), C.c_int64(k_caches.stride(0)),
        _ptr(workspace), C.c_size_t(workspace.numel()), _stream(stream)))
    return workspace


def profile_start():
    """Benchmarking aid: bracket every kernel launch with HIP events until profile_stop()."""
    _check(library().mustdrop_profile_start())


def profile_stop(cap: int = 64) -> Dict[str, Dict[str, float]]:
    """Returns {kernel name: {"ms": summed milliseconds, "calls": launches}}."""
    names = C.create_string_buffer(64 * cap)
    ms = (C.c_float * cap)()
    calls = (C.c_int * cap)()
    n = C.c_int(0)
    _check(library().mustdrop_profile_stop(names, ms, calls, C.c_int(cap), C.byref(n)))
    out = {}
    for i in range(n.value):
        nm = names.raw[64 * i:64 * (i + 1)].split(b"\0", 1)[0].decode()
        out[nm] = {"ms": float(ms[i]), "calls": int(calls[i])}
    return out
