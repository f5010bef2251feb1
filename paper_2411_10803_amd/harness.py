"""Host <-> device plumbing for tests, the smoke check and the benchmark: numpy arrays (bf16 as
uint16 bit patterns) to torch device tensors and back.  No arithmetic of the method lives here."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from . import binding as md


def to_dev(a: Optional[np.ndarray], bf16: bool = False, device="cuda"):
    import torch
    if a is None:
        return None
    if a.dtype == np.uint16:
        t = torch.from_numpy(a.view(np.int16)).to(device)
        return t.view(torch.bfloat16) if bf16 else t
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def to_host(t) -> Optional[np.ndarray]:
    import torch
    if t is None:
        return None
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def outputs_to_host(out: Dict) -> Dict[str, np.ndarray]:
    return {k: to_host(v) for k, v in out.items() if k != "workspace" and v is not None}


def encode_on_gpu(x, x_dtype, q_cls, k_cls, qk_dtype, mass_in, valid, T, Hg, Wg, kt, kh, kw, tau, key_budget):
    out = md.mustdrop_encode_merge(
        to_dev(x, x_dtype == md.BF16), to_dev(q_cls, qk_dtype == md.BF16), to_dev(k_cls, qk_dtype == md.BF16),
        to_dev(mass_in), to_dev(valid), T, Hg, Wg, kt, kh, kw, tau, key_budget)
    g = outputs_to_host(out)
    if key_budget == 0:
        g["key_index"] = np.zeros((x.shape[0], 0), dtype=np.int32)
    return g


def encode_adaptive_on_gpu(x, x_dtype, q_cls, k_cls, qk_dtype, mass_in, valid, T, Hg, Wg, kt, kh, kw, tau, key_lambda,
                           key_cap):
    out = md.mustdrop_encode_merge_adaptive(
        to_dev(x, x_dtype == md.BF16), to_dev(q_cls, qk_dtype == md.BF16), to_dev(k_cls, qk_dtype == md.BF16),
        to_dev(mass_in), to_dev(valid), T, Hg, Wg, kt, kh, kw, tau, key_lambda, key_cap)
    g = outputs_to_host(out)
    if key_cap == 0:
        g["key_index"] = np.zeros((x.shape[0], 0), dtype=np.int32)
    return g


def prefill_on_gpu(t, Mv, vis_valid, txt_len, is_key, scale, mode, budget, gamma, alpha, Rcap=None, row_lse=None):
    out = md.mustdrop_prefill_filter(
        to_dev(t["q_txt"], True), to_dev(t["k"], True), to_dev(t["v"], True), to_dev(t["hidden"], True),
        to_dev(vis_valid), to_dev(txt_len), to_dev(is_key), Mv, scale, mode, budget, gamma, alpha, Rcap,
        row_lse=to_dev(row_lse))
    return outputs_to_host(out)


def decode_state_to_dev(s):
    """s: dict with k, v (uint16), acc, ids, protect, len numpy arrays -> device tensors (copies)."""
    return {"k": to_dev(s["k"], True), "v": to_dev(s["v"], True), "acc": to_dev(s["acc"]), "ids": to_dev(s["ids"]),
            "protect": to_dev(s["protect"]), "len": to_dev(s["len"])}


def decode_on_gpu(q, d, scale, decay, budget, workspace=None):
    """One decode step on a device state dict (in place); returns evicted ids / counts as device tensors."""
    import torch
    B, Lcap = d["ids"].shape
    ev = torch.full((B, Lcap), -1, dtype=torch.int32, device=d["ids"].device)
    evc = torch.zeros((B,), dtype=torch.int32, device=d["ids"].device)
    md.mustdrop_decode_evict(q, d["k"], d["v"], d["acc"], d["ids"], d["protect"], d["len"], scale, decay, budget,
                             ev, evc, workspace)
    return ev, evc


def decode_state_to_host(d, ev=None, evc=None):
    g = {k: to_host(v) for k, v in d.items()}
    if ev is not None:
        g["evicted_ids"], g["evicted_count"] = to_host(ev), to_host(evc)
    return g
