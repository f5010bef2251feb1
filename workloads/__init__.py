"""Seeded synthetic inputs for the MustDrop token-reduction path.

This module only *draws inputs* (random fields, Gaussian tensors, masks).  It
contains none of the method's arithmetic: no similarity, softmax, selection or
compaction lives here.  Both the CPU oracle's tests and the GPU path's tests /
benchmark take their inputs from here so that they see identical bit patterns.

The shapes stand in for the workloads the paper evaluates (LLaVA-1.5: a 24x24
patch grid = 576 vision tokens; LLaVA-NeXT: 5 tiles = 2880 tokens; video: 8
frames) -- see Sec. 4.2 / Tables 1, 2 and 6 of the paper.  No dataset item is
reproduced; everything is a seeded random field.

bf16 tensors are carried as ``numpy.uint16`` bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

MASTER_SEED = 20241110

F32 = 0
BF16 = 1


# --------------------------------------------------------------------------
# bf16 helpers (storage format only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    out = (r >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    """Exact widening of a stored tensor (F32 array or BF16 bits) to float64."""
    if dtype == BF16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def store(a: np.ndarray, dtype: int) -> np.ndarray:
    """float array -> storage array of the requested dtype."""
    if dtype == BF16:
        return f32_to_bf16_bits(a.astype(np.float32))
    return np.ascontiguousarray(a, dtype=np.float32)


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    """One synthetic workload.  Vision grid is T x Hg x Wg (T = frames or tiles)."""
    name: str
    number: int                     # 1..5 -> seed offset
    B: int
    T: int = 1
    Hg: int = 24
    Wg: int = 24
    D: int = 1024                   # vision feature dim
    Hc: int = 16                    # CLS-attention heads (Hc*dc == D)
    dc: int = 64
    x_dtype: int = BF16
    kt: int = 1
    kh: int = 2
    kw: int = 2
    tau: float = 0.85
    bench_tau: float = 0.955        # merge threshold of the benchmark: leaves about three quarters of the tokens,
                                    # the merge rate of Table 3 (440 of 576), on this workload's random fields
    key_budget: int = 32
    N: int = 64                     # text tokens
    H: int = 32                     # LLM heads
    d: int = 128                    # head dim
    C: int = 4096                   # LLM hidden
    budgets: Tuple[int, ...] = (192,)
    field_kind: str = "image"       # image | tiles | video
    ell: Tuple[float, float] = (2.0, 2.0)   # correlation length range (cells)
    sigma_n: float = 0.1
    drift: float = 0.05
    # decode
    L0: int = 0
    steps: int = 0
    decode_budget: int = 0
    n_protect: int = 0
    heavy_frac: float = 0.05

    @property
    def M(self) -> int:
        return self.T * self.Hg * self.Wg

    @property
    def L(self) -> int:
        return self.M + self.N

    @property
    def seed(self) -> int:
        return MASTER_SEED + self.number


CONFIGS: Dict[int, Config] = {
    1: Config("cfg1_llava15_single", 1, B=1, x_dtype=F32, N=32, key_budget=32,
              budgets=(192,), ell=(2.0, 2.0), bench_tau=0.913),
    2: Config("cfg2_llava15_b16", 2, B=16, N=64, key_budget=32,
              budgets=(192, 128, 64), ell=(1.0, 4.0)),
    3: Config("cfg3_llavanext_b8", 3, B=8, T=5, N=128, key_budget=128,
              budgets=(320,), field_kind="tiles", bench_tau=0.942),
    4: Config("cfg4_video_b4", 4, B=4, T=8, kt=2, N=64, key_budget=128,
              budgets=(512,), field_kind="video", bench_tau=0.9215),
    5: Config("cfg5_decode_b64", 5, B=64, L0=4096, steps=256, decode_budget=1024,
              n_protect=128),
}


def tiny(cfg: Config, **kw) -> Config:
    """A reduced copy of a config (tests)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------
# random fields
# --------------------------------------------------------------------------
def smooth_field(rng: np.random.Generator, n_chan: int, Hg: int, Wg: int, ell: float) -> np.ndarray:
    """[Hg*Wg, n_chan] float32: per channel, periodic white noise convolved with a
    Gaussian kernel of std ``ell`` cells, scaled to unit expected variance.
    The autocorrelation at lag r is exp(-r^2 / (4 ell^2)) (up to periodic wrap)."""
    w = rng.standard_normal((n_chan, Hg, Wg), dtype=np.float32)
    fy = np.fft.fftfreq(Hg)[:, None]
    fx = np.fft.rfftfreq(Wg)[None, :]
    tf = np.exp(-2.0 * (np.pi * ell) ** 2 * (fy * fy + fx * fx))
    # gain^2 = mean over all frequencies of |tf|^2 (Parseval), using the full grid
    fx_full = np.fft.fftfreq(Wg)[None, :]
    tf_full = np.exp(-2.0 * (np.pi * ell) ** 2 * (fy * fy + fx_full * fx_full))
    gain = np.sqrt(np.mean(tf_full ** 2))
    f = np.fft.irfft2(np.fft.rfft2(w, axes=(1, 2)) * tf[None], s=(Hg, Wg), axes=(1, 2))
    f = (f / gain).astype(np.float32)
    return np.ascontiguousarray(f.reshape(n_chan, Hg * Wg).T)


def _sample_rngs(seed: int, B: int, stream: int):
    ss = np.random.SeedSequence([seed, stream])
    return [np.random.default_rng(s) for s in ss.spawn(B)]


def vision_features(cfg: Config, samples: Optional[Sequence[int]] = None):
    """Patch features and CLS row for the encode stage.

    Returns (x [b, M, D] float32, cls [b, D] float32, ell [b]) before storage
    rounding.  ``samples`` selects a subset of batch entries (same values as in
    the full batch)."""
    rngs = _sample_rngs(cfg.seed, cfg.B, 1)
    idx = list(range(cfg.B)) if samples is None else list(samples)
    xs, cs, ells = [], [], []
    P = cfg.Hg * cfg.Wg
    for b in idx:
        rng = rngs[b]
        ell = float(rng.uniform(cfg.ell[0], cfg.ell[1])) if cfg.ell[0] != cfg.ell[1] else float(cfg.ell[0])
        if cfg.field_kind == "image":
            frames = [smooth_field(rng, cfg.D, cfg.Hg, cfg.Wg, ell) for _ in range(cfg.T)]
            frames = [f + cfg.sigma_n * rng.standard_normal(f.shape, dtype=np.float32) for f in frames]
        elif cfg.field_kind == "tiles":
            shared = smooth_field(rng, cfg.D, cfg.Hg, cfg.Wg, 4.0)
            frames = []
            for _ in range(cfg.T):
                own = smooth_field(rng, cfg.D, cfg.Hg, cfg.Wg, 2.0)
                f = np.float32(np.sqrt(0.5)) * (shared + own)
                frames.append(f + cfg.sigma_n * rng.standard_normal(f.shape, dtype=np.float32))
        elif cfg.field_kind == "video":
            f = smooth_field(rng, cfg.D, cfg.Hg, cfg.Wg, ell)
            f = f + cfg.sigma_n * rng.standard_normal(f.shape, dtype=np.float32)
            frames = [f]
            for _ in range(cfg.T - 1):
                f = f + cfg.drift * rng.standard_normal(f.shape, dtype=np.float32)
                frames.append(f)
        else:
            raise ValueError(cfg.field_kind)
        x = np.concatenate(frames, axis=0).astype(np.float32)
        assert x.shape == (cfg.T * P, cfg.D)
        cls = x.mean(axis=0) + rng.standard_normal(cfg.D, dtype=np.float32)
        xs.append(x)
        cs.append(cls.astype(np.float32))
        ells.append(ell)
    return np.stack(xs), np.stack(cs), np.asarray(ells)


def encode_inputs(cfg: Config, samples: Optional[Sequence[int]] = None) -> Dict[str, np.ndarray]:
    """Stored tensors for the encode stage.

    x      [b, M, D]        cfg.x_dtype (patch tokens; index = (t*Hg + y)*Wg + x)
    k_cls  [b, 1+M, Hc, dc] cfg.x_dtype (row 0 = CLS key, rows 1.. = patch keys;
                            the synthetic keys are the features viewed as Hc x dc)
    q_cls  [b, Hc, dc]      cfg.x_dtype (CLS query = the CLS row)
    """
    x, cls, ell = vision_features(cfg, samples)
    b = x.shape[0]
    k = np.concatenate([cls[:, None, :], x], axis=1)
    return {
        "x": store(x, cfg.x_dtype),
        "k_cls": store(k, cfg.x_dtype).reshape(b, 1 + cfg.M, cfg.Hc, cfg.dc),
        "q_cls": store(cls, cfg.x_dtype).reshape(b, cfg.Hc, cfg.dc),
        "ell": ell,
    }


def random_valid_mask(cfg: Config, frac_invalid: float, stream: int = 7) -> np.ndarray:
    """[B, M] uint8 mask with about ``frac_invalid`` of slots marked padding."""
    rng = np.random.default_rng([cfg.seed, stream])
    return (rng.random((cfg.B, cfg.M)) >= frac_invalid).astype(np.uint8)


def random_key_mask(cfg: Config, n_keys: int, stream: int = 8, valid: Optional[np.ndarray] = None) -> np.ndarray:
    """[B, M] uint8 with exactly ``n_keys`` ones per sample (stand-in key set)."""
    rng = np.random.default_rng([cfg.seed, stream])
    out = np.zeros((cfg.B, cfg.M), dtype=np.uint8)
    for b in range(cfg.B):
        cand = np.arange(cfg.M) if valid is None else np.flatnonzero(valid[b])
        pick = rng.choice(cand, size=min(n_keys, cand.size), replace=False)
        out[b, pick] = 1
    return out


def _normal_bf16(rng: np.random.Generator, shape, scale: float = 1.0) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    return f32_to_bf16_bits(a)


def prefill_inputs(cfg: Config, samples: Optional[Sequence[int]] = None, literal_scale: bool = False,
                   with_payload: bool = True) -> Dict[str, np.ndarray]:
    """bf16 tensors of one LLM layer at prefill, sequence = [vision M | text N].

    q_txt [b, N, H, d], k, v [b, L, H, d], hidden [b, L, C]; elements ~ N(0,1)
    (the benchmark uses softmax_scale = 1/sqrt(d), i.e. unit-variance logits).
    ``literal_scale`` divides Q and K elements by sqrt(d) as well (near-uniform
    softmax: a near-tie stress case)."""
    rngs = _sample_rngs(cfg.seed, cfg.B, 2)
    idx = list(range(cfg.B)) if samples is None else list(samples)
    s = 1.0 / np.sqrt(cfg.d) if literal_scale else 1.0
    q, k, v, h = [], [], [], []
    for b in idx:
        rng = rngs[b]
        q.append(_normal_bf16(rng, (cfg.N, cfg.H, cfg.d), s))
        k.append(_normal_bf16(rng, (cfg.L, cfg.H, cfg.d), s))
        if with_payload:
            v.append(_normal_bf16(rng, (cfg.L, cfg.H, cfg.d)))
            h.append(_normal_bf16(rng, (cfg.L, cfg.C)))
    out = {"q_txt": np.stack(q), "k": np.stack(k)}
    if with_payload:
        out["v"] = np.stack(v)
        out["hidden"] = np.stack(h)
    return out


def layer_text_queries(cfg: Config, layer: int, samples: Optional[Sequence[int]] = None) -> np.ndarray:
    """q_txt [b, N, H, d] bf16 of a later LLM layer (layer >= 1) for chained, progressively smaller
    prefill calls; elements ~ N(0,1), independent of the layer-0 queries of prefill_inputs()."""
    assert layer >= 1
    rngs = _sample_rngs(cfg.seed, cfg.B, 20 + layer)
    idx = list(range(cfg.B)) if samples is None else list(samples)
    return np.stack([_normal_bf16(rngs[b], (cfg.N, cfg.H, cfg.d)) for b in idx])


def random_bf16_payload(rng: np.random.Generator, shape) -> np.ndarray:
    """Cheap finite bf16 bit patterns (|value| < 2) for tensors that are only moved."""
    bits = rng.integers(0, 1 << 16, size=shape, dtype=np.uint16)
    # clear the top exponent bit -> exponent field <= 127 -> finite, |v| < 2
    return bits & np.uint16(0xBFFF)


def decode_inputs(cfg: Config, samples: Optional[Sequence[int]] = None, Lcap: Optional[int] = None,
                  steps: Optional[int] = None, literal_scale: bool = False) -> Dict[str, np.ndarray]:
    """KV cache state and per-step queries / appended entries for decode eviction.

    k_cache, v_cache [b, Lcap, H, d] bf16 (entries >= len0 are zero)
    q_steps [steps, b, H, d], k_new, v_new [steps, b, H, d] bf16
    protect [b, Lcap] uint8 (n_protect seeded entries of the initial cache)
    heavy   [b, L0]  uint8 (the planted heavy-hitter keys)

    Keys ~ N(0,1); a seeded ``heavy_frac`` of them get +mu on every element and
    each query gets +mu, with mu^2 * d / sqrt(d) = 3, so heavy hitters' scaled
    logits sit about three standard deviations above the rest."""
    steps = cfg.steps if steps is None else steps
    Lcap = cfg.L0 + steps if Lcap is None else Lcap
    assert Lcap >= cfg.L0 + max(steps - 1, 0)
    rngs = _sample_rngs(cfg.seed, cfg.B, 3)
    idx = list(range(cfg.B)) if samples is None else list(samples)
    mu = np.float32(np.sqrt(3.0 / np.sqrt(cfg.d)))
    s = np.float32(1.0 / np.sqrt(cfg.d)) if literal_scale else np.float32(1.0)
    nb = len(idx)
    kc = np.zeros((nb, Lcap, cfg.H, cfg.d), dtype=np.uint16)
    vc = np.zeros((nb, Lcap, cfg.H, cfg.d), dtype=np.uint16)
    qs = np.zeros((steps, nb, cfg.H, cfg.d), dtype=np.uint16)
    kn = np.zeros((steps, nb, cfg.H, cfg.d), dtype=np.uint16)
    vn = np.zeros((steps, nb, cfg.H, cfg.d), dtype=np.uint16)
    protect = np.zeros((nb, Lcap), dtype=np.uint8)
    heavy = np.zeros((nb, cfg.L0), dtype=np.uint8)
    for o, b in enumerate(idx):
        rng = rngs[b]
        hv = rng.random(cfg.L0) < cfg.heavy_frac
        heavy[o] = hv
        k = rng.standard_normal((cfg.L0, cfg.H, cfg.d), dtype=np.float32)
        k[hv] += mu
        kc[o, :cfg.L0] = f32_to_bf16_bits(k * s)
        del k
        vc[o, :cfg.L0] = random_bf16_payload(rng, (cfg.L0, cfg.H, cfg.d))
        pick = rng.choice(cfg.L0, size=min(cfg.n_protect, cfg.L0), replace=False)
        protect[o, pick] = 1
        q = rng.standard_normal((steps, cfg.H, cfg.d), dtype=np.float32) + mu
        qs[:, o] = f32_to_bf16_bits(q * s)
        kn[:, o] = _normal_bf16(rng, (steps, cfg.H, cfg.d), float(s))
        vn[:, o] = random_bf16_payload(rng, (steps, cfg.H, cfg.d))
    return {"k_cache": kc, "v_cache": vc, "q_steps": qs, "k_new": kn, "v_new": vn,
            "protect": protect, "heavy": heavy,
            "len0": np.full(nb, cfg.L0, dtype=np.int32), "Lcap": Lcap}
