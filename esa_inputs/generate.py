"""Seeded generation of one attention layer's tensors for an ESA workload.

Recipe (per batch element):
  * Q [S,H,d], K [S,H_kv,d], V [S,H_kv,d] ~ N(0,1) from Philox streams keyed by
    (seed, tensor, batch) with the counter advanced per block of ROW_BLOCK rows, so
    any row range can be regenerated alone;
  * rotary position encoding (rotate-half form, absolute positions) on Q and K
    when the configuration names a base;
  * W_q [H*d, d_c], W_k [H_kv*d, d_c] ~ N(0, std 1/sqrt(fan_in));
  * planted structure: every chunk with a large enough middle segment owns a
    random unit direction u in R^{d_c}.  The chunk's queries get the extra
    component beta * (u P_q) and `needles` middle tokens (or spans of tokens) get
    the key alpha_i * (u P_k), where P = pinv(W) is the least-norm pre-image map of
    the stored weights, i.e. (u P) W = u.  The compressed needle keys are
    therefore aligned with the chunk's mean compressed query.
  * push_keys_down: adds a small multiple of the pre-image of -u to chosen key rows; test
    harnesses use it to clear a band of near-tied scores below a selection boundary (they
    decide which rows; this module only edits the data).
Values are produced in fp32 and stored as fp32 or as bf16 bit patterns (uint16,
round-to-nearest-even).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

from .configs import EsaConfig, segment_bounds, chunk_starts

ROW_BLOCK = 1024

_T_Q, _T_K, _T_V, _T_WQ, _T_WK, _T_DIR, _T_POS, _T_AMP = range(1, 9)


# ----------------------------------------------------------------------------- storage
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern, round to nearest, ties to even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a stored tensor to float64."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- streams
def _stream(seed: int, tensor: int, batch: int, block: int = 0, sub: int = 0) -> np.random.Generator:
    key = np.array([np.uint64(seed), (np.uint64(tensor) << np.uint64(40)) | np.uint64(batch)], dtype=np.uint64)
    counter = np.array([0, 0, np.uint64(block), np.uint64(sub)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key, counter=counter))


def _normal_rows(seed: int, tensor: int, batch: int, r0: int, r1: int, width: int) -> np.ndarray:
    """Rows [r0,r1) of an N(0,1) fp32 matrix with `width` columns, independent of the range asked."""
    out = np.empty((r1 - r0, width), dtype=np.float32)
    b0, b1 = r0 // ROW_BLOCK, (r1 + ROW_BLOCK - 1) // ROW_BLOCK
    for b in range(b0, b1):
        blk = _stream(seed, tensor, batch, b).standard_normal((ROW_BLOCK, width), dtype=np.float32)
        lo, hi = max(r0, b * ROW_BLOCK), min(r1, (b + 1) * ROW_BLOCK)
        out[lo - r0:hi - r0] = blk[lo - b * ROW_BLOCK:hi - b * ROW_BLOCK]
    return out


def _rope_inplace(x: np.ndarray, r0: int, n_heads: int, d: int, base: float) -> None:
    """Rotate-half rotary encoding at absolute positions r0.. on x [rows, n_heads*d] (fp32)."""
    rows = x.shape[0]
    half = d // 2
    inv_freq = base ** (-np.arange(half, dtype=np.float64) * 2.0 / d)
    ang = np.arange(r0, r0 + rows, dtype=np.float64)[:, None] * inv_freq[None, :]
    cos = np.cos(ang).astype(np.float32)[:, None, :]
    sin = np.sin(ang).astype(np.float32)[:, None, :]
    xv = x.reshape(rows, n_heads, d)
    x1 = xv[:, :, :half].copy()
    x2 = xv[:, :, half:].copy()
    xv[:, :, :half] = x1 * cos - x2 * sin
    xv[:, :, half:] = x2 * cos + x1 * sin


# ----------------------------------------------------------------------------- weights
def make_weights(cfg: EsaConfig):
    """Compression weights in storage form: W_q [H*d, d_c], W_k [H_kv*d, d_c]."""
    wq = _stream(cfg.seed, _T_WQ, 0).standard_normal((cfg.d_Hq, cfg.d_c), dtype=np.float32)
    wk = _stream(cfg.seed, _T_WK, 0).standard_normal((cfg.d_K, cfg.d_c), dtype=np.float32)
    wq *= np.float32(1.0 / np.sqrt(cfg.d_Hq))
    wk *= np.float32(1.0 / np.sqrt(cfg.d_K))
    return to_storage(wq, cfg.dtype), to_storage(wk, cfg.dtype)


# ----------------------------------------------------------------------------- planted structure
@dataclass
class NeedlePlan:
    """Which chunk owns which planted tokens, and with what direction and amplitudes."""
    t0: List[int] = field(default_factory=list)              # chunk start of every planted chunk
    direction: Dict[int, np.ndarray] = field(default_factory=dict)   # t0 -> u [d_c] (float64, unit)
    positions: Dict[int, np.ndarray] = field(default_factory=dict)   # t0 -> absolute token positions
    amplitude: Dict[int, np.ndarray] = field(default_factory=dict)   # t0 -> alpha_i per position
    beta: float = 0.0


def needle_plan(cfg: EsaConfig, batch: int = 0) -> NeedlePlan:
    plan = NeedlePlan(beta=float(np.sqrt(cfg.d_c)))
    alpha = 4.0 * np.sqrt(cfg.d_c)
    used = np.zeros(cfg.S, dtype=bool)
    span = cfg.needle_span
    for j, t0 in enumerate(chunk_starts(cfg)):
        i_end, l_start = segment_bounds(t0, cfg.l_I, cfg.l_L)
        n_mid = l_start - i_end
        if cfg.needles == 0 or n_mid < 4 * cfg.needles * span:
            continue
        rng = _stream(cfg.seed, _T_POS, batch, j)
        starts = i_end + span * np.arange(n_mid // span)
        taken = used[i_end:i_end + starts.shape[0] * span].reshape(-1, span).any(axis=1)
        free = starts[~taken]
        pick = np.sort(rng.choice(free, size=cfg.needles, replace=False))
        pos = (pick[:, None] + np.arange(span)[None, :]).reshape(-1)
        used[pos] = True
        u = _stream(cfg.seed, _T_DIR, batch, j).standard_normal(cfg.d_c)
        u /= np.linalg.norm(u)
        amp = alpha * (1.0 + 0.25 * _stream(cfg.seed, _T_AMP, batch, j).random(pos.shape[0]))
        plan.t0.append(t0)
        plan.direction[t0] = u
        plan.positions[t0] = pos.astype(np.int64)
        plan.amplitude[t0] = amp
    return plan


_PINV_CACHE: Dict[tuple, np.ndarray] = {}


def _pinv_wk(cfg: EsaConfig) -> np.ndarray:
    key = (cfg.seed, cfg.dtype, cfg.d_K, cfg.d_c)
    if key not in _PINV_CACHE:
        _PINV_CACHE[key] = np.linalg.pinv(storage_to_f64(make_weights(cfg)[1], cfg.dtype))
    return _PINV_CACHE[key]


def push_keys_down(cfg: EsaConfig, batch: int, key_rows: np.ndarray, away_from, plan: NeedlePlan,
                   delta: float) -> np.ndarray:
    """Stored key rows [n, H_kv, d] with a small planted component added, re-rounded to storage.

    Row i gets the pre-image of -delta * u for every chunk start t0 in away_from[i] that owns a
    planted direction u.  All queries of that chunk share the component +beta * u in compressed
    space, so the row's compressed score drops for every one of them (by delta * (beta + noise)),
    while for other chunks the change is a small random perturbation.  Test harnesses use this to
    open a gap below a selection boundary; which rows to push is their decision.
    """
    rows = storage_to_f64(key_rows, cfg.dtype).reshape(-1, cfg.d_K)
    p_k = _pinv_wk(cfg)
    for i in range(rows.shape[0]):
        push = np.zeros(cfg.d_c)
        for t0 in away_from[i]:
            if t0 in plan.direction:
                push -= delta * plan.direction[t0]
        rows[i] += push @ p_k
    return to_storage(rows.astype(np.float32), cfg.dtype).reshape(-1, cfg.H_kv, cfg.d)


# ----------------------------------------------------------------------------- the layer
@dataclass
class LayerInputs:
    cfg: EsaConfig
    batch: int
    Q: np.ndarray        # [S, H, d]     storage form
    K: np.ndarray        # [S, H_kv, d]
    V: np.ndarray        # [S, H_kv, d]
    W_q: np.ndarray      # [H*d, d_c]
    W_k: np.ndarray      # [H_kv*d, d_c]
    plan: NeedlePlan

    def f64(self, name: str, r0: Optional[int] = None, r1: Optional[int] = None) -> np.ndarray:
        a = getattr(self, name)
        if r0 is not None:
            a = a[r0:r1]
        return storage_to_f64(a, self.cfg.dtype)


def make_layer(cfg: EsaConfig, batch: int = 0, q_rows: Optional[tuple] = None) -> LayerInputs:
    """Generate one batch element.  `q_rows=(r0,r1)` limits Q to those rows (K and V are
    always whole, since every step reads the whole cache); Q is then [r1-r0, H, d]."""
    S = cfg.S
    wq_s, wk_s = make_weights(cfg)
    plan = needle_plan(cfg, batch)
    p_q = np.linalg.pinv(storage_to_f64(wq_s, cfg.dtype))   # [d_c, H*d]
    p_k = np.linalg.pinv(storage_to_f64(wk_s, cfg.dtype))   # [d_c, H_kv*d]

    qr0, qr1 = (0, S) if q_rows is None else q_rows
    sdt = np.float32 if cfg.dtype == "f32" else np.uint16
    Q = np.empty((qr1 - qr0, cfg.d_Hq), dtype=sdt)
    K = np.empty((S, cfg.d_K), dtype=sdt)
    V = np.empty((S, cfg.d_K), dtype=sdt)

    needle_img = {t0: plan.direction[t0] @ p_k for t0 in plan.t0}                # [H_kv*d] each
    query_add = {t0: (plan.beta * (plan.direction[t0] @ p_q)).astype(np.float32) for t0 in plan.t0}

    step = 4 * ROW_BLOCK

    def kv_block(r0: int) -> None:
        r1 = min(S, r0 + step)
        k = _normal_rows(cfg.seed, _T_K, batch, r0, r1, cfg.d_K)
        if cfg.rope_base:
            _rope_inplace(k, r0, cfg.H_kv, cfg.d, cfg.rope_base)
        for t0 in plan.t0:
            pos = plan.positions[t0]
            sel = (pos >= r0) & (pos < r1)
            if sel.any():
                k[pos[sel] - r0] = (plan.amplitude[t0][sel, None] * needle_img[t0][None, :]).astype(np.float32)
        K[r0:r1] = to_storage(k, cfg.dtype)
        V[r0:r1] = to_storage(_normal_rows(cfg.seed, _T_V, batch, r0, r1, cfg.d_K), cfg.dtype)

    def q_block(r0: int) -> None:
        a, b = max(r0, qr0), min(r0 + step, qr1, S)
        if a >= b:
            return
        q = _normal_rows(cfg.seed, _T_Q, batch, a, b, cfg.d_Hq)
        if cfg.rope_base:
            _rope_inplace(q, a, cfg.H, cfg.d, cfg.rope_base)
        for t0 in plan.t0:
            lo, hi = max(a, t0), min(b, t0 + cfg.l_C)
            if lo < hi:
                q[lo - a:hi - a] += query_add[t0][None, :]
        Q[a - qr0:b - qr0] = to_storage(q, cfg.dtype)

    # Row blocks are independent (each has its own counter range), so they are drawn by a
    # few threads; the result does not depend on the thread count.
    with ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1))) as pool:
        list(pool.map(kv_block, range(0, S, step)))
        list(pool.map(q_block, range(qr0 - qr0 % step, qr1, step)))

    return LayerInputs(cfg, batch,
                       Q.reshape(-1, cfg.H, cfg.d), K.reshape(S, cfg.H_kv, cfg.d),
                       V.reshape(S, cfg.H_kv, cfg.d), wq_s, wk_s, plan)
