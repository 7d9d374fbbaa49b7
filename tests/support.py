"""Glue shared by the GPU parity tests: storage <-> torch conversion and one ESA step on each side."""
from __future__ import annotations

import numpy as np
import torch

from esa_inputs import segment_bounds
from oracle import esa_oracle as orc


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Stored numpy tensor (fp32, or uint16 bf16 patterns) -> CUDA tensor of the matching torch dtype."""
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def f64_to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float64 values already representable in the storage type -> CUDA tensor."""
    return to_dev(orc.narrow_to_bits(x, dtype), dtype)


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bf16 numbers around x (x != 0)."""
    e = np.floor(np.log2(np.maximum(np.abs(x), 1e-30)))
    return 2.0 ** (e - 7)


def oracle_step(layer, kc64, t0, eps=0):
    """Oracle result for the step at t0: (O, lse, selected, F, qc)."""
    cfg = layer.cfg
    q_lo = getattr(layer, "q_row0", 0)
    t1 = min(t0 + cfg.l_C, cfg.S)
    q = orc.widen(layer.Q[t0 - q_lo:t1 - q_lo], cfg.dtype)
    K = orc.widen(layer.K[:t1], cfg.dtype)
    V = orc.widen(layer.V[:t1], cfg.dtype)
    qc = orc.compress(q, orc.widen(layer.W_q, cfg.dtype), None, cfg.dtype)
    O, lse, sel, F = orc.esa_step(q, K, V, kc64, qc, t0, cfg.l_I, cfg.l_L, cfg.k, 1.0 / np.sqrt(cfg.d), eps=eps)
    return O, lse, sel, F, qc


def gpu_step(esa, dev, cfg, t0, kc_dev=None, two_calls=False, eps=0, fused=False, indexed=False):
    """The five library calls for the step at t0.  dev: dict of device tensors Q,K,V,W_q,W_k
    (Q may start at row dev['q_row0']).  kc_dev: compressed-key cache [S, d_c]; rows of the current
    tokens are (re)written by esa_compress.  Returns dict of device tensors."""
    q_lo = dev.get("q_row0", 0)
    t1 = min(t0 + cfg.l_C, cfg.S)
    q = dev["Q"][t0 - q_lo:t1 - q_lo]
    if kc_dev is None:
        kc_dev = esa.esa_compress(dev["K"][:t1], dev["W_k"])
    else:
        esa.esa_compress(dev["K"][t0:t1], dev["W_k"], out=kc_dev[t0:t1])
    qc = esa.esa_compress(q, dev["W_q"])
    i_end, l_start = esa.esa_segments(t0, cfg.l_I, cfg.l_L)
    assert (i_end, l_start) == segment_bounds(t0, cfg.l_I, cfg.l_L)
    n_mid = l_start - i_end
    out = {"qc": qc, "kc": kc_dev, "score": None}
    if n_mid > 0 and indexed:
        # the benchmark's default step: score + select as one call, the attention follows the index list itself
        out["score"], idx, _, _ = esa.esa_score_select_gather(qc, kc_dev, i_end, l_start, cfg.k, eps=eps)
        O, lse = esa.esa_attend_indexed(q, dev["K"], dev["V"], t0, cfg.l_I, cfg.l_L, idx, return_lse=True)
        out.update(idx=idx, k_sel=None, v_sel=None, O=O, lse=lse)
        return out
    if n_mid > 0 and fused:
        out["score"], idx, ks, vs = esa.esa_score_select_gather(qc, kc_dev, i_end, l_start, cfg.k, dev["K"], dev["V"], eps=eps)
    elif n_mid > 0:
        if n_mid > cfg.k:
            out["score"] = esa.esa_score(qc, kc_dev, i_end, l_start, eps=eps)
            idx = esa.esa_select_topk(out["score"], cfg.k, base=i_end)
        else:
            # k covers the middle segment: every middle token is taken and the scores are never read
            idx = esa.esa_select_topk(torch.empty(n_mid, dtype=torch.float32, device="cuda"), cfg.k, base=i_end)
        ks, vs = esa.esa_gather_kv(dev["K"], dev["V"], idx)
    else:
        idx = torch.empty(0, dtype=torch.int32, device="cuda")
        ks = vs = None
    if two_calls:
        esa.esa_attend_local(q, dev["K"], dev["V"], t0, cfg.l_I, cfg.l_L)
        O, lse = esa.esa_attend_finish(q, dev["K"], dev["V"], t0, cfg.l_I, cfg.l_L, ks, vs, return_lse=True)
    else:
        O, lse = esa.esa_attend(q, dev["K"], dev["V"], t0, cfg.l_I, cfg.l_L, ks, vs, return_lse=True)
    out.update(idx=idx, k_sel=ks, v_sel=vs, O=O, lse=lse)
    return out


def layer_to_dev(layer):
    cfg = layer.cfg
    d = {n: to_dev(getattr(layer, n), cfg.dtype) for n in ("Q", "K", "V", "W_q", "W_k")}
    d["q_row0"] = getattr(layer, "q_row0", 0)
    return d


def pack_layer_weights(esa, dev):
    """Switch a device layer to packed compression weights (the layout the benchmark uses)."""
    dev["W_q"] = esa.esa_pack_weights(dev["W_q"])
    dev["W_k"] = esa.esa_pack_weights(dev["W_k"])
    return dev
