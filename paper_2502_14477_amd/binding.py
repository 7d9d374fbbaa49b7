"""ctypes binding over libesa.so: argument marshalling only.

Every function has the name and meaning of its C entry point (include/esa.h).  Tensors are
torch CUDA tensors (torch provides device memory and the current stream, nothing else); a
leading batch dimension is optional.  Outputs and workspaces are torch allocations made here.
Nothing in this module computes: with the library missing, import fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

ESA_F32, ESA_BF16 = 0, 1
ESA_W_ROWMAJOR, ESA_W_PACKED = 0, 1
_PKG = os.path.dirname(os.path.abspath(__file__))


class EsaError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("libesa error %d: %s" % (code, text))
        self.code = code


def lib_path() -> str:
    return os.path.join(_PKG, "libesa.so")


def _load() -> ctypes.CDLL:
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(
            "%s is missing: build it with `python -m paper_2502_14477_amd.build` "
            "(there is no fallback path)" % path)
    L = ctypes.CDLL(path)
    i32, i64, vp, sz, f32 = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
    L.esa_version.restype = i32
    L.esa_version.argtypes = []
    L.esa_last_error.restype = ctypes.c_char_p
    L.esa_last_error.argtypes = []
    L.esa_segments.restype = i32
    L.esa_segments.argtypes = [i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.esa_compress.restype = i32
    L.esa_pack_weights.restype = i32
    L.esa_pack_weights.argtypes = [vp, i64, i32, i32, vp, vp]
    L.esa_compress.argtypes = [vp, i64, i64, i64, vp, i32, vp, i32, vp, i64, i32, i32, i64, i64, vp]
    L.esa_compress_qk.restype = i32
    L.esa_compress_qk.argtypes = [vp, i64, i64, vp, vp, vp, i64, i64, i64, vp, i64, i64, vp, vp, vp, i64, i64, i64,
                                  i64, i32, i32, i32, i32, vp]
    L.esa_score_workspace_bytes.restype = sz
    L.esa_score_workspace_bytes.argtypes = [i32, i64, i32, i32]
    L.esa_score.restype = i32
    L.esa_score.argtypes = [vp, i32, vp, i64, i64, i32, i32, vp, i32, i32, i64, i64, i64, vp, sz, vp]
    L.esa_select_topk_workspace_bytes.restype = sz
    L.esa_select_topk_workspace_bytes.argtypes = [i64, i32, i32]
    L.esa_select_topk.restype = i32
    L.esa_select_topk.argtypes = [vp, i64, i32, i64, vp, i32, i64, i64, vp, sz, vp]
    L.esa_score_select_gather_workspace_bytes.restype = sz
    L.esa_score_select_gather_workspace_bytes.argtypes = [i32, i64, i32, i32, i32]
    L.esa_score_select_gather.restype = i32
    L.esa_score_select_gather.argtypes = [vp, i32, vp, i64, i64, i32, i32, i32, vp, vp, vp, vp, i64, i32, i32, vp, vp, i32, i32,
                                          i64, i64, i64, i64, i64, i64, vp, sz, vp]
    L.esa_select_topk_static_capacity.restype = sz
    L.esa_select_topk_static_capacity.argtypes = []
    L.esa_select_topk_static_prepare.restype = i32
    L.esa_select_topk_static_prepare.argtypes = []
    L.esa_select_topk_static.restype = i32
    L.esa_select_topk_static.argtypes = [vp, i64, i32, i64, vp, i32, i64, i64, vp]
    L.esa_gather_kv.restype = i32
    L.esa_gather_kv.argtypes = [vp, vp, i64, vp, i32, i32, i32, vp, vp, i32, i32, i64, i64, i64, vp]
    L.esa_attend_workspace_bytes.restype = sz
    L.esa_attend_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    L.esa_attend.restype = i32
    L.esa_attend.argtypes = [vp, i32, i32, i32, i32, vp, vp, i64, i64, i64, i64, vp, vp, i32, f32, vp, vp,
                             i32, i32, i64, i64, i64, i64, vp, sz, vp]
    L.esa_attend_indexed_workspace_bytes.restype = sz
    L.esa_attend_indexed_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32, i32]
    L.esa_attend_indexed.restype = i32
    L.esa_attend_indexed.argtypes = [vp, i32, i32, i32, i32, vp, vp, i64, i64, i64, i64, vp, i32, i64, f32, vp, vp,
                                     i32, i32, i64, i64, i64, vp, sz, vp]
    L.esa_attend_finish.restype = i32
    L.esa_attend_finish.argtypes = [vp, i32, i32, i32, i32, vp, vp, i64, i64, i64, i64, vp, vp, i32, f32, i32, vp, vp,
                                    i32, i32, i64, i64, i64, i64, vp, sz, vp]
    L.esa_attend_local.restype = i32
    L.esa_attend_local.argtypes = [vp, i32, i32, i32, i32, vp, vp, i64, i64, i64, i64, f32, i32, i32, i32, i64, i64,
                                   vp, sz, vp]
    f64 = ctypes.c_double
    L.esa_rope.restype = i32
    L.esa_rope.argtypes = [vp, i64, i32, i32, i64, f64, f64, f64, vp, i64, i32, i32, i64, i64, vp]
    L.esa_attend_reencoded_workspace_bytes.restype = sz
    L.esa_attend_reencoded_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32, i64]
    L.esa_attend_reencoded.restype = i32
    L.esa_attend_reencoded.argtypes = [vp, i32, i32, i32, i32, vp, vp, i64, i64, i64, i64, vp, vp, i32, f32, f64, f64,
                                       vp, vp, i32, i32, i64, i64, i64, i64, vp, sz, vp]
    return L


lib = _load()

EXPORTS = ("esa_version", "esa_last_error", "esa_segments", "esa_pack_weights", "esa_compress", "esa_score_workspace_bytes",
           "esa_score", "esa_select_topk_workspace_bytes", "esa_select_topk", "esa_gather_kv",
           "esa_attend_workspace_bytes", "esa_attend", "esa_attend_local", "esa_attend_finish",
           "esa_attend_indexed_workspace_bytes", "esa_attend_indexed", "esa_rope",
           "esa_attend_reencoded_workspace_bytes", "esa_attend_reencoded", "esa_compress_qk",
           "esa_select_topk_static_capacity", "esa_select_topk_static_prepare", "esa_select_topk_static",
           "esa_score_select_gather_workspace_bytes", "esa_score_select_gather")


def _check(code: int) -> None:
    if code != 0:
        raise EsaError(code, lib.esa_last_error().decode())


def _dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return ESA_F32
    if t.dtype == torch.bfloat16:
        return ESA_BF16
    raise EsaError(-2, "unsupported torch dtype %s" % t.dtype)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


_hip = None


def _cache_ptr(t: torch.Tensor) -> int:
    """Device address of a KV cache: a GPU tensor, or pinned host memory (the KV cache offloaded to the
    host as in Appendix B; the gather kernel then fetches the selected rows over the host link)."""
    if t.is_cuda:
        return t.data_ptr()
    if not t.is_pinned():
        raise ValueError("a KV cache in host memory must be pinned (torch's pin_memory), pageable memory is not "
                         "addressable by the GPU")
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipHostGetDevicePointer.restype = ctypes.c_int
        _hip.hipHostGetDevicePointer.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, ctypes.c_uint]
    dptr = ctypes.c_void_p()
    err = _hip.hipHostGetDevicePointer(ctypes.byref(dptr), ctypes.c_void_p(t.data_ptr()), 0)
    if err != 0 or not dptr.value:
        raise EsaError(-4, "hipHostGetDevicePointer failed (%d): the pinned cache is not mapped into the GPU" % err)
    return dptr.value


_ws_cache = {}


def _workspace(nbytes: int, device, tag: str) -> torch.Tensor:
    """A reusable 256-byte aligned scratch tensor per (device, call)."""
    key = (device, tag)
    t = _ws_cache.get(key)
    if t is None or t.numel() < nbytes:
        t = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        assert t.data_ptr() % 256 == 0
        _ws_cache[key] = t
    return t


def _batched(t: torch.Tensor, rank: int) -> Tuple[torch.Tensor, bool]:
    if t.dim() == rank:
        return t.unsqueeze(0), False
    if t.dim() == rank + 1:
        return t, True
    raise EsaError(-1, "expected %d or %d dimensions, got %d" % (rank, rank + 1, t.dim()))


def esa_version() -> int:
    return lib.esa_version()


def esa_segments(t0: int, l_i: int, l_l: int) -> Tuple[int, int]:
    a, b = ctypes.c_int64(), ctypes.c_int64()
    _check(lib.esa_segments(t0, l_i, l_l, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


class PackedWeights:
    """Compression weights in the packed layout [d_c, d_in] (see esa_pack_weights)."""

    def __init__(self, data: torch.Tensor, d_in: int, d_c: int):
        self.data, self.d_in, self.d_c = data, d_in, d_c


def esa_pack_weights(W: torch.Tensor) -> PackedWeights:
    """W [d_in, d_c] -> packed weights; done once per layer."""
    d_in, d_c = W.shape
    assert W.is_contiguous()
    out = torch.empty((d_c, d_in), dtype=W.dtype, device=W.device)
    _check(lib.esa_pack_weights(_ptr(W), d_in, d_c, _dtype(W), _ptr(out), _stream()))
    return PackedWeights(out, d_in, d_c)


def esa_compress(x: torch.Tensor, W, bias: Optional[torch.Tensor] = None,
                 out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x [B?, n_tok, heads, d] or [B?, n_tok, d_in] -> [B?, n_tok, d_c].  W is a [d_in, d_c] tensor or
    PackedWeights.  `out` may be a row-strided view (e.g. rows t0.. of the compressed-key cache)."""
    if isinstance(W, PackedWeights):
        layout, d_in, d_c, W = ESA_W_PACKED, W.d_in, W.d_c, W.data
    else:
        layout = ESA_W_ROWMAJOR
        d_in, d_c = W.shape
    if x.shape[-1] != d_in:
        x = x.flatten(-2)
    xb, had_batch = _batched(x, 2)
    B, n_tok = xb.shape[0], xb.shape[1]
    assert xb.shape[2] == d_in and xb.stride(2) == 1 and W.is_contiguous()
    if out is None:
        ob = torch.empty((B, n_tok, d_c), dtype=x.dtype, device=x.device)
    else:
        ob, _ = _batched(out, 2)
        assert ob.shape == (B, n_tok, d_c) and ob.stride(2) == 1 and ob.dtype == x.dtype
    _check(lib.esa_compress(_ptr(xb), n_tok, d_in, xb.stride(1), _ptr(W), layout, _ptr(bias), d_c, _ptr(ob), ob.stride(1),
                            _dtype(x), B, xb.stride(0), ob.stride(0), _stream()))
    return ob if had_batch else ob[0]


def esa_compress_qk(xq: torch.Tensor, Wq, xk: torch.Tensor, Wk, bias_q: Optional[torch.Tensor] = None,
                    bias_k: Optional[torch.Tensor] = None, out_q: Optional[torch.Tensor] = None,
                    out_k: Optional[torch.Tensor] = None):
    """Both compressions of Eq. 5 in one call (shapes per tensor as esa_compress; `out_k` is typically the rows
    t0.. of the compressed-key cache).  Returns (q', k')."""
    packed = isinstance(Wq, PackedWeights)
    assert packed == isinstance(Wk, PackedWeights), "both weight matrices in the same layout"
    if packed:
        layout, (dq, dc, wq), (dk, dck, wk) = ESA_W_PACKED, (Wq.d_in, Wq.d_c, Wq.data), (Wk.d_in, Wk.d_c, Wk.data)
    else:
        layout, (dq, dc, wq), (dk, dck, wk) = ESA_W_ROWMAJOR, (*Wq.shape, Wq), (*Wk.shape, Wk)
    assert dc == dck and wq.is_contiguous() and wk.is_contiguous()

    def prep(x, d_in, out):
        if x.shape[-1] != d_in:
            x = x.flatten(-2)
        xb, had_batch = _batched(x, 2)
        assert xb.shape[2] == d_in and xb.stride(2) == 1
        if out is None:
            ob = torch.empty((xb.shape[0], xb.shape[1], dc), dtype=x.dtype, device=x.device)
        else:
            ob, _ = _batched(out, 2)
            assert ob.shape == (xb.shape[0], xb.shape[1], dc) and ob.stride(2) == 1 and ob.dtype == x.dtype
        return xb, ob, had_batch

    xqb, oq, had_batch = prep(xq, dq, out_q)
    xkb, ok, _ = prep(xk, dk, out_k)
    assert xqb.shape[:2] == xkb.shape[:2] and xqb.dtype == xkb.dtype
    B, n_tok = xqb.shape[0], xqb.shape[1]
    _check(lib.esa_compress_qk(_ptr(xqb), dq, xqb.stride(1), _ptr(wq), _ptr(bias_q), _ptr(oq), oq.stride(1), xqb.stride(0),
                               oq.stride(0), _ptr(xkb), dk, xkb.stride(1), _ptr(wk), _ptr(bias_k), _ptr(ok), ok.stride(1),
                               xkb.stride(0), ok.stride(0), n_tok, dc, layout, _dtype(xq), B, _stream()))
    return (oq, ok) if had_batch else (oq[0], ok[0])


def esa_score(qc: torch.Tensor, kc_cache: torch.Tensor, m_lo: int, m_hi: int, eps: int = 0,
              out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """qc [B?, l_c, d_c], kc_cache [B?, S, d_c] -> score [B?, m_hi-m_lo] fp32."""
    qb, had_batch = _batched(qc, 2)
    kb, _ = _batched(kc_cache, 2)
    B, l_c, d_c = qb.shape
    assert kb.shape[0] == B and kb.shape[2] == d_c and qb.stride(2) == 1 and kb.stride(2) == 1
    assert qb.stride(1) == d_c and kb.stride(1) == d_c and kb.dtype == qb.dtype
    n = m_hi - m_lo
    if out is None:
        sb = torch.empty((B, max(n, 0)), dtype=torch.float32, device=qc.device)
    else:
        sb, _ = _batched(out, 1)
    nbytes = lib.esa_score_workspace_bytes(l_c, n, eps, B)
    ws = _workspace(nbytes, qc.device, "score")
    _check(lib.esa_score(_ptr(qb), l_c, _ptr(kb), m_lo, m_hi, d_c, eps, _ptr(sb), _dtype(qc), B, qb.stride(0),
                         kb.stride(0), sb.stride(0) if B > 1 else max(n, 1), _ptr(ws), ws.numel(), _stream()))
    return sb if had_batch else sb[0]


def esa_select_topk(score: torch.Tensor, k: int, base: int = 0) -> torch.Tensor:
    """score [B?, n] fp32 -> idx [B?, min(k, n)] int32, ascending absolute positions."""
    sb, had_batch = _batched(score, 1)
    B, n = sb.shape
    assert sb.dtype == torch.float32 and (n == 0 or sb.stride(1) == 1)
    k_eff = min(k, n)
    idx = torch.empty((B, k_eff), dtype=torch.int32, device=score.device)
    nbytes = lib.esa_select_topk_workspace_bytes(n, k, B)
    ws = _workspace(nbytes, score.device, "topk")
    _check(lib.esa_select_topk(_ptr(sb), n, k, base, _ptr(idx), B, sb.stride(0) if B > 1 else max(n, 1),
                               max(k_eff, 1), _ptr(ws), ws.numel(), _stream()))
    return idx if had_batch else idx[0]


def esa_score_select_gather(qc: torch.Tensor, kc_cache: torch.Tensor, m_lo: int, m_hi: int, k: int,
                            k_cache: Optional[torch.Tensor] = None, v_cache: Optional[torch.Tensor] = None, eps: int = 0):
    """esa_score + esa_select_topk (+ esa_gather_kv when the caches are given) in one call.
    Returns (score or None, idx, k_sel, v_sel); k_sel / v_sel are None without caches."""
    qb, had_batch = _batched(qc, 2)
    kb, _ = _batched(kc_cache, 2)
    B, l_c, d_c = qb.shape
    assert kb.shape[0] == B and kb.shape[2] == d_c and qb.stride(2) == 1 and kb.stride(2) == 1
    assert qb.stride(1) == d_c and kb.stride(1) == d_c and kb.dtype == qb.dtype
    n = m_hi - m_lo
    k_eff = min(k, max(n, 0))
    score = torch.empty((B, max(n, 0)), dtype=torch.float32, device=qc.device) if n > k else None
    idx = torch.empty((B, k_eff), dtype=torch.int32, device=qc.device)
    ks = vs = kcb = vcb = None
    tok_stride = h_kv = d = cache_bs = sel_bs = 0
    if k_cache is not None:
        kcb, _ = _batched(k_cache, 3)
        vcb, _ = _batched(v_cache, 3)
        _, S, h_kv, d = kcb.shape
        assert vcb.shape == kcb.shape and vcb.stride() == kcb.stride() and kcb.stride(3) == 1 and kcb.stride(2) == d
        assert kcb.shape[0] == B and kcb.is_cuda
        ks = torch.empty((B, k_eff, h_kv, d), dtype=k_cache.dtype, device=qc.device)
        vs = torch.empty_like(ks)
        tok_stride, cache_bs, sel_bs = kcb.stride(1), kcb.stride(0), k_eff * h_kv * d
    nbytes = lib.esa_score_select_gather_workspace_bytes(l_c, n, eps, k, B)
    ws = _workspace(nbytes, qc.device, "score_select")
    _check(lib.esa_score_select_gather(_ptr(qb), l_c, _ptr(kb), m_lo, m_hi, d_c, eps, k, _ptr(score), _ptr(idx), _ptr(kcb), _ptr(vcb),
                                       tok_stride, h_kv, d, _ptr(ks), _ptr(vs), _dtype(qc), B, qb.stride(0), kb.stride(0),
                                       max(n, 1), max(k_eff, 1), cache_bs, sel_bs, _ptr(ws), ws.numel(), _stream()))
    if not had_batch:
        score = None if score is None else score[0]
        idx = idx[0]
        ks = None if ks is None else ks[0]
        vs = None if vs is None else vs[0]
    return score, idx, ks, vs


def esa_select_topk_static_capacity() -> int:
    return lib.esa_select_topk_static_capacity()


def esa_select_topk_static_prepare() -> None:
    _check(lib.esa_select_topk_static_prepare())


def esa_select_topk_static(score: torch.Tensor, k: int, base: int = 0, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """esa_select_topk on the library's own scratch.  With `out` given ([B?, min(k, n)] int32) this
    function allocates nothing either."""
    sb, had_batch = _batched(score, 1)
    B, n = sb.shape
    assert sb.dtype == torch.float32 and (n == 0 or sb.stride(1) == 1)
    k_eff = min(k, n)
    if out is None:
        idx = torch.empty((B, k_eff), dtype=torch.int32, device=score.device)
    else:
        idx, _ = _batched(out, 1)
        assert idx.dtype == torch.int32 and idx.shape == (B, k_eff) and idx.is_contiguous()
    _check(lib.esa_select_topk_static(_ptr(sb), n, k, base, _ptr(idx), B, sb.stride(0) if B > 1 else max(n, 1),
                                      max(k_eff, 1), _stream()))
    return idx if had_batch else idx[0]


def esa_gather_kv(k_cache: torch.Tensor, v_cache: torch.Tensor, idx: torch.Tensor):
    """caches [B?, S, h_kv, d] (GPU memory, or pinned host memory for an offloaded cache), idx [B?, n_sel]
    int32 on the GPU -> (k_sel, v_sel) [B?, n_sel, h_kv, d] on the GPU."""
    kb, had_batch = _batched(k_cache, 3)
    vb, _ = _batched(v_cache, 3)
    ib, _ = _batched(idx, 1)
    B, S, h_kv, d = kb.shape
    n_sel = ib.shape[1]
    assert vb.shape == kb.shape and vb.stride() == kb.stride() and kb.stride(3) == 1 and kb.stride(2) == d
    assert ib.dtype == torch.int32 and ib.shape[0] == B and (n_sel == 0 or ib.stride(1) == 1)
    ks = torch.empty((B, n_sel, h_kv, d), dtype=k_cache.dtype, device=idx.device)
    vs = torch.empty_like(ks)
    _check(lib.esa_gather_kv(_cache_ptr(kb), _cache_ptr(vb), kb.stride(1), _ptr(ib), n_sel, h_kv, d, _ptr(ks), _ptr(vs),
                             _dtype(k_cache), B, kb.stride(0), ib.stride(0) if B > 1 else max(n_sel, 1),
                             n_sel * h_kv * d, _stream()))
    return (ks, vs) if had_batch else (ks[0], vs[0])


ESA_SPLIT_I_EARLY, ESA_SPLIT_ALGORITHM1 = 0, 1


def esa_attend_indexed(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, t0: int, l_i: int, l_l: int,
                       idx: Optional[torch.Tensor], scale: Optional[float] = None, return_lse: bool = False):
    """esa_gather_kv + esa_attend in one call: idx [B?, n_sel] int32 positions of the selected tokens."""
    qb, had_batch = _batched(q, 3)
    kb, _ = _batched(k_cache, 3)
    vb, _ = _batched(v_cache, 3)
    B, l_c, h, d = qb.shape
    h_kv = kb.shape[2]
    assert qb.is_contiguous() and kb.stride(3) == 1 and kb.stride(2) == d and vb.stride() == kb.stride()
    assert kb.shape[1] >= t0 + l_c, "the cache must already hold the current tokens"
    n_sel, idx_bs, ib = 0, 0, None
    if idx is not None and idx.numel() > 0:
        ib, _ = _batched(idx, 1)
        assert ib.dtype == torch.int32 and ib.stride(1) == 1 and ib.shape[0] == B
        n_sel, idx_bs = ib.shape[1], ib.stride(0)
    out = torch.empty_like(qb)
    lse = torch.empty((B, l_c, h), dtype=torch.float32, device=q.device) if return_lse else None
    scale = float(d) ** -0.5 if scale is None else float(scale)
    nbytes = lib.esa_attend_indexed_workspace_bytes(l_c, h, h_kv, d, _dtype(q), B, n_sel)
    ws = _workspace(nbytes, q.device, "attend")
    _check(lib.esa_attend_indexed(_ptr(qb), l_c, h, h_kv, d, _ptr(kb), _ptr(vb), kb.stride(1), t0, l_i, l_l, _ptr(ib),
                                  n_sel, idx_bs, scale, _ptr(out), _ptr(lse), _dtype(q), B, qb.stride(0), kb.stride(0),
                                  out.stride(0), _ptr(ws), ws.numel(), _stream()))
    if not had_batch:
        out = out[0]
        lse = None if lse is None else lse[0]
    return (out, lse) if return_lse else out


def esa_rope(x: torch.Tensor, pos0: float, pos_step: float, base: float, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Rotary encoding of x [B?, n_tok, heads, d]: row i goes to position pos0 + i*pos_step.  `out` may be
    x itself (in place) or a view with the same shape (e.g. rows of a cache)."""
    xb, had_batch = _batched(x, 3)
    B, n_tok, heads, d = xb.shape
    if out is None:
        ob = torch.empty((B, n_tok, heads, d), dtype=x.dtype, device=x.device)
        out = ob if had_batch else ob[0]
    else:
        ob, _ = _batched(out, 3)
        assert ob.shape == xb.shape and ob.dtype == xb.dtype
    for t in (xb, ob):
        assert t.stride(3) == 1 and t.stride(2) == d
    _check(lib.esa_rope(_ptr(xb), n_tok, heads, d, xb.stride(1), float(pos0), float(pos_step), float(base), _ptr(ob),
                        ob.stride(1), _dtype(x), B, xb.stride(0), ob.stride(0), _stream()))
    return out


def esa_attend_reencoded(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, t0: int, l_i: int, l_l: int,
                         k_sel: Optional[torch.Tensor], v_sel: Optional[torch.Tensor], w: float, rope_base: float,
                         scale: Optional[float] = None, return_lse: bool = False):
    """Section 3.2's attention on un-encoded q, key cache and gathered keys (shapes as esa_attend)."""
    qb, had_batch = _batched(q, 3)
    kb, _ = _batched(k_cache, 3)
    vb, _ = _batched(v_cache, 3)
    B, l_c, h, d = qb.shape
    h_kv = kb.shape[2]
    assert qb.is_contiguous() and kb.stride(3) == 1 and kb.stride(2) == d and vb.stride() == kb.stride()
    assert kb.shape[1] >= t0 + l_c, "the cache must already hold the current tokens"
    n_sel, sel_bs, ksb, vsb = 0, 0, None, None
    if k_sel is not None and k_sel.numel() > 0:
        ksb, _ = _batched(k_sel, 3)
        vsb, _ = _batched(v_sel, 3)
        assert ksb.is_contiguous() and vsb.is_contiguous() and ksb.shape == vsb.shape
        n_sel, sel_bs = ksb.shape[1], ksb.stride(0)
    out = torch.empty_like(qb)
    lse = torch.empty((B, l_c, h), dtype=torch.float32, device=q.device) if return_lse else None
    scale = float(d) ** -0.5 if scale is None else float(scale)
    nbytes = lib.esa_attend_reencoded_workspace_bytes(l_c, h, h_kv, d, _dtype(q), B, l_l)
    ws = _workspace(nbytes, q.device, "attend")
    _check(lib.esa_attend_reencoded(_ptr(qb), l_c, h, h_kv, d, _ptr(kb), _ptr(vb), kb.stride(1), t0, l_i, l_l, _ptr(ksb),
                                    _ptr(vsb), n_sel, scale, float(w), float(rope_base), _ptr(out), _ptr(lse), _dtype(q), B,
                                    qb.stride(0), kb.stride(0), sel_bs, out.stride(0), _ptr(ws), ws.numel(), _stream()))
    if not had_batch:
        out = out[0]
        lse = None if lse is None else lse[0]
    return (out, lse) if return_lse else out


def esa_attend_local(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, t0: int, l_i: int, l_l: int,
                     scale: Optional[float] = None, split: int = ESA_SPLIT_I_EARLY) -> None:
    """First half of the two-call form of esa_attend: the keys that do not depend on the selection
    ([I, L, C], or [L, C] with split = ESA_SPLIT_ALGORITHM1).  Leaves partial results in the attend
    workspace for esa_attend_finish (same sizes and split, ordered after it)."""
    qb, _ = _batched(q, 3)
    kb, _ = _batched(k_cache, 3)
    vb, _ = _batched(v_cache, 3)
    B, l_c, h, d = qb.shape
    h_kv = kb.shape[2]
    assert qb.is_contiguous() and kb.stride(3) == 1 and kb.stride(2) == d and vb.stride() == kb.stride()
    assert kb.shape[1] >= t0 + l_c, "the cache must already hold the current tokens"
    scale = float(d) ** -0.5 if scale is None else float(scale)
    nbytes = lib.esa_attend_workspace_bytes(l_c, h, h_kv, d, _dtype(q), B)
    ws = _workspace(nbytes, q.device, "attend")
    _check(lib.esa_attend_local(_ptr(qb), l_c, h, h_kv, d, _ptr(kb), _ptr(vb), kb.stride(1), t0, l_i, l_l, scale, split,
                                _dtype(q), B, qb.stride(0), kb.stride(0), _ptr(ws), ws.numel(), _stream()))


def esa_attend_finish(q, k_cache, v_cache, t0, l_i, l_l, k_sel, v_sel, scale=None, return_lse=False,
                      split: int = ESA_SPLIT_I_EARLY):
    """Second half of the two-call form: the selected keys (with the initial tokens if split =
    ESA_SPLIT_ALGORITHM1), then the merge.  Arguments as esa_attend."""
    return esa_attend(q, k_cache, v_cache, t0, l_i, l_l, k_sel, v_sel, scale, return_lse, _split=split)


def esa_attend(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, t0: int, l_i: int, l_l: int,
               k_sel: Optional[torch.Tensor], v_sel: Optional[torch.Tensor], scale: Optional[float] = None,
               return_lse: bool = False, _split: Optional[int] = None):
    """q [B?, l_c, h, d]; caches [B?, S, h_kv, d] holding the current tokens at rows t0..; gathered
    buffers [B?, n_sel, h_kv, d] -> out [B?, l_c, h, d] (and lse [B?, l_c, h] fp32)."""
    qb, had_batch = _batched(q, 3)
    kb, _ = _batched(k_cache, 3)
    vb, _ = _batched(v_cache, 3)
    B, l_c, h, d = qb.shape
    h_kv = kb.shape[2]
    assert qb.is_contiguous() and kb.stride(3) == 1 and kb.stride(2) == d and vb.stride() == kb.stride()
    assert kb.shape[1] >= t0 + l_c, "the cache must already hold the current tokens"
    n_sel = 0
    sel_bs = 0
    ksb = vsb = None
    if k_sel is not None and k_sel.numel() > 0:
        ksb, _ = _batched(k_sel, 3)
        vsb, _ = _batched(v_sel, 3)
        assert ksb.is_contiguous() and vsb.is_contiguous() and ksb.shape == vsb.shape
        n_sel = ksb.shape[1]
        sel_bs = ksb.stride(0)
    out = torch.empty_like(qb)
    lse = torch.empty((B, l_c, h), dtype=torch.float32, device=q.device) if return_lse else None
    scale = float(d) ** -0.5 if scale is None else float(scale)
    nbytes = lib.esa_attend_workspace_bytes(l_c, h, h_kv, d, _dtype(q), B)
    ws = _workspace(nbytes, q.device, "attend")
    if _split is None:
        _check(lib.esa_attend(_ptr(qb), l_c, h, h_kv, d, _ptr(kb), _ptr(vb), kb.stride(1), t0, l_i, l_l, _ptr(ksb),
                              _ptr(vsb), n_sel, scale, _ptr(out), _ptr(lse), _dtype(q), B, qb.stride(0), kb.stride(0),
                              sel_bs, out.stride(0), _ptr(ws), ws.numel(), _stream()))
    else:
        _check(lib.esa_attend_finish(_ptr(qb), l_c, h, h_kv, d, _ptr(kb), _ptr(vb), kb.stride(1), t0, l_i, l_l,
                                     _ptr(ksb), _ptr(vsb), n_sel, scale, _split, _ptr(out), _ptr(lse), _dtype(q), B,
                                     qb.stride(0), kb.stride(0), sel_bs, out.stride(0), _ptr(ws), ws.numel(), _stream()))
    if not had_batch:
        out = out[0]
        lse = None if lse is None else lse[0]
    return (out, lse) if return_lse else out
