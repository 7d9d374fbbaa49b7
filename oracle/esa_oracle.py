"""CPU oracle for the Efficient Selective Attention (ESA) step.  TEST INFRASTRUCTURE ONLY.

A plain, slow float64 numpy implementation of what one ESA step computes, written
from the paper's definitions.  It exists so that the HIP library can be checked
element by element; it shares no code with that library and must never be imported
by it.  Only tests, the smoke check and the benchmark's CPU-baseline leg call it.

Every function cites the passage it follows.  Inputs are float64 arrays holding the
exactly widened stored values (fp32 or bf16); arithmetic is float64 throughout.
The only rounding the oracle performs on purpose is `round_to_storage`, applied to
the compressed queries/keys because the compressed-key cache is kept in the
storage type (Section 3.1, "cached and reused"; Section 3.3, cache analysis).

Pins (tests/test_oracle_*.py): full-causal-attention reduction when k covers the
middle tokens (Eq. 1 vs Eq. 10), chunk-size independence, probability rows summing to
one, the log-sum-exp merge identity of Algorithm 1, permutation invariance of the
selected set, the one-key case, identity-weight compression, Eq. 4 invariants,
the head-concatenation identity behind Eq. 3, brute-force sorting for Eq. 2, a
clamped maximum filter for Eq. 8, and the closed forms of Eq. 9 and of the cache
overhead.  Selection *quality* (how well compressed top-k approximates
full-dimension top-k) needs trained weights and model activations: parity unpinned,
out of scope.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- storage precision
def widen(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored tensor (fp32 array, or uint16 bf16 bit patterns) -> exact float64."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        # a bf16 pattern is the top 16 bits of an fp32 pattern
        return (np.asarray(x, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the storage type (nearest, ties to even); result stays float64."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype == "bf16":
        # bf16 keeps 7 of the 52 fraction bits: drop 45 with round-to-nearest-even.
        # Valid inside the normal range shared by bf16 and float64, which is asserted.
        nz = x[x != 0.0]
        if nz.size:
            a = np.abs(nz)
            assert a.min() > 1e-30 and a.max() < 1e30, "outside the range this rounding covers"
        u = x.view(np.uint64).copy()
        lsb = (u >> np.uint64(45)) & np.uint64(1)
        u = u + np.uint64((1 << 44) - 1) + lsb
        u &= ~np.uint64((1 << 45) - 1)
        return u.view(np.float64)
    raise ValueError(dtype)


def narrow_to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Already-rounded float64 values -> stored form (fp32 array or uint16 bf16 patterns)."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "bf16":
        return (np.asarray(x, dtype=np.float64).astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- Section 3.1: segments
def segments(t0: int, l_I: int, l_L: int):
    """Preceding tokens [0,t0) -> initial [0,i_end), middle [i_end,l_start), local [l_start,t0).

    Section 3.1: fixed-length initial and local parts, the middle is what lies between.
    Early steps with fewer than l_I + l_L preceding tokens have an empty middle.
    """
    i_end = min(l_I, t0)
    l_start = max(t0 - l_L, i_end)
    return i_end, l_start


# ----------------------------------------------------------------------------- Eq. 5: compression
def compress(x: np.ndarray, W: np.ndarray, bias=None, dtype: str = "f32") -> np.ndarray:
    """q' = f_theta(q): one linear layer on the head-concatenated vector (Eq. 5).

    x [n, heads, d] or [n, heads*d] (concatenation is head-major, Section 3.1), W [heads*d, d_c].
    The result is rounded to the storage type of the compressed cache.
    """
    x2 = np.asarray(x, dtype=np.float64).reshape(x.shape[0], -1)
    y = x2 @ np.asarray(W, dtype=np.float64)
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return round_to_storage(y, dtype)


# ----------------------------------------------------------------------------- Eq. 6 / Eq. 4: scores
def pair_scores(qc: np.ndarray, kc: np.ndarray) -> np.ndarray:
    """f_s(m;c) ~= q'_c . k'_m for every current token c and middle token m (Eq. 6). -> [l_C, N]"""
    return np.asarray(qc, dtype=np.float64) @ np.asarray(kc, dtype=np.float64).T


def importance(qc: np.ndarray, kc_mid: np.ndarray) -> np.ndarray:
    """F_s(m;C) = max_c ( f_s(m;c) - max_{m'} f_s(m';c) ) over the middle tokens (Eq. 4). -> [N]"""
    s = pair_scores(qc, kc_mid)
    mu = s.max(axis=1, keepdims=True)          # per current token, its best middle token
    return (s - mu).max(axis=0)


def proximity(score: np.ndarray, eps: int) -> np.ndarray:
    """s'_j = max of s over [j-eps, j+eps] clamped to the middle segment (Eq. 8)."""
    score = np.asarray(score, dtype=np.float64)
    n = score.shape[0]
    out = np.empty_like(score)
    for j in range(n):
        out[j] = score[max(j - eps, 0):min(j + eps, n - 1) + 1].max()
    return out


# ----------------------------------------------------------------------------- Eq. 2: selection
def select_topk(score: np.ndarray, k: int, base: int = 0) -> np.ndarray:
    """M_k = the k middle tokens with the highest score (Eq. 2), as ascending absolute positions.

    The paper is silent on ties; equal scores are resolved towards the lower position.
    If k >= N every middle token is returned (the paper requires k <= l_M).
    """
    score = np.asarray(score, dtype=np.float64)
    n = score.shape[0]
    k_eff = min(int(k), n)
    if k_eff <= 0:
        return np.empty(0, dtype=np.int32)
    order = np.argsort(-score, kind="stable")   # descending score; stable => lower position first
    chosen = np.sort(order[:k_eff])
    return (chosen + base).astype(np.int32)


# ----------------------------------------------------------------------------- gather
def gather_rows(cache: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Full-size keys or values of the selected tokens (Section 1: the attention step uses the
    full-sized keys and values of the selected tokens; Appendix B: only these are fetched)."""
    return np.asarray(cache)[np.asarray(idx, dtype=np.int64)]


# ----------------------------------------------------------------------------- Eq. 1: attention
def attend(q: np.ndarray, K: np.ndarray, V: np.ndarray, t0: int, l_I: int, l_L: int,
           selected: np.ndarray, scale: float, return_probs: bool = False):
    """O = Attn(Q_C, K_[I,M_k,L,C], V_[I,M_k,L,C]) (Eq. 1), softmax with scale, per head.

    q [l_C, H, d] are the current tokens at positions t0..t0+l_C-1; K, V [>=t0+l_C, H_kv, d]
    are the caches including the current tokens.  Query head h uses key/value head
    h // (H / H_kv).  Initial, selected and local tokens are visible to every current token;
    inside C a token sees itself and earlier ones (Algorithm 1: the local call is causal
    with queries aligned to the end of the keys, the global call is not causal).
    Returns O [l_C, H, d] and lse [l_C, H] (natural-log of the softmax normaliser).
    """
    q = np.asarray(q, dtype=np.float64)
    l_C, H, d = q.shape
    H_kv = K.shape[1]
    G = H // H_kv
    i_end, l_start = segments(t0, l_I, l_L)
    pos = np.concatenate([np.arange(0, i_end, dtype=np.int64),
                          np.asarray(selected, dtype=np.int64),
                          np.arange(l_start, t0 + l_C, dtype=np.int64)])
    visible = pos[None, :] <= (t0 + np.arange(l_C, dtype=np.int64))[:, None]   # [l_C, n_keys]
    Ks = np.asarray(K, dtype=np.float64)[pos]
    Vs = np.asarray(V, dtype=np.float64)[pos]
    O = np.empty((l_C, H, d), dtype=np.float64)
    lse = np.empty((l_C, H), dtype=np.float64)
    probs = np.empty((H, l_C, pos.shape[0]), dtype=np.float64) if return_probs else None
    for h in range(H):
        g = h // G
        a = (q[:, h, :] @ Ks[:, g, :].T) * scale
        a = np.where(visible, a, -np.inf)
        amax = a.max(axis=1, keepdims=True)
        e = np.exp(a - amax)
        z = e.sum(axis=1, keepdims=True)
        p = e / z
        O[:, h, :] = p @ Vs[:, g, :]
        lse[:, h] = (amax + np.log(z))[:, 0]
        if return_probs:
            probs[h] = p
    if return_probs:
        return O, lse, probs, pos
    return O, lse


def merge_partial_attention(outs, lses):
    """Algorithm 1: combine attentions over disjoint key sets with weights exp(lse_i)/sum exp(lse).

    Evaluated with the maximum subtracted before exponentiation.
    """
    lses = np.stack(lses)                        # [parts, l_C, H]
    top = lses.max(axis=0, keepdims=True)
    w = np.exp(lses - top)
    share = w / w.sum(axis=0, keepdims=True)     # each part's share of the joint normaliser
    return sum(s[..., None] * o for s, o in zip(share, outs))


# ----------------------------------------------------------------------------- Section 3.2: position encoding
def rope(x: np.ndarray, positions, base: float) -> np.ndarray:
    """Rotary position encoding of x [n, heads, d] at the given positions [n] (rotate-half form:
    element i of the first half pairs with element i of the second half, angle pos * base^(-2i/d)).
    Section 3.2 assumes a model "that utilizes RoPE"; position 0 leaves x unchanged.
    """
    x = np.asarray(x, dtype=np.float64)
    n, _, d = x.shape
    half = d // 2
    freq = np.asarray(base, dtype=np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(positions, dtype=np.float64).reshape(n, 1) * freq[None, :]
    c, s_ = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[:, :, :half], x[:, :, half:]
    return np.concatenate([x1 * c - x2 * s_, x2 * c + x1 * s_], axis=2)


def attend_two_encodings(q_l, q_g, K_l, K_g, V, t0: int, l_I: int, l_L: int, selected, scale: float):
    """Eq. 1 with Algorithm 1's two groups of keys seen through their own encodings.

    Logits of the local group (L and C, causal inside C) are q_l . K_l, logits of the global group
    (I and the selected middle tokens, all visible) are q_g . K_g; one softmax over the union
    ("we fuse the two categories of attention based on their respective weights", Section 3.2),
    values shared.  q_* [l_C, H, d]; K_*, V [>= t0 + l_C, H_kv, d] indexed by absolute position.
    Returns O [l_C, H, d] and lse [l_C, H].
    """
    q_l, q_g = np.asarray(q_l, dtype=np.float64), np.asarray(q_g, dtype=np.float64)
    K_l, K_g, V = (np.asarray(a, dtype=np.float64) for a in (K_l, K_g, V))
    l_C, H, d = q_l.shape
    G = H // K_l.shape[1]
    i_end, l_start = segments(t0, l_I, l_L)
    pos_g = np.concatenate([np.arange(0, i_end, dtype=np.int64), np.asarray(selected, dtype=np.int64)])
    pos_l = np.arange(l_start, t0 + l_C, dtype=np.int64)
    visible_l = pos_l[None, :] <= (t0 + np.arange(l_C, dtype=np.int64))[:, None]
    O = np.empty((l_C, H, d), dtype=np.float64)
    lse = np.empty((l_C, H), dtype=np.float64)
    for h in range(H):
        g = h // G
        a_g = (q_g[:, h, :] @ K_g[pos_g, g, :].T) * scale
        a_l = np.where(visible_l, (q_l[:, h, :] @ K_l[pos_l, g, :].T) * scale, -np.inf)
        a = np.concatenate([a_g, a_l], axis=1)
        amax = a.max(axis=1, keepdims=True)
        e = np.exp(a - amax)
        z = e.sum(axis=1, keepdims=True)
        O[:, h, :] = (e / z) @ np.concatenate([V[pos_g, g, :], V[pos_l, g, :]], axis=0)
        lse[:, h] = (amax + np.log(z))[:, 0]
    return O, lse


def attend_reencoded(q_raw, K_raw, V, t0: int, l_I: int, l_L: int, selected, scale: float, w: float, base: float):
    """Section 3.2 on un-encoded queries and keys: local keys at positions 0 .. n_L + l_C - 1 and local
    queries at n_L .. n_L + l_C - 1 (n_L = number of local tokens actually present), global queries
    all at position w, initial and selected keys at position 0."""
    q_raw, K_raw = np.asarray(q_raw, dtype=np.float64), np.asarray(K_raw, dtype=np.float64)
    l_C = q_raw.shape[0]
    i_end, l_start = segments(t0, l_I, l_L)
    n_L = t0 - l_start
    K_l = np.zeros_like(K_raw)
    K_l[l_start:t0 + l_C] = rope(K_raw[l_start:t0 + l_C], np.arange(n_L + l_C), base)
    q_l = rope(q_raw, n_L + np.arange(l_C), base)
    q_g = rope(q_raw, np.full(l_C, w, dtype=np.float64), base)
    return attend_two_encodings(q_l, q_g, K_l, K_raw, V, t0, l_I, l_L, selected, scale)


# ----------------------------------------------------------------------------- Eq. 10: plain attention
def full_causal_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """Ordinary causal attention of all S tokens (Eq. 10 applied at every step); S small."""
    from scipy.special import softmax
    Q = np.asarray(Q, dtype=np.float64)
    S, H, d = Q.shape
    G = H // K.shape[1]
    mask = np.tril(np.ones((S, S), dtype=bool))
    out = np.empty_like(Q)
    for h in range(H):
        logits = scale * np.einsum("sd,td->st", Q[:, h], np.asarray(K, dtype=np.float64)[:, h // G])
        logits[~mask] = -np.inf
        out[:, h] = softmax(logits, axis=1) @ np.asarray(V, dtype=np.float64)[:, h // G]
    return out


# ----------------------------------------------------------------------------- one step, whole sequence
def esa_step(q_chunk, K, V, kc_cache, qc_chunk, t0, l_I, l_L, k, scale, eps: int = 0):
    """One step for the current tokens at t0: score the middle tokens, select, attend.

    kc_cache [>=l_start, d_c] holds the stored compressed keys, qc_chunk [l_C, d_c] the
    compressed queries.  Returns (O, lse, selected positions, F or None).
    """
    l_C = q_chunk.shape[0]
    i_end, l_start = segments(t0, l_I, l_L)
    n_mid = l_start - i_end
    F = None
    if n_mid <= 0:
        sel = np.empty(0, dtype=np.int32)
    elif n_mid <= k:
        sel = np.arange(i_end, l_start, dtype=np.int32)     # k covers the middle: keep all of it
    else:
        F = importance(qc_chunk, kc_cache[i_end:l_start])
        Fp = proximity(F, eps) if eps > 0 else F
        sel = select_topk(Fp, k, base=i_end)
    O, lse = attend(q_chunk, K, V, t0, l_I, l_L, sel, scale)
    return O, lse, sel, F


def esa_prefill(Q, K, V, W_q, W_k, l_I, l_L, l_C, k, dtype, scale=None, eps: int = 0, chunks=None):
    """Chunked prefill of a whole sequence (Section 3.1).  Q [S,H,d], K,V [S,H_kv,d] float64.

    Returns dict t0 -> (O, lse, selected, F).  `chunks` restricts to the given start positions
    (steps of one layer are independent of each other given Q, K, V).
    """
    S, H, d = Q.shape
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    kc = compress(K, W_k, None, dtype)
    out = {}
    for t0 in (range(0, S, l_C) if chunks is None else chunks):
        t1 = min(t0 + l_C, S)
        qc = compress(Q[t0:t1], W_q, None, dtype)
        out[t0] = esa_step(Q[t0:t1], K[:t1], V[:t1], kc, qc, t0, l_I, l_L, k, scale, eps)
    return out


# ----------------------------------------------------------------------------- Appendix A: cost model
def flops_full_step(l_C, n_prev_and_cur, d_H, H):
    """(4 d_H + 3 H) l_C l_{I,M,L,C}: one step of full attention (Eq. 14)."""
    return (4 * d_H + 3 * H) * l_C * n_prev_and_cur


def flops_esa_step(l_C, l_I, l_M, l_L, k, d_H, H, d_c):
    """Compression, selection, sparse attention (Eq. 15, 16, 17)."""
    comp = 2 * 2 * l_C * d_H * d_c + 2 * l_C * d_c
    sel = 2 * l_M * l_C * d_c + l_M * l_C
    att = (4 * d_H + 3 * H) * l_C * (l_I + l_L + l_C + k)
    return comp, sel, att
