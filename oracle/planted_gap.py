"""Score gap at the selection boundary, planted with the oracle's own scores.  TEST INFRASTRUCTURE.

Adjacent order statistics of the importance score near rank k are closer together than
the rounding differences between an fp32-accumulating GPU kernel and float64, so the
selected *set* is only well defined if rank k and rank k+1 are separated.  For every
step under test, tokens ranked below k whose score lies within `tau` of the k-th score get
their key pushed (by the input generator) against the direction that step's queries share:
their score for that step drops, while other steps see only a small random change.  A push can
still move a token across another step's boundary, so the procedure repeats, with a growing
push, until no step has a token inside its band.
"""
from __future__ import annotations

import numpy as np

from esa_inputs import push_keys_down, segment_bounds
from . import esa_oracle as orc


def plant_gap(layer, steps, tau: float, max_rounds: int = 30, eps: int = 0):
    """Modify layer.K in place.  `steps` = chunk start positions to protect.

    With eps > 0 the selection acts on the max-pooled score of Eq. 8: tokens that share a pooled value
    (the same source token inside their windows) are tied exactly on any implementation and the tie
    rule orders them, so the band to clear is the pooled values strictly between f_k - tau and
    f_k + tau other than f_k itself, and what gets pushed is the source token of such a value.

    Returns (sorted array of modified positions, compressed keys K' as float64 [S, d_c]).
    Steps without a planted direction cannot be protected this way and raise.
    """
    cfg = layer.cfg
    W_q = orc.widen(layer.W_q, cfg.dtype)
    W_k = orc.widen(layer.W_k, cfg.dtype)
    kc = orc.compress(orc.widen(layer.K, cfg.dtype), W_k, None, cfg.dtype)
    q_lo = getattr(layer, "q_row0", 0)
    touched = set()
    for rnd in range(max_rounds):
        bad = {}
        for t0 in steps:
            i_end, l_start = segment_bounds(t0, cfg.l_I, cfg.l_L)
            n_mid = l_start - i_end
            if n_mid <= cfg.k:
                continue
            if t0 not in layer.plan.direction:
                raise ValueError("step %d has no planted direction to push against" % t0)
            t1 = min(t0 + cfg.l_C, cfg.S)
            qc = orc.compress(orc.widen(layer.Q[t0 - q_lo:t1 - q_lo], cfg.dtype), W_q, None, cfg.dtype)
            F = orc.importance(qc, kc[i_end:l_start])
            if eps > 0:
                Fp = orc.proximity(F, eps)
                f_k = Fp[np.argsort(-Fp, kind="stable")[cfg.k - 1]]
                near = np.nonzero((np.abs(Fp - f_k) < tau) & (Fp != f_k))[0]
                src = set()
                for j in near.tolist():           # the tokens inside j's window that carry its pooled value
                    lo, hi = max(j - eps, 0), min(j + eps, n_mid - 1)
                    src.update((lo + np.nonzero(F[lo:hi + 1] == Fp[j])[0]).tolist())
                for p in sorted(src):
                    bad.setdefault(p + i_end, []).append(t0)
                continue
            order = np.argsort(-F, kind="stable")
            f_k = F[order[cfg.k - 1]]
            below = order[cfg.k:]
            for p in (below[F[below] > f_k - tau] + i_end).tolist():
                bad.setdefault(p, []).append(t0)
        if not bad:
            return np.array(sorted(touched), dtype=np.int64), kc
        pos = np.array(sorted(bad), dtype=np.int64)
        delta = (2.0 * tau / layer.plan.beta) * 2.0 ** min(rnd, 12)
        layer.K[pos] = push_keys_down(cfg, layer.batch, layer.K[pos], [bad[p] for p in pos.tolist()],
                                      layer.plan, delta)
        kc[pos] = orc.compress(orc.widen(layer.K[pos], cfg.dtype), W_k, None, cfg.dtype)
        touched.update(pos.tolist())
    raise RuntimeError("planted gap did not converge")
