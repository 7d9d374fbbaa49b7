"""The seeded generator: determinism, slicing, distributions, and the planted structure
as seen through the oracle (needles selected, boundary gap present after planting it)."""
import numpy as np
import pytest

from esa_inputs import (CONFIGS, get_config, make_layer, make_weights, needle_plan, segment_bounds,
                        chunk_starts, f32_to_bf16_bits, bf16_bits_to_f32, storage_to_f64)
from oracle import esa_oracle as orc
from oracle.planted_gap import plant_gap


def test_bf16_bit_helpers_round_trip_and_agree_with_the_oracles_rounding():
    x = (np.random.default_rng(0).standard_normal(50000) * 10).astype(np.float32)
    bits = f32_to_bf16_bits(x)
    back = bf16_bits_to_f32(bits)
    assert np.array_equal(f32_to_bf16_bits(back), bits)
    assert np.array_equal(back.astype(np.float64), orc.round_to_storage(x.astype(np.float64), "bf16"))
    assert np.array_equal(orc.widen(bits, "bf16"), storage_to_f64(bits, "bf16"))


def test_generation_is_deterministic_and_sliceable():
    cfg = get_config("C1")
    a, b = make_layer(cfg), make_layer(cfg)
    for n in ("Q", "K", "V", "W_q", "W_k"):
        assert np.array_equal(getattr(a, n), getattr(b, n))
    part = make_layer(cfg, q_rows=(640, 768))
    assert np.array_equal(part.Q, a.Q[640:768]) and np.array_equal(part.K, a.K)
    other = make_layer(cfg, batch=1)
    assert not np.array_equal(other.K, a.K)
    assert np.array_equal(other.W_q, a.W_q)          # weights belong to the layer, not the batch element


def test_shapes_and_distributions():
    cfg = get_config("C1")
    L = make_layer(cfg)
    assert L.Q.shape == (2048, 4, 64) and L.K.shape == (2048, 2, 64) and L.V.shape == (2048, 2, 64)
    assert L.W_q.shape == (256, 32) and L.W_k.shape == (128, 32)
    assert abs(L.V.std() - 1.0) < 0.01 and abs(L.V.mean()) < 0.01
    assert abs(L.W_q.std() * 16.0 - 1.0) < 0.02 and abs(L.W_k.std() * np.sqrt(128.0) - 1.0) < 0.03
    small = get_config("C2").scaled(S=4096)
    Lb = make_layer(small)
    assert Lb.Q.dtype == np.uint16 and Lb.Q.shape == (4096, 32, 128)
    k = Lb.f64("K")
    assert abs(k.std() - 1.0) < 0.1
    # rotary encoding preserves the norm of every (i, i + d/2) pair; V is untouched noise
    raw = get_config("C2").scaled(S=4096, rope_base=None, needles=0)
    rot = get_config("C2").scaled(S=4096, needles=0)
    a, b = make_layer(raw).f64("K"), make_layer(rot).f64("K")
    na = a[..., :64] ** 2 + a[..., 64:] ** 2
    nb = b[..., :64] ** 2 + b[..., 64:] ** 2
    assert np.allclose(na, nb, rtol=0.05, atol=0.02)            # bf16 storage on both sides
    assert np.array_equal(a[0], b[0])                            # position 0 is not rotated


def test_table_of_configurations():
    n_chunks = {n: len(chunk_starts(c)) for n, c in CONFIGS.items()}
    assert n_chunks == {"C1": 16, "C2": 64, "C3": 256, "C4": 1, "C5": 256, "C6": 256}
    c3 = get_config("C3")
    i_end, l_start = segment_bounds(chunk_starts(c3)[-1], c3.l_I, c3.l_L)
    assert l_start - i_end == 128384
    c4 = get_config("C4")
    i_end, l_start = segment_bounds(chunk_starts(c4)[-1], c4.l_I, c4.l_L)
    assert l_start - i_end == 259967 and chunk_starts(c4) == [262143]
    c6 = get_config("C6")                     # the second model's shape: local length 4096 (Section 4.1, "Parameters")
    i_end, l_start = segment_bounds(chunk_starts(c6)[-1], c6.l_I, c6.l_L)
    assert (c6.l_L, c6.k, c6.l_I, c6.d_c) == (4096, 2048, 128, 128) and l_start - i_end == 126336


def test_needles_lie_in_the_owning_chunks_middle_and_never_collide():
    for name in ("C1", "C2"):
        cfg = get_config(name)
        plan = needle_plan(cfg)
        seen = set()
        for t0 in plan.t0:
            i_end, l_start = segment_bounds(t0, cfg.l_I, cfg.l_L)
            pos = plan.positions[t0]
            assert pos.shape[0] == cfg.needles * cfg.needle_span
            assert pos.min() >= i_end and pos.max() < l_start
            assert not (seen & set(pos.tolist()))
            seen |= set(pos.tolist())
            assert abs(np.linalg.norm(plan.direction[t0]) - 1.0) < 1e-12
    c5 = get_config("C5").scaled(S=65536)
    plan = needle_plan(c5)
    pos = plan.positions[plan.t0[-1]].reshape(c5.needles, c5.needle_span)
    assert np.all(np.diff(pos, axis=1) == 1)                      # contiguous spans


def test_oracle_selects_every_needle_and_gap_planting_separates_the_boundary():
    cfg = get_config("C1")
    L = make_layer(cfg)
    steps = [t0 for t0 in chunk_starts(cfg) if segment_bounds(t0, cfg.l_I, cfg.l_L)[1] - min(cfg.l_I, t0) > cfg.k]
    assert steps[0] == 640
    tau = 0.05
    replaced, kc = plant_gap(L, steps, tau)
    assert replaced.shape[0] < 200
    planted = np.concatenate([L.plan.positions[t] for t in L.plan.t0])
    W_q = orc.widen(L.W_q, cfg.dtype)
    for t0 in steps:
        i_end, l_start = segment_bounds(t0, cfg.l_I, cfg.l_L)
        qc = orc.compress(L.f64("Q", t0, t0 + cfg.l_C), W_q, None, cfg.dtype)
        F = orc.importance(qc, kc[i_end:l_start])
        srt = np.sort(F)[::-1]
        assert srt[cfg.k - 1] - srt[cfg.k] >= tau
        sel = orc.select_topk(F, cfg.k, base=i_end)
        if t0 in L.plan.positions:
            needles = np.setdiff1d(L.plan.positions[t0], replaced)     # a needle may sit in another step's band
            assert needles.shape[0] >= cfg.needles - 2
            assert set(needles.tolist()) <= set(sel.tolist())
            # every needle outranks every token of this chunk's middle segment that was not planted
            others = np.setdiff1d(np.arange(i_end, l_start), planted)
            assert F[needles - i_end].min() > F[others - i_end].max()


def test_gap_planting_on_pooled_scores_clears_both_sides_of_the_boundary_value():
    """With Eq. 8's pooling the k-th pooled value may be shared by several tokens (ties, ordered by
    position); every other pooled value must stay at least tau away from it."""
    cfg = get_config("C1")
    L = make_layer(cfg)
    steps, tau, eps = [1152, 1920], 1.5, 3
    replaced, kc = plant_gap(L, steps, tau, eps=eps)
    assert 0 < replaced.shape[0] < 200
    W_q = orc.widen(L.W_q, cfg.dtype)
    for t0 in steps:
        i_end, l_start = segment_bounds(t0, cfg.l_I, cfg.l_L)
        qc = orc.compress(L.f64("Q", t0, t0 + cfg.l_C), W_q, None, cfg.dtype)
        Fp = orc.proximity(orc.importance(qc, kc[i_end:l_start]), eps)
        f_k = np.sort(Fp)[::-1][cfg.k - 1]
        dist = np.abs(Fp - f_k)
        assert dist[dist > 0].min() >= tau
