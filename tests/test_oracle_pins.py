"""Pins for the CPU oracle: what the paper and the mathematics fix, not the oracle's own output.

Each test names the mistake it is meant to catch.
"""
import os

import numpy as np
import pytest
from scipy.ndimage import maximum_filter1d
from scipy.special import logsumexp, softmax

from oracle import esa_oracle as orc

RNG = np.random.default_rng(12345)


def _qkv(S, H, H_kv, d, rng=RNG):
    return (rng.standard_normal((S, H, d)), rng.standard_normal((S, H_kv, d)),
            rng.standard_normal((S, H_kv, d)))


def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_closed_forms.txt")
    vals = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            name, value = line.split()[:2]
            vals[name] = float(value)
    return vals


# ------------------------------------------------------------------ storage rounding
def test_bf16_rounding_matches_ieee_definition():
    # nearest-even on hand-picked cases: exact, below half, above half, ties both ways
    x = np.array([1.0, 1.0 + 2**-9, 1.0 + 2**-8 - 2**-20, 1.0 + 2**-8 + 2**-20,
                  1.0 + 2**-8, 1.0 + 3 * 2**-8, -1.0 - 2**-8, 0.0, 3.0e-3, 255.5])
    want = np.array([1.0, 1.0, 1.0, 1.0 + 2**-7, 1.0, 1.0 + 2**-6, -1.0, 0.0, 197.0 / 65536.0, 256.0])  # 3e-3 = 196.608 * 2^-16
    got = orc.round_to_storage(x, "bf16")
    assert np.array_equal(got, want)
    # round trip through the 16-bit pattern is exact
    assert np.array_equal(orc.widen(orc.narrow_to_bits(got, "bf16"), "bf16"), got)
    # error bound of round-to-nearest with 8 significant bits
    y = RNG.standard_normal(100000) * 37.0
    assert np.all(np.abs(orc.round_to_storage(y, "bf16") - y) <= np.abs(y) * 2.0**-8)


# ------------------------------------------------------------------ segments (Section 3.1)
def test_segments_partition_the_preceding_tokens():
    for t0, l_I, l_L in [(0, 32, 256), (10, 32, 256), (32, 32, 256), (100, 32, 256), (288, 32, 256),
                         (289, 32, 256), (640, 32, 256), (130560, 128, 2048)]:
        i_end, l_start = orc.segments(t0, l_I, l_L)
        assert 0 <= i_end <= l_start <= t0
        assert i_end == min(l_I, t0)
        assert t0 - l_start <= l_L
        if t0 >= l_I + l_L:                      # steady state: both fixed parts are full
            assert i_end == l_I and t0 - l_start == l_L
    assert orc.segments(640, 32, 256) == (32, 384)       # 352 middle tokens
    assert orc.segments(130560, 128, 2048) == (128, 128512)


# ------------------------------------------------------------------ Eq. 5 compression
def test_compress_identity_and_hand_example():
    x = RNG.standard_normal((5, 3, 4))
    assert np.array_equal(orc.compress(x, np.eye(12), None, "f32"),
                          x.reshape(5, 12).astype(np.float32).astype(np.float64))
    # head-major concatenation: token 0 = heads [1,2 | 3,4]; W picks (head0,dim1) and (head1,dim0)
    x = np.array([[[1.0, 2.0], [3.0, 4.0]]])
    W = np.zeros((4, 2)); W[1, 0] = 1.0; W[2, 1] = 10.0
    assert np.array_equal(orc.compress(x, W, None, "f32"), [[2.0, 30.0]])       # transposed W or wrong concat fails
    assert np.array_equal(orc.compress(x, W, np.array([0.5, -1.0]), "f32"), [[2.5, 29.0]])
    # library routine on random data (rounding to fp32 only)
    x = RNG.standard_normal((7, 2, 8)); W = RNG.standard_normal((16, 5))
    assert np.allclose(orc.compress(x, W, None, "f32"), np.matmul(x.reshape(7, 16), W), rtol=1e-6, atol=1e-6)
    # bf16 storage: result is representable and within half an ulp
    y = orc.compress(x, W, None, "bf16")
    exact = x.reshape(7, 16) @ W
    assert np.all(np.abs(y - exact) <= np.abs(exact) * 2.0**-8)


# ------------------------------------------------------------------ Eq. 3 / Eq. 6 head concatenation
def test_full_dimension_score_is_a_special_case_of_compressed_score():
    H, H_kv, d, n_c, n_m = 4, 2, 8, 6, 40
    G = H // H_kv
    q = RNG.standard_normal((n_c, H, d)); kk = RNG.standard_normal((n_m, H_kv, d))
    # Eq. 3 written out with explicit loops over heads
    want = np.zeros((n_c, n_m))
    for c in range(n_c):
        for m in range(n_m):
            for h in range(H):
                want[c, m] += float(np.dot(q[c, h], kk[m, h // G]))
    # d' = d_H, W_q = identity, W_k = the GQA repeat map (key head g feeds query heads g*G..g*G+G-1)
    W_k = np.zeros((H_kv * d, H * d))
    for h in range(H):
        W_k[(h // G) * d:(h // G + 1) * d, h * d:(h + 1) * d] = np.eye(d)
    qc = q.reshape(n_c, -1)
    kc = kk.reshape(n_m, -1) @ W_k
    assert np.allclose(orc.pair_scores(qc, kc), want, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ Eq. 4 invariants
def test_importance_invariants():
    qc = RNG.standard_normal((16, 8)); kc = RNG.standard_normal((300, 8))
    F = orc.importance(qc, kc)
    S = qc @ kc.T
    assert F.shape == (300,)
    assert np.all(F <= 0.0) and F.max() == 0.0
    assert np.all(F[np.argmax(S, axis=1)] == 0.0)           # every current token's best middle token scores 0
    # a token that is nobody's best is strictly negative
    others = np.setdiff1d(np.arange(300), np.argmax(S, axis=1))
    assert np.all(F[others] < 0.0)
    # shifting one current token's scores by a constant (e.g. scaling its norm) cannot change F's argmax set:
    # direct definition on a 2x3 example, by hand
    q2 = np.array([[1.0, 0.0], [0.0, 2.0]]); k2 = np.array([[3.0, 1.0], [1.0, 5.0], [2.0, 2.0]])
    # S = [[3,1,2],[2,10,4]]; row max = [3,10]; S-mu = [[0,-2,-1],[-8,0,-6]]; column max = [0,0,-1]
    assert np.array_equal(orc.importance(q2, k2), [0.0, 0.0, -1.0])


def test_single_current_token_ranks_like_raw_dot_product():
    qc = RNG.standard_normal((1, 8)); kc = RNG.standard_normal((500, 8))
    F = orc.importance(qc, kc)
    raw = (kc @ qc[0])
    assert np.array_equal(np.argsort(-F, kind="stable"), np.argsort(-raw, kind="stable"))
    assert np.allclose(F, raw - raw.max(), rtol=0, atol=1e-12)


# ------------------------------------------------------------------ Eq. 8 proximity influence
@pytest.mark.parametrize("eps", [0, 1, 3, 5])
def test_proximity_is_a_clamped_maximum_filter(eps):
    s = RNG.standard_normal(257)
    got = orc.proximity(s, eps)
    if eps == 0:
        assert np.array_equal(got, s)
    # 'nearest' padding repeats edge values, which never raises a maximum beyond the clamped window's
    want = maximum_filter1d(s, size=2 * eps + 1, mode="nearest")
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ Eq. 2 selection
def test_select_topk_against_brute_force():
    for n, k in [(50, 7), (50, 1), (50, 50), (50, 80), (1, 1), (300, 299)]:
        s = RNG.standard_normal(n)
        got = orc.select_topk(s, k, base=100)
        # brute force: repeatedly take the best remaining
        rem = list(range(n)); chosen = []
        for _ in range(min(k, n)):
            b = max(rem, key=lambda i: (s[i], -i)); chosen.append(b); rem.remove(b)
        assert got.dtype == np.int32
        assert np.array_equal(got, np.array(sorted(chosen)) + 100)
    assert orc.select_topk(np.zeros(0), 5).shape == (0,)
    assert orc.select_topk(np.ones(4), 0).shape == (0,)


def test_select_topk_ties_go_to_the_lower_position():
    s = np.array([0.0, -1.0, 0.0, -1.0, -1.0, 0.0, -2.0, -1.0])
    assert np.array_equal(orc.select_topk(s, 2), [0, 2])
    assert np.array_equal(orc.select_topk(s, 4), [0, 1, 2, 5])
    assert np.array_equal(orc.select_topk(s, 5), [0, 1, 2, 3, 5])
    assert np.array_equal(orc.select_topk(s, 7), [0, 1, 2, 3, 4, 5, 7])


# ------------------------------------------------------------------ gather
def test_gather_is_row_indexing():
    cache = RNG.standard_normal((40, 2, 3)); idx = np.array([3, 17, 39, 0], dtype=np.int32)
    got = orc.gather_rows(cache, idx)
    for i, p in enumerate(idx):
        assert np.array_equal(got[i], cache[p])


# ------------------------------------------------------------------ Eq. 1 attention
def test_attend_with_k_covering_the_middle_is_full_causal_attention():
    """Eq. 1 with M_k = M is Eq. 10.  Catches: wrong GQA map, wrong causal alignment, dropped
    segment, off-by-one at any of the three boundaries, wrong scale."""
    S, H, H_kv, d = 96, 4, 2, 8
    Q, K, V = _qkv(S, H, H_kv, d)
    scale = 1.0 / np.sqrt(d)
    want = orc.full_causal_attention(Q, K, V, scale)
    for l_I, l_L, l_C in [(4, 16, 8), (4, 16, 32), (1, 1, 5), (0, 3, 7), (10, 0, 12), (200, 200, 96)]:
        for t0 in range(0, S, l_C):
            t1 = min(t0 + l_C, S)
            i_end, l_start = orc.segments(t0, l_I, l_L)
            sel = np.arange(i_end, l_start)
            O, lse = orc.attend(Q[t0:t1], K[:t1], V[:t1], t0, l_I, l_L, sel, scale)
            assert np.allclose(O, want[t0:t1], rtol=1e-11, atol=1e-12), (l_I, l_L, l_C, t0)
            # lse against the library routine on the plain causal logits
            for h in range(H):
                lg = scale * Q[t0:t1, h] @ K[:t1, h // (H // H_kv)].T
                for c in range(t1 - t0):
                    assert abs(lse[c, h] - logsumexp(lg[c, :t0 + c + 1])) < 1e-11


def test_prefill_is_independent_of_chunk_size_when_k_covers_the_middle():
    S, H, H_kv, d, d_c = 80, 4, 2, 8, 4
    Q, K, V = _qkv(S, H, H_kv, d)
    W_q = RNG.standard_normal((H * d, d_c)); W_k = RNG.standard_normal((H_kv * d, d_c))
    full = orc.full_causal_attention(Q, K, V, 1.0 / np.sqrt(d))
    for l_C in (1, 7, 16, 80):
        res = orc.esa_prefill(Q, K, V, W_q, W_k, l_I=4, l_L=8, l_C=l_C, k=S, dtype="f32")
        O = np.concatenate([res[t0][0] for t0 in sorted(res)])
        assert np.allclose(O, full, rtol=1e-11, atol=1e-12)


def test_attention_probabilities_sum_to_one_and_respect_visibility():
    S, H, H_kv, d = 64, 4, 2, 8
    Q, K, V = _qkv(S, H, H_kv, d)
    t0, l_C, l_I, l_L = 48, 16, 4, 8
    sel = np.array([7, 19, 30], dtype=np.int32)
    O, lse, P, pos = orc.attend(Q[t0:], K, V, t0, l_I, l_L, sel, 0.3, return_probs=True)
    assert np.all(np.abs(P.sum(axis=2) - 1.0) < 1e-12)
    assert np.array_equal(pos, np.concatenate([np.arange(4), sel, np.arange(40, 64)]))
    for c in range(l_C):
        assert np.all(P[:, c, pos > t0 + c] == 0.0)
        assert np.all(P[:, c, pos <= t0 + c] > 0.0)
    # against the library softmax on the same key set, one query at a time
    c, h = 5, 3
    keys = pos[pos <= t0 + c]
    p_lib = softmax(0.3 * K[keys, h // 2] @ Q[t0 + c, h])
    assert np.allclose(O[c, h], p_lib @ V[keys, h // 2], rtol=1e-12, atol=1e-13)


def test_merge_identity_of_algorithm_1():
    """Local (L and C, causal) and global (I and M_k) attentions merged by exp(lse) weights
    equal one softmax over the union."""
    S, H, H_kv, d = 64, 4, 2, 8
    Q, K, V = _qkv(S, H, H_kv, d)
    t0, l_C, l_I, l_L, scale = 48, 16, 4, 8, 0.35
    sel = np.array([9, 21, 22, 35], dtype=np.int32)
    joint, lse_joint = orc.attend(Q[t0:], K, V, t0, l_I, l_L, sel, scale)
    # local part: no initial tokens, nothing selected
    loc, lse_loc = orc.attend(Q[t0:], K, V, t0, 0, l_L, np.empty(0, np.int32), scale)
    # global part alone, with library softmax (not causal)
    gpos = np.concatenate([np.arange(l_I), sel])
    glo = np.empty_like(joint); lse_glo = np.empty_like(lse_joint)
    for h in range(H):
        lg = scale * Q[t0:, h] @ K[gpos, h // 2].T
        glo[:, h] = softmax(lg, axis=1) @ V[gpos, h // 2]
        lse_glo[:, h] = logsumexp(lg, axis=1)
    merged = orc.merge_partial_attention([loc, glo], [lse_loc, lse_glo])
    assert np.allclose(merged, joint, rtol=1e-11, atol=1e-12)
    assert np.allclose(np.logaddexp(lse_loc, lse_glo), lse_joint, rtol=1e-12, atol=1e-12)


def test_attend_ignores_the_order_of_selected_tokens_and_handles_one_key():
    S, H, H_kv, d = 40, 2, 1, 4
    Q, K, V = _qkv(S, H, H_kv, d)
    sel = np.array([5, 9, 14, 20], dtype=np.int32)
    a, _ = orc.attend(Q[32:], K, V, 32, 2, 4, sel, 0.5)
    b, _ = orc.attend(Q[32:], K, V, 32, 2, 4, sel[::-1].copy(), 0.5)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-13)
    # first token of a sequence attends only to itself
    O, lse = orc.attend(Q[:1], K[:1], V[:1], 0, 2, 4, np.empty(0, np.int32), 0.5)
    assert np.array_equal(O[0, 0], V[0, 0]) and np.array_equal(O[0, 1], V[0, 0])
    assert np.allclose(lse[0], 0.5 * np.array([Q[0, 0] @ K[0, 0], Q[0, 1] @ K[0, 0]]))


def test_step_selects_planted_tokens_and_decode_equals_prefill_with_one_token():
    S, H, H_kv, d, d_c = 200, 2, 1, 8, 8
    Q, K, V = _qkv(S, H, H_kv, d)
    W_q = np.eye(H * d)[:, :d_c] * 1.0
    W_k = np.eye(H_kv * d)[:, :d_c] * 1.0
    t0, l_I, l_L, k = 199, 4, 16, 5
    planted = np.array([20, 77, 150])
    K[planted, 0, :d_c] = 25.0 * Q[t0, 0, :d_c] / np.linalg.norm(Q[t0, 0, :d_c])
    res = orc.esa_prefill(Q, K, V, W_q, W_k, l_I, l_L, 1, k, "f32", chunks=[t0])
    O, lse, sel, F = res[t0]
    assert set(planted.tolist()) <= set(sel.tolist()) and sel.shape == (k,)
    assert np.all(np.diff(sel) > 0) and sel.min() >= l_I and sel.max() < t0 - l_L
    # one decode step == a one-token chunk: same arithmetic by construction; check against raw top-k of q'.k'
    kc = orc.compress(K, W_k, None, "f32"); qc = orc.compress(Q[t0:t0 + 1], W_q, None, "f32")
    raw = kc[l_I:t0 - l_L] @ qc[0]
    assert set((np.argsort(-raw, kind="stable")[:k] + l_I).tolist()) == set(sel.tolist())


# ------------------------------------------------------------------ Eq. 9, cache overhead, Appendix A
# ----------------------------------------------------------------------------- Section 3.2
def test_rope_is_a_rotation_that_composes_and_depends_on_relative_position_only():
    """Catches: wrong pairing of elements, wrong sign of the sine term, wrong frequency exponent."""
    rng = np.random.default_rng(5)
    n, heads, d, base = 7, 3, 8, 10000.0
    x, y = rng.standard_normal((n, heads, d)), rng.standard_normal((n, heads, d))
    pos = rng.integers(0, 500, n)
    assert np.array_equal(orc.rope(x, np.zeros(n), base), x)                       # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(orc.rope(x, pos, base), axis=2), np.linalg.norm(x, axis=2), rtol=1e-12)
    np.testing.assert_allclose(orc.rope(orc.rope(x, pos, base), 3 * pos, base), orc.rope(x, 4 * pos, base), atol=1e-9)
    # <R_a x, R_b y> = <R_(a+s) x, R_(b+s) y>
    a, b, shift = rng.integers(0, 300, n), rng.integers(0, 300, n), 1234
    dots = lambda pa, pb: np.einsum("nhd,nhd->nh", orc.rope(x, pa, base), orc.rope(y, pb, base))
    np.testing.assert_allclose(dots(a, b), dots(a + shift, b + shift), atol=1e-9)
    # closed form for one pair of elements: element i and i + d/2 turn by pos * base^(-2i/d), counter-clockwise
    v = np.zeros((1, 1, d))
    v[0, 0, 1], v[0, 0, 1 + d // 2] = 2.0, 0.5
    ang = 11.0 * base ** (-2.0 * 1 / d)
    got = orc.rope(v, [11], base)[0, 0]
    np.testing.assert_allclose([got[1], got[1 + d // 2]],
                               [2.0 * np.cos(ang) - 0.5 * np.sin(ang), 0.5 * np.cos(ang) + 2.0 * np.sin(ang)], rtol=1e-12)
    assert np.count_nonzero(got) == 2


def test_two_encodings_reduce_to_eq1_and_fuse_as_algorithm_1_says():
    """Same tensors for both groups give Eq. 1 back; different tensors equal the two groups' own
    softmaxes (written out here with scipy) fused by exp(lse) weights (Algorithm 1).
    Catches: a group's logits taken from the wrong encoding, the causal mask applied to the global
    group, I placed in the local group."""
    rng = np.random.default_rng(6)
    S, H, H_kv, d, l_C, l_I, l_L, t0 = 90, 4, 2, 8, 6, 5, 20, 84
    Q, K, V = _qkv(S, H, H_kv, d, rng)
    sel = np.array([7, 19, 33, 40, 61])
    q = Q[t0:t0 + l_C]
    want, want_lse = orc.attend(q, K, V, t0, l_I, l_L, sel, 0.3)
    got, got_lse = orc.attend_two_encodings(q, q, K, K, V, t0, l_I, l_L, sel, 0.3)
    np.testing.assert_allclose(got, want, atol=1e-12)
    np.testing.assert_allclose(got_lse, want_lse, atol=1e-12)
    # different encodings per group
    q_g, K_g = rng.standard_normal(q.shape), rng.standard_normal(K.shape)
    O, lse = orc.attend_two_encodings(q, q_g, K, K_g, V, t0, l_I, l_L, sel, 0.3)
    glob = np.concatenate([np.arange(l_I), sel])
    for c in range(l_C):
        for h in range(H):
            g = h // (H // H_kv)
            a_g = 0.3 * K_g[glob, g] @ q_g[c, h]
            loc = np.arange(t0 - l_L, t0 + c + 1)
            a_l = 0.3 * K[loc, g] @ q[c, h]
            o_g, o_l = softmax(a_g) @ V[glob, g], softmax(a_l) @ V[loc, g]
            w_g, w_l = np.exp(logsumexp(a_g)), np.exp(logsumexp(a_l))
            np.testing.assert_allclose(O[c, h], (w_g * o_g + w_l * o_l) / (w_g + w_l), atol=1e-12)
            np.testing.assert_allclose(lse[c, h], np.log(w_g + w_l), atol=1e-12)


def test_reencoded_positions_follow_section_3_2():
    """Local logits depend on relative position only, so encoding L and C in order from 0 equals
    encoding them at their absolute positions; global logits are those of relative position w for
    every pair.  Catches: local positions not starting where the local window starts, w applied
    to keys, selected keys encoded at their own position."""
    rng = np.random.default_rng(7)
    S, H, H_kv, d, l_C, l_I, l_L, t0, w, base = 80, 2, 1, 16, 4, 3, 12, 70, 37.0, 10000.0
    Q, K, V = _qkv(S, H, H_kv, d, rng)
    sel = np.array([9, 21, 22, 50])
    q = Q[t0:t0 + l_C]
    O, lse = orc.attend_reencoded(q, K, V, t0, l_I, l_L, sel, 0.25, w, base)
    K_abs = orc.rope(K, np.arange(S), base)
    q_abs = orc.rope(q, t0 + np.arange(l_C), base)
    q_w = orc.rope(q, np.full(l_C, w), base)
    want, want_lse = orc.attend_two_encodings(q_abs, q_w, K_abs, K, V, t0, l_I, l_L, sel, 0.25)
    np.testing.assert_allclose(O, want, atol=1e-10)
    np.testing.assert_allclose(lse, want_lse, atol=1e-10)
    # a global logit is the dot product at relative position w whatever the key's own position
    p = 21
    assert np.isclose(q_w[1, 0] @ K[p, 0], orc.rope(q[1:2], [p + w], base)[0, 0] @ orc.rope(K[p:p + 1], [p], base)[0, 0])
    # early chunk: fewer local tokens than l_L, no middle tokens
    O2, _ = orc.attend_reencoded(Q[8:12], K, V, 8, l_I, l_L, np.empty(0, int), 0.25, w, base)
    want2, _ = orc.attend_two_encodings(orc.rope(Q[8:12], 8 + np.arange(4), base), orc.rope(Q[8:12], np.full(4, w), base),
                                        K_abs, K, V, 8, l_I, l_L, np.empty(0, int), 0.25)
    np.testing.assert_allclose(O2, want2, atol=1e-10)


def test_cost_model_reproduces_the_papers_numbers():
    g = _golden()
    d_c, d_H, H, H_G = int(g["d_prime"]), int(g["d_H"]), int(g["H"]), int(g["H_G"])
    r_closed = (2 * d_c + 1) / (4 * d_H + 3 * H)
    assert round(100 * r_closed, 2) == g["reduction_ratio_percent"]
    assert 100 * d_c / (2 * H_G * (d_H // H)) == g["cache_overhead_percent"]
    # the step-level FLOP counts approach the closed form as the middle segment grows (Eq. 18)
    l_I, l_L, l_C, k = 128, 4096, 512, 2048
    prev = None
    for l_M in (10**6, 10**7, 10**8, 10**9):
        comp, sel, att = orc.flops_esa_step(l_C, l_I, l_M, l_L, k, d_H, H, d_c)
        r = (comp + sel + att) / orc.flops_full_step(l_C, l_I + l_M + l_L + l_C, d_H, H)
        assert r > r_closed
        if prev is not None:
            assert r < prev
        prev = r
    assert abs(prev - r_closed) / r_closed < 1e-3
    # term by term at a size small enough to count by hand: l_C=2, l_M=10, d_H=8, H=2, d'=4, l_I=1, l_L=3, k=5
    comp, sel, att = orc.flops_esa_step(2, 1, 10, 3, 5, 8, 2, 4)
    assert comp == 2 * 2 * 2 * 8 * 4 + 2 * 2 * 4 and sel == 2 * 10 * 2 * 4 + 10 * 2
    assert att == (4 * 8 + 3 * 2) * 2 * (1 + 3 + 2 + 5)
    assert orc.flops_full_step(2, 16, 8, 2) == (32 + 6) * 2 * 16
