"""GPU parity: every libesa call against the float64 oracle, on the same seeded inputs.

Stage-wise tests feed a call the oracle's own inputs, so each call is judged alone; pipeline
tests chain the five calls on the GPU and compare the step's final results.
Bars: indices bit-exact; attention outputs max-abs 1e-5 (fp32) / 2e-2 (bf16); compressed
values within one unit in the last place of the storage type; scores within the tolerance
derived from fp32 accumulation of d_c exact products.
"""
import sys

import numpy as np
import pytest
import torch

from esa_inputs import get_config, make_layer, segment_bounds, chunk_starts
from oracle import esa_oracle as orc
from oracle.planted_gap import plant_gap

from support import to_dev, to_f64, f64_to_dev, bf16_ulp, oracle_step, gpu_step, layer_to_dev, pack_layer_weights

pytestmark = pytest.mark.gpu

O_TOL = {"f32": 1e-5, "bf16": 2e-2}
# |F_gpu - F_oracle| for identical stored inputs: fp32 accumulation of d_c exact (bf16) or
# once-rounded (fp32) products of magnitude <= ~600 -> a few 1e-4 absolute.
F_TOL = {"f32": 2e-4, "bf16": 1e-3}
# boundary gap planted for end-to-end index parity (the GPU chain scores its own K', Q', which differ from the
# oracle's in a few last places: one bf16 step in a compressed component moves a score by up to ~0.1)
TAU_E2E = {"f32": 2e-3, "bf16": 0.5}


@pytest.fixture(scope="module")
def esa():
    import paper_2502_14477_amd as lib
    return lib


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


# ------------------------------------------------------------------------------------------ top-k
def _scores(rng, n, kind):
    if kind == "normal":
        return rng.standard_normal(n).astype(np.float32)
    if kind == "ties":          # few distinct values: the tie rule decides almost everything
        return (rng.integers(-3, 1, n) * 0.5).astype(np.float32)
    if kind == "importance":    # like Eq. 4 output: non-positive, some exact zeros, narrow exponent range
        s = (-400.0 - 40.0 * np.abs(rng.standard_normal(n))).astype(np.float32)
        s[rng.choice(n, size=min(n, 7), replace=False)] = 0.0
        return s
    if kind == "constant":
        return np.full(n, -1.25, dtype=np.float32)
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["normal", "ties", "importance", "constant"])
@pytest.mark.parametrize("n,k", [(1, 1), (5, 3), (300, 1), (2047, 256), (2048, 2048), (2049, 2048), (2049, 5000),
                                 (5000, 17), (40000, 2048), (128384, 2048), (259967, 2048), (70000, 69999),
                                 (700001, 4096)])     # more workgroups than compute units, one tile each
def test_select_topk_is_bit_exact(esa, kind, n, k):
    say(f"topk kind={kind} n={n} k={k}")
    rng = np.random.default_rng(n * 7919 + k)
    s = _scores(rng, n, kind)
    want = orc.select_topk(s.astype(np.float64), k, base=1000)
    got = esa.esa_select_topk(torch.from_numpy(s).cuda(), k, base=1000).cpu().numpy()
    assert got.dtype == np.int32 and np.array_equal(got, want)


def test_select_topk_batched_rows_with_stride(esa):
    say("topk batch=5 strided")
    rng = np.random.default_rng(5)
    B, n, k = 5, 9001, 777
    buf = torch.full((B, n + 13), 1e30, dtype=torch.float32)       # padding that must never be read as data
    s = np.stack([_scores(rng, n, kd) for kd in ("normal", "ties", "importance", "normal", "ties")])
    buf[:, :n] = torch.from_numpy(s)
    got = esa.esa_select_topk(buf.cuda()[:, :n], k, base=3).cpu().numpy()
    for b in range(B):
        assert np.array_equal(got[b], orc.select_topk(s[b].astype(np.float64), k, base=3)), b


@pytest.mark.parametrize("B,n,k", [(6, 300001, 2048), (16, 259967, 2048), (40, 1500000 // 8, 5)])
def test_select_topk_many_rows_several_tiles_per_workgroup(esa, B, n, k):
    """Enough rows that a workgroup takes several tiles (2, 3 and 6 here): offsets run across tiles."""
    say(f"topk batch={B} n={n} k={k}")
    rng = np.random.default_rng(B * 31 + k)
    kinds = ("normal", "ties", "importance", "constant")
    s = np.stack([_scores(rng, n, kinds[b % 4]) for b in range(B)])
    got = esa.esa_select_topk(torch.from_numpy(s).cuda(), k, base=11).cpu().numpy()
    for b in range(B):
        assert np.array_equal(got[b], orc.select_topk(s[b].astype(np.float64), k, base=11)), b


# ------------------------------------------------------------------------------------------ gather
@pytest.mark.parametrize("dtype,h_kv,d,pad", [("f32", 2, 64, 0), ("bf16", 8, 128, 0), ("bf16", 2, 64, 24),
                                              ("f32", 1, 32, 5), ("bf16", 3, 32, 1)])
def test_gather_is_byte_exact(esa, dtype, h_kv, d, pad):
    say(f"gather dtype={dtype} h_kv={h_kv} d={d} pad={pad}")
    rng = np.random.default_rng(11)
    B, S, n_sel = 2, 700, 133
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    kfull = torch.randn((B, S, h_kv * d + pad), generator=torch.Generator().manual_seed(1)).to(tdt).cuda()
    vfull = torch.randn((B, S, h_kv * d + pad), generator=torch.Generator().manual_seed(2)).to(tdt).cuda()
    kc = kfull[:, :, :h_kv * d].unflatten(2, (h_kv, d))
    vc = vfull[:, :, :h_kv * d].unflatten(2, (h_kv, d))
    idx = np.stack([np.sort(rng.choice(S, n_sel, replace=False)) for _ in range(B)]).astype(np.int32)
    ks, vs = esa.esa_gather_kv(kc, vc, torch.from_numpy(idx).cuda())
    for b in range(B):
        assert torch.equal(ks[b], kc[b][torch.from_numpy(idx[b]).long().cuda()])
        assert torch.equal(vs[b], vc[b][torch.from_numpy(idx[b]).long().cuda()])
    # the oracle's definition on the widened values
    want = orc.gather_rows(to_f64(kc[0]), idx[0])
    assert np.array_equal(to_f64(ks[0]), want)


def test_gather_from_a_kv_cache_offloaded_to_pinned_host_memory(esa):
    """Appendix B's deployment: the KV cache lives in host memory and only the selected rows are
    loaded per step.  The same kernel reads the pinned cache through its device mapping."""
    say("gather from pinned host memory")
    rng = np.random.default_rng(404)
    S, h_kv, d, n_sel = 20000, 8, 128, 2048
    K = torch.from_numpy(rng.integers(0, 2**15, (S, h_kv, d), dtype=np.int16)).view(torch.bfloat16).pin_memory()
    V = torch.from_numpy(rng.integers(0, 2**15, (S, h_kv, d), dtype=np.int16)).view(torch.bfloat16).pin_memory()
    idx = torch.from_numpy(np.sort(rng.choice(S, n_sel, replace=False)).astype(np.int32))
    ks, vs = esa.esa_gather_kv(K, V, idx.cuda())
    assert ks.is_cuda and torch.equal(ks.cpu().view(torch.int16), K[idx.long()].view(torch.int16))
    assert torch.equal(vs.cpu().view(torch.int16), V[idx.long()].view(torch.int16))
    with pytest.raises(ValueError):
        esa.esa_gather_kv(K.clone(), V.clone(), idx.cuda())       # pageable host memory is refused, not dereferenced


# ------------------------------------------------------------------------------------------ compress
@pytest.mark.parametrize("dtype,n_tok,heads,d,d_c,bias", [
    ("f32", 128, 4, 64, 32, False), ("f32", 37, 2, 64, 32, True), ("f32", 1, 4, 64, 32, False),
    ("bf16", 512, 32, 128, 128, False), ("bf16", 100, 8, 128, 128, True), ("bf16", 1, 32, 128, 128, False),
    ("bf16", 77, 4, 64, 48, True)])
def test_compress_matches_oracle(esa, dtype, n_tok, heads, d, d_c, bias):
    say(f"compress dtype={dtype} n_tok={n_tok} heads={heads} d={d} d_c={d_c} bias={bias}")
    rng = np.random.default_rng(n_tok + d_c)
    d_in = heads * d
    x = orc.round_to_storage(rng.standard_normal((n_tok, heads, d)), dtype)
    W = orc.round_to_storage(rng.standard_normal((d_in, d_c)) / np.sqrt(d_in), dtype)
    b = orc.round_to_storage(rng.standard_normal(d_c), dtype) if bias else None
    want = orc.compress(x, W, b, dtype)
    xd, Wd = f64_to_dev(x, dtype), f64_to_dev(W, dtype)
    bd = None if b is None else f64_to_dev(b, dtype)
    _assert_compressed_close(to_f64(esa.esa_compress(xd, Wd, bd)), want, x, W, b, dtype)
    # the packed weight layout computes the same thing
    Wp = esa.esa_pack_weights(Wd)
    assert torch.equal(Wp.data, Wd.t().contiguous())
    _assert_compressed_close(to_f64(esa.esa_compress(xd, Wp, bd)), want, x, W, b, dtype)


def _assert_compressed_close(got, want, x, W, b, dtype):
    if dtype == "f32":
        assert np.max(np.abs(got - want)) <= 1e-5
        return
    exact = x.reshape(x.shape[0], -1) @ W + (0.0 if b is None else b[None, :])
    diff = got != want
    # a mismatch is a rounding-boundary flip: the fp32-accumulated sum (absolute error ~ sqrt(d_in) * 2^-24 for
    # unit-scale terms) fell on the other side of a bf16 midpoint; still half a step from the float64 value, and rare
    assert np.all(np.abs(got - exact)[diff] <= bf16_ulp(exact)[diff] * 0.5 + 4e-6)
    assert np.all(np.abs(got - want)[diff] <= bf16_ulp(want)[diff] + 4e-6)
    assert diff.mean() < 5e-3, diff.mean()


def test_compress_writes_rows_of_a_strided_cache_in_place(esa):
    say("compress into cache rows, batch=2")
    rng = np.random.default_rng(3)
    B, S, t0, l_c, hk, d, d_c = 2, 96, 40, 24, 2, 64, 32
    K = rng.standard_normal((B, S, hk, d)).astype(np.float32)
    W = (rng.standard_normal((hk * d, d_c)) / np.sqrt(hk * d)).astype(np.float32)
    cache = torch.full((B, S, d_c), 7.0, dtype=torch.float32, device="cuda")
    esa.esa_compress(torch.from_numpy(K).cuda()[:, t0:t0 + l_c], torch.from_numpy(W).cuda(), out=cache[:, t0:t0 + l_c])
    got = cache.cpu().numpy()
    assert np.all(got[:, :t0] == 7.0) and np.all(got[:, t0 + l_c:] == 7.0)
    for b in range(B):
        want = orc.compress(K[b, t0:t0 + l_c].astype(np.float64), W.astype(np.float64), None, "f32")
        assert np.max(np.abs(got[b, t0:t0 + l_c] - want)) <= 1e-5


@pytest.mark.parametrize("dtype,B,n_tok,hq,hk,d,d_c,packed", [
    ("bf16", 1, 512, 32, 8, 128, 128, True),      # the chunk of configuration 3: one launch for both
    ("bf16", 2, 37, 8, 4, 128, 64, True),         # ragged token count, batched
    ("bf16", 1, 1, 32, 8, 128, 128, True),        # decode: one workgroup per output
    ("bf16", 2, 3, 32, 8, 128, 128, True),        # three tokens, batched: the same kernel
    ("bf16", 3, 4, 8, 4, 128, 64, True),          # four tokens (its limit), short reductions
    ("bf16", 5, 2, 8, 4, 128, 64, True),          # batch of five: back to the matrix-core kernel
    ("bf16", 1, 5, 8, 4, 128, 64, True),          # five tokens: back to the matrix-core kernel
    ("bf16", 1, 40, 4, 2, 64, 32, True),          # d_in not a multiple of 512: one launch each
    ("bf16", 1, 40, 8, 4, 128, 64, False),        # row-major weights
    ("f32", 2, 24, 4, 2, 64, 32, False)])
def test_compress_qk_equals_two_compress_calls(esa, dtype, B, n_tok, hq, hk, d, d_c, packed):
    say(f"compress_qk dtype={dtype} B={B} n_tok={n_tok} hq={hq} hk={hk} d={d} d_c={d_c} packed={packed}")
    rng = np.random.default_rng(90 + n_tok + hq)
    S, t0 = n_tok + 11, 5
    q = orc.round_to_storage(rng.standard_normal((B, n_tok, hq, d)), dtype)
    Kc = orc.round_to_storage(rng.standard_normal((B, S, hk, d)), dtype)
    Wq = orc.round_to_storage(rng.standard_normal((hq * d, d_c)) / np.sqrt(hq * d), dtype)
    Wk = orc.round_to_storage(rng.standard_normal((hk * d, d_c)) / np.sqrt(hk * d), dtype)
    bq = orc.round_to_storage(rng.standard_normal(d_c) * 0.1, dtype)
    qd, Kd, Wqd, Wkd, bqd = (f64_to_dev(a, dtype) for a in (q, Kc, Wq, Wk, bq))
    if packed:
        Wqd, Wkd = esa.esa_pack_weights(Wqd), esa.esa_pack_weights(Wkd)
    cache = torch.full((B, S, d_c), 3.0, dtype=qd.dtype, device="cuda")
    cache_ref = cache.clone()
    got_q, got_k = esa.esa_compress_qk(qd, Wqd, Kd[:, t0:t0 + n_tok], Wkd, bias_q=bqd, out_k=cache[:, t0:t0 + n_tok])
    ref_q = esa.esa_compress(qd, Wqd, bias=bqd)
    esa.esa_compress(Kd[:, t0:t0 + n_tok], Wkd, out=cache_ref[:, t0:t0 + n_tok])
    assert torch.equal(got_q, ref_q) and torch.equal(cache, cache_ref)     # the same arithmetic, bit for bit
    assert got_k.data_ptr() == cache[:, t0:t0 + n_tok].data_ptr()
    tol = 1e-5 if dtype == "f32" else None
    for b in range(B):
        want_q = orc.compress(q[b].reshape(n_tok, -1), Wq, bq, dtype)
        want_k = orc.compress(Kc[b, t0:t0 + n_tok].reshape(n_tok, -1), Wk, None, dtype)
        for got, want in ((to_f64(got_q[b]), want_q), (to_f64(cache[b, t0:t0 + n_tok]), want_k)):
            if tol is not None:
                assert np.max(np.abs(got - want)) <= tol
            else:       # within one bf16 step (fp32 accumulation crossing a rounding midpoint)
                assert np.all(np.abs(got - want) <= bf16_ulp(want) * 1.001)


# ------------------------------------------------------------------------------------------ score
@pytest.mark.parametrize("dtype,l_c,n,d_c,m_lo", [
    ("f32", 128, 1632, 32, 32), ("f32", 1, 999, 32, 0), ("f32", 5, 63, 16, 7),
    ("bf16", 512, 30080, 128, 128), ("bf16", 1, 20000, 128, 128), ("bf16", 37, 2433, 128, 5),
    ("bf16", 64, 4097, 64, 0), ("bf16", 700, 5003, 128, 3), ("bf16", 1024, 33, 128, 0)])
def test_score_matches_oracle_and_keeps_eq4_invariants(esa, dtype, l_c, n, d_c, m_lo):
    say(f"score dtype={dtype} l_c={l_c} n={n} d_c={d_c} m_lo={m_lo}")
    rng = np.random.default_rng(l_c * 31 + n)
    qc = orc.round_to_storage(rng.standard_normal((l_c, d_c)) * 1.5, dtype)
    kc = orc.round_to_storage(rng.standard_normal((m_lo + n + 9, d_c)), dtype)
    kc[m_lo + rng.choice(n, size=min(n, 5), replace=False)] *= 6.0          # a few dominant tokens
    kc = orc.round_to_storage(kc, dtype)
    want = orc.importance(qc, kc[m_lo:m_lo + n])
    got = to_f64(esa.esa_score(f64_to_dev(qc, dtype), f64_to_dev(kc, dtype), m_lo, m_lo + n))
    assert got.shape == (n,)
    assert np.max(np.abs(got - want)) <= F_TOL[dtype]
    assert np.all(got <= 0.0) and got.max() == 0.0
    S = qc @ kc[m_lo:m_lo + n].T
    srt = np.sort(S, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 10 * F_TOL[dtype] if n > 1 else np.ones(l_c, bool)
    assert np.all(got[np.argmax(S, axis=1)[clear]] == 0.0)                 # each row's best token scores exactly 0


@pytest.mark.parametrize("eps", [1, 3])
def test_score_with_proximity_influence(esa, eps):
    say(f"score eps={eps}")
    rng = np.random.default_rng(eps)
    qc = orc.round_to_storage(rng.standard_normal((16, 32)), "f32")
    kc = orc.round_to_storage(rng.standard_normal((3000, 32)), "f32")
    want = orc.proximity(orc.importance(qc, kc[10:2990]), eps)
    got = to_f64(esa.esa_score(f64_to_dev(qc, "f32"), f64_to_dev(kc, "f32"), 10, 2990, eps=eps))
    assert np.max(np.abs(got - want)) <= F_TOL["f32"]


@pytest.mark.parametrize("B,n,d_c,m_lo", [(4, 20000, 128, 128), (16, 9000, 128, 0), (3, 5003, 64, 7), (2, 4100, 256, 3)])
def test_score_one_current_token_batched(esa, B, n, d_c, m_lo):
    """The decode shape of the score call (one current token per sequence) with several independent
    sequences in one call: every batch element against the oracle, and Eq. 4's invariants per row."""
    say(f"score l_c=1 batch={B} n={n} d_c={d_c} m_lo={m_lo}")
    rng = np.random.default_rng(B * 1009 + n)
    qc = orc.round_to_storage(rng.standard_normal((B, 1, d_c)) * 1.5, "bf16")
    kc = orc.round_to_storage(rng.standard_normal((B, m_lo + n + 5, d_c)), "bf16")
    got = to_f64(esa.esa_score(f64_to_dev(qc, "bf16"), f64_to_dev(kc, "bf16"), m_lo, m_lo + n))
    assert got.shape == (B, n)
    for b in range(B):
        want = orc.importance(qc[b], kc[b, m_lo:m_lo + n])
        assert np.max(np.abs(got[b] - want)) <= F_TOL["bf16"], b
        assert np.all(got[b] <= 0.0) and got[b].max() == 0.0


def test_score_batched(esa):
    say("score batch=3")
    rng = np.random.default_rng(9)
    B, l_c, S, d_c = 3, 4, 1500, 32
    qc = orc.round_to_storage(rng.standard_normal((B, l_c, d_c)), "bf16")
    kc = orc.round_to_storage(rng.standard_normal((B, S, d_c)), "bf16")
    got = to_f64(esa.esa_score(f64_to_dev(qc, "bf16"), f64_to_dev(kc, "bf16"), 100, 1400))
    for b in range(B):
        assert np.max(np.abs(got[b] - orc.importance(qc[b], kc[b, 100:1400]))) <= F_TOL["bf16"]


@pytest.mark.parametrize("seed", range(10))
def test_score_random_shapes(esa, seed):
    rng = np.random.default_rng(7000 + seed)
    dtype = str(rng.choice(["bf16", "bf16", "f32"]))
    d_c = int(rng.choice([128, 128, 64, 32])) if dtype == "bf16" else int(rng.choice([32, 48]))
    B, l_c = int(rng.choice([1, 2, 3])), int(rng.choice([1, 5, 31, 64, 200, 513]))
    n, m_lo, eps = int(rng.integers(1, 9000)), int(rng.integers(0, 300)), int(rng.choice([0, 0, 1, 4]))
    say(f"score random seed={seed}: dtype={dtype} B={B} l_c={l_c} n={n} d_c={d_c} m_lo={m_lo} eps={eps}")
    qc = orc.round_to_storage(rng.standard_normal((B, l_c, d_c)), dtype)
    kc = orc.round_to_storage(rng.standard_normal((B, m_lo + n + 3, d_c)), dtype)
    got = to_f64(esa.esa_score(f64_to_dev(qc, dtype), f64_to_dev(kc, dtype), m_lo, m_lo + n, eps=eps))
    for b in range(B):
        want = orc.proximity(orc.importance(qc[b], kc[b, m_lo:m_lo + n]), eps)
        assert np.max(np.abs(got[b] - want)) <= F_TOL[dtype]


def test_score_batched_on_the_matrix_core_path_with_proximity_influence(esa):
    say("score batch=3 d_c=128 l_c=100 eps=2")
    rng = np.random.default_rng(10)
    B, l_c, S, d_c, eps = 3, 100, 3300, 128, 2
    qc = orc.round_to_storage(rng.standard_normal((B, l_c, d_c)), "bf16")
    kc = orc.round_to_storage(rng.standard_normal((B, S, d_c)), "bf16")
    plain = to_f64(esa.esa_score(f64_to_dev(qc, "bf16"), f64_to_dev(kc, "bf16"), 128, 3203))
    pooled = to_f64(esa.esa_score(f64_to_dev(qc, "bf16"), f64_to_dev(kc, "bf16"), 128, 3203, eps=eps))
    for b in range(B):
        F = orc.importance(qc[b], kc[b, 128:3203])
        assert np.max(np.abs(plain[b] - F)) <= F_TOL["bf16"]
        assert np.max(np.abs(pooled[b] - orc.proximity(F, eps))) <= F_TOL["bf16"]


def test_score_batched_with_two_blocks_of_queries(esa):
    """Batch of two on the matrix-core path with more than 512 queries: the second sweep reads each batch entry's
    own copy of the query fragments, one per block of queries."""
    say("score batch=2 d_c=128 l_c=600")
    rng = np.random.default_rng(11)
    B, l_c, S, d_c = 2, 600, 2600, 128
    qc = orc.round_to_storage(rng.standard_normal((B, l_c, d_c)), "bf16")
    kc = orc.round_to_storage(rng.standard_normal((B, S, d_c)), "bf16")
    got = to_f64(esa.esa_score(f64_to_dev(qc, "bf16"), f64_to_dev(kc, "bf16"), 64, 2575))
    for b in range(B):
        F = orc.importance(qc[b], kc[b, 64:2575])
        assert np.max(np.abs(got[b] - F)) <= F_TOL["bf16"]
        assert np.all(got[b] <= 0.0) and got[b].max() == 0.0


# ------------------------------------------------------------------------------------------ score + select + gather fused
@pytest.mark.parametrize("dtype,B,l_c,n,d_c,m_lo,k,h_kv,d,pad", [
    ("bf16", 1, 512, 30080, 128, 128, 2048, 8, 128, 0),     # matrix-core sweeps, histogram left by the second one
    ("bf16", 2, 100, 5003, 128, 7, 300, 2, 128, 64),        # batched, ragged share of the last workgroup, padded cache rows
    ("bf16", 1, 1, 20000, 128, 128, 2048, 8, 128, 0),       # decode: histogram left by the subtract pass
    ("bf16", 4, 1, 9000, 128, 0, 500, 2, 64, 0),            # decode, batched
    ("bf16", 1, 700, 70000, 128, 3, 2048, 2, 128, 0),       # more than one block of queries
    ("bf16", 1, 33, 4097, 64, 0, 64, 2, 64, 4),             # plain score kernel; cache rows not 16-byte aligned
    ("f32", 2, 16, 3000, 32, 10, 256, 2, 64, 0),            # fp32: plain kernels throughout
    ("bf16", 1, 64, 900, 128, 5, 2048, 2, 128, 0),          # k covers the middle: nothing is scored
    ("bf16", 1, 512, 2049, 128, 128, 2048, 8, 128, 0)])     # all but one selected
def test_score_select_gather_equals_the_three_calls(esa, dtype, B, l_c, n, d_c, m_lo, k, h_kv, d, pad):
    say(f"fused score+select+gather dtype={dtype} B={B} l_c={l_c} n={n} d_c={d_c} m_lo={m_lo} k={k} h_kv={h_kv} d={d} pad={pad}")
    rng = np.random.default_rng(l_c * 7 + n + k)
    S = m_lo + n + 9
    qc = orc.round_to_storage(rng.standard_normal((B, l_c, d_c)) * 1.5, dtype)
    kc = orc.round_to_storage(rng.standard_normal((B, S, d_c)), dtype)
    qd, kd = f64_to_dev(qc, dtype), f64_to_dev(kc, dtype)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    Kbuf = torch.randn((B, S, h_kv * d + pad), generator=torch.Generator().manual_seed(3)).to(tdt).cuda()
    Vbuf = torch.randn((B, S, h_kv * d + pad), generator=torch.Generator().manual_seed(4)).to(tdt).cuda()
    Kc, Vc = Kbuf[:, :, :h_kv * d].unflatten(2, (h_kv, d)), Vbuf[:, :, :h_kv * d].unflatten(2, (h_kv, d))
    if B == 1:
        qd, kd, Kc, Vc = qd[0], kd[0], Kc[0], Vc[0]
    score, idx, ks, vs = esa.esa_score_select_gather(qd, kd, m_lo, m_lo + n, k, Kc, Vc)
    want_score = esa.esa_score(qd, kd, m_lo, m_lo + n)
    want_idx = esa.esa_select_topk(want_score, k, base=m_lo)
    want_ks, want_vs = esa.esa_gather_kv(Kc, Vc, want_idx)
    assert torch.equal(idx, want_idx)
    assert torch.equal(ks, want_ks) and torch.equal(vs, want_vs)
    if k < n:
        assert torch.equal(score, want_score)
    else:
        assert score is None
    # without the gather
    score2, idx2, ks2, vs2 = esa.esa_score_select_gather(qd, kd, m_lo, m_lo + n, k)
    assert torch.equal(idx2, want_idx) and ks2 is None and vs2 is None
    # and against the oracle (first batch element)
    F = orc.importance(qc[0], kc[0, m_lo:m_lo + n])
    if k < n:
        got_F = to_f64(score if B == 1 else score[0])
        assert np.max(np.abs(got_F - F)) <= F_TOL[dtype]
        srt = np.sort(F)[::-1]
        if srt[k - 1] - srt[k] > 4 * F_TOL[dtype]:          # the boundary is clear of rounding: the set is the oracle's
            assert np.array_equal((idx if B == 1 else idx[0]).cpu().numpy(), orc.select_topk(F, k, base=m_lo))


@pytest.mark.parametrize("B,l_c,n,d_c,eps", [(1, 512, 30080, 128, 3), (2, 1, 20000, 128, 2), (1, 33, 4097, 64, 1), (1, 16, 3000, 32, 5)])
def test_score_select_gather_with_proximity_influence_equals_the_three_calls(esa, B, l_c, n, d_c, eps):
    """Eq. 8 inside the fused call: the pooling pass leaves the selection's first histogram."""
    say(f"fused score+select+gather with eps={eps}: B={B} l_c={l_c} n={n} d_c={d_c}")
    rng = np.random.default_rng(n + eps)
    dtype = "f32" if d_c == 32 else "bf16"
    m_lo, k, h_kv, d = 9, 700, 2, 128
    qc = orc.round_to_storage(rng.standard_normal((B, l_c, d_c)) * 1.5, dtype)
    kc = orc.round_to_storage(rng.standard_normal((B, m_lo + n + 4, d_c)), dtype)
    qd, kd = f64_to_dev(qc, dtype), f64_to_dev(kc, dtype)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    Kc = torch.randn((B, m_lo + n + 4, h_kv, d), generator=torch.Generator().manual_seed(7)).to(tdt).cuda()
    Vc = torch.randn((B, m_lo + n + 4, h_kv, d), generator=torch.Generator().manual_seed(8)).to(tdt).cuda()
    score, idx, ks, vs = esa.esa_score_select_gather(qd, kd, m_lo, m_lo + n, k, Kc, Vc, eps=eps)
    want_score = esa.esa_score(qd, kd, m_lo, m_lo + n, eps=eps)
    want_idx = esa.esa_select_topk(want_score, k, base=m_lo)
    want_ks, want_vs = esa.esa_gather_kv(Kc, Vc, want_idx)
    assert torch.equal(score, want_score) and torch.equal(idx, want_idx)
    assert torch.equal(ks, want_ks) and torch.equal(vs, want_vs)
    for b in range(B):
        F = orc.proximity(orc.importance(qc[b], kc[b, m_lo:m_lo + n]), eps)
        assert np.max(np.abs(to_f64(score[b]) - F)) <= F_TOL[dtype]


def test_score_select_gather_with_massive_ties(esa):
    """Identical compressed keys give identical scores: the tie rule (lower position first) decides the
    whole selection, and the gathering write pass copies long runs of consecutive rows."""
    say("fused score+select+gather, tied scores")
    rng = np.random.default_rng(99)
    l_c, n, d_c, m_lo, k, h_kv, d = 64, 6000, 128, 11, 1500, 2, 128
    qc = orc.round_to_storage(rng.standard_normal((l_c, d_c)), "bf16")
    # four distinct compressed keys, each repeated over a quarter of the cache
    kc = np.repeat(orc.round_to_storage(rng.standard_normal((4, d_c)), "bf16"), (m_lo + n + 3) // 4 + 1, axis=0)[:m_lo + n + 3]
    Kc = torch.randn((m_lo + n + 3, h_kv, d), generator=torch.Generator().manual_seed(5)).to(torch.bfloat16).cuda()
    Vc = torch.randn((m_lo + n + 3, h_kv, d), generator=torch.Generator().manual_seed(6)).to(torch.bfloat16).cuda()
    score, idx, ks, vs = esa.esa_score_select_gather(f64_to_dev(qc, "bf16"), f64_to_dev(kc, "bf16"), m_lo, m_lo + n, k, Kc, Vc)
    F = orc.importance(qc, kc[m_lo:m_lo + n])
    assert np.unique(F).size <= 4
    want = orc.select_topk(to_f64(score), k, base=m_lo)       # ties are exact on both sides: the GPU's own scores decide
    assert np.array_equal(idx.cpu().numpy(), want)
    assert torch.equal(ks, Kc[idx.long()]) and torch.equal(vs, Vc[idx.long()])


# ------------------------------------------------------------------------------------------ attend
@pytest.mark.parametrize("dtype,H,H_kv,d,S,t0,l_C,l_I,l_L,n_sel", [
    ("f32", 4, 2, 64, 2048, 1920, 128, 32, 256, 256),
    ("f32", 4, 2, 64, 300, 0, 128, 32, 256, 0),          # first chunk: only the causal part
    ("f32", 4, 2, 64, 300, 128, 128, 32, 256, 0),        # I and L touch, empty middle
    ("f32", 2, 1, 32, 500, 499, 1, 4, 16, 9),            # decode step
    ("bf16", 32, 8, 128, 8192, 7680, 512, 128, 2048, 2048),
    ("bf16", 32, 8, 128, 6000, 5999, 1, 128, 2048, 2048),
    ("bf16", 32, 8, 128, 40, 39, 1, 128, 2048, 0),       # decode, fewer keys than one slice
    ("bf16", 8, 8, 128, 3000, 2990, 3, 16, 500, 200),    # three current tokens (causal inside C), G = 1
    ("bf16", 16, 2, 128, 2500, 2485, 15, 8, 300, 1000),  # G = 8, largest chunk of the decode kernel
    ("bf16", 4, 2, 128, 150000, 149999, 1, 128, 120000, 0),  # slices near their maximum length
    ("bf16", 4, 2, 128, 150000, 149999, 1, 128, 140000, 0),  # more keys than the decode kernel covers
    ("bf16", 8, 2, 128, 1500, 1203, 77, 16, 100, 55),    # ragged sizes
    ("bf16", 4, 4, 128, 2300, 2000, 300, 16, 700, 333),  # matrix-core kernel, one query head per KV head
    ("bf16", 4, 2, 128, 1900, 1700, 200, 16, 500, 100),  # two query heads per KV head
    ("bf16", 16, 2, 128, 1000, 936, 64, 16, 400, 77),    # eight query heads per KV head
    ("bf16", 4, 4, 64, 900, 800, 100, 8, 64, 31)])
def test_attend_matches_oracle(esa, dtype, H, H_kv, d, S, t0, l_C, l_I, l_L, n_sel):
    say(f"attend dtype={dtype} H={H} H_kv={H_kv} d={d} t0={t0} l_C={l_C} l_I={l_I} l_L={l_L} n_sel={n_sel}")
    rng = np.random.default_rng(t0 + l_C)
    t1 = t0 + l_C
    Q = orc.round_to_storage(rng.standard_normal((l_C, H, d)), dtype)
    K = orc.round_to_storage(rng.standard_normal((t1, H_kv, d)), dtype)
    V = orc.round_to_storage(rng.standard_normal((t1, H_kv, d)), dtype)
    i_end, l_start = segment_bounds(t0, l_I, l_L)
    sel = np.sort(rng.choice(np.arange(i_end, l_start), n_sel, replace=False)).astype(np.int32) if n_sel else \
        np.empty(0, np.int32)
    scale = 1.0 / np.sqrt(d)
    want_O, want_lse = orc.attend(Q, K, V, t0, l_I, l_L, sel, scale)
    Kd, Vd = f64_to_dev(K, dtype), f64_to_dev(V, dtype)
    ks = vs = None
    if n_sel:
        ks, vs = esa.esa_gather_kv(Kd, Vd, torch.from_numpy(sel).cuda())
    Qd = f64_to_dev(Q, dtype)
    O, lse = esa.esa_attend(Qd, Kd, Vd, t0, l_I, l_L, ks, vs, return_lse=True)
    assert np.max(np.abs(to_f64(O) - want_O)) <= O_TOL[dtype]
    assert np.max(np.abs(to_f64(lse) - want_lse)) <= (1e-5 if dtype == "f32" else 1e-3)
    # the two-call form (Algorithm 1's split: keys known before the selection, then the selected keys)
    esa.esa_attend_local(Qd, Kd, Vd, t0, l_I, l_L)
    O2, lse2 = esa.esa_attend_finish(Qd, Kd, Vd, t0, l_I, l_L, ks, vs, return_lse=True)
    assert np.max(np.abs(to_f64(O2) - want_O)) <= O_TOL[dtype]
    assert np.max(np.abs(to_f64(lse2) - want_lse)) <= (1e-5 if dtype == "f32" else 1e-3)


@pytest.mark.parametrize("seed", range(16))
def test_attend_random_shapes_all_three_forms(esa, seed):
    """Seeded random geometry (segment lengths, chunk length, group size, batch, selection size): the one-call,
    two-call and index-driven forms against the oracle."""
    rng = np.random.default_rng(9000 + seed)
    G = int(rng.choice([1, 2, 4, 8]))
    H_kv = int(rng.choice([1, 2, 3]))
    H, d, B = G * H_kv, 128, int(rng.choice([1, 1, 2, 3]))
    l_C = int(rng.choice([1, 7, 16, 33, 64, 100, 257, 300]))
    l_I, l_L = int(rng.integers(0, 70)), int(rng.integers(0, 400))
    t0 = int(rng.integers(0, 1500))
    i_end, l_start = segment_bounds(t0, l_I, l_L)
    n_mid = l_start - i_end
    n_sel = int(rng.integers(0, min(n_mid, 300) + 1)) if n_mid > 0 else 0
    say(f"attend random seed={seed}: B={B} H={H} H_kv={H_kv} t0={t0} l_C={l_C} l_I={l_I} l_L={l_L} n_sel={n_sel}")
    S = t0 + l_C
    Q = orc.round_to_storage(rng.standard_normal((B, l_C, H, d)), "bf16")
    K = orc.round_to_storage(rng.standard_normal((B, S, H_kv, d)), "bf16")
    V = orc.round_to_storage(rng.standard_normal((B, S, H_kv, d)), "bf16")
    sel = np.stack([np.sort(rng.choice(np.arange(i_end, l_start), n_sel, replace=False)) for _ in range(B)]).astype(np.int32) \
        if n_sel else np.empty((B, 0), np.int32)
    Qd, Kd, Vd, idx = f64_to_dev(Q, "bf16"), f64_to_dev(K, "bf16"), f64_to_dev(V, "bf16"), torch.from_numpy(sel).cuda()
    ks = vs = None
    if n_sel:
        ks, vs = esa.esa_gather_kv(Kd, Vd, idx)
    O1 = esa.esa_attend(Qd, Kd, Vd, t0, l_I, l_L, ks, vs)
    esa.esa_attend_local(Qd, Kd, Vd, t0, l_I, l_L)
    O2 = esa.esa_attend_finish(Qd, Kd, Vd, t0, l_I, l_L, ks, vs)
    O3 = esa.esa_attend_indexed(Qd, Kd, Vd, t0, l_I, l_L, idx)
    for b in range(B):
        want, _ = orc.attend(Q[b], K[b], V[b], t0, l_I, l_L, sel[b], 1.0 / np.sqrt(d))
        for O in (O1, O2, O3):
            assert np.max(np.abs(to_f64(O[b]) - want)) <= O_TOL["bf16"]


@pytest.mark.parametrize("vmax", [1.0e5, 1.0e29])
def test_attend_with_values_beyond_the_fp16_range_on_the_multi_slice_path(esa, vmax):
    """bf16 storage admits |v| far above 65504: key slices of the matrix-core kernel must hand such
    rows to the merge without overflow (one dominant key per row makes the output as large as the value)."""
    say(f"attend bf16 with |V| up to {vmax:g}, key slices merged")
    rng = np.random.default_rng(8181)
    H, H_kv, d, t0, l_C, l_I, l_L, n_sel = 8, 2, 128, 1400, 96, 16, 300, 200
    S = t0 + l_C
    u = rng.standard_normal(d)
    u /= np.linalg.norm(u)
    Q = orc.round_to_storage(rng.standard_normal((l_C, H, d)) + 6.0 * u, "bf16")     # every query leans towards u
    K = rng.standard_normal((S, H_kv, d))
    K[3] = 8.0 * np.sqrt(d) * u                                  # an initial token every query attends to almost alone
    K = orc.round_to_storage(K, "bf16")
    V = rng.standard_normal((S, H_kv, d))
    big = np.concatenate([[3], rng.choice(S, 40, replace=False)])
    V[big] *= vmax / 2.0                                         # some rows huge, most of unit scale
    V = orc.round_to_storage(np.clip(V, -vmax, vmax), "bf16")
    i_end, l_start = segment_bounds(t0, l_I, l_L)
    sel = np.sort(rng.choice(np.arange(i_end, l_start), n_sel, replace=False)).astype(np.int32)
    want, _ = orc.attend(Q, K, V, t0, l_I, l_L, sel, 1.0 / np.sqrt(d))
    Qd, Kd, Vd = f64_to_dev(Q, "bf16"), f64_to_dev(K, "bf16"), f64_to_dev(V, "bf16")
    ks, vs = esa.esa_gather_kv(Kd, Vd, torch.from_numpy(sel).cuda())
    O1 = esa.esa_attend(Qd, Kd, Vd, t0, l_I, l_L, ks, vs)
    esa.esa_attend_local(Qd, Kd, Vd, t0, l_I, l_L)
    O2 = esa.esa_attend_finish(Qd, Kd, Vd, t0, l_I, l_L, ks, vs)
    for O in (O1, O2):
        got = to_f64(O)
        assert np.all(np.isfinite(got))
        # bf16 probabilities (8 significant bits) times values of this size: the error of an output element
        # scales with the values its row mixes, so rows are judged relative to their largest output
        row_scale = np.maximum(1.0, np.abs(want).max(axis=2, keepdims=True))
        assert np.all(np.abs(got - want) <= O_TOL["bf16"] * row_scale)
    assert np.abs(want).max() > 70000.0


def test_attend_batched(esa):
    say("attend batch=2 decode")
    rng = np.random.default_rng(77)
    B, H, H_kv, d, S, l_I, l_L, n_sel = 2, 8, 2, 128, 3000, 16, 256, 128
    t0 = S - 1
    Q = orc.round_to_storage(rng.standard_normal((B, 1, H, d)), "bf16")
    K = orc.round_to_storage(rng.standard_normal((B, S, H_kv, d)), "bf16")
    V = orc.round_to_storage(rng.standard_normal((B, S, H_kv, d)), "bf16")
    sel = np.stack([np.sort(rng.choice(np.arange(l_I, t0 - l_L), n_sel, replace=False)) for _ in range(B)]).astype(np.int32)
    Kd, Vd = f64_to_dev(K, "bf16"), f64_to_dev(V, "bf16")
    ks, vs = esa.esa_gather_kv(Kd, Vd, torch.from_numpy(sel).cuda())
    O = esa.esa_attend(f64_to_dev(Q, "bf16"), Kd, Vd, t0, l_I, l_L, ks, vs)
    for b in range(B):
        want, _ = orc.attend(Q[b], K[b], V[b], t0, l_I, l_L, sel[b], 1.0 / np.sqrt(d))
        assert np.max(np.abs(to_f64(O[b]) - want)) <= O_TOL["bf16"]


def test_attend_in_two_calls_batched_with_the_local_part_on_a_side_stream(esa):
    say("attend batch=3, l_C=96, local part on a second stream")
    rng = np.random.default_rng(78)
    B, H, H_kv, d, l_C, l_I, l_L, n_sel = 3, 8, 2, 128, 96, 16, 300, 200
    t0 = 1400
    Q = orc.round_to_storage(rng.standard_normal((B, l_C, H, d)), "bf16")
    K = orc.round_to_storage(rng.standard_normal((B, t0 + l_C, H_kv, d)), "bf16")
    V = orc.round_to_storage(rng.standard_normal((B, t0 + l_C, H_kv, d)), "bf16")
    sel = np.stack([np.sort(rng.choice(np.arange(l_I, t0 - l_L), n_sel, replace=False)) for _ in range(B)]).astype(np.int32)
    Qd, Kd, Vd = f64_to_dev(Q, "bf16"), f64_to_dev(K, "bf16"), f64_to_dev(V, "bf16")
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    side.wait_stream(main)
    with torch.cuda.stream(side):
        esa.esa_attend_local(Qd, Kd, Vd, t0, l_I, l_L)
    ks, vs = esa.esa_gather_kv(Kd, Vd, torch.from_numpy(sel).cuda())
    main.wait_stream(side)
    O, lse = esa.esa_attend_finish(Qd, Kd, Vd, t0, l_I, l_L, ks, vs, return_lse=True)
    for b in range(B):
        want, want_lse = orc.attend(Q[b], K[b], V[b], t0, l_I, l_L, sel[b], 1.0 / np.sqrt(d))
        assert np.max(np.abs(to_f64(O[b]) - want)) <= O_TOL["bf16"]
        assert np.max(np.abs(to_f64(lse[b]) - want_lse)) <= 1e-3


@pytest.mark.parametrize("dtype,H,H_kv,d,t0,l_C,l_I,l_L,n_sel", [
    ("bf16", 8, 2, 128, 1400, 96, 16, 300, 200),     # matrix-core kernel
    ("bf16", 32, 8, 128, 5000, 512, 128, 2048, 2048),
    ("bf16", 8, 2, 128, 40, 32, 16, 300, 0),         # early chunk: no middle tokens, I and L touch
    ("bf16", 8, 2, 128, 0, 64, 16, 300, 0),          # first chunk: nothing but C
    ("f32", 4, 2, 64, 900, 100, 8, 64, 31),          # plain kernel, one launch per part
    ("bf16", 8, 2, 128, 2999, 1, 16, 256, 128)])     # decode shape
def test_attend_with_the_position_encoding_of_section_3_2(esa, dtype, H, H_kv, d, t0, l_C, l_I, l_L, n_sel):
    """Algorithm 1's grouping with separately encoded queries and keys: esa_attend_local on the in-order
    encoding of L and C, esa_attend_finish on queries at the fixed position w against I and M_k at
    position 0.  The encodings are applied on the host (the library takes Q and K as given)."""
    say(f"attend, Section 3.2 encodings, dtype={dtype} H={H} H_kv={H_kv} d={d} t0={t0} l_C={l_C} n_sel={n_sel}")
    rng = np.random.default_rng(1000 + t0 + l_C)
    S, w, base = t0 + l_C, 4096.0, 500000.0
    q_raw = rng.standard_normal((l_C, H, d))
    K_raw = rng.standard_normal((S, H_kv, d))
    V = orc.round_to_storage(rng.standard_normal((S, H_kv, d)), dtype)
    i_end, l_start = segment_bounds(t0, l_I, l_L)
    n_L = t0 - l_start
    K_l = np.zeros_like(K_raw)
    K_l[l_start:] = orc.rope(K_raw[l_start:], np.arange(n_L + l_C), base)
    q_l = orc.round_to_storage(orc.rope(q_raw, n_L + np.arange(l_C), base), dtype)
    q_g = orc.round_to_storage(orc.rope(q_raw, np.full(l_C, w), base), dtype)
    K_l, K_g = orc.round_to_storage(K_l, dtype), orc.round_to_storage(K_raw, dtype)
    sel = np.sort(rng.choice(np.arange(i_end, l_start), n_sel, replace=False)).astype(np.int32) if n_sel else \
        np.empty(0, np.int32)
    scale = 1.0 / np.sqrt(d)
    want_O, want_lse = orc.attend_two_encodings(q_l, q_g, K_l, K_g, V, t0, l_I, l_L, sel, scale)
    Vd, Kld, Kgd = f64_to_dev(V, dtype), f64_to_dev(K_l, dtype), f64_to_dev(K_g, dtype)
    ks = vs = None
    if n_sel:
        ks, vs = esa.esa_gather_kv(Kgd, Vd, torch.from_numpy(sel).cuda())
    esa.esa_attend_local(f64_to_dev(q_l, dtype), Kld, Vd, t0, l_I, l_L, split=esa.ESA_SPLIT_ALGORITHM1)
    O, lse = esa.esa_attend_finish(f64_to_dev(q_g, dtype), Kgd, Vd, t0, l_I, l_L, ks, vs, return_lse=True,
                                   split=esa.ESA_SPLIT_ALGORITHM1)
    assert np.max(np.abs(to_f64(O) - want_O)) <= O_TOL[dtype]
    assert np.max(np.abs(to_f64(lse) - want_lse)) <= (1e-5 if dtype == "f32" else 1e-3)


@pytest.mark.parametrize("dtype,B,n_tok,heads,d,pos0,step,pad", [
    ("bf16", 1, 700, 8, 128, 0.0, 1.0, 0),           # local keys in order from 0
    ("bf16", 1, 512, 32, 128, 2048.0, 1.0, 0),       # local queries behind a window of 2048
    ("bf16", 2, 96, 8, 128, 4096.0, 0.0, 64),        # global queries at w; padded rows; batched
    ("bf16", 1, 33, 3, 64, 130000.0, 1.0, 8),        # large absolute positions
    ("bf16", 2, 20, 2, 64, 5.0, 1.0, 3),             # odd row stride: the element-wise path
    ("f32", 2, 100, 4, 64, 7.5, 1.0, 0),
    ("f32", 1, 9, 3, 128, 300.0, 1.0, 1),
    ("f32", 1, 5, 2, 32, 0.0, 0.0, 0)])              # position 0: identity
def test_rope_matches_the_fp64_definition_rounded_once(esa, dtype, B, n_tok, heads, d, pos0, step, pad):
    say(f"rope dtype={dtype} B={B} n_tok={n_tok} heads={heads} d={d} pos0={pos0} step={step} pad={pad}")
    rng = np.random.default_rng(4000 + n_tok + heads)
    base = 500000.0
    x = orc.round_to_storage(rng.standard_normal((B, n_tok, heads, d)), dtype)
    want = np.stack([orc.round_to_storage(orc.rope(x[b], pos0 + step * np.arange(n_tok), base), dtype) for b in range(B)])
    buf = torch.zeros((B, n_tok, heads * d + pad), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32,
                      device="cuda")
    xd = buf[:, :, :heads * d].unflatten(2, (heads, d))
    xd.copy_(f64_to_dev(x, dtype))
    got = to_f64(esa.esa_rope(xd, pos0, step, base))
    # one rounding on each side of the same fp64 value: equal except where the two fp64 results differ in
    # their last bits across a rounding boundary
    ulp = np.abs(want) * (2.0 ** -7 if dtype == "bf16" else 2.0 ** -23)
    assert np.all(np.abs(got - want) <= ulp)
    assert np.count_nonzero(got != want) <= 1e-5 * want.size
    if pos0 == 0.0 and step == 0.0:
        assert np.array_equal(got, x)
    esa.esa_rope(xd, pos0, step, base, out=xd)      # in place, strided rows
    assert np.array_equal(to_f64(xd), got)
    assert pad == 0 or float(buf[:, :, heads * d:].abs().max()) == 0.0


@pytest.mark.parametrize("dtype,B,H,H_kv,d,t0,l_C,l_I,l_L,n_sel", [
    ("bf16", 1, 8, 2, 128, 1400, 96, 16, 300, 200),     # matrix-core kernel
    ("bf16", 1, 32, 8, 128, 5000, 512, 128, 2048, 2048),
    ("bf16", 2, 8, 2, 128, 1400, 80, 16, 300, 150),     # batched
    ("bf16", 1, 8, 2, 128, 40, 32, 16, 300, 0),         # early chunk: no middle tokens, I and L touch
    ("bf16", 1, 8, 2, 128, 0, 64, 16, 300, 0),          # first chunk: nothing but C
    ("f32", 1, 4, 2, 64, 900, 100, 8, 64, 31),          # plain kernel, one launch per part
    ("f32", 2, 4, 2, 64, 900, 7, 8, 64, 31),
    ("bf16", 1, 8, 2, 128, 2999, 1, 16, 256, 128),      # decode shape: split-key kernel, one launch per part
    ("bf16", 3, 32, 8, 128, 6000, 2, 128, 2048, 2048),  # decode, batched, Llama shape
    ("bf16", 2, 8, 2, 128, 40, 3, 16, 300, 0),          # decode in an early chunk: the global part is I alone
    ("bf16", 1, 8, 8, 128, 0, 5, 16, 300, 0)])          # decode at the very start: no global keys at all
def test_attend_reencoded_from_unencoded_queries_and_caches(esa, dtype, B, H, H_kv, d, t0, l_C, l_I, l_L, n_sel):
    """Section 3.2 inside the library: un-encoded q, K cache and gathered keys in, esa_attend_reencoded
    encodes and attends; the oracle applies the section's positions in fp64 without intermediate rounding."""
    say(f"attend re-encoded dtype={dtype} B={B} H={H} H_kv={H_kv} d={d} t0={t0} l_C={l_C} l_I={l_I} l_L={l_L} n_sel={n_sel}")
    rng = np.random.default_rng(2000 + t0 + l_C + B)
    S, w, base = t0 + l_C + 3, 4096.0, 500000.0
    q = orc.round_to_storage(rng.standard_normal((B, l_C, H, d)), dtype)
    K = orc.round_to_storage(rng.standard_normal((B, S, H_kv, d)), dtype)
    V = orc.round_to_storage(rng.standard_normal((B, S, H_kv, d)), dtype)
    i_end, l_start = segment_bounds(t0, l_I, l_L)
    sel = np.stack([np.sort(rng.choice(np.arange(i_end, l_start), n_sel, replace=False)) for _ in range(B)]).astype(np.int32) \
        if n_sel else np.empty((B, 0), np.int32)
    scale = 1.0 / np.sqrt(d)
    qd, Kd, Vd = f64_to_dev(q, dtype), f64_to_dev(K, dtype), f64_to_dev(V, dtype)
    K_before = Kd.clone()
    ks = vs = None
    if n_sel:
        ks, vs = esa.esa_gather_kv(Kd, Vd, torch.from_numpy(sel).cuda())
    O, lse = esa.esa_attend_reencoded(qd, Kd, Vd, t0, l_I, l_L, ks, vs, w, base, return_lse=True)
    for b in range(B):
        want_O, want_lse = orc.attend_reencoded(q[b], K[b], V[b], t0, l_I, l_L, sel[b], scale, w, base)
        assert np.max(np.abs(to_f64(O[b]) - want_O)) <= O_TOL[dtype]
        assert np.max(np.abs(to_f64(lse[b]) - want_lse)) <= (2e-5 if dtype == "f32" else 4e-3)
    assert torch.equal(Kd, K_before)                  # the caller's cache stays un-encoded


@pytest.mark.parametrize("dtype,B,H,H_kv,d,t0,l_C,l_I,l_L,n_sel", [
    ("bf16", 1, 32, 8, 128, 5999, 1, 128, 2048, 2048),   # decode: indices followed inside the kernel
    ("bf16", 3, 8, 2, 128, 2999, 2, 16, 256, 128),
    ("bf16", 2, 8, 2, 128, 1400, 96, 16, 300, 200),      # matrix-core kernel: gathers into its workspace first
    ("f32", 1, 4, 2, 64, 900, 100, 8, 64, 31),           # plain kernel
    ("bf16", 1, 8, 2, 128, 300, 1, 16, 400, 0)])         # nothing selected
def test_attend_indexed_equals_gather_then_attend(esa, dtype, B, H, H_kv, d, t0, l_C, l_I, l_L, n_sel):
    say(f"attend_indexed dtype={dtype} B={B} H={H} H_kv={H_kv} d={d} t0={t0} l_C={l_C} n_sel={n_sel}")
    rng = np.random.default_rng(2000 + t0 + l_C)
    S = t0 + l_C
    Q = orc.round_to_storage(rng.standard_normal((B, l_C, H, d)), dtype)
    K = orc.round_to_storage(rng.standard_normal((B, S, H_kv, d)), dtype)
    V = orc.round_to_storage(rng.standard_normal((B, S, H_kv, d)), dtype)
    i_end, l_start = segment_bounds(t0, l_I, l_L)
    sel = np.stack([np.sort(rng.choice(np.arange(i_end, l_start), n_sel, replace=False)) for _ in range(B)]).astype(np.int32) \
        if n_sel else np.empty((B, 0), np.int32)
    Qd, Kd, Vd = f64_to_dev(Q, dtype), f64_to_dev(K, dtype), f64_to_dev(V, dtype)
    idx = torch.from_numpy(sel).cuda()
    if B == 1:
        Qd, Kd, Vd, idx = Qd[0], Kd[0], Vd[0], idx[0]
    ks = vs = None
    if n_sel:
        ks, vs = esa.esa_gather_kv(Kd, Vd, idx)
    want_O, want_lse = esa.esa_attend(Qd, Kd, Vd, t0, l_I, l_L, ks, vs, return_lse=True)
    O, lse = esa.esa_attend_indexed(Qd, Kd, Vd, t0, l_I, l_L, idx, return_lse=True)
    assert torch.equal(O, want_O) and torch.equal(lse, want_lse)       # the same arithmetic in the same order
    for b in range(B):
        o64, _ = orc.attend(Q[b], K[b], V[b], t0, l_I, l_L, sel[b], 1.0 / np.sqrt(d))
        got = to_f64(O if B == 1 else O[b])
        assert np.max(np.abs(got - o64)) <= O_TOL[dtype]


@pytest.mark.parametrize("l_C", [1, 3, 96])
def test_attend_indexed_clamps_indices_that_leave_the_cache(esa, l_C):
    """Entries below 0 or at or beyond the local window's start cannot be selected tokens; the kernels
    clamp them into [0, l_start) instead of following them (decode kernel and matrix-core kernel alike)."""
    say(f"attend_indexed with out-of-range entries, l_C={l_C}")
    rng = np.random.default_rng(31 + l_C)
    H, H_kv, d, t0, l_I, l_L, n_sel = 8, 2, 128, 1500, 16, 300, 200
    S = t0 + l_C
    bf = torch.bfloat16
    q = torch.from_numpy(rng.standard_normal((l_C, H, d)).astype(np.float32)).cuda().to(bf)
    K = torch.from_numpy(rng.standard_normal((S, H_kv, d)).astype(np.float32)).cuda().to(bf)
    V = torch.from_numpy(rng.standard_normal((S, H_kv, d)).astype(np.float32)).cuda().to(bf)
    i_end, l_start = segment_bounds(t0, l_I, l_L)
    sel = np.sort(rng.choice(np.arange(i_end, l_start), n_sel, replace=False)).astype(np.int64)
    bad = sel.copy()
    bad[[0, 7, 64, 65, 130, 199]] = [-5, -(2 ** 31), l_start, 2 ** 31 - 1, S + 100000, l_start + 1]
    clamped = np.clip(bad, 0, l_start - 1).astype(np.int32)
    got = esa.esa_attend_indexed(q, K, V, t0, l_I, l_L, torch.from_numpy(bad.astype(np.int32)).cuda())
    want = esa.esa_attend_indexed(q, K, V, t0, l_I, l_L, torch.from_numpy(clamped).cuda())
    assert torch.equal(got, want)


# ------------------------------------------------------------------------------------------ whole steps
def _check_step(esa, layer, dev, kc64, kc_dev, t0, two_calls=False, eps=0):
    cfg = layer.cfg
    O, lse, sel, F, qc = oracle_step(layer, kc64, t0, eps=eps)
    g = gpu_step(esa, dev, cfg, t0, kc_dev, two_calls=two_calls, eps=eps)
    got_idx = g["idx"].cpu().numpy()
    assert np.array_equal(got_idx, sel), f"t0={t0}: selected sets differ in {np.sum(got_idx != sel)} slots"
    if g["score"] is not None:
        # End to end the score inherits the last-place differences of the GPU's own K' and Q': where the fp32
        # and the fp64 sum fall on opposite sides of a rounding boundary, one stored element differs by one
        # unit in the last place, which moves S[c, m] by |q'_cj| ulp(k'_mj).  The sanity bound here is a
        # quarter of the planted gap plus one such flip in the token's own row and one in the row that sets
        # mu_c; the bar for the score call itself is F_TOL, held by the stage-wise tests above, which feed it
        # the oracle's compressed vectors.
        want_F = orc.proximity(F, eps) if eps > 0 else F
        ulp = 2.0 ** -7 if cfg.dtype == "bf16" else 2.0 ** -23
        flip = float(np.max(np.abs(qc))) * ulp * float(np.max(np.abs(kc64[:t0])))
        assert np.max(np.abs(to_f64(g["score"]) - want_F)) <= TAU_E2E[cfg.dtype] / 4 + 2 * flip
    assert np.max(np.abs(to_f64(g["O"]) - O)) <= O_TOL[cfg.dtype], f"t0={t0}"
    if g["k_sel"] is not None:
        assert torch.equal(g["k_sel"], dev["K"][torch.from_numpy(sel).long().cuda()])
    return g


def test_tiny_layer_full_prefill_fp32(esa):
    """Configuration 1, every chunk, the five calls chained on the GPU."""
    cfg = get_config("C1")
    layer = make_layer(cfg)
    steps = chunk_starts(cfg)
    replaced, kc64 = plant_gap(layer, steps, TAU_E2E["f32"])
    say(f"C1 prefill, {len(steps)} chunks, {replaced.shape[0]} rows replaced for the boundary gap")
    dev = layer_to_dev(layer)
    kc_dev = torch.zeros((cfg.S, cfg.d_c), dtype=torch.float32, device="cuda")
    n_selecting = 0
    for t0 in steps:
        g = _check_step(esa, layer, dev, kc64, kc_dev, t0)
        fused = gpu_step(esa, dev, cfg, t0, kc_dev, fused=True)      # one call for score + select + gather
        assert torch.equal(fused["idx"], g["idx"]) and torch.equal(fused["O"], g["O"])
        n_selecting += g["score"] is not None
        # needles of this chunk (those still in place) are all selected
        if t0 in layer.plan.positions and g["score"] is not None:
            needles = np.setdiff1d(layer.plan.positions[t0], replaced)
            assert set(needles.tolist()) <= set(g["idx"].cpu().numpy().tolist())
    assert n_selecting == 11
    # the cache now holds K' of every token, written chunk by chunk
    assert np.max(np.abs(to_f64(kc_dev) - kc64)) <= 1e-5


def test_k_covering_the_middle_reproduces_full_causal_attention_on_gpu(esa):
    """Eq. 1 with M_k = M equals Eq. 10: the GPU path against plain causal attention."""
    cfg = get_config("C1").scaled(S=768, k=4096, needles=0)
    layer = make_layer(cfg)
    say("C1-shaped, k covers the middle: GPU vs full causal attention")
    dev = layer_to_dev(layer)
    full = orc.full_causal_attention(layer.f64("Q"), layer.f64("K"), layer.f64("V"), 1.0 / np.sqrt(cfg.d))
    for t0 in chunk_starts(cfg):
        g = gpu_step(esa, dev, cfg, t0)
        assert np.max(np.abs(to_f64(g["O"]) - full[t0:t0 + cfg.l_C])) <= 1e-5, t0


@pytest.mark.parametrize("S,sample", [(8192, (0, 2048, 4608, 7680))])
def test_llama_shaped_layer_sampled_chunks_bf16(esa, S, sample):
    """Configuration 2's shape at a length the oracle finishes in seconds."""
    cfg = get_config("C2").scaled(S=S)
    layer = make_layer(cfg)
    replaced, kc64 = plant_gap(layer, sample, TAU_E2E["bf16"])
    say(f"C2-shaped S={S}, chunks {sample}, {replaced.shape[0]} rows replaced")
    dev = pack_layer_weights(esa, layer_to_dev(layer))
    kc_dev = esa.esa_compress(dev["K"], dev["W_k"])
    _assert_compressed_close(to_f64(kc_dev), kc64, layer.f64("K"), orc.widen(layer.W_k, "bf16"), None, "bf16")
    for t0 in sample:
        _check_step(esa, layer, dev, kc64, kc_dev, t0)


def test_decode_step_equals_one_token_chunk_bf16(esa):
    """Configuration 4's shape on a shorter cache, batch of 2 independent caches."""
    cfg = get_config("C4").scaled(S=20000)
    t0 = cfg.S - 1
    for b in range(2):
        layer = make_layer(cfg, batch=b)
        replaced, kc64 = plant_gap(layer, [t0], TAU_E2E["bf16"])
        say(f"decode S={cfg.S} batch element {b}, {replaced.shape[0]} rows replaced")
        dev = layer_to_dev(layer)
        kc_dev = esa.esa_compress(dev["K"][:t0], dev["W_k"])
        kc_dev = torch.cat([kc_dev, torch.zeros((1, cfg.d_c), dtype=kc_dev.dtype, device="cuda")])
        g = _check_step(esa, layer, dev, kc64, kc_dev, t0)
        needles = np.setdiff1d(layer.plan.positions[t0], replaced)
        assert set(needles.tolist()) <= set(g["idx"].cpu().numpy().tolist())


def test_decode_step_batched_call_chain_bf16(esa):
    """Configuration 4's shape on shorter caches: four independent sequences stacked and taken through
    the five calls as ONE batched call each (batch strides of every tensor in use), every sequence
    compared with its own oracle step."""
    cfg = get_config("C4").scaled(S=20000)
    t0, B = cfg.S - 1, 4
    layers, kc64s = [], []
    for b in range(B):
        layer = make_layer(cfg, batch=b)
        replaced, kc64 = plant_gap(layer, [t0], TAU_E2E["bf16"])
        say(f"batched decode S={cfg.S} batch element {b}, {replaced.shape[0]} rows replaced")
        layers.append(layer)
        kc64s.append(kc64)
    Q = torch.stack([to_dev(l.Q[t0:t0 + 1], "bf16") for l in layers])          # [B, 1, H, d]
    K = torch.stack([to_dev(l.K, "bf16") for l in layers])                      # [B, S, H_kv, d]
    V = torch.stack([to_dev(l.V, "bf16") for l in layers])
    Wq = esa.esa_pack_weights(to_dev(layers[0].W_q, "bf16"))
    Wk = esa.esa_pack_weights(to_dev(layers[0].W_k, "bf16"))
    kc = torch.zeros((B, cfg.S, cfg.d_c), dtype=torch.bfloat16, device="cuda")
    esa.esa_compress(K[:, :t0], Wk, out=kc[:, :t0])                             # state left by the earlier steps
    qc, _ = esa.esa_compress_qk(Q, Wq, K[:, t0:t0 + 1], Wk, out_k=kc[:, t0:t0 + 1])
    i_end, l_start = esa.esa_segments(t0, cfg.l_I, cfg.l_L)
    score = esa.esa_score(qc, kc, i_end, l_start)
    idx = esa.esa_select_topk(score, cfg.k, base=i_end)
    ks, vs = esa.esa_gather_kv(K, V, idx)
    O, lse = esa.esa_attend(Q, K, V, t0, cfg.l_I, cfg.l_L, ks, vs, return_lse=True)
    O_idx = esa.esa_attend_indexed(Q, K, V, t0, cfg.l_I, cfg.l_L, idx)
    assert idx.shape == (B, cfg.k) and O.shape == (B, 1, cfg.H, cfg.d)
    for b in range(B):
        want_O, want_lse, sel, F, _ = oracle_step(layers[b], kc64s[b], t0)
        got_idx = idx[b].cpu().numpy()
        assert np.array_equal(got_idx, sel), f"batch element {b}: {np.sum(got_idx != sel)} slots differ"
        assert np.max(np.abs(to_f64(score[b]) - F)) <= TAU_E2E["bf16"] / 4
        assert torch.equal(ks[b], K[b][torch.from_numpy(sel).long().cuda()])
        assert np.max(np.abs(to_f64(O[b]) - want_O)) <= O_TOL["bf16"], b
        assert np.max(np.abs(to_f64(O_idx[b]) - want_O)) <= O_TOL["bf16"], b
        assert np.max(np.abs(to_f64(lse[b]) - want_lse)) <= 1e-3, b


@pytest.mark.parametrize("eps", [3])
def test_whole_step_with_proximity_influence_selects_the_oracles_set(esa, eps):
    """Eq. 8 between Eq. 4 and Eq. 2 in a whole step: pooling makes neighbouring tokens share a score
    exactly, so the tie rule decides much of the selected set.  Configuration 1's shape, two steps."""
    cfg = get_config("C1")
    layer = make_layer(cfg)
    steps = [1152, 1920]
    replaced, kc64 = plant_gap(layer, steps, TAU_E2E["f32"], eps=eps)
    say(f"C1 steps {steps} with eps={eps}, {replaced.shape[0]} rows replaced")
    dev = layer_to_dev(layer)
    kc_dev = esa.esa_compress(dev["K"], dev["W_k"])
    for t0 in steps:
        g = _check_step(esa, layer, dev, kc64, kc_dev, t0, eps=eps)
        fused = gpu_step(esa, dev, cfg, t0, kc_dev, eps=eps, fused=True)      # pooling inside the fused call
        assert torch.equal(fused["idx"], g["idx"]) and torch.equal(fused["score"], g["score"])
        # the pooled scores are full of exact ties: fewer distinct values than tokens among the selected
        pooled = to_f64(g["score"])
        i_end, _ = segment_bounds(t0, cfg.l_I, cfg.l_L)
        assert np.unique(pooled[g["idx"].cpu().numpy() - i_end]).size < cfg.k // 2


@pytest.mark.parametrize("name,chunk", [("C2", -1), ("C3", -1), ("C5", -1), ("C4", -1), ("C6", -1),
                                        ("C3", 0), ("C3", 9), ("C3", 128)])
def test_full_size_step_in_the_benchmark_launch_configuration(esa, name, chunk):
    """The configurations at their full sizes, one step (chunk -1: the last, the one the benchmark times; for
    configuration 3 also the first chunk, the first chunk whose middle segment exceeds k, and a middle one),
    launched the way the benchmark launches it: packed weights, compressed-key cache filled 16384 tokens at a
    time.  One step is within the oracle's reach at any of these sizes, so every output is compared."""
    cfg = get_config(name)
    t0 = chunk_starts(cfg)[chunk]
    t1 = min(t0 + cfg.l_C, cfg.S)
    layer = make_layer(cfg, q_rows=(t0, t1))
    layer.q_row0 = t0
    # the oracle side only needs the tokens up to the end of the step
    layer.K, layer.V = layer.K[:max(t1, 1)], layer.V[:max(t1, 1)]
    cfg_step = cfg.scaled(S=t1)
    layer.cfg = cfg_step
    replaced, kc64 = plant_gap(layer, [t0], TAU_E2E["bf16"])
    say(f"{name} full size S={cfg.S}, step at t0={t0} (l_C={t1 - t0}, k={cfg.k}), {replaced.shape[0]} rows replaced")
    cfg = cfg_step
    dev = pack_layer_weights(esa, layer_to_dev(layer))
    kc_dev = torch.zeros((cfg.S, cfg.d_c), dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, t0, 16384):
        r1 = min(r0 + 16384, t0)
        esa.esa_compress(dev["K"][r0:r1], dev["W_k"], out=kc_dev[r0:r1])
    rows = np.unique(np.concatenate([np.arange(0, t0, 997), replaced[replaced < t0]])).astype(np.int64)
    if rows.size:
        _assert_compressed_close(to_f64(kc_dev[torch.from_numpy(rows).cuda()]), kc64[rows],
                                 orc.widen(layer.K[rows], "bf16").reshape(rows.shape[0], -1),
                                 orc.widen(layer.W_k, "bf16"), None, "bf16")
    g = _check_step(esa, layer, dev, kc64, kc_dev, t0, two_calls=True)
    one = gpu_step(esa, dev, cfg, t0, kc_dev)     # esa_attend in one call: same selection, same output to rounding
    assert torch.equal(one["idx"], g["idx"])
    assert float((one["O"].float() - g["O"].float()).abs().max()) <= O_TOL["bf16"]
    # score, select and gather as one call (the benchmark's default step): identical to the separate calls
    fused = gpu_step(esa, dev, cfg, t0, kc_dev, fused=True)
    assert torch.equal(fused["idx"], one["idx"]) and torch.equal(fused["O"], one["O"])
    if one["score"] is not None:
        assert torch.equal(fused["score"], one["score"])
        assert torch.equal(fused["k_sel"], one["k_sel"]) and torch.equal(fused["v_sel"], one["v_sel"])
    # ... and with the gather left to the attention kernel (what the benchmark times): the same arithmetic in the same order
    via_idx = gpu_step(esa, dev, cfg, t0, kc_dev, indexed=True)
    assert torch.equal(via_idx["idx"], one["idx"]) and torch.equal(via_idx["O"], one["O"]) and torch.equal(via_idx["lse"], one["lse"])
    if one["score"] is not None:
        assert torch.equal(via_idx["score"], one["score"])
    if t0 in layer.plan.positions:
        needles = np.setdiff1d(layer.plan.positions[t0], replaced)
        assert needles.size and set(needles.tolist()) <= set(g["idx"].cpu().numpy().tolist())
    else:
        assert chunk == 0 and g["idx"].numel() == 0          # the first chunk has no middle segment


@pytest.mark.parametrize("fused", [False, True, "indexed"])
def test_step_captured_as_a_graph_replays_identically(esa, fused):
    """The five calls captured once and replayed, with eager work and synchronisations between the
    replays: every replay must reproduce the eager result bit for bit (nothing in the library
    records a memset node, and no call keeps state between launches)."""
    cfg = get_config("C2").scaled(S=8192)
    layer = make_layer(cfg)
    say(f"graph capture of one step, C2-shaped S=8192, fused={fused}")
    dev = pack_layer_weights(esa, layer_to_dev(layer))
    t0 = 7680
    kc_dev = esa.esa_compress(dev["K"], dev["W_k"])
    form = dict(indexed=True) if fused == "indexed" else dict(fused=fused)
    eager = gpu_step(esa, dev, cfg, t0, kc_dev, **form)
    torch.cuda.synchronize()
    want_O, want_idx = eager["O"].clone(), eager["idx"].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gpu_step(esa, dev, cfg, t0, kc_dev, **form)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        g = gpu_step(esa, dev, cfg, t0, kc_dev, **form)
    for rep in range(4):
        g["O"].zero_()
        g["idx"].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g["O"], want_O) and torch.equal(g["idx"], want_idx), rep
        other = gpu_step(esa, dev, cfg, 4608, kc_dev)          # eager work between replays
        torch.cuda.synchronize()
        assert other["O"].shape == want_O.shape


def test_variant_calls_captured_as_a_graph_replay_identically(esa):
    """The calls beside the five (both compressions at once, index-driven attention, the two-call form,
    Section 3.2's re-encoding) captured in one graph: every replay reproduces the eager results."""
    say("graph capture of the variant calls")
    rng = np.random.default_rng(77)
    H, H_kv, d, d_c, t0, l_C, l_I, l_L, n_sel = 8, 2, 128, 64, 1400, 96, 16, 300, 200
    S = t0 + l_C
    bf = torch.bfloat16
    q = torch.from_numpy(rng.standard_normal((l_C, H, d)).astype(np.float32)).cuda().to(bf)
    K = torch.from_numpy(rng.standard_normal((S, H_kv, d)).astype(np.float32)).cuda().to(bf)
    V = torch.from_numpy(rng.standard_normal((S, H_kv, d)).astype(np.float32)).cuda().to(bf)
    Wq = esa.esa_pack_weights((torch.randn(H * d, d_c, device="cuda") / 32).to(bf))
    Wk = esa.esa_pack_weights((torch.randn(H_kv * d, d_c, device="cuda") / 16).to(bf))
    i_end, l_start = segment_bounds(t0, l_I, l_L)
    idx = torch.from_numpy(np.sort(rng.choice(np.arange(i_end, l_start), n_sel, replace=False)).astype(np.int32)).cuda()
    kc = torch.zeros((S, d_c), dtype=bf, device="cuda")

    def calls():
        qc, _ = esa.esa_compress_qk(q, Wq, K[t0:], Wk, out_k=kc[t0:])
        o_idx = esa.esa_attend_indexed(q, K, V, t0, l_I, l_L, idx)
        ks, vs = esa.esa_gather_kv(K, V, idx)
        esa.esa_attend_local(q, K, V, t0, l_I, l_L)
        o_two = esa.esa_attend_finish(q, K, V, t0, l_I, l_L, ks, vs)
        o_re = esa.esa_attend_reencoded(q, K, V, t0, l_I, l_L, ks, vs, 4096.0, 500000.0)
        return qc, o_idx, o_two, o_re

    want = [t.clone() for t in calls()]
    want_kc = kc.clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        got = calls()
    for rep in range(3):
        for t in got:
            t.zero_()
        kc.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for g, w in zip(got, want):
            assert torch.equal(g, w), rep
        assert torch.equal(kc, want_kc), rep
        calls()                                              # eager work between replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("l_C,pad,n_sel", [(64, 64, 100),      # matrix-core kernel, token rows wider than h_kv*d
                                           (64, 4, 100),       # rows not 16-byte aligned: the plain kernel
                                           (1, 64, 100),       # decode kernel
                                           (48, 64, 0)])
def test_attend_reads_caches_with_padded_token_rows(esa, l_C, pad, n_sel):
    """The caches as strided views (tok_stride > h_kv*d), for every attention form; the padding holds
    huge values that must never be read."""
    say(f"attend with padded token rows l_C={l_C} pad={pad} n_sel={n_sel}")
    rng = np.random.default_rng(600 + l_C + pad)
    H, H_kv, d, t0, l_I, l_L = 8, 2, 128, 900, 16, 200
    S = t0 + l_C
    q = orc.round_to_storage(rng.standard_normal((l_C, H, d)), "bf16")
    K = orc.round_to_storage(rng.standard_normal((S, H_kv, d)), "bf16")
    V = orc.round_to_storage(rng.standard_normal((S, H_kv, d)), "bf16")
    i_end, l_start = segment_bounds(t0, l_I, l_L)
    sel = np.sort(rng.choice(np.arange(i_end, l_start), n_sel, replace=False)).astype(np.int32) if n_sel else \
        np.empty(0, np.int32)

    def padded(x):
        buf = torch.full((S, H_kv * d + pad), 3.0e38, dtype=torch.bfloat16, device="cuda")
        view = buf[:, :H_kv * d].unflatten(1, (H_kv, d))
        view.copy_(f64_to_dev(x, "bf16"))
        return view

    Kd, Vd, qd = padded(K), padded(V), f64_to_dev(q, "bf16")
    assert Kd.stride(0) == H_kv * d + pad
    idx = torch.from_numpy(sel).cuda()
    ks, vs = esa.esa_gather_kv(Kd, Vd, idx) if n_sel else (None, None)
    want, want_lse = orc.attend(q, K, V, t0, l_I, l_L, sel, 1.0 / np.sqrt(d))
    O1, lse1 = esa.esa_attend(qd, Kd, Vd, t0, l_I, l_L, ks, vs, return_lse=True)
    esa.esa_attend_local(qd, Kd, Vd, t0, l_I, l_L)
    O2 = esa.esa_attend_finish(qd, Kd, Vd, t0, l_I, l_L, ks, vs)
    O3 = esa.esa_attend_indexed(qd, Kd, Vd, t0, l_I, l_L, idx if n_sel else None)
    for O in (O1, O2, O3):
        assert np.max(np.abs(to_f64(O) - want)) <= O_TOL["bf16"]
    assert np.max(np.abs(to_f64(lse1) - want_lse)) <= 1e-3


@pytest.mark.parametrize("dtype,n_tok,d_in,d_c,pad,packed", [("bf16", 70, 1024, 128, 64, True), ("bf16", 70, 1024, 128, 3, True),
                                                              ("bf16", 33, 256, 64, 8, False), ("f32", 20, 128, 32, 5, False)])
def test_compress_reads_rows_with_a_stride(esa, dtype, n_tok, d_in, d_c, pad, packed):
    """x as a strided view (ldx > d_in): aligned padding keeps the matrix-core kernel, odd padding takes the
    plain one; the padding holds huge values that must never be read."""
    say(f"compress strided rows dtype={dtype} n_tok={n_tok} d_in={d_in} d_c={d_c} pad={pad} packed={packed}")
    rng = np.random.default_rng(31 + n_tok + pad)
    x = orc.round_to_storage(rng.standard_normal((n_tok, d_in)), dtype)
    W = orc.round_to_storage(rng.standard_normal((d_in, d_c)) / np.sqrt(d_in), dtype)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    buf = torch.full((n_tok, d_in + pad), 3.0e38, dtype=tdt, device="cuda")
    xd = buf[:, :d_in]
    xd.copy_(f64_to_dev(x, dtype))
    Wd = f64_to_dev(W, dtype)
    if packed:
        Wd = esa.esa_pack_weights(Wd)
    got = to_f64(esa.esa_compress(xd, Wd))
    want = orc.compress(x, W, None, dtype)
    if dtype == "f32":
        assert np.max(np.abs(got - want)) <= 1e-5
    else:
        assert np.all(np.abs(got - want) <= bf16_ulp(want) * 1.001)
