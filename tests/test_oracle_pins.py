"""Pins for the CPU oracle: everything here checks oracle/flashblock_oracle.py against
something that is not the oracle - hand-derived closed forms, library routines (torch SDPA,
scipy softmax / logsumexp) on the special cases that are plain attention, brute force on tiny
inputs, and the figures the paper prints in Table 5.  CPU only."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import flashblock_oracle as orc
from paper_2602_05305_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TOL = 1e-12


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def _sdpa(Q, K, V, scale):
    """Library pin: torch's scaled_dot_product_attention in float64 (GQA by repeating KV)."""
    q, k, v = (torch.from_numpy(np.asarray(x, dtype=np.float64)) for x in (Q, K, V))
    G = q.shape[1] // k.shape[1]
    k = k.repeat_interleave(G, dim=1)
    v = v.repeat_interleave(G, dim=1)
    return torch.nn.functional.scaled_dot_product_attention(q, k, v, scale=scale).numpy()


def _small_problem(seed, B=2, Hq=4, Hkv=2, d=16, P=37, Bq=5):
    Q = _rand((B, Hq, Bq, d), seed)
    Kp, Vp = _rand((B, Hkv, P, d), seed + 1), _rand((B, Hkv, P, d), seed + 2)
    Kb, Vb = _rand((B, Hkv, Bq, d), seed + 3), _rand((B, Hkv, Bq, d), seed + 4)
    return Q, Kp, Vp, Kb, Vb


# ------------------------------------------------------------------ hand-derived closed forms
def test_hand_case_scale_and_weights():
    """golden/softmax_hand_cases.txt case A: pins scale = 1/sqrt(head_dim), the sign of the
    exponent and which operand the weights multiply."""
    q = np.zeros((1, 1, 1, 4)); q[0, 0, 0, 0] = 2.0
    K = np.zeros((1, 1, 2, 4)); K[0, 0, 0, 0] = math.log(3.0)
    V = np.zeros((1, 1, 2, 4)); V[0, 0, 0, 0] = 1.0; V[0, 0, 1, 1] = 1.0
    p = orc.partial(q, K, V)
    A = orc.normalized(p)
    assert np.allclose(A[0, 0, 0], [0.75, 0.25, 0.0, 0.0], atol=TOL)
    assert abs(p["lse"][0, 0, 0] - math.log(4.0)) < TOL
    assert abs(p["m"][0, 0, 0] - math.log(3.0)) < TOL
    # unnormalised o is paired with m: o = e^{s-m} v summed = (1, 1/3, 0, 0)
    assert np.allclose(p["o"][0, 0, 0], [1.0, 1.0 / 3.0, 0, 0], atol=TOL)
    a, logz = orc.full_attention(q, K, V)
    assert np.allclose(a[0, 0, 0], [0.75, 0.25, 0, 0], atol=TOL) and abs(logz[0, 0, 0] - math.log(4)) < TOL


def test_hand_case_merge():
    """case B: external {k1}, internal {k2}: Eq. 5 and Eq. 9 both give (0.75, 0.25, 0, 0)."""
    q = np.zeros((1, 1, 1, 4)); q[0, 0, 0, 0] = 2.0
    K1 = np.zeros((1, 1, 1, 4)); K1[0, 0, 0, 0] = math.log(3.0)
    V1 = np.zeros((1, 1, 1, 4)); V1[0, 0, 0, 0] = 1.0
    K2 = np.zeros((1, 1, 1, 4)); V2 = np.zeros((1, 1, 1, 4)); V2[0, 0, 0, 1] = 1.0
    ext, inn = orc.partial(q, K1, V1), orc.partial(q, K2, V2)
    assert abs(ext["lse"][0, 0, 0] - math.log(3.0)) < TOL and abs(inn["lse"][0, 0, 0]) < TOL
    out, L = orc.merge(ext, inn)
    assert np.allclose(out[0, 0, 0], [0.75, 0.25, 0, 0], atol=TOL) and abs(L[0, 0, 0] - math.log(4)) < TOL
    out2, L2 = orc.merge_uz(ext, inn)
    assert np.allclose(out2, out, atol=TOL) and np.allclose(L2, L, atol=TOL)
    # the external side must weigh 3x the internal side, not the other way round
    out_swapped, _ = orc.merge(inn, ext)
    assert np.allclose(out_swapped, out, atol=TOL)  # symmetric operands, same key union


def test_zero_keys_uniform_weights():
    """case C: K = 0 => A_out = mean(V_prefix), L_out = ln P, out = weighted mean of means."""
    B, Hq, Hkv, d, P, Bq = 1, 4, 2, 8, 23, 3
    Q = _rand((B, Hq, Bq, d), 1)
    Vp, Vb = _rand((B, Hkv, P, d), 2), _rand((B, Hkv, Bq, d), 3)
    ext = orc.partial(Q, np.zeros((B, Hkv, P, d)), Vp)
    inn = orc.partial(Q, np.zeros((B, Hkv, Bq, d)), Vb)
    A = orc.normalized(ext)
    for h in range(Hq):
        assert np.allclose(A[0, h], Vp[0, h // 2].mean(axis=0)[None], atol=TOL)
    assert np.allclose(ext["lse"], math.log(P), atol=TOL)
    out, L = orc.merge(ext, inn)
    for h in range(Hq):
        want = (P * Vp[0, h // 2].mean(0) + Bq * Vb[0, h // 2].mean(0)) / (P + Bq)
        assert np.allclose(out[0, h], want[None], atol=TOL)
    assert np.allclose(L, math.log(P + Bq), atol=TOL)


def test_constant_values_and_dominant_key():
    Q, Kp, Vp, Kb, Vb = _small_problem(10)
    c = 3.25
    out, _ = orc.merge(orc.partial(Q, Kp, np.full_like(Vp, c)), orc.partial(Q, Kb, np.full_like(Vb, c)))
    assert np.allclose(out, c, atol=1e-12)
    # one key aligned with the query with a huge score dominates
    d = Q.shape[-1]
    Kp2 = Kp.copy()
    Kp2[0, 0, 7] = Q[0, 0, 2] * (60.0 * math.sqrt(d) / np.dot(Q[0, 0, 2], Q[0, 0, 2]))  # score 60
    out2, _ = orc.merge(orc.partial(Q, Kp2, Vp), orc.partial(Q, Kb, Vb))
    assert np.allclose(out2[0, 0, 2], Vp[0, 0, 7], atol=1e-9)


def test_shift_invariance_and_convexity():
    """Adding a constant c to every score of a row (via an extra feature) moves L by c and
    leaves A unchanged; every output lies in the convex hull of the values."""
    Q, Kp, Vp, Kb, Vb = _small_problem(20)
    d = Q.shape[-1]
    c = 1.7
    scale = 1.0 / math.sqrt(d)
    Qa = np.concatenate([Q, np.full(Q.shape[:-1] + (1,), c / scale)], axis=-1)
    Ka = np.concatenate([Kp, np.ones(Kp.shape[:-1] + (1,))], axis=-1)
    p0, p1 = orc.partial(Q, Kp, Vp, scale), orc.partial(Qa, Ka, Vp, scale)
    assert np.allclose(p1["lse"], p0["lse"] + c, atol=1e-12)
    assert np.allclose(orc.normalized(p1), orc.normalized(p0), atol=1e-12)
    A = orc.normalized(p0)
    for h in range(Q.shape[1]):
        lo, hi = Vp[:, h // 2].min(axis=1), Vp[:, h // 2].max(axis=1)
        assert (A[:, h] >= lo[:, None] - 1e-12).all() and (A[:, h] <= hi[:, None] + 1e-12).all()


# ------------------------------------------------------------------ library pins
@pytest.mark.parametrize("seed,shape", [(1, dict()), (2, dict(B=1, Hq=6, Hkv=6, d=8, P=64, Bq=8)),
                                        (3, dict(B=1, Hq=8, Hkv=2, d=32, P=130, Bq=1))])
def test_refresh_step_equals_plain_attention_sdpa(seed, shape):
    """Eq. 5: at a refresh step merge(external, internal) is plain attention over
    [prefix | block]; checked against torch SDPA (float64) and scipy logsumexp."""
    Q, Kp, Vp, Kb, Vb = _small_problem(seed, **shape)
    d = Q.shape[-1]
    scale = 1.0 / math.sqrt(d)
    out, L = orc.merge(orc.partial(Q, Kp, Vp), orc.partial(Q, Kb, Vb))
    Kall, Vall = np.concatenate([Kp, Kb], axis=2), np.concatenate([Vp, Vb], axis=2)
    assert np.allclose(out, _sdpa(Q, Kall, Vall, scale), atol=1e-12)
    G = Q.shape[1] // Kp.shape[1]
    s = np.einsum("bhqd,bhkd->bhqk", Q, np.repeat(Kall, G, axis=1)) * scale
    assert np.allclose(L, scipy.special.logsumexp(s, axis=-1), atol=1e-12)
    a, logz = orc.full_attention(Q, Kall, Vall)
    assert np.allclose(a, out, atol=1e-12) and np.allclose(logz, L, atol=1e-12)
    w = scipy.special.softmax(s, axis=-1)
    assert np.allclose(a, np.einsum("bhqk,bhkd->bhqd", w, np.repeat(Vall, G, axis=1)), atol=1e-12)


def test_explicit_scale_overrides_default():
    Q, Kp, Vp, _, _ = _small_problem(5)
    out = orc.normalized(orc.partial(Q, Kp, Vp, scale=0.3))
    assert np.allclose(out, _sdpa(Q, Kp, Vp, 0.3), atol=1e-12)
    assert not np.allclose(out, _sdpa(Q, Kp, Vp, 0.25), atol=1e-6)


def _augmented(Q_stale, Q_now, K_out, V_out, K_in, V_in):
    """Plain attention whose scores are q_stale.k for J_out keys and q_now.k for J_in keys:
    queries [q_stale | q_now], J_out keys [k | 0], J_in keys [0 | k]."""
    Qa = np.concatenate([Q_stale, Q_now], axis=-1)
    Ko = np.concatenate([K_out, np.zeros_like(K_out)], axis=-1)
    Ki = np.concatenate([np.zeros_like(K_in), K_in], axis=-1)
    return Qa, np.concatenate([Ko, Ki], axis=2), np.concatenate([V_out, V_in], axis=2)


def test_reuse_step_equals_augmented_sdpa_and_bruteforce():
    """A reuse step (Eq. 9 with a stale external pair) is plain attention on an augmented
    problem; checked against torch SDPA and against the oracle's own exponential-sum form."""
    Q0, Kp, Vp, Kb0, Vb0 = _small_problem(30)
    d = Q0.shape[-1]
    scale = 1.0 / math.sqrt(d)
    steps = [(Q0, Kb0, Vb0)]
    for t in range(1, 4):
        steps.append(tuple(x + 0.3 * _rand(x.shape, 40 + 3 * t + i) for i, x in enumerate(steps[-1])))
    res = orc.run_block_dense(Kp, Vp, steps, R=4)
    assert [r["refreshed"] for r in res] == [True, False, False, False]
    for t, (Q, Kb, Vb) in enumerate(steps):
        Qa, Ka, Va = _augmented(Q0, Q, Kp, Vp, Kb, Vb)
        assert np.allclose(res[t]["out"], _sdpa(Qa, Ka, Va, scale), atol=1e-12), t
        assert np.allclose(res[t]["out"], orc.stale_query_bruteforce(Q0, Q, Kp, Vp, Kb, Vb), atol=1e-12)
    # reuse steps really differ from exact attention when the query moved
    exact, _ = orc.full_attention(steps[2][0], np.concatenate([Kp, steps[2][1]], 2),
                                  np.concatenate([Vp, steps[2][2]], 2))
    assert np.abs(res[2]["out"] - exact).max() > 1e-3


@pytest.mark.parametrize("R", [1, 2, 3, 8])
def test_refresh_schedule_and_interval_one(R):
    """R = 1 => every step is plain attention; otherwise steps with t mod R == 0 are, and the
    cache in force at step t is the one computed at the last refresh step."""
    Q0, Kp, Vp, Kb0, Vb0 = _small_problem(50)
    scale = 1.0 / math.sqrt(Q0.shape[-1])
    steps = [(Q0, Kb0, Vb0)]
    for t in range(1, 6):
        steps.append(tuple(x + 0.2 * _rand(x.shape, 60 + 3 * t + i) for i, x in enumerate(steps[-1])))
    res = orc.run_block_dense(Kp, Vp, steps, R=R)
    for t, (Q, Kb, Vb) in enumerate(steps):
        t_r = (t // R) * R
        assert res[t]["refreshed"] == (t % R == 0)
        Qa, Ka, Va = _augmented(steps[t_r][0], Q, Kp, Vp, Kb, Vb)
        assert np.allclose(res[t]["out"], _sdpa(Qa, Ka, Va, scale), atol=1e-12)
        if t % R == 0:
            assert np.allclose(res[t]["out"], _sdpa(Q, np.concatenate([Kp, Kb], 2),
                                                    np.concatenate([Vp, Vb], 2), scale), atol=1e-12)


def test_zero_perturbation_reuse_is_exact():
    Q0, Kp, Vp, Kb0, Vb0 = _small_problem(70)
    res = orc.run_block_dense(Kp, Vp, [(Q0, Kb0, Vb0)] * 4, R=4)
    exact, _ = orc.full_attention(Q0, np.concatenate([Kp, Kb0], 2), np.concatenate([Vp, Vb0], 2))
    for r in res:
        assert np.allclose(r["out"], exact, atol=1e-12)


# ------------------------------------------------------------------ structure
def test_chunk_associativity_any_order():
    """Folding per-chunk partials with merge_partials in any order equals one partial over the
    whole key set (pins the split-KV combine and selected (+) residual)."""
    Q, Kp, Vp, _, _ = _small_problem(80, P=53)
    whole = orc.partial(Q, Kp, Vp)
    cuts = [0, 7, 8, 29, 53]
    chunks = [orc.partial(Q, Kp[:, :, a:b], Vp[:, :, a:b]) for a, b in zip(cuts[:-1], cuts[1:])]
    for order in ([0, 1, 2, 3], [3, 1, 0, 2], [2, 3, 1, 0]):
        acc = orc.empty_partial(*Q.shape)
        for i in order:
            acc = orc.merge_partials(acc, chunks[i])
        assert np.allclose(acc["lse"], whole["lse"], atol=1e-12)
        assert np.allclose(orc.normalized(acc), orc.normalized(whole), atol=1e-12)
        assert np.allclose(acc["m"], whole["m"], atol=0)
        assert np.allclose(acc["o"], whole["o"], atol=1e-12)


def test_empty_sets():
    Q, Kp, Vp, Kb, Vb = _small_problem(90)
    B, Hq, Bq, d = Q.shape
    e = orc.partial(Q, Kp[:, :, :0], Vp[:, :, :0])
    assert np.isneginf(e["lse"]).all() and np.isneginf(e["m"]).all() and (e["o"] == 0).all()
    inn = orc.partial(Q, Kb, Vb)
    out, L = orc.merge(e, inn)                       # prefix_len = 0 => out = A_in exactly
    assert np.allclose(out, orc.normalized(inn), atol=0) and np.allclose(L, inn["lse"], atol=0)
    out2, L2 = orc.merge(e, e)
    assert (out2 == 0).all() and np.isneginf(L2).all() and not np.isnan(out2).any()
    m2 = orc.merge_partials(e, inn)
    assert np.allclose(m2["o"], inn["o"]) and np.allclose(m2["lse"], inn["lse"])


def test_single_key_block_closed_form():
    """Bq = 1: out = (Z_out A_out + e^{s} v) / (Z_out + e^{s})."""
    Q, Kp, Vp, Kb, Vb = _small_problem(95, B=1, Hq=2, Hkv=2, d=8, P=11, Bq=1)
    ext = orc.partial(Q, Kp, Vp)
    out, _ = orc.merge(ext, orc.partial(Q, Kb, Vb))
    for h in range(2):
        s = float(Q[0, h, 0] @ Kb[0, h, 0]) / math.sqrt(8)
        Z = math.exp(ext["lse"][0, h, 0])
        want = (Z * orc.normalized(ext)[0, h, 0] + math.exp(s) * Vb[0, h, 0]) / (Z + math.exp(s))
        assert np.allclose(out[0, h, 0], want, atol=1e-12)


def test_large_scores_stay_finite():
    """Eq. 8-9 exist for stability: scores near +-600 must not overflow in merge()."""
    Q, Kp, Vp, Kb, Vb = _small_problem(97, d=4)
    out, L = orc.merge(orc.partial(Q * 40, Kp * 10, Vp), orc.partial(Q * 40, Kb * 10, Vb))
    assert np.isfinite(out).all() and np.isfinite(L).all()
    ref = _sdpa(Q * 40, np.concatenate([Kp, Kb], 2) * 10, np.concatenate([Vp, Vb], 2), 0.5)
    assert np.allclose(out, ref, atol=1e-10)


# ------------------------------------------------------------------ sparse variant
def test_pool_and_topk_hand_example():
    """4 key blocks of 2 tokens (last block short), d = 1: pooled means and scores by hand."""
    K = np.array([1.0, 3.0, -2.0, 0.0, 5.0, 5.0, 4.0]).reshape(1, 1, 7, 1)
    pooled = orc.pool_keys(K, 2)
    assert np.allclose(pooled[0, 0, :, 0], [2.0, -1.0, 5.0, 4.0])
    Q = np.array([1.0, 3.0]).reshape(1, 1, 2, 1)              # q-bar = 2 => scores 4,-2,10,8
    assert np.allclose(orc.select_scores(Q, pooled)[0, 0], [4.0, -2.0, 10.0, 8.0])
    assert orc.select_topk(Q, K, 2, 2)[0, 0].tolist() == [2, 3]
    assert orc.select_topk(Q, K, 2, 3)[0, 0].tolist() == [0, 2, 3]
    assert orc.select_topk(-Q, K, 2, 1)[0, 0].tolist() == [1]
    assert orc.select_topk(Q, K, 2, 9)[0, 0].tolist() == [0, 1, 2, 3]     # clamped


def test_topk_ties_go_to_lower_index_and_bruteforce():
    K = np.zeros((1, 1, 8, 2)); K[0, 0, :, 0] = [1, 1, 2, 2, 1, 1, 2, 2]   # blocks: 1,2,1,2
    Q = np.ones((1, 1, 1, 2))
    assert orc.select_topk(Q, K, 2, 1)[0, 0].tolist() == [1]
    assert orc.select_topk(Q, K, 2, 3)[0, 0].tolist() == [0, 1, 3]
    rng = np.random.default_rng(5)
    Qr, Kr = rng.standard_normal((2, 4, 3, 8)), rng.standard_normal((2, 2, 50, 8))
    idx = orc.select_topk(Qr, Kr, 4, 5)
    for b in range(2):
        for h in range(4):
            sc = [float(Kr[b, h // 2, c * 4:min(50, c * 4 + 4)].mean(0) @ Qr[b, h].mean(0)) for c in range(13)]
            assert idx[b, h].tolist() == sorted(np.argsort(-np.array(sc), kind="stable")[:5].tolist())


def test_block_mass_closed_forms():
    """Attention mass per key block.  (1) All-zero keys: uniform weights, mass = block size / P,
    short last block included.  (2) d = 1 hand case: q = ln 2, keys (0, 1 | 1, 2): weights
    proportional to 1, 2, 2, 4, so the two blocks of two hold 3/9 and 6/9 (scale 1).  (3) One key far
    above the rest takes (almost) all the mass of its block, for every head that reads it (GQA)."""
    Q = np.random.default_rng(1).standard_normal((2, 4, 3, 8))
    m = orc.block_mass(Q, np.zeros((2, 2, 7, 8)), 3)
    assert m.shape == (2, 4, 3) and np.allclose(m, np.array([3, 3, 1]) / 7.0)
    q = np.full((1, 1, 2, 1), np.log(2.0))
    K = np.array([0.0, 1.0, 1.0, 2.0]).reshape(1, 1, 4, 1)
    assert np.allclose(orc.block_mass(q, K, 2, scale=1.0)[0, 0], [3.0 / 9.0, 6.0 / 9.0])
    K = np.zeros((1, 2, 8, 4)); K[0, 1, 5] = 50.0
    m = orc.block_mass(np.ones((1, 4, 2, 4)), K, 4, scale=1.0)
    assert np.allclose(m[0, :2], 0.5) and np.allclose(m[0, 2:], [0.0, 1.0], atol=1e-12)


def test_block_mass_matches_library_softmax_and_sums_to_one():
    """Against scipy's softmax on scores written out here with einsum (GQA: head h reads KV head
    h // G), summed per block by reduceat; each (batch, head) row of masses sums to 1."""
    from scipy.special import softmax
    rng = np.random.default_rng(8)
    Q, K = rng.standard_normal((2, 6, 5, 16)), rng.standard_normal((2, 3, 45, 16))
    m = orc.block_mass(Q, K, 8)
    Kh = np.repeat(K, 2, axis=1)                               # KV head of each query head
    pr = softmax(np.einsum("bhid,bhjd->bhij", Q, Kh) / 4.0, axis=-1)
    want = np.add.reduceat(pr, np.arange(0, 45, 8), axis=-1).mean(axis=2)
    assert np.allclose(m, want, atol=1e-13)
    assert np.allclose(m.sum(-1), 1.0)


def test_select_topk_scores_hand_and_bruteforce():
    sc = np.array([[[0.1, 0.4, 0.4, 0.05, 0.05]]])
    assert orc.select_topk_scores(sc, 1)[0, 0].tolist() == [1]               # tie -> lower index
    assert orc.select_topk_scores(sc, 2)[0, 0].tolist() == [1, 2]
    assert orc.select_topk_scores(sc, 4)[0, 0].tolist() == [0, 1, 2, 3]      # tie among the last again
    assert orc.select_topk_scores(sc, 9)[0, 0].tolist() == [0, 1, 2, 3, 4]   # clamped
    r = np.random.default_rng(3).standard_normal((2, 3, 17))
    idx = orc.select_topk_scores(r, 6)
    for b in range(2):
        for h in range(3):
            assert idx[b, h].tolist() == sorted(np.argsort(-r[b, h], kind="stable")[:6].tolist())


def test_selection_key_mask_hand_example():
    """Block c covers tokens [c*kb, min(P, (c+1)*kb)): 7 tokens in blocks of 3, last block short."""
    idx = np.array([[[1], [2]]], dtype=np.int32)
    m = orc.selection_key_mask(idx, 7, 3)
    assert m[0, 0].tolist() == [False, False, False, True, True, True, False]
    assert m[0, 1].tolist() == [False] * 6 + [True]
    both = orc.selection_key_mask(np.array([[[0, 2], [-1, 1]]], dtype=np.int32), 7, 3)
    assert both[0, 0].tolist() == [True, True, True, False, False, False, True]
    assert both[0, 1].tolist() == [False, False, False, True, True, True, False]      # negative entries are skipped


def _sparse_steps(seed):
    Q0, Kp, Vp, Kb0, Vb0 = _small_problem(seed, B=1, Hq=4, Hkv=2, d=8, P=45, Bq=4)
    steps = [(Q0, Kb0, Vb0)]
    for t in range(1, 4):
        steps.append(tuple(x + 0.3 * _rand(x.shape, seed + 3 * t + i) for i, x in enumerate(steps[-1])))
    return Kp, Vp, steps


def test_sparse_reuse_equals_augmented_sdpa():
    """Sparse reuse step = plain attention where unselected prefix keys see the refresh-step
    query and selected prefix keys + block keys see the current query."""
    Kp, Vp, steps = _sparse_steps(100)
    kb, topk, P = 8, 2, 45
    scale = 1.0 / math.sqrt(8)
    res = orc.run_block_sparse(Kp, Vp, steps, R=4, key_block=kb, topk=topk)
    idx = res[0]["idx"]
    assert all((r["idx"] == idx).all() for r in res)            # selection frozen within the block
    kmask = np.zeros((1, 4, P), dtype=bool)          # built here, not by the oracle's own helper
    for h in range(4):
        for c in idx[0, h]:
            kmask[0, h, int(c) * kb:min(P, (int(c) + 1) * kb)] = True
    assert kmask.sum(axis=-1).max() <= topk * kb
    Q0 = steps[0][0]
    for t, (Q, Kb, Vb) in enumerate(steps):
        for h in range(4):
            sel = kmask[0, h]
            g = h // 2
            Qa, Ka, Va = _augmented(Q0[:, h:h + 1], Q[:, h:h + 1], Kp[:, g:g + 1, ~sel], Vp[:, g:g + 1, ~sel],
                                    np.concatenate([Kp[:, g:g + 1, sel], Kb[:, g:g + 1]], 2),
                                    np.concatenate([Vp[:, g:g + 1, sel], Vb[:, g:g + 1]], 2))
            assert np.allclose(res[t]["out"][:, h:h + 1], _sdpa(Qa, Ka, Va, scale), atol=1e-12), (t, h)
    # refresh step is exact full attention for any k
    exact, _ = orc.full_attention(Q0, np.concatenate([Kp, steps[0][1]], 2), np.concatenate([Vp, steps[0][2]], 2))
    assert np.allclose(res[0]["out"], exact, atol=1e-12)


def test_sparse_limits_all_and_none_selected():
    """k >= #blocks: residual empty, every step is plain attention.  k = 0: the residual is the
    whole prefix and the sparse path is the dense cached path."""
    Kp, Vp, steps = _sparse_steps(120)
    res_all = orc.run_block_sparse(Kp, Vp, steps, R=4, key_block=8, topk=99)
    for t, (Q, Kb, Vb) in enumerate(steps):
        exact, lz = orc.full_attention(Q, np.concatenate([Kp, Kb], 2), np.concatenate([Vp, Vb], 2))
        assert np.allclose(res_all[t]["out"], exact, atol=1e-12) and np.allclose(res_all[t]["lse"], lz, atol=1e-12)
        assert np.isneginf(res_all[t]["residual"]["lse"]).all()
    res_none = orc.run_block_sparse(Kp, Vp, steps, R=4, key_block=8, topk=0)
    dense = orc.run_block_dense(Kp, Vp, steps, R=4)
    for a, b in zip(res_none, dense):
        assert np.allclose(a["out"], b["out"], atol=1e-12)


def test_residual_reuse_reduces_gap_to_full_attention():
    """Direction of Table 3: adding the cached residual brings sparse attention closer to
    full attention than dropping the unselected keys (synthetic data, only the inequality)."""
    w = wl.CONFIGS["tiny_f32"].with_(prefix_len=512, key_block=32, topk=4)
    Kp, Vp = wl.make_prefix(w, 7)
    steps = wl.make_block_steps(w, 7)
    res = orc.run_block_sparse(Kp, Vp, steps, R=4, key_block=32, topk=4)
    for t in range(1, 4):
        Q, Kb, Vb = steps[t]
        exact, _ = orc.full_attention(Q, np.concatenate([Kp, Kb], 2), np.concatenate([Vp, Vb], 2))
        with_res = np.abs(res[t]["out"] - exact).mean()
        without = np.abs(res[t]["sparse_only"] - exact).mean()
        assert with_res < without


# ------------------------------------------------------------------ paper-printed figures
def test_cache_bytes_match_table5():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table5_cache_bytes.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for batch, mib, layers, heads, brow, d in rows:
        got = orc.cache_bytes_paper_layout(int(layers), int(heads), int(brow), int(d), batch=int(batch))
        assert abs(got / 2 ** 20 - float(mib)) < 0.006, (got / 2 ** 20, mib)
    # independent of context length by construction: no context argument exists
    assert orc.cache_bytes_paper_layout(36, 32, 4, 128) == 36 * 32 * 4 * 260


# ------------------------------------------------------------------ input generator sanity
def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 3
    x = np.concatenate([x, np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.0e38], dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(wl.round_bf16(x), want)


def test_workload_generator_shapes_and_determinism():
    w = wl.CONFIGS["tiny_f32"]
    K, V = wl.make_prefix(w, 3)
    assert K.shape == (1, 4, 256, 64) and K.dtype == np.float32
    s1, s2 = wl.make_block_steps(w, 3), wl.make_block_steps(w, 3)
    assert len(s1) == 4 and all(np.array_equal(a[0], b[0]) for a, b in zip(s1, s2))
    d = s1[1][0] - s1[0][0]
    assert 0.03 < d.std() < 0.07
    wb = wl.CONFIGS["llm_32k"].with_(prefix_len=64)
    Kb, _ = wl.make_prefix(wb, 3)
    assert np.array_equal(Kb, wl.round_bf16(Kb)) and abs(Kb.std() - 1 / math.sqrt(128)) < 0.01


def test_head_similarity_hand_cases():
    """Cosine similarity of A_out rows: identical partials -> 1, orthogonal outputs -> 0, and the
    value must not depend on the row normalisers (A = o * positive scalar)."""
    o = np.zeros((1, 2, 2, 4)); o[0, 0, :, 0] = 1.0; o[0, 1, 0, 0] = 3.0; o[0, 1, 1, 1] = 2.0
    a = {"o": o, "m": np.zeros((1, 2, 2)), "lse": np.log(np.full((1, 2, 2), 5.0))}
    o2 = np.zeros((1, 2, 2, 4)); o2[0, 0, :, 1] = 7.0; o2[0, 1, 0, 0] = 1.0; o2[0, 1, 1, 1] = 1.0; o2[0, 1, 1, 0] = 1.0
    b = {"o": o2, "m": np.ones((1, 2, 2)), "lse": np.log(np.full((1, 2, 2), 11.0))}
    assert np.allclose(orc.head_similarity(a, a), 1.0)
    s = orc.head_similarity(a, b)
    assert abs(s[0, 0]) < 1e-15                                  # orthogonal rows
    assert abs(s[0, 1] - 0.5 * (1.0 + 1.0 / math.sqrt(2.0))) < 1e-12   # rows: parallel, 45 degrees
