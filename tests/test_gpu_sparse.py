"""GPU parity of the sparse variant with residual reuse (key-block selection, refresh pass that
routes key blocks into selected / residual statistics, reuse pass over selected blocks only)
against the numpy float64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import flashblock_oracle as orc
from paper_2602_05305_amd import flashblock as fb
from paper_2602_05305_amd import workloads as wl

import fb_testlib as T

pytestmark = pytest.mark.gpu


def _wl(dtype, B, Hq, Hkv, d, P, Bq, kb, topk, S=4, R=4, scale_in=1.0):
    return wl.Workload(f"sparse_{dtype}_{B}_{Hq}_{Hkv}_{d}_{P}_{Bq}_{kb}_{topk}", B, Hq, Hkv, d, P, Bq, S, R, dtype,
                       scale_in, key_block=kb, topk=topk)


def _compare_sparse(w, seed, R=None):
    """Attention parity with the ORACLE's selection fed to the GPU (near-ties in the selection
    scores may legitimately differ between fp64 and fp32; selection has its own test)."""
    print(f"[case] {w.name} seed={seed} R={R}", flush=True)
    R = w.refresh if R is None else R
    Kp, Vp = wl.make_prefix(w, seed)
    steps = wl.make_block_steps(w, seed)
    ora = orc.run_block_sparse(Kp, Vp, steps, R, w.key_block, w.topk)
    idx = {t: ora[t]["idx"] for t in range(len(steps)) if t % R == 0}
    gpu = T.run_sparse_block_gpu(w, Kp, Vp, steps, idx_per_refresh=idx, R=R)
    for t, (g, o) in enumerate(zip(gpu, ora)):
        T.assert_close(g["out"], o["out"], w.dtype, f"{w.name} step {t} out")
        T.assert_close(g["lse"], o["lse"], w.dtype, f"{w.name} step {t} lse", lse=True)
        T.check_partial(g["ext"], o["ext"], w.dtype, f"{w.name} step {t} sel(+)res")
        T.check_partial(g["residual"], o["residual"], w.dtype, f"{w.name} step {t} residual")
    return gpu, ora


@pytest.mark.parametrize("dtype,B,Hq,Hkv,d,P,Bq,kb,topk", [
    ("f32", 1, 4, 2, 64, 640, 8, 64, 3),       # 10 blocks, 3 selected per head
    ("f32", 2, 2, 2, 128, 700, 5, 128, 2),     # 128-token key blocks, short last block
    ("f32", 1, 4, 1, 64, 333, 3, 64, 1),       # G = 4, short last block of 13 tokens
    ("bf16", 1, 8, 2, 128, 2048, 32, 64, 8),   # LLM group shape: 32 blocks, 8 selected
    ("bf16", 1, 8, 2, 128, 1999, 32, 64, 5),   # short last block
    ("bf16", 1, 4, 2, 128, 1500, 40, 128, 3),  # wavefronts straddle query heads (per-lane routing)
    ("bf16", 2, 4, 4, 64, 900, 16, 64, 4),     # d = 64, MHA
])
def test_sparse_shapes(dtype, B, Hq, Hkv, d, P, Bq, kb, topk):
    _compare_sparse(_wl(dtype, B, Hq, Hkv, d, P, Bq, kb, topk), seed=41)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sparse_all_blocks_selected_equals_full_attention(dtype):
    """k >= #blocks: the residual is empty and every step is plain attention."""
    w = _wl(dtype, 1, 4, 2, 128 if dtype == "bf16" else 64, 500, 32 if dtype == "bf16" else 6, 64, 99)
    gpu, _ = _compare_sparse(w, seed=43)
    Kp, Vp = wl.make_prefix(w, 43)
    steps = wl.make_block_steps(w, 43)
    for t, (Q, Kb, Vb) in enumerate(steps):
        a, _ = orc.full_attention(Q, np.concatenate([Kp, Kb], 2), np.concatenate([Vp, Vb], 2))
        T.assert_close(gpu[t]["out"], a, dtype, f"k=all step {t}")
        assert np.isneginf(gpu[t]["residual"]["lse"]).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sparse_nothing_selected_equals_dense_cached_path(dtype):
    """k = 0: the residual is the whole prefix; the sparse path is the dense cached path."""
    d, Bq = (128, 32) if dtype == "bf16" else (64, 6)
    w = _wl(dtype, 1, 4, 2, d, 500, Bq, 64, 0)
    Kp, Vp = wl.make_prefix(w, 45)
    steps = wl.make_block_steps(w, 45)
    gpu = T.run_sparse_block_gpu(w, Kp, Vp, steps, idx_per_refresh=None)
    dense = orc.run_block_dense(Kp, Vp, steps, w.refresh)
    for t in range(len(steps)):
        T.assert_close(gpu[t]["out"], dense[t]["out"], dtype, f"k=0 step {t}")


def test_sparse_refresh_step_is_exact_and_negative_or_duplicate_indices():
    """Negative entries are skipped, duplicates count once; the refresh step is exact attention."""
    w = _wl("bf16", 1, 4, 2, 128, 1024, 32, 64, 4, S=2, R=2)
    Kp, Vp = wl.make_prefix(w, 47)
    steps = wl.make_block_steps(w, 47)
    idx = np.array([[[3, 3, -1, 9], [0, 15, 15, -1], [-1, -1, -1, -1], [1, 2, 3, 4]]], dtype=np.int32)
    gpu = T.run_sparse_block_gpu(w, Kp, Vp, steps, idx_per_refresh={0: idx})
    Q, Kb, Vb = steps[0]
    a, _ = orc.full_attention(Q, np.concatenate([Kp, Kb], 2), np.concatenate([Vp, Vb], 2))
    T.assert_close(gpu[0]["out"], a, "bf16", "refresh step exact")
    # reuse step against the oracle with the de-duplicated selection
    kmask = np.zeros((1, 4, 1024), dtype=bool)
    for h in range(4):
        for c in set(int(c) for c in idx[0, h] if c >= 0):
            kmask[0, h, c * 64:(c + 1) * 64] = True
    Q1, Kb1, Vb1 = steps[1]
    res = orc.partial(Q, Kp, Vp, key_mask=~kmask)
    sel = orc.partial(Q1, Kp, Vp, key_mask=kmask)
    out, _ = orc.merge(orc.merge_partials(sel, res), orc.partial(Q1, Kb1, Vb1))
    T.assert_close(gpu[1]["out"], out, "bf16", "reuse step with duplicates")


@pytest.mark.parametrize("dtype,B,Hq,Hkv,d,P,Bq,kb,topk", [
    ("f32", 1, 4, 2, 64, 4096, 16, 64, 16),
    ("bf16", 2, 8, 2, 128, 8000, 32, 64, 30),
    ("bf16", 1, 2, 2, 128, 700, 8, 128, 9),     # topk beyond the 6 blocks: tail filled with -1
    ("f32", 1, 6, 2, 128, 64 * 37 + 5, 12, 64, 7),   # 3 heads per group, ragged last block, rows not a lane multiple
    ("bf16", 1, 8, 1, 64, 64 * 70, 40, 64, 20),      # 8 heads per group, head_dim 64, more rows than one trip
])
def test_select_topk_matches_oracle(dtype, B, Hq, Hkv, d, P, Bq, kb, topk):
    """fb_pool_keys + fb_select_topk against the oracle's selection.  The selected sets must be
    equal, except for members whose oracle score is within 1e-3 (relative to the score spread)
    of the k-th score, where fp32 and fp64 may order near-ties differently."""
    w = _wl(dtype, B, Hq, Hkv, d, P, Bq, kb, topk)
    Kp, _ = wl.make_prefix(w, 51)
    Q = wl.make_block_steps(w, 51, steps=1)[0][0]
    shape = T.shape_of(w)
    nblk = -(-P // kb)
    pooled = torch.empty((B, Hkv, nblk, d), device=T.DEV, dtype=torch.float32)
    fb.fb_pool_keys(shape, T.to_dev(Kp, dtype), kb, pooled)
    idx = torch.full((B, Hq, topk), -7, device=T.DEV, dtype=torch.int32)
    fb.fb_select_topk(shape, T.to_dev(Q, dtype), pooled, kb, topk, idx)
    # the same selection with the scoring spread over the chip (workspace given): identical indices
    idx_ws = torch.full((B, Hq, topk), -7, device=T.DEV, dtype=torch.int32)
    sws = torch.empty(fb.fb_select_workspace_bytes(shape, kb), device=T.DEV, dtype=torch.uint8)
    fb.fb_select_topk(shape, T.to_dev(Q, dtype), pooled, kb, topk, idx_ws, sws)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx_ws)
    ora_pooled = orc.pool_keys(Kp, kb)
    assert np.abs(pooled.double().cpu().numpy() - ora_pooled).max() < 1e-5
    sc = orc.select_scores(Q, ora_pooled)
    want = orc.select_topk(Q, Kp, kb, topk)
    got = idx.cpu().numpy()
    k = min(topk, nblk)
    assert (got[:, :, k:] == -1).all()
    for b in range(B):
        for h in range(Hq):
            g = got[b, h, :k]
            assert (np.diff(g) > 0).all() and g.min() >= 0 and g.max() < nblk      # ascending, unique, valid
            diff = set(g.tolist()) ^ set(want[b, h].tolist())
            if diff:
                kth = np.sort(sc[b, h])[::-1][k - 1]
                spread = sc[b, h].max() - sc[b, h].min()
                assert all(abs(sc[b, h, c] - kth) <= 1e-3 * spread for c in diff), (b, h, diff)


def test_sparse_gpu_selection_end_to_end():
    """Whole sparse path with the GPU's own selection: valid selection + parity of the attention
    computed with exactly that selection."""
    w = _wl("bf16", 1, 8, 2, 128, 4096, 32, 64, 16)
    Kp, Vp = wl.make_prefix(w, 53)
    steps = wl.make_block_steps(w, 53)
    gpu = T.run_sparse_block_gpu(w, Kp, Vp, steps, idx_per_refresh=None)
    idx = gpu[0]["idx"]
    kmask = orc.selection_key_mask(idx, w.prefix_len, w.key_block)
    res = orc.partial(steps[0][0], Kp, Vp, key_mask=~kmask)
    for t, (Q, Kb, Vb) in enumerate(steps):
        sel = orc.partial(Q, Kp, Vp, key_mask=kmask)
        out, _ = orc.merge(orc.merge_partials(sel, res), orc.partial(Q, Kb, Vb))
        T.assert_close(gpu[t]["out"], out, "bf16", f"gpu-selected step {t}")


# ------------------------------------------------------------------ selection by attention mass
@pytest.mark.parametrize("dtype,B,Hq,Hkv,d,P,Bq,kb,topk", [
    ("f32", 1, 4, 2, 64, 700, 7, 64, 3),
    ("f32", 2, 4, 4, 128, 256, 16, 128, 1),
    ("bf16", 1, 8, 2, 128, 2048 + 37, 32, 64, 8),
    ("bf16", 2, 4, 4, 64, 1000, 16, 128, 5),
    ("bf16", 1, 32, 8, 128, 8192, 32, 256, 8),
    ("bf16", 1, 4, 4, 128, 1024, 200, 64, 20),       # several row tiles; topk > number of key blocks
])
def test_select_topk_mass_matches_oracle(dtype, B, Hq, Hkv, d, P, Bq, kb, topk):
    """fb_select_topk_mass: the block scores (attention mass) against the oracle within the
    storage tolerance (relative: masses are of order 1/nblk), rows summing to 1, and the selection
    = the oracle's top-k of the oracle's masses except for near-ties at the k-th score."""
    w = _wl(dtype, B, Hq, Hkv, d, P, Bq, kb, topk)
    print(f"[case] mass {w.name}", flush=True)
    Kp, Vp = wl.make_prefix(w, 61)
    Q = wl.make_block_steps(w, 61, steps=1)[0][0]
    shape = T.shape_of(w)
    q, kp, vp = T.to_dev(Q, dtype), T.to_dev(Kp, dtype), T.to_dev(Vp, dtype)
    ext = T.Partial(w)
    fb.fb_external_partial(shape, q, kp, vp, ext.o, ext.m, ext.lse, T.workspace(shape))
    nblk = -(-P // kb)
    idx = torch.full((B, Hq, topk), -7, device=T.DEV, dtype=torch.int32)
    mass = torch.full((B, Hq, nblk), -1.0, device=T.DEV, dtype=torch.float32)
    ws = torch.empty(fb.fb_select_mass_workspace_bytes(shape, kb), device=T.DEV, dtype=torch.uint8)
    fb.fb_select_topk_mass(shape, q, kp, ext.lse, kb, topk, idx, mass, ws)
    torch.cuda.synchronize()
    want_mass = orc.block_mass(Q, Kp, kb)
    got_mass = mass.double().cpu().numpy()
    rel = 2e-5 if dtype == "f32" else 1e-2
    assert np.abs(got_mass - want_mass).max() <= rel * want_mass.max() + 1e-7, np.abs(got_mass - want_mass).max()
    assert np.abs(got_mass.sum(-1) - 1.0).max() <= (1e-4 if dtype == "f32" else 1e-2)
    want = orc.select_topk_scores(want_mass, topk)
    got = idx.cpu().numpy()
    k = min(topk, nblk)
    assert (got[:, :, k:] == -1).all()
    for b in range(B):
        for h in range(Hq):
            g = got[b, h, :k]
            assert (np.diff(g) > 0).all() and g.min() >= 0 and g.max() < nblk
            diff = set(g.tolist()) ^ set(want[b, h].tolist())
            if diff:
                kth = np.sort(want_mass[b, h])[::-1][k - 1]
                assert all(abs(want_mass[b, h, c] - kth) <= rel * want_mass[b, h].max() for c in diff), (b, h, diff)
    # the kernel's own scores and its own selection are consistent: exact top-k of mass_out, ties low
    own = orc.select_topk_scores(got_mass, topk)
    assert np.array_equal(own, got[:, :, :k])


def test_mass_selection_feeds_the_sparse_path():
    """Mass-selected blocks go through fb_sparse_external_residual like any other selection; the
    refresh step stays exact attention."""
    w = _wl("bf16", 1, 8, 2, 128, 4096, 32, 64, 16)
    Kp, Vp = wl.make_prefix(w, 63)
    Q, Kb, Vb = wl.make_block_steps(w, 63, steps=1)[0]
    shape = T.shape_of(w)
    q, kp, vp = T.to_dev(Q, "bf16"), T.to_dev(Kp, "bf16"), T.to_dev(Vp, "bf16")
    ext, res, tot = T.Partial(w), T.Partial(w), T.Partial(w)
    ws = T.workspace(shape, w.key_block, w.topk)
    fb.fb_external_partial(shape, q, kp, vp, ext.o, ext.m, ext.lse, ws)
    idx = torch.empty((1, 8, 16), device=T.DEV, dtype=torch.int32)
    wsm = torch.empty(fb.fb_select_mass_workspace_bytes(shape, 64), device=T.DEV, dtype=torch.uint8)
    fb.fb_select_topk_mass(shape, q, kp, ext.lse, 64, 16, idx, None, wsm)
    fb.fb_sparse_external_residual(shape, fb.FB_SPARSE_REFRESH, q, kp, vp, 64, 16, idx, res.o, res.m, res.lse,
                                   tot.o, tot.m, tot.lse, ws)
    torch.cuda.synchronize()
    T.check_partial(tot.numpy(), orc.partial(Q, Kp, Vp), "bf16", "mass-selected refresh total")
    kmask = orc.selection_key_mask(idx.cpu().numpy(), w.prefix_len, w.key_block)
    T.check_partial(res.numpy(), orc.partial(Q, Kp, Vp, key_mask=~kmask), "bf16", "mass-selected residual")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sparse_reuse_with_the_previous_calls_selection(dtype):
    """FB_SPARSE_REUSE_SAME_SELECTION: reuse steps that take the selection masks the refresh call left
    in the workspace give bit-identical results to reuse steps that rebuild them from sel_idx."""
    w = _wl(dtype, 2, 8, 2, 128 if dtype == "bf16" else 64, 1500, 16, 64, 5, S=4, R=4)
    Kp, Vp = wl.make_prefix(w, 67)
    steps = wl.make_block_steps(w, 67)
    idx = {0: orc.select_topk(steps[0][0], Kp, w.key_block, w.topk)}
    a = T.run_sparse_block_gpu(w, Kp, Vp, steps, idx_per_refresh=idx)
    b = T.run_sparse_block_gpu(w, Kp, Vp, steps, idx_per_refresh=idx, same_selection=True)
    ora = orc.run_block_sparse(Kp, Vp, steps, w.refresh, w.key_block, w.topk)
    for t in range(w.steps):
        assert np.array_equal(a[t]["out"], b[t]["out"]) and np.array_equal(a[t]["lse"], b[t]["lse"]), t
        T.assert_close(b[t]["out"], ora[t]["out"], dtype, f"same-selection step {t}")
