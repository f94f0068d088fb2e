"""Seeded random shapes through the C ABI against the numpy float64 oracle.  The HIP path picks its
kernel variant from the shape (rows per KV group, tiles per split, number of splits, block size), so
shapes drawn across those thresholds reach variant combinations the hand-picked cases may miss.
Same tolerances as everywhere: fp32 storage 1e-5 max-abs, bf16 storage 1e-2 abs + 1e-2 rel."""
import numpy as np
import pytest
import torch

from oracle import flashblock_oracle as orc
from paper_2602_05305_amd import flashblock as fb
from paper_2602_05305_amd import workloads as wl

import fb_testlib as T

pytestmark = pytest.mark.gpu


def _draw_dense(rng):
    dtype = "bf16" if rng.random() < 0.75 else "f32"
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.choice([1, 1, 2, 4, 8]))
    B = int(rng.choice([1, 1, 2, 3]))
    if dtype == "f32":
        Bq = int(rng.integers(1, 40))
        P = int(rng.integers(0, 700))
    else:
        Bq = int(rng.choice([1, 3, 4, 8, 16, 31, 32, 33, 64, 96, 130, 300]))
        P = int(rng.choice([0, 1, 63, 64, 65, 500, 1024, 1500, 2048, 3000, 4500]))
        if G * Bq > 1200:
            P = min(P, 1500)
    n_splits = int(rng.choice([0, 0, 0, 1, 2, 3, 5, 9]))
    return dtype, B, Hkv * G, Hkv, d, P, Bq, n_splits


@pytest.mark.parametrize("case", range(36))
def test_random_dense_shape(case):
    rng = np.random.default_rng([20260205, case])
    dtype, B, Hq, Hkv, d, P, Bq, n_splits = _draw_dense(rng)
    w = wl.Workload(f"rand{case}", B, Hq, Hkv, d, P, Bq, 3, 2, dtype, 1.0 if rng.random() < 0.5 else 1.0 / np.sqrt(d))
    print(f"[case {case}] {dtype} B={B} Hq={Hq} Hkv={Hkv} d={d} P={P} Bq={Bq} n_splits={n_splits}", flush=True)
    Kp, Vp = wl.make_prefix(w, 900 + case)
    steps = wl.make_block_steps(w, 900 + case)
    ora = orc.run_block_dense(Kp, Vp, steps, 2)
    gpu = T.run_dense_block_gpu(w, Kp, Vp, steps, R=2, n_splits=n_splits)
    for t, (g, o) in enumerate(zip(gpu, ora)):
        T.assert_close(g["out"], o["out"], dtype, f"case {case} step {t} out")
        T.assert_close(g["lse"], o["lse"], dtype, f"case {case} step {t} lse", lse=True)
        T.check_partial(g["ext"], o["ext"], dtype, f"case {case} step {t} ext")
    # the one-call refresh step on the same inputs: identical contract (partial + final output)
    shape = T.shape_of(w)
    ws = T.workspace(shape)
    Q, Kb, Vb = steps[0]
    q, kb, vb = T.to_dev(Q, dtype), T.to_dev(Kb, dtype), T.to_dev(Vb, dtype)
    kp = T.to_dev(Kp, dtype) if P > 0 else None
    vp = T.to_dev(Vp, dtype) if P > 0 else None
    ext = T.Partial(w)
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], device=T.DEV, dtype=torch.float32)
    fb.fb_refresh_step(shape, q, kp, vp, kb, vb, ext.o, ext.m, ext.lse, out, lse, ws)
    torch.cuda.synchronize()
    T.assert_close(out.double().cpu().numpy(), ora[0]["out"], dtype, f"case {case} refresh_step out")
    T.assert_close(lse.double().cpu().numpy(), ora[0]["lse"], dtype, f"case {case} refresh_step lse", lse=True)
    T.check_partial(ext.numpy(), ora[0]["ext"], dtype, f"case {case} refresh_step ext")


@pytest.mark.parametrize("case", range(14))
def test_random_sparse_shape(case):
    rng = np.random.default_rng([20260206, case])
    dtype = "bf16" if rng.random() < 0.8 else "f32"
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 4, 8]))
    B = int(rng.choice([1, 2]))
    Bq = int(rng.choice([4, 16, 32, 40])) if dtype == "bf16" else int(rng.integers(2, 20))
    kb = int(rng.choice([64, 128]))
    nblk = int(rng.integers(1, 40 if dtype == "bf16" else 10))
    P = nblk * kb - int(rng.integers(0, kb))          # last block possibly short
    P = max(P, 1)
    topk = int(rng.integers(0, nblk + 3))
    w = wl.Workload(f"rsp{case}", B, Hkv * G, Hkv, d, P, Bq, 3, 2, dtype, 1.0 / np.sqrt(d), key_block=kb, topk=topk)
    print(f"[case {case}] {dtype} B={B} Hq={Hkv * G} Hkv={Hkv} d={d} P={P} Bq={Bq} key_block={kb} topk={topk}", flush=True)
    Kp, Vp = wl.make_prefix(w, 700 + case)
    steps = wl.make_block_steps(w, 700 + case)
    ora = orc.run_block_sparse(Kp, Vp, steps, 2, kb, topk)
    idx = {t: o["idx"] for t, o in enumerate(ora) if t % 2 == 0}
    gpu = T.run_sparse_block_gpu(w, Kp, Vp, steps, idx_per_refresh=idx, R=2, same_selection=bool(case % 2))
    for t, (g, o) in enumerate(zip(gpu, ora)):
        T.assert_close(g["out"], o["out"], dtype, f"case {case} step {t} out")
        T.assert_close(g["lse"], o["lse"], dtype, f"case {case} step {t} lse", lse=True)
        T.check_partial(g["ext"], o["ext"], dtype, f"case {case} step {t} ext")
        if t % 2 == 0:
            T.check_partial(g["residual"], o["residual"], dtype, f"case {case} step {t} residual")


@pytest.mark.parametrize("case", range(12))
def test_random_paged_shape(case):
    import test_gpu_paged as PG
    rng = np.random.default_rng([20260207, case])
    dtype = "bf16" if rng.random() < 0.75 else "f32"
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 4]))
    B = int(rng.integers(1, 7))
    page = int(rng.choice([64, 128, 256]))
    pmax = int(rng.integers(1, 24 if dtype == "bf16" else 6)) * page
    Bq = int(rng.choice([4, 16, 32, 48])) if dtype == "bf16" else int(rng.integers(1, 12))
    lens = rng.integers(0, pmax + 1, size=B)
    lens[int(rng.integers(0, B))] = pmax if rng.random() < 0.5 else int(lens.max())
    n_splits = int(rng.choice([0, 0, 1, 2, 5]))
    w = wl.Workload(f"rpg{case}", B, Hkv * G, Hkv, d, pmax, Bq, 1, 1, dtype, 1.0)
    PG._run_paged(w, seed=300 + case, page_size=page, lens=[int(x) for x in lens], n_splits=n_splits)


@pytest.mark.parametrize("case", range(10))
def test_random_head_mask_shape(case):
    """Per-head refresh with random masks and hints (0 = none, the true count, or a wrong count)."""
    import test_gpu_dense as DN
    rng = np.random.default_rng([20260208, case])
    dtype = "bf16" if rng.random() < 0.8 else "f32"
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3, 6]))
    G = int(rng.choice([1, 1, 2, 4]))
    B = int(rng.choice([1, 2]))
    if dtype == "bf16":
        Bq = int(rng.choice([8, 32, 48, 150, 300]))
        P = int(rng.choice([200, 700, 2100, 4200]))
    else:
        Bq, P = int(rng.integers(1, 10)), int(rng.integers(1, 400))
    Hq = Hkv * G
    mask = (rng.random(B * Hq) < rng.choice([0.15, 0.5, 0.9])).astype(int).tolist()
    hint = int(rng.choice([0, sum(mask), max(1, sum(mask) // 2), Hq]))
    DN.test_head_wise_selective_refresh(dtype, B, Hq, Hkv, d, P, Bq, mask, hint)
