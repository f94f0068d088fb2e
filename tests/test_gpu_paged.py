"""GPU parity of the paged external pass (block table + per-sequence prefix lengths) against the
numpy float64 oracle.  The oracle never sees pages: it gets each sequence's contiguous K, V from
the input generator and computes that sequence's partial on its own."""
import numpy as np
import pytest
import torch

from oracle import flashblock_oracle as orc
from paper_2602_05305_amd import flashblock as fb
from paper_2602_05305_amd import workloads as wl

import fb_testlib as T

pytestmark = pytest.mark.gpu


def _oracle_partial(w, Q, seqs, scale=None):
    parts = [orc.partial(Q[b:b + 1], Kb[None], Vb[None], scale) if Kb.shape[1] > 0
             else orc.empty_partial(1, w.n_q_heads, w.block_len, w.head_dim)
             for b, (Kb, Vb) in enumerate(seqs)]
    return {k: np.concatenate([p[k] for p in parts], axis=0) for k in ("o", "m", "lse")}


def _run_paged(w, seed, page_size, lens, n_splits=0):
    print(f"[case] paged {w.name} seed={seed} page={page_size} lens={list(lens)}", flush=True)
    seqs, Kpool, Vpool, table, lens = wl.make_paged_prefix(w, seed, page_size, lens)
    Q, Kb, Vb = wl.make_block_steps(w, seed, 1)[0]
    shape = T.shape_of(w)
    q = T.to_dev(Q, w.dtype)
    kpool, vpool = T.to_dev(Kpool, w.dtype), T.to_dev(Vpool, w.dtype)
    tbl = torch.from_numpy(table).to(T.DEV)
    ln = torch.from_numpy(lens).to(T.DEV)
    kv = fb.make_paged_kv(kpool, vpool, tbl, ln)
    ws = T.workspace(shape, n_splits=n_splits or fb.fb_paged_splits(shape))
    ext = T.Partial(w)
    fb.fb_external_partial_paged(shape, q, kv, ext.o, ext.m, ext.lse, ws, n_splits)
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], device=T.DEV, dtype=torch.float32)
    fb.fb_internal_merge(shape, q, T.to_dev(Kb, w.dtype), T.to_dev(Vb, w.dtype), ext.o, ext.m, ext.lse, out, lse)
    torch.cuda.synchronize()
    ora_ext = _oracle_partial(w, Q, seqs)
    T.check_partial(ext.numpy(), ora_ext, w.dtype, f"{w.name} paged ext")
    ora_out, ora_lse = orc.merge(ora_ext, orc.partial(Q, Kb, Vb))
    T.assert_close(out.double().cpu().numpy(), ora_out, w.dtype, f"{w.name} paged out")
    T.assert_close(lse.double().cpu().numpy(), ora_lse, w.dtype, f"{w.name} paged lse", lse=True)
    return ext, (q, kpool, vpool, tbl, ln, shape, ws)


def _wl(dtype, B, Hq, Hkv, d, P, Bq):
    return wl.Workload(f"paged_{dtype}_{B}_{Hq}_{Hkv}_{d}_{P}_{Bq}", B, Hq, Hkv, d, P, Bq, 1, 1, dtype, 1.0)


@pytest.mark.parametrize("dtype,B,Hq,Hkv,d,P,Bq,page,lens", [
    ("f32", 3, 4, 2, 64, 576, 5, 64, [200, 0, 513]),
    ("f32", 2, 4, 4, 128, 640, 16, 128, [640, 129]),
    ("bf16", 4, 8, 2, 128, 2048, 32, 128, [1617, 64, 1, 1000]),
    ("bf16", 3, 4, 4, 64, 1024, 16, 64, [0, 1024, 65]),
    ("bf16", 2, 8, 2, 128, 8192, 32, 256, [8192, 3000]),        # two wavefront groups per workgroup
    ("bf16", 5, 32, 8, 128, 4096, 32, 256, [4096, 17, 2048, 3333, 255]),
])
def test_paged_external_matches_oracle(dtype, B, Hq, Hkv, d, P, Bq, page, lens):
    _run_paged(_wl(dtype, B, Hq, Hkv, d, P, Bq), seed=41, page_size=page, lens=lens)


def test_paged_large_batch_uses_the_ordering_kernel():
    """More than 128 sequences: the longest-first order comes from the separate ranking kernel
    (smaller batches rank inside the attention kernel).  Lengths with many ties."""
    rng = np.random.default_rng(9)
    lens = rng.integers(0, 5, size=130) * 64 + rng.integers(0, 2, size=130) * 17
    _run_paged(_wl("bf16", 130, 2, 1, 64, 320, 8), seed=44, page_size=64, lens=np.minimum(lens, 320))


@pytest.mark.parametrize("n_splits", [1, 3, 16])
def test_paged_split_counts(n_splits):
    """Every sequence's own tile list is cut into n_splits ranges; short sequences leave some empty."""
    _run_paged(_wl("bf16", 3, 8, 2, 128, 2048, 32), seed=42, page_size=128, lens=[2048, 130, 700], n_splits=n_splits)
    _run_paged(_wl("f32", 2, 4, 2, 64, 512, 8), seed=42, page_size=64, lens=[512, 70], n_splits=n_splits)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_paged_equals_contiguous_when_all_sequences_are_full(dtype):
    """With every sequence at the maximum length the paged pass walks the same tiles with the same
    split as the contiguous pass.  fp32: bit for bit.  bf16: the workgroups visit their tiles in a
    rotated order that depends on the workgroup index, which the two passes assign differently, so
    the probabilities are rounded to bf16 against different lazily
    updated references and the results agree to a fraction of the bf16 tolerance only."""
    w = _wl(dtype, 2, 8, 2, 128, 1536, 32)
    ns = fb.fb_external_splits(T.shape_of(w))
    ext, (q, kpool, vpool, tbl, ln, shape, ws) = _run_paged(w, seed=43, page_size=256, lens=[1536, 1536], n_splits=ns)
    seqs, *_ = wl.make_paged_prefix(w, 43, 256, [1536, 1536])
    K = np.stack([s[0] for s in seqs])
    V = np.stack([s[1] for s in seqs])
    ref = T.Partial(w)
    fb.fb_external_partial(shape, q, T.to_dev(K, dtype), T.to_dev(V, dtype), ref.o, ref.m, ref.lse, ws)
    torch.cuda.synchronize()
    if dtype == "f32":
        assert torch.equal(ref.o, ext.o) and torch.equal(ref.m, ext.m) and torch.equal(ref.lse, ext.lse)
    else:
        a, b = orc.normalized(ref.numpy()), orc.normalized(ext.numpy())
        assert np.abs(a - b).max() <= 2e-3
        assert np.abs(ref.lse.double().cpu().numpy() - ext.lse.double().cpu().numpy()).max() <= 2e-3


def test_paged_lengths_are_clamped_and_bad_pages_stay_in_pool():
    """prefix_lens above shape.prefix_len are clamped to it; page ids outside the pool are clamped
    into it (wrong values, but no access outside the pool): the call completes and is finite."""
    w = _wl("bf16", 2, 4, 2, 128, 512, 32)
    seqs, Kpool, Vpool, table, lens = wl.make_paged_prefix(w, 47, 128, [512, 300])
    Q = wl.make_block_steps(w, 47, 1)[0][0]
    shape = T.shape_of(w)
    q, kpool, vpool = T.to_dev(Q, w.dtype), T.to_dev(Kpool, w.dtype), T.to_dev(Vpool, w.dtype)
    big = torch.tensor([10 ** 6, 300], dtype=torch.int32, device=T.DEV)
    tbl = torch.from_numpy(table).to(T.DEV)
    ext = T.Partial(w)
    ws = T.workspace(shape, n_splits=fb.fb_paged_splits(shape))
    fb.fb_external_partial_paged(shape, q, fb.make_paged_kv(kpool, vpool, tbl, big), ext.o, ext.m, ext.lse, ws)
    torch.cuda.synchronize()
    T.check_partial(ext.numpy(), _oracle_partial(w, Q, seqs), w.dtype, "clamped lengths")
    bad = tbl.clone()
    bad[1, 0] = 10 ** 6
    bad[1, 1] = -5
    fb.fb_external_partial_paged(shape, q, fb.make_paged_kv(kpool, vpool, bad, big), ext.o, ext.m, ext.lse, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(ext.o).all() and torch.isfinite(ext.lse).all()


def test_paged_serving_shape_batch32_full_tensors():
    """The benchmark's paged shape at full size, library-chosen split count: batch 32, 32 q / 8 kv
    heads, d128, block 32, prefix lengths uniform in [512, 8192] (one at the maximum, one a single
    ragged tile), 256-token pages.  The oracle computes every sequence."""
    w = wl.Workload("paged_b32", 32, 32, 8, 128, 8192, 32, 1, 1, "bf16", 1.0 / np.sqrt(128.0))
    rng = np.random.default_rng(4100)
    lens = rng.integers(512, 8193, size=32)
    lens[0], lens[5] = 8192, 37
    _run_paged(w, seed=4100, page_size=256, lens=lens)


def test_paged_head_dim_64_and_wide_grouping():
    """head_dim 64 (other tile geometry) and G = 8 with a block that spans two row tiles."""
    _run_paged(_wl("bf16", 3, 8, 1, 64, 1536, 40), seed=45, page_size=128, lens=[1536, 700, 64])
    _run_paged(_wl("f32", 2, 8, 1, 128, 384, 3), seed=46, page_size=64, lens=[384, 65])


@pytest.mark.parametrize("block_len", [4, 8])
def test_paged_deployment_shape_batch128_small_blocks(block_len):
    """The paper's language-model deployment shape (Section 5 implementation details, Table 1): 128 sequences under
    one token budget, blocks of 4 or 8 tokens, 32 q / 8 kv heads, d128, 256-token pages, library-chosen split count.
    Lengths are uniform in [512, 12288] with the extremes planted (maximum, one ragged tile, a single key, empty).
    The oracle recomputes 24 of the 128 sequences, among them every planted one."""
    w = wl.Workload(f"paged_b128_blk{block_len}", 128, 32, 8, 128, 12288, block_len, 1, 1, "bf16", 1.0 / np.sqrt(128.0))
    print(f"[case] {w.name}", flush=True)
    rng = np.random.default_rng(4200 + block_len)
    lens = rng.integers(512, 12289, size=128).astype(np.int32)
    lens[0], lens[7], lens[64], lens[127] = 12288, 37, 1, 0
    seqs, Kpool, Vpool, table, lens = wl.make_paged_prefix(w, 4200 + block_len, 256, lens)
    Q = wl.make_block_steps(w, 4200 + block_len, 1)[0][0]
    shape = T.shape_of(w)
    # the descriptor holds raw device addresses: the tensors behind them stay referenced until the call has run
    kpool, vpool = T.to_dev(Kpool, "bf16"), T.to_dev(Vpool, "bf16")
    tbl, ln = torch.from_numpy(table).to(T.DEV), torch.from_numpy(lens).to(T.DEV)
    kv = fb.make_paged_kv(kpool, vpool, tbl, ln)
    del Kpool, Vpool
    ext = T.Partial(w)
    fb.fb_external_partial_paged(shape, T.to_dev(Q, "bf16"), kv, ext.o, ext.m, ext.lse,
                                 T.workspace(shape, n_splits=fb.fb_paged_splits(shape)))
    torch.cuda.synchronize()
    got = ext.numpy()
    check = sorted(set([0, 7, 64, 127] + rng.choice(128, 20, replace=False).tolist()))
    for b in check:
        Kb, Vb = seqs[b]
        ora = (orc.partial(Q[b:b + 1], Kb[None], Vb[None]) if Kb.shape[1] > 0
               else orc.empty_partial(1, w.n_q_heads, w.block_len, w.head_dim))
        T.check_partial({k: v[b:b + 1] for k, v in got.items()}, ora, "bf16", f"{w.name} seq {b}")


@pytest.mark.parametrize("dtype,B,Hq,Hkv,d,P,Bq,page,lens,n_splits", [
    ("bf16", 4, 8, 2, 128, 2048, 32, 128, [1617, 64, 0, 1000], 0),     # library split count
    ("bf16", 3, 8, 2, 128, 4096, 8, 256, [4096, 300, 2222], 4),        # several splits, small block: fold kernel
    ("bf16", 2, 8, 2, 64, 1024, 16, 64, [1024, 65], 1),                # one split: paged pass writes the partial
    ("bf16", 2, 4, 4, 128, 1024, 70, 128, [1000, 512], 3),             # block above 64 rows: combine + internal pass
    ("f32", 3, 4, 2, 64, 576, 8, 64, [200, 0, 513], 2),
    ("f32", 2, 4, 4, 64, 640, 5, 128, [640, 129], 2),                  # block not a multiple of 4
])
def test_paged_refresh_step(dtype, B, Hq, Hkv, d, P, Bq, page, lens, n_splits):
    """fb_refresh_step_paged: cached partial, output and log-normaliser of a whole refresh step on the paged cache."""
    w = _wl(dtype, B, Hq, Hkv, d, P, Bq)
    print(f"[case] paged refresh step {w.name} lens={lens} n_splits={n_splits}", flush=True)
    seqs, Kpool, Vpool, table, lens = wl.make_paged_prefix(w, 51, page, lens)
    Q, Kb, Vb = wl.make_block_steps(w, 51, 1)[0]
    shape = T.shape_of(w)
    q, kb, vb = T.to_dev(Q, dtype), T.to_dev(Kb, dtype), T.to_dev(Vb, dtype)
    kpool, vpool = T.to_dev(Kpool, dtype), T.to_dev(Vpool, dtype)
    tbl, ln = torch.from_numpy(table).to(T.DEV), torch.from_numpy(lens).to(T.DEV)
    kv = fb.make_paged_kv(kpool, vpool, tbl, ln)
    ext = T.Partial(w)
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], device=T.DEV, dtype=torch.float32)
    ws = T.workspace(shape, n_splits=n_splits or fb.fb_paged_splits(shape))
    fb.fb_refresh_step_paged(shape, q, kv, kb, vb, ext.o, ext.m, ext.lse, out, lse, ws, n_splits)
    torch.cuda.synchronize()
    ora_ext = _oracle_partial(w, Q, seqs)
    T.check_partial(ext.numpy(), ora_ext, dtype, f"{w.name} paged refresh ext")
    ora_out, ora_lse = orc.merge(ora_ext, orc.partial(Q, Kb, Vb))
    T.assert_close(out.double().cpu().numpy(), ora_out, dtype, f"{w.name} paged refresh out")
    T.assert_close(lse.double().cpu().numpy(), ora_lse, dtype, f"{w.name} paged refresh lse", lse=True)
