"""Seeded synthetic workloads for the FlashBlock hot path.

This module only draws random tensors of the benchmark configurations' shapes and rounds them
to the configuration's storage type.  It holds none of the method's arithmetic and is the one
module that both the CPU oracle's tests and the HIP path's tests / benchmark use, so that both
sides see bit-identical inputs.  numpy only.

A workload is a prefix KV cache that stays fixed while one block is denoised, plus per-step
block tensors (Q_t, K_block_t, V_block_t) that follow a cumulative random walk between
diffusion steps (the block's tokens are refined step by step while the prefix is frozen,
Section 4.1 of the paper): X_{t+1} = round(X_t + sigma * eps_t), eps_t ~ N(0, 1).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prefix_len: int
    block_len: int
    steps: int            # diffusion steps per block
    refresh: int          # refresh interval R
    dtype: str            # "f32" | "bf16"  (storage type of Q, K, V and the output)
    input_scale: float    # Q, K, V ~ N(0,1) * input_scale
    step_sigma: float = 0.05
    key_block: int = 0    # sparse variant: tokens per key block (0 = dense workload)
    topk: int = 0         # sparse variant: key blocks selected per query head

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)

    @property
    def kv_bytes(self) -> int:
        """Bytes of the prefix K and V together."""
        esz = 4 if self.dtype == "f32" else 2
        return 2 * self.batch * self.n_kv_heads * self.prefix_len * self.head_dim * esz


_S128 = 1.0 / np.sqrt(128.0)

CONFIGS = {
    # tiny fp32 case the oracle finishes instantly
    "tiny_f32": Workload("tiny_f32", 1, 4, 4, 64, 256, 16, 4, 4, "f32", 1.0),
    # LLM-shaped GQA, 32K prefix
    "llm_32k": Workload("llm_32k", 1, 32, 8, 128, 32768, 32, 8, 8, "bf16", _S128),
    # long context, 128K prefix (batch 1 and 4)
    "long_128k": Workload("long_128k", 1, 32, 8, 128, 131072, 32, 8, 8, "bf16", _S128),
    "long_128k_b4": Workload("long_128k_b4", 4, 32, 8, 128, 131072, 32, 8, 8, "bf16", _S128),
    # video-shaped MHA: block = 3 latent frames x 1560 tokens, prefix = 8 previous blocks
    "video": Workload("video", 1, 12, 12, 128, 37440, 4680, 4, 4, "bf16", 1.0),
    # sparse + residual reuse: 64K prefix, 64-token key blocks, 256 of 1024 selected
    "sparse_64k": Workload("sparse_64k", 1, 32, 8, 128, 65536, 32, 8, 8, "bf16", _S128,
                           key_block=64, topk=256),
}


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def round_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    return round_bf16(x) if dtype == "bf16" else x


def make_prefix(w: Workload, seed: int):
    """K, V of the prefix: float32 arrays [B,Hkv,P,d] holding values exactly representable in
    the workload's storage type."""
    rng = np.random.default_rng([seed, 1])
    shape = (w.batch, w.n_kv_heads, w.prefix_len, w.head_dim)
    K = round_storage(rng.standard_normal(shape, dtype=np.float32) * np.float32(w.input_scale), w.dtype)
    V = round_storage(rng.standard_normal(shape, dtype=np.float32) * np.float32(w.input_scale), w.dtype)
    return K, V


def make_block_steps(w: Workload, seed: int, steps: int | None = None):
    """List of (Q_t, K_block_t, V_block_t), t = 0..steps-1, as float32 arrays of storage-exact
    values.  Q [B,Hq,Bq,d]; K_block, V_block [B,Hkv,Bq,d]."""
    rng = np.random.default_rng([seed, 2])
    n = w.steps if steps is None else steps
    qs = (w.batch, w.n_q_heads, w.block_len, w.head_dim)
    ks = (w.batch, w.n_kv_heads, w.block_len, w.head_dim)
    sc = np.float32(w.input_scale)
    Q = round_storage(rng.standard_normal(qs, dtype=np.float32) * sc, w.dtype)
    K = round_storage(rng.standard_normal(ks, dtype=np.float32) * sc, w.dtype)
    V = round_storage(rng.standard_normal(ks, dtype=np.float32) * sc, w.dtype)
    out = [(Q, K, V)]
    sg = np.float32(w.step_sigma)
    for _ in range(1, n):
        Q = round_storage(Q + sg * rng.standard_normal(qs, dtype=np.float32), w.dtype)
        K = round_storage(K + sg * rng.standard_normal(ks, dtype=np.float32), w.dtype)
        V = round_storage(V + sg * rng.standard_normal(ks, dtype=np.float32), w.dtype)
        out.append((Q, K, V))
    return out


def make_paged_prefix(w: Workload, seed: int, page_size: int, lens, spare_pages: int = 3):
    """A paged prefix cache for per-sequence prefix lengths `lens` (one per batch element, each
    <= w.prefix_len).  Returns (seqs, K_pool, V_pool, block_table, lens):
      seqs        list over the batch of (K_b, V_b), float32 [Hkv, lens[b], d]: the contiguous view
      K_pool/V_pool  float32 [num_pages, Hkv, page_size, d]; pages are handed out in a seeded random
                  order, rows past a sequence's length and the spare pages hold random values (reading
                  them would change the result)
      block_table int32 [B, max_pages], -1 where a sequence has no page
      lens        int32 [B]
    """
    rng = np.random.default_rng([seed, 3])
    lens = np.asarray(lens, dtype=np.int32)
    assert lens.shape == (w.batch,) and (lens >= 0).all() and (lens <= w.prefix_len).all()
    max_pages = max(1, -(-w.prefix_len // page_size))
    need = [-(-int(n) // page_size) for n in lens]
    num_pages = sum(need) + spare_pages
    sc = np.float32(w.input_scale)
    pshape = (num_pages, w.n_kv_heads, page_size, w.head_dim)
    K_pool = round_storage(rng.standard_normal(pshape, dtype=np.float32) * sc, w.dtype)
    V_pool = round_storage(rng.standard_normal(pshape, dtype=np.float32) * sc, w.dtype)
    order = rng.permutation(num_pages)
    table = np.full((w.batch, max_pages), -1, dtype=np.int32)
    seqs, nxt = [], 0
    for b in range(w.batch):
        table[b, :need[b]] = order[nxt:nxt + need[b]]
        nxt += need[b]
        n = int(lens[b])
        Kb = np.empty((w.n_kv_heads, n, w.head_dim), dtype=np.float32)
        Vb = np.empty_like(Kb)
        for j in range(need[b]):
            lo, hi = j * page_size, min(n, (j + 1) * page_size)
            Kb[:, lo:hi] = K_pool[table[b, j], :, :hi - lo]
            Vb[:, lo:hi] = V_pool[table[b, j], :, :hi - lo]
        seqs.append((Kb, Vb))
    return seqs, K_pool, V_pool, table, lens
