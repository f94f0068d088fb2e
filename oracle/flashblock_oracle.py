"""CPU oracle for the FlashBlock attention hot path (arxiv 2602.05305).

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct numpy float64
statement of what the HIP library computes.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it; the product path never does.  It shares no code,
tables or helpers with the HIP path and imports nothing from the package.

Notation follows the paper (Section 4.1-4.2, Appendix D):
    s_ij  = q_i . k_j * scale, scale = 1/sqrt(head_dim)                 (Eq. 1)
    Z_i   = sum_j e^{s_ij},  U_i = sum_j e^{s_ij} v_j,  a_i = U_i/Z_i      (Eq. 2)
    in/out decomposition of Z and U over a key partition                 (Eq. 3-4)
    a_i   = (U_out + U_in) / (Z_out + Z_in)                              (Eq. 5)
    cached A_out = U_out/Z_out, L_out = log Z_out                        (Eq. 6)
    recomputed A_in, L_in                                                (Eq. 7)
    m = max(L_out, L_in); log-space composition                          (Eq. 8-9)

Layouts (all numpy float64):
    Q            [B, Hq,  Bq, d]      queries of the current block
    K, V prefix  [B, Hkv, P,  d]      prefix KV cache (block-external keys)
    K, V block   [B, Hkv, Bq, d]      the current block's own keys/values
    a "partial"  dict(o=[B,Hq,Bq,d], m=[B,Hq,Bq], lse=[B,Hq,Bq])
        o   = sum_j e^{s_ij - m_i} v_j      (unnormalised, paired with m)
        m   = max_j s_ij
        lse = m + ln sum_j e^{s_ij - m_i} = log Z                        (Eq. 6)
      An empty key set gives o = 0, m = lse = -inf.
    Query head h reads KV head h // (Hq // Hkv) (grouped-query attention; the paper does not
    discuss GQA, the partial/cache is kept per query head).

Readings of the paper taken here (the paper is silent or garbled on these):
  * d in Eq. 1 is the head dimension.
  * log is the natural logarithm.
  * inside the block the mask is bidirectional; J_out is the whole prefix handed in.
  * Algorithm 1's cache-update lines are read as: on a reuse step the cached pair is carried
    over unchanged; on a refresh step it is overwritten by the freshly computed external pair.
  * refresh rule: a fixed interval R, refresh iff t mod R == 0 (t 0-based within the block);
    the first step of a block always refreshes (Section 4.2, selective reuse).
  * sparse variant (Section 4.2 "Compatibility with Sparse Attention", Appendix D): J_in is the
    selected prefix keys plus the block's keys, J_out the unselected prefix keys; the selection
    and the residual are taken at the refresh step and frozen until the next refresh.  The
    selection rule itself (mean-pooled q . mean-pooled key block, top-k, ties to the lower block
    index) is this build's workload definition, not the paper's.

Pins (tests/test_oracle_pins.py): hand-computed closed forms, torch SDPA / scipy softmax and
logsumexp in float64 on the plain-attention special cases, an augmented-feature construction
that reduces the stale-query reuse step and the sparse reuse step to plain attention, chunk
associativity, brute force top-k, and the cache-size figures printed in Table 5.
"""
from __future__ import annotations

import math

import numpy as np

NEG_INF = -np.inf


# --------------------------------------------------------------------------------------
# Eq. 1-4, 6: statistics of one query block against one key set
# --------------------------------------------------------------------------------------
def default_scale(head_dim: int) -> float:
    """Eq. 1: 1/sqrt(d) with d read as the head dimension."""
    return 1.0 / math.sqrt(float(head_dim))


def scores(Q, K, scale=None):
    """Eq. 1.  Q [B,Hq,Bq,d], K [B,Hkv,P,d] -> s [B,Hq,Bq,P] (float64)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    B, Hq, Bq, d = Q.shape
    Hkv, P = K.shape[1], K.shape[2]
    assert K.shape[0] == B and K.shape[3] == d and Hq % Hkv == 0
    G = Hq // Hkv
    if scale is None:
        scale = default_scale(d)
    s = np.empty((B, Hq, Bq, P), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            s[b, h] = (Q[b, h] @ K[b, h // G].T) * scale
    return s


def partial(Q, K, V, scale=None, key_mask=None):
    """Eq. 3-4 and 6 for one key set: the unnormalised weighted value sum, the row maximum and
    log Z of every query row.

    key_mask: optional bool [B,Hq,P]; False keys do not belong to the key set of that query
    head (used for the selected / unselected split of the sparse variant).
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, Hq, Bq, d = Q.shape
    Hkv, P = K.shape[1], K.shape[2]
    G = Hq // Hkv
    if scale is None:
        scale = default_scale(d)
    o = np.zeros((B, Hq, Bq, V.shape[3]), dtype=np.float64)   # value width may differ from d
    m = np.full((B, Hq, Bq), NEG_INF, dtype=np.float64)
    lse = np.full((B, Hq, Bq), NEG_INF, dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            kk, vv = K[b, h // G], V[b, h // G]
            if key_mask is not None:
                keep = np.asarray(key_mask[b, h], dtype=bool)
                kk, vv = kk[keep], vv[keep]
            if kk.shape[0] == 0:
                continue
            s = (Q[b, h] @ kk.T) * scale                    # [Bq, n]           Eq. 1
            mi = s.max(axis=1)                               # row max
            p = np.exp(s - mi[:, None])                      # e^{s - m}
            z = p.sum(axis=1)                                # Z e^{-m}          Eq. 3-4
            o[b, h] = p @ vv                                 # U e^{-m}          Eq. 3-4
            m[b, h] = mi
            lse[b, h] = mi + np.log(z)                       # L = log Z         Eq. 6
    return {"o": o, "m": m, "lse": lse}


def normalized(part):
    """Eq. 6: A = U/Z from an (o, m, lse) partial; rows of an empty key set give 0."""
    o, m, lse = part["o"], part["m"], part["lse"]
    with np.errstate(invalid="ignore"):
        w = np.where(np.isneginf(lse), 0.0, np.exp(m - lse))   # e^{m}/Z
    return o * w[..., None]


def empty_partial(B, Hq, Bq, d):
    return {"o": np.zeros((B, Hq, Bq, d)), "m": np.full((B, Hq, Bq), NEG_INF),
            "lse": np.full((B, Hq, Bq), NEG_INF)}


# --------------------------------------------------------------------------------------
# Eq. 5 / 8-9: composition
# --------------------------------------------------------------------------------------
def merge(ext, inn):
    """Eq. 8-9: compose the cached external pair (A_out, L_out) with the recomputed internal
    pair (A_in, L_in).  Returns (A_full [B,Hq,Bq,d], L_full [B,Hq,Bq]).  If both sides are empty
    the output row is 0 and L_full = -inf."""
    A_out, L_out = normalized(ext), ext["lse"]
    A_in, L_in = normalized(inn), inn["lse"]
    mm = np.maximum(L_out, L_in)                                             # Eq. 8
    safe = np.where(np.isneginf(mm), 0.0, mm)
    w_out = np.where(np.isneginf(L_out), 0.0, np.exp(L_out - safe))
    w_in = np.where(np.isneginf(L_in), 0.0, np.exp(L_in - safe))
    den = w_out + w_in
    num = w_out[..., None] * A_out + w_in[..., None] * A_in                 # Eq. 9
    with np.errstate(divide="ignore", invalid="ignore"):
        A_full = np.where(den[..., None] > 0, num / np.where(den > 0, den, 1.0)[..., None], 0.0)
        L_full = np.where(den > 0, mm + np.log(np.where(den > 0, den, 1.0)), NEG_INF)
    return A_full, L_full


def merge_uz(ext, inn):
    """Eq. 5 taken literally, with plain (unshifted) exponentials: (U_out+U_in)/(Z_out+Z_in).
    Only safe for moderate score ranges; kept as the comparator for Eq. 8-9."""
    U_out = normalized(ext) * np.exp(ext["lse"])[..., None]
    U_in = normalized(inn) * np.exp(inn["lse"])[..., None]
    Z = np.exp(ext["lse"]) + np.exp(inn["lse"])
    return (U_out + U_in) / Z[..., None], np.log(Z)


def merge_partials(a, b):
    """Eq. 5 applied to two partials, result again a partial (used to fold split-KV chunks and
    to form selected (+) residual in the sparse variant)."""
    M = np.maximum(a["m"], b["m"])
    safe = np.where(np.isneginf(M), 0.0, M)
    wa = np.where(np.isneginf(a["m"]), 0.0, np.exp(a["m"] - safe))
    wb = np.where(np.isneginf(b["m"]), 0.0, np.exp(b["m"] - safe))
    o = a["o"] * wa[..., None] + b["o"] * wb[..., None]
    with np.errstate(invalid="ignore"):
        za = np.where(np.isneginf(a["lse"]), 0.0, np.exp(a["lse"] - a["m"])) * wa
        zb = np.where(np.isneginf(b["lse"]), 0.0, np.exp(b["lse"] - b["m"])) * wb
    z = za + zb
    with np.errstate(divide="ignore"):
        lse = np.where(z > 0, M + np.log(np.where(z > 0, z, 1.0)), NEG_INF)
    return {"o": o, "m": M, "lse": lse}


# --------------------------------------------------------------------------------------
# Comparators: plain attention, and the reuse step written without any LSE machinery
# --------------------------------------------------------------------------------------
def full_attention(Q, K, V, scale=None):
    """Eq. 1-2 directly: softmax(Q K^T scale) V over all given keys.  Returns (a, log Z)."""
    s = scores(Q, K, scale)
    B, Hq, Bq, d = np.asarray(Q).shape
    G = Hq // np.asarray(K).shape[1]
    V = np.asarray(V, dtype=np.float64)
    a = np.empty((B, Hq, Bq, V.shape[3]))
    logz = np.empty((B, Hq, Bq))
    for b in range(B):
        for h in range(Hq):
            sm = s[b, h].max(axis=1, keepdims=True)
            e = np.exp(s[b, h] - sm)
            z = e.sum(axis=1, keepdims=True)
            a[b, h] = (e / z) @ V[b, h // G]
            logz[b, h] = (sm + np.log(z))[:, 0]
    return a, logz


def stale_query_bruteforce(Q_refresh, Q_now, K_prefix, V_prefix, K_block, V_block, scale=None):
    """What a reuse step returns, written from Eq. 3-5 with the step superscripts of Eq. 6-7
    and 9: prefix terms use the query of the last refresh step, block terms the current query.
    Plain exponentials, no shift (float64, moderate score ranges only)."""
    s_out = scores(Q_refresh, K_prefix, scale)
    s_in = scores(Q_now, K_block, scale)
    B, Hq, Bq, d = np.asarray(Q_now).shape
    G = Hq // np.asarray(K_prefix).shape[1]
    Vp = np.asarray(V_prefix, dtype=np.float64)
    Vb = np.asarray(V_block, dtype=np.float64)
    out = np.empty((B, Hq, Bq, Vp.shape[3]))
    for b in range(B):
        for h in range(Hq):
            e_out, e_in = np.exp(s_out[b, h]), np.exp(s_in[b, h])
            U = e_out @ Vp[b, h // G] + e_in @ Vb[b, h // G]
            Z = e_out.sum(axis=1) + e_in.sum(axis=1)
            out[b, h] = U / Z[:, None]
    return out


# --------------------------------------------------------------------------------------
# Key-block selection (workload definition for the sparse configuration)
# --------------------------------------------------------------------------------------
def pool_keys(K, key_block):
    """Mean of every key block's tokens (the last block may be short): [B,Hkv,ceil(P/kb),d]."""
    K = np.asarray(K, dtype=np.float64)
    B, Hkv, P, d = K.shape
    nblk = -(-P // key_block)
    out = np.zeros((B, Hkv, nblk, d))
    for c in range(nblk):
        out[:, :, c] = K[:, :, c * key_block:min(P, (c + 1) * key_block)].mean(axis=2)
    return out


def select_scores(Q, K_pooled):
    """Mean over the block's query rows of head h, dotted with each pooled key block of KV head
    h // G.  [B,Hq,nblk]."""
    Q = np.asarray(Q, dtype=np.float64)
    B, Hq, Bq, d = Q.shape
    G = Hq // K_pooled.shape[1]
    qbar = Q.mean(axis=2)
    sc = np.empty((B, Hq, K_pooled.shape[2]))
    for b in range(B):
        for h in range(Hq):
            sc[b, h] = K_pooled[b, h // G] @ qbar[b, h]
    return sc


def select_topk(Q, K, key_block, topk):
    """Indices of the top-k key blocks per (batch, query head), ascending; ties go to the lower
    block index; topk is clamped to the number of key blocks.  int32 [B,Hq,min(topk,nblk)]."""
    sc = select_scores(Q, pool_keys(K, key_block))
    B, Hq, nblk = sc.shape
    k = min(int(topk), nblk)
    idx = np.empty((B, Hq, k), dtype=np.int32)
    for b in range(B):
        for h in range(Hq):
            order = sorted(range(nblk), key=lambda c: (-sc[b, h, c], c))
            idx[b, h] = np.array(sorted(order[:k]), dtype=np.int32)
    return idx


def block_mass(Q, K, key_block, scale=None):
    """Attention mass per key block at a step that computes full attention over the prefix (the
    step the sparse mask is derived from, Appendix "Adapting SparseD to Block dLLM"): with
    p_ij = softmax_j(s_ij) over all prefix keys (Eq. 1-2 restricted to J_out), the mass of block c
    for query head h is the mean over the block's query rows i of sum_{j in c} p_ij.
    [B,Hq,nblk]; every (b, h) row sums to 1."""
    S = scores(Q, K, scale)                                   # [B,Hq,Bq,P]
    P = S.shape[-1]
    nblk = -(-P // key_block)
    mx = S.max(axis=-1, keepdims=True)
    e = np.exp(S - mx)
    prob = e / e.sum(axis=-1, keepdims=True)
    mass = np.zeros(S.shape[:2] + (nblk,))
    for c in range(nblk):
        mass[:, :, c] = prob[..., c * key_block:min(P, (c + 1) * key_block)].sum(axis=-1).mean(axis=-1)
    return mass


def select_topk_scores(sc, topk):
    """Top-k key blocks per (batch, query head) of given block scores [B,Hq,nblk]: ascending
    indices, ties to the lower block index, topk clamped to nblk.  int32 [B,Hq,min(topk,nblk)]."""
    sc = np.asarray(sc, dtype=np.float64)
    B, Hq, nblk = sc.shape
    k = min(int(topk), nblk)
    idx = np.empty((B, Hq, k), dtype=np.int32)
    for b in range(B):
        for h in range(Hq):
            order = sorted(range(nblk), key=lambda c: (-sc[b, h, c], c))
            idx[b, h] = np.array(sorted(order[:k]), dtype=np.int32)
    return idx


def selection_key_mask(idx, P, key_block):
    """bool [B,Hq,P]: True for prefix keys inside a selected key block."""
    B, Hq, k = idx.shape
    mask = np.zeros((B, Hq, P), dtype=bool)
    for b in range(B):
        for h in range(Hq):
            for c in idx[b, h]:
                if c >= 0:
                    mask[b, h, int(c) * key_block:min(P, (int(c) + 1) * key_block)] = True
    return mask


# --------------------------------------------------------------------------------------
# The per-block step drivers (Algorithm 1 around a fixed refresh interval R)
# --------------------------------------------------------------------------------------
def run_block_dense(K_prefix, V_prefix, steps, R, scale=None):
    """steps: list of (Q_t, K_block_t, V_block_t).  Returns one dict per step with
    out, lse (Eq. 9 result and its log-normaliser), ext (the external partial in force),
    refreshed (bool)."""
    res, ext = [], None
    for t, (Q, Kb, Vb) in enumerate(steps):
        refreshed = (t % R == 0)
        if refreshed:
            ext = partial(Q, K_prefix, V_prefix, scale)      # refresh: recompute and cache
        inn = partial(Q, Kb, Vb, scale)                      # always recomputed (Eq. 7)
        out, lse = merge(ext, inn)                           # Eq. 8-9
        res.append({"out": out, "lse": lse, "ext": ext, "int": inn, "refreshed": refreshed})
    return res


def run_block_sparse(K_prefix, V_prefix, steps, R, key_block, topk, scale=None):
    """Sparse variant with residual reuse (Appendix D).  Per step: idx, residual partial
    (cached at refresh), selected partial (recomputed with the current query and the frozen
    idx), ext = selected (+) residual, out/lse = merge(ext, internal)."""
    P = np.asarray(K_prefix).shape[2]
    res, idx, residual = [], None, None
    for t, (Q, Kb, Vb) in enumerate(steps):
        refreshed = (t % R == 0)
        if refreshed:
            idx = select_topk(Q, K_prefix, key_block, topk)
            kmask = selection_key_mask(idx, P, key_block)
            residual = partial(Q, K_prefix, V_prefix, scale, key_mask=~kmask)
        kmask = selection_key_mask(idx, P, key_block)
        sel = partial(Q, K_prefix, V_prefix, scale, key_mask=kmask)
        ext = merge_partials(sel, residual)
        inn = partial(Q, Kb, Vb, scale)
        out, lse = merge(ext, inn)
        sparse_only, _ = merge(sel, inn)                      # sparse attention without the residual
        res.append({"out": out, "lse": lse, "ext": ext, "sel": sel, "residual": residual, "int": inn,
                    "idx": idx, "refreshed": refreshed, "sparse_only": sparse_only})
    return res


# --------------------------------------------------------------------------------------
# Cross-step similarity (Section 3, Figure 1; calibration of the head-wise threshold, Section 4.2)
# --------------------------------------------------------------------------------------
def head_similarity(part_a, part_b):
    """[B,Hq]: mean over the block's rows of the cosine similarity between the normalised
    block-external outputs A_out of two partials (a zero row counts as similarity 0)."""
    A, Bm = normalized(part_a), normalized(part_b)
    num = (A * Bm).sum(axis=-1)
    den = np.sqrt((A * A).sum(axis=-1)) * np.sqrt((Bm * Bm).sum(axis=-1))
    with np.errstate(divide="ignore", invalid="ignore"):
        cos = np.where(den > 0, num / np.where(den > 0, den, 1.0), 0.0)
    return cos.mean(axis=-1)


# --------------------------------------------------------------------------------------
# Cache footprint (Section 4.4 complexity paragraph; Table 5 "Extra Mem.")
# --------------------------------------------------------------------------------------
def cache_bytes_paper_layout(n_layers, n_heads, block_rows, head_dim, batch=1,
                             a_bytes=2, l_bytes=4):
    """Bytes of the cached (A_out, L_out) pair: one head_dim vector (half precision) and one
    fp32 log-normaliser per (layer, head, block query row) - independent of context length."""
    return batch * n_layers * n_heads * block_rows * (head_dim * a_bytes + l_bytes)
