"""The pins in test_oracle_pins.py are only worth something if a plausible mistake in the oracle
makes one of them fail.  Each case here plants one such mistake in the oracle (on the CPU, by
patching one function) and checks that the named pin catches it."""
import math

import numpy as np
import pytest

from oracle import flashblock_oracle as orc

import test_oracle_pins as pins


def _wrong_scale(head_dim):                       # 1/d instead of 1/sqrt(d)
    return 1.0 / float(head_dim)


def _partial_wrong_gqa(Q, K, V, scale=None, key_mask=None):     # head h reads KV head h % Hkv
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    Hq, Hkv = Q.shape[1], K.shape[1]
    perm = [h % Hkv for h in range(Hq)]
    G = Hq // Hkv
    K2 = np.stack([K[:, perm[h]] for h in range(Hq)], axis=1)
    V2 = np.stack([V[:, perm[h]] for h in range(Hq)], axis=1)
    km = key_mask
    return _ORIG["partial"](Q, K2, V2, scale if scale is not None else 1.0 / math.sqrt(Q.shape[-1]), km)


def _partial_log2(Q, K, V, scale=None, key_mask=None):          # lse in base 2
    p = _ORIG["partial"](Q, K, V, scale, key_mask)
    z = np.where(np.isneginf(p["lse"]), 0.0, np.exp(p["lse"] - p["m"]))
    with np.errstate(divide="ignore"):
        p["lse"] = np.where(z > 0, p["m"] + np.log2(np.where(z > 0, z, 1.0)), -np.inf)
    return p


def _partial_transposed_pv(Q, K, V, scale=None, key_mask=None):  # weights applied to K instead of V
    return _ORIG["partial"](Q, K, K, scale, key_mask)


def _merge_swapped_weights(ext, inn):                            # w_out multiplies A_in
    A_out, L_out = orc.normalized(ext), ext["lse"]
    A_in, L_in = orc.normalized(inn), inn["lse"]
    mm = np.maximum(L_out, L_in)
    w_out, w_in = np.exp(L_out - mm), np.exp(L_in - mm)
    return (w_out[..., None] * A_in + w_in[..., None] * A_out) / (w_out + w_in)[..., None], mm + np.log(w_out + w_in)


def _merge_dropped_normaliser(ext, inn):                         # denominator forgets the external weight
    A_out, L_out = orc.normalized(ext), ext["lse"]
    A_in, L_in = orc.normalized(inn), inn["lse"]
    mm = np.maximum(L_out, L_in)
    w_out, w_in = np.exp(L_out - mm), np.exp(L_in - mm)
    return (w_out[..., None] * A_out + w_in[..., None] * A_in) / w_in[..., None], mm + np.log(w_out + w_in)


def _merge_partials_no_rescale(a, b):                            # forgets e^{m_b - M} on the second operand
    M = np.maximum(a["m"], b["m"])
    wa = np.where(np.isneginf(a["m"]), 0.0, np.exp(a["m"] - np.where(np.isneginf(M), 0.0, M)))
    o = a["o"] * wa[..., None] + b["o"]
    za = np.where(np.isneginf(a["lse"]), 0.0, np.exp(a["lse"] - a["m"])) * wa
    zb = np.where(np.isneginf(b["lse"]), 0.0, np.exp(b["lse"] - b["m"]))
    z = za + zb
    with np.errstate(divide="ignore"):
        return {"o": o, "m": M, "lse": np.where(z > 0, M + np.log(np.where(z > 0, z, 1.0)), -np.inf)}


def _run_block_dense_fresh_query(K_prefix, V_prefix, steps, R, scale=None):   # "reuse" recomputes with the new query
    return _ORIG["run_block_dense"](K_prefix, V_prefix, steps, 1, scale)


def _run_block_dense_late_refresh(K_prefix, V_prefix, steps, R, scale=None):  # refreshes at t % R == R-1 (and t = 0)
    res, ext = [], None
    for t, (Q, Kb, Vb) in enumerate(steps):
        refreshed = (t == 0) or (t % R == R - 1)
        if refreshed:
            ext = orc.partial(Q, K_prefix, V_prefix, scale)
        inn = orc.partial(Q, Kb, Vb, scale)
        out, lse = orc.merge(ext, inn)
        res.append({"out": out, "lse": lse, "ext": ext, "int": inn, "refreshed": refreshed})
    return res


def _select_topk_ties_high(Q, K, key_block, topk):               # ties go to the higher block index
    sc = orc.select_scores(Q, orc.pool_keys(K, key_block))
    B, Hq, nblk = sc.shape
    k = min(int(topk), nblk)
    idx = np.empty((B, Hq, k), dtype=np.int32)
    for b in range(B):
        for h in range(Hq):
            order = sorted(range(nblk), key=lambda c: (-sc[b, h, c], -c))
            idx[b, h] = np.array(sorted(order[:k]), dtype=np.int32)
    return idx


def _pool_keys_sum(K, key_block):                                # sum instead of mean: the short last block ranks wrong
    K = np.asarray(K, dtype=np.float64)
    B, Hkv, P, d = K.shape
    nblk = -(-P // key_block)
    out = np.zeros((B, Hkv, nblk, d))
    for c in range(nblk):
        out[:, :, c] = K[:, :, c * key_block:min(P, (c + 1) * key_block)].sum(axis=2)
    return out


def _selection_mask_off_by_one(idx, P, key_block):               # selected blocks shifted by one token
    m = _ORIG["selection_key_mask"](idx, P, key_block)
    return np.roll(m, 1, axis=-1)


def _block_mass_unnormalised(Q, K, key_block, scale=None):       # weights against the row maximum, not the row sum
    S = orc.scores(Q, K, scale)
    e = np.exp(S - S.max(axis=-1, keepdims=True))
    nblk = -(-S.shape[-1] // key_block)
    return np.stack([e[..., c * key_block:(c + 1) * key_block].sum(-1).mean(-1) for c in range(nblk)], axis=-1)


def _block_mass_wrong_kv_head(Q, K, key_block, scale=None):      # head h reads KV head h % Hkv
    Q, K = np.asarray(Q), np.asarray(K)
    Hq, Hkv = Q.shape[1], K.shape[1]
    out = [_ORIG["block_mass"](Q[:, h:h + 1], K[:, (h % Hkv):(h % Hkv) + 1], key_block, scale) for h in range(Hq)]
    return np.concatenate(out, axis=1)


def _select_topk_scores_ties_high(sc, topk):                     # ties go to the higher index
    sc = np.asarray(sc, dtype=np.float64)
    B, Hq, nblk = sc.shape
    k = min(int(topk), nblk)
    idx = np.empty((B, Hq, k), dtype=np.int32)
    for b in range(B):
        for h in range(Hq):
            order = sorted(range(nblk), key=lambda c: (-sc[b, h, c], -c))
            idx[b, h] = np.array(sorted(order[:k]), dtype=np.int32)
    return idx


def _cache_bytes_fp32_a(n_layers, n_heads, block_rows, head_dim, batch=1, a_bytes=4, l_bytes=4):
    return _ORIG["cache_bytes_paper_layout"](n_layers, n_heads, block_rows, head_dim, batch, a_bytes, l_bytes)


_ORIG = {n: getattr(orc, n) for n in ("partial", "run_block_dense", "selection_key_mask", "cache_bytes_paper_layout",
                                      "block_mass")}

MUTATIONS = [
    ("default_scale", _wrong_scale, pins.test_hand_case_scale_and_weights),
    ("partial", _partial_wrong_gqa, lambda: pins.test_refresh_step_equals_plain_attention_sdpa(1, dict())),
    ("partial", _partial_log2, pins.test_hand_case_scale_and_weights),
    ("partial", _partial_transposed_pv, pins.test_zero_keys_uniform_weights),
    ("merge", _merge_swapped_weights, lambda: pins.test_refresh_step_equals_plain_attention_sdpa(1, dict())),
    ("merge", _merge_dropped_normaliser, pins.test_hand_case_merge),
    ("merge_partials", _merge_partials_no_rescale, pins.test_chunk_associativity_any_order),
    ("run_block_dense", _run_block_dense_fresh_query, pins.test_reuse_step_equals_augmented_sdpa_and_bruteforce),
    ("run_block_dense", _run_block_dense_late_refresh, lambda: pins.test_refresh_schedule_and_interval_one(3)),
    ("select_topk", _select_topk_ties_high, pins.test_topk_ties_go_to_lower_index_and_bruteforce),
    ("pool_keys", _pool_keys_sum, pins.test_pool_and_topk_hand_example),
    ("selection_key_mask", _selection_mask_off_by_one, pins.test_selection_key_mask_hand_example),
    ("selection_key_mask", _selection_mask_off_by_one, pins.test_sparse_reuse_equals_augmented_sdpa),
    ("cache_bytes_paper_layout", _cache_bytes_fp32_a, pins.test_cache_bytes_match_table5),
    ("block_mass", _block_mass_unnormalised, pins.test_block_mass_closed_forms),
    ("block_mass", _block_mass_wrong_kv_head, pins.test_block_mass_closed_forms),
    ("block_mass", _block_mass_wrong_kv_head, pins.test_block_mass_matches_library_softmax_and_sums_to_one),
    ("select_topk_scores", _select_topk_scores_ties_high, pins.test_select_topk_scores_hand_and_bruteforce),
]


@pytest.mark.parametrize("name,mutant,pin", MUTATIONS, ids=[f"{n}:{m.__name__}" for n, m, _ in MUTATIONS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant, pin):
    pin()                                          # the pin holds on the real oracle
    monkeypatch.setattr(orc, name, mutant)
    with pytest.raises((AssertionError, ValueError)):
        pin()
