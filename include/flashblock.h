/*
 * flashblock.h - C ABI of the FlashBlock attention hot path for AMD MI355X (gfx950).
 *
 * Block-diffusion attention with a cached block-external partial (arxiv 2602.05305,
 * Section 4.2): the current block's queries against the prefix KV cache are reduced, at a
 * refresh step, to an unnormalised partial output with a per-row reference maximum and the
 * log-normaliser log Z (Eq. 3-4, 6).  That partial is kept by the caller and reused on the
 * following diffusion steps; every step recomputes only the block-internal attention (Eq. 7)
 * and composes the two in log space (Eq. 8-9).  A sparse variant recomputes only selected key
 * blocks and reuses the cached residual of the unselected ones (Section 4.2 "Compatibility
 * with Sparse Attention", Appendix D).
 *
 * General conventions
 *   - Every tensor argument is a DEVICE pointer unless it says "host".  The fb_shape struct is
 *     a host pointer.  Tensors are dense, row-major, last index contiguous:
 *         Q, out            [batch, n_q_heads,  block_len,  head_dim]   dtype
 *         K/V prefix        [batch, n_kv_heads, prefix_len, head_dim]   dtype
 *         K/V block         [batch, n_kv_heads, block_len,  head_dim]   dtype
 *         partial o         [batch, n_q_heads,  block_len,  head_dim]   float
 *         partial m, lse    [batch, n_q_heads,  block_len]              float
 *         pooled keys       [batch, n_kv_heads, ceil(prefix_len/key_block), head_dim] float
 *         selection idx     [batch, n_q_heads,  topk]                   int32
 *     Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - A "partial" (o, m, lse) over a key set J of a query row i means, with natural logarithms
 *     and s_ij = (q_i . k_j) * scale (Eq. 1):
 *         o_i   = sum_{j in J} exp(s_ij - m_i) v_j
 *         lse_i = log sum_{j in J} exp(s_ij)                   ( = L of Eq. 6 )
 *         m_i   = the reference the sum in o_i was taken against; m_i >= max_j s_ij is NOT
 *                 guaranteed to be the exact maximum (split-KV folding keeps the largest
 *                 per-split maximum), only that (o_i, m_i) are paired exactly.
 *     The normalised pair of Eq. 6 is A_i = o_i * exp(m_i - lse_i), L_i = lse_i.
 *     An empty key set gives o = 0, m = lse = -inf.
 *   - Ownership: the caller allocates and frees every buffer, including the workspace.  The
 *     library allocates no device memory, never synchronises the device and launches only on the
 *     HIP stream passed in (hipStream_t cast to void*; NULL is the default stream).  The only
 *     state it keeps between calls is, per kernel, the set of devices on which the kernel's
 *     dynamic-LDS limit has been raised (a one-time hipFuncSetAttribute per kernel and device,
 *     remembered in an atomic word, safe to race from several host threads) and the text of the
 *     last HIP error per thread.  Calls are asynchronous; buffers must stay valid until the stream
 *     has passed the call.  Two calls that share a workspace must be ordered on one stream.
 *   - Alignment: every tensor pointer must be 16-byte aligned (FB_ERR_ALIGN otherwise).
 *   - Errors: every entry point returns an fb_status; nothing throws or aborts.  Arguments are
 *     validated on the host before the first launch, so every error except FB_ERR_HIP leaves
 *     the outputs untouched and can be provoked without a GPU.
 *   - Supported: head_dim in {64, 128}; dtype FB_F32 or FB_BF16 (accumulation, partials and the
 *     merge are always fp32); n_q_heads a multiple of n_kv_heads with at most 32 query heads
 *     per KV head; block_len >= 1; prefix_len >= 0; scale > 0, or 0 for 1/sqrt(head_dim).
 *     key_block (sparse calls) must be a positive multiple of 64.
 */
#ifndef FLASHBLOCK_H_
#define FLASHBLOCK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FB_VERSION 110

typedef enum fb_status {
  FB_OK = 0,
  FB_ERR_NULL = 1,        /* a required pointer is NULL */
  FB_ERR_SHAPE = 2,       /* a dimension, head grouping, scale or mode is out of range */
  FB_ERR_DTYPE = 3,       /* dtype is not FB_F32 / FB_BF16 */
  FB_ERR_ALIGN = 4,       /* a tensor pointer is not 16-byte aligned */
  FB_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than fb_workspace_bytes() */
  FB_ERR_UNSUPPORTED = 6, /* valid request outside what the kernels cover (head_dim, key_block) */
  FB_ERR_HIP = 7          /* a HIP launch failed; hipGetLastError text via fb_last_hip_error() */
} fb_status;

typedef enum fb_dtype { FB_F32 = 0, FB_BF16 = 1 } fb_dtype;

typedef enum fb_sparse_mode {
  FB_SPARSE_REFRESH = 0,  /* stream the whole prefix: write the residual AND selected(+)residual */
  FB_SPARSE_REUSE = 1,    /* stream selected key blocks only, fold in the cached residual */
  FB_SPARSE_REUSE_SAME_SELECTION = 2   /* FB_SPARSE_REUSE with the selection of the previous call (see below) */
} fb_sparse_mode;

/* Problem shape.  Plain data, host memory, caller-owned.  struct_size = sizeof(fb_shape). */
typedef struct fb_shape {
  uint32_t struct_size;
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t block_len;   /* Bq: query rows of the block == rows of the block's own K/V */
  int32_t prefix_len;  /* P: number of prefix (block-external) keys; 0 is legal */
  int32_t dtype;       /* fb_dtype of Q, K, V and out */
  float scale;         /* score scale of Eq. 1; 0 selects 1/sqrt(head_dim) */
} fb_shape;

int fb_version(void);
const char* fb_status_string(int status);
/* Text of the last HIP error seen by this thread's failing call ("" if none). Host string,
 * owned by the library, valid until the next failing call on the same thread. */
const char* fb_last_hip_error(void);

/* Validate a shape exactly as the entry points do (host only, no GPU needed). */
fb_status fb_check_shape(const fb_shape* shape);

/* Number of prefix splits (split-KV workgroups per KV head and row tile) the external pass
 * uses for this shape when the caller passes n_splits = 0.  Host only.  0 on invalid shape. */
int32_t fb_external_splits(const fb_shape* shape);

/* Name (as a profiler's kernel trace prints it, without the namespace) of the streaming attention
 * kernel fb_external_partial launches for this shape with the library's own split count: the
 * kernel whose duration the roofline of the external pass is about.  Host only.  Host string owned
 * by the library, valid until the next call on the same thread; "" on an invalid shape. */
const char* fb_external_kernel_name(const fb_shape* shape);

/* Bytes of device workspace one call needs on this shape.  n_splits = 0 sizes for the
 * library's own split choice (what fb_external_partial and fb_sparse_external_residual use),
 * otherwise for fb_external_partial_ex with that split count.  key_block = 0 sizes the dense
 * external pass only; key_block > 0 sizes both sparse modes as well.  Host only.  Returns 0 on
 * invalid arguments, otherwise at least 256. */
#define FB_MAX_SPLITS 256
size_t fb_workspace_bytes(const fb_shape* shape, int32_t key_block, int32_t topk, int32_t n_splits);

/*
 * External partial at a refresh step: Eq. 3-4 and 6 over J_out = all prefix_len prefix keys.
 * The prefix is cut into splits streamed by separate workgroups; the per-split partials go
 * through `workspace` and are folded by Eq. 5 in a fixed order (bit-reproducible).
 *   in : q [B,Hq,Bq,d], k_prefix/v_prefix [B,Hkv,P,d] (may be NULL iff prefix_len == 0)
 *   out: o_part [B,Hq,Bq,d] float, m_part / lse_part [B,Hq,Bq] float (all overwritten)
 *   workspace: >= fb_workspace_bytes(shape, 0, 0, 0) bytes, contents undefined before and after.
 */
fb_status fb_external_partial(const fb_shape* shape, const void* q, const void* k_prefix,
                              const void* v_prefix, float* o_part, float* m_part, float* lse_part,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* Same, with the number of prefix splits given (1..FB_MAX_SPLITS; 0 = library's choice);
 * workspace >= fb_workspace_bytes(shape, 0, 0, n_splits). */
fb_status fb_external_partial_ex(const fb_shape* shape, const void* q, const void* k_prefix,
                                 const void* v_prefix, float* o_part, float* m_part,
                                 float* lse_part, int32_t n_splits, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);

/*
 * fb_external_partial for callers that cannot allocate device memory at all, not even a workspace: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation, arguments and results as fb_external_partial (library's own split count); the split
 * partials go through a scratch array built into the library (device memory of
 * fb_builtin_workspace_bytes() = 20 MiB per GPU, held until the process ends) instead of a caller
 * workspace.  The call allocates and frees nothing.  Shapes whose fb_workspace_bytes(shape, 0, 0, 0)
 * exceeds that size are rejected with FB_ERR_WORKSPACE before anything is launched (every batch-1
 * LLM-shaped configuration up to 128K context fits; batch 4 at 128K and the video shape do not).
 * All calls on one GPU share the one array: calls that may overlap in time (different streams, or
 * different threads) race on it and must be ordered by the caller; nothing in it has to be cleared
 * between calls.  More than 16 GPUs per process: FB_ERR_UNSUPPORTED.  The first call on a device looks up
 * the array's device address (hipGetSymbolAddress): make it outside graph capture.
 */
size_t fb_builtin_workspace_bytes(void);
fb_status fb_external_partial_builtin_ws(const fb_shape* shape, const void* q, const void* k_prefix,
                                         const void* v_prefix, float* o_part, float* m_part,
                                         float* lse_part, void* hip_stream);

/*
 * Head-wise selective refresh (Section 4.2, "Selective reuse": for video models only heads whose
 * block-external attention is not stable enough across steps are recomputed): fb_external_partial
 * restricted to the query heads with head_mask[b * n_q_heads + h] != 0.  The (o, m, lse) rows of
 * the other heads are left exactly as they are (their cached partial stays in force).  Which
 * heads to refresh is the caller's policy.  head_mask: device, uint8 [B,Hq], required.
 * KV groups none of whose query heads is flagged are not streamed at all.
 * n_active_heads: host-side hint, the largest number of flagged heads in any batch element
 * (0 = unknown, sized as if all were flagged).  The mask lives in device memory, so this is the
 * only way the library can tell that few workgroups will do real work and cut the prefix into
 * more splits to keep the GPU full; a wrong hint costs speed, never correctness.
 * workspace: >= fb_workspace_bytes(shape, 0, 0, fb_external_heads_splits(shape, n_active_heads)).
 */
int32_t fb_external_heads_splits(const fb_shape* shape, int32_t n_active_heads);
fb_status fb_external_partial_heads(const fb_shape* shape, const void* q, const void* k_prefix,
                                    const void* v_prefix, const uint8_t* head_mask,
                                    int32_t n_active_heads, float* o_part, float* m_part,
                                    float* lse_part, void* workspace, size_t workspace_bytes,
                                    void* hip_stream);

/*
 * Paged prefix cache with per-sequence prefix lengths: the deployment shape of the language-model
 * experiments (Section 5, implementation details: a serving framework with a paged KV cache,
 * batches of up to 128 sequences under one token budget; the limitations section asks for kernels
 * compatible with such a cache).  Same operation as fb_external_partial (Eq. 3-4 / Eq. 6 over the
 * block-external keys), but sequence b attends to its own prefix_lens[b] keys, which live in
 * fixed-size pages of a shared pool.
 *
 *   k_pool, v_pool  device, element type shape->dtype, layout [num_pages, n_kv_heads, page_size, head_dim]
 *                   (one KV head's keys of a page are contiguous: a 64-key tile is one 8/16/32 KB run)
 *   block_table     device, int32 [batch, max_pages]: block_table[b][j] = pool page holding keys
 *                   [j*page_size, (j+1)*page_size) of sequence b.  Only entries j < ceil(prefix_lens[b]
 *                   / page_size) are read; each is clamped to [0, num_pages) inside the kernel, so a bad
 *                   id gives a wrong result, never an out-of-pool access.
 *   prefix_lens     device, int32 [batch]; clamped to [0, shape->prefix_len] inside the kernel.
 *                   A sequence with 0 keys gets the empty partial (o = 0, m = lse = -inf).
 *   page_size       multiple of 64 (FB_ERR_UNSUPPORTED otherwise); max_pages * page_size >= shape->prefix_len.
 * shape->prefix_len is the maximum prefix length over the batch: it sizes the work split and the
 * workspace.  n_splits: 0 = library heuristic (fb_paged_splits), else as in fb_external_partial_ex;
 * every sequence's own tile list is cut into that many ranges.  Workspace:
 * fb_workspace_bytes(shape, 0, 0, n_splits > 0 ? n_splits : fb_paged_splits(shape)).  All pointers are borrowed for the
 * duration of the enqueued work; nothing is written except o_part / m_part / lse_part / workspace.
 */
typedef struct fb_paged_kv {
  uint32_t struct_size;        /* sizeof(fb_paged_kv), checked */
  int32_t num_pages;
  int32_t page_size;
  int32_t max_pages;           /* row length of block_table */
  const void* k_pool;
  const void* v_pool;
  const int32_t* block_table;
  const int32_t* prefix_lens;
} fb_paged_kv;

/* Split count fb_external_partial_paged uses for n_splits = 0: ragged lengths make workgroups of
 * unequal length, so it asks for several workgroups per compute unit and lets the hardware
 * dispatcher balance them.  0 if the shape is invalid. */
int32_t fb_paged_splits(const fb_shape* shape);

fb_status fb_external_partial_paged(const fb_shape* shape, const void* q, const fb_paged_kv* kv,
                                    float* o_part, float* m_part, float* lse_part, int32_t n_splits,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * A whole refresh step on the paged cache: fb_external_partial_paged followed by the step's block-internal
 * attention and Eq. 8-9 merge (what fb_internal_merge would return), in two launches where the shape allows it:
 * with one split the paged pass writes the partial itself and the internal pass follows; with several
 * splits and a block of at most 64 rows (a multiple of 4) one kernel folds the splits, computes the rows'
 * block-internal attention and merges; otherwise split combine + internal pass (three launches).
 * Arguments as in fb_external_partial_paged and fb_internal_merge; lse_out may be NULL.  Workspace as for
 * fb_external_partial_paged.  (Batches above 128 sequences add the sequence-ordering launch.)
 */
fb_status fb_refresh_step_paged(const fb_shape* shape, const void* q, const fb_paged_kv* kv,
                                const void* k_block, const void* v_block, float* o_part, float* m_part,
                                float* lse_part, void* out, float* lse_out, int32_t n_splits,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Cross-step similarity of block-external attention per head (Section 3 / Figure 1, used to
 * calibrate the head-wise reuse threshold of Section 4.2): sim[b,h] = mean over the block's rows
 * of the cosine similarity between the external attention outputs A_out of two partials, e.g.
 * the cached one and a freshly computed one.  Only the o tensors are needed: A_out is o times a
 * positive per-row scalar.  A row that is zero in either partial counts as similarity 0.
 *   in : o_a, o_b [B,Hq,Bq,d] float;  out: sim [B,Hq] float.
 */
fb_status fb_head_similarity(const fb_shape* shape, const float* o_a, const float* o_b, float* sim,
                             void* hip_stream);

/*
 * One diffusion step with a cached external partial (Algorithm 1): block-internal attention
 * of q against the block's own current k_block/v_block, bidirectional (Eq. 7), composed in
 * the kernel's epilogue with the cached (o_part, m_part, lse_part) by Eq. 8-9.
 *   in : q [B,Hq,Bq,d], k_block/v_block [B,Hkv,Bq,d]; cached partial, read-only.  Passing
 *        o_part = m_part = lse_part = NULL means "no external keys" (out = A_in).
 *   out: out [B,Hq,Bq,d] in the shape's dtype (round-to-nearest-even for bf16);
 *        lse_out [B,Hq,Bq] float = log(Z_out + Z_in), may be NULL.
 * prefix_len of the shape is ignored here.
 */
fb_status fb_internal_merge(const fb_shape* shape, const void* q, const void* k_block,
                            const void* v_block, const float* o_part, const float* m_part,
                            const float* lse_part, void* out, float* lse_out, void* hip_stream);

/*
 * A whole refresh step in two launches: the single-pass formulation of Section 4.4 (one attention
 * pass over [prefix || block] whose block-external statistics are kept at the block boundary), cut
 * into splits for a 256-CU part.  One streaming launch covers the prefix splits and, as one more
 * split, the block's own keys; the combine launch folds the prefix splits into the partial to
 * cache (o_part, m_part, lse_part: exactly what fb_external_partial returns, up to the order of
 * floating-point sums) and, in the same pass, merges it with the block-internal statistics by
 * Eq. 8-9 into out / lse_out (what fb_internal_merge would return for this step).
 * Arguments as in fb_external_partial and fb_internal_merge; lse_out may be NULL.
 * workspace: >= fb_workspace_bytes(shape, 0, 0, 0).
 */
fb_status fb_refresh_step(const fb_shape* shape, const void* q, const void* k_prefix,
                          const void* v_prefix, const void* k_block, const void* v_block,
                          float* o_part, float* m_part, float* lse_part, void* out, float* lse_out,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Sparse variant, key-block selection (this library's workload rule; the paper leaves the
 * sparse policy to the sparse-attention method it is combined with, Appendix D).
 * fb_pool_keys: mean over the tokens of every key block of key_block tokens (last block may be
 *   short) -> k_pooled [B,Hkv,ceil(P/key_block),d] float.
 * fb_select_topk: score(h, c) = mean_rows(q[b,h]) . k_pooled[b,h/G,c]; the topk blocks with
 *   the largest score, ties to the lower block index, written in ascending block order to
 *   sel_idx [B,Hq,topk] int32.  If topk exceeds the number of blocks the tail is filled
 *   with -1 (consumers skip negative entries).  Scores are computed in fp32.
 *   workspace: device scratch of >= fb_select_workspace_bytes(shape, key_block) bytes (mean
 *   queries and block scores), or NULL.  With it the scoring runs as kernels of its own across
 *   the whole GPU and only the selection proper runs one workgroup per head; without it one
 *   kernel does both (same result bit for bit, slower for prefixes of many key blocks).
 *   A workspace that is given but too small is FB_ERR_WORKSPACE.
 */
fb_status fb_pool_keys(const fb_shape* shape, const void* k_prefix, int32_t key_block,
                       float* k_pooled, void* hip_stream);
size_t fb_select_workspace_bytes(const fb_shape* shape, int32_t key_block);
fb_status fb_select_topk(const fb_shape* shape, const void* q, const float* k_pooled,
                         int32_t key_block, int32_t topk, int32_t* sel_idx, void* workspace,
                         size_t workspace_bytes, void* hip_stream);

/*
 * Key-block selection by attention mass (appendix on adapting the sparse method to block
 * diffusion: the sparse mask of a block is derived from full attention at the block's first
 * diffusion step and frozen for the block).  With p_ij = exp(s_ij - lse_i) the softmax weights of
 * full attention over the prefix (lse_part = the log-normaliser a refresh step's external partial
 * carries for the same q), the score of key block c for query head h is the mean over the block's
 * query rows of sum_{j in c} p_ij; sel_idx gets the topk highest-scoring blocks per head, in the
 * format fb_select_topk writes (ascending, ties to the lower index, -1 padding).
 *   in : q [B,Hq,Bq,d], k_prefix [B,Hkv,P,d], lse_part [B,Hq,Bq] float
 *   out: sel_idx int32 [B,Hq,topk]; mass_out float [B,Hq,nblk] (the scores; may be NULL)
 *   workspace: >= fb_select_mass_workspace_bytes(shape, key_block) bytes (per-row masses).
 * Reads K once (no V).  topk = 0 or prefix_len = 0: nothing is launched.
 */
size_t fb_select_mass_workspace_bytes(const fb_shape* shape, int32_t key_block);
fb_status fb_select_topk_mass(const fb_shape* shape, const void* q, const void* k_prefix,
                              const float* lse_part, int32_t key_block, int32_t topk,
                              int32_t* sel_idx, float* mass_out, void* workspace,
                              size_t workspace_bytes, void* hip_stream);

/*
 * Sparse external pass with residual reuse (Section 4.2 sparse paragraph, Appendix D).
 * J_sel(h) = prefix keys inside the key blocks listed in sel_idx[b,h,:]; J_res(h) = the rest.
 *   mode FB_SPARSE_REFRESH: one pass over the whole prefix with the current q; keys of J_res
 *     feed the residual partial (res_o, res_m, res_lse: written, to be cached by the caller),
 *     keys of J_sel the selected partial; (o_part, m_part, lse_part) = selected (+) residual,
 *     i.e. the exact partial over the whole prefix.
 *   mode FB_SPARSE_REUSE: only key blocks selected by at least one query head of a KV group
 *     are read; the selected partial is recomputed with the current q and folded with the
 *     cached residual (res_*: read-only) into (o_part, m_part, lse_part).
 *   mode FB_SPARSE_REUSE_SAME_SELECTION: FB_SPARSE_REUSE without rebuilding the per-KV-group
 *     selection masks: the selection is frozen between refresh steps, and the masks that the
 *     preceding FB_SPARSE_REFRESH / FB_SPARSE_REUSE call (same shape, key_block, topk, same
 *     workspace, earlier on the same stream) left in the workspace are used again.  sel_idx is
 *     ignored.  The caller guarantees that nothing else wrote the workspace in between; this is
 *     the one case in which workspace contents carry over from call to call.
 * The result is external-shaped and feeds fb_internal_merge unchanged.
 *   sel_idx [B,Hq,topk] int32, entries in [0, n_blocks) or negative (ignored); duplicates
 *   are allowed and count once.  topk = 0 (then sel_idx may be NULL) selects nothing.
 *   workspace: >= fb_workspace_bytes(shape, key_block, topk, 0).
 */
fb_status fb_sparse_external_residual(const fb_shape* shape, int32_t mode, const void* q,
                                      const void* k_prefix, const void* v_prefix,
                                      int32_t key_block, int32_t topk, const int32_t* sel_idx,
                                      float* res_o, float* res_m, float* res_lse, float* o_part,
                                      float* m_part, float* lse_part, void* workspace,
                                      size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FLASHBLOCK_H_ */
