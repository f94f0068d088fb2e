// Internal interface between the C-ABI layer (fb_api.hip) and the gfx950 kernels.
// Not installed; the public contract is include/flashblock.h.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

namespace fb {

constexpr int kKeyTile = 64;  // keys per main-loop iteration in every attention kernel

// Division of a non-negative 31-bit integer by a launch-time constant, without the ~25
// instruction integer-division sequence in the (cold, run-once) kernel prologue:
// q = (mulhi(n, magic) + n) >> shift with magic = floor(2^32 (2^shift - d) / d) + 1, shift = ceil(log2 d).
struct FastDiv {
  uint32_t magic, shift, d;
};

inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  uint32_t s = 0;
  while ((1ull << s) < d) ++s;
  f.shift = s;
  f.magic = (uint32_t)((((1ull << s) - d) << 32) / d + 1);
  return f;
}

__host__ __device__ __forceinline__ uint32_t fastdiv(uint32_t n, const FastDiv& f) {
#if defined(__HIP_DEVICE_COMPILE__)
  const uint64_t t = (uint64_t)__umulhi(n, f.magic) + n;
#else
  const uint64_t t = (((uint64_t)n * f.magic) >> 32) + n;
#endif
  return (uint32_t)(t >> f.shift);
}

// Kernels with more than 64 KiB of dynamic LDS need their per-kernel limit raised before the first launch on a
// device.  One flag word per kernel remembers the devices on which that was done (bit d = device d): the only
// state the library keeps between calls.  It is an atomic, so concurrent first calls from several host threads are
// safe (the attribute call is idempotent), and it is per device, so a second GPU gets its own call.
struct LdsLimit {
  std::atomic<uint32_t> devices{0};
};

// bytes: what this launch needs; limit: what to ask for (the kernel's fixed size, or, for kernels whose size
// varies from call to call, kLdsLimitMax, which leaves room for their small static arrays).
constexpr size_t kLdsLimitMax = 160 * 1024 - 2048;

template <typename K>
hipError_t raise_lds_limit(K kern, size_t bytes, LdsLimit& st, size_t limit) {
  if (bytes <= 48 * 1024) return hipSuccess;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint32_t bit = (dev >= 0 && dev < 32) ? (1u << dev) : 0u;
  if (bit != 0u && (st.devices.load(std::memory_order_acquire) & bit) != 0u) return hipSuccess;
  e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)limit);
  if (e == hipSuccess && bit != 0u) st.devices.fetch_or(bit, std::memory_order_release);
  return e;
}

// Measurement hook (include/flashblock_prof.h): events that the NEXT bf16 attention launch of this host thread is to
// carry as its own start / stop events (hipExtLaunchKernelGGL: the timestamps of the kernel's dispatch, what a
// profiler's kernel trace reports, instead of markers recorded around it).  Cleared by the launch that takes them.
struct KernelEvents {
  hipEvent_t start = nullptr, stop = nullptr;
};
inline thread_local KernelEvents tl_kernel_events;

template <typename K, typename P>
void launch_attn_kernel(K kern, dim3 grid, dim3 block, size_t lds, hipStream_t s, const P& params) {
  KernelEvents& ev = tl_kernel_events;
  if (ev.start != nullptr || ev.stop != nullptr) {
    hipExtLaunchKernelGGL(kern, grid, block, lds, s, ev.start, ev.stop, 0, params);
    ev = KernelEvents{};
  } else {
    hipLaunchKernelGGL(kern, grid, block, lds, s, params);
  }
}

// What a pass iterates over and what it emits.
enum PassMode : int {
  kPassDense = 0,          // keys [0, nkeys) cut into nsplit tile ranges -> split partials
  kPassInternal = 1,       // keys [0, nkeys), no split; epilogue = Eq. 8-9 merge with cached partial
  kPassSparseRefresh = 2,  // like dense, but every key block is routed to the selected or the residual set
  kPassSparseReuse = 3,    // only key blocks of the per-KV-group union list; selected set only
  kPassDenseHeads = 4,     // dense, but only query heads flagged in head_on take part (others keep their cache)
  kPassDensePaged = 5,     // dense over a paged KV pool with a block table and per-sequence prefix lengths
  kPassRefreshFused = 6    // dense over the prefix plus one extra split over the block's own keys (partial set 1)
};

// One attention pass.  Rows of one KV group are addressed "group-flattened": query head
// kvh*G+g, block row i  <->  flat row g*Bq+i, which is contiguous in Q / partial / out memory.
struct PassParams {
  const void* q;        // [B,Hq,Bq,D]
  const void* k;        // [B,Hkv,nkeys,D]
  const void* v;        // [B,Hkv,nkeys,D]
  int B, Hq, Hkv, G, Bq, nkeys;
  int nsplit;
  float scale_log2;     // scale * log2(e): scores are kept in the log2 domain inside the kernels
  // split partial sets in the workspace, layout [set][split][B*Hq*Bq] rows:
  //   o [.., D] sum exp2(s2 - m2) v ; m2 (log2 domain reference) ; l = sum exp2(s2 - m2)
  float* ws_o;  float* ws_m;  float* ws_l;      // set 0: dense / selected
  float* ws_o2; float* ws_m2; float* ws_l2;     // set 1: residual (sparse refresh only)
  // internal pass epilogue
  const float* ext_o; const float* ext_m; const float* ext_lse;   // cached partial (natural log), may be null
  void* out; float* lse_out;
  // sparse passes
  const uint32_t* blk_mask;   // [B,Hkv,nblk] bit g set: head g of the group selected the block
  const int32_t* union_list;  // [B,Hkv,nblk] ascending blocks with mask != 0
  const uint32_t* union_mask; // [B,Hkv,nblk] mask of the i-th listed block (no dependent lookup in the reuse pass)
  const int32_t* union_cnt;   // [B,Hkv]
  int key_block, nblk;
  const uint8_t* head_on;     // [B,Hq] per-head refresh flags (kPassDenseHeads), else null
  // paged pass: k/v point at the pools [num_pages, Hkv, page_size, D]
  const int32_t* block_table; // [B, max_pages] page ids
  const int32_t* prefix_lens; // [B] keys per sequence (<= nkeys)
  int page_size, max_pages, num_pages;
  const int32_t* seq_order;   // [B] sequences by descending prefix length (longest work is dispatched first), or null
  int order_inline;           // seq_order == null and 1: each workgroup ranks the (few) sequences itself
  // fused refresh pass: the block's own K/V [B,Hkv,Bq,D] go into partial set 1 (bf16: second phase of the last
  // split's workgroup, which gets blk_cost prefix tiles fewer; fp32: one extra split index)
  const void* k2; const void* v2; int blk_cost;
  // dense / heads / paged pass with nsplit == 1: ws_o / ws_m / ws_l are the caller's final (o, m, lse)
  // arrays and the kernel emits natural-log units itself (no combine pass)
  int direct;
  // streaming bf16 pass: 1 = splits alternate between the even and the odd XCD of a pair and the odd XCDs' splits are a
  // little shorter (see biased_range)
  int xcd_bias;
  FastDiv div_rowtiles, div_nsplit, div_hkv;   // bf16 pass: decomposition of the linear workgroup index
  FastDiv div_page;                            // bf16 paged pass: key index -> page slot
  FastDiv div_tpb;                             // streaming sparse passes: tile index -> key block (tiles per key block)
};

// Fold split partials (and optionally a cached residual) into final (o, m, lse) partials.
struct CombineParams {
  int rows, D, nsplit;
  const float* ws_o;  const float* ws_m;  const float* ws_l;    // selected / dense set, may be null when nsplit==0
  const float* ws_o2; const float* ws_m2; const float* ws_l2;   // residual set (refresh) or null
  const float* res_in_o; const float* res_in_m; const float* res_in_lse;   // cached residual (reuse) or null
  float* res_out_o; float* res_out_m; float* res_out_lse;                  // residual out (refresh) or null
  float* o; float* m; float* lse;                                          // total out
  const uint8_t* head_on; int Bq;   // if head_on != null: rows of heads with a zero flag are left untouched
  // fused refresh step: block-internal partial (one split, log2 domain) merged with the total by Eq. 8-9 into
  // the normalised output (storage type) and its log-normaliser; null = no final output
  const float* blk_o; const float* blk_m; const float* blk_l;
  void* fin_out; float* fin_lse; int fin_bf16;
  // ... or, for a block of at most kMaxInlineBlock keys, the block's q / k / v themselves (storage type
  // fin_bf16): the fold kernel computes the block-internal attention of its rows itself
  const void* blk_q; const void* blk_k; const void* blk_v;
  int Hq, Hkv, G; float scale_log2;
};

struct SelectParams {
  const void* q; const float* k_pooled; int32_t* sel_idx;
  int B, Hq, Hkv, G, Bq, D, nblk, topk, is_bf16;
  // score source "attention mass": per-row masses [B][nblk][Hq*Bq] (then q / k_pooled are unused), and an
  // optional copy of the block scores [B,Hq,nblk]
  const float* rowmass; float* score_out;
  // optional scratch: mean queries [B,Hq,D] and block scores [B,Hq,nblk]; both set = scoring runs as kernels of
  // its own over the whole chip instead of inside the (one workgroup per head) selection kernel
  float* qbar_ws; float* scores_ws;
};

// Attention mass of every (query row, key block): sum over the block's keys of exp(s - lse).
struct MassParams {
  const void* q; const void* k; const float* lse; float* rowmass;   // rowmass [B][nblk][Hq*Bq]
  int B, Hq, Hkv, G, Bq, nkeys, key_block, nblk, nsplit;            // nsplit: key-block ranges per row tile
  float scale_log2;
};

struct PoolParams {
  const void* k; float* k_pooled;
  int BH, nkeys, D, key_block, nblk, is_bf16;
};

struct MaskParams {
  const int32_t* sel_idx; uint32_t* blk_mask; int32_t* union_list; uint32_t* union_mask; int32_t* union_cnt;
  int B, Hq, Hkv, G, topk, nblk;
};

// Host-side launchers; each returns the hipError_t of its launch(es).
hipError_t launch_attn_f32(const PassParams& p, int D, PassMode mode, hipStream_t s);
hipError_t launch_attn_bf16(const PassParams& p, int D, PassMode mode, hipStream_t s);
// Streaming form of the bf16 pass (direct-to-LDS tile ring); covers a subset of (shape, mode) combinations.
bool stream_bf16_covers(const PassParams& p, int D, PassMode mode);
hipError_t launch_stream_bf16(const PassParams& p, int D, PassMode mode, hipStream_t s);
int stream_bf16_name(const PassParams& p, int D, PassMode mode, char* buf, size_t n);
// Name of the kernel launch_attn_bf16 runs for the dense external pass of p (profiler spelling, no namespace).
int attn_bf16_dense_name(const PassParams& p, int D, char* buf, size_t n);
hipError_t launch_combine(const CombineParams& p, hipStream_t s);
// Fold + block-internal attention + merge in one kernel; needs blk_q/k/v, Bq <= kMaxInlineBlock, Bq % kFoldRows == 0.
hipError_t launch_refresh_fold(const CombineParams& p, hipStream_t s);
constexpr int kMaxInlineBlock = 64;
constexpr int kFoldRows = 4;
hipError_t launch_pool_keys(const PoolParams& p, hipStream_t s);
hipError_t launch_select_topk(const SelectParams& p, hipStream_t s);
hipError_t launch_build_masks(const MaskParams& p, hipStream_t s);
hipError_t launch_block_mass_f32(const MassParams& p, int D, hipStream_t s);
hipError_t launch_block_mass_bf16(const MassParams& p, int D, hipStream_t s);
hipError_t launch_seq_order(const int32_t* prefix_lens, int32_t* seq_order, int B, hipStream_t s);
hipError_t launch_head_similarity(const float* o_a, const float* o_b, float* sim, int BH, int Bq, int D, hipStream_t s);

// Row tiles (workgroups along the group-flattened row axis) per KV group, per kernel family.
constexpr int kRowsPerWgBf16 = 128;  // 4 waves x 32 rows
constexpr int kRowsPerWgF32 = 4;     // 4 waves x 1 row
// bf16 dense external pass: KV groups of more than 128 rows run row-pair workgroups (8 wavefronts, 256 rows, one
// shared tile stream), so every K/V tile is staged once per 256 rows.  At head_dim 64 that measures the same as
// 128-row workgroups (32.6 vs 33.8 us at 256 rows, 32K keys) but leaves twice the splits to fold, so there only
// from 1024 rows on, where the pass is compute-bound.  Shared by the split heuristic and the launcher.
inline bool dense_row_pairs(int nrows, int head_dim) {
  return nrows >= 1024 || (head_dim >= 128 && nrows > kRowsPerWgBf16);
}

// ---- device helpers shared by the attention kernels -------------------------------------
// Tile schedule of one workgroup: which 64-key tiles it visits.
struct TileRange {
  int begin, end;   // entries [begin, end) of the pass's tile list
};

__device__ __forceinline__ TileRange split_range(int total, int nsplit, int split) {
  // balanced contiguous cut of `total` entries into nsplit pieces: the first total % nsplit
  // pieces get one entry more (one 32-bit division, no 64-bit arithmetic)
  const int base = total / nsplit, rem = total - base * nsplit;
  TileRange r;
  r.begin = split * base + min(split, rem);
  r.end = r.begin + base + (split < rem ? 1 : 0);
  return r;
}

// Cut of `total` tiles into an even number of pieces in which the even-numbered pieces are 1/64 longer and the
// odd-numbered ones 1/64 shorter than the mean (weights 65 : 63).  Used with a workgroup mapping that puts the
// odd-numbered splits on the odd-numbered XCDs: on the MI355X boards measured, the odd XCD of each pair streams
// about 4 % slower than the even one whichever KV head it reads (finish times of 128K passes per XCD, in-kernel
// clocks, with the head-to-XCD assignment rotated), and the pass ends with its slowest XCD.  A fixed, deterministic
// cut, deliberately a little weaker than the measured asymmetry: 128K pass 99.4 -> 97.4 us, batch 4 neutral; on a
// board without the asymmetry it would cost under 2 %.
__device__ __forceinline__ TileRange biased_range(int total, int nsplit, int split) {
  auto cum = [](int s) -> unsigned long long { return 64ull * (unsigned)s + (unsigned long long)(s & 1); };
  const unsigned long long den = 64ull * (unsigned)nsplit;
  TileRange r;
  r.begin = (int)(((unsigned long long)(unsigned)total * cum(split)) / den);
  r.end = (split + 1 == nsplit) ? total : (int)(((unsigned long long)(unsigned)total * cum(split + 1)) / den);
  return r;
}

// The same cut with the division by nsplit done through its precomputed magic number.
__device__ __forceinline__ TileRange split_range(int total, const FastDiv& by_nsplit, int split) {
  const int base = (int)fastdiv((uint32_t)total, by_nsplit), rem = total - base * (int)by_nsplit.d;
  TileRange r;
  r.begin = split * base + min(split, rem);
  r.end = r.begin + base + (split < rem ? 1 : 0);
  return r;
}

}  // namespace fb
