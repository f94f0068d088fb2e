// bf16 attention pass for gfx950 (MI355X): MFMA 32x32x16 tiles, fp32 statistics.
//
// Computes the per-row statistics of Eq. 3-4/6 (arxiv 2602.05305, Section 4.2) of a block of
// query rows against a stream of keys, and either stores split partials (external passes) or
// finishes with the log-space composition of Eq. 8-9 against a cached partial (internal pass).
//
// Work decomposition
//   workgroup = 4 wavefronts = 128 group-flattened query rows of one KV head (with 4 query
//   heads per KV head and a 32-row block that is exactly the whole KV group, so every K/V
//   byte is fetched once per pass); wavefront w owns rows [32w, 32w+32).
//   grid = batch * Hkv * row_tiles * nsplit workgroups, remapped so that workgroups that share
//   K/V (row tiles of one KV head) land on the same XCD / L2.
//   Variants of the one kernel template <D, MODE, KT, WS, NG, VAR> (picked on the host, launch_d):
//   NG = 2: 8 wavefronts, two groups stream interleaved tiles and merge through LDS (or, in the
//   sparse refresh pass, own one accumulator set each); WS = 2/4: wavefronts share 32 rows and
//   split the output columns (few rows per KV group); KT = 32: internal pass over <= 32 keys;
//   VAR = 1: row pair (the two groups own different rows, 256 per workgroup, one shared tile
//   stream: compute-bound passes with many rows); VAR = 2: tiles fetched two ahead (long streams);
//   VAR = 3: both.
//   MODE: dense external, internal + merge epilogue, sparse refresh, sparse reuse, per-head
//   refresh, paged external, fused refresh step (PassMode in fb_kernels.h).
// Per 64-key tile
//   K tile  -> LDS row-major [key][D] (row stride D*2+16 bytes: conflict-free ds_read_b128)
//   V tile  -> LDS transposed [d][key slot] (stride 64*2+16 bytes); the transpose happens in
//              registers on the way from global memory, keys are stored in the slot order in
//              which the score MFMA leaves them in registers.
//   S^T = K Q^T  : A = K rows from LDS, B = Q^T held in registers for the whole pass.
//                  Each lane ends up with 32 scores of ONE query row (row = lane%32), so the
//                  row max / row sum are in-lane reductions plus one exchange with lane^32.
//   O^T += V^T P^T: A = V^T from LDS, B = P^T = the lane's own exp2'd scores packed to bf16.
//   Tiles are double-buffered: global loads of tile t+1 are in flight (in registers) while
//   tile t is computed from LDS; one barrier per tile.
// Precision: bf16 operands, fp32 MFMA accumulation, fp32 max / sum / rescale, probabilities
// rounded to bf16 for the PV product; scores live in the log2 domain (scale*log2(e) folded).
#include <stdio.h>

#include "fb_kernels.h"

namespace fb {
namespace {

struct SteadyYes { static constexpr bool value = true; };
struct SteadyNo { static constexpr bool value = false; };

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int D, int KT_>
struct Cfg {
  static constexpr int KT = KT_;                    // keys per tile: 64, or 32 for the short internal pass
  static constexpr int KSTR = D * 2 + 16;           // bytes per K row in LDS
  static constexpr int VSTR = KT * 2 + 16;          // bytes per V^T row in LDS
  static constexpr int KBYTES = KT * KSTR;
  static constexpr int VBYTES = D * VSTR;
  static constexpr int STAGE = KBYTES + VBYTES;
  static constexpr int LDS = 2 * STAGE;
  static constexpr int NK = (KT * (D / 8) + 255) / 256;   // 16-byte K chunks per thread per tile
  static constexpr int KCHUNKS = KT * (D / 8);
  static constexpr int VUNITS = (KT / 4) * (D / 8); // (4 keys x 8 d) transpose units per tile
  static constexpr int NKS = D / 16;                // MFMA k-steps of the score product
  static constexpr int NDB = D / 32;                // 32-wide output column blocks
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef const __attribute__((address_space(1))) u32x4* gptr128;   // global address space: global_load_dwordx4

struct TileRegs {
  u32x4 k[4];
  u32x4 v[4];
};

__device__ __forceinline__ u32x4 gload128(const __bf16* p) { return *(gptr128)(p); }

// Global -> registers for one 64-key tile.  Keys past the end of the key range are clamped to
// the last key: the loads stay in bounds and branch-free, the duplicated rows are finite, and
// their scores are masked to -inf before the softmax so they never contribute.
template <int D, int KT>
__device__ __forceinline__ void load_k(u32x4 (&r)[4], const __bf16* __restrict__ K, int k0, int nkeys, int tid) {
  using C = Cfg<D, KT>;
  const int last = nkeys - 1;
#pragma unroll
  for (int i = 0; i < C::NK; ++i) {
    const int c = tid + 256 * i;
    const int row = c / (D / 8), col = c % (D / 8);
    const int key = min(k0 + row, last);
    if (C::KCHUNKS % 256 == 0 || c < C::KCHUNKS) r[i] = gload128(K + (size_t)key * D + col * 8);
    else r[i] = u32x4{0u, 0u, 0u, 0u};
  }
  // every element defined on every path: a partly written array is kept in scratch memory by the compiler, and
  // the store to it waits for the tile load right after issuing it
#pragma unroll
  for (int i = C::NK; i < 4; ++i) r[i] = u32x4{0u, 0u, 0u, 0u};
}

template <int D, int KT>
__device__ __forceinline__ void load_v(u32x4 (&r)[4], const __bf16* __restrict__ V, int k0, int nkeys, int tid) {
  using C = Cfg<D, KT>;
  const int last = nkeys - 1;
  if (C::VUNITS >= 256 || tid < C::VUNITS) {
    const int kq = tid % (C::KT / 4), doct = tid / (C::KT / 4);   // see store_v: lanes vary the key quad
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int key = min(k0 + 4 * kq + j, last);
      r[j] = gload128(V + (size_t)key * D + doct * 8);
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = u32x4{0u, 0u, 0u, 0u};
  }
}

template <int D, int KT>
__device__ __forceinline__ void store_k(const u32x4 (&r)[4], unsigned char* __restrict__ stage, int tid) {
  using C = Cfg<D, KT>;
#pragma unroll
  for (int i = 0; i < C::NK; ++i) {
    const int c = tid + 256 * i;
    const int row = c / (D / 8), col = c % (D / 8);
    if (C::KCHUNKS % 256 == 0 || c < C::KCHUNKS) *(u32x4*)(stage + row * C::KSTR + col * 16) = r[i];
  }
}

template <int D, int KT>
__device__ __forceinline__ void store_v(const u32x4 (&r)[4], unsigned char* __restrict__ stage, int tid) {
  using C = Cfg<D, KT>;
  unsigned char* Vt = stage + C::KBYTES;
  if (C::VUNITS >= 256 || tid < C::VUNITS) {
    const int kq = tid % (C::KT / 4), doct = tid / (C::KT / 4);
    // Lane -> unit mapping: the 16 key quads vary fastest across lanes.  One ds_write_b64 of a
    // wavefront then covers 16 x 8 contiguous bytes of two adjacent V^T rows per 32 lanes, which
    // is bank-conflict-free; with the d-octet varying fastest, lanes would hit rows 8 apart
    // (8 * VSTR = 32 dwords mod 64 banks: an 8-way conflict, measured 10x slower).
    // key quad kq of a 16-key group goes to slot quad {0,2,1,3}[kq%4]: the order in which the
    // 32x32 score accumulators hand keys to the two lane halves.
    const int g4 = kq & 3;
    const int sq = ((g4 & 1) << 1) | (g4 >> 1);
    const int slot = 16 * (kq >> 2) + 4 * sq;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t a = r[0][w], b = r[1][w], c = r[2][w], d = r[3][w];
      u32x2 lo, hi;   // column 2w (low halves) and 2w+1 (high halves) of the 4 keys
      // one byte-permute each: {first.lo16, second.lo16} and {first.hi16, second.hi16}
      lo.x = __builtin_amdgcn_perm(b, a, 0x05040100u);
      lo.y = __builtin_amdgcn_perm(d, c, 0x05040100u);
      hi.x = __builtin_amdgcn_perm(b, a, 0x07060302u);
      hi.y = __builtin_amdgcn_perm(d, c, 0x07060302u);
      const int dcol = doct * 8 + 2 * w;
      *(u32x2*)(Vt + dcol * C::VSTR + slot * 2) = lo;
      *(u32x2*)(Vt + (dcol + 1) * C::VSTR + slot * 2) = hi;
    }
  }
}

// Whole tile by one 256-thread group, or (SPLIT) K by wavefront group 0 and V by group 1, each
// into the same four staging registers.
template <int D, int KT, bool SPLIT>
__device__ __forceinline__ void tile_load(TileRegs& t, const __bf16* __restrict__ K, const __bf16* __restrict__ V,
                                          int k0, int nkeys, int tid, int grp) {
  if constexpr (SPLIT) {
    if (grp == 0) load_k<D, KT>(t.k, K, k0, nkeys, tid);
    else load_v<D, KT>(t.k, V, k0, nkeys, tid);
  } else {
    load_k<D, KT>(t.k, K, k0, nkeys, tid);
    load_v<D, KT>(t.v, V, k0, nkeys, tid);
  }
}

template <int D, int KT, bool SPLIT>
__device__ __forceinline__ void tile_store(const TileRegs& t, unsigned char* __restrict__ stage, int tid, int grp) {
  if constexpr (SPLIT) {
    if (grp == 0) store_k<D, KT>(t.k, stage, tid);
    else store_v<D, KT>(t.k, stage, tid);
  } else {
    store_k<D, KT>(t.k, stage, tid);
    store_v<D, KT>(t.v, stage, tid);
  }
}

// Running softmax state of the 32 rows a wavefront owns (one row per lane pair l, l^32).
template <int NDB>
struct WaveState {
  float m, l;          // log2-domain running reference; per-lane partial row sum
  f32x16 o[NDB];       // O^T: lane (row = lane%32, h = lane/32) holds d = 32db + 8(r/4) + 4h + r%4
  __device__ __forceinline__ void init() {
    m = -INFINITY;
    l = 0.f;
#pragma unroll
    for (int i = 0; i < NDB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
  }
};

// One 64-key tile for one wavefront: scores, online softmax update, value accumulation.
//   lane_on : this lane's query row takes part in this tile for this accumulator set
//   nvalid  : keys of the tile that exist (ragged tail); 64 for full tiles
template <int D, int KT, int WS>
__device__ __forceinline__ void tile_compute(WaveState<Cfg<D, KT>::NDB / WS>& st, const bf16x8 (&qreg)[Cfg<D, KT>::NKS],
                                             const unsigned char* __restrict__ stage, float scale_log2,
                                             bool lane_on, int nvalid, int l32, int h, int db_base) {
  using C = Cfg<D, KT>;
  constexpr int NDBL = C::NDB / WS;   // output column blocks this wavefront owns
  const unsigned char* Ks = stage;
  const unsigned char* Vt = stage + C::KBYTES;
  // scheduling hint: interleave the LDS operand reads with the MFMAs of this region (measured +2 % at the
  // compute-bound video shape, neutral where the pass is HBM-bound)
  __builtin_amdgcn_iglp_opt(0);

  constexpr int NKB = KT / 32;
  f32x16 s[NKB];
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
  // LDS operands are fetched in batches (2 k-steps x NKB key blocks) ahead of the MFMAs that use
  // them, and the key blocks' independent accumulator chains alternate.
#pragma unroll
  for (int ks0 = 0; ks0 < C::NKS; ks0 += 2) {
    bf16x8 a[2][NKB];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
        a[u][kb] = *(const bf16x8*)(Ks + (kb * 32 + l32) * C::KSTR + ((ks0 + u) * 16 + 8 * h) * 2);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u][kb], qreg[ks0 + u], s[kb], 0, 0, 0);
  }
  // s[kb][r] is the raw dot product of query row l32 with key kb*32 + 8*(r/4) + 4*h + r%4
  if (nvalid < C::KT) {
    // the empty asm keeps this a real (wavefront-uniform) branch: left alone, the compiler turns the
    // test into 62 compare/select instructions executed on every tile
    asm volatile("" ::: "memory");
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = kb * 32 + 8 * (r / 4) + 4 * h + (r % 4);
        if (key >= nvalid) s[kb][r] = -INFINITY;
      }
  }
  float tmax = -INFINITY;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[kb][r]);
  tmax = lane_on ? tmax * scale_log2 : -INFINITY;
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
  // Lazy reference update: the running reference m only moves when the tile maximum exceeds it
  // by more than kLazy (log2 units).  Weights then stay below 2^kLazy, which fp32 sums and the
  // relative precision of bf16 weights absorb, and (o, l, m) remain exactly paired; in return
  // the 16*NDB accumulator registers are rescaled on a small fraction of the tiles only.
  constexpr float kLazy = 8.f;
  const float m_new = (tmax > st.m + kLazy) ? tmax : st.m;
  const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_use);
  float lsum = 0.f;
  bf16x8 pb[2 * NKB];
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      // raw v_exp_f32: exp2(-inf) = 0, results below 2^-126 flush to 0 (irrelevant for weights)
      float pf = __builtin_amdgcn_exp2f(fmaf(s[kb][r], scale_log2, -m_use));
      if (!lane_on) pf = 0.f;                        // rows that sit this tile out
      lsum += pf;
      pb[2 * kb + r / 8][r % 8] = (__bf16)pf;
    }
  st.l = st.l * alpha + lsum;
  st.m = m_new;
  if (__any(alpha != 1.f)) {
#pragma unroll
    for (int db = 0; db < NDBL; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
  }
#pragma unroll
  for (int t0 = 0; t0 < 2 * NKB; t0 += 2) {
    bf16x8 a[2][NDBL];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int db = 0; db < NDBL; ++db)
        a[u][db] = *(const bf16x8*)(Vt + ((db_base + db) * 32 + l32) * C::VSTR + ((t0 + u) * 16 + 8 * h) * 2);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int db = 0; db < NDBL; ++db)
        st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u][db], pb[t0 + u], st.o[db], 0, 0, 0);
  }
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, v);
}

// NG = wavefront groups per workgroup (1 or 2).  With NG = 2 a workgroup is 8 wavefronts: both
// groups own the same 128 rows, stream alternate tiles of the workgroup's key range through their
// own pair of LDS stages, and group 1 hands its statistics to group 0 through LDS at the end.
// Same wavefronts per CU as two 4-wave workgroups, half as many split partials to write and fold.
template <int D, int MODE, int KT, int WS, int NG, int VAR = 0>
__global__ __launch_bounds__(256 * NG, (NG > 1 || (MODE == kPassInternal && WS > 1) || MODE == kPassSparseRefresh) ? 1 : 2) void attn_bf16_kernel(const PassParams p) {
  using C = Cfg<D, KT>;
  extern __shared__ __align__(16) unsigned char smem_all[];
  // Sparse refresh with NG = 2: the two wavefront groups are specialised by accumulator set
  // instead (group 0 = selected keys, group 1 = residual keys).  Both see every tile in shared
  // LDS stages (group 0 loads K, group 1 loads V), each wavefront computes a tile only if its
  // head routes it to its set, and every wavefront keeps ONE set: two wavefronts per SIMD
  // instead of the one that two sets in a single wavefront allow.
  constexpr bool RP = (VAR & 1) != 0;
  constexpr bool kSetSplit = (MODE == kPassSparseRefresh && NG == 2);
  // RP ("row pair", compute-bound passes with many rows): the two wavefront groups own DIFFERENT rows (256 per
  // workgroup) and share one tile stream and its LDS stages, so a staged tile serves twice the rows.
  static_assert(!RP || (NG == 2 && WS == 1 && (MODE == kPassDense || MODE == kPassInternal || MODE == kPassRefreshFused)), "row-pair mode");
  constexpr bool kShare = kSetSplit || RP;        // one tile stream, loaded cooperatively by both groups
  constexpr int TG = kShare ? 1 : NG;             // wavefront groups that own separate tile streams
  static_assert(NG == 1 || MODE == kPassDense || MODE == kPassDenseHeads || MODE == kPassDensePaged || MODE == kPassRefreshFused ||
                    MODE == kPassSparseReuse || kSetSplit || MODE == kPassInternal,
                "unsupported group mode");

  // wavefront-uniform by construction; in the list-driven passes (paged, sparse reuse), telling the compiler
  // so turns the per-tile table lookups into scalar loads, which do not queue behind the tile's vector loads
  const int grp = (NG > 1) ? ((MODE == kPassDensePaged || MODE == kPassSparseReuse || MODE == kPassSparseRefresh || (VAR & 1) != 0)
                                  ? __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 8))
                                  : (int)(threadIdx.x >> 8))
                           : 0;
  const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  unsigned char* smem = smem_all + (kShare ? 0 : grp) * 2 * C::STAGE;

  // XCD-aware remap: hardware deals consecutive workgroup ids round-robin to the 8 XCDs; make
  // each XCD own a contiguous range of work items (row tiles of one KV head are adjacent).
  const int nwg = gridDim.x;
  const int nrows = p.G * p.Bq;
  uint32_t rest;
  int rt;
  if constexpr (MODE == kPassDensePaged) {
    // Ragged sequences: contiguous ranges per XCD would give the XCDs unequal work.  Deal the
    // (sequence, KV head, split) units round-robin instead; the row tiles of one unit, which share
    // its K/V, stay on one XCD.  The grid is rounded up to a multiple of 8 units.
    const uint32_t j = blockIdx.x >> 3, xcd = blockIdx.x & 7;
    const uint32_t jq = fastdiv(j, p.div_rowtiles);
    rt = (int)(j - jq * p.div_rowtiles.d);
    rest = jq * 8 + xcd;
    if (rest >= (uint32_t)(p.B * p.Hkv * p.nsplit)) return;   // workgroup-uniform
  } else {
    const int bid = blockIdx.x, q8 = nwg / 8, r8 = nwg % 8;
    const int xcd = bid % 8, j = bid / 8;
    int w = (xcd < r8 ? xcd * (q8 + 1) : r8 * (q8 + 1) + (xcd - r8) * q8) + j;
    if constexpr (MODE == kPassDenseHeads) {
      // Per-head refresh over many row tiles: whole heads drop out, so a head's row tiles are dealt
      // round-robin over the XCDs (each XCD's L2 then holds that head's K/V stream once) instead of
      // filling one XCD, which would leave the XCDs of unflagged heads idle.
      if (p.div_rowtiles.d > 1) w = bid;
    }
    rest = fastdiv((uint32_t)w, p.div_rowtiles);
    rt = w - (int)(rest * p.div_rowtiles.d);
  }
  const uint32_t unit = rest;   // (batch, KV head, split) index: the same for all row tiles that share K/V
  int split = 0;
  if constexpr (MODE != kPassInternal) {
    const uint32_t r2 = fastdiv(rest, p.div_nsplit);
    split = (int)(rest - r2 * p.div_nsplit.d);
    rest = r2;
  }
  int b = (int)fastdiv(rest, p.div_hkv);
  const int kvh = (int)(rest - (uint32_t)b * p.div_hkv.d);
  if constexpr (MODE == kPassDensePaged) {
    if (p.seq_order != nullptr) {
      b = p.seq_order[b];
    } else if (p.order_inline) {
      // Small batch: this workgroup finds the sequence with the b-th longest prefix itself (ties: lower
      // index first) instead of waiting for a separate ordering kernel: lengths to LDS, one rank per
      // thread, the thread whose sequence has rank b publishes it.  The LDS is not yet in use.
      int* lens_s = (int*)smem_all;
      __shared__ int chosen;
      const int nthr = 256 * NG;
      for (int i = threadIdx.x; i < p.B; i += nthr) lens_s[i] = p.prefix_lens[i];
      __syncthreads();
      for (int i = threadIdx.x; i < p.B; i += nthr) {
        const int li = lens_s[i];
        int rank = 0;
        for (int j = 0; j < p.B; ++j) {
          const int lj = lens_s[j];
          rank += (lj > li || (lj == li && j < i)) ? 1 : 0;
        }
        if (rank == b) chosen = i;
      }
      __syncthreads();
      b = chosen;
    }
  }
  const int bk = b * p.Hkv + kvh;
  int nkeys_pass = p.nkeys;
  if constexpr (MODE == kPassDensePaged) nkeys_pass = min(p.nkeys, max(0, p.prefix_lens[b]));   // this sequence's prefix

  // WS wavefronts share one 32-row group and split the output columns between them (each repeats
  // the cheap score / softmax work): used when the pass has too few rows to fill the GPU, where
  // the time is a single wavefront's instruction stream, not throughput.
  constexpr int ROWS = RP ? 2 * kRowsPerWgBf16 : kRowsPerWgBf16 / WS;
  constexpr int NDBL = C::NDB / WS;
  const int db_base = (wave % WS) * NDBL;
  const int row = rt * ROWS + (RP ? (int)(threadIdx.x >> 6) * 32 : (wave / WS) * 32) + l32;      // group-flattened row of this lane
  const bool row_ok = row < nrows;
  const size_t grow = (size_t)(b * p.Hq + kvh * p.G) * p.Bq + row;   // global row index
  const size_t grow_last = (size_t)(b * p.Hq + kvh * p.G) * p.Bq + (nrows - 1);
  bool head_active = true;
  if constexpr (MODE == kPassDenseHeads) {
    // per-head refresh: rows of heads whose flag is 0 sit every tile out; a workgroup none of
    // whose rows is active leaves before it touches K/V
    head_active = row_ok && p.head_on[b * p.Hq + kvh * p.G + row / p.Bq] != 0;
    if (!__syncthreads_or(head_active ? 1 : 0)) return;
  }

  // One pass over a key range with fresh statistics, from the first tile load to the result's store.
  // Every mode runs it once, except the fused refresh pass, where the workgroup of the last prefix
  // split runs it a second time over the block's own keys (partial set 1).
  constexpr bool kFused = (MODE == kPassRefreshFused);
  auto run_pass = [&](const bool own_block) __attribute__((always_inline)) {
    const int nkeys = own_block ? p.Bq : nkeys_pass;
    const __bf16* __restrict__ Q = (const __bf16*)p.q;
    // contiguous cache: this KV head's [nkeys, D] slab; paged cache: the pool (tiles add their page offset)
    const __bf16* __restrict__ K = (const __bf16*)p.k + ((MODE == kPassDensePaged) ? (size_t)0 : (size_t)bk * nkeys * D);
    const __bf16* __restrict__ V = (const __bf16*)p.v + ((MODE == kPassDensePaged) ? (size_t)0 : (size_t)bk * nkeys * D);
    if constexpr (kFused) {
      if (own_block) {
        K = (const __bf16*)p.k2 + (size_t)bk * nkeys * D;
        V = (const __bf16*)p.v2 + (size_t)bk * nkeys * D;
      }
    }

    // tile list of this workgroup
    int tpb = 1, total;
    if constexpr (MODE == kPassSparseReuse) {
      tpb = p.key_block / KT;
      total = p.union_cnt[bk] * tpb;
    } else {
      total = (nkeys + KT - 1) / KT;
    }
    TileRange tr = (MODE == kPassInternal) ? TileRange{0, total}     // never split: no run-time division in its short prologue
                                           : split_range(total, p.div_nsplit, split);
    if constexpr (kFused) {
      if (own_block) {
        tr = TileRange{0, total};
      } else {
        // the last split's workgroup also runs the block phase: it gets blk_cost tiles fewer
        tr = split_range(total + p.blk_cost, p.div_nsplit, split);
        tr.begin = min(tr.begin, total);
        tr.end = min(tr.end, total);
      }
    }
    const uint32_t* __restrict__ bmask = p.blk_mask ? p.blk_mask + (size_t)bk * p.nblk : nullptr;
    const int32_t* __restrict__ ulist = p.union_list ? p.union_list + (size_t)bk * p.nblk : nullptr;
    const uint32_t my_bit = 1u << ((row_ok ? row : 0) / p.Bq);

    auto entry_k0 = [&](int e, uint32_t& mask) -> int {
      if constexpr (MODE == kPassSparseReuse) {
        const int blk = ulist[e / tpb];
        mask = bmask[blk];
        return blk * p.key_block + KT * (e % tpb);
      } else if constexpr (MODE == kPassSparseRefresh) {
        mask = bmask[(e * KT) / p.key_block];
        return e * KT;
      } else if constexpr (MODE == kPassDensePaged) {
        // descriptor word = page id, clamped into the pool
        const uint32_t slot = fastdiv((uint32_t)(e * KT), p.div_page);
        mask = (uint32_t)min(max(p.block_table[(size_t)b * p.max_pages + slot], 0), p.num_pages - 1);
        return e * KT;
      } else {
        mask = 0xffffffffu;
        return e * KT;
      }
    };

    // The first tile's loads go out before anything else touches memory: the start of the kernel
    // is a chain of cold latencies (instruction fetch, TLB, HBM), so the longest one starts first.
    // Tiles are visited in a rotated order (start offset differs per workgroup): workgroups that
    // run in lockstep would otherwise all read the same offset of their 2^k-strided chunks, i.e.
    // the same HBM channels, at the same time.  Row tiles of one unit share the offset: they run side
    // by side on one XCD, and walking the same K/V tiles at the same time is what lets its L2 serve
    // all but the first of them.  The statistics do not depend on the tile order.
    const int ntiles = tr.end - tr.begin;
    const uint32_t rsrc = (p.div_rowtiles.d == 1) ? blockIdx.x : unit;
    const int rot = (MODE == kPassInternal || ntiles <= 0) ? 0      // the block's K/V are small and cache-resident
                                                            : (int)((rsrc * 13u + (rsrc >> 5) * 7u) % (unsigned)ntiles);
    auto tile_entry = [&](int i) -> int {   // i-th tile of this wavefront group
      int j = TG * i + (kShare ? 0 : grp) + rot;
      if (j >= ntiles) j -= ntiles;
      return tr.begin + j;
    };
    const int common = ntiles / TG;                 // tiles every group has
    const bool extra = !kShare && (ntiles % TG) > grp;   // this group has one more
    TileRegs regs;
    // Tile descriptors (first key, selection mask) are looked up two tiles ahead: in the list-driven
    // sparse reuse pass they come from dependent scalar loads, whose latency would otherwise sit
    // in front of every tile's global loads.
    const int mine = common + (extra ? 1 : 0);
    auto load_tile = [&](int k0, uint32_t aux) {
      if constexpr (MODE == kPassDensePaged) {
        // page `aux` holds keys [j * page_size, (j+1) * page_size) of this sequence; rebase so that key
        // index k0 + r addresses row (k0 % page_size) + r of this KV head's slab of the page
        const int in_page = k0 - (int)(fastdiv((uint32_t)k0, p.div_page) * p.div_page.d);
        const long long off = (((long long)aux * p.Hkv + kvh) * p.page_size + in_page - k0) * D;
        tile_load<D, KT, kShare>(regs, K + off, V + off, k0, nkeys, tid, grp);
      } else {
        tile_load<D, KT, kShare>(regs, K, V, k0, nkeys, tid, grp);
      }
    };
    uint32_t mask_cur = 0, mask_next = 0, mask_nn = 0;
    int k0_cur = 0, k0_next = 0, k0_nn = 0;
    if (mine > 0) {
      k0_cur = entry_k0(tile_entry(0), mask_cur);
      load_tile(k0_cur, mask_cur);
      if (mine > 1) k0_next = entry_k0(tile_entry(1), mask_next);
    }

    bf16x8 qreg[C::NKS];
#pragma unroll
    for (int ks = 0; ks < C::NKS; ++ks) {
      // rows past the end load the group's last row instead (branch-free, in bounds); whatever
      // they compute is never stored
      const u32x4 u = gload128(Q + (row_ok ? grow : grow_last) * D + ks * 16 + 8 * h);
      qreg[ks] = __builtin_bit_cast(bf16x8, u);
    }

    // Internal pass: the cached external partial is independent of everything computed here.  In
    // the small (column-split) pass, which is a chain of memory latencies, its loads are issued up
    // front and complete under the attention work; in the large pass, where registers decide how
    // many wavefronts fit a SIMD, they are issued only in front of the epilogue.
    constexpr int NEO = (MODE == kPassInternal) ? NDBL * 4 : 1;
    constexpr bool kExtEarly = (WS > 1);
    // eo is deliberately left unset when there is no cached partial (it is only read under has_ext):
    // a zero default would have to be merged with the loaded values at the end of the branch, which
    // makes the compiler wait for the loads right there, in front of the first tile.
    f32x4 eo[NEO];
    float ext_m_v = -INFINITY, ext_lse_v = -INFINITY;
    const bool has_ext = (MODE == kPassInternal) && (p.ext_o != nullptr);     // workgroup-uniform
    auto load_ext = [&]() {
      typedef const __attribute__((address_space(1))) f32x4* gptr_f4;
      typedef const __attribute__((address_space(1))) float* gptr_f;
      if (has_ext) {
        const size_t er = row_ok ? grow : grow_last;   // rows past the end read the group's last row; never stored
        ext_m_v = *((gptr_f)p.ext_m + er);
        ext_lse_v = *((gptr_f)p.ext_lse + er);
#pragma unroll
        for (int db = 0; db < NDBL; ++db)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4)
            eo[db * 4 + q4] = *(gptr_f4)(p.ext_o + er * D + 32 * (db_base + db) + 8 * q4 + 4 * h);
      }
    };
    if constexpr (MODE == kPassInternal && kExtEarly) { if (ntiles == 0) load_ext(); }
    WaveState<NDBL> sel;
    sel.init();
    WaveState<(MODE == kPassSparseRefresh && !kSetSplit) ? NDBL : 1> res;
    res.init();

    // Steady state per iteration: issue the global loads of tile i+1 (they stay in flight in
    // registers), compute tile i from LDS, park tile i+1 in the other LDS stage, one barrier.
    auto run_tile = [&](auto& st, const unsigned char* stage, bool on, int nvalid) {
      tile_compute<D, KT, WS>(st, qreg, stage, p.scale_log2, on, nvalid, l32, h, db_base);
    };
    auto compute = [&](const unsigned char* stage, int k0, uint32_t mask) {
      const int nvalid = min(C::KT, nkeys - k0);      // <= 0 only for a reuse-list tile past the end
      if constexpr (MODE == kPassSparseReuse) {
        if (nvalid <= 0) return;
      }
      if constexpr (kSetSplit) {
        const bool on = row_ok && (((mask & my_bit) != 0u) == (grp == 0));
        if (__any(on)) run_tile(sel, stage, on, nvalid);
      } else if constexpr (MODE == kPassSparseRefresh) {
        const bool on = row_ok && (mask & my_bit);
        if (__any(on)) run_tile(sel, stage, on, nvalid);
        const bool off = row_ok && !(mask & my_bit);
        if (__any(off)) run_tile(res, stage, off, nvalid);
      } else if constexpr (MODE == kPassSparseReuse) {
        const bool on = row_ok && (mask & my_bit);
        if (__any(on)) run_tile(sel, stage, on, nvalid);
      } else if constexpr (MODE == kPassDenseHeads) {
        if (__any(head_active)) run_tile(sel, stage, head_active, nvalid);
      } else {
        run_tile(sel, stage, true, nvalid);
      }
    };

    // Long streams: tiles are fetched TWO ahead (two register sets that alternate).  Dense split pass with two
    // wavefront groups: each group then keeps two 32 KB tiles in flight instead of one; with one, the bytes in
    // flight per CU are just what the HBM latency-bandwidth product asks for, with no slack.  Sparse refresh
    // pass: its two groups share ONE tile stream (each loads half of every tile), so one-ahead leaves a single
    // tile in flight per CU, half of that product.
    constexpr bool kDeep = (VAR & 2) != 0;
    static_assert(!kDeep || (NG == 2 && WS == 1 && (MODE == kPassDense || MODE == kPassSparseRefresh || (RP && MODE == kPassInternal))),
                  "deep-prefetch variant");
    if constexpr (kDeep) {
      if (ntiles > 0) {
        const int maxmine = common + ((ntiles % TG) != 0 ? 1 : 0);      // workgroup-uniform trip count
        auto k0_of = [&](int i) -> int { return tile_entry(i) * KT; };
        TileRegs regs_b;
        if (mine > 1) tile_load<D, KT, kShare>(regs_b, K, V, k0_of(1), nkeys, tid, grp);
        if (mine > 0) tile_store<D, KT, kShare>(regs, smem, tid, grp);
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < C::NKS; ++ks) asm volatile("" ::"v"(qreg[ks]));
        // mask_cur / mask_next hold the selection masks of tiles i and i+1 (all ones in the dense pass).
        // The steady-state steps are unconditional: a load under a condition would make the number of loads in
        // flight path-dependent, and the wait in front of the LDS store would then have to be for all of them,
        // the just-issued tile included.
        auto step = [&](int i, TileRegs& r_load, TileRegs& r_store, auto steady) __attribute__((always_inline)) {
          constexpr bool kSteady = decltype(steady)::value;
          if (kSteady || i + 2 < mine) {
            k0_nn = entry_k0(tile_entry(i + 2), mask_nn);
            tile_load<D, KT, kShare>(r_load, K, V, k0_nn, nkeys, tid, grp);
          }
          if (kSteady || i < mine) compute(smem + (i & 1) * C::STAGE, k0_of(i), mask_cur);
          if (kSteady || i + 1 < mine) tile_store<D, KT, kShare>(r_store, smem + ((i + 1) & 1) * C::STAGE, tid, grp);
          __syncthreads();
          mask_cur = mask_next;
          mask_next = mask_nn;
        };
        int i = 0;
        for (; kShare && i + 3 < common; i += 2) {          // every group has tiles i .. i+3 (shared stream only: in the dense pass the unguarded steps cost 97 spilled registers)
          step(i, regs, regs_b, SteadyYes{});
          step(i + 1, regs_b, regs, SteadyYes{});
        }
        for (; i < maxmine; i += 2) {
          step(i, regs, regs_b, SteadyNo{});
          if (i + 1 < maxmine) step(i + 1, regs_b, regs, SteadyNo{});
        }
      }
    } else
    if (ntiles > 0) {
      if (common > 0 || extra) tile_store<D, KT, kShare>(regs, smem, tid, grp);
      __syncthreads();
      // the query registers have arrived by now (their loads went out with the first tile's); saying so here
      // keeps waits for them out of the tile loop, where in-order load counters would turn them into waits
      // for the next tile's prefetch
#pragma unroll
      for (int ks = 0; ks < C::NKS; ++ks) asm volatile("" ::"v"(qreg[ks]));
      if constexpr (MODE == kPassInternal && kExtEarly) load_ext();   // in flight under the attention work
      for (int i = 0; i < common - 1; ++i) {       // steady state: one barrier per tile
        if (i + 2 < mine) k0_nn = entry_k0(tile_entry(i + 2), mask_nn);
        load_tile(k0_next, mask_next);
        compute(smem + (i & 1) * C::STAGE, k0_cur, mask_cur);
        tile_store<D, KT, kShare>(regs, smem + ((i + 1) & 1) * C::STAGE, tid, grp);
        __syncthreads();
        k0_cur = k0_next;
        mask_cur = mask_next;
        k0_next = k0_nn;
        mask_next = mask_nn;
      }
      if (common > 0) {
        const int i = common - 1;
        if (extra) load_tile(k0_next, mask_next);
        compute(smem + (i & 1) * C::STAGE, k0_cur, mask_cur);
        if (TG > 1 && (ntiles % TG) != 0) {         // some group has one more tile (workgroup-uniform)
          if (extra) tile_store<D, KT, kShare>(regs, smem + ((i + 1) & 1) * C::STAGE, tid, grp);
          __syncthreads();
          if (extra) compute(smem + ((i + 1) & 1) * C::STAGE, k0_next, mask_next);
        }
      } else if (extra) {
        compute(smem, k0_cur, mask_cur);
      }
    }
    if constexpr (TG > 1) {
      // hand group 1's statistics to group 0: [wave][register][lane] floats in the (now idle) LDS
      constexpr int REC = NDBL * 16 + 2;
      float* mbuf = (float*)smem_all + (size_t)wave * REC * 64 + lane;
      __syncthreads();
      if (grp == 1) {
#pragma unroll
        for (int db = 0; db < NDBL; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) mbuf[(db * 16 + r) * 64] = sel.o[db][r];
        mbuf[(NDBL * 16) * 64] = sel.m;
        mbuf[(NDBL * 16 + 1) * 64] = sel.l;
      }
      __syncthreads();
      if (grp == 1) return;
      const float m1 = mbuf[(NDBL * 16) * 64], l1 = mbuf[(NDBL * 16 + 1) * 64];
      const float M = fmaxf(sel.m, m1);
      const float Mu = (M == -INFINITY) ? 0.f : M;
      const float w0 = __builtin_amdgcn_exp2f(sel.m - Mu), w1 = __builtin_amdgcn_exp2f(m1 - Mu);
#pragma unroll
      for (int db = 0; db < NDBL; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) sel.o[db][r] = sel.o[db][r] * w0 + mbuf[(db * 16 + r) * 64] * w1;
      sel.l = sel.l * w0 + l1 * w1;
      sel.m = M;
    }
    // ---------------------------------------------------------------- epilogue
    const float l_sel = sel.l + __shfl_xor(sel.l, 32, 64);
    if constexpr (MODE == kPassInternal) {
      if constexpr (!kExtEarly) load_ext();
      if (!row_ok) return;
      // keep the use of the cached statistics down here: hoisted into the prologue, it would make the
      // first tile wait for the cached partial's loads
      asm volatile("" : "+v"(ext_m_v), "+v"(ext_lse_v));
      if constexpr (kExtEarly) {
#pragma unroll
        for (int i = 0; i < NEO; ++i) asm volatile("" : "+v"(eo[i]));
      }
      float me2 = -INFINITY, le = 0.f;
      if (ext_lse_v != -INFINITY) {
        me2 = ext_m_v * kLog2e;
        le = exp2f((ext_lse_v - ext_m_v) * kLog2e);
      }
      // Eq. 8-9 with the cached pair expressed through (o, m, lse): A_out e^{L_out-M} = o e^{m-M}
      const float M2 = fmaxf(me2, sel.m);
      const float Mu = (M2 == -INFINITY) ? 0.f : M2;
      const float we = exp2f(me2 - Mu), wi = exp2f(sel.m - Mu);
      const float den = le * we + l_sel * wi;
      const float inv = den > 0.f ? 1.f / den : 0.f;
      __bf16* out = (__bf16*)p.out + grow * D;
#pragma unroll
      for (int db = 0; db < NDBL; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d0 = 32 * (db_base + db) + 8 * q4 + 4 * h;
          const f32x4 e = has_ext ? eo[(MODE == kPassInternal) ? db * 4 + q4 : 0] : f32x4{0.f, 0.f, 0.f, 0.f};
          float r[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) r[i] = (sel.o[db][4 * q4 + i] * wi + e[i] * we) * inv;
          u32x2 pk;
          pk.x = pack_bf16x2(r[0], r[1]);
          pk.y = pack_bf16x2(r[2], r[3]);
          *(u32x2*)(out + d0) = pk;
        }
      if (p.lse_out != nullptr && h == 0 && db_base == 0) p.lse_out[grow] = den > 0.f ? (M2 + log2f(den)) * kLn2 : -INFINITY;
    } else {
      if constexpr (MODE == kPassDense || MODE == kPassDenseHeads || MODE == kPassDensePaged) {
        if (p.direct) {
          // single split: this is the final partial.  Same conversion as the split combine: m is
          // rounded when converted to natural-log units, o is rescaled to the reference consumers
          // recover from it.
          if (!(row_ok && head_active)) return;
          float m_nat = -INFINITY, L = -INFINITY, adj = 0.f;
          if (l_sel > 0.f) {
            m_nat = sel.m * kLn2;
            adj = exp2f(sel.m - m_nat * kLog2e);
            L = (sel.m + log2f(l_sel)) * kLn2;
          }
#pragma unroll
          for (int db = 0; db < NDBL; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const int d0 = 32 * (db_base + db) + 8 * q4 + 4 * h;
              f32x4 o4 = {sel.o[db][4 * q4] * adj, sel.o[db][4 * q4 + 1] * adj, sel.o[db][4 * q4 + 2] * adj,
                          sel.o[db][4 * q4 + 3] * adj};
              *(f32x4*)(p.ws_o + grow * D + d0) = o4;
            }
          if (h == 0 && db_base == 0) {
            p.ws_m[grow] = m_nat;
            p.ws_l[grow] = L;
          }
          return;
        }
      }
      const size_t rows_total = (size_t)p.B * p.Hq * p.Bq;
      const size_t wrow = (own_block ? (size_t)0 : (size_t)split * rows_total) + grow;
      const bool set1 = (kSetSplit && grp == 1) || own_block;
      float* __restrict__ w_o = set1 ? p.ws_o2 : p.ws_o;
      float* __restrict__ w_m = set1 ? p.ws_m2 : p.ws_m;
      float* __restrict__ w_l = set1 ? p.ws_l2 : p.ws_l;
      if (row_ok) {
#pragma unroll
        for (int db = 0; db < NDBL; ++db)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int d0 = 32 * (db_base + db) + 8 * q4 + 4 * h;
            f32x4 o4 = {sel.o[db][4 * q4], sel.o[db][4 * q4 + 1], sel.o[db][4 * q4 + 2], sel.o[db][4 * q4 + 3]};
            // streaming store: the partials are read next by another kernel, never again by this
            // one; written through, they do not pile up as dirty L2 lines to flush at kernel end
            __builtin_nontemporal_store(o4, (f32x4*)(w_o + wrow * D + d0));
          }
        if (h == 0 && db_base == 0) {
          w_m[wrow] = sel.m;
          w_l[wrow] = l_sel;
        }
      }
      if constexpr (MODE == kPassSparseRefresh && !kSetSplit) {
        const float l_res = res.l + __shfl_xor(res.l, 32, 64);
        if (row_ok) {
#pragma unroll
          for (int db = 0; db < NDBL; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const int d0 = 32 * (db_base + db) + 8 * q4 + 4 * h;
              f32x4 o4 = {res.o[db][4 * q4], res.o[db][4 * q4 + 1], res.o[db][4 * q4 + 2], res.o[db][4 * q4 + 3]};
              *(f32x4*)(p.ws_o2 + wrow * D + d0) = o4;
            }
          if (h == 0 && db_base == 0) {
            p.ws_m2[wrow] = res.m;
            p.ws_l2[wrow] = l_res;
          }
        }
      }
    }
  };
  run_pass(false);
  if constexpr (kFused) {
    if (split == p.nsplit - 1) {   // workgroup-uniform
      __syncthreads();             // group 0 has read group 1's statistics out of LDS
      run_pass(true);
    }
  }
}

// Attention mass per (query row, key block) at a step that has the log-normaliser of full attention
// over the prefix: p_ij = exp(s_ij - lse_i), summed over the keys of each block.  Reads K only.
// Workgroup = 128 group-flattened rows of one KV head x a range of key blocks; scores as in the
// attention pass (S^T = K Q^T on the MFMA units, K tiles double-buffered in LDS).
template <int D>
__global__ __launch_bounds__(256) void block_mass_bf16_kernel(const MassParams p) {
  using C = Cfg<D, kKeyTile>;
  __shared__ __align__(16) unsigned char stages[2 * C::KBYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, h = lane >> 5;
  const int rt = blockIdx.x, split = blockIdx.y, bk = blockIdx.z;
  const int b = bk / p.Hkv, kvh = bk % p.Hkv;
  const int nrows = p.G * p.Bq, nkeys = p.nkeys;
  const int row = rt * kRowsPerWgBf16 + wave * 32 + l32;
  const bool row_ok = row < nrows;
  const size_t hrow = (size_t)kvh * nrows + (row_ok ? row : nrows - 1);   // head * Bq + i within the batch element
  const size_t grow = (size_t)b * p.Hq * p.Bq + hrow;
  const __bf16* __restrict__ Q = (const __bf16*)p.q;
  const __bf16* __restrict__ K = (const __bf16*)p.k + (size_t)bk * nkeys * D;

  const int tpb = p.key_block / kKeyTile;
  const TileRange br = split_range(p.nblk, p.nsplit, split);            // key blocks of this workgroup
  const int t0 = br.begin * tpb, t1 = min(br.end * tpb, (nkeys + kKeyTile - 1) / kKeyTile);
  if (t0 >= t1) return;                                                 // workgroup-uniform

  u32x4 kr[4];
  load_k<D, kKeyTile>(kr, K, t0 * kKeyTile, nkeys, tid);
  bf16x8 qreg[C::NKS];
#pragma unroll
  for (int ks = 0; ks < C::NKS; ++ks) qreg[ks] = __builtin_bit_cast(bf16x8, gload128(Q + grow * D + ks * 16 + 8 * h));
  const float lse = p.lse[grow];
  const bool live = lse != -INFINITY;
  const float lse2 = live ? lse * kLog2e : 0.f;
  store_k<D, kKeyTile>(kr, stages, tid);
  __syncthreads();
  // Touch the query registers here: otherwise the waits for their loads end up inside the loop, where
  // (load counters being in order) they would also wait for the next tile's prefetch on every trip.
#pragma unroll
  for (int ks = 0; ks < C::NKS; ++ks) asm volatile("" ::"v"(qreg[ks]));

  float acc = 0.f;
  for (int t = t0; t < t1; ++t) {
    const int cur = (t - t0) & 1;
    const bool more = t + 1 < t1;                                       // workgroup-uniform
    if (more) load_k<D, kKeyTile>(kr, K, (t + 1) * kKeyTile, nkeys, tid);
    const unsigned char* Ks = stages + cur * C::KBYTES;
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::NKS; ++ks)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8 a = *(const bf16x8*)(Ks + (kb * 32 + l32) * C::KSTR + (ks * 16 + 8 * h) * 2);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], s[kb], 0, 0, 0);
      }
    const int nvalid = min(kKeyTile, nkeys - t * kKeyTile);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = kb * 32 + 8 * (r / 4) + 4 * h + (r % 4);          // key of this accumulator register
        const float pf = __builtin_amdgcn_exp2f(fmaf(s[kb][r], p.scale_log2, -lse2));
        acc += (key < nvalid) ? pf : 0.f;
      }
    if (more) store_k<D, kKeyTile>(kr, stages + (cur ^ 1) * C::KBYTES, tid);
    __syncthreads();
    if ((t + 1) % tpb == 0 || !more) {                                  // the key block is complete
      const float tot = acc + __shfl_xor(acc, 32, 64);
      if (h == 0 && row_ok)
        p.rowmass[((size_t)b * p.nblk + t / tpb) * ((size_t)p.Hq * p.Bq) + hrow] = live ? tot : 0.f;
      acc = 0.f;
    }
  }
}

template <int D, int MODE, int KT, int WS, int NG, int VAR = 0>
hipError_t launch_one(const PassParams& p, hipStream_t s) {
  static LdsLimit lim;
  constexpr bool RP = (VAR & 1) != 0;
  auto kern = attn_bf16_kernel<D, MODE, KT, WS, NG, VAR>;
  constexpr int lds = Cfg<D, KT>::LDS * ((MODE == kPassSparseRefresh || RP) ? 1 : NG);
  {
    hipError_t e = raise_lds_limit(kern, lds, lim, lds);
    if (e != hipSuccess) return e;
  }
  constexpr int rows_per_wg = RP ? 2 * kRowsPerWgBf16 : kRowsPerWgBf16 / WS;
  const int nrows = p.G * p.Bq;
  const int ntile_rows = (nrows + rows_per_wg - 1) / rows_per_wg;
  long long nwg = (long long)p.B * p.Hkv * ntile_rows * p.nsplit;
  if (MODE == kPassDensePaged) nwg = (((long long)p.B * p.Hkv * p.nsplit + 7) / 8) * 8 * ntile_rows;
  if (nwg >= (1ll << 31)) return hipErrorInvalidValue;
  PassParams q = p;
  if (MODE == kPassDensePaged) q.div_page = make_fastdiv((uint32_t)p.page_size);
  q.div_rowtiles = make_fastdiv((uint32_t)ntile_rows);
  q.div_nsplit = make_fastdiv((uint32_t)p.nsplit);
  q.div_hkv = make_fastdiv((uint32_t)p.Hkv);
  launch_attn_kernel(kern, dim3((unsigned)nwg), dim3(256 * NG), lds, s, q);
  return hipGetLastError();
}

// Internal and fused passes (never or rarely split): row-pair workgroups when the pass is compute-bound, i.e. many
// rows per KV head and enough 256-row workgroups to give every CU one.  (The dense external pass uses them for
// every KV group above 128 rows, see dense_row_pairs.)
inline bool use_row_pairs(const PassParams& p) {
  const int nrows = p.G * p.Bq;
  const long long wgs = (long long)p.B * p.Hkv * ((nrows + 2 * kRowsPerWgBf16 - 1) / (2 * kRowsPerWgBf16)) * p.nsplit;
  return nrows >= 1024 && wgs >= 128;
}

// Template arguments <column split, wavefront groups, variant> of the dense external pass for a shape: the one
// place that decides them, for the launcher and for the name the benchmark reports.
struct DenseVariant {
  int ws, ng, var;
};

template <int D>
DenseVariant dense_variant(const PassParams& p) {
  constexpr int WSMAX = (D / 32 >= 4) ? 4 : 2;
  // 8-wave workgroups for split-KV streaming when every wavefront group gets >= 4 tiles; the
  // split heuristic (fb_api) then asks for one such workgroup per CU.
  // Small blocks (the paper's 4- and 8-token blocks: G*Bq <= 32 or 64 rows per KV group) would
  // leave three of the four row groups of a workgroup computing padding rows; there the
  // wavefronts share one or two 32-row groups and split the output columns instead.
  // (row pair + two tiles ahead, VAR = 3, measured: 0.6 % faster with 9 spilled registers; not used)
  if (dense_row_pairs(p.G * p.Bq, D)) return {1, 2, 1};
  const int tiles = (p.nkeys + kKeyTile - 1) / kKeyTile;
  const bool groups2 = p.nsplit > 1 && tiles >= 8 * p.nsplit;
  const int nrows = p.G * p.Bq;
  if (nrows <= 32) return {WSMAX, groups2 ? 2 : 1, 0};
  if (nrows <= 64) return {2, groups2 ? 2 : 1, 0};
  // long streams (>= 48 tiles per workgroup): tiles fetched two ahead; measured 4-6 % faster at 64 tiles
  // per workgroup (128K prefix), neutral at 32, and 1 us slower at 16 (32K prefix: longer start-up)
  if (groups2) return {1, 2, tiles >= 48 * p.nsplit ? 2 : 0};
  return {1, 1, 0};
}

template <int D>
hipError_t launch_d(const PassParams& p, PassMode mode, hipStream_t s) {
  constexpr int WSMAX = (D / 32 >= 4) ? 4 : 2;
  switch (mode) {
    case kPassDense: {
      const DenseVariant v = dense_variant<D>(p);
      if (v.var == 1) return launch_one<D, kPassDense, kKeyTile, 1, 2, 1>(p, s);
      if (v.ws == WSMAX && WSMAX > 2) {
        if (v.ng == 2) return launch_one<D, kPassDense, kKeyTile, WSMAX, 2>(p, s);
        return launch_one<D, kPassDense, kKeyTile, WSMAX, 1>(p, s);
      }
      if (v.ws == 2) {
        if (v.ng == 2) return launch_one<D, kPassDense, kKeyTile, 2, 2>(p, s);
        return launch_one<D, kPassDense, kKeyTile, 2, 1>(p, s);
      }
      if (v.ng == 2) {
        if (v.var == 2) return launch_one<D, kPassDense, kKeyTile, 1, 2, 2>(p, s);
        return launch_one<D, kPassDense, kKeyTile, 1, 2>(p, s);
      }
      return launch_one<D, kPassDense, kKeyTile, 1, 1>(p, s);
    }
    case kPassInternal: {
      // Few rows (an LLM-sized block): the pass is one wavefront's run-once instruction stream.
      // Spread each 32-row group over WSMAX wavefronts (columns split) and, for a block of at
      // most 32 keys, use the 32-key tile: both shorten that stream.
      if (use_row_pairs(p)) return launch_one<D, kPassInternal, kKeyTile, 1, 2, 1>(p, s);
      const long long wgs = (long long)p.B * p.Hkv * ((p.G * p.Bq + kRowsPerWgBf16 - 1) / kRowsPerWgBf16);
      if (wgs < 128) {
        if (p.nkeys <= 32) return launch_one<D, kPassInternal, 32, WSMAX, 1>(p, s);
        return launch_one<D, kPassInternal, kKeyTile, WSMAX, 1>(p, s);
      }
      return launch_one<D, kPassInternal, kKeyTile, 1, 1>(p, s);
    }
    case kPassSparseRefresh: {
      // 8 wavefronts, the two groups specialised by accumulator set (see the kernel); tiles two ahead unless
      // the workgroups' streams are short
      const int tiles = (p.nkeys + kKeyTile - 1) / kKeyTile;
      if (tiles >= 8 * p.nsplit) return launch_one<D, kPassSparseRefresh, kKeyTile, 1, 2, 2>(p, s);
      return launch_one<D, kPassSparseRefresh, kKeyTile, 1, 2>(p, s);
    }
    case kPassDenseHeads: {
      const int tiles = (p.nkeys + kKeyTile - 1) / kKeyTile;
      // 8-wavefront workgroups also without splits: workgroups of unflagged heads leave at once, and the
      // remaining ones should each be able to use a whole CU
      if (tiles >= 8 * p.nsplit) return launch_one<D, kPassDenseHeads, kKeyTile, 1, 2>(p, s);
      return launch_one<D, kPassDenseHeads, kKeyTile, 1, 1>(p, s);
    }
    case kPassRefreshFused: {
      const int tiles = (p.nkeys + kKeyTile - 1) / kKeyTile;
      if (p.nsplit == 1 && use_row_pairs(p)) return launch_one<D, kPassRefreshFused, kKeyTile, 1, 2, 1>(p, s);   // many rows, unsplit
      if (p.nsplit > 1 && tiles >= 8 * p.nsplit) return launch_one<D, kPassRefreshFused, kKeyTile, 1, 2>(p, s);
      return launch_one<D, kPassRefreshFused, kKeyTile, 1, 1>(p, s);   // unsplit (many row tiles): as the dense pass
    }
    case kPassDensePaged: {
      const int tiles = (p.nkeys + kKeyTile - 1) / kKeyTile;
      // two wavefront groups also without splits: the longest sequence's workgroup sets the pass time
      if (tiles >= 16 * p.nsplit) return launch_one<D, kPassDensePaged, kKeyTile, 1, 2>(p, s);
      return launch_one<D, kPassDensePaged, kKeyTile, 1, 1>(p, s);
    }
    case kPassSparseReuse:
      if (p.nsplit > 1) return launch_one<D, kPassSparseReuse, kKeyTile, 1, 2>(p, s);
      return launch_one<D, kPassSparseReuse, kKeyTile, 1, 1>(p, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_block_mass_bf16(const MassParams& p, int D, hipStream_t s) {
  const int rowtiles = (p.G * p.Bq + kRowsPerWgBf16 - 1) / kRowsPerWgBf16;
  const dim3 grid(rowtiles, p.nsplit, p.B * p.Hkv);
  if (D == 64) hipLaunchKernelGGL(block_mass_bf16_kernel<64>, grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL(block_mass_bf16_kernel<128>, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

int attn_bf16_dense_name(const PassParams& p, int D, char* buf, size_t n) {
  if (stream_bf16_covers(p, D, kPassDense)) return stream_bf16_name(p, D, kPassDense, buf, n);
  const DenseVariant v = D == 64 ? dense_variant<64>(p) : dense_variant<128>(p);
  return snprintf(buf, n, "attn_bf16_kernel<%d, %d, %d, %d, %d, %d>", D, (int)kPassDense, kKeyTile, v.ws, v.ng, v.var);
}

hipError_t launch_attn_bf16(const PassParams& p, int D, PassMode mode, hipStream_t s) {
  if (stream_bf16_covers(p, D, mode)) return launch_stream_bf16(p, D, mode, s);
  if (D == 64) return launch_d<64>(p, mode, s);
  return launch_d<128>(p, mode, s);
}

}  // namespace fb
