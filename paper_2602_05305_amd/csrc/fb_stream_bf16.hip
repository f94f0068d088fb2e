// bf16 streaming attention pass for gfx950 (MI355X): K/V tiles travel from global memory straight into a ring
// of LDS stages (direct-to-LDS 16-byte loads, no register staging), K operands are read back with
// ds_read_b128 from a rotation-swizzled row-major layout, V operands with the transposing LDS read
// (ds_read_b64_tr_b16) from row-major V, so nothing is transposed or re-stored on the way.
//
// Computes the per-row statistics of Eq. 3-4/6 (arxiv 2602.05305, Section 4.2) of a block of query rows
// against a stream of keys and either stores split partials / the final partial (external passes) or finishes
// with the log-space composition of Eq. 8-9 against a cached partial (internal pass).
//
// Work decomposition: one workgroup streams one list of 64-key tiles through NS ring stages.
//   kKeySplit  NRG = 4, 2 or 1 groups of 32 group-flattened rows (8, 4 or 2 wavefronts); wavefront w owns row group
//              w % NRG and the key half w / NRG of every tile; the two halves exchange accumulator halves through LDS
//              after the last tile and each finishes and stores half of the output columns.  (LLM-shaped blocks:
//              the whole KV group is one workgroup, every K/V byte is fetched once; NRG = 2 / 1 for KV groups of
//              at most 64 / 32 rows, the 4- and 8-token blocks, where more row groups would compute padding.)
//              Sparse refresh pass: the same layout with two accumulator sets per wavefront (selected /
//              residual key blocks); a tile's scores are computed once and go to the set the row's head routes
//              the tile's key block to, so the eight wavefronts stay evenly loaded whatever the selection.
//   kRowPair   256 rows, wavefront w owns rows [32 w, +32) and whole tiles (many rows per KV head: a staged
//              tile serves twice the rows).  Two tiles per barrier: inside an iteration the two wavefronts of a SIMD
//              are free to drift apart by a tile, so that one's softmax can run under the other's MFMAs.
//   Per tile and wavefront: S^T = K Q^T on v_mfma_f32_32x32x16_bf16 (A = K rows from LDS, B = Q^T in
//   registers), in-lane online softmax with a lazily moved reference, O^T += V^T P^T with the lane's own
//   probabilities as the B operand (register layout reasoning: fb_attn_bf16.hip, which is the same).
// LDS layout of a stage: [K: 64 rows x D*2 bytes][V: 64 rows x D*2 bytes], rows unpadded, the 16-byte chunks
//   of a row rotated by a row-dependent amount (K: by row, V: by 4*row at head_dim 128; by row/2 and
//   4*(row/2) at head_dim 64) so that both read patterns are bank-conflict-free.  A direct-to-LDS load puts
//   the 64 lanes' chunks at consecutive LDS addresses, so the rotation is applied on the global-address side.
// Synchronisation: the direct-to-LDS loads are issued from inline assembly, invisible to the compiler's
//   wait-count insertion (which would otherwise drain every outstanding load before any LDS read); each
//   wavefront waits for its own loads of a tile with an explicit s_waitcnt vmcnt(n), then the workgroup
//   barrier makes the tile visible to all.  The stage refilled after barrier t is the one last read in
//   iteration t-1, which every wavefront has left by then.
#include <stdio.h>

#include "fb_kernels.h"

namespace fb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

enum StreamLayout : int { kKeySplit = 0, kRowPair = 2 };

// NRG: 32-row groups of a key-split workgroup (4: 128 rows, 8 wavefronts; 2: 64 rows, 4 wavefronts; 1: 32 rows, 2
// wavefronts: the small blocks of 4- and 8-token diffusion steps, where more row groups would compute padding rows)
template <int D, int LAYOUT, int NSETS = 1, int NRG = 4>
struct SCfg {
  static constexpr int NW = (LAYOUT == kRowPair) ? 8 : 2 * NRG;   // wavefronts per workgroup
  static constexpr int THREADS = 64 * NW;
  static constexpr int KT = 64;                       // keys per tile
  static constexpr int ROWB = D * 2;                  // bytes per key row
  static constexpr int CPR = ROWB / 16;               // 16-byte chunks per row
  static constexpr int OPB = KT * ROWB;               // bytes per operand (K or V) per tile
  static constexpr int STAGE = 2 * OPB;
  static constexpr int NLOAD = OPB / (THREADS * 16);  // direct-to-LDS loads per lane, operand and tile
  static constexpr int LSTEP = NW * 1024;             // LDS bytes one load of every wavefront covers
  static constexpr int LPT = 2 * NLOAD;               // loads per lane and tile
  static constexpr int NS = (D == 128) ? 4 : 6;       // ring stages
  static constexpr int NKS = D / 16;                  // MFMA k-steps of the score product
  static constexpr int NDB = D / 32;                  // 32-wide output column blocks
  static constexpr int ROWS = (LAYOUT == kRowPair) ? 256 : 32 * NRG;
  static constexpr int NKB = (LAYOUT == kKeySplit) ? 1 : 2;    // 32-key blocks of a tile one wavefront computes
  static constexpr int QPARTS = (ROWS + 63) / 64;             // the query rows are loaded 64 at a time, like a K operand
  static constexpr int QSTAGES = (QPARTS * OPB + STAGE - 1) / STAGE;   // ring stages they pass through at start
  static constexpr int MERGE = (LAYOUT == kKeySplit) ? NSETS * NRG * 2 * (NDB / 2 * 16 + 2) * 64 * 4 : 0;   // key-half exchange
  static constexpr int RING = NS * STAGE;
  static constexpr int FIFO = RING > MERGE ? RING : MERGE;
  static constexpr int LDS = FIFO;
  static_assert(QSTAGES >= 1 && QSTAGES < NS && NLOAD >= 1, "ring geometry");
  static_assert((NS - 1) * LPT <= 63, "the loads of NS - 1 tiles in flight must fit the 6-bit load counter");
  // rotation (in chunks) of row `row`
  __device__ static __forceinline__ int rot_k(int row) { return D == 128 ? row : (row >> 1); }
  __device__ static __forceinline__ int rot_v(int row) { return D == 128 ? 4 * row : 4 * (row >> 1); }
};

// One 16-byte direct-to-LDS load per lane: lane l's chunk lands at LDS byte lds_base + 16 l.  Global address =
// base (wavefront-uniform) + off (per lane, unsigned 32-bit).
__device__ __forceinline__ void dma16(const void* base, uint32_t off, uint32_t lds_base) {
  // base and lds_base are wavefront-uniform by construction; readfirstlane says so to the compiler, which
  // otherwise may hand the "s" operands over in vector registers (not encodable here)
  // (the builtin returns int: each half goes through uint32_t so that nothing is sign-extended)
  const uint64_t b = (uint64_t)(uintptr_t)base;
  const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32));
  const uint64_t bu = ((uint64_t)b_hi << 32) | (uint64_t)b_lo;
  const uint32_t lu = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(off), "s"(bu), "s"(lu)
               : "memory", "m0");
}

// Wavefront-uniform table lookup as a scalar load (constant address space).  The tables were written by earlier
// kernels, so they are constant here; without this the compiler, which sees the inline assembly's memory
// clobber, falls back to vector loads, and its wait for them (vmcnt(0)) would also drain every direct-to-LDS
// load in flight.
__device__ __forceinline__ int32_t sload(const void* table, int idx) {
  typedef const __attribute__((address_space(4))) int32_t* cptr;
  return ((cptr)(uintptr_t)table)[__builtin_amdgcn_readfirstlane(idx)];
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// wait until at most `tiles` tiles' worth of this lane's direct-to-LDS loads are outstanding
// (the counter has 6 bits: counts above 63 cannot be asked for, and no ring here keeps that many loads in flight)
template <int LPT>
__device__ __forceinline__ void wait_tiles(int tiles) {
  constexpr int kMax = 63 / LPT;       // largest tile count the counter can express
  if (kMax >= 5 && tiles >= 5) wait_vm<(kMax >= 5 ? 5 : 0) * LPT>();
  else if (kMax >= 4 && tiles >= 4) wait_vm<(kMax >= 4 ? 4 : 0) * LPT>();
  else if (kMax >= 3 && tiles >= 3) wait_vm<(kMax >= 3 ? 3 : 0) * LPT>();
  else if (kMax >= 2 && tiles >= 2) wait_vm<(kMax >= 2 ? 2 : 0) * LPT>();
  else if (kMax >= 1 && tiles >= 1) wait_vm<(kMax >= 1 ? 1 : 0) * LPT>();
  else wait_vm<0>();
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, v);
}

// Running softmax state of the 32 rows a wavefront owns (one row per lane pair l, l^32).
template <int NDB>
struct WaveAcc {
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

// Scores of this wavefront's 32 rows against key blocks [kb0, kb0 + NKB) of the tile in `stage`.
// kaddr[ks] = per-lane byte address (within a stage, key block 0) of the K chunk of k-step ks.
template <int D, int NKB>
__device__ __forceinline__ void tile_scores(f32x16 (&s)[NKB], const bf16x8 (&qreg)[D / 16],
                                            const unsigned char* __restrict__ stage, const uint32_t (&kaddr)[D / 16],
                                            int kb0) {
  constexpr int NKS = D / 16, ROWB = D * 2;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
  for (int ks0 = 0; ks0 < NKS; ks0 += 2) {
    bf16x8 a[2][NKB];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
        a[u][kb] = *(const bf16x8*)(stage + kaddr[ks0 + u] + (kb0 + kb) * 32 * ROWB);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u][kb], qreg[ks0 + u], s[kb], 0, 0, 0);
  }
}

// Online softmax update with the tile's scores: moves the running reference if needed (rescaling the accumulators),
// adds the row sums, and leaves the tile's probabilities, rounded to bf16, in pb (B operands of the value product).
//   s[kb][r] = raw dot product of query row lane%32 with key 32 (kb0 + kb) + 8 (r/4) + 4 h + r%4
template <int D, int NKB>
__device__ __forceinline__ void tile_softmax(WaveAcc<D / 32>& st, f32x16 (&s)[NKB], bf16x8 (&pb)[2 * NKB], int kb0,
                                             float scale_log2, bool lane_on, int nvalid, int h) {
  constexpr int NDB = D / 32;
  if (nvalid < 64) {
    // the empty asm keeps this a real (wavefront-uniform) branch instead of per-score selects on every tile
    asm volatile("" ::: "memory");
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = (kb0 + kb) * 32 + 8 * (r / 4) + 4 * h + (r % 4);
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
  // Lazy reference: m moves only when the tile maximum exceeds it by more than kLazy (log2 units); weights
  // stay below 2^kLazy, (o, l, m) remain exactly paired, and the accumulators are rescaled on few tiles only.
  constexpr float kLazy = 8.f;
  const float m_new = (tmax > st.m + kLazy) ? tmax : st.m;
  const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_use);
  float lsum = 0.f;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float pf = __builtin_amdgcn_exp2f(fmaf(s[kb][r], scale_log2, -m_use));
      if (!lane_on) pf = 0.f;
      lsum += pf;
      pb[2 * kb + r / 8][r % 8] = (__bf16)pf;
    }
  st.l = st.l * alpha + lsum;
  st.m = m_new;
  if (__any(alpha != 1.f)) {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
  }
}

// Value accumulation O^T[db] += V^T P^T over 16-key steps: A operand element e of lane half h is key
// 16u + 8(e/4) + 4h + e%4 of the key block, i.e. two transposing reads of 4 consecutive keys each.
//   vaddr[db] = per-lane byte address (within a stage) of the lane's share of the transposing V read of column block
//               db, key offset 0 (the lane's own 4h + i/4 row offset is inside); the 4-key groups are reached
//               through immediate offsets
template <int D, int NKB>
__device__ __forceinline__ void tile_pv(WaveAcc<D / 32>& st, const bf16x8 (&pb)[2 * NKB],
                                        const unsigned char* __restrict__ stage, const uint32_t (&vaddr)[D / 32], int kb0) {
  constexpr int NDB = D / 32, ROWB = D * 2, OPB = 64 * ROWB;
#pragma unroll
  for (int t = 0; t < 2 * NKB; ++t) {
    const int krow = (kb0 + t / 2) * 32 + 16 * (t % 2);
    bf16x8 a[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db) {
      const unsigned char* base = stage + OPB + vaddr[db] + krow * ROWB;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base + 8 * ROWB));
      const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      a[db] = __builtin_bit_cast(bf16x8, both);
    }
#pragma unroll
    for (int db = 0; db < NDB; ++db)
      st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[db], pb[t], st.o[db], 0, 0, 0);
  }
}

template <int D, int NKB>
__device__ __forceinline__ void tile_softmax_pv(WaveAcc<D / 32>& st, f32x16 (&s)[NKB],
                                                const unsigned char* __restrict__ stage,
                                                const uint32_t (&vaddr)[D / 32], int kb0, float scale_log2,
                                                bool lane_on, int nvalid, int h) {
  bf16x8 pb[2 * NKB];
  tile_softmax<D, NKB>(st, s, pb, kb0, scale_log2, lane_on, nvalid, h);
  tile_pv<D, NKB>(st, pb, stage, vaddr, kb0);
}

// A tile of the stream (all wavefront-uniform).  TileRaw is what the table lookups deliver (fetched one iteration
// before the tile is issued, with no arithmetic on the loaded words, so that the wait for them falls into the
// next iteration); TileDesc adds the addresses.
struct TileRaw {
  int e;            // entry of the pass's tile list
  int word;         // sparse reuse: key block; paged: page id; else unused
  uint32_t mask;    // selection mask of the tile's key block (sparse passes), else all ones
};
struct TileDesc {
  int k0;
  uint32_t mask;
  const unsigned char* kt;
  const unsigned char* vt;
};

template <int D, int MODE, int LAYOUT, int NRG>
__global__ __launch_bounds__(((LAYOUT == kRowPair) ? 8 : 2 * NRG) * 64, 1) void attn_stream_kernel(const PassParams p) {
  constexpr int NSETS = (MODE == kPassSparseRefresh) ? 2 : 1;
  using C = SCfg<D, LAYOUT, NSETS, NRG>;
  static_assert(MODE == kPassDense || MODE == kPassDenseHeads || MODE == kPassDensePaged || MODE == kPassSparseReuse ||
                    MODE == kPassSparseRefresh || MODE == kPassInternal, "modes of the streaming kernel");
  static_assert(MODE != kPassSparseRefresh || LAYOUT == kKeySplit, "two accumulator sets: key-split layout");
  static_assert(MODE != kPassInternal || LAYOUT == kRowPair, "internal pass: row-pair layout");
  // Row-pair layout: two tiles per barrier (tiles t, t+1 are computed while t+2, t+3 are in flight), measured 2 % faster
  // at the video shape than one tile per barrier; every other layout: one tile per barrier, NS - 1 tiles in flight.
  constexpr bool kPairs = LAYOUT == kRowPair;
  constexpr int AHEAD = kPairs ? C::NS - 2 : C::NS - 1;
  static_assert(!kPairs || (C::NS == 4 || C::NS == 6), "pairs of tiles: an even number of stages");
  // passes whose tiles come from a table (paged, sparse): the lookups are made one iteration ahead of the tile's
  // issue, and (first key, mask) travel to the tile's compute in a register queue
  constexpr bool kListed = (MODE == kPassDensePaged || MODE == kPassSparseReuse || MODE == kPassSparseRefresh);
  extern __shared__ __align__(16) unsigned char ring[];
  const int lane = threadIdx.x & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));     // wavefront-uniform (scalar)
  const int rg = (LAYOUT == kRowPair) ? wave : (wave % NRG);     // 32-row group
  const int kb0 = (LAYOUT == kKeySplit) ? (wave / NRG) : 0;      // first 32-key block of every tile

  // ---- workgroup -> (row tile, batch, KV head, split).  Hardware deals consecutive workgroup ids round-robin
  // to the 8 XCDs; each XCD gets a contiguous range of units so that row tiles sharing K/V share an L2.
  const int nwg = gridDim.x;
  const int nrows = p.G * p.Bq;
  int rt;
  uint32_t rest;
  if constexpr (MODE == kPassDensePaged) {
    // ragged sequences: contiguous ranges would give the XCDs unequal work; deal the units round-robin
    const uint32_t j = blockIdx.x >> 3, xcd = blockIdx.x & 7;
    const uint32_t jq = fastdiv(j, p.div_rowtiles);
    rt = (int)(j - jq * p.div_rowtiles.d);
    rest = jq * 8 + xcd;
    if (rest >= (uint32_t)(p.B * p.Hkv * p.nsplit)) return;   // workgroup-uniform
  } else {
    const int bid = blockIdx.x, q8 = nwg / 8, r8 = nwg % 8;
    const int xcd = bid % 8, j = bid / 8;
    int w = (xcd < r8 ? xcd * (q8 + 1) : r8 * (q8 + 1) + (xcd - r8) * q8) + j;
    // biased cut (the host sets it only for one row tile, an even split count and a grid that is a multiple of 8):
    // the two XCDs of a pair take alternate work items of the pair's contiguous range, so that even-numbered splits
    // run on even XCDs and odd-numbered ones on odd XCDs
    if (p.xcd_bias) w = (xcd >> 1) * (2 * q8) + 2 * j + (xcd & 1);
    if constexpr (MODE == kPassDenseHeads) {
      if (p.div_rowtiles.d > 1) w = bid;     // whole heads drop out: deal a head's row tiles over the XCDs
    }
    rest = fastdiv((uint32_t)w, p.div_rowtiles);
    rt = w - (int)(rest * p.div_rowtiles.d);
  }
  const uint32_t unit = rest;
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
      b = sload(p.seq_order, b);
    } else if (p.order_inline) {
      // small batch: this workgroup finds the sequence with the b-th longest prefix itself (ties: lower index
      // first): lengths to LDS, one rank per thread, the thread whose sequence has rank b publishes it
      int* lens_s = (int*)ring;
      __shared__ int chosen;
      for (int i = threadIdx.x; i < p.B; i += C::THREADS) lens_s[i] = p.prefix_lens[i];
      __syncthreads();
      for (int i = threadIdx.x; i < p.B; i += C::THREADS) {
        const int li = lens_s[i];
        int rank = 0;
        for (int j = 0; j < p.B; ++j) {
          const int lj = lens_s[j];
          rank += (lj > li || (lj == li && j < i)) ? 1 : 0;
        }
        if (rank == b) chosen = i;
      }
      __syncthreads();
      b = __builtin_amdgcn_readfirstlane(chosen);
      __syncthreads();                       // the ring is free again before the first direct-to-LDS load
    }
  }
  const int bk = b * p.Hkv + kvh;
  int nkeys = p.nkeys;
  if constexpr (MODE == kPassDensePaged) nkeys = min(p.nkeys, max(0, sload(p.prefix_lens, b)));   // this sequence's prefix

  const int row0 = rt * C::ROWS;                               // first group-flattened row of the workgroup
  const int row = row0 + rg * 32 + l32;
  const bool row_ok = row < nrows;
  const size_t grow_base = (size_t)(b * p.Hq + kvh * p.G) * p.Bq;
  const size_t grow = grow_base + row;
  bool head_active = true;
  if constexpr (MODE == kPassDenseHeads) {
    head_active = row_ok && p.head_on[b * p.Hq + kvh * p.G + row / p.Bq] != 0;
    if (!__syncthreads_or(head_active ? 1 : 0)) return;
  }

  // contiguous cache: this KV head's [nkeys, D] slab; paged cache: the pool (tiles add their page offset)
  const unsigned char* __restrict__ Kg =
      (const unsigned char*)p.k + ((MODE == kPassDensePaged) ? (size_t)0 : (size_t)bk * nkeys * C::ROWB);
  const unsigned char* __restrict__ Vg =
      (const unsigned char*)p.v + ((MODE == kPassDensePaged) ? (size_t)0 : (size_t)bk * nkeys * C::ROWB);

  // ---- tile list of this workgroup: a contiguous range of the pass's tile list, visited in rotated order
  // (workgroups that run in lockstep would otherwise read the same offset of their chunks, i.e. the same
  // channels, at once; row tiles of one unit share the offset so that one L2 serves them)
  int tpb = 1, total;
  if constexpr (MODE == kPassSparseReuse) {
    tpb = p.key_block / C::KT;
    total = sload(p.union_cnt, bk) * tpb;
  } else {
    total = (nkeys + C::KT - 1) / C::KT;
  }
  const TileRange tr = (MODE == kPassInternal) ? TileRange{0, total}
                       : p.xcd_bias ? biased_range(total, p.nsplit, split) : split_range(total, p.div_nsplit, split);
  const int ntiles = tr.end - tr.begin;
  const uint32_t rsrc = (p.div_rowtiles.d == 1) ? blockIdx.x : unit;
  const int rot = (MODE == kPassInternal || ntiles <= 0) ? 0 : (int)((rsrc * 13u + (rsrc >> 5) * 7u) % (unsigned)ntiles);
  const uint32_t* __restrict__ bmask = p.blk_mask ? p.blk_mask + (size_t)bk * p.nblk : nullptr;
  const int32_t* __restrict__ ulist = p.union_list ? p.union_list + (size_t)bk * p.nblk : nullptr;
  const uint32_t* __restrict__ umask = p.union_mask ? p.union_mask + (size_t)bk * p.nblk : nullptr;
  auto tile_raw = [&](int i) -> TileRaw {        // i-th tile of this workgroup: table lookups only
    int j = i + rot;
    if (j >= ntiles) j -= ntiles;
    TileRaw r;
    r.e = tr.begin + j;
    r.word = 0;
    r.mask = 0xffffffffu;
    if constexpr (MODE == kPassSparseReuse) {
      const int blk_i = (int)fastdiv((uint32_t)r.e, p.div_tpb);     // entry of the union list
      r.word = sload(ulist, blk_i);
      r.mask = (uint32_t)sload(umask, blk_i);
    } else if constexpr (MODE == kPassSparseRefresh) {
      r.mask = (uint32_t)sload(bmask, (int)fastdiv((uint32_t)r.e, p.div_tpb));
    } else if constexpr (MODE == kPassDensePaged) {
      r.word = sload(p.block_table + (size_t)b * p.max_pages, (int)fastdiv((uint32_t)(r.e * C::KT), p.div_page));
    }
    return r;
  };
  auto tile_desc = [&](const TileRaw& r) -> TileDesc {
    TileDesc d;
    d.mask = r.mask;
    d.k0 = (MODE == kPassSparseReuse)
               ? r.word * p.key_block + C::KT * (r.e - (int)(fastdiv((uint32_t)r.e, p.div_tpb) * p.div_tpb.d))
               : r.e * C::KT;
    if constexpr (MODE == kPassDensePaged) {
      const uint32_t slot = fastdiv((uint32_t)d.k0, p.div_page);
      const int page = min(max(r.word, 0), p.num_pages - 1);       // clamped into the pool
      const int in_page = d.k0 - (int)(slot * p.div_page.d);
      const size_t off = (((size_t)page * p.Hkv + kvh) * p.page_size + in_page) * C::ROWB;
      d.kt = Kg + off;
      d.vt = Vg + off;
    } else {
      // a list entry past the end of the keys (reuse pass, short last key block) is skipped by the compute; its
      // loads, issued all the same so that every tile counts the same number of loads, read the head's first keys
      const int kload = (MODE == kPassSparseReuse && d.k0 >= nkeys) ? 0 : d.k0;
      d.kt = Kg + (size_t)kload * C::ROWB;
      d.vt = Vg + (size_t)kload * C::ROWB;
    }
    return d;
  };

  // ---- direct-to-LDS load slots of this lane: operand chunk pidx = (j*8 + wave)*64 + lane lives at LDS row
  // pidx / CPR, chunk position pidx % CPR, and holds logical chunk (position - rotation(row)) of that row.
  const uint32_t ring_base = (uint32_t)(uintptr_t)ring;
  int ld_row[C::NLOAD];
  uint32_t off_k[C::NLOAD], off_v[C::NLOAD];     // byte offsets inside a full tile
  int ck[C::NLOAD], cv[C::NLOAD];
#pragma unroll
  for (int j = 0; j < C::NLOAD; ++j) {
    const int pidx = (j * C::NW + wave) * 64 + lane;
    const int r = pidx / C::CPR, pc = pidx % C::CPR;
    ld_row[j] = r;
    ck[j] = (pc - C::rot_k(r)) & (C::CPR - 1);
    cv[j] = (pc - C::rot_v(r)) & (C::CPR - 1);
    off_k[j] = (uint32_t)(r * C::ROWB + ck[j] * 16);
    off_v[j] = (uint32_t)(r * C::ROWB + cv[j] * 16);
  }
  // (first key, mask) of the tiles in the ring, oldest first: [0] is the tile computed in this iteration
  int qk0[C::NS];
  uint32_t qmask[C::NS];
#pragma unroll
  for (int i = 0; i < C::NS; ++i) { qk0[i] = 0; qmask[i] = 0u; }
  auto issue_tile = [&](int i, const TileDesc& d) {
    const uint32_t sbase = ring_base + (uint32_t)(i % C::NS) * C::STAGE + wave * 1024;
    const int nvalid = nkeys - d.k0;
    if (nvalid >= C::KT) {
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j) dma16(d.kt, off_k[j], sbase + j * C::LSTEP);
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j) dma16(d.vt, off_v[j], sbase + C::OPB + j * C::LSTEP);
    } else {
      // ragged tile: rows past the end read the last key (in bounds; their scores are masked); an entry past the
      // end of the keys reads one row of the address tile_desc gave it
      const int last = max(nvalid, 1) - 1;
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j)
        dma16(d.kt, (uint32_t)(min(ld_row[j], last) * C::ROWB + ck[j] * 16), sbase + j * C::LSTEP);
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j)
        dma16(d.vt, (uint32_t)(min(ld_row[j], last) * C::ROWB + cv[j] * 16), sbase + C::OPB + j * C::LSTEP);
    }
  };

  // ---- prologue: the query rows go through the last ring stage(s), then the first tiles; everything is in
  // flight before the first wait.
  {
    const unsigned char* qg = (const unsigned char*)p.q + (grow_base + row0) * C::ROWB;
    const int qvalid = nrows - row0;                     // >= 1
    const uint32_t qbase = ring_base + (uint32_t)(C::NS - C::QSTAGES) * C::STAGE + wave * 1024;
#pragma unroll
    for (int part = 0; part < C::QPARTS; ++part)         // 64 rows at a time, each laid out like a K operand
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j) {
        const int r = min(64 * part + ld_row[j], qvalid - 1);
        dma16(qg, (uint32_t)(r * C::ROWB + ck[j] * 16), qbase + part * C::OPB + j * C::LSTEP);
      }
  }
  constexpr int kPre = (AHEAD < C::NS - C::QSTAGES) ? AHEAD : C::NS - C::QSTAGES;   // tiles issued while the queries sit in the ring
  {
    int pre = 0;
#pragma unroll
    for (int i = 0; i < kPre; ++i)
      if (i < ntiles) {
        const TileDesc d = tile_desc(tile_raw(i));
        issue_tile(i, d);
        qk0[i] = d.k0;
        qmask[i] = d.mask;
        ++pre;
      }
    wait_tiles<C::LPT>(pre);                             // the query loads were issued first
  }
  __syncthreads();
  bf16x8 qreg[C::NKS];
  {
    const int r = rg * 32 + l32;
    const unsigned char* qs = ring + (C::NS - C::QSTAGES) * C::STAGE + (r / 64) * C::OPB + (r % 64) * C::ROWB;
#pragma unroll
    for (int ks = 0; ks < C::NKS; ++ks)
      qreg[ks] = *(const bf16x8*)(qs + ((2 * ks + h + C::rot_k(r % 64)) & (C::CPR - 1)) * 16);
  }
  if constexpr (kPre < AHEAD) {
    // the queries took more than the last stage: the remaining start-up tiles go out once everyone has read them
    __syncthreads();
#pragma unroll
    for (int i = kPre; i < AHEAD; ++i)
      if (i < ntiles) {
        const TileDesc d = tile_desc(tile_raw(i));
        issue_tile(i, d);
        qk0[i] = d.k0;
        qmask[i] = d.mask;
      }
  }
  // table words of the next tile to be issued, fetched one iteration ahead (lookups off the critical path)
  TileRaw rnext;
  rnext.e = 0; rnext.word = 0; rnext.mask = 0u;
  if (AHEAD < ntiles) rnext = tile_raw(AHEAD);

  // per-lane LDS read addresses inside a stage
  uint32_t kaddr[C::NKS], vaddr[C::NDB];
#pragma unroll
  for (int ks = 0; ks < C::NKS; ++ks)
    kaddr[ks] = (uint32_t)(l32 * C::ROWB + ((2 * ks + h + C::rot_k(l32)) & (C::CPR - 1)) * 16);
  {
    const int i16 = lane & 15, blk1 = (lane >> 4) & 1;
    const int rrow = 4 * h + (i16 >> 2);                 // row of this lane inside an 8-key group
#pragma unroll
    for (int db = 0; db < C::NDB; ++db) {
      const int c = 4 * db + 2 * blk1 + ((i16 & 3) >> 1);
      const int pc = (c + C::rot_v(rrow)) & (C::CPR - 1);   // 8-key groups start at multiples of 8: same rotation
      vaddr[db] = (uint32_t)(rrow * C::ROWB + pc * 16 + (i16 & 1) * 8);
    }
  }

  WaveAcc<C::NDB> accs[NSETS];
#pragma unroll
  for (int i = 0; i < NSETS; ++i) accs[i].init();
  WaveAcc<C::NDB>& acc = accs[0];
  const uint32_t my_bit = 1u << ((row_ok ? row : 0) / p.Bq);

  auto lane_on_of = [&](uint32_t mask, int set) -> bool {
    if constexpr (MODE == kPassDenseHeads) return head_active;
    else if constexpr (MODE == kPassSparseReuse) return row_ok && (mask & my_bit) != 0u;
    else if constexpr (MODE == kPassSparseRefresh) return row_ok && (((mask & my_bit) != 0u) == (set == 0));
    else return true;
  };
  constexpr bool kMasked = (MODE == kPassDenseHeads || MODE == kPassSparseReuse || MODE == kPassSparseRefresh);
  // issue of tile t + AHEAD (into a stage every wavefront has left for good), then the lookups of the tile after it;
  // the queue then holds tiles t .. t + AHEAD
  auto refill = [&](int t) {
    if (t + AHEAD < ntiles) {
      const TileDesc d = tile_desc(rnext);
      issue_tile(t + AHEAD, d);
      qk0[AHEAD] = d.k0;
      qmask[AHEAD] = d.mask;
      if (t + AHEAD + 1 < ntiles) rnext = tile_raw(t + AHEAD + 1);
    }
  };
  auto advance = [&]() {
#pragma unroll
    for (int i = 0; i + 1 < C::NS; ++i) {
      qk0[i] = qk0[i + 1];
      qmask[i] = qmask[i + 1];
    }
  };

  if constexpr (kPairs) {
    // two tiles per barrier; the prologue put tiles 0 .. AHEAD-1 in flight, iteration t adds tiles t+AHEAD, t+AHEAD+1
    // into the stages of tiles t-2, t-1 (or the query stages), which every wavefront left before this barrier
    static_assert(!kListed, "row-pair layout: dense passes only");
    for (int t = 0; t < ntiles; t += 2) {
      wait_tiles<C::LPT>(min(AHEAD - 2, max(ntiles - 2 - t, 0)));   // tiles issued after tile t+1 so far
      __syncthreads();
#pragma unroll
      for (int u = 0; u < 2; ++u)
        if (t + AHEAD + u < ntiles) {
          const TileDesc d = tile_desc(tile_raw(t + AHEAD + u));
          issue_tile(t + AHEAD + u, d);
          qk0[AHEAD + u] = d.k0;
        }
#pragma unroll
      for (int u = 0; u < 2; ++u)
        if (t + u < ntiles) {
          const unsigned char* stage = ring + ((t + u) % C::NS) * C::STAGE;
          const int nvalid = min(C::KT, nkeys - qk0[u]);
          f32x16 s[C::NKB];
          tile_scores<D, C::NKB>(s, qreg, stage, kaddr, kb0);
          tile_softmax_pv<D, C::NKB>(acc, s, stage, vaddr, kb0, p.scale_log2, true, nvalid, h);
        }
#pragma unroll
      for (int i = 0; i + 2 < C::NS; ++i) qk0[i] = qk0[i + 2];
    }
  } else {
    for (int t = 0; t < ntiles; ++t) {
      wait_tiles<C::LPT>(min(AHEAD - 1, ntiles - 1 - t));      // tiles issued after tile t so far
      __syncthreads();
      refill(t);
      const unsigned char* stage = ring + (t % C::NS) * C::STAGE;
      const int k0 = qk0[0];
      const uint32_t mask = qmask[0];
      advance();
      const int nvalid = min(C::KT, nkeys - k0);
      if constexpr (MODE == kPassSparseReuse) {
        if (nvalid <= 0) continue;                             // a list entry past the end of the keys
      }
      bool on[NSETS];
      bool any_on = false;
#pragma unroll
      for (int i = 0; i < NSETS; ++i) {
        on[i] = lane_on_of(mask, i);
        any_on = any_on || on[i];
      }
      if (kMasked && !__any(any_on)) continue;
      f32x16 s[C::NKB];
      tile_scores<D, C::NKB>(s, qreg, stage, kaddr, kb0);
#pragma unroll
      for (int i = 0; i < NSETS; ++i) {
        if (NSETS > 1 && !__any(on[i])) continue;
        tile_softmax_pv<D, C::NKB>(accs[i], s, stage, vaddr, kb0, p.scale_log2, on[i], nvalid, h);
      }
    }
  }

  // Output column blocks this wavefront finishes and stores.  Row-pair layout: all of them.  Key-split layout: the two
  // wavefronts of a row group exchange halves, so that both take part in the merge and in the stores (the wavefront of
  // key half 0 keeps the lower column blocks, the other one the upper ones).
  constexpr int NDBK = (LAYOUT == kKeySplit) ? C::NDB / 2 : C::NDB;
  const int db_keep = (LAYOUT == kKeySplit) ? kb0 * NDBK : 0;
  if constexpr (LAYOUT == kKeySplit) {
    // ---- merge the two key halves through LDS.  Record per (set, row group, key half): the NDBK column blocks the
    // wavefront gives away, then its m and l; [register][lane] so that neighbouring lanes hit neighbouring banks.
    constexpr int REC = NDBK * 16 + 2;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NSETS; ++i) {
      float* mine = (float*)ring + (((size_t)i * NRG + rg) * 2 + kb0) * REC * 64 + lane;
#pragma unroll
      for (int db = 0; db < NDBK; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          // static register indices: select between the two halves instead of indexing by kb0
          mine[(db * 16 + r) * 64] = kb0 ? accs[i].o[db][r] : accs[i].o[NDBK + db][r];
        }
      mine[(NDBK * 16) * 64] = accs[i].m;
      mine[(NDBK * 16 + 1) * 64] = accs[i].l;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NSETS; ++i) {
      const float* other = (const float*)ring + (((size_t)i * NRG + rg) * 2 + (kb0 ^ 1)) * REC * 64 + lane;
      WaveAcc<C::NDB>& a = accs[i];
      const float mo = other[(NDBK * 16) * 64], lo = other[(NDBK * 16 + 1) * 64];
      // both wavefronts of the pair evaluate the same expressions on (key half 0, key half 1) in that order
      const float m0 = kb0 ? mo : a.m, m1 = kb0 ? a.m : mo;
      const float l0 = kb0 ? lo : a.l, l1 = kb0 ? a.l : lo;
      const float M = fmaxf(m0, m1);
      const float Mu = (M == -INFINITY) ? 0.f : M;
      const float w0 = __builtin_amdgcn_exp2f(m0 - Mu), w1 = __builtin_amdgcn_exp2f(m1 - Mu);
      const float ws = kb0 ? w1 : w0, wo = kb0 ? w0 : w1;
#pragma unroll
      for (int db = 0; db < NDBK; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float x = other[(db * 16 + r) * 64];
          // kept block = lower ones for key half 0, upper ones for key half 1; result parked in o[db]
          const float own = kb0 ? a.o[NDBK + db][r] : a.o[db][r];
          a.o[db][r] = kb0 ? (x * wo + own * ws) : (own * ws + x * wo);
        }
      a.l = l0 * w0 + l1 * w1;
      a.m = M;
    }
  }

  // ---- epilogue
  const float l_row = acc.l + __shfl_xor(acc.l, 32, 64);
  if constexpr (MODE == kPassInternal) {
    if (!row_ok) return;
    // Eq. 8-9 with the cached pair expressed through (o, m, lse): A_out e^{L_out-M} = o e^{m-M}
    const bool has_ext = p.ext_o != nullptr;             // workgroup-uniform
    float me2 = -INFINITY, le = 0.f;
    if (has_ext) {
      const float em = p.ext_m[grow], el = p.ext_lse[grow];
      if (el != -INFINITY) {
        me2 = em * kLog2e;
        le = exp2f((el - em) * kLog2e);
      }
    }
    const float M2 = fmaxf(me2, acc.m);
    const float Mu = (M2 == -INFINITY) ? 0.f : M2;
    const float we = exp2f(me2 - Mu), wi = exp2f(acc.m - Mu);
    const float den = le * we + l_row * wi;
    const float inv = den > 0.f ? 1.f / den : 0.f;
    __bf16* out = (__bf16*)p.out + grow * D;
#pragma unroll
    for (int db = 0; db < NDBK; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int d0 = 32 * (db_keep + db) + 8 * q4 + 4 * h;
        f32x4 e = {0.f, 0.f, 0.f, 0.f};
        if (has_ext) e = *(const f32x4*)(p.ext_o + grow * D + d0);
        float r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = (acc.o[db][4 * q4 + i] * wi + e[i] * we) * inv;
        u32x2 pk;
        pk.x = pack_bf16x2(r[0], r[1]);
        pk.y = pack_bf16x2(r[2], r[3]);
        *(u32x2*)(out + d0) = pk;
      }
    if (p.lse_out != nullptr && h == 0) p.lse_out[grow] = den > 0.f ? (M2 + log2f(den)) * kLn2 : -INFINITY;
    return;
  } else {
    if (p.direct) {
      // single split: this is the final partial.  Same conversion as the split combine: m is rounded when
      // converted to natural-log units, o is rescaled to the reference consumers recover from it.
      if (!(row_ok && head_active)) return;
      float m_nat = -INFINITY, L = -INFINITY, adj = 0.f;
      if (l_row > 0.f) {
        m_nat = acc.m * kLn2;
        adj = exp2f(acc.m - m_nat * kLog2e);
        L = (acc.m + log2f(l_row)) * kLn2;
      }
#pragma unroll
      for (int db = 0; db < NDBK; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d0 = 32 * (db_keep + db) + 8 * q4 + 4 * h;
          f32x4 o4 = {acc.o[db][4 * q4] * adj, acc.o[db][4 * q4 + 1] * adj, acc.o[db][4 * q4 + 2] * adj,
                      acc.o[db][4 * q4 + 3] * adj};
          *(f32x4*)(p.ws_o + grow * D + d0) = o4;
        }
      if (h == 0 && kb0 == 0) {
        p.ws_m[grow] = m_nat;
        p.ws_l[grow] = L;
      }
      return;
    }
    if (!row_ok) return;
    const size_t rows_total = (size_t)p.B * p.Hq * p.Bq;
    const size_t wrow = (size_t)split * rows_total + grow;
#pragma unroll
    for (int i = 0; i < NSETS; ++i) {
      float* __restrict__ w_o = i ? p.ws_o2 : p.ws_o;
      float* __restrict__ w_m = i ? p.ws_m2 : p.ws_m;
      float* __restrict__ w_l = i ? p.ws_l2 : p.ws_l;
      const WaveAcc<C::NDB>& a = accs[i];
      const float l_i = (i == 0) ? l_row : a.l + __shfl_xor(a.l, 32, 64);
#pragma unroll
      for (int db = 0; db < NDBK; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int d0 = 32 * (db_keep + db) + 8 * q4 + 4 * h;
          f32x4 o4 = {a.o[db][4 * q4], a.o[db][4 * q4 + 1], a.o[db][4 * q4 + 2], a.o[db][4 * q4 + 3]};
          // streaming store: read next by another kernel, never again by this one (measured: faster than staging
          // the rows through LDS for whole-row stores, and faster than write-back stores)
          __builtin_nontemporal_store(o4, (f32x4*)(w_o + wrow * D + d0));
        }
      if (h == 0 && kb0 == 0) {
        w_m[wrow] = a.m;
        w_l[wrow] = l_i;
      }
    }
  }
}

template <int D, int MODE, int LAYOUT, int NRG = 4>
hipError_t launch_stream(const PassParams& p, hipStream_t s) {
  using C = SCfg<D, LAYOUT, (MODE == kPassSparseRefresh) ? 2 : 1, NRG>;
  auto kern = attn_stream_kernel<D, MODE, LAYOUT, NRG>;
  static LdsLimit lim;
  hipError_t e = raise_lds_limit(kern, C::LDS, lim, C::LDS);
  if (e != hipSuccess) return e;
  const int nrows = p.G * p.Bq;
  const int ntile_rows = (nrows + C::ROWS - 1) / C::ROWS;
  long long nwg = (long long)p.B * p.Hkv * ntile_rows * p.nsplit;
  if (MODE == kPassDensePaged) nwg = (((long long)p.B * p.Hkv * p.nsplit + 7) / 8) * 8 * ntile_rows;
  if (nwg >= (1ll << 31)) return hipErrorInvalidValue;
  PassParams q = p;
  if (MODE == kPassDensePaged) q.div_page = make_fastdiv((uint32_t)p.page_size);
  q.div_tpb = make_fastdiv((uint32_t)(p.key_block > 0 ? p.key_block / kKeyTile : 1));
  {
    // long streams only: below 64 tiles per split a 1/64 bias rounds away
    const int tiles = (p.nkeys + kKeyTile - 1) / kKeyTile;
    q.xcd_bias = ((MODE == kPassDense || MODE == kPassSparseRefresh) && ntile_rows == 1 && p.nsplit % 2 == 0 &&
                  nwg % 8 == 0 && tiles >= 64 * p.nsplit) ? 1 : 0;
  }
  q.div_rowtiles = make_fastdiv((uint32_t)ntile_rows);
  q.div_nsplit = make_fastdiv((uint32_t)p.nsplit);
  q.div_hkv = make_fastdiv((uint32_t)p.Hkv);
  launch_attn_kernel(kern, dim3((unsigned)nwg), dim3(C::THREADS), C::LDS, s, q);
  return hipGetLastError();
}

// key-split layout with as many 32-row groups per workgroup as the KV group has rows for
template <int D, int MODE>
hipError_t launch_key_split(const PassParams& p, hipStream_t s) {
  const int nrows = p.G * p.Bq;
  if (nrows <= 32) return launch_stream<D, MODE, kKeySplit, 1>(p, s);
  if (nrows <= 64) return launch_stream<D, MODE, kKeySplit, 2>(p, s);
  return launch_stream<D, MODE, kKeySplit, 4>(p, s);
}

template <int D>
hipError_t launch_stream_d(const PassParams& p, PassMode mode, hipStream_t s) {
  const int nrows = p.G * p.Bq;
  switch (mode) {
    case kPassDense:
      if (dense_row_pairs(nrows, D)) return launch_stream<D, kPassDense, kRowPair>(p, s);
      return launch_key_split<D, kPassDense>(p, s);
    case kPassDenseHeads: return launch_key_split<D, kPassDenseHeads>(p, s);
    case kPassDensePaged: return launch_key_split<D, kPassDensePaged>(p, s);
    case kPassSparseReuse: return launch_key_split<D, kPassSparseReuse>(p, s);
    case kPassSparseRefresh: return launch_key_split<D, kPassSparseRefresh>(p, s);
    case kPassInternal: return launch_stream<D, kPassInternal, kRowPair>(p, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

// Shapes the streaming kernel takes over from the register-staged one: KV groups of up to 128 rows (and the many-row
// shapes of the row-pair layout) whose workgroups stream at least 8 tiles each.
bool stream_bf16_covers(const PassParams& p, int D, PassMode mode) {
  const int nrows = p.G * p.Bq;
  const int tiles = (p.nkeys + kKeyTile - 1) / kKeyTile;
  switch (mode) {
    case kPassDense:
      if (dense_row_pairs(nrows, D)) return tiles >= 8 * p.nsplit;
      return nrows <= 128 && tiles >= 8 * p.nsplit;
    case kPassDenseHeads:
    case kPassDensePaged:
    case kPassSparseReuse:
    case kPassSparseRefresh:
      return nrows <= 128 && tiles >= 8 * p.nsplit;
    case kPassInternal: {
      // compute-bound internal pass: many rows per KV head and a 256-row workgroup for (almost) every CU
      const long long wgs = (long long)p.B * p.Hkv * ((nrows + 255) / 256);
      return nrows >= 1024 && wgs >= 128 && tiles >= 8;
    }
    default: return false;
  }
}

// Name of the instantiation launch_stream_bf16 picks, as a kernel trace prints it (without the namespaces).
int stream_bf16_name(const PassParams& p, int D, PassMode mode, char* buf, size_t n) {
  const bool rp = (mode == kPassDense && dense_row_pairs(p.G * p.Bq, D)) || mode == kPassInternal;
  const int nrows = p.G * p.Bq;
  return snprintf(buf, n, "attn_stream_kernel<%d, %d, %d, %d>", D, (int)mode, rp ? (int)kRowPair : (int)kKeySplit,
                  (rp || nrows > 64) ? 4 : nrows > 32 ? 2 : 1);
}

hipError_t launch_stream_bf16(const PassParams& p, int D, PassMode mode, hipStream_t s) {
  return D == 64 ? launch_stream_d<64>(p, mode, s) : launch_stream_d<128>(p, mode, s);
}

}  // namespace fb
