// bf16 streaming attention pass for gfx950 (MI355X): K/V tiles travel from global memory straight into a ring
// of LDS stages (direct-to-LDS 16-byte loads, no register staging), K operands are read back with
// ds_read_b128 from a rotation-swizzled row-major layout, V operands with the transposing LDS read
// (ds_read_b64_tr_b16) from row-major V, so nothing is transposed or re-stored on the way.
//
// Computes the per-row statistics of Eq. 3-4/6 (arxiv 2602.05305, Section 4.2) of a block of query rows
// against a long stream of keys and stores split partials (or, with one split, the final partial).
//
// Work decomposition
//   workgroup = 8 wavefronts, one tile stream of 64-key tiles, NS ring stages (NS - 1 tiles in flight).
//   KSPLIT = 2: 128 group-flattened rows; wavefront w owns rows [32 (w%4), +32) and the key half w/4 of every
//               tile; the two halves' statistics are merged through LDS after the last tile.
//   Per tile and wavefront: S^T = K Q^T on v_mfma_f32_32x32x16_bf16 (A = K rows from LDS, B = Q^T in
//   registers), in-lane online softmax with a lazily moved reference, O^T += V^T P^T with the lane's own
//   probabilities as the B operand (see fb_attn_bf16.hip for the register layout reasoning, which is the same).
// LDS layout of a stage: [K: 64 rows x D*2 bytes][V: 64 rows x D*2 bytes], rows unpadded, the 16-byte chunks
//   of a row rotated by a row-dependent amount (K: by row, V: by 4*row at head_dim 128; by row/2 and
//   4*(row/2) at head_dim 64) so that both read patterns are bank-conflict-free.  A direct-to-LDS load puts
//   the 64 lanes' chunks at consecutive LDS addresses, so the rotation is applied on the global-address side.
// Synchronisation: the direct-to-LDS loads are issued from inline assembly, invisible to the compiler's
//   wait-count insertion (which would otherwise drain every outstanding load before any LDS read); each
//   wavefront waits for its own loads of a tile with an explicit s_waitcnt vmcnt(n), then the workgroup
//   barrier makes the tile visible to all.  The stage refilled after barrier t is the one read in iteration
//   t-1, which every wavefront has left by then.
#include "fb_kernels.h"
#include <stdlib.h>

namespace fb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kStreamThreads = 512;

template <int D>
struct SCfg {
  static constexpr int KT = 64;                       // keys per tile
  static constexpr int ROWB = D * 2;                  // bytes per key row
  static constexpr int CPR = ROWB / 16;               // 16-byte chunks per row
  static constexpr int OPB = KT * ROWB;               // bytes per operand (K or V) per tile
  static constexpr int STAGE = 2 * OPB;
  static constexpr int NLOAD = OPB / (kStreamThreads * 16);   // direct-to-LDS loads per lane, operand and tile
  static constexpr int LPT = 2 * NLOAD;               // loads per lane and tile
  static constexpr int NS = (D == 128) ? 4 : 6;       // ring stages
  static constexpr int NKS = D / 16;                  // MFMA k-steps of the score product
  static constexpr int NDB = D / 32;                  // 32-wide output column blocks
  static constexpr int QSTAGES = (128 * ROWB + STAGE - 1) / STAGE;   // stages the 128 query rows occupy at start
  static constexpr int LDS = NS * STAGE;
  // rotation (in chunks) of row `row`
  __device__ static __forceinline__ int rot_k(int row) { return D == 128 ? row : (row >> 1); }
  __device__ static __forceinline__ int rot_v(int row) { return D == 128 ? 4 * row : 4 * (row >> 1); }
};

// One 16-byte direct-to-LDS load per lane: lane l's chunk lands at LDS byte lds_base + 16 l.  Global address =
// base (wavefront-uniform) + off (per lane, unsigned 32-bit).
__device__ __forceinline__ void dma16(const void* base, uint32_t off, uint32_t lds_base) {
  // base and lds_base are wavefront-uniform by construction; readfirstlane says so to the compiler, which
  // otherwise may hand the "s" operands over in vector registers (not encodable here)
  const uint64_t b = (uint64_t)(uintptr_t)base;
  // (the builtin returns int: each half goes through uint32_t so that nothing is sign-extended)
  const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32));
  const uint64_t bu = ((uint64_t)b_hi << 32) | (uint64_t)b_lo;
  const uint32_t lu = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(off), "s"(bu), "s"(lu)
               : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
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

// Scores of this wavefront's 32 rows against key blocks [KB0, KB0 + NKB) of the tile in `stage`.
// kaddr[ks] = per-lane byte address (within a stage, key block 0) of the K chunk of k-step ks.
template <int D, int NKB>
__device__ __forceinline__ void tile_scores(f32x16 (&s)[NKB], const bf16x8 (&qreg)[SCfg<D>::NKS],
                                            const unsigned char* __restrict__ stage, const uint32_t (&kaddr)[SCfg<D>::NKS],
                                            int kb0) {
  using C = SCfg<D>;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
  for (int ks0 = 0; ks0 < C::NKS; ks0 += 2) {
    bf16x8 a[2][NKB];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
        a[u][kb] = *(const bf16x8*)(stage + kaddr[ks0 + u] + (kb0 + kb) * 32 * C::ROWB);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u][kb], qreg[ks0 + u], s[kb], 0, 0, 0);
  }
}

// Online softmax update with the tile's scores and value accumulation.
//   s[kb][r] = raw dot product of query row lane%32 with key 32 (kb0 + kb) + 8 (r/4) + 4 h + r%4
//   vaddr[db] = per-lane byte address (within a stage) of the lane's share of the transposing V read of
//               column block db, key offset 0; the 4-key groups are reached through immediate offsets
template <int D, int NKB>
__device__ __forceinline__ void tile_softmax_pv(WaveAcc<SCfg<D>::NDB>& st, f32x16 (&s)[NKB],
                                                const unsigned char* __restrict__ stage,
                                                const uint32_t (&vaddr)[SCfg<D>::NDB], int kb0, float scale_log2,
                                                bool lane_on, int nvalid, int h) {
  using C = SCfg<D>;
  if (nvalid < C::KT) {
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
  bf16x8 pb[2 * NKB];
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
    for (int db = 0; db < C::NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
  }
  // O^T[db] += V^T P^T over 16-key steps: A operand element e of lane half h is key 16u + 8(e/4) + 4h + e%4 of
  // the key block, i.e. two transposing reads of 4 consecutive keys each (the lane's own 4h + i/4 row offset
  // is inside vaddr).
#pragma unroll
  for (int t = 0; t < 2 * NKB; ++t) {
    const int krow = (kb0 + t / 2) * 32 + 16 * (t % 2);
    bf16x8 a[C::NDB];
#pragma unroll
    for (int db = 0; db < C::NDB; ++db) {
      const unsigned char* base = stage + C::OPB + vaddr[db] + krow * C::ROWB;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base + 8 * C::ROWB));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      a[db] = __builtin_bit_cast(bf16x8, both);
    }
#pragma unroll
    for (int db = 0; db < C::NDB; ++db)
      st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[db], pb[t], st.o[db], 0, 0, 0);
  }
}

template <int D, int MODE>
__global__ __launch_bounds__(kStreamThreads, 1) void attn_stream_kernel(const PassParams p) {
  using C = SCfg<D>;
  static_assert(MODE == kPassDense || MODE == kPassDenseHeads, "modes of the streaming kernel");
  extern __shared__ __align__(16) unsigned char ring[];
  const int lane = threadIdx.x & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));     // wavefront-uniform (scalar)
  const int rg = wave & 3;        // 32-row group
  const int kb0 = wave >> 2;      // key half of every tile

  // XCD-aware remap: hardware deals consecutive workgroup ids round-robin to the 8 XCDs; make each XCD own a
  // contiguous range of (batch, KV head, split) units.
  const int nwg = gridDim.x;
  const int nrows = p.G * p.Bq;
  int rt;
  uint32_t rest;
  {
    const int bid = blockIdx.x, q8 = nwg / 8, r8 = nwg % 8;
    const int xcd = bid % 8, j = bid / 8;
    int w = (xcd < r8 ? xcd * (q8 + 1) : r8 * (q8 + 1) + (xcd - r8) * q8) + j;
    if constexpr (MODE == kPassDenseHeads) {
      if (p.div_rowtiles.d > 1) w = bid;     // whole heads drop out: deal a head's row tiles over the XCDs
    }
    rest = fastdiv((uint32_t)w, p.div_rowtiles);
    rt = w - (int)(rest * p.div_rowtiles.d);
  }
  const uint32_t unit = rest;
  const uint32_t r2 = fastdiv(rest, p.div_nsplit);
  const int split = (int)(rest - r2 * p.div_nsplit.d);
  rest = r2;
  const int b = (int)fastdiv(rest, p.div_hkv);
  const int kvh = (int)(rest - (uint32_t)b * p.div_hkv.d);
  const int bk = b * p.Hkv + kvh;
  const int nkeys = p.nkeys;

  const int row0 = rt * 128;                                   // first group-flattened row of the workgroup
  const int row = row0 + rg * 32 + l32;
  const bool row_ok = row < nrows;
  const size_t grow_base = (size_t)(b * p.Hq + kvh * p.G) * p.Bq;
  const size_t grow = grow_base + row;
  bool head_active = true;
  if constexpr (MODE == kPassDenseHeads) {
    head_active = row_ok && p.head_on[b * p.Hq + kvh * p.G + row / p.Bq] != 0;
    if (!__syncthreads_or(head_active ? 1 : 0)) return;
  }

  const unsigned char* __restrict__ Kg = (const unsigned char*)p.k + (size_t)bk * nkeys * C::ROWB;
  const unsigned char* __restrict__ Vg = (const unsigned char*)p.v + (size_t)bk * nkeys * C::ROWB;

  // tile list of this workgroup: a contiguous range of the prefix's tiles, visited in rotated order (workgroups
  // that run in lockstep would otherwise read the same offset of their chunks, i.e. the same channels, at once)
  const int total = (nkeys + C::KT - 1) / C::KT;
  const TileRange tr = split_range(total, p.div_nsplit, split);
  const int ntiles = tr.end - tr.begin;
  const uint32_t rsrc = (p.div_rowtiles.d == 1) ? blockIdx.x : unit;
  const int rot = ntiles <= 0 ? 0 : (int)((rsrc * 13u + (rsrc >> 5) * 7u) % (unsigned)ntiles);
  auto tile_k0 = [&](int i) -> int {
    int j = i + rot;
    if (j >= ntiles) j -= ntiles;
    return (tr.begin + j) * C::KT;
  };

  // ---- direct-to-LDS load slots of this lane: operand chunk p = (j*8 + wave)*64 + lane lives at LDS row
  // p / CPR, chunk position p % CPR, and holds logical chunk (position - rotation(row)) of that row.
  const uint32_t ring_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)ring);
  int ld_row[C::NLOAD];
  uint32_t off_k[C::NLOAD], off_v[C::NLOAD];     // byte offsets inside a full tile
  int ck[C::NLOAD], cv[C::NLOAD];
#pragma unroll
  for (int j = 0; j < C::NLOAD; ++j) {
    const int pidx = (j * 8 + wave) * 64 + lane;
    const int r = pidx / C::CPR, pc = pidx % C::CPR;
    ld_row[j] = r;
    ck[j] = (pc - C::rot_k(r)) & (C::CPR - 1);
    cv[j] = (pc - C::rot_v(r)) & (C::CPR - 1);
    off_k[j] = (uint32_t)(r * C::ROWB + ck[j] * 16);
    off_v[j] = (uint32_t)(r * C::ROWB + cv[j] * 16);
  }
  auto issue_tile = [&](int i) {
    const int k0 = tile_k0(i);
    const uint32_t sbase = ring_base + (uint32_t)(i % C::NS) * C::STAGE + wave * 1024;
    const unsigned char* kt = Kg + (size_t)k0 * C::ROWB;
    const unsigned char* vt = Vg + (size_t)k0 * C::ROWB;
    const int nvalid = nkeys - k0;
    if (nvalid >= C::KT) {
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j) dma16(kt, off_k[j], sbase + j * 8192);
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j) dma16(vt, off_v[j], sbase + C::OPB + j * 8192);
    } else {
      // ragged last tile: rows past the end read the last key (in bounds; their scores are masked)
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j)
        dma16(kt, (uint32_t)(min(ld_row[j], nvalid - 1) * C::ROWB + ck[j] * 16), sbase + j * 8192);
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j)
        dma16(vt, (uint32_t)(min(ld_row[j], nvalid - 1) * C::ROWB + cv[j] * 16), sbase + C::OPB + j * 8192);
    }
  };

  // ---- prologue: the 128 query rows go through the last ring stage(s) (free until tile NS - QSTAGES is
  // issued), then the first tiles; everything is in flight before the first wait.
  {
    const unsigned char* qg = (const unsigned char*)p.q + (grow_base + row0) * C::ROWB;
    const int qvalid = nrows - row0;                     // >= 1
    const uint32_t qbase = ring_base + (uint32_t)(C::NS - C::QSTAGES) * C::STAGE + wave * 1024;
#pragma unroll
    for (int half = 0; half < 2; ++half)                 // rows [0,64) and [64,128): each laid out like a K operand
#pragma unroll
      for (int j = 0; j < C::NLOAD; ++j) {
        const int r = min(64 * half + ld_row[j], qvalid - 1);
        dma16(qg, (uint32_t)(r * C::ROWB + ck[j] * 16), qbase + half * C::OPB + j * 8192);
      }
  }
  constexpr int kPre = C::NS - C::QSTAGES;               // tiles issued before the queries have been read
  static_assert(C::QSTAGES == 1 && kPre == C::NS - 1, "the query rows fit the last stage");
#pragma unroll
  for (int i = 0; i < kPre; ++i)
    if (i < ntiles) issue_tile(i);
  // every lane issued 2*NLOAD query loads first and LPT loads per tile after them
  {
    const int pre = min(kPre, max(ntiles, 0));
    if (pre >= 3) wait_vm<3 * C::LPT>();
    else if (pre == 2) wait_vm<2 * C::LPT>();
    else if (pre == 1) wait_vm<C::LPT>();
    else wait_vm<0>();
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

  WaveAcc<C::NDB> acc;
  acc.init();

  for (int t = 0; t < ntiles; ++t) {
    const int younger = min(C::NS - 2, ntiles - 1 - t);    // tiles issued after tile t so far
    if (younger >= 4) wait_vm<4 * C::LPT>();
    else if (younger == 3) wait_vm<3 * C::LPT>();
    else if (younger == 2) wait_vm<2 * C::LPT>();
    else if (younger == 1) wait_vm<C::LPT>();
    else wait_vm<0>();
    __syncthreads();
    if (t + C::NS - 1 < ntiles) issue_tile(t + C::NS - 1);
    const unsigned char* stage = ring + (t % C::NS) * C::STAGE;
    const int nvalid = min(C::KT, nkeys - tile_k0(t));
    f32x16 s[1];
    tile_scores<D, 1>(s, qreg, stage, kaddr, kb0);
    if constexpr (MODE == kPassDenseHeads) {
      tile_softmax_pv<D, 1>(acc, s, stage, vaddr, kb0, p.scale_log2, head_active, nvalid, h);
    } else {
      tile_softmax_pv<D, 1>(acc, s, stage, vaddr, kb0, p.scale_log2, true, nvalid, h);
    }
  }

  // ---- merge the two key halves through LDS: wavefronts 4..7 hand their statistics to wavefronts 0..3
  {
    constexpr int REC = C::NDB * 16 + 2;
    float* mbuf = (float*)ring + (size_t)rg * REC * 64 + lane;
    __syncthreads();
    if (kb0 == 1) {
#pragma unroll
      for (int db = 0; db < C::NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) mbuf[(db * 16 + r) * 64] = acc.o[db][r];
      mbuf[(C::NDB * 16) * 64] = acc.m;
      mbuf[(C::NDB * 16 + 1) * 64] = acc.l;
    }
    __syncthreads();
    if (kb0 == 1) return;
    const float m1 = mbuf[(C::NDB * 16) * 64], l1 = mbuf[(C::NDB * 16 + 1) * 64];
    const float M = fmaxf(acc.m, m1);
    const float Mu = (M == -INFINITY) ? 0.f : M;
    const float w0 = __builtin_amdgcn_exp2f(acc.m - Mu), w1 = __builtin_amdgcn_exp2f(m1 - Mu);
#pragma unroll
    for (int db = 0; db < C::NDB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc.o[db][r] = acc.o[db][r] * w0 + mbuf[(db * 16 + r) * 64] * w1;
    acc.l = acc.l * w0 + l1 * w1;
    acc.m = M;
  }

  // ---- epilogue
  const float l_row = acc.l + __shfl_xor(acc.l, 32, 64);
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
    for (int db = 0; db < C::NDB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int d0 = 32 * db + 8 * q4 + 4 * h;
        f32x4 o4 = {acc.o[db][4 * q4] * adj, acc.o[db][4 * q4 + 1] * adj, acc.o[db][4 * q4 + 2] * adj,
                    acc.o[db][4 * q4 + 3] * adj};
        *(f32x4*)(p.ws_o + grow * D + d0) = o4;
      }
    if (h == 0) {
      p.ws_m[grow] = m_nat;
      p.ws_l[grow] = L;
    }
    return;
  }
  if (!row_ok) return;
  const size_t rows_total = (size_t)p.B * p.Hq * p.Bq;
  const size_t wrow = (size_t)split * rows_total + grow;
#pragma unroll
  for (int db = 0; db < C::NDB; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int d0 = 32 * db + 8 * q4 + 4 * h;
      f32x4 o4 = {acc.o[db][4 * q4], acc.o[db][4 * q4 + 1], acc.o[db][4 * q4 + 2], acc.o[db][4 * q4 + 3]};
      // streaming store: read next by another kernel, never again by this one
      __builtin_nontemporal_store(o4, (f32x4*)(p.ws_o + wrow * D + d0));
    }
  if (h == 0) {
    p.ws_m[wrow] = acc.m;
    p.ws_l[wrow] = l_row;
  }
  __builtin_amdgcn_s_waitcnt(0);
}

template <int D, int MODE>
hipError_t launch_stream(const PassParams& p, hipStream_t s) {
  auto kern = attn_stream_kernel<D, MODE>;
  constexpr int lds = SCfg<D>::LDS;
  // raising the dynamic-LDS limit is a host-only call; made on every launch so that no process-wide flag is kept
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return e;
  const int nrows = p.G * p.Bq;
  const int ntile_rows = (nrows + 127) / 128;
  const long long nwg = (long long)p.B * p.Hkv * ntile_rows * p.nsplit;
  if (nwg >= (1ll << 31)) return hipErrorInvalidValue;
  PassParams q = p;
  q.div_rowtiles = make_fastdiv((uint32_t)ntile_rows);
  q.div_nsplit = make_fastdiv((uint32_t)p.nsplit);
  q.div_hkv = make_fastdiv((uint32_t)p.Hkv);
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kStreamThreads), lds, s, q);
  return hipGetLastError();
}

}  // namespace

bool stream_bf16_covers(const PassParams& p, PassMode mode) {

  if (mode != kPassDense && mode != kPassDenseHeads) return false;
  const int nrows = p.G * p.Bq;
  const int tiles = (p.nkeys + kKeyTile - 1) / kKeyTile;
  return nrows > 64 && nrows <= 128 && tiles >= 8 * p.nsplit;
}

hipError_t launch_stream_bf16(const PassParams& p, int D, PassMode mode, hipStream_t s) {
  if (mode == kPassDense) return D == 64 ? launch_stream<64, kPassDense>(p, s) : launch_stream<128, kPassDense>(p, s);
  if (mode == kPassDenseHeads) return D == 64 ? launch_stream<64, kPassDenseHeads>(p, s) : launch_stream<128, kPassDenseHeads>(p, s);
  return hipErrorInvalidValue;
}

}  // namespace fb
