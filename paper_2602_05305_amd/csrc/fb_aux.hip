// Small kernels around the attention passes: the split-KV combine (Eq. 5 applied to the
// per-split partials, fixed order), key-block pooling / top-k selection for the sparse
// variant, and the per-KV-group selection masks + union list the sparse passes iterate over.
#include "fb_kernels.h"

namespace fb {
namespace {

// Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of work items, the same
// cut the attention pass uses for its (batch, KV head, split) units, so that rows are folded on the XCD whose
// L2 their split partials were written through.
__device__ __forceinline__ uint32_t xcd_contiguous(uint32_t bid, uint32_t n) {
  const uint32_t q8 = n / 8, r8 = n % 8, xcd = bid % 8, j = bid / 8;
  return (xcd < r8 ? xcd * (q8 + 1) : r8 * (q8 + 1) + (xcd - r8) * q8) + j;
}


constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// v_exp_f32 directly: every use below has an argument that is <= 0, -inf, or a small positive number,
// where the library exp2f's extra range handling (denormal results) buys nothing.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ------------------------------------------------------------------------------ combine
// A folded partial in the log2 domain: o4 (4 columns of this thread), reference m2, sum l.
struct Folded {
  float4 o;
  float m2, l;
};

__device__ __forceinline__ Folded fold_two(const Folded& a, const Folded& b) {
  Folded f;
  f.m2 = fmaxf(a.m2, b.m2);
  const float mu = (f.m2 == -INFINITY) ? 0.f : f.m2;
  const float wa = fast_exp2(a.m2 - mu), wb = fast_exp2(b.m2 - mu);
  f.o.x = a.o.x * wa + b.o.x * wb;
  f.o.y = a.o.y * wa + b.o.y * wb;
  f.o.z = a.o.z * wa + b.o.z * wb;
  f.o.w = a.o.w * wa + b.o.w * wb;
  f.l = a.l * wa + b.l * wb;
  return f;
}

// Emit (o, m, lse) in natural-log units.  m is rounded when converted, so o and l are
// rescaled to the reference that consumers recover as m * log2(e): the pair stays exact.
__device__ __forceinline__ void emit(const Folded& f, float* __restrict__ o, float* __restrict__ m,
                                     float* __restrict__ lse, size_t row, int D, int c4) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  float m_nat = -INFINITY, L = -INFINITY;
  if (f.l > 0.f) {
    m_nat = f.m2 * kLn2;
    const float back = m_nat * kLog2e;
    const float adj = fast_exp2(f.m2 - back);
    v = make_float4(f.o.x * adj, f.o.y * adj, f.o.z * adj, f.o.w * adj);
    L = (f.m2 + log2f(f.l)) * kLn2;
  }
  *(float4*)(o + row * D + c4 * 4) = v;
  if (c4 == 0) {
    m[row] = m_nat;
    lse[row] = L;
  }
}

// float -> bf16 bits, round to nearest even (inputs are finite)
__device__ __forceinline__ uint32_t bf16_rne(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ Folded empty_folded() {
  Folded f;
  f.o = make_float4(0.f, 0.f, 0.f, 0.f);
  f.m2 = -INFINITY;
  f.l = 0.f;
  return f;
}

// Everything after the split fold: residual in/out, total, emission (shared by both kernels).
__device__ __forceinline__ void finish_row(const CombineParams& p, const Folded& sel, Folded res,
                                           bool have_res_set, size_t row, int c4) {
  if (!have_res_set && p.res_in_o != nullptr) {   // reuse: cached residual, natural-log units
    const float lse = p.res_in_lse[row];
    if (lse != -INFINITY) {
      const float m = p.res_in_m[row];
      res.m2 = m * kLog2e;
      res.l = fast_exp2((lse - m) * kLog2e);
      res.o = *(const float4*)(p.res_in_o + row * p.D + c4 * 4);
    }
  }
  if (p.res_out_o != nullptr) emit(res, p.res_out_o, p.res_out_m, p.res_out_lse, row, p.D, c4);
  const Folded total = fold_two(sel, res);
  emit(total, p.o, p.m, p.lse, row, p.D, c4);
  if (p.fin_out != nullptr) {
    // fused refresh step: Eq. 8-9 with the block-internal partial, then normalise
    Folded in;
    in.m2 = p.blk_m[row];
    in.l = p.blk_l[row];
    in.o = *(const float4*)(p.blk_o + row * p.D + c4 * 4);
    const Folded f = fold_two(total, in);
    const float inv = f.l > 0.f ? 1.f / f.l : 0.f;
    const float4 r = make_float4(f.o.x * inv, f.o.y * inv, f.o.z * inv, f.o.w * inv);
    if (p.fin_bf16) {
      uint2 pk;
      pk.x = bf16_rne(r.x) | (bf16_rne(r.y) << 16);
      pk.y = bf16_rne(r.z) | (bf16_rne(r.w) << 16);
      *(uint2*)((uint16_t*)p.fin_out + row * p.D + c4 * 4) = pk;
    } else {
      *(float4*)((float*)p.fin_out + row * p.D + c4 * 4) = r;
    }
    if (p.fin_lse != nullptr && c4 == 0) p.fin_lse[row] = f.l > 0.f ? (f.m2 + log2f(f.l)) * kLn2 : -INFINITY;
  }
}

// Fold of the splits first, first + stride, ... of one row (4 columns of it).
__device__ __forceinline__ Folded fold_strided(const float* __restrict__ ws_o, const float* __restrict__ ws_m,
                                               const float* __restrict__ ws_l, int nsplit, size_t rows,
                                               size_t row, int D, int c4, int first, int stride) {
  // Chunks of CH splits: all loads of a chunk are independent (one memory round trip), then the
  // chunk is folded into the running result with an online reference update.
  constexpr int CH = 4;
  Folded f = empty_folded();
  for (int s0 = first; s0 < nsplit; s0 += stride * CH) {
    float mv[CH], lv[CH];
    float4 ov[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int s = s0 + c * stride;
      mv[c] = -INFINITY;
      lv[c] = 0.f;
      ov[c] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (s < nsplit) {
        const size_t r = (size_t)s * rows + row;
        mv[c] = ws_m[r];
        lv[c] = ws_l[r];
        ov[c] = *(const float4*)(ws_o + r * D + c4 * 4);
      }
    }
    float cm = mv[0];
#pragma unroll
    for (int c = 1; c < CH; ++c) cm = fmaxf(cm, mv[c]);
    const float Mn = fmaxf(f.m2, cm);
    if (Mn == -INFINITY) continue;
    const float a = fast_exp2(f.m2 - Mn);
    f.o.x *= a; f.o.y *= a; f.o.z *= a; f.o.w *= a;
    f.l *= a;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const float w = fast_exp2(mv[c] - Mn);
      f.o.x = fmaf(ov[c].x, w, f.o.x);
      f.o.y = fmaf(ov[c].y, w, f.o.y);
      f.o.z = fmaf(ov[c].z, w, f.o.z);
      f.o.w = fmaf(ov[c].w, w, f.o.w);
      f.l = fmaf(lv[c], w, f.l);
    }
    f.m2 = Mn;
  }
  return f;
}

// Few splits: one thread per (row, 4 columns) walks the splits.
__global__ __launch_bounds__(256) void combine_kernel(const CombineParams p) {
  const int per_row = p.D / 4;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)p.rows * per_row) return;
  const size_t row = idx / per_row;
  const int c4 = (int)(idx % per_row);
  if (p.head_on != nullptr && p.head_on[row / p.Bq] == 0) return;
  Folded sel = empty_folded(), res = empty_folded();
  // chunks of four splits with all loads in flight (one memory round trip for up to four splits)
  if (p.ws_o != nullptr && p.nsplit > 0) sel = fold_strided(p.ws_o, p.ws_m, p.ws_l, p.nsplit, p.rows, row, p.D, c4, 0, 1);
  const bool have_res_set = p.ws_o2 != nullptr;
  if (have_res_set) res = fold_strided(p.ws_o2, p.ws_m2, p.ws_l2, p.nsplit, p.rows, row, p.D, c4, 0, 1);
  finish_row(p, sel, res, have_res_set, row, c4);
}

// Many splits: one workgroup per row; NSL = 256/(D/4) thread groups each fold every NSL-th split
// (fold_strided above), then one group folds the NSL results in fixed order.
__global__ __launch_bounds__(256) void combine_wide_kernel(const CombineParams p) {
  __shared__ Folded sh[2][256];
  const int per_row = p.D / 4, nsl = 256 / per_row;
  const int tid = threadIdx.x, sl = tid / per_row, c4 = tid % per_row;
  const size_t row = xcd_contiguous(blockIdx.x, gridDim.x);
  if (p.head_on != nullptr && p.head_on[row / p.Bq] == 0) return;   // workgroup-uniform
  const bool have_res_set = p.ws_o2 != nullptr;
  sh[0][tid] = fold_strided(p.ws_o, p.ws_m, p.ws_l, p.nsplit, p.rows, row, p.D, c4, sl, nsl);
  if (have_res_set) sh[1][tid] = fold_strided(p.ws_o2, p.ws_m2, p.ws_l2, p.nsplit, p.rows, row, p.D, c4, sl, nsl);
  __syncthreads();
  if (sl != 0) return;
  Folded sel = sh[0][c4], res = empty_folded();
  for (int j = 1; j < nsl; ++j) sel = fold_two(sel, sh[0][j * per_row + c4]);
  if (have_res_set) {
    res = sh[1][c4];
    for (int j = 1; j < nsl; ++j) res = fold_two(res, sh[1][j * per_row + c4]);
  }
  finish_row(p, sel, res, have_res_set, row, c4);
}

// ------------------------------------------------------------------------------ refresh fold
// Refresh step with a small block (at most kMaxInlineBlock keys): after the streaming pass over the
// prefix, ONE kernel folds the split partials (Eq. 5), writes the folded external partial to the
// caller's cache, computes the block-internal attention of its rows with plain FMAs (Eq. 7) and
// writes the Eq. 8-9 merge as the step's output.  Workgroup = kFoldRows rows of one query head
// (the block's K/V are staged in LDS once per workgroup); wavefront w owns row w for the
// attention part, all 256 threads share the split loads of every row.
__device__ __forceinline__ float4 load4(const void* base, size_t i, int is_bf16) {
  if (is_bf16) {
    const uint2 u = *(const uint2*)((const uint16_t*)base + i);
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                       __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u));
  }
  return *(const float4*)((const float*)base + i);
}
__device__ __forceinline__ float wave_max_f(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ float wave_sum_f(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

template <int D>
__global__ __launch_bounds__(256) void refresh_fold_kernel(const CombineParams p) {
  constexpr int RW = kFoldRows;
  static_assert(RW % 4 == 0 && RW <= 4, "block length is a multiple of RW: the value loop below steps by 4 keys; one wavefront per row");
  constexpr int per_row = D / 4, nsl = 256 / per_row;
  constexpr int ST = D + 4;                        // floats per K / V row in LDS: conflict-free 128-bit row reads
  constexpr int ES = D + 4;                        // folded external row: o[D], m2, l
  constexpr int NACC = D / 64;
  extern __shared__ __align__(16) float lds_f[];
  float* k_s = lds_f;                              // [Bq][ST]
  float* v_s = k_s + p.Bq * ST;                    // [Bq][ST]
  float* q_s = v_s + p.Bq * ST;                    // [RW][D]
  float* e_s = q_s + RW * D;                       // [RW][ES]
  Folded* sh = (Folded*)(e_s + RW * ES);           // [RW][256]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sl = tid / per_row, c4 = tid % per_row;
  const size_t row0 = (size_t)xcd_contiguous(blockIdx.x, gridDim.x) * RW;     // Bq % RW == 0: the RW rows belong to one query head

  // first CH splits of this thread for all RW rows: every load is issued before any is used, and the
  // block's K / V / q staging below runs while they are in flight
  {
    constexpr int CH = 4;
    float mv[RW][CH], lv[RW][CH];
    float4 ov[RW][CH];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int sp = sl + c * nsl;
        mv[r][c] = -INFINITY;
        lv[r][c] = 0.f;
        ov[r][c] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (sp < p.nsplit) {
          const size_t g = (size_t)sp * p.rows + row0 + r;
          mv[r][c] = p.ws_m[g];
          lv[r][c] = p.ws_l[g];
          ov[r][c] = *(const float4*)(p.ws_o + g * D + c4 * 4);
        }
      }
    // block K / V / q -> LDS.  All global loads of the staging are issued before the first LDS store
    // (a load-then-store loop would wait for every load in flight, the split loads included, on
    // each trip); chunks past the block's end are clamped to its last chunk and not stored.
    // (the head arithmetic needs integer divisions: it comes after the split loads have been issued)
    const int bh = (int)(row0 / p.Bq), b = bh / p.Hq, kvh = (bh % p.Hq) / p.G;
    const size_t kvbase = (size_t)(b * p.Hkv + kvh) * p.Bq * D;
    constexpr int NST = kMaxInlineBlock * per_row / 256;      // staging trips at the largest block
    const int nchunk = p.Bq * per_row;
    const size_t qoff = (row0 + (size_t)((tid % (RW * per_row)) / per_row)) * D + (tid % per_row) * 4;
    if (p.fin_bf16) {
      uint2 kr[NST], vr[NST];
#pragma unroll
      for (int it = 0; it < NST; ++it) {
        const int c = min(tid + 256 * it, nchunk - 1);
        const size_t g = kvbase + (size_t)(c / per_row) * D + (c % per_row) * 4;
        kr[it] = *(const uint2*)((const uint16_t*)p.blk_k + g);
        vr[it] = *(const uint2*)((const uint16_t*)p.blk_v + g);
      }
      const uint2 qr = *(const uint2*)((const uint16_t*)p.blk_q + qoff);
#pragma unroll
      for (int it = 0; it < NST; ++it) {
        const int c = tid + 256 * it;
        if (c < nchunk) {
          const int j = c / per_row, cc = c % per_row;
          *(float4*)(k_s + j * ST + cc * 4) = make_float4(__uint_as_float(kr[it].x << 16), __uint_as_float(kr[it].x & 0xffff0000u),
                                                          __uint_as_float(kr[it].y << 16), __uint_as_float(kr[it].y & 0xffff0000u));
          *(float4*)(v_s + j * ST + cc * 4) = make_float4(__uint_as_float(vr[it].x << 16), __uint_as_float(vr[it].x & 0xffff0000u),
                                                          __uint_as_float(vr[it].y << 16), __uint_as_float(vr[it].y & 0xffff0000u));
        }
      }
      if (tid < RW * per_row)
        *(float4*)(q_s + (tid / per_row) * D + (tid % per_row) * 4) =
            make_float4(__uint_as_float(qr.x << 16), __uint_as_float(qr.x & 0xffff0000u), __uint_as_float(qr.y << 16),
                        __uint_as_float(qr.y & 0xffff0000u));
    } else {
      float4 kr[NST], vr[NST];
#pragma unroll
      for (int it = 0; it < NST; ++it) {
        const int c = min(tid + 256 * it, nchunk - 1);
        const size_t g = kvbase + (size_t)(c / per_row) * D + (c % per_row) * 4;
        kr[it] = *(const float4*)((const float*)p.blk_k + g);
        vr[it] = *(const float4*)((const float*)p.blk_v + g);
      }
      const float4 qr = *(const float4*)((const float*)p.blk_q + qoff);
#pragma unroll
      for (int it = 0; it < NST; ++it) {
        const int c = tid + 256 * it;
        if (c < nchunk) {
          *(float4*)(k_s + (c / per_row) * ST + (c % per_row) * 4) = kr[it];
          *(float4*)(v_s + (c / per_row) * ST + (c % per_row) * 4) = vr[it];
        }
      }
      if (tid < RW * per_row) *(float4*)(q_s + (tid / per_row) * D + (tid % per_row) * 4) = qr;
    }
#pragma unroll
    for (int r = 0; r < RW; ++r) {
      Folded f = empty_folded();
      float cm = mv[r][0];
#pragma unroll
      for (int c = 1; c < CH; ++c) cm = fmaxf(cm, mv[r][c]);
      if (cm != -INFINITY) {
        f.m2 = cm;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const float w = fast_exp2(mv[r][c] - cm);
          f.o.x = fmaf(ov[r][c].x, w, f.o.x);
          f.o.y = fmaf(ov[r][c].y, w, f.o.y);
          f.o.z = fmaf(ov[r][c].z, w, f.o.z);
          f.o.w = fmaf(ov[r][c].w, w, f.o.w);
          f.l = fmaf(lv[r][c], w, f.l);
        }
      }
      if (p.nsplit > CH * nsl)     // more splits than one chunk per thread covers
        f = fold_two(f, fold_strided(p.ws_o, p.ws_m, p.ws_l, p.nsplit, p.rows, row0 + r, D, c4, sl + CH * nsl, nsl));
      sh[r * 256 + tid] = f;
    }
  }
  __syncthreads();

  const bool has_row = wave < RW;                  // wavefronts beyond the workgroup's rows only took part in the loads
  const size_t row = row0 + (has_row ? wave : 0);
  if (has_row && lane < per_row) {                 // finish this wavefront's row: fold the split groups in order
    Folded ext = sh[wave * 256 + lane];
    for (int j = 1; j < nsl; ++j) ext = fold_two(ext, sh[wave * 256 + j * per_row + lane]);
    emit(ext, p.o, p.m, p.lse, row, D, lane);
    *(float4*)(e_s + wave * ES + lane * 4) = ext.o;
    if (lane == 0) {
      e_s[wave * ES + D] = ext.m2;
      e_s[wave * ES + D + 1] = ext.l;
    }
  }
  // block-internal scores of the row: lane = key
  float s2 = -INFINITY;
  if (has_row && lane < p.Bq) {
    const float4* kr = (const float4*)(k_s + lane * ST);
    const float4* qr = (const float4*)(q_s + wave * D);
    float d = 0.f;
#pragma unroll 8
    for (int i = 0; i < D / 4; ++i) {
      const float4 a = kr[i], c = qr[i];
      d = fmaf(a.x, c.x, d);
      d = fmaf(a.y, c.y, d);
      d = fmaf(a.z, c.z, d);
      d = fmaf(a.w, c.w, d);
    }
    s2 = d * p.scale_log2;
  }
  const float mi = wave_max_f(s2);
  const float w = (lane < p.Bq) ? fast_exp2(s2 - mi) : 0.f;
  const float li = wave_sum_f(w);
  __syncthreads();                                 // the row's folded external statistics are in LDS
  if (!has_row) return;

  // value accumulation: lane owns columns lane, lane + 64; key j's weight is broadcast from lane j
  float acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i) acc[i] = 0.f;
  for (int j = 0; j < p.Bq; j += 4) {             // Bq % 4 == 0 on this path; four keys' LDS reads in flight per trip
    float pj[4], vv[4][NACC];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      pj[u] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w), j + u));
#pragma unroll
      for (int i = 0; i < NACC; ++i) vv[u][i] = v_s[(j + u) * ST + lane + 64 * i];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < NACC; ++i) acc[i] = fmaf(pj[u], vv[u][i], acc[i]);
  }
  // Eq. 8-9 against the folded external statistics of the row
  const float me = e_s[wave * ES + D], le = e_s[wave * ES + D + 1];
  const float M = fmaxf(me, mi);
  const float we = fast_exp2(me - M), wi = fast_exp2(mi - M);      // mi is finite (the block has at least one key)
  const float den = le * we + li * wi;
  const float inv = 1.f / den;
#pragma unroll
  for (int i = 0; i < NACC; ++i) {
    const float val = (e_s[wave * ES + lane + 64 * i] * we + acc[i] * wi) * inv;
    if (p.fin_bf16) ((uint16_t*)p.fin_out)[row * D + lane + 64 * i] = (uint16_t)bf16_rne(val);
    else ((float*)p.fin_out)[row * D + lane + 64 * i] = val;
  }
  if (p.fin_lse != nullptr && lane == 0) p.fin_lse[row] = (M + log2f(den)) * kLn2;
}

// ------------------------------------------------------------------------------ pooling
__device__ __forceinline__ float load_elem(const void* base, size_t i, int is_bf16) {
  if (is_bf16) {
    const uint32_t u = ((uint32_t)((const uint16_t*)base)[i]) << 16;
    return __uint_as_float(u);
  }
  return ((const float*)base)[i];
}

// grid (nblk, B*Hkv), 256 threads: column d = tid % D, token lane = tid / D (fp32 storage).
__global__ __launch_bounds__(256) void pool_keys_kernel(const PoolParams p) {
  __shared__ float red[256];
  const int c = blockIdx.x, bh = blockIdx.y;
  const int D = p.D, tid = threadIdx.x;
  const int d = tid % D, tl = tid / D, ntl = 256 / D;
  const int k0 = c * p.key_block, k1 = min(p.nkeys, k0 + p.key_block);
  float s = 0.f;
  for (int k = k0 + tl; k < k1; k += ntl) s += load_elem(p.k, ((size_t)bh * p.nkeys + k) * D + d, p.is_bf16);
  red[tid] = s;
  __syncthreads();
  if (tl == 0) {
    for (int j = 1; j < ntl; ++j) s += red[j * D + d];
    p.k_pooled[((size_t)bh * p.nblk + c) * D + d] = s / (float)(k1 - k0);
  }
}

// bf16 storage: 16-byte loads (8 columns per thread), D/8 threads per key row, 256/(D/8) rows in
// flight per step; the row lanes are folded through LDS in a fixed order.
template <int D>
__global__ __launch_bounds__(256) void pool_keys_bf16_kernel(const PoolParams p) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef const __attribute__((address_space(1))) u32x4* gptr128;
  constexpr int CPR = D / 8, NRL = 256 / CPR;
  __shared__ float red[NRL][D + 1];
  const int c = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x;
  const int col = tid % CPR, rl = tid / CPR;
  const int k0 = c * p.key_block, k1 = min(p.nkeys, k0 + p.key_block);
  const uint16_t* base = (const uint16_t*)p.k + (size_t)bh * p.nkeys * D + col * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int k = k0 + rl; k < k1; k += NRL) {
    const u32x4 u = *(gptr128)(base + (size_t)k * D);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      acc[2 * w] += __uint_as_float(u[w] << 16);
      acc[2 * w + 1] += __uint_as_float(u[w] & 0xffff0000u);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) red[rl][col * 8 + i] = acc[i];
  __syncthreads();
  if (tid < D) {
    float s = 0.f;
    for (int j = 0; j < NRL; ++j) s += red[j][tid];
    p.k_pooled[((size_t)bh * p.nblk + c) * D + tid] = s / (float)(k1 - k0);
  }
}

// ------------------------------------------------------------------------------ top-k
// Order-preserving map of a float onto uint32 (larger float <-> larger key).
__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sum of one int per thread over a 256-thread workgroup: shuffles inside each
// wavefront, wavefront totals through wtot[4] (two barriers; wtot may be reused afterwards).
__device__ __forceinline__ int block_exclusive_prefix(int v, int* wtot, int tid) {
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int dn = __shfl_up(inc, o, 64);
    if ((tid & 63) >= o) inc += dn;
  }
  __syncthreads();                      // earlier readers of wtot are done
  if ((tid & 63) == 63) wtot[tid >> 6] = inc;
  __syncthreads();
  int base = 0;
  for (int wv = 0; wv < (tid >> 6); ++wv) base += wtot[wv];
  return base + inc - v;
}

typedef uint32_t sel_u32x4 __attribute__((ext_vector_type(4)));

// Mean over the Bq rows of query head bh -> qbar[D] (LDS).  Thread = (row lane, 16-byte chunk of a row):
// up to eight row loads in flight per trip, per-lane sums in row order, then the row lanes meet through
// red[256 * 8] in lane order.  Ends with a barrier.
__device__ __forceinline__ void head_qbar(const void* q, int bh, int Bq, int D, int is_bf16, float* qbar,
                                          float* red, int tid) {
  const int E = is_bf16 ? 8 : 4, esz = is_bf16 ? 2 : 4;
  const int cpr = D / E, nrl = 256 / cpr, chunk = tid % cpr, rl = tid / cpr;
  const size_t rowbytes = (size_t)D * esz;
  const char* base = (const char*)q + (size_t)bh * Bq * rowbytes + (size_t)chunk * 16;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int r0 = rl; r0 < Bq; r0 += 8 * nrl) {
    sel_u32x4 x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = r0 + u * nrl;
      if (r < Bq) x[u] = *(const sel_u32x4*)(base + (size_t)r * rowbytes);
      else x[u] = sel_u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (is_bf16) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          acc[2 * w] += __uint_as_float(x[u][w] << 16);
          acc[2 * w + 1] += __uint_as_float(x[u][w] & 0xffff0000u);
        }
      } else {
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[w] += __uint_as_float(x[u][w]);
      }
    }
  }
  for (int i = 0; i < E; ++i) red[rl * D + chunk * E + i] = acc[i];
  __syncthreads();
  if (tid < D) {
    float t = 0.f;
    for (int j = 0; j < nrl; ++j) t += red[j * D + tid];
    qbar[tid] = t / (float)Bq;
  }
  __syncthreads();
}

// One 16-byte chunk of a pooled-key row against the same chunk of a mean query.
__device__ __forceinline__ float chunk_dot(const float4 a, const float4 q4) {
  return fmaf(a.w, q4.w, fmaf(a.z, q4.z, fmaf(a.y, q4.y, a.x * q4.x)));
}

// grid (B*Hq), 256 threads: qbar_out[bh][D] = mean query of the head (first kernel of the three-kernel selection).
__global__ __launch_bounds__(256) void head_qbar_kernel(const SelectParams p) {
  __shared__ float qbar[128];
  __shared__ float red[256 * 8];
  head_qbar(p.q, blockIdx.x, p.Bq, p.D, p.is_bf16, qbar, red, threadIdx.x);
  if ((int)threadIdx.x < p.D) p.qbar_ws[(size_t)blockIdx.x * p.D + threadIdx.x] = qbar[threadIdx.x];
}

// grid (ceil(nblk / rows per workgroup), B*Hkv), 256 threads: scores of a run of key blocks for the G heads of
// a KV group: every pooled row is read once for the whole group.  A wavefront instruction covers 64 / (D/4)
// rows; kScoreU of them are in flight; a row's partial sums meet by xor-shuffles inside its lane group (the
// same arithmetic, in the same order, as the one-kernel selection).
constexpr int kScoreU = 4;
__global__ __launch_bounds__(256) void block_scores_kernel(const SelectParams p) {
  extern __shared__ __align__(16) float qb[];              // [G][D]
  const int D = p.D, nblk = p.nblk, tid = threadIdx.x;
  const int bk = blockIdx.y, b = bk / p.Hkv, kvh = bk % p.Hkv;
  const int cpr = D / 4, rpw = 64 / cpr;
  const int lane = tid & 63, wave = tid >> 6, c = lane % cpr, rsub = lane / cpr;
  const int r_base = blockIdx.x * (4 * rpw * kScoreU) + wave * (rpw * kScoreU) + rsub;
  const float* kp = p.k_pooled + (size_t)bk * nblk * D;
  float4 a[kScoreU];
#pragma unroll
  for (int u = 0; u < kScoreU; ++u) {
    const int r = min(r_base + u * rpw, nblk - 1);         // clamped: in bounds, result discarded
    a[u] = *(const float4*)(kp + (size_t)r * D + 4 * c);
  }
  const float* qsrc = p.qbar_ws + (size_t)(b * p.Hq + kvh * p.G) * D;
  for (int i = tid; i < p.G * D; i += 256) qb[i] = qsrc[i];
  __syncthreads();
  for (int g = 0; g < p.G; ++g) {
    const float4 q4 = *(const float4*)(qb + g * D + 4 * c);
    float part[kScoreU];
#pragma unroll
    for (int u = 0; u < kScoreU; ++u) part[u] = chunk_dot(a[u], q4);
    for (int o = cpr / 2; o > 0; o >>= 1)
#pragma unroll
      for (int u = 0; u < kScoreU; ++u) part[u] += __shfl_xor(part[u], o, 64);
    float* dst = p.scores_ws + (size_t)(b * p.Hq + kvh * p.G + g) * nblk;
#pragma unroll
    for (int u = 0; u < kScoreU; ++u) {
      const int r = r_base + u * rpw;
      if (c == 0 && r < nblk) dst[r] = part[u];
    }
  }
}

// grid (B*Hq), 256 threads, dynamic LDS: qbar[D] | red[256 * 8] | key[nblk] | flag[nblk]
// Selection = the k largest scores, ties to the lower block index: the k-th largest key T is
// found by a 4-pass radix select over its bytes (256-bin LDS histogram of the keys that match the
// digits fixed so far), then blocks with key > T are taken plus the first k - count(key > T)
// blocks with key == T in index order.
__global__ __launch_bounds__(256) void select_topk_kernel(const SelectParams p) {
  extern __shared__ __align__(16) float lds[];
  float* qbar = lds;
  float* red = qbar + p.D;
  uint32_t* key = (uint32_t*)(red + 256 * 8);
  int* flag = (int*)(key + p.nblk);
  __shared__ int sel_digit, sel_rest, wtot[4];

  const int bh = blockIdx.x, b = bh / p.Hq, h = bh % p.Hq, kvh = h / p.G;
  const int D = p.D, tid = threadIdx.x, nblk = p.nblk;
  const int k = min(p.topk, nblk);

  if (p.rowmass != nullptr) {
    // score = attention mass of the block: mean over the head's rows of the per-row masses (fixed order)
    const float* rm = p.rowmass + (size_t)b * nblk * ((size_t)p.Hq * p.Bq) + (size_t)h * p.Bq;
    for (int c = tid; c < nblk; c += 256) {
      const float* r = rm + (size_t)c * ((size_t)p.Hq * p.Bq);
      float s = 0.f;
      int i = 0;
      if ((p.Bq & 3) == 0) {                   // 16-byte aligned rows: up to 32 masses per trip in eight wide loads
        for (; i < p.Bq; i += 32) {
          float4 x[8];
#pragma unroll
          for (int u = 0; u < 8; ++u)
            x[u] = (i + 4 * u < p.Bq) ? *(const float4*)(r + i + 4 * u) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
          for (int u = 0; u < 8; ++u) s += x[u].x, s += x[u].y, s += x[u].z, s += x[u].w;
        }
      }
      for (; i + 8 <= p.Bq; i += 8) {          // eight independent loads per trip, summed in index order
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = r[i + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += x[u];
      }
      for (; i < p.Bq; ++i) s += r[i];
      s /= (float)p.Bq;
      key[c] = order_key(s);
      if (p.score_out != nullptr) p.score_out[(size_t)bh * nblk + c] = s;
    }
  } else if (p.scores_ws != nullptr) {
    // scores already computed by block_scores_kernel
    const float* sc = p.scores_ws + (size_t)bh * nblk;
    for (int c = tid; c < nblk; c += 256) key[c] = order_key(sc[c]);
  } else {
    head_qbar(p.q, bh, p.Bq, D, p.is_bf16, qbar, red, tid);
    // score = qbar . pooled key of the block.  A wavefront reads 64 consecutive 16-byte chunks per
    // instruction (2 rows at D = 128, 4 at D = 64); a row's partial sums meet by xor-shuffles inside
    // its lane group; 8 such loads are in flight per wavefront.
    const float* kp = p.k_pooled + (size_t)(b * p.Hkv + kvh) * nblk * D;
    const int cpr = D / 4, rpw = 64 / cpr;            // chunks per row, rows per wavefront instruction
    const int lane = tid & 63, wave = tid >> 6;
    const int c = lane % cpr, rsub = lane / cpr;
    const float4 q4 = *(const float4*)(qbar + 4 * c);
    constexpr int U = 8;
    for (int r0 = wave * rpw; r0 < nblk; r0 += 4 * rpw * U) {
      float part[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int r = min(r0 + u * 4 * rpw + rsub, nblk - 1);       // clamped: in bounds, result discarded
        const float4 a = *(const float4*)(kp + (size_t)r * D + 4 * c);
        part[u] = chunk_dot(a, q4);
      }
      for (int o = cpr / 2; o > 0; o >>= 1)
#pragma unroll
        for (int u = 0; u < U; ++u) part[u] += __shfl_xor(part[u], o, 64);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int r = r0 + u * 4 * rpw + rsub;
        if (c == 0 && r < nblk) key[r] = order_key(part[u]);
      }
    }
  }
  __syncthreads();

  // radix select of the k-th largest key, most significant byte first
  uint32_t T = 0u;
  int rest = k;                                   // how many keys with the fixed prefix are still to take
  int* hist = (int*)red;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t himask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    hist[tid] = 0;
    __syncthreads();
    for (int cidx = tid; cidx < nblk; cidx += 256) {
      const uint32_t kc = key[cidx];
      if ((kc & himask) == (T & himask)) atomicAdd(&hist[(kc >> shift) & 0xffu], 1);
    }
    __syncthreads();
    // thread t: keys (with the prefix) whose digit is >= t, and > t: suffix sums over the 256 bins,
    // by shuffles inside each wavefront plus the totals of the wavefronts above
    const int mine_h = hist[tid];
    int ge = mine_h;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_down(ge, o, 64);
      if ((tid & 63) + o < 64) ge += up;
    }
    if ((tid & 63) == 0) wtot[tid >> 6] = ge;
    __syncthreads();
    for (int wv = (tid >> 6) + 1; wv < 4; ++wv) ge += wtot[wv];
    const int gt = ge - mine_h;
    if (ge >= rest && gt < rest) {               // exactly one digit qualifies (rest >= 1)
      sel_digit = tid;
      sel_rest = rest - gt;
    }
    __syncthreads();
    T |= (uint32_t)sel_digit << shift;
    rest = sel_rest;
    __syncthreads();
  }
  // ties with the k-th key to take, lowest index first
  const int need_eq = rest;

  // ascending passes over contiguous chunks: thread t owns blocks [t*per, (t+1)*per)
  const int per = (nblk + 255) / 256;
  const int c0 = min(nblk, tid * per), c1 = min(nblk, c0 + per);
  int mine = 0;
  for (int c = c0; c < c1; ++c) mine += key[c] == T;
  int eq_before = block_exclusive_prefix(mine, wtot, tid);
  mine = 0;
  for (int c = c0; c < c1; ++c) {
    const uint32_t kc = key[c];
    int f = kc > T;
    if (kc == T) f = (eq_before++ < need_eq);
    flag[c] = f;
    mine += f;
  }
  int pos = block_exclusive_prefix(mine, wtot, tid);
  int32_t* out = p.sel_idx + (size_t)bh * p.topk;
  for (int c = c0; c < c1; ++c)
    if (flag[c]) out[pos++] = c;
  for (int j = k + tid; j < p.topk; j += 256) out[j] = -1;
}

// ------------------------------------------------------------------------------ masks + union
// grid (B*Hkv), 256 threads, dynamic LDS: mask[nblk]
__global__ __launch_bounds__(256) void build_masks_kernel(const MaskParams p) {
  extern __shared__ __align__(16) uint32_t lmask[];
  __shared__ int wtot[4];
  const int bk = blockIdx.x, b = bk / p.Hkv, kvh = bk % p.Hkv;
  const int tid = threadIdx.x, nblk = p.nblk;
  for (int c = tid; c < nblk; c += 256) lmask[c] = 0u;
  __syncthreads();
  if (p.sel_idx != nullptr) {
    const int n = p.G * p.topk;
    const int32_t* base = p.sel_idx + (size_t)(b * p.Hq + kvh * p.G) * p.topk;
    // four selection entries per thread and trip, loaded before any is used (one memory round trip per trip)
    for (int i0 = tid; i0 < n; i0 += 4 * 256) {
      int c[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + 256 * u;
        c[u] = (i < n) ? base[i] : -1;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + 256 * u;
        if (c[u] >= 0 && c[u] < nblk) atomicOr(&lmask[c[u]], 1u << (i / p.topk));
      }
    }
  }
  __syncthreads();
  const int per = (nblk + 255) / 256;
  const int c0 = min(nblk, tid * per), c1 = min(nblk, c0 + per);
  int mine = 0;
  for (int c = c0; c < c1; ++c) {
    const uint32_t m = lmask[c];
    p.blk_mask[(size_t)bk * nblk + c] = m;
    mine += (m != 0u);
  }
  int pos = block_exclusive_prefix(mine, wtot, tid);
  int32_t* list = p.union_list + (size_t)bk * nblk;
  uint32_t* lm = p.union_mask + (size_t)bk * nblk;
  for (int c = c0; c < c1; ++c)
    if (lmask[c] != 0u) {
      list[pos] = c;
      lm[pos] = lmask[c];
      ++pos;
    }
  if (tid == 255) p.union_cnt[bk] = pos;
}

// ------------------------------------------------------------------------------ similarity
// Mean over a head's rows of the cosine similarity between two partials' output rows.  The
// normalised output A = o * e^{m-lse} is o times a positive scalar, so cos(A_a, A_b) = cos(o_a, o_b).
// grid (B*Hq), 256 threads: wavefront w takes rows w, w+4, ...; lanes stride the columns.
__global__ __launch_bounds__(256) void head_similarity_kernel(const float* __restrict__ oa, const float* __restrict__ ob,
                                                              float* __restrict__ sim, int Bq, int D) {
  __shared__ float part[4];
  const int bh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float acc = 0.f;
  for (int r = wave; r < Bq; r += 4) {
    const float* a = oa + ((size_t)bh * Bq + r) * D;
    const float* b = ob + ((size_t)bh * Bq + r) * D;
    float ab = 0.f, aa = 0.f, bb = 0.f;
    for (int d = lane; d < D; d += 64) {
      const float x = a[d], y = b[d];
      ab = fmaf(x, y, ab);
      aa = fmaf(x, x, aa);
      bb = fmaf(y, y, bb);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      ab += __shfl_xor(ab, o, 64);
      aa += __shfl_xor(aa, o, 64);
      bb += __shfl_xor(bb, o, 64);
    }
    const float den = sqrtf(aa) * sqrtf(bb);
    acc += den > 0.f ? ab / den : 0.f;       // a zero row (empty key set) counts as similarity 0
  }
  if (lane == 0) part[wave] = acc;
  __syncthreads();
  if (tid == 0) sim[bh] = (part[0] + part[1] + part[2] + part[3]) / (float)Bq;
}

}  // namespace

// order[r] = index of the sequence with the r-th longest prefix (ties: lower index first).  Rank by
// counting: B is a batch size, so B^2 comparisons are cheap; the lengths are staged through LDS in
// chunks of 256 so that the kernel is one memory round trip per chunk, not one per comparison.
__global__ __launch_bounds__(256) void seq_order_kernel(const int32_t* __restrict__ lens, int32_t* __restrict__ order, int B) {
  __shared__ int chunk[256];
  const int i = blockIdx.x * 256 + threadIdx.x;
  const int li = (i < B) ? lens[i] : 0;
  int rank = 0;
  for (int j0 = 0; j0 < B; j0 += 256) {
    const int j = j0 + threadIdx.x;
    __syncthreads();
    chunk[threadIdx.x] = (j < B) ? lens[j] : 0;
    __syncthreads();
    const int n = min(256, B - j0);
    for (int t = 0; t < n; ++t) {
      const int lj = chunk[t];
      rank += (lj > li || (lj == li && j0 + t < i)) ? 1 : 0;
    }
  }
  if (i < B) order[rank] = i;
}

hipError_t launch_seq_order(const int32_t* prefix_lens, int32_t* seq_order, int B, hipStream_t s) {
  hipLaunchKernelGGL(seq_order_kernel, dim3((B + 255) / 256), dim3(256), 0, s, prefix_lens, seq_order, B);
  return hipGetLastError();
}

hipError_t launch_head_similarity(const float* o_a, const float* o_b, float* sim, int BH, int Bq, int D, hipStream_t s) {
  hipLaunchKernelGGL(head_similarity_kernel, dim3(BH), dim3(256), 0, s, o_a, o_b, sim, Bq, D);
  return hipGetLastError();
}

hipError_t launch_combine(const CombineParams& p, hipStream_t s) {
  const size_t n = (size_t)p.rows * (p.D / 4);
  if (n == 0) return hipSuccess;
  if (p.nsplit >= 8 && p.ws_o != nullptr)
    hipLaunchKernelGGL(combine_wide_kernel, dim3((unsigned)p.rows), dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_pool_keys(const PoolParams& p, hipStream_t s) {
  if (p.nblk == 0 || p.BH == 0) return hipSuccess;
  const dim3 grid(p.nblk, p.BH), block(256);
  if (p.is_bf16 && p.D == 128) hipLaunchKernelGGL(pool_keys_bf16_kernel<128>, grid, block, 0, s, p);
  else if (p.is_bf16 && p.D == 64) hipLaunchKernelGGL(pool_keys_bf16_kernel<64>, grid, block, 0, s, p);
  else hipLaunchKernelGGL(pool_keys_kernel, grid, block, 0, s, p);
  return hipGetLastError();
}

hipError_t launch_refresh_fold(const CombineParams& p, hipStream_t s) {
  if (p.rows == 0) return hipSuccess;
  if (p.Bq > kMaxInlineBlock || p.Bq % kFoldRows != 0 || p.blk_q == nullptr || p.nsplit < 1) return hipErrorInvalidValue;
  const size_t lds = ((size_t)2 * p.Bq * (p.D + 4) + kFoldRows * p.D + kFoldRows * (p.D + 4)) * sizeof(float) +
                     (size_t)kFoldRows * 256 * sizeof(Folded);
  static LdsLimit lim64, lim128;
  hipError_t e = p.D == 64 ? raise_lds_limit(refresh_fold_kernel<64>, lds, lim64, kLdsLimitMax) : raise_lds_limit(refresh_fold_kernel<128>, lds, lim128, kLdsLimitMax);
  if (e != hipSuccess) return e;
  const dim3 grid((unsigned)(p.rows / kFoldRows));
  if (p.D == 64) hipLaunchKernelGGL(refresh_fold_kernel<64>, grid, dim3(256), lds, s, p);
  else hipLaunchKernelGGL(refresh_fold_kernel<128>, grid, dim3(256), lds, s, p);
  return hipGetLastError();
}

hipError_t launch_select_topk(const SelectParams& p, hipStream_t s) {
  static LdsLimit lim;
  const size_t lds = (size_t)(p.D + 256 * 8 + 2 * p.nblk) * 4;
  hipError_t e = raise_lds_limit(select_topk_kernel, lds, lim, kLdsLimitMax);
  if (e != hipSuccess) return e;
  if (p.scores_ws != nullptr && p.rowmass == nullptr && p.nblk > 0) {
    // three kernels: mean queries, block scores spread over the whole chip, then the selection proper
    hipLaunchKernelGGL(head_qbar_kernel, dim3(p.B * p.Hq), dim3(256), 0, s, p);
    const int rows_per_wg = 4 * (64 / (p.D / 4)) * kScoreU;
    const dim3 grid((unsigned)((p.nblk + rows_per_wg - 1) / rows_per_wg), (unsigned)(p.B * p.Hkv));
    hipLaunchKernelGGL(block_scores_kernel, grid, dim3(256), (size_t)p.G * p.D * sizeof(float), s, p);
  }
  hipLaunchKernelGGL(select_topk_kernel, dim3(p.B * p.Hq), dim3(256), lds, s, p);
  return hipGetLastError();
}

hipError_t launch_build_masks(const MaskParams& p, hipStream_t s) {
  static LdsLimit lim;
  const size_t lds = (size_t)p.nblk * 4;
  hipError_t e = raise_lds_limit(build_masks_kernel, lds, lim, kLdsLimitMax);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(build_masks_kernel, dim3(p.B * p.Hkv), dim3(256), lds, s, p);
  return hipGetLastError();
}

}  // namespace fb
