// fp32 attention pass for gfx950: plain-FMA scores, wavefront-shuffle softmax statistics.
//
// Computes the per-row statistics of Eq. 3-4/6 (arxiv 2602.05305, Section 4.2) over a key
// range, for storage type float.  This is the exactness path (max-abs 1e-5 against a float64
// reference): scores are fp32 FMA chains, the running maximum is exact, and every reduction
// has a fixed order, so results are bit-reproducible.
//
// Work decomposition: one workgroup = 4 wavefronts = 4 consecutive query rows of one query
// head; grid = (row chunks, batch*Hq, splits).  Per 64-key tile the workgroup stages K in LDS
// (row stride D+4 floats: conflict-free 128-bit reads), lane j of each wavefront scores key j
// against its wavefront's query row, max/sum go through 6-step xor shuffles, and the value
// accumulation has lanes own output columns (lane, lane+64) with p_j broadcast by readlane
// while V rows are read coalesced from global memory (L1/L2 serve the 4 rows' re-reads).
#include "fb_kernels.h"

namespace fb {
namespace {

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

template <int NACC>
struct RowState {
  float m, l;
  float acc[NACC];
  __device__ __forceinline__ void init() {
    m = -INFINITY;
    l = 0.f;
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = 0.f;
  }
};

// One online-softmax update of a row's state with the 64 scores held one per lane
// (log2 domain; -inf marks keys outside the set).
template <int D, int NACC>
__device__ __forceinline__ void row_update(RowState<NACC>& st, float s, const float* __restrict__ V,
                                           int k0, int nvalid, int lane) {
  const float tmax = wave_max(s);
  const float m_new = fmaxf(st.m, tmax);
  const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
  const float p = exp2f(s - m_use);
  const float alpha = exp2f(st.m - m_use);
  st.l = st.l * alpha + wave_sum(p);
#pragma unroll
  for (int i = 0; i < NACC; ++i) st.acc[i] *= alpha;
  const float* vrow = V + (size_t)k0 * D + lane;
  for (int j = 0; j < nvalid; ++j) {
    const float pj = __shfl(p, j, 64);
#pragma unroll
    for (int i = 0; i < NACC; ++i) st.acc[i] = fmaf(pj, vrow[(size_t)j * D + 64 * i], st.acc[i]);
  }
  st.m = m_new;
}

template <int D, int MODE>
__global__ __launch_bounds__(256) void attn_f32_kernel(const PassParams p) {
  constexpr int KSTR = D + 4;
  constexpr int NACC = D / 64;
  __shared__ __align__(16) float Ks[kKeyTile * KSTR];
  __shared__ __align__(16) float Qs[4 * D];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x;
  const int bh = blockIdx.y;
  int b = bh / p.Hq;
  const int h = bh % p.Hq;
  if constexpr (MODE == kPassDensePaged) {
    if (p.seq_order != nullptr) b = p.seq_order[b];
  }
  const int kvh = h / p.G, g = h % p.G;
  const int split = blockIdx.z;
  const int row = chunk * 4 + wave;
  const bool valid = row < p.Bq;
  if constexpr (MODE == kPassDenseHeads) {
    if (p.head_on[bh] == 0) return;     // workgroup-uniform: this head keeps its cached partial
  }
  int nkeys = p.nkeys;
  if constexpr (MODE == kPassDensePaged) nkeys = min(p.nkeys, max(0, p.prefix_lens[b]));   // this sequence's prefix
  const int bk = b * p.Hkv + kvh;
  // fused refresh pass: the workgroups of split index nsplit take the block's own keys
  const bool own_block = (MODE == kPassRefreshFused) && (split == p.nsplit);
  if (own_block) nkeys = p.Bq;

  const float* __restrict__ Q = (const float*)p.q + (size_t)(b * p.Hq + h) * p.Bq * D;
  // contiguous cache: this KV head's [nkeys, D] slab; paged cache: the pool (tiles add their page offset)
  const float* __restrict__ K = (const float*)p.k + ((MODE == kPassDensePaged) ? (size_t)0 : (size_t)bk * nkeys * D);
  const float* __restrict__ V = (const float*)p.v + ((MODE == kPassDensePaged) ? (size_t)0 : (size_t)bk * nkeys * D);
  if (own_block) {
    K = (const float*)p.k2 + (size_t)bk * nkeys * D;
    V = (const float*)p.v2 + (size_t)bk * nkeys * D;
  }

  for (int i = tid; i < 4 * D; i += 256) {
    const int r = chunk * 4 + i / D;
    Qs[i] = (r < p.Bq) ? Q[(size_t)r * D + (i % D)] : 0.f;
  }

  // tile list of this workgroup
  int tpb = 1, total;
  if constexpr (MODE == kPassSparseReuse) {
    tpb = p.key_block / kKeyTile;
    total = p.union_cnt[bk] * tpb;
  } else {
    total = (nkeys + kKeyTile - 1) / kKeyTile;
  }
  TileRange tr = split_range(total, p.nsplit, split);
  if (own_block) tr = TileRange{0, total};

  RowState<NACC> sel, res;   // res only used by the sparse refresh pass
  sel.init();
  res.init();

  for (int e = tr.begin; e < tr.end; ++e) {
    int k0;
    bool is_sel = true;
    if constexpr (MODE == kPassSparseReuse) {
      const int blk = p.union_list[(size_t)bk * p.nblk + e / tpb];
      k0 = blk * p.key_block + kKeyTile * (e % tpb);
      is_sel = (p.blk_mask[(size_t)bk * p.nblk + blk] >> g) & 1u;
      if (!is_sel || k0 >= nkeys) continue;   // uniform over the workgroup
    } else {
      k0 = e * kKeyTile;
      if constexpr (MODE == kPassSparseRefresh)
        is_sel = (p.blk_mask[(size_t)bk * p.nblk + k0 / p.key_block] >> g) & 1u;
    }
    const float* Kt = K;
    const float* Vt = V;
    if constexpr (MODE == kPassDensePaged) {
      // rebase so that key index k0 + r addresses row (k0 % page_size) + r of this head's slab of the page
      const long long page = min(max(p.block_table[(size_t)b * p.max_pages + k0 / p.page_size], 0), p.num_pages - 1);
      const long long off = ((page * p.Hkv + kvh) * p.page_size + (k0 % p.page_size) - k0) * D;
      Kt = K + off;
      Vt = V + off;
    }
    __syncthreads();   // all wavefronts are done with the previous K tile (and Qs is written)
    for (int c = tid; c < kKeyTile * (D / 4); c += 256) {
      const int r = c / (D / 4), c4 = c % (D / 4);
      const int key = k0 + r;
      float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
      if (key < nkeys) val = *(const float4*)(Kt + (size_t)key * D + c4 * 4);
      *(float4*)(Ks + r * KSTR + c4 * 4) = val;
    }
    __syncthreads();
    if (valid) {
      const float4* kr = (const float4*)(Ks + lane * KSTR);
      const float4* qr = (const float4*)(Qs + wave * D);
      float s = 0.f;
#pragma unroll 8
      for (int i = 0; i < D / 4; ++i) {
        const float4 a = kr[i], c = qr[i];
        s = fmaf(a.x, c.x, s);
        s = fmaf(a.y, c.y, s);
        s = fmaf(a.z, c.z, s);
        s = fmaf(a.w, c.w, s);
      }
      s *= p.scale_log2;
      if (k0 + lane >= nkeys) s = -INFINITY;
      const int nvalid = min(kKeyTile, nkeys - k0);
      if (MODE == kPassSparseRefresh && !is_sel)
        row_update<D, NACC>(res, s, Vt, k0, nvalid, lane);
      else
        row_update<D, NACC>(sel, s, Vt, k0, nvalid, lane);
    }
  }

  if (!valid) return;
  const size_t grow = (size_t)(b * p.Hq + h) * p.Bq + row;
  if constexpr (MODE == kPassInternal) {
    // Eq. 8-9 with the cached pair expressed through (o, m, lse): A_out e^{L_out-M} = o e^{m-M}.
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    float me2 = -INFINITY, le = 0.f;
    if (p.ext_o != nullptr) {
      const float me = p.ext_m[grow], lse = p.ext_lse[grow];
      if (lse != -INFINITY) {
        me2 = me * kLog2e;
        le = exp2f((lse - me) * kLog2e);
      }
    }
    const float M2 = fmaxf(me2, sel.m);
    const float Mu = (M2 == -INFINITY) ? 0.f : M2;
    const float we = exp2f(me2 - Mu), wi = exp2f(sel.m - Mu);
    const float den = le * we + sel.l * wi;
    const float inv = den > 0.f ? 1.f / den : 0.f;
    float* out = (float*)p.out + grow * D;
#pragma unroll
    for (int i = 0; i < NACC; ++i) {
      float num = sel.acc[i] * wi;
      if (le > 0.f) num = fmaf(p.ext_o[grow * D + lane + 64 * i], we, num);
      out[lane + 64 * i] = num * inv;
    }
    if (p.lse_out != nullptr && lane == 0)
      p.lse_out[grow] = den > 0.f ? (M2 + log2f(den)) * kLn2 : -INFINITY;
  } else {
    if constexpr (MODE == kPassDense || MODE == kPassDenseHeads || MODE == kPassDensePaged) {
      if (p.direct) {
        // single split: this is the final partial; same unit conversion as the split combine
        constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
        float m_nat = -INFINITY, L = -INFINITY, adj = 0.f;
        if (sel.l > 0.f) {
          m_nat = sel.m * kLn2;
          adj = exp2f(sel.m - m_nat * kLog2e);
          L = (sel.m + log2f(sel.l)) * kLn2;
        }
#pragma unroll
        for (int i = 0; i < NACC; ++i) p.ws_o[grow * D + lane + 64 * i] = sel.acc[i] * adj;
        if (lane == 0) {
          p.ws_m[grow] = m_nat;
          p.ws_l[grow] = L;
        }
        return;
      }
    }
    const size_t rows_total = (size_t)p.B * p.Hq * p.Bq;
    const size_t wrow = (own_block ? (size_t)0 : (size_t)split * rows_total) + grow;
    float* __restrict__ w_o = own_block ? p.ws_o2 : p.ws_o;
    float* __restrict__ w_m = own_block ? p.ws_m2 : p.ws_m;
    float* __restrict__ w_l = own_block ? p.ws_l2 : p.ws_l;
#pragma unroll
    for (int i = 0; i < NACC; ++i) w_o[wrow * D + lane + 64 * i] = sel.acc[i];
    if (lane == 0) {
      w_m[wrow] = sel.m;
      w_l[wrow] = sel.l;
    }
    if constexpr (MODE == kPassSparseRefresh) {
#pragma unroll
      for (int i = 0; i < NACC; ++i) p.ws_o2[wrow * D + lane + 64 * i] = res.acc[i];
      if (lane == 0) {
        p.ws_m2[wrow] = res.m;
        p.ws_l2[wrow] = res.l;
      }
    }
  }
}

// Attention mass per (query row, key block): sum over the block's keys of exp(s - lse), fp32 storage.
// Same work decomposition as the attention pass (one wavefront per query row, lane j scores key j).
template <int D>
__global__ __launch_bounds__(256) void block_mass_f32_kernel(const MassParams p) {
  constexpr int KSTR = D + 4;
  constexpr float kLog2e = 1.4426950408889634f;
  __shared__ __align__(16) float Ks[kKeyTile * KSTR];
  __shared__ __align__(16) float Qs[4 * D];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x, bh = blockIdx.y, split = blockIdx.z;
  const int b = bh / p.Hq, h = bh % p.Hq, kvh = h / p.G;
  const int row = chunk * 4 + wave, nkeys = p.nkeys;
  const bool valid = row < p.Bq;
  const float* __restrict__ Q = (const float*)p.q + (size_t)bh * p.Bq * D;
  const float* __restrict__ K = (const float*)p.k + (size_t)(b * p.Hkv + kvh) * nkeys * D;
  for (int i = tid; i < 4 * D; i += 256) {
    const int r = chunk * 4 + i / D;
    Qs[i] = (r < p.Bq) ? Q[(size_t)r * D + (i % D)] : 0.f;
  }
  const float lse = valid ? p.lse[(size_t)bh * p.Bq + row] : 0.f;
  const bool live = lse != -INFINITY;
  const float lse2 = live ? lse * kLog2e : 0.f;
  const int tpb = p.key_block / kKeyTile;
  const TileRange br = split_range(p.nblk, p.nsplit, split);
  const int t0 = br.begin * tpb, t1 = min(br.end * tpb, (nkeys + kKeyTile - 1) / kKeyTile);
  float acc = 0.f;
  for (int t = t0; t < t1; ++t) {
    const int k0 = t * kKeyTile;
    __syncthreads();
    for (int c = tid; c < kKeyTile * (D / 4); c += 256) {
      const int r = c / (D / 4), c4 = c % (D / 4);
      float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
      if (k0 + r < nkeys) val = *(const float4*)(K + (size_t)(k0 + r) * D + c4 * 4);
      *(float4*)(Ks + r * KSTR + c4 * 4) = val;
    }
    __syncthreads();
    const float4* kr = (const float4*)(Ks + lane * KSTR);
    const float4* qr = (const float4*)(Qs + wave * D);
    float s = 0.f;
#pragma unroll 8
    for (int i = 0; i < D / 4; ++i) {
      const float4 a = kr[i], c = qr[i];
      s = fmaf(a.x, c.x, s);
      s = fmaf(a.y, c.y, s);
      s = fmaf(a.z, c.z, s);
      s = fmaf(a.w, c.w, s);
    }
    acc += (k0 + lane < nkeys) ? exp2f(s * p.scale_log2 - lse2) : 0.f;
    if ((t + 1) % tpb == 0 || t + 1 == t1) {
      const float tot = wave_sum(acc);
      if (valid && lane == 0)
        p.rowmass[((size_t)b * p.nblk + t / tpb) * ((size_t)p.Hq * p.Bq) + (size_t)h * p.Bq + row] = live ? tot : 0.f;
      acc = 0.f;
    }
  }
}

template <int D>
hipError_t launch_d(const PassParams& p, PassMode mode, hipStream_t s) {
  const dim3 grid((p.Bq + kRowsPerWgF32 - 1) / kRowsPerWgF32, p.B * p.Hq, p.nsplit + (mode == kPassRefreshFused ? 1 : 0));
  const dim3 block(256);
  switch (mode) {
    case kPassDense: hipLaunchKernelGGL((attn_f32_kernel<D, kPassDense>), grid, block, 0, s, p); break;
    case kPassInternal: hipLaunchKernelGGL((attn_f32_kernel<D, kPassInternal>), grid, block, 0, s, p); break;
    case kPassSparseRefresh: hipLaunchKernelGGL((attn_f32_kernel<D, kPassSparseRefresh>), grid, block, 0, s, p); break;
    case kPassSparseReuse: hipLaunchKernelGGL((attn_f32_kernel<D, kPassSparseReuse>), grid, block, 0, s, p); break;
    case kPassDenseHeads: hipLaunchKernelGGL((attn_f32_kernel<D, kPassDenseHeads>), grid, block, 0, s, p); break;
    case kPassDensePaged: hipLaunchKernelGGL((attn_f32_kernel<D, kPassDensePaged>), grid, block, 0, s, p); break;
    case kPassRefreshFused: hipLaunchKernelGGL((attn_f32_kernel<D, kPassRefreshFused>), grid, block, 0, s, p); break;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_block_mass_f32(const MassParams& p, int D, hipStream_t s) {
  const dim3 grid((p.Bq + kRowsPerWgF32 - 1) / kRowsPerWgF32, p.B * p.Hq, p.nsplit);
  if (D == 64) hipLaunchKernelGGL(block_mass_f32_kernel<64>, grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL(block_mass_f32_kernel<128>, grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_attn_f32(const PassParams& p, int D, PassMode mode, hipStream_t s) {
  if (D == 64) return launch_d<64>(p, mode, s);
  return launch_d<128>(p, mode, s);
}

}  // namespace fb
