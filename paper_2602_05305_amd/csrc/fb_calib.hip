// Calibration kernels for the benchmark (libfbcalib.so): what this GPU sustains on the two resources the
// attention passes are priced against, measured with kernels that do nothing else.  Not part of the product
// library and not declared in include/flashblock.h; bench.py loads it next to libflashblock.so and reports
// its numbers beside the nominal peaks.
//   fbc_read_vgpr   every workgroup streams a contiguous chunk with 16-byte loads into registers
//   fbc_read_lds    the same stream through direct-to-LDS loads into a ring of stages (the data path of the
//                   streaming attention pass, with the arithmetic taken out)
//   fbc_copy        plain device copy of a known size (scale factor of the profiler's HBM byte counters)
//   fbc_mfma        back-to-back v_mfma_f32_32x32x16_bf16 on independent accumulators, no memory traffic; with operands
//                   that change from MFMA to MFMA (what a real contraction presents) or with one constant pair
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* gptr128;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int UNROLL>
__global__ __launch_bounds__(256) void read_vgpr_kernel(const u32x4* __restrict__ src, size_t chunks_per_wg,
                                                        uint32_t* __restrict__ sink) {
  gptr128 p = (gptr128)(src + (size_t)blockIdx.x * chunks_per_wg);
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (size_t i = threadIdx.x; i < chunks_per_wg; i += 256 * UNROLL) {
    u32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) v[u] = p[i + u * 256];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) acc ^= v[u];
  }
  // never true for the benchmark's data; keeps the loads alive
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;
}

// One 16-byte direct-to-LDS load per lane: the wavefront's 64 chunks land contiguously at lds_base.
__device__ __forceinline__ void lds_load16(const void* gaddr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(gaddr), "s"(lds_base)
               : "memory", "m0");
}

constexpr int kStageBytes = 32768;     // one 64-key K+V tile at head_dim 128
constexpr int kRingThreads = 512;
constexpr int kLoadsPerStage = kStageBytes / (kRingThreads * 16);   // 4 loads per lane per stage

// DEPTH stages in flight per workgroup.  Every wavefront waits for its own loads of the oldest stage, the
// workgroup meets at a barrier (as a consumer of the stage would require), and the stage is refilled.
template <int DEPTH>
__global__ __launch_bounds__(kRingThreads, 1) void read_lds_kernel(const unsigned char* __restrict__ src,
                                                                   int stages_per_wg, uint32_t* __restrict__ sink) {
  extern __shared__ __align__(16) unsigned char ring[];
  const unsigned char* p = src + (size_t)blockIdx.x * stages_per_wg * kStageBytes + threadIdx.x * 16;
  // wavefront-uniform values, said so explicitly: the LDS base of a direct-to-LDS load travels in M0
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t ring_base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)ring);
  auto issue = [&](int t) {
    const uint32_t lbase = ring_base + (uint32_t)(t % DEPTH) * kStageBytes + wave * 1024;
#pragma unroll
    for (int j = 0; j < kLoadsPerStage; ++j)
      lds_load16(p + (size_t)t * kStageBytes + j * (kRingThreads * 16), lbase + j * (kRingThreads * 16));
  };
  for (int t = 0; t < DEPTH - 1 && t < stages_per_wg; ++t) issue(t);
  for (int t = 0; t < stages_per_wg; ++t) {
    // loads of the DEPTH-2 younger stages may stay in flight
    if (t + DEPTH - 1 <= stages_per_wg) {
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DEPTH - 2) * kLoadsPerStage) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    if (t + DEPTH - 1 < stages_per_wg) issue(t + DEPTH - 1);
  }
  if (ring[threadIdx.x * 16] == 0x5a && ring[threadIdx.x] == 0xa5 && src[0] == 0x77) sink[0] = 1u;
}

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = ((gptr128)src)[i];
}

// Each wavefront: iters x 4 MFMAs on four independent accumulators (no dependency between neighbours).  The operands
// rotate through four register sets of pseudo-random bf16 values per lane, so that the multipliers see changing bits as
// they do on real data (with one constant operand pair the part draws less power and holds a higher clock than any real
// contraction does).
template <bool VARY>
__global__ __launch_bounds__(256) void mfma_kernel(int iters, float* __restrict__ sink) {
  bf16x8 a[4], b[4];
  uint32_t h = (uint32_t)(blockIdx.x * 256 + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      h = h * 1664525u + 1013904223u;
      a[k][i] = (__bf16)(((float)(h >> 8) * (1.0f / 16777216.0f) - 0.5f) * 0.25f);
      h = h * 1664525u + 1013904223u;
      b[k][i] = (__bf16)(((float)(h >> 8) * (1.0f / 16777216.0f) - 0.5f) * 0.25f);
      if (!VARY) {                       // one constant operand pair for every MFMA: the best case for the clock
        a[k][i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[k][i] = (__bf16)(float)((threadIdx.x * 3 + i) & 1);
      }
    }
  f32x16 c[4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) c[k][r] = 0.f;
  for (int it = 0; it < iters; it += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int k = 0; k < 4; ++k) c[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(k + u) & 3], b[u], c[k], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c[k][r];
  if (s == -1.f) sink[0] = s;
}

}  // namespace

extern "C" {

// All pointers are device pointers; `stream` is a hipStream_t.  Each call launches exactly one kernel and
// returns the hipError_t of the launch.  bytes must be a multiple of wgs * 32768.
int fbc_read_vgpr(const void* src, size_t bytes, int wgs, void* sink, void* stream) {
  if (wgs <= 0 || bytes % ((size_t)wgs * 32768) != 0) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(read_vgpr_kernel<8>, dim3(wgs), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src,
                     bytes / 16 / wgs, (uint32_t*)sink);
  return (int)hipGetLastError();
}

int fbc_read_lds(const void* src, size_t bytes, int wgs, int depth, void* sink, void* stream) {
  if (wgs <= 0 || bytes % ((size_t)wgs * kStageBytes) != 0) return (int)hipErrorInvalidValue;
  const int stages = (int)(bytes / kStageBytes / wgs);
  hipError_t e;
  auto go = [&](auto kern, int d) {
    e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, d * kStageBytes);
    if (e != hipSuccess) return;
    hipLaunchKernelGGL(kern, dim3(wgs), dim3(kRingThreads), d * kStageBytes, (hipStream_t)stream,
                       (const unsigned char*)src, stages, (uint32_t*)sink);
    e = hipGetLastError();
  };
  switch (depth) {
    case 2: go(read_lds_kernel<2>, 2); break;
    case 3: go(read_lds_kernel<3>, 3); break;
    case 4: go(read_lds_kernel<4>, 4); break;
    case 5: go(read_lds_kernel<5>, 5); break;
    default: return (int)hipErrorInvalidValue;
  }
  return (int)e;
}

int fbc_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (bytes % 16 != 0) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(copy_kernel, dim3(2048), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, (u32x4*)dst, bytes / 16);
  return (int)hipGetLastError();
}

// flops per launch = wgs * 4 wavefronts * iters * 4 MFMAs * 32768 (iters a multiple of 4)
int fbc_mfma(int iters, int wgs, int vary, void* sink, void* stream) {
  if (wgs <= 0 || iters <= 0 || iters % 4 != 0) return (int)hipErrorInvalidValue;
  if (vary) hipLaunchKernelGGL(mfma_kernel<true>, dim3(wgs), dim3(256), 0, (hipStream_t)stream, iters, (float*)sink);
  else hipLaunchKernelGGL(mfma_kernel<false>, dim3(wgs), dim3(256), 0, (hipStream_t)stream, iters, (float*)sink);
  return (int)hipGetLastError();
}

}  // extern "C"
