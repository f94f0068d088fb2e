// C-ABI layer of libflashblock.so: argument validation (host only, no GPU touched), split
// heuristics, workspace carving and kernel dispatch.  Contract: include/flashblock.h.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <string>

#include "../../include/flashblock_prof.h"
#include "fb_kernels.h"

namespace {

thread_local std::string g_last_hip_error;

constexpr long long kFoldKernelMaxRows = 4096;   // largest row count the one-kernel split fold + internal attention is used for
constexpr int kMaxKeyBlocks = 16384;   // LDS-resident per-KV-group block tables in the sparse helpers
constexpr float kLog2e = 1.4426950408889634f;

fb_status hip_fail(hipError_t e) {
  g_last_hip_error = hipGetErrorString(e);
  return FB_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

fb_status check_shape(const fb_shape* s) {
  if (s == nullptr) return FB_ERR_NULL;
  if (s->struct_size != sizeof(fb_shape)) return FB_ERR_SHAPE;
  if (s->dtype != FB_F32 && s->dtype != FB_BF16) return FB_ERR_DTYPE;
  if (s->batch < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->block_len < 1 || s->prefix_len < 0)
    return FB_ERR_SHAPE;
  if (s->n_q_heads % s->n_kv_heads != 0) return FB_ERR_SHAPE;
  if (s->n_q_heads / s->n_kv_heads > 32) return FB_ERR_SHAPE;
  if (!(s->scale >= 0.f) || isinf(s->scale)) return FB_ERR_SHAPE;   // rejects NaN and negatives
  if (s->head_dim < 1) return FB_ERR_SHAPE;
  if (s->head_dim != 64 && s->head_dim != 128) return FB_ERR_UNSUPPORTED;
  if ((long long)s->batch * s->n_q_heads > 65535) return FB_ERR_UNSUPPORTED;   // grid.y of the fp32 pass
  const long long rows = (long long)s->batch * s->n_q_heads * s->block_len;
  if (rows > (1ll << 28)) return FB_ERR_UNSUPPORTED;
  return FB_OK;
}

float eff_scale(const fb_shape* s) { return s->scale > 0.f ? s->scale : 1.0f / sqrtf((float)s->head_dim); }

long long rows_of(const fb_shape* s) { return (long long)s->batch * s->n_q_heads * s->block_len; }

int auto_splits(const fb_shape* s, int active_heads = 0) {
  const int tiles = (s->prefix_len + fb::kKeyTile - 1) / fb::kKeyTile;
  if (s->dtype == FB_BF16 && active_heads > 0 && active_heads < s->n_q_heads) {
    // Per-head refresh with a hint: only the KV groups of flagged heads do work (at most
    // min(Hkv, active) of them per batch element).  8-wavefront workgroups, one per CU; among the two
    // split counts around 256 / groups take the one with the shorter critical path
    // (rounds of 256 workgroups x tiles per split), never fewer than 8 tiles per split.
    const int G = s->n_q_heads / s->n_kv_heads;
    const long long kvg = active_heads < s->n_kv_heads ? active_heads : s->n_kv_heads;
    const long long groups = (long long)s->batch * kvg * ((G * s->block_len + fb::kRowsPerWgBf16 - 1) / fb::kRowsPerWgBf16);
    long long best = 1, best_cost = -1;
    const long long lo = 256 / groups > 1 ? 256 / groups : 1;
    for (long long ns = lo; ns <= lo + 1; ++ns) {
      if (ns > 1 && tiles < 8 * ns) continue;
      if (ns > FB_MAX_SPLITS) continue;
      const long long cost = ((groups * ns + 255) / 256) * ((tiles + ns - 1) / ns);
      if (best_cost < 0 || cost < best_cost) { best = ns; best_cost = cost; }
    }
    return (int)best;
  }
  if (s->dtype == FB_BF16) {
    // Every split costs a 128-row fp32 partial written and read back, so splits are as few as
    // still fill the GPU.
    const int G = s->n_q_heads / s->n_kv_heads;
    const long long groups =
        (long long)s->batch * s->n_kv_heads * ((G * s->block_len + fb::kRowsPerWgBf16 - 1) / fb::kRowsPerWgBf16);
    // Long prefixes: one 8-wavefront workgroup per CU (256 CUs), each streaming >= 8 tiles.
    // Shorter ones: 4-wavefront workgroups, up to two per CU, never fewer than 4 tiles per split.
    const long long per_cu = (256 + groups - 1) / groups;
    long long ns;
    if (tiles >= 8 * per_cu) {
      ns = per_cu;
    } else {
      ns = tiles / 4;
      const long long hi = (512 + groups - 1) / groups;
      if (ns > hi) ns = hi;
    }
    if (ns > FB_MAX_SPLITS) ns = FB_MAX_SPLITS;
    if (ns < 1) ns = 1;
    return (int)ns;
  }
  const long long groups =
      (long long)s->batch * s->n_q_heads * ((s->block_len + fb::kRowsPerWgF32 - 1) / fb::kRowsPerWgF32);
  long long ns = (1024 + groups - 1) / groups;
  if (ns > tiles) ns = tiles;
  if (ns > FB_MAX_SPLITS) ns = FB_MAX_SPLITS;
  if (ns < 1) ns = 1;
  return (int)ns;
}

// Split counts of the sparse passes (bf16): one workgroup per CU in both modes - 8 wavefronts in
// the reuse pass, 4 wavefronts with two accumulator sets in the refresh pass.
// Splits of the plain dense external pass.  KV groups above 128 rows run 256-row, 8-wavefront workgroups, one per
// CU: as many splits as keep the workgroup count within the 256 CUs (one round), each with at least 8 tiles.
int dense_splits(const fb_shape* s) {
  const int G = s->n_q_heads / s->n_kv_heads;
  const long long nrows = (long long)G * s->block_len;
  if (s->dtype != FB_BF16 || !fb::dense_row_pairs((int)std::min<long long>(nrows, 1 << 30), s->head_dim)) return auto_splits(s);
  const int tiles = (s->prefix_len + fb::kKeyTile - 1) / fb::kKeyTile;
  const long long groups = (long long)s->batch * s->n_kv_heads * ((nrows + 2 * fb::kRowsPerWgBf16 - 1) / (2 * fb::kRowsPerWgBf16));
  long long ns = 256 / groups;
  if (ns > tiles / 8) ns = tiles / 8;
  if (ns > FB_MAX_SPLITS) ns = FB_MAX_SPLITS;
  if (ns < 1) ns = 1;
  return (int)ns;
}

int sparse_splits(const fb_shape* s, bool refresh) {
  (void)refresh;
  if (s->dtype != FB_BF16) return auto_splits(s);
  const int tiles = (s->prefix_len + fb::kKeyTile - 1) / fb::kKeyTile;
  const int G = s->n_q_heads / s->n_kv_heads;
  const long long groups =
      (long long)s->batch * s->n_kv_heads * ((G * s->block_len + fb::kRowsPerWgBf16 - 1) / fb::kRowsPerWgBf16);
  long long ns = (256 + groups - 1) / groups;
  const long long cap = tiles / 4;
  if (ns > cap) ns = cap;
  if (ns > FB_MAX_SPLITS) ns = FB_MAX_SPLITS;
  if (ns < 1) ns = 1;
  return (int)ns;
}

// Paged pass: sequences differ in length, so equal split counts give unequal workgroups.  Aim at
// ~2 eight-wavefront workgroups per CU (dispatched longest sequence first, the hardware dispatcher
// evens them out), each with at least 16 tiles on the longest sequence.
int paged_splits(const fb_shape* s) {
  if (s->dtype != FB_BF16) return auto_splits(s);
  const int tiles = (s->prefix_len + fb::kKeyTile - 1) / fb::kKeyTile;
  const int G = s->n_q_heads / s->n_kv_heads;
  const long long groups =
      (long long)s->batch * s->n_kv_heads * ((G * s->block_len + fb::kRowsPerWgBf16 - 1) / fb::kRowsPerWgBf16);
  long long ns = (512 + groups - 1) / groups;
  const long long cap = tiles / 16;
  if (ns > cap) ns = cap;
  if (ns > FB_MAX_SPLITS) ns = FB_MAX_SPLITS;
  if (ns < 1) ns = 1;
  return (int)ns;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct WsLayout {
  size_t o[2], m[2], l[2], mask, ulist, umask, ucnt, order, total;
};

WsLayout ws_layout(const fb_shape* s, int nsplit, int nsets, int nblk, int nsplit2 = -1) {
  WsLayout w;
  const size_t rows = (size_t)rows_of(s);
  size_t off = 0;
  for (int i = 0; i < 2; ++i) {
    const size_t n = (i < nsets) ? (size_t)((i == 1 && nsplit2 >= 0) ? nsplit2 : nsplit) * rows : 0;
    w.o[i] = off; off = align256(off + n * s->head_dim * sizeof(float));
    w.m[i] = off; off = align256(off + n * sizeof(float));
    w.l[i] = off; off = align256(off + n * sizeof(float));
  }
  const size_t nb = (size_t)s->batch * s->n_kv_heads * nblk;
  w.mask = off;  off = align256(off + nb * sizeof(uint32_t));
  w.ulist = off; off = align256(off + nb * sizeof(int32_t));
  w.umask = off; off = align256(off + nb * sizeof(uint32_t));
  w.ucnt = off;  off = align256(off + (nblk > 0 ? (size_t)s->batch * s->n_kv_heads * sizeof(int32_t) : 0));
  w.order = off; off = align256(off + (size_t)s->batch * sizeof(int32_t));   // paged pass: sequences by length
  w.total = off;
  return w;
}

fb_status check_key_block(const fb_shape* s, int32_t key_block, int32_t topk, int* nblk) {
  if (key_block <= 0 || topk < 0) return FB_ERR_SHAPE;
  if (key_block % fb::kKeyTile != 0) return FB_ERR_UNSUPPORTED;
  const long long nb = ((long long)s->prefix_len + key_block - 1) / key_block;
  if (nb > kMaxKeyBlocks) return FB_ERR_UNSUPPORTED;
  *nblk = (int)nb;
  return FB_OK;
}

fb::PassParams base_pass(const fb_shape* s, const void* q, const void* k, const void* v, int nkeys, int nsplit) {
  fb::PassParams p;
  memset(&p, 0, sizeof(p));
  p.q = q; p.k = k; p.v = v;
  p.B = s->batch; p.Hq = s->n_q_heads; p.Hkv = s->n_kv_heads; p.G = s->n_q_heads / s->n_kv_heads;
  p.Bq = s->block_len; p.nkeys = nkeys; p.nsplit = nsplit;
  p.scale_log2 = eff_scale(s) * kLog2e;
  p.key_block = fb::kKeyTile;
  return p;
}

hipError_t launch_attn(const fb_shape* s, const fb::PassParams& p, fb::PassMode mode, hipStream_t st) {
  return s->dtype == FB_BF16 ? fb::launch_attn_bf16(p, s->head_dim, mode, st)
                             : fb::launch_attn_f32(p, s->head_dim, mode, st);
}

// Attention launch with optional measurement events.  bf16 kernels take them as their own start / stop events
// (the kernel's dispatch timestamps); where the launch does not (fp32 kernel), they are recorded around it.
hipError_t timed_attn(const fb_shape* s, const fb::PassParams& p, fb::PassMode mode, hipStream_t st, void* ev_begin,
                      void* ev_end) {
  hipError_t e = hipSuccess;
  const bool in_launch = s->dtype == FB_BF16 && (ev_begin || ev_end);
  if (in_launch) {
    fb::tl_kernel_events.start = (hipEvent_t)ev_begin;
    fb::tl_kernel_events.stop = (hipEvent_t)ev_end;
  } else if (ev_begin && (e = hipEventRecord((hipEvent_t)ev_begin, st)) != hipSuccess) {
    return e;
  }
  e = launch_attn(s, p, mode, st);
  fb::tl_kernel_events = fb::KernelEvents{};      // never left behind for an unrelated launch
  if (e != hipSuccess) return e;
  if (!in_launch && ev_end) e = hipEventRecord((hipEvent_t)ev_end, st);
  return e;
}

}  // namespace

extern "C" {

int fb_version(void) { return FB_VERSION; }

const char* fb_status_string(int status) {
  switch (status) {
    case FB_OK: return "FB_OK";
    case FB_ERR_NULL: return "FB_ERR_NULL: required pointer is NULL";
    case FB_ERR_SHAPE: return "FB_ERR_SHAPE: dimension, head grouping, scale or mode out of range";
    case FB_ERR_DTYPE: return "FB_ERR_DTYPE: dtype is not FB_F32 / FB_BF16";
    case FB_ERR_ALIGN: return "FB_ERR_ALIGN: tensor pointer not 16-byte aligned";
    case FB_ERR_WORKSPACE: return "FB_ERR_WORKSPACE: workspace NULL or too small";
    case FB_ERR_UNSUPPORTED: return "FB_ERR_UNSUPPORTED: request outside what the kernels cover";
    case FB_ERR_HIP: return "FB_ERR_HIP: HIP launch failed";
    default: return "unknown fb_status";
  }
}

const char* fb_last_hip_error(void) { return g_last_hip_error.c_str(); }

fb_status fb_check_shape(const fb_shape* shape) { return check_shape(shape); }

int32_t fb_external_splits(const fb_shape* shape) {
  if (check_shape(shape) != FB_OK) return 0;
  return dense_splits(shape);
}

const char* fb_external_kernel_name(const fb_shape* shape) {
  thread_local char name[96];
  name[0] = 0;
  if (check_shape(shape) != FB_OK) return name;
  if (shape->dtype != FB_BF16) {
    snprintf(name, sizeof(name), "attn_f32_kernel<%d, %d>", shape->head_dim, (int)fb::kPassDense);
    return name;
  }
  const fb::PassParams p = base_pass(shape, nullptr, nullptr, nullptr, shape->prefix_len, dense_splits(shape));
  fb::attn_bf16_dense_name(p, shape->head_dim, name, sizeof(name));
  return name;
}

int32_t fb_paged_splits(const fb_shape* shape) {
  if (check_shape(shape) != FB_OK) return 0;
  return paged_splits(shape);
}

size_t fb_workspace_bytes(const fb_shape* shape, int32_t key_block, int32_t topk, int32_t n_splits) {
  if (check_shape(shape) != FB_OK) return 0;
  if (n_splits < 0 || n_splits > FB_MAX_SPLITS) return 0;
  const int ns = n_splits > 0 ? n_splits : std::max(auto_splits(shape), dense_splits(shape));
  size_t t = ws_layout(shape, ns, 2, 0, 1).total;   // + one block-internal partial for fb_refresh_step
  if (key_block != 0) {
    int nblk = 0;
    if (check_key_block(shape, key_block, topk, &nblk) != FB_OK) return 0;
    const size_t ts = ws_layout(shape, sparse_splits(shape, false), 2, nblk).total;
    if (ts > t) t = ts;
  }
  return t > 0 ? t : 256;
}

}  // extern "C"

namespace {

fb_status external_partial_impl(const fb_shape* shape, const void* q, const void* k_prefix,
                                const void* v_prefix, const fb_paged_kv* paged, const uint8_t* head_mask,
                                bool use_head_mask, int n_active_heads, float* o_part, float* m_part, float* lse_part,
                                int32_t n_splits, void* workspace, size_t workspace_bytes,
                                void* ev_begin, void* ev_attn_end, void* ev_end, void* hip_stream,
                                fb::CombineParams* fold_out = nullptr) {
  // fold_out: the caller folds the split partials itself (with a kernel that does more than the plain combine); it
  // gets the combine's parameters instead of the combine launch.  Left with nsplit = 0 when there was one split
  // and the attention kernel wrote the final partial itself.
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  if (!q || !o_part || !m_part || !lse_part) return FB_ERR_NULL;
  if (use_head_mask && !head_mask) return FB_ERR_NULL;
  if (paged) {
    if (paged->struct_size != sizeof(fb_paged_kv)) return FB_ERR_SHAPE;
    if (!paged->block_table || !paged->prefix_lens) return FB_ERR_NULL;
    if (paged->num_pages <= 0 || paged->page_size <= 0 || paged->max_pages <= 0) return FB_ERR_SHAPE;
    if (paged->page_size % fb::kKeyTile != 0) return FB_ERR_UNSUPPORTED;
    if ((long long)paged->max_pages * paged->page_size < shape->prefix_len) return FB_ERR_SHAPE;
    k_prefix = paged->k_pool;
    v_prefix = paged->v_pool;
  }
  if (shape->prefix_len > 0 && (!k_prefix || !v_prefix)) return FB_ERR_NULL;
  if (n_splits < 0 || n_splits > FB_MAX_SPLITS) return FB_ERR_SHAPE;
  if (!aligned16(q) || !aligned16(k_prefix) || !aligned16(v_prefix) || !aligned16(o_part) ||
      !aligned16(m_part) || !aligned16(lse_part) || !aligned16(workspace))
    return FB_ERR_ALIGN;
  if (n_active_heads < 0) return FB_ERR_SHAPE;
  const int ns = n_splits > 0 ? n_splits
                             : (paged ? paged_splits(shape)
                                      : use_head_mask ? auto_splits(shape, n_active_heads) : dense_splits(shape));
  const WsLayout w = ws_layout(shape, ns, 1, 0);
  if (!workspace || workspace_bytes < w.total) return FB_ERR_WORKSPACE;

  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  fb::PassParams p = base_pass(shape, q, k_prefix, v_prefix, shape->prefix_len, ns);
  p.ws_o = (float*)(ws + w.o[0]); p.ws_m = (float*)(ws + w.m[0]); p.ws_l = (float*)(ws + w.l[0]);
  p.head_on = use_head_mask ? head_mask : nullptr;
  fb::PassMode mode = use_head_mask ? fb::kPassDenseHeads : fb::kPassDense;
  if (paged) {
    mode = fb::kPassDensePaged;
    p.block_table = paged->block_table; p.prefix_lens = paged->prefix_lens;
    p.page_size = paged->page_size; p.max_pages = paged->max_pages; p.num_pages = paged->num_pages;
    if (shape->batch > 1 && shape->batch <= 128 && shape->dtype == FB_BF16) {
      p.order_inline = 1;       // the bf16 kernel ranks up to 128 sequences in its prologue
    } else if (shape->batch > 1) {
      p.seq_order = (int32_t*)(ws + w.order);
      hipError_t eo = fb::launch_seq_order(paged->prefix_lens, (int32_t*)(ws + w.order), shape->batch, stream);
      if (eo != hipSuccess) return hip_fail(eo);
    }
  }
  if (ns == 1) {   // the attention kernel writes the final partial itself
    p.direct = 1;
    p.ws_o = o_part; p.ws_m = m_part; p.ws_l = lse_part;
  }
  hipError_t e = timed_attn(shape, p, mode, stream, ev_begin, ev_attn_end);
  if (e != hipSuccess) return hip_fail(e);

  if (fold_out) memset(fold_out, 0, sizeof(*fold_out));
  if (!p.direct) {
    fb::CombineParams c;
    memset(&c, 0, sizeof(c));
    c.rows = (int)rows_of(shape); c.D = shape->head_dim; c.nsplit = ns;
    c.ws_o = p.ws_o; c.ws_m = p.ws_m; c.ws_l = p.ws_l;
    c.o = o_part; c.m = m_part; c.lse = lse_part;
    c.head_on = p.head_on; c.Bq = shape->block_len;
    if (fold_out) {
      *fold_out = c;
    } else {
      e = fb::launch_combine(c, stream);
      if (e != hipSuccess) return hip_fail(e);
    }
  }
  if (ev_end && (e = hipEventRecord((hipEvent_t)ev_end, stream)) != hipSuccess) return hip_fail(e);
  return FB_OK;
}

}  // namespace

extern "C" {

fb_status fb_external_partial_prof(const fb_shape* shape, const void* q, const void* k_prefix,
                                   const void* v_prefix, float* o_part, float* m_part, float* lse_part,
                                   int32_t n_splits, void* workspace, size_t workspace_bytes,
                                   void* ev_begin, void* ev_attn_end, void* ev_end, void* hip_stream) {
  return external_partial_impl(shape, q, k_prefix, v_prefix, nullptr, nullptr, false, 0, o_part, m_part, lse_part, n_splits,
                               workspace, workspace_bytes, ev_begin, ev_attn_end, ev_end, hip_stream);
}

int32_t fb_external_heads_splits(const fb_shape* shape, int32_t n_active_heads) {
  if (check_shape(shape) != FB_OK || n_active_heads < 0) return 0;
  return auto_splits(shape, n_active_heads);
}

fb_status fb_external_partial_heads(const fb_shape* shape, const void* q, const void* k_prefix,
                                    const void* v_prefix, const uint8_t* head_mask, int32_t n_active_heads,
                                    float* o_part, float* m_part, float* lse_part, void* workspace,
                                    size_t workspace_bytes, void* hip_stream) {
  return external_partial_impl(shape, q, k_prefix, v_prefix, nullptr, head_mask, true, n_active_heads, o_part, m_part, lse_part, 0,
                               workspace, workspace_bytes, nullptr, nullptr, nullptr, hip_stream);
}

fb_status fb_external_partial_paged(const fb_shape* shape, const void* q, const fb_paged_kv* kv, float* o_part,
                                    float* m_part, float* lse_part, int32_t n_splits, void* workspace,
                                    size_t workspace_bytes, void* hip_stream) {
  if (!kv) return FB_ERR_NULL;
  return external_partial_impl(shape, q, nullptr, nullptr, kv, nullptr, false, 0, o_part, m_part, lse_part, n_splits,
                               workspace, workspace_bytes, nullptr, nullptr, nullptr, hip_stream);
}

fb_status fb_external_partial_ex(const fb_shape* shape, const void* q, const void* k_prefix,
                                 const void* v_prefix, float* o_part, float* m_part, float* lse_part,
                                 int32_t n_splits, void* workspace, size_t workspace_bytes,
                                 void* hip_stream) {
  return fb_external_partial_prof(shape, q, k_prefix, v_prefix, o_part, m_part, lse_part, n_splits,
                                  workspace, workspace_bytes, nullptr, nullptr, nullptr, hip_stream);
}

fb_status fb_external_partial(const fb_shape* shape, const void* q, const void* k_prefix,
                              const void* v_prefix, float* o_part, float* m_part, float* lse_part,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  return fb_external_partial_ex(shape, q, k_prefix, v_prefix, o_part, m_part, lse_part, 0, workspace,
                                workspace_bytes, hip_stream);
}

}  // extern "C"

namespace {

// Scratch memory of fb_external_partial_builtin_ws: the split partials of one call.  One copy per GPU the
// library runs on, held until the process ends.
constexpr size_t kBuiltinWsBytes = (size_t)20 * 1024 * 1024;
static __device__ __align__(256) unsigned char scratch[kBuiltinWsBytes];

constexpr int kMaxDevices = 16;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // device address of `scratch` per device, looked up on first use

// The array's name is only a host-side handle: its device address comes from hipGetSymbolAddress, asked once
// per device with that device current, and that address is what kernels and copies get.
fb_status builtin_ws(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return FB_ERR_UNSUPPORTED;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr == nullptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (ptr == nullptr) return FB_ERR_HIP;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // racing first calls store the same address
  }
  *out = ptr;
  return FB_OK;
}

}  // namespace

extern "C" {

size_t fb_builtin_workspace_bytes(void) { return kBuiltinWsBytes; }

fb_status fb_external_partial_builtin_ws(const fb_shape* shape, const void* q, const void* k_prefix,
                                         const void* v_prefix, float* o_part, float* m_part, float* lse_part,
                                         void* hip_stream) {
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  if (fb_workspace_bytes(shape, 0, 0, 0) > kBuiltinWsBytes) return FB_ERR_WORKSPACE;   // too large for the built-in scratch
  if (!q || !o_part || !m_part || !lse_part) return FB_ERR_NULL;      // host-side checks before any HIP call
  if (shape->prefix_len > 0 && (!k_prefix || !v_prefix)) return FB_ERR_NULL;
  void* ws = nullptr;
  st = builtin_ws(&ws);
  if (st != FB_OK) return st;
  return external_partial_impl(shape, q, k_prefix, v_prefix, nullptr, nullptr, false, 0, o_part, m_part, lse_part, 0,
                               ws, kBuiltinWsBytes, nullptr, nullptr, nullptr, hip_stream);
}

fb_status fb_head_similarity(const fb_shape* shape, const float* o_a, const float* o_b, float* sim,
                             void* hip_stream) {
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  if (!o_a || !o_b || !sim) return FB_ERR_NULL;
  if (!aligned16(o_a) || !aligned16(o_b) || !aligned16(sim)) return FB_ERR_ALIGN;
  hipError_t e = fb::launch_head_similarity(o_a, o_b, sim, shape->batch * shape->n_q_heads, shape->block_len,
                                            shape->head_dim, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e);
  return FB_OK;
}

fb_status fb_internal_merge(const fb_shape* shape, const void* q, const void* k_block,
                            const void* v_block, const float* o_part, const float* m_part,
                            const float* lse_part, void* out, float* lse_out, void* hip_stream) {
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  if (!q || !k_block || !v_block || !out) return FB_ERR_NULL;
  const int n_ext = (o_part != nullptr) + (m_part != nullptr) + (lse_part != nullptr);
  if (n_ext != 0 && n_ext != 3) return FB_ERR_NULL;   // all three or none
  if (!aligned16(q) || !aligned16(k_block) || !aligned16(v_block) || !aligned16(o_part) ||
      !aligned16(m_part) || !aligned16(lse_part) || !aligned16(out) || !aligned16(lse_out))
    return FB_ERR_ALIGN;
  fb::PassParams p = base_pass(shape, q, k_block, v_block, shape->block_len, 1);
  p.ext_o = o_part; p.ext_m = m_part; p.ext_lse = lse_part;
  p.out = out; p.lse_out = lse_out;
  hipError_t e = launch_attn(shape, p, fb::kPassInternal, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e);
  return FB_OK;
}

fb_status fb_refresh_step_prof(const fb_shape* shape, const void* q, const void* k_prefix, const void* v_prefix,
                               const void* k_block, const void* v_block, float* o_part, float* m_part,
                               float* lse_part, void* out, float* lse_out, void* workspace,
                               size_t workspace_bytes, void* ev_begin, void* ev_attn_end, void* ev_end,
                               void* hip_stream) {
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  if (!q || !k_block || !v_block || !o_part || !m_part || !lse_part || !out) return FB_ERR_NULL;
  if (shape->prefix_len > 0 && (!k_prefix || !v_prefix)) return FB_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_prefix) || !aligned16(v_prefix) || !aligned16(k_block) ||
      !aligned16(v_block) || !aligned16(o_part) || !aligned16(m_part) || !aligned16(lse_part) ||
      !aligned16(out) || !aligned16(lse_out) || !aligned16(workspace))
    return FB_ERR_ALIGN;
  // Small block and many splits (the LLM shapes): the prefix splits already fill every CU, so the
  // block's own keys are not streamed by the attention kernel at all (plain dense pass, with its split
  // count); one fold kernel (4 rows per workgroup) folds the splits, computes the rows' block-internal
  // attention and merges.
  const bool small_block = shape->block_len <= fb::kMaxInlineBlock && shape->block_len % fb::kFoldRows == 0 &&
                           dense_splits(shape) >= 8;
  const int ns = small_block ? dense_splits(shape) : auto_splits(shape);
  const WsLayout w = ws_layout(shape, ns, 2, 0, 1);
  if (!workspace || workspace_bytes < w.total) return FB_ERR_WORKSPACE;

  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  fb::PassParams p = base_pass(shape, q, k_prefix, v_prefix, shape->prefix_len, ns);
  p.k2 = k_block; p.v2 = v_block;
  {
    // prefix tiles the block phase is worth (its cold load, LDS hand-over and epilogue), capped at half a split
    const int tiles = (shape->prefix_len + fb::kKeyTile - 1) / fb::kKeyTile;
    const int btiles = (shape->block_len + fb::kKeyTile - 1) / fb::kKeyTile;
    p.blk_cost = ns > 1 ? std::min(2 + btiles, tiles / ns / 2) : 0;
  }
  p.ws_o = (float*)(ws + w.o[0]); p.ws_m = (float*)(ws + w.m[0]); p.ws_l = (float*)(ws + w.l[0]);
  p.ws_o2 = (float*)(ws + w.o[1]); p.ws_m2 = (float*)(ws + w.m[1]); p.ws_l2 = (float*)(ws + w.l[1]);
  hipError_t e = timed_attn(shape, p, small_block ? fb::kPassDense : fb::kPassRefreshFused, stream, ev_begin, ev_attn_end);
  if (e != hipSuccess) return hip_fail(e);

  fb::CombineParams c;
  memset(&c, 0, sizeof(c));
  c.rows = (int)rows_of(shape); c.D = shape->head_dim; c.nsplit = ns;
  c.ws_o = p.ws_o; c.ws_m = p.ws_m; c.ws_l = p.ws_l;
  c.o = o_part; c.m = m_part; c.lse = lse_part;
  c.Bq = shape->block_len;
  c.fin_out = out; c.fin_lse = lse_out; c.fin_bf16 = shape->dtype == FB_BF16;
  if (small_block) {
    c.blk_q = q; c.blk_k = k_block; c.blk_v = v_block;
    c.Hq = shape->n_q_heads; c.Hkv = shape->n_kv_heads; c.G = shape->n_q_heads / shape->n_kv_heads;
    c.scale_log2 = p.scale_log2;
    e = fb::launch_refresh_fold(c, stream);
  } else {
    c.blk_o = p.ws_o2; c.blk_m = p.ws_m2; c.blk_l = p.ws_l2;
    e = fb::launch_combine(c, stream);
  }
  if (e != hipSuccess) return hip_fail(e);
  if (ev_end && (e = hipEventRecord((hipEvent_t)ev_end, stream)) != hipSuccess) return hip_fail(e);
  return FB_OK;
}

fb_status fb_refresh_step_paged(const fb_shape* shape, const void* q, const fb_paged_kv* kv, const void* k_block,
                                const void* v_block, float* o_part, float* m_part, float* lse_part, void* out,
                                float* lse_out, int32_t n_splits, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
  if (!kv) return FB_ERR_NULL;
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  if (!k_block || !v_block || !out) return FB_ERR_NULL;
  if (!aligned16(k_block) || !aligned16(v_block) || !aligned16(out) || !aligned16(lse_out)) return FB_ERR_ALIGN;
  // With several splits and a small block the split fold, the block-internal attention and the merge are one
  // kernel (as in fb_refresh_step); with one split the paged pass writes the partial itself and the internal pass
  // follows; otherwise combine + internal pass.
  // (the fold kernel runs 4 rows per workgroup and is a latency chain: beyond a few thousand rows the plain
  // combine and the MFMA internal pass are faster, measured 219 vs ~165 us per step at batch 32, block 32)
  const bool fold_kernel = shape->block_len <= fb::kMaxInlineBlock && shape->block_len % fb::kFoldRows == 0 &&
                           rows_of(shape) <= kFoldKernelMaxRows;
  fb::CombineParams c;
  st = external_partial_impl(shape, q, nullptr, nullptr, kv, nullptr, false, 0, o_part, m_part, lse_part, n_splits,
                             workspace, workspace_bytes, nullptr, nullptr, nullptr, hip_stream, fold_kernel ? &c : nullptr);
  if (st != FB_OK) return st;
  if (fold_kernel && c.nsplit > 0) {
    c.fin_out = out; c.fin_lse = lse_out; c.fin_bf16 = shape->dtype == FB_BF16;
    c.blk_q = q; c.blk_k = k_block; c.blk_v = v_block;
    c.Hq = shape->n_q_heads; c.Hkv = shape->n_kv_heads; c.G = shape->n_q_heads / shape->n_kv_heads;
    c.scale_log2 = eff_scale(shape) * kLog2e;
    hipError_t e = fb::launch_refresh_fold(c, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e);
    return FB_OK;
  }
  return fb_internal_merge(shape, q, k_block, v_block, o_part, m_part, lse_part, out, lse_out, hip_stream);
}

fb_status fb_refresh_step(const fb_shape* shape, const void* q, const void* k_prefix, const void* v_prefix,
                          const void* k_block, const void* v_block, float* o_part, float* m_part,
                          float* lse_part, void* out, float* lse_out, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  return fb_refresh_step_prof(shape, q, k_prefix, v_prefix, k_block, v_block, o_part, m_part, lse_part, out,
                              lse_out, workspace, workspace_bytes, nullptr, nullptr, nullptr, hip_stream);
}

fb_status fb_pool_keys(const fb_shape* shape, const void* k_prefix, int32_t key_block, float* k_pooled,
                       void* hip_stream) {
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  int nblk = 0;
  st = check_key_block(shape, key_block, 0, &nblk);
  if (st != FB_OK) return st;
  if (shape->prefix_len > 0 && (!k_prefix || !k_pooled)) return FB_ERR_NULL;
  if (!aligned16(k_prefix) || !aligned16(k_pooled)) return FB_ERR_ALIGN;
  fb::PoolParams p;
  p.k = k_prefix; p.k_pooled = k_pooled;
  p.BH = shape->batch * shape->n_kv_heads; p.nkeys = shape->prefix_len; p.D = shape->head_dim;
  p.key_block = key_block; p.nblk = nblk; p.is_bf16 = shape->dtype == FB_BF16;
  hipError_t e = fb::launch_pool_keys(p, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e);
  return FB_OK;
}

size_t fb_select_workspace_bytes(const fb_shape* shape, int32_t key_block) {
  if (check_shape(shape) != FB_OK) return 0;
  int nblk = 0;
  if (check_key_block(shape, key_block, 0, &nblk) != FB_OK) return 0;
  const size_t heads = (size_t)shape->batch * shape->n_q_heads;
  return align256(heads * shape->head_dim * sizeof(float)) + align256(heads * nblk * sizeof(float)) + 256;
}

fb_status fb_select_topk(const fb_shape* shape, const void* q, const float* k_pooled, int32_t key_block,
                         int32_t topk, int32_t* sel_idx, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  int nblk = 0;
  st = check_key_block(shape, key_block, topk, &nblk);
  if (st != FB_OK) return st;
  if (topk == 0) return FB_OK;
  if (!q || !sel_idx || (nblk > 0 && !k_pooled)) return FB_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_pooled) || !aligned16(sel_idx) || !aligned16(workspace)) return FB_ERR_ALIGN;
  if (workspace && workspace_bytes < fb_select_workspace_bytes(shape, key_block)) return FB_ERR_WORKSPACE;
  fb::SelectParams p;
  memset(&p, 0, sizeof(p));
  p.q = q; p.k_pooled = k_pooled; p.sel_idx = sel_idx;
  if (workspace) {
    p.qbar_ws = (float*)workspace;
    p.scores_ws = (float*)((char*)workspace +
                           align256((size_t)shape->batch * shape->n_q_heads * shape->head_dim * sizeof(float)));
  }
  p.B = shape->batch; p.Hq = shape->n_q_heads; p.Hkv = shape->n_kv_heads;
  p.G = shape->n_q_heads / shape->n_kv_heads; p.Bq = shape->block_len; p.D = shape->head_dim;
  p.nblk = nblk; p.topk = topk; p.is_bf16 = shape->dtype == FB_BF16;
  hipError_t e = fb::launch_select_topk(p, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e);
  return FB_OK;
}

size_t fb_select_mass_workspace_bytes(const fb_shape* shape, int32_t key_block) {
  if (check_shape(shape) != FB_OK) return 0;
  int nblk = 0;
  if (check_key_block(shape, key_block, 0, &nblk) != FB_OK) return 0;
  return align256((size_t)rows_of(shape) * nblk * sizeof(float)) + 256;
}

fb_status fb_select_topk_mass(const fb_shape* shape, const void* q, const void* k_prefix, const float* lse_part,
                              int32_t key_block, int32_t topk, int32_t* sel_idx, float* mass_out,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  int nblk = 0;
  st = check_key_block(shape, key_block, topk, &nblk);
  if (st != FB_OK) return st;
  if (topk == 0 || nblk == 0) return FB_OK;
  if (!q || !k_prefix || !lse_part || !sel_idx) return FB_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_prefix) || !aligned16(lse_part) || !aligned16(sel_idx) ||
      !aligned16(mass_out) || !aligned16(workspace))
    return FB_ERR_ALIGN;
  if (!workspace || workspace_bytes < fb_select_mass_workspace_bytes(shape, key_block)) return FB_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)hip_stream;
  const bool bf16 = shape->dtype == FB_BF16;

  fb::MassParams m;
  memset(&m, 0, sizeof(m));
  m.q = q; m.k = k_prefix; m.lse = lse_part; m.rowmass = (float*)workspace;
  m.B = shape->batch; m.Hq = shape->n_q_heads; m.Hkv = shape->n_kv_heads;
  m.G = shape->n_q_heads / shape->n_kv_heads; m.Bq = shape->block_len;
  m.nkeys = shape->prefix_len; m.key_block = key_block; m.nblk = nblk;
  m.scale_log2 = eff_scale(shape) * kLog2e;
  {
    // key-block ranges per row tile: enough workgroups for ~2 per CU, never more than key blocks
    const long long groups = bf16
        ? (long long)m.B * m.Hkv * ((m.G * m.Bq + fb::kRowsPerWgBf16 - 1) / fb::kRowsPerWgBf16)
        : (long long)m.B * m.Hq * ((m.Bq + fb::kRowsPerWgF32 - 1) / fb::kRowsPerWgF32);
    long long ns = ((bf16 ? 512 : 1024) + groups - 1) / groups;
    if (ns > nblk) ns = nblk;
    if (ns > 65535) ns = 65535;
    m.nsplit = (int)ns;
  }
  hipError_t e = bf16 ? fb::launch_block_mass_bf16(m, shape->head_dim, stream)
                      : fb::launch_block_mass_f32(m, shape->head_dim, stream);
  if (e != hipSuccess) return hip_fail(e);

  fb::SelectParams p;
  memset(&p, 0, sizeof(p));
  p.sel_idx = sel_idx; p.rowmass = m.rowmass; p.score_out = mass_out;
  p.B = m.B; p.Hq = m.Hq; p.Hkv = m.Hkv; p.G = m.G; p.Bq = m.Bq; p.D = shape->head_dim;
  p.nblk = nblk; p.topk = topk; p.is_bf16 = bf16;
  e = fb::launch_select_topk(p, stream);
  if (e != hipSuccess) return hip_fail(e);
  return FB_OK;
}

fb_status fb_sparse_external_residual(const fb_shape* shape, int32_t mode, const void* q,
                                      const void* k_prefix, const void* v_prefix, int32_t key_block,
                                      int32_t topk, const int32_t* sel_idx, float* res_o, float* res_m,
                                      float* res_lse, float* o_part, float* m_part, float* lse_part,
                                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  fb_status st = check_shape(shape);
  if (st != FB_OK) return st;
  if (mode != FB_SPARSE_REFRESH && mode != FB_SPARSE_REUSE && mode != FB_SPARSE_REUSE_SAME_SELECTION)
    return FB_ERR_SHAPE;
  const bool keep_masks = mode == FB_SPARSE_REUSE_SAME_SELECTION;
  if (keep_masks) mode = FB_SPARSE_REUSE;
  int nblk = 0;
  st = check_key_block(shape, key_block, topk, &nblk);
  if (st != FB_OK) return st;
  if (!q || !res_o || !res_m || !res_lse || !o_part || !m_part || !lse_part) return FB_ERR_NULL;
  if (shape->prefix_len > 0 && (!k_prefix || !v_prefix)) return FB_ERR_NULL;
  if (topk > 0 && !sel_idx && !keep_masks) return FB_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_prefix) || !aligned16(v_prefix) || !aligned16(sel_idx) ||
      !aligned16(res_o) || !aligned16(res_m) || !aligned16(res_lse) || !aligned16(o_part) ||
      !aligned16(m_part) || !aligned16(lse_part) || !aligned16(workspace))
    return FB_ERR_ALIGN;
  const int ns = sparse_splits(shape, mode == FB_SPARSE_REFRESH);
  const WsLayout w = ws_layout(shape, ns, 2, nblk);
  if (!workspace || workspace_bytes < ws_layout(shape, sparse_splits(shape, false), 2, nblk).total)
    return FB_ERR_WORKSPACE;

  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;

  fb::MaskParams mp;
  mp.sel_idx = topk > 0 ? sel_idx : nullptr;
  mp.blk_mask = (uint32_t*)(ws + w.mask); mp.union_list = (int32_t*)(ws + w.ulist);
  mp.union_mask = (uint32_t*)(ws + w.umask);
  mp.union_cnt = (int32_t*)(ws + w.ucnt);
  mp.B = shape->batch; mp.Hq = shape->n_q_heads; mp.Hkv = shape->n_kv_heads;
  mp.G = shape->n_q_heads / shape->n_kv_heads; mp.topk = topk; mp.nblk = nblk;
  hipError_t e = hipSuccess;
  if (nblk > 0 && !keep_masks) {
    e = fb::launch_build_masks(mp, stream);
    if (e != hipSuccess) return hip_fail(e);
  }

  fb::PassParams p = base_pass(shape, q, k_prefix, v_prefix, shape->prefix_len, ns);
  p.ws_o = (float*)(ws + w.o[0]); p.ws_m = (float*)(ws + w.m[0]); p.ws_l = (float*)(ws + w.l[0]);
  p.ws_o2 = (float*)(ws + w.o[1]); p.ws_m2 = (float*)(ws + w.m[1]); p.ws_l2 = (float*)(ws + w.l[1]);
  p.blk_mask = mp.blk_mask; p.union_list = mp.union_list; p.union_mask = mp.union_mask; p.union_cnt = mp.union_cnt;
  p.key_block = key_block; p.nblk = nblk;

  fb::CombineParams c;
  memset(&c, 0, sizeof(c));
  c.rows = (int)rows_of(shape); c.D = shape->head_dim; c.nsplit = ns;
  c.o = o_part; c.m = m_part; c.lse = lse_part;
  if (nblk > 0) {
    c.ws_o = p.ws_o; c.ws_m = p.ws_m; c.ws_l = p.ws_l;
    e = launch_attn(shape, p, mode == FB_SPARSE_REFRESH ? fb::kPassSparseRefresh : fb::kPassSparseReuse, stream);
    if (e != hipSuccess) return hip_fail(e);
  } else {
    c.nsplit = 0;   // empty prefix: nothing selected, nothing residual
  }
  if (mode == FB_SPARSE_REFRESH) {
    if (nblk > 0) { c.ws_o2 = p.ws_o2; c.ws_m2 = p.ws_m2; c.ws_l2 = p.ws_l2; }
    c.res_out_o = res_o; c.res_out_m = res_m; c.res_out_lse = res_lse;
  } else {
    c.res_in_o = res_o; c.res_in_m = res_m; c.res_in_lse = res_lse;
  }
  e = fb::launch_combine(c, stream);
  if (e != hipSuccess) return hip_fail(e);
  return FB_OK;
}

}  // extern "C"
