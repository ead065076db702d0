// Partitioned tree attention (Section "Redundancy-Free Tree Partitioning", Appendix "Zero-Overhead
// Partition Boundaries"): one attention pass per partition over [cached slice ; own tokens], driven
// from whole-tree tensors.  The data movement around each pass -- row gathers, row scatters, fp32
// accumulation of cached-key gradients, the final rounding -- is a handful of HBM-bound copy
// kernels, 16 bytes per lane, rows addressed through the planner's token index lists.
#include <hip/hip_runtime.h>
#include <algorithm>
#include "tt_internal.h"
#include "tt_kernels.h"

namespace tt {
namespace {

constexpr int COPY_THREADS = 256;

// dst[r][:] = src[idx[r]][:]  (rows of `vec_per_row` 16-byte vectors; src rows `src_stride` vectors apart)
__global__ __launch_bounds__(COPY_THREADS) void gather_rows_kernel(
    int64_t n_vec, int vec_per_row, const uint4* __restrict__ src, int64_t src_stride,
    const int32_t* __restrict__ idx, uint4* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * COPY_THREADS + threadIdx.x;
  if (i >= n_vec) return;
  const int64_t r = i / vec_per_row;
  const int c = (int)(i - r * vec_per_row);
  dst[i] = src[(int64_t)idx[r] * src_stride + c];
}

// dst[idx[r]][:] = src[r][:]
__global__ __launch_bounds__(COPY_THREADS) void scatter_rows_kernel(
    int64_t n_vec, int vec_per_row, const uint4* __restrict__ src, const int32_t* __restrict__ idx,
    uint4* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * COPY_THREADS + threadIdx.x;
  if (i >= n_vec) return;
  const int64_t r = i / vec_per_row;
  const int c = (int)(i - r * vec_per_row);
  dst[(int64_t)idx[r] * vec_per_row + c] = src[i];
}

// dst[idx[r]][:] += src[r][:] in fp32.  The indices of one call are distinct, so plain read-modify-
// write is exact and deterministic; calls on one stream are ordered.
__global__ __launch_bounds__(COPY_THREADS) void scatter_add_rows_kernel(
    int64_t n_vec, int vec_per_row, const float4* __restrict__ src, const int32_t* __restrict__ idx,
    float4* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * COPY_THREADS + threadIdx.x;
  if (i >= n_vec) return;
  const int64_t r = i / vec_per_row;
  const int c = (int)(i - r * vec_per_row);
  const float4 s = src[i];
  float4* p = dst + (int64_t)idx[r] * vec_per_row + c;
  float4 d = *p;
  d.x += s.x; d.y += s.y; d.z += s.z; d.w += s.w;
  *p = d;
}

// lse is [heads][tokens]: local[h][i] = whole[h][idx[i]] (GATHER) or the reverse.
template <bool GATHER>
__global__ __launch_bounds__(COPY_THREADS) void lse_move_kernel(
    int n_local, int n_whole, int heads, const int32_t* __restrict__ idx, const float* __restrict__ src,
    float* __restrict__ dst) {
  const int i = blockIdx.x * COPY_THREADS + threadIdx.x;
  const int h = blockIdx.y;
  if (i >= n_local) return;
  if (GATHER) dst[(int64_t)h * n_local + i] = src[(int64_t)h * n_whole + idx[i]];
  else        dst[(int64_t)h * n_whole + idx[i]] = src[(int64_t)h * n_local + i];
}

__global__ __launch_bounds__(COPY_THREADS) void fill_zero_kernel(int64_t n_vec, uint4* __restrict__ dst) {
  const int64_t i = (int64_t)blockIdx.x * COPY_THREADS + threadIdx.x;
  if (i < n_vec) dst[i] = uint4{0u, 0u, 0u, 0u};
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {     // round to nearest even; NaN stays NaN
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// grad = round(grad + acc): the own-partition gradient (already rounded once to the tensor dtype)
// plus the fp32 sum of what the descendant partitions sent back for the same key.
template <bool BF16>
__global__ __launch_bounds__(COPY_THREADS) void finalize_kernel(int64_t n_quads, void* __restrict__ grad,
                                                                const float4* __restrict__ acc) {
  const int64_t i = (int64_t)blockIdx.x * COPY_THREADS + threadIdx.x;
  if (i >= n_quads) return;
  const float4 a = acc[i];
  if (BF16) {
    ushort4* g = reinterpret_cast<ushort4*>(grad) + i;
    ushort4 v = *g;
    v.x = f32_to_bf16(bf16_to_f32(v.x) + a.x);
    v.y = f32_to_bf16(bf16_to_f32(v.y) + a.y);
    v.z = f32_to_bf16(bf16_to_f32(v.z) + a.z);
    v.w = f32_to_bf16(bf16_to_f32(v.w) + a.w);
    *g = v;
  } else {
    float4* g = reinterpret_cast<float4*>(grad) + i;
    float4 v = *g;
    v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
    *g = v;
  }
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + COPY_THREADS - 1) / COPY_THREADS); }

size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }

struct Dims {
  int32_t n, np;           // whole-tree tokens, partitions
  int32_t max_own, max_prefix;
  int32_t hq;
  size_t esz;
  size_t q_row, kv_row;    // bytes per token row of q-like / k-like tensors (contiguous)
  size_t attn_ws;          // largest attention workspace over the partitions
};

// Carves the driver's buffers out of the workspace, in a fixed order.
struct Carve {
  char* base;
  size_t used = 0;
  explicit Carve(void* p) : base((char*)p) {}
  void* take(size_t bytes) {
    void* r = base ? base + used : nullptr;
    used += up256(bytes);
    return r;
  }
};

struct Buffers {
  void *q, *k, *v, *o, *d_o, *dq, *dk, *dv, *kp, *vp;
  float *dkp, *dvp, *lse, *acc_dk, *acc_dv;
  void* attn_ws;
  size_t total;
};

Buffers carve(void* ws, const Dims& d, bool backward) {
  Carve c(ws);
  Buffers b{};
  const size_t nq = (size_t)d.max_own * d.q_row, nk = (size_t)d.max_own * d.kv_row, npk = (size_t)d.max_prefix * d.kv_row;
  b.q = c.take(nq); b.k = c.take(nk); b.v = c.take(nk); b.o = c.take(nq);
  b.kp = c.take(npk); b.vp = c.take(npk);
  b.lse = (float*)c.take(sizeof(float) * (size_t)d.hq * (size_t)d.max_own);
  if (backward) {
    b.d_o = c.take(nq); b.dq = c.take(nq); b.dk = c.take(nk); b.dv = c.take(nk);
    b.dkp = (float*)c.take(npk / d.esz * sizeof(float));
    b.dvp = (float*)c.take(npk / d.esz * sizeof(float));
    b.acc_dk = (float*)c.take((size_t)d.n * d.kv_row / d.esz * sizeof(float));
    b.acc_dv = (float*)c.take((size_t)d.n * d.kv_row / d.esz * sizeof(float));
  }
  b.attn_ws = c.take(d.attn_ws);
  b.total = c.used + 256;
  return b;
}

// Descriptor of one partition's pass.  `in_place`: q, k, v are read from the whole-tree tensors
// (their token strides apply); otherwise from gathered, contiguous rows.
tt_attn_desc part_desc(const tt_attn_desc* whole, int32_t n_own, int32_t n_prefix, bool in_place = false) {
  tt_attn_desc d = *whole;
  d.n_q = n_own;
  d.n_prefix = n_prefix;
  if (!in_place) d.q_stride_tok = d.k_stride_tok = d.v_stride_tok = 0;
  return d;
}

// One partition's view of the plan.
struct Part {
  int32_t t0, n_own, n_pre;
  int64_t p0;
  int32_t own_start;      // >= 0: own rows are whole-tree rows [own_start, own_start + n_own)
  int32_t pre_start;      // >= 0: the cached slice is whole-tree rows [pre_start, pre_start + n_pre)
};

Part part_of(const tt_partition_plan* plan, int32_t p, bool kv_contiguous) {
  Part x;
  x.t0 = plan->part_tok_off[p];
  x.n_own = plan->part_tok_off[p + 1] - x.t0;
  x.p0 = plan->part_prefix_off[p];
  x.n_pre = (int32_t)(plan->part_prefix_off[p + 1] - x.p0);
  x.own_start = plan->part_own_start && x.n_own > 0 ? plan->part_own_start[p] : -1;
  // the attention calls take the cached slice as contiguous rows, so in-place use needs unpadded k, v
  x.pre_start = plan->part_prefix_start && kv_contiguous && x.n_pre > 0 ? plan->part_prefix_start[p] : -1;
  return x;
}

inline const void* row_ptr(const void* base, int64_t row, int64_t stride_bytes) { return (const char*)base + row * stride_bytes; }
inline void* row_ptr(void* base, int64_t row, int64_t stride_bytes) { return (char*)base + row * stride_bytes; }

tt_status check_plan(const tt_attn_desc* desc, const tt_partition_plan* plan, bool backward, Dims& dm) {
  if (!desc || !plan) return fail(TT_ERR_NULL, "desc / plan is NULL");
  // the whole-tree descriptor must be valid by itself (dtype, heads, d, strides, scale)
  if (tt_status s = tt::check_attn_desc(desc)) return s;
  if (desc->n_prefix != 0) return fail(TT_ERR_SHAPE, "the whole-tree descriptor must have n_prefix = 0, got %d", desc->n_prefix);
  if (plan->n_parts < 0 || plan->n_tokens != desc->n_q)
    return fail(TT_ERR_SHAPE, "plan covers %d tokens in %d partitions, descriptor has n_q=%d", plan->n_tokens, plan->n_parts, desc->n_q);
  if (plan->n_parts > 0 && (!plan->part_tok_off || !plan->part_prefix_off || !plan->part_ktile_off))
    return fail(TT_ERR_NULL, "a host offset table of the plan is NULL");
  dm.n = plan->n_tokens; dm.np = plan->n_parts; dm.hq = desc->hq;
  dm.esz = desc->dtype == TT_DTYPE_BF16 ? 2 : 4;
  dm.q_row = (size_t)desc->hq * desc->d * dm.esz;
  dm.kv_row = (size_t)desc->hkv * desc->d * dm.esz;
  dm.max_own = 0; dm.max_prefix = 0; dm.attn_ws = 0;
  for (int32_t p = 0; p < dm.np; p++) {
    const int64_t n_own = (int64_t)plan->part_tok_off[p + 1] - plan->part_tok_off[p];
    const int64_t n_pre = plan->part_prefix_off[p + 1] - plan->part_prefix_off[p];
    const int64_t n_kt = plan->part_ktile_off[p + 1] - plan->part_ktile_off[p];
    if (n_own < 0 || n_pre < 0 || n_own + n_pre >= INT32_MAX || plan->part_tok_off[p] < 0 || plan->part_tok_off[p + 1] > dm.n ||
        n_kt != tt::ceil_div(n_pre, TT_KTILE) + tt::ceil_div(n_own, TT_KTILE))
      return fail(TT_ERR_SHAPE, "plan offsets of partition %d are inconsistent", p);
    if (plan->part_own_start && plan->part_own_start[p] >= 0 && (int64_t)plan->part_own_start[p] + n_own > dm.n)
      return fail(TT_ERR_SHAPE, "part_own_start[%d]=%d runs past the last token", p, plan->part_own_start[p]);
    if (plan->part_prefix_start && plan->part_prefix_start[p] >= 0 && (int64_t)plan->part_prefix_start[p] + n_pre > dm.n)
      return fail(TT_ERR_SHAPE, "part_prefix_start[%d]=%d runs past the last token", p, plan->part_prefix_start[p]);
    dm.max_own = std::max<int32_t>(dm.max_own, (int32_t)n_own);
    dm.max_prefix = std::max<int32_t>(dm.max_prefix, (int32_t)n_pre);
    if (n_own > 0) {
      const tt_attn_desc d = part_desc(desc, (int32_t)n_own, (int32_t)n_pre);
      dm.attn_ws = std::max(dm.attn_ws, tt_tree_attn_workspace(&d, backward ? 1 : 0));
    }
  }
  if (dm.np == 0 && dm.n > 0) return fail(TT_ERR_SHAPE, "plan has no partitions for %d tokens", dm.n);
  if (dm.np > 0 && (plan->part_tok_off[0] != 0 || plan->part_tok_off[dm.np] != dm.n))
    return fail(TT_ERR_SHAPE, "plan's own-token offsets do not cover [0, %d)", dm.n);
  tt::clear_error();
  return TT_OK;
}

tt_status hip_ok(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return TT_OK;
  return fail(TT_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

struct Mover {
  hipStream_t st;
  void gather(const void* src, int64_t src_stride_bytes, const int32_t* idx, int64_t rows, size_t row_bytes, void* dst) const {
    if (rows == 0) return;
    tt::KernelTimer t(TT_KERNEL_PART_GATHER, st);
    const int vpr = (int)(row_bytes / 16);
    const int64_t n_vec = rows * vpr;
    gather_rows_kernel<<<blocks_for(n_vec), COPY_THREADS, 0, st>>>(n_vec, vpr, (const uint4*)src, src_stride_bytes / 16, idx, (uint4*)dst);
  }
  void scatter(const void* src, const int32_t* idx, int64_t rows, size_t row_bytes, void* dst) const {
    if (rows == 0) return;
    tt::KernelTimer t(TT_KERNEL_PART_SCATTER, st);
    const int vpr = (int)(row_bytes / 16);
    const int64_t n_vec = rows * vpr;
    scatter_rows_kernel<<<blocks_for(n_vec), COPY_THREADS, 0, st>>>(n_vec, vpr, (const uint4*)src, idx, (uint4*)dst);
  }
  void scatter_add(const float* src, const int32_t* idx, int64_t rows, size_t row_floats, float* dst) const {
    if (rows == 0) return;
    tt::KernelTimer t(TT_KERNEL_PART_SCATTER, st);
    const int vpr = (int)(row_floats / 4);
    const int64_t n_vec = rows * vpr;
    scatter_add_rows_kernel<<<blocks_for(n_vec), COPY_THREADS, 0, st>>>(n_vec, vpr, (const float4*)src, idx, (float4*)dst);
  }
  void zero(void* dst, size_t bytes) const {
    if (bytes == 0) return;
    tt::KernelTimer t(TT_KERNEL_PART_SCATTER, st);
    fill_zero_kernel<<<blocks_for((int64_t)(bytes / 16)), COPY_THREADS, 0, st>>>((int64_t)(bytes / 16), (uint4*)dst);
  }
  void lse_gather(const float* whole, int n_whole, const int32_t* idx, int n_local, int heads, float* local) const {
    tt::KernelTimer t(TT_KERNEL_PART_GATHER, st);
    lse_move_kernel<true><<<dim3(blocks_for(n_local), heads), COPY_THREADS, 0, st>>>(n_local, n_whole, heads, idx, whole, local);
  }
  void lse_scatter(const float* local, int n_local, const int32_t* idx, int n_whole, int heads, float* whole) const {
    tt::KernelTimer t(TT_KERNEL_PART_SCATTER, st);
    lse_move_kernel<false><<<dim3(blocks_for(n_local), heads), COPY_THREADS, 0, st>>>(n_local, n_whole, heads, idx, local, whole);
  }
};

int64_t stride_bytes(int64_t stride_tok, int heads, int d, size_t esz) {
  return (stride_tok ? stride_tok : (int64_t)heads * d) * (int64_t)esz;
}

tt_status check_tensors(const tt_attn_desc* desc, const tt_partition_plan* plan, std::initializer_list<const void*> ptrs) {
  if (desc->n_q == 0) return TT_OK;
  for (const void* p : ptrs) {
    if (!p) return fail(TT_ERR_NULL, "a tensor pointer is NULL");
    if (!tt::aligned16(p)) return fail(TT_ERR_ALIGN, "device pointer %p is not 16-byte aligned", p);
  }
  if (!plan->own_tok || !plan->kend || !plan->kt_min || !plan->kt_max) return fail(TT_ERR_NULL, "a device array of the plan is NULL");
  if (plan->part_prefix_off[plan->n_parts] > 0 && !plan->prefix_tok) return fail(TT_ERR_NULL, "plan->prefix_tok is NULL");
  return TT_OK;
}

}  // namespace
}  // namespace tt

using namespace tt;

extern "C" size_t tt_tree_attn_partitioned_workspace(const tt_attn_desc* desc, const tt_partition_plan* plan, int32_t backward) {
  tt::clear_error();
  Dims dm;
  if (check_plan(desc, plan, backward != 0, dm) != TT_OK) return 0;
  return carve(nullptr, dm, backward != 0).total;
}

extern "C" tt_status tt_tree_attn_partitioned_fwd(const tt_attn_desc* desc, const tt_partition_plan* plan,
                                                  const void* q, const void* k, const void* v, void* o, float* lse,
                                                  void* workspace, size_t workspace_bytes, void* stream) {
  tt::clear_error();
  Dims dm;
  if (tt_status s = check_plan(desc, plan, false, dm)) return s;
  if (tt_status s = check_tensors(desc, plan, {q, k, v, o, (const void*)lse})) return s;
  const Buffers b = carve(workspace, dm, false);
  if (!workspace || !tt::aligned16(workspace) || workspace_bytes < b.total)
    return fail(TT_ERR_WORKSPACE, "partitioned forward needs %zu bytes of 16-byte aligned workspace, got %zu", b.total, workspace_bytes);
  const Mover mv{(hipStream_t)stream};
  const int64_t qs = stride_bytes(desc->q_stride_tok, desc->hq, desc->d, dm.esz);
  const int64_t ks = stride_bytes(desc->k_stride_tok, desc->hkv, desc->d, dm.esz);
  const int64_t vs = stride_bytes(desc->v_stride_tok, desc->hkv, desc->d, dm.esz);
  const bool kv_contig = ks == (int64_t)dm.kv_row && vs == (int64_t)dm.kv_row;
  for (int32_t p = 0; p < dm.np; p++) {
    const Part x = part_of(plan, p, kv_contig);
    if (x.n_own == 0) continue;
    const int32_t* own = plan->own_tok + x.t0;
    const int32_t* pre = x.n_pre ? plan->prefix_tok + x.p0 : nullptr;
    const bool own_ip = x.own_start >= 0, pre_ip = x.pre_start >= 0;
    const void *qp = b.q, *kp = b.k, *vp = b.v, *kpre = nullptr, *vpre = nullptr;
    void* op = b.o;
    if (own_ip) {
      qp = row_ptr(q, x.own_start, qs); kp = row_ptr(k, x.own_start, ks); vp = row_ptr(v, x.own_start, vs);
      op = row_ptr(o, x.own_start, (int64_t)dm.q_row);
    } else {
      mv.gather(q, qs, own, x.n_own, dm.q_row, b.q);
      mv.gather(k, ks, own, x.n_own, dm.kv_row, b.k);
      mv.gather(v, vs, own, x.n_own, dm.kv_row, b.v);
    }
    if (pre_ip) {
      kpre = row_ptr(k, x.pre_start, ks); vpre = row_ptr(v, x.pre_start, vs);
    } else if (x.n_pre) {
      mv.gather(k, ks, pre, x.n_pre, dm.kv_row, b.kp);
      mv.gather(v, vs, pre, x.n_pre, dm.kv_row, b.vp);
      kpre = b.kp; vpre = b.vp;
    }
    if (tt_status s = hip_ok("partition gather")) return s;
    const tt_attn_desc d = part_desc(desc, x.n_own, x.n_pre, own_ip);
    if (tt_status s = tt_tree_attn_fwd(&d, qp, kp, vp, kpre, vpre,
                                       plan->kend + x.p0 + x.t0, plan->kt_min + plan->part_ktile_off[p],
                                       plan->kt_max + plan->part_ktile_off[p], op, b.lse, b.attn_ws, dm.attn_ws, stream))
      return s;
    if (!own_ip) mv.scatter(b.o, own, x.n_own, dm.q_row, o);
    mv.lse_scatter(b.lse, x.n_own, own, dm.n, desc->hq, lse);
    if (tt_status s = hip_ok("partition scatter")) return s;
  }
  return TT_OK;
}

extern "C" tt_status tt_tree_attn_partitioned_bwd(const tt_attn_desc* desc, const tt_partition_plan* plan,
                                                  const void* q, const void* k, const void* v,
                                                  const void* o, const void* d_o, const float* lse,
                                                  void* dq, void* dk, void* dv,
                                                  void* workspace, size_t workspace_bytes, void* stream) {
  tt::clear_error();
  Dims dm;
  if (tt_status s = check_plan(desc, plan, true, dm)) return s;
  if (tt_status s = check_tensors(desc, plan, {q, k, v, o, d_o, (const void*)lse, (const void*)dq, (const void*)dk, (const void*)dv})) return s;
  const Buffers b = carve(workspace, dm, true);
  if (!workspace || !tt::aligned16(workspace) || workspace_bytes < b.total)
    return fail(TT_ERR_WORKSPACE, "partitioned backward needs %zu bytes of 16-byte aligned workspace, got %zu", b.total, workspace_bytes);
  const Mover mv{(hipStream_t)stream};
  const int64_t qs = stride_bytes(desc->q_stride_tok, desc->hq, desc->d, dm.esz);
  const int64_t ks = stride_bytes(desc->k_stride_tok, desc->hkv, desc->d, dm.esz);
  const int64_t vs = stride_bytes(desc->v_stride_tok, desc->hkv, desc->d, dm.esz);
  const size_t kv_floats = (size_t)desc->hkv * desc->d;
  const bool any_prefix = dm.max_prefix > 0;
  if (any_prefix) {
    mv.zero(b.acc_dk, (size_t)dm.n * kv_floats * sizeof(float));
    mv.zero(b.acc_dv, (size_t)dm.n * kv_floats * sizeof(float));
  }
  const bool kv_contig = ks == (int64_t)dm.kv_row && vs == (int64_t)dm.kv_row;
  for (int32_t p = dm.np - 1; p >= 0; p--) {          // children before parents
    const Part x = part_of(plan, p, kv_contig);
    if (x.n_own == 0) continue;
    const int32_t* own = plan->own_tok + x.t0;
    const int32_t* pre = x.n_pre ? plan->prefix_tok + x.p0 : nullptr;
    const bool own_ip = x.own_start >= 0, pre_ip = x.pre_start >= 0;
    const void *qp = b.q, *kp = b.k, *vp = b.v, *op = b.o, *dop = b.d_o, *kpre = nullptr, *vpre = nullptr;
    void *dqp = b.dq, *dkp = b.dk, *dvp = b.dv;
    float *dk_acc = nullptr, *dv_acc = nullptr;
    if (own_ip) {
      qp = row_ptr(q, x.own_start, qs); kp = row_ptr(k, x.own_start, ks); vp = row_ptr(v, x.own_start, vs);
      op = row_ptr(o, x.own_start, (int64_t)dm.q_row); dop = row_ptr(d_o, x.own_start, (int64_t)dm.q_row);
      dqp = row_ptr(dq, x.own_start, (int64_t)dm.q_row);
      dkp = row_ptr(dk, x.own_start, (int64_t)dm.kv_row); dvp = row_ptr(dv, x.own_start, (int64_t)dm.kv_row);
    } else {
      mv.gather(q, qs, own, x.n_own, dm.q_row, b.q);
      mv.gather(k, ks, own, x.n_own, dm.kv_row, b.k);
      mv.gather(v, vs, own, x.n_own, dm.kv_row, b.v);
      mv.gather(o, (int64_t)dm.q_row, own, x.n_own, dm.q_row, b.o);
      mv.gather(d_o, (int64_t)dm.q_row, own, x.n_own, dm.q_row, b.d_o);
    }
    mv.lse_gather(lse, dm.n, own, x.n_own, desc->hq, b.lse);
    if (pre_ip) {
      // the kernels add straight into the whole-tree fp32 accumulators
      kpre = row_ptr(k, x.pre_start, ks); vpre = row_ptr(v, x.pre_start, vs);
      dk_acc = b.acc_dk + (size_t)x.pre_start * kv_floats; dv_acc = b.acc_dv + (size_t)x.pre_start * kv_floats;
    } else if (x.n_pre) {
      mv.gather(k, ks, pre, x.n_pre, dm.kv_row, b.kp);
      mv.gather(v, vs, pre, x.n_pre, dm.kv_row, b.vp);
      mv.zero(b.dkp, (size_t)x.n_pre * kv_floats * sizeof(float));
      mv.zero(b.dvp, (size_t)x.n_pre * kv_floats * sizeof(float));
      kpre = b.kp; vpre = b.vp; dk_acc = b.dkp; dv_acc = b.dvp;
    }
    if (tt_status s = hip_ok("partition gather")) return s;
    const tt_attn_desc d = part_desc(desc, x.n_own, x.n_pre, own_ip);
    if (tt_status s = tt_tree_attn_bwd(&d, qp, kp, vp, kpre, vpre,
                                       plan->kend + x.p0 + x.t0, plan->kt_min + plan->part_ktile_off[p],
                                       plan->kt_max + plan->part_ktile_off[p], op, dop, b.lse, dqp, dkp, dvp,
                                       dk_acc, dv_acc, b.attn_ws, dm.attn_ws, stream))
      return s;
    if (!own_ip) {
      mv.scatter(b.dq, own, x.n_own, dm.q_row, dq);
      mv.scatter(b.dk, own, x.n_own, dm.kv_row, dk);
      mv.scatter(b.dv, own, x.n_own, dm.kv_row, dv);
    }
    if (!pre_ip && x.n_pre) {
      mv.scatter_add(b.dkp, pre, x.n_pre, kv_floats, b.acc_dk);
      mv.scatter_add(b.dvp, pre, x.n_pre, kv_floats, b.acc_dv);
    }
    if (tt_status s = hip_ok("partition scatter")) return s;
  }
  if (any_prefix && dm.n > 0) {
    tt::KernelTimer t(TT_KERNEL_PART_SCATTER, (hipStream_t)stream);
    const int64_t n_quads = (int64_t)dm.n * (int64_t)kv_floats / 4;
    if (dm.esz == 2) {
      finalize_kernel<true><<<blocks_for(n_quads), COPY_THREADS, 0, (hipStream_t)stream>>>(n_quads, dk, (const float4*)b.acc_dk);
      finalize_kernel<true><<<blocks_for(n_quads), COPY_THREADS, 0, (hipStream_t)stream>>>(n_quads, dv, (const float4*)b.acc_dv);
    } else {
      finalize_kernel<false><<<blocks_for(n_quads), COPY_THREADS, 0, (hipStream_t)stream>>>(n_quads, dk, (const float4*)b.acc_dk);
      finalize_kernel<false><<<blocks_for(n_quads), COPY_THREADS, 0, (hipStream_t)stream>>>(n_quads, dv, (const float4*)b.acc_dv);
    }
    if (tt_status s = hip_ok("partition finalize")) return s;
  }
  return TT_OK;
}
