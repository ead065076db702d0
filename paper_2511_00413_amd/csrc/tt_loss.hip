// Fused log-softmax / gather / loss weighting (paper Eq. 4: L_tree = sum_t (g_t/K) * l_t with
// l_t = -log p(y_t | x_<=t); "Loss Weights" paragraph: one multiply per token).
//
// HBM-bound: each logits row is streamed from memory exactly once with 16-byte loads; every
// thread keeps an online (max, sum-of-exp) pair in base 2, the pairs are merged across the
// workgroup, and the target logit is fetched separately (one element).  The weighted sum over
// rows is a second, single-workgroup kernel that adds the rows in a fixed order in fp64, so the
// loss is bit-reproducible.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <hip/hip_bf16.h>
#include "tt_kernels.h"

namespace tt {
namespace {

constexpr int LOSS_THREADS = 256;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct MS { float m, s; };   // running max (natural units) and sum of exp(z - m)

// 2^x as the bare hardware instruction: every argument here is <= 0, and a term below 2^-126 may
// flush to zero (it could not change a sum whose largest term is 1).  The library exp2f spends
// several more instructions per element on that range, which made the kernel ALU-bound.
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ MS merge(MS a, MS b) {
  const float m = fmaxf(a.m, b.m);
  // exp2(-inf) = 0 handles empty partners; (-inf) - (-inf) is avoided by the select
  const float sa = a.m == -INFINITY ? 0.f : a.s * ex2((a.m - m) * LOG2E);
  const float sb = b.m == -INFINITY ? 0.f : b.s * ex2((b.m - m) * LOG2E);
  return {m, sa + sb};
}

__device__ __forceinline__ void push8(MS& st, const float (&z)[8]) {  // z may hold -inf (masked vocabulary entries)
  float vm = fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])), fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7])));
  const float m_new = fmaxf(st.m, vm);
  const float mref = m_new == -INFINITY ? 0.f : m_new;      // all -inf so far: keep the sum at 0, no NaN
  // the difference is taken before the scaling so that large |z| loses nothing
  float acc = st.m == -INFINITY ? 0.f : st.s * ex2((st.m - mref) * LOG2E);
#pragma unroll
  for (int e = 0; e < 8; e++) acc += ex2((z[e] - mref) * LOG2E);
  st.m = m_new;
  st.s = acc;
}

__device__ __forceinline__ void push1(MS& st, float z) {
  const float m_new = fmaxf(st.m, z);
  const float old = st.m == -INFINITY ? 0.f : st.s * ex2((st.m - m_new) * LOG2E);
  st.s = old + ex2((z - m_new) * LOG2E);
  st.m = m_new;
}

__device__ __forceinline__ float elem(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float elem(const __hip_bfloat16* p, int64_t i) { return __bfloat162float(p[i]); }

__device__ __forceinline__ void unpack8(const u32x4& v, float (&z)[8]) {
  // bf16 -> fp32 is a 16-bit shift
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; i++) {
    z[2 * i] = __uint_as_float(w[i] << 16);
    z[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

// One workgroup per row.  T = float: a 16-byte load holds 4 elements (two loads per push8).
template <typename T>
__global__ void __launch_bounds__(LOSS_THREADS)
row_logprob_kernel(int vocab, const T* __restrict__ logits, int64_t row_stride,
                   const int32_t* __restrict__ target, float* __restrict__ logp, float* __restrict__ lse_out) {
  constexpr int EPV = 16 / sizeof(T);               // elements per 16-byte vector
  const int64_t r = blockIdx.x;
  const T* row = logits + r * row_stride;
  const int t = threadIdx.x;
  // split the row into [0, head) scalar, [head, head + nvec*EPV) vector, rest scalar
  const uintptr_t addr = reinterpret_cast<uintptr_t>(row);
  int head = (int)(((16 - (addr & 15)) & 15) / sizeof(T));
  head = head < vocab ? head : vocab;
  const int nvec = (vocab - head) / EPV;
  const int tail0 = head + nvec * EPV;
  MS st = {-INFINITY, 0.f};
  const u32x4* vp = reinterpret_cast<const u32x4*>(row + head);
  if constexpr (sizeof(T) == 2) {
    int i = t;
    // 4 loads in flight per thread
    for (; i + 3 * LOSS_THREADS < nvec; i += 4 * LOSS_THREADS) {
      const u32x4 v0 = __builtin_nontemporal_load(vp + i);
      const u32x4 v1 = __builtin_nontemporal_load(vp + i + LOSS_THREADS);
      const u32x4 v2 = __builtin_nontemporal_load(vp + i + 2 * LOSS_THREADS);
      const u32x4 v3 = __builtin_nontemporal_load(vp + i + 3 * LOSS_THREADS);
      float z[8];
      unpack8(v0, z); push8(st, z);
      unpack8(v1, z); push8(st, z);
      unpack8(v2, z); push8(st, z);
      unpack8(v3, z); push8(st, z);
    }
    for (; i < nvec; i += LOSS_THREADS) {
      const u32x4 v0 = __builtin_nontemporal_load(vp + i);
      float z[8];
      unpack8(v0, z); push8(st, z);
    }
  } else {
    int i = t;
    for (; i + LOSS_THREADS < nvec; i += 2 * LOSS_THREADS) {
      const u32x4 v0 = __builtin_nontemporal_load(vp + i);
      const u32x4 v1 = __builtin_nontemporal_load(vp + i + LOSS_THREADS);
      const float z[8] = {__uint_as_float(v0.x), __uint_as_float(v0.y), __uint_as_float(v0.z), __uint_as_float(v0.w),
                          __uint_as_float(v1.x), __uint_as_float(v1.y), __uint_as_float(v1.z), __uint_as_float(v1.w)};
      push8(st, z);
    }
    for (; i < nvec; i += LOSS_THREADS) {
      const u32x4 v0 = __builtin_nontemporal_load(vp + i);
      push1(st, __uint_as_float(v0.x)); push1(st, __uint_as_float(v0.y));
      push1(st, __uint_as_float(v0.z)); push1(st, __uint_as_float(v0.w));
    }
  }
  for (int e = t; e < head; e += LOSS_THREADS) push1(st, elem(row, e));
  for (int e = tail0 + t; e < vocab; e += LOSS_THREADS) push1(st, elem(row, e));

  // merge across the wavefront, then across the 4 wavefronts
  for (int o = 32; o > 0; o >>= 1) {
    MS other = {__shfl_xor(st.m, o), __shfl_xor(st.s, o)};
    st = merge(st, other);
  }
  __shared__ MS part[LOSS_THREADS / 64];
  if ((t & 63) == 0) part[t >> 6] = st;
  __syncthreads();
  if (t == 0) {
    MS a = part[0];
    for (int w = 1; w < LOSS_THREADS / 64; w++) a = merge(a, part[w]);
    const float ln_s = LN2 * log2f(a.s);
    const float lse = a.m + ln_s;
    const int32_t y = target[r];
    // (z_y - m) - ln(sum) keeps full precision when |m| is large
    logp[r] = (y >= 0 && y < vocab) ? (elem(row, y) - a.m) - ln_s : 0.f;
    if (lse_out) lse_out[r] = lse;
  }
}

// loss_acc += sum_r weight_r * (-logp_r), rows added in a fixed order (fp64 partials).
__global__ void __launch_bounds__(1024)
weighted_sum_kernel(int64_t n_rows, const float* __restrict__ logp, const float* __restrict__ weight,
                    const int32_t* __restrict__ target, float* __restrict__ loss_acc) {
  __shared__ double part[1024];
  double acc = 0.0;
  for (int64_t r = threadIdx.x; r < n_rows; r += 1024) {
    const float w = weight ? weight[r] : 1.f;
    if (target[r] >= 0 && w != 0.f) acc += (double)w * (double)(-logp[r]);
  }
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 512; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss_acc = (float)((double)*loss_acc + part[0]);
}

// ---- backward: dlogits = grad_scale * weight * (softmax - onehot) --------------------------------
typedef float f32x8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));

// w_r (exp(z - lse) - [v == y]) for the 8 (bf16) or 4 (fp32) elements of one 16-byte vector whose
// first element has index `base` in the row
__device__ __forceinline__ u32x4 grad_vec_bf16(const u32x4& v, float lse, float w, int base, int y) {
  float z[8];
  unpack8(v, z);
  f32x8v g;
#pragma unroll
  for (int e = 0; e < 8; e++) g[e] = w * ex2((z[e] - lse) * LOG2E);
  if ((unsigned)(y - base) < 8u) {              // the target element lives in this vector (at most once per row)
#pragma unroll
    for (int e = 0; e < 8; e++) g[e] -= (base + e == y) ? w : 0.f;
  }
  const bf16x8v b = __builtin_convertvector(g, bf16x8v);     // round to nearest even
  return __builtin_bit_cast(u32x4, b);
}
__device__ __forceinline__ u32x4 grad_vec_f32(const u32x4& v, float lse, float w, int base, int y) {
  const float z[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
  float g[4];
#pragma unroll
  for (int e = 0; e < 4; e++) g[e] = w * ex2((z[e] - lse) * LOG2E) - ((base + e == y) ? w : 0.f);
  u32x4 o;
  o.x = __float_as_uint(g[0]); o.y = __float_as_uint(g[1]); o.z = __float_as_uint(g[2]); o.w = __float_as_uint(g[3]);
  return o;
}
__device__ __forceinline__ void store_elem(float* p, int64_t i, float g) { p[i] = g; }
__device__ __forceinline__ void store_elem(__hip_bfloat16* p, int64_t i, float g) { p[i] = __float2bfloat16(g); }

// A row is cut into gridDim.y parts of `part_vecs` 16-byte vectors (a multiple of the workgroup size) and one
// workgroup handles one part: one 16-byte load and one 16-byte store per vector, four vectors in flight.  Many
// small workgroups stream faster than one per row here (a bare one-read-one-write stream measures 6.4 TB/s with
// 16 KB per workgroup against 5.9 with long grid-stride loops).  The last part also does the row's scalar tail.
template <typename T>
__global__ void __launch_bounds__(LOSS_THREADS)
row_dlogits_kernel(int vocab, const T* logits, int64_t row_stride, const int32_t* __restrict__ target,
                   const float* __restrict__ weight, const float* __restrict__ lse_in, float grad_scale,
                   T* dlogits, int64_t out_stride, int part_vecs) {
  constexpr int EPV = 16 / sizeof(T);
  const int64_t r = blockIdx.x;
  const T* row = logits + r * row_stride;
  T* out = dlogits + r * out_stride;
  const int t = threadIdx.x;
  const int y = target[r];
  // A row whose target is negative or not below the vocabulary size is ignored, as in the forward (logp = 0,
  // nothing added to the loss): its gradient is exactly zero -- weight 0 and lse = +inf, so that every
  // exponential is 0 whatever the logits and whatever the caller left in lse[r].
  const bool used = y >= 0 && y < vocab;
  const float w = used ? grad_scale * (weight ? weight[r] : 1.f) : 0.f;
  const float lse = used ? lse_in[r] : INFINITY;
  const bool vec_ok = ((reinterpret_cast<uintptr_t>(row) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
  const int nvec = vec_ok ? vocab / EPV : 0;
  const u32x4* vp = reinterpret_cast<const u32x4*>(row);
  u32x4* op = reinterpret_cast<u32x4*>(out);
  auto grad = [&](const u32x4& v, int i) {
    if constexpr (sizeof(T) == 2) return grad_vec_bf16(v, lse, w, i * EPV, y);
    else return grad_vec_f32(v, lse, w, i * EPV, y);
  };
  const int v_end = min(nvec, ((int)blockIdx.y + 1) * part_vecs);
  int i = (int)blockIdx.y * part_vecs + t;
  for (; i + 3 * LOSS_THREADS < v_end; i += 4 * LOSS_THREADS) {
    const u32x4 v0 = __builtin_nontemporal_load(vp + i);
    const u32x4 v1 = __builtin_nontemporal_load(vp + i + LOSS_THREADS);
    const u32x4 v2 = __builtin_nontemporal_load(vp + i + 2 * LOSS_THREADS);
    const u32x4 v3 = __builtin_nontemporal_load(vp + i + 3 * LOSS_THREADS);
    __builtin_nontemporal_store(grad(v0, i), op + i);
    __builtin_nontemporal_store(grad(v1, i + LOSS_THREADS), op + i + LOSS_THREADS);
    __builtin_nontemporal_store(grad(v2, i + 2 * LOSS_THREADS), op + i + 2 * LOSS_THREADS);
    __builtin_nontemporal_store(grad(v3, i + 3 * LOSS_THREADS), op + i + 3 * LOSS_THREADS);
  }
  for (; i < v_end; i += LOSS_THREADS) {
    const u32x4 v0 = __builtin_nontemporal_load(vp + i);
    __builtin_nontemporal_store(grad(v0, i), op + i);
  }
  // the rest of the row (everything, for a row that is not 16-byte aligned), element by element
  if (blockIdx.y == gridDim.y - 1)
    for (int e = nvec * EPV + t; e < vocab; e += LOSS_THREADS) {
      const float g = w * ex2((elem(row, e) - lse) * LOG2E) - (e == y ? w : 0.f);
      store_elem(out, e, g);
    }
}

// ---- forward and backward in one pass ----------------------------------------------------------------
// When the gradient is wanted together with the loss (the usual training step), a row is read from memory
// once: the workgroup streams it, keeps its first `lds_vecs` 16-byte vectors in LDS while it accumulates
// (max, sum of exp), and then forms the gradient from that copy; what did not fit (a vocabulary beyond
// FUSED_LDS_BYTES per row) is read a second time, right behind the first read, so that it mostly comes out of
// the caches.  Both the row and the gradient row must start on a 16-byte boundary (the host checks that and
// uses the two separate kernels otherwise).  Same arithmetic per element as the separate kernels.
constexpr int FUSED_THREADS = 512;
constexpr int FUSED_LDS_BYTES = 64 * 1024;             // two workgroups per compute unit

template <typename T>
__global__ void __launch_bounds__(FUSED_THREADS)
row_logprob_dlogits_kernel(int vocab, const T* logits, int64_t row_stride, const int32_t* __restrict__ target,
                           const float* __restrict__ weight, float grad_scale, float* __restrict__ logp,
                           float* __restrict__ lse_out, T* dlogits, int64_t out_stride, int lds_vecs) {
  constexpr int EPV = 16 / sizeof(T);
  extern __shared__ u32x4 rowbuf[];
  __shared__ MS part[FUSED_THREADS / 64];
  __shared__ float row_stat[2];                        // max, ln(sum)
  const int64_t r = blockIdx.x;
  const T* row = logits + r * row_stride;
  T* out = dlogits + r * out_stride;
  const int t = threadIdx.x;
  const int nvec = vocab / EPV;
  const u32x4* vp = reinterpret_cast<const u32x4*>(row);
  u32x4* op = reinterpret_cast<u32x4*>(out);
  const int y = target[r];
  const bool used = y >= 0 && y < vocab;
  const float w = used ? grad_scale * (weight ? weight[r] : 1.f) : 0.f;

  // ---- pass 1: statistics; the part of the row that is kept goes to LDS ----
  MS st = {-INFINITY, 0.f};
  auto push_vec = [&](const u32x4& v) {
    if constexpr (sizeof(T) == 2) {
      float z[8];
      unpack8(v, z);
      push8(st, z);
    } else {
      push1(st, __uint_as_float(v.x)); push1(st, __uint_as_float(v.y));
      push1(st, __uint_as_float(v.z)); push1(st, __uint_as_float(v.w));
    }
  };
  const int n_kept = min(nvec, lds_vecs);
  {
    int i = t;
    for (; i + 3 * FUSED_THREADS < n_kept; i += 4 * FUSED_THREADS) {      // 4 loads in flight per thread
      const u32x4 v0 = __builtin_nontemporal_load(vp + i);
      const u32x4 v1 = __builtin_nontemporal_load(vp + i + FUSED_THREADS);
      const u32x4 v2 = __builtin_nontemporal_load(vp + i + 2 * FUSED_THREADS);
      const u32x4 v3 = __builtin_nontemporal_load(vp + i + 3 * FUSED_THREADS);
      rowbuf[i] = v0; rowbuf[i + FUSED_THREADS] = v1; rowbuf[i + 2 * FUSED_THREADS] = v2; rowbuf[i + 3 * FUSED_THREADS] = v3;
      push_vec(v0); push_vec(v1); push_vec(v2); push_vec(v3);
    }
    for (; i < n_kept; i += FUSED_THREADS) {
      const u32x4 v0 = __builtin_nontemporal_load(vp + i);
      rowbuf[i] = v0;
      push_vec(v0);
    }
  }
  {
    int i = n_kept + t;                                 // the rest: ordinary loads, they are wanted again soon
    for (; i + 3 * FUSED_THREADS < nvec; i += 4 * FUSED_THREADS) {
      const u32x4 v0 = vp[i], v1 = vp[i + FUSED_THREADS], v2 = vp[i + 2 * FUSED_THREADS], v3 = vp[i + 3 * FUSED_THREADS];
      push_vec(v0); push_vec(v1); push_vec(v2); push_vec(v3);
    }
    for (; i < nvec; i += FUSED_THREADS) push_vec(vp[i]);
  }
  for (int e = nvec * EPV + t; e < vocab; e += FUSED_THREADS) push1(st, elem(row, e));
  for (int o = 32; o > 0; o >>= 1) {
    MS other = {__shfl_xor(st.m, o), __shfl_xor(st.s, o)};
    st = merge(st, other);
  }
  if ((t & 63) == 0) part[t >> 6] = st;
  __syncthreads();
  if (t == 0) {
    MS a = part[0];
    for (int wv = 1; wv < FUSED_THREADS / 64; wv++) a = merge(a, part[wv]);
    const float ln_s = LN2 * log2f(a.s);
    row_stat[0] = a.m; row_stat[1] = ln_s;
    logp[r] = used ? (elem(row, y) - a.m) - ln_s : 0.f;
    if (lse_out) lse_out[r] = a.m + ln_s;
  }
  __syncthreads();                                      // also: every kept vector is in LDS
  // an ignored row gets an exactly zero gradient whatever its logits are (weight 0, lse = +inf)
  const float lse = used ? row_stat[0] + row_stat[1] : INFINITY;

  // ---- pass 2: gradient ----
  auto grad = [&](const u32x4& v, int i) {
    if constexpr (sizeof(T) == 2) return grad_vec_bf16(v, lse, w, i * EPV, y);
    else return grad_vec_f32(v, lse, w, i * EPV, y);
  };
  for (int i = t; i < n_kept; i += FUSED_THREADS) __builtin_nontemporal_store(grad(rowbuf[i], i), op + i);
  {
    int i = n_kept + t;
    for (; i + 3 * FUSED_THREADS < nvec; i += 4 * FUSED_THREADS) {
      const u32x4 v0 = __builtin_nontemporal_load(vp + i);
      const u32x4 v1 = __builtin_nontemporal_load(vp + i + FUSED_THREADS);
      const u32x4 v2 = __builtin_nontemporal_load(vp + i + 2 * FUSED_THREADS);
      const u32x4 v3 = __builtin_nontemporal_load(vp + i + 3 * FUSED_THREADS);
      __builtin_nontemporal_store(grad(v0, i), op + i);
      __builtin_nontemporal_store(grad(v1, i + FUSED_THREADS), op + i + FUSED_THREADS);
      __builtin_nontemporal_store(grad(v2, i + 2 * FUSED_THREADS), op + i + 2 * FUSED_THREADS);
      __builtin_nontemporal_store(grad(v3, i + 3 * FUSED_THREADS), op + i + 3 * FUSED_THREADS);
    }
    for (; i < nvec; i += FUSED_THREADS) {
      const u32x4 v0 = __builtin_nontemporal_load(vp + i);
      __builtin_nontemporal_store(grad(v0, i), op + i);
    }
  }
  for (int e = nvec * EPV + t; e < vocab; e += FUSED_THREADS) {
    const float g = w * ex2((elem(row, e) - lse) * LOG2E) - (e == y ? w : 0.f);
    store_elem(out, e, g);
  }
}

}  // namespace

bool weighted_logprob_fused_ok(bool bf16, const void* logits, int64_t row_stride, const void* dlogits, int64_t out_stride) {
  const int esz = bf16 ? 2 : 4;
  return ((reinterpret_cast<uintptr_t>(logits) | reinterpret_cast<uintptr_t>(dlogits)) & 15) == 0 && (row_stride * esz) % 16 == 0 &&
         (out_stride * esz) % 16 == 0;
}

hipError_t weighted_logprob_fused(int64_t n_rows, int vocab, bool bf16, const void* logits, int64_t row_stride,
                                  const int32_t* target, const float* weight, float grad_scale, float* logp, float* lse,
                                  float* loss_acc, void* dlogits, int64_t out_stride, hipStream_t st) {
  if (n_rows == 0) return hipSuccess;
  const int nvec = vocab / (bf16 ? 8 : 4);
  const int lds_vecs = std::min(nvec, FUSED_LDS_BYTES / 16);
  const size_t lds = (size_t)lds_vecs * 16;
  {
    KernelTimer timer(TT_KERNEL_LOSS_FUSED, st);
    if (bf16) {
      if (hipError_t e = hipFuncSetAttribute((const void*)row_logprob_dlogits_kernel<__hip_bfloat16>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, FUSED_LDS_BYTES))
        return e;
      row_logprob_dlogits_kernel<__hip_bfloat16><<<(unsigned)n_rows, FUSED_THREADS, lds, st>>>(
          vocab, (const __hip_bfloat16*)logits, row_stride, target, weight, grad_scale, logp, lse, (__hip_bfloat16*)dlogits,
          out_stride, lds_vecs);
    } else {
      if (hipError_t e = hipFuncSetAttribute((const void*)row_logprob_dlogits_kernel<float>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, FUSED_LDS_BYTES))
        return e;
      row_logprob_dlogits_kernel<float><<<(unsigned)n_rows, FUSED_THREADS, lds, st>>>(
          vocab, (const float*)logits, row_stride, target, weight, grad_scale, logp, lse, (float*)dlogits, out_stride, lds_vecs);
    }
  }
  if (hipError_t e = hipGetLastError()) return e;
  if (loss_acc) {
    KernelTimer timer(TT_KERNEL_LOSS_SUM, st);
    weighted_sum_kernel<<<1, 1024, 0, st>>>(n_rows, logp, weight, target, loss_acc);
    return hipGetLastError();
  }
  return hipSuccess;
}

hipError_t weighted_logprob(int64_t n_rows, int vocab, bool bf16, const void* logits, int64_t row_stride,
                            const int32_t* target, const float* weight, float* logp, float* lse,
                            float* loss_acc, hipStream_t st) {
  if (n_rows == 0) return hipSuccess;
  // grid.x is limited to 2^31-1 workgroups; rows beyond that are rejected by the API layer
  {
  KernelTimer timer(TT_KERNEL_LOSS_ROWS, st);
  if (bf16)
    row_logprob_kernel<__hip_bfloat16><<<(unsigned)n_rows, LOSS_THREADS, 0, st>>>(
        vocab, (const __hip_bfloat16*)logits, row_stride, target, logp, lse);
  else
    row_logprob_kernel<float><<<(unsigned)n_rows, LOSS_THREADS, 0, st>>>(
        vocab, (const float*)logits, row_stride, target, logp, lse);
  }
  if (hipError_t e = hipGetLastError()) return e;
  if (loss_acc) {
    KernelTimer timer(TT_KERNEL_LOSS_SUM, st);
    weighted_sum_kernel<<<1, 1024, 0, st>>>(n_rows, logp, weight, target, loss_acc);
    return hipGetLastError();
  }
  return hipSuccess;
}

hipError_t weighted_logprob_bwd(int64_t n_rows, int vocab, bool bf16, const void* logits, int64_t row_stride,
                                const int32_t* target, const float* weight, const float* lse, float grad_scale,
                                void* dlogits, int64_t out_stride, hipStream_t st) {
  if (n_rows == 0) return hipSuccess;
  // parts of 4 vectors per thread (16 KB), at most 65535 of them (grid.y limit); a part is a multiple of the
  // workgroup size so that the four-in-flight loop keeps its stride pattern
  const int nvec = vocab / (bf16 ? 8 : 4);
  int part_vecs = 4 * LOSS_THREADS;
  while ((nvec + part_vecs - 1) / part_vecs > 65535) part_vecs *= 2;
  const unsigned parts = (unsigned)std::max(1, (nvec + part_vecs - 1) / part_vecs);
  const dim3 grid((unsigned)n_rows, parts);
  KernelTimer timer(TT_KERNEL_LOSS_BWD, st);
  if (bf16)
    row_dlogits_kernel<__hip_bfloat16><<<grid, LOSS_THREADS, 0, st>>>(
        vocab, (const __hip_bfloat16*)logits, row_stride, target, weight, lse, grad_scale, (__hip_bfloat16*)dlogits, out_stride,
        part_vecs);
  else
    row_dlogits_kernel<float><<<grid, LOSS_THREADS, 0, st>>>(
        vocab, (const float*)logits, row_stride, target, weight, lse, grad_scale, (float*)dlogits, out_stride, part_vecs);
  return hipGetLastError();
}

}  // namespace tt
