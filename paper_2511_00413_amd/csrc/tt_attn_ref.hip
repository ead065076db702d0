// Reference-grade tree attention kernels: plain fp32 arithmetic, one wavefront per query row
// (forward, dQ) or per key (dK/dV), no matrix cores.  This is the TT_DTYPE_FP32 path of the
// library (the paper verifies its gradients in float32, Appendix "Numerical Verification"); the
// same code also runs on bf16 tensors for cross-checking the MFMA kernels.
//
// Mask (Section "Attention Mask"): key j is visible to query i  <=>  j <= i + P < kend[j].
// Deterministic: every output element is produced by one wavefront in a fixed order.
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include "tt_kernels.h"

namespace tt {
namespace {

constexpr int WAVE = 64;
constexpr int ROWS_PER_BLOCK = 4;

__device__ __forceinline__ float to_f(float x) { return x; }
__device__ __forceinline__ float to_f(__hip_bfloat16 x) { return __bfloat162float(x); }
__device__ __forceinline__ void from_f(float* p, float x) { *p = x; }
__device__ __forceinline__ void from_f(__hip_bfloat16* p, float x) { *p = __float2bfloat16(x); }

__device__ __forceinline__ float wave_max(float x) {
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

template <typename T>
__device__ __forceinline__ float dot_row(const float* __restrict__ a_lds, const T* __restrict__ b, int d) {
  float acc = 0.f;
  for (int e = 0; e < d; e++) acc = fmaf(a_lds[e], to_f(b[e]), acc);
  return acc;
}

// Row of key j on the unified key axis.
template <typename T>
__device__ __forceinline__ const T* key_row(const T* own, const T* prefix, int64_t own_stride, int hkv, int d,
                                            int P, int j, int kvh) {
  return j < P ? prefix + ((int64_t)j * hkv + kvh) * d : own + (int64_t)(j - P) * own_stride + (int64_t)kvh * d;
}

// ---------------------------------------------------------------------------------------------
// Forward: wave <-> (query i, head h).  Lanes own keys for the scores and head-dim elements for
// the output accumulation (d = lane + 64 u).
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(WAVE * ROWS_PER_BLOCK)
ref_fwd_kernel(RefArgs a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int i = blockIdx.x * ROWS_PER_BLOCK + w;
  const int h = blockIdx.y, kvh = h / (a.hq / a.hkv);
  float* q_s = lds + w * a.d;
  const bool active = i < a.n_q;
  if (active) {
    const T* qp = (const T*)a.q + (int64_t)i * a.q_stride + (int64_t)h * a.d;
    for (int e = lane; e < a.d; e += WAVE) q_s[e] = to_f(qp[e]);
  }
  __syncthreads();
  if (!active) return;
  const int gi = i + a.n_prefix;
  float m = -INFINITY, l = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int c = 0; c <= gi; c += WAVE) {
    const int j = c + lane;
    const bool vis = j <= gi && gi < a.kend[j < a.n_prefix + a.n_q ? j : 0] && j < a.n_prefix + a.n_q;
    if (__ballot(vis) == 0) continue;
    float s = -INFINITY;
    if (vis) s = a.scale * dot_row(q_s, key_row((const T*)a.k_own, (const T*)a.k_prefix, a.k_stride, a.hkv, a.d, a.n_prefix, j, kvh), a.d);
    const float m_new = fmaxf(m, wave_max(s));
    const float alpha = expf(m - m_new);          // m = -inf on the first visited chunk: alpha = 0
    const float p = vis ? expf(s - m_new) : 0.f;
    l = l * alpha + wave_sum(p);
    m = m_new;
#pragma unroll
    for (int u = 0; u < 4; u++) acc[u] *= alpha;
    const uint64_t vmask = __ballot(vis);
    for (int jj = 0; jj < WAVE; jj++) {
      if (!((vmask >> jj) & 1)) continue;
      const float pj = __shfl(p, jj);
      const T* vr = key_row((const T*)a.v_own, (const T*)a.v_prefix, a.v_stride, a.hkv, a.d, a.n_prefix, c + jj, kvh);
#pragma unroll
      for (int u = 0; u < 4; u++) {
        const int e = lane + u * WAVE;
        if (e < a.d) acc[u] = fmaf(pj, to_f(vr[e]), acc[u]);
      }
    }
  }
  T* op = (T*)a.o + ((int64_t)i * a.hq + h) * a.d;
#pragma unroll
  for (int u = 0; u < 4; u++) {
    const int e = lane + u * WAVE;
    if (e < a.d) from_f(op + e, acc[u] / l);
  }
  if (lane == 0) a.lse[(int64_t)h * a.n_q + i] = m + logf(l);
}

// D_i = <dO_i, O_i>  -> delta[h][i]
template <typename T>
__global__ void __launch_bounds__(WAVE * ROWS_PER_BLOCK)
ref_delta_kernel(RefArgs a) {
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int i = blockIdx.x * ROWS_PER_BLOCK + w;
  const int h = blockIdx.y;
  if (i >= a.n_q) return;
  const T* op = (const T*)a.o + ((int64_t)i * a.hq + h) * a.d;
  const T* gp = (const T*)a.d_o + ((int64_t)i * a.hq + h) * a.d;
  float s = 0.f;
  for (int e = lane; e < a.d; e += WAVE) s = fmaf(to_f(op[e]), to_f(gp[e]), s);
  s = wave_sum(s);
  if (lane == 0) a.delta[(int64_t)h * a.n_q + i] = s;
}

// dQ: wave <-> (query i, head h)
template <typename T>
__global__ void __launch_bounds__(WAVE * ROWS_PER_BLOCK)
ref_dq_kernel(RefArgs a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int i = blockIdx.x * ROWS_PER_BLOCK + w;
  const int h = blockIdx.y, kvh = h / (a.hq / a.hkv);
  float* q_s = lds + (2 * w) * a.d;
  float* g_s = lds + (2 * w + 1) * a.d;
  const bool active = i < a.n_q;
  if (active) {
    const T* qp = (const T*)a.q + (int64_t)i * a.q_stride + (int64_t)h * a.d;
    const T* gp = (const T*)a.d_o + ((int64_t)i * a.hq + h) * a.d;
    for (int e = lane; e < a.d; e += WAVE) { q_s[e] = to_f(qp[e]); g_s[e] = to_f(gp[e]); }
  }
  __syncthreads();
  if (!active) return;
  const int gi = i + a.n_prefix;
  const float lse = a.lse[(int64_t)h * a.n_q + i];
  const float delta = a.delta[(int64_t)h * a.n_q + i];
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int c = 0; c <= gi; c += WAVE) {
    const int j = c + lane;
    const bool vis = j < a.n_prefix + a.n_q && j <= gi && gi < a.kend[j < a.n_prefix + a.n_q ? j : 0];
    const uint64_t vmask = __ballot(vis);
    if (vmask == 0) continue;
    float ds = 0.f;
    if (vis) {
      const float s = a.scale * dot_row(q_s, key_row((const T*)a.k_own, (const T*)a.k_prefix, a.k_stride, a.hkv, a.d, a.n_prefix, j, kvh), a.d);
      const float p = expf(s - lse);
      const float dp = dot_row(g_s, key_row((const T*)a.v_own, (const T*)a.v_prefix, a.v_stride, a.hkv, a.d, a.n_prefix, j, kvh), a.d);
      ds = p * (dp - delta);
    }
    for (int jj = 0; jj < WAVE; jj++) {
      if (!((vmask >> jj) & 1)) continue;
      const float dsj = __shfl(ds, jj);
      const T* kr = key_row((const T*)a.k_own, (const T*)a.k_prefix, a.k_stride, a.hkv, a.d, a.n_prefix, c + jj, kvh);
#pragma unroll
      for (int u = 0; u < 4; u++) {
        const int e = lane + u * WAVE;
        if (e < a.d) acc[u] = fmaf(dsj, to_f(kr[e]), acc[u]);
      }
    }
  }
  T* dp_ = (T*)a.dq + ((int64_t)i * a.hq + h) * a.d;
#pragma unroll
  for (int u = 0; u < 4; u++) {
    const int e = lane + u * WAVE;
    if (e < a.d) from_f(dp_ + e, a.scale * acc[u]);
  }
}

// dK/dV: wave <-> (key j on the unified axis, kv head).  The visible queries of key j form the
// contiguous range [max(j - P, 0), kend[j] - P).
template <typename T>
__global__ void __launch_bounds__(WAVE * ROWS_PER_BLOCK)
ref_dkv_kernel(RefArgs a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int j = blockIdx.x * ROWS_PER_BLOCK + w;
  const int kvh = blockIdx.y, G = a.hq / a.hkv;
  float* k_s = lds + (2 * w) * a.d;
  float* v_s = lds + (2 * w + 1) * a.d;
  const int n_k = a.n_prefix + a.n_q;
  const bool active = j < n_k;
  if (active) {
    const T* kr = key_row((const T*)a.k_own, (const T*)a.k_prefix, a.k_stride, a.hkv, a.d, a.n_prefix, j, kvh);
    const T* vr = key_row((const T*)a.v_own, (const T*)a.v_prefix, a.v_stride, a.hkv, a.d, a.n_prefix, j, kvh);
    for (int e = lane; e < a.d; e += WAVE) { k_s[e] = to_f(kr[e]); v_s[e] = to_f(vr[e]); }
  }
  __syncthreads();
  if (!active) return;
  const int i_lo = j > a.n_prefix ? j - a.n_prefix : 0;
  const int ke = a.kend[j];
  const int i_hi = ke - a.n_prefix < a.n_q ? ke - a.n_prefix : a.n_q;    // ke = INT32_MAX or 0 for prefix keys
  float dk[4] = {0.f, 0.f, 0.f, 0.f}, dv[4] = {0.f, 0.f, 0.f, 0.f};
  for (int g = 0; g < G; g++) {
    const int h = kvh * G + g;
    for (int c = i_lo; c < i_hi; c += WAVE) {
      const int i = c + lane;
      const bool vis = i < i_hi;
      float p = 0.f, ds = 0.f;
      if (vis) {
        const T* qp = (const T*)a.q + (int64_t)i * a.q_stride + (int64_t)h * a.d;
        const T* gp = (const T*)a.d_o + ((int64_t)i * a.hq + h) * a.d;
        const float s = a.scale * dot_row(k_s, qp, a.d);
        p = expf(s - a.lse[(int64_t)h * a.n_q + i]);
        const float dp = dot_row(v_s, gp, a.d);
        ds = p * (dp - a.delta[(int64_t)h * a.n_q + i]);
      }
      const int cnt = i_hi - c < WAVE ? i_hi - c : WAVE;
      for (int ii = 0; ii < cnt; ii++) {
        const float pi = __shfl(p, ii), dsi = __shfl(ds, ii);
        const T* qp = (const T*)a.q + (int64_t)(c + ii) * a.q_stride + (int64_t)h * a.d;
        const T* gp = (const T*)a.d_o + ((int64_t)(c + ii) * a.hq + h) * a.d;
#pragma unroll
        for (int u = 0; u < 4; u++) {
          const int e = lane + u * WAVE;
          if (e < a.d) {
            dv[u] = fmaf(pi, to_f(gp[e]), dv[u]);
            dk[u] = fmaf(dsi, to_f(qp[e]), dk[u]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < 4; u++) {
    const int e = lane + u * WAVE;
    if (e >= a.d) continue;
    if (j < a.n_prefix) {
      if (i_hi > i_lo) {
        a.dk_prefix_acc[((int64_t)j * a.hkv + kvh) * a.d + e] += a.scale * dk[u];
        a.dv_prefix_acc[((int64_t)j * a.hkv + kvh) * a.d + e] += dv[u];
      }
    } else {
      from_f((T*)a.dk_own + ((int64_t)(j - a.n_prefix) * a.hkv + kvh) * a.d + e, a.scale * dk[u]);
      from_f((T*)a.dv_own + ((int64_t)(j - a.n_prefix) * a.hkv + kvh) * a.d + e, dv[u]);
    }
  }
}

template <typename T>
hipError_t launch_fwd(const RefArgs& a, hipStream_t st) {
  if (a.n_q == 0) return hipSuccess;
  dim3 grid((a.n_q + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, a.hq);
  KernelTimer timer(TT_KERNEL_REF_FWD, st);
  ref_fwd_kernel<T><<<grid, WAVE * ROWS_PER_BLOCK, sizeof(float) * a.d * ROWS_PER_BLOCK, st>>>(a);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_bwd(const RefArgs& a, hipStream_t st) {
  if (a.n_q == 0) return hipSuccess;
  dim3 grid((a.n_q + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, a.hq);
  KernelTimer timer(TT_KERNEL_REF_BWD, st);
  ref_delta_kernel<T><<<grid, WAVE * ROWS_PER_BLOCK, 0, st>>>(a);
  if (hipError_t e = hipGetLastError()) return e;
  ref_dq_kernel<T><<<grid, WAVE * ROWS_PER_BLOCK, sizeof(float) * a.d * ROWS_PER_BLOCK * 2, st>>>(a);
  if (hipError_t e = hipGetLastError()) return e;
  dim3 gridk((a.n_prefix + a.n_q + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, a.hkv);
  ref_dkv_kernel<T><<<gridk, WAVE * ROWS_PER_BLOCK, sizeof(float) * a.d * ROWS_PER_BLOCK * 2, st>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t ref_attn_fwd(const RefArgs& a, bool bf16, hipStream_t st) {
  return bf16 ? launch_fwd<__hip_bfloat16>(a, st) : launch_fwd<float>(a, st);
}
hipError_t ref_attn_bwd(const RefArgs& a, bool bf16, hipStream_t st) {
  return bf16 ? launch_bwd<__hip_bfloat16>(a, st) : launch_bwd<float>(a, st);
}

}  // namespace tt
