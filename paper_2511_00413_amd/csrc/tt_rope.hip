// Rotary position embedding driven by the tree position ids (paper Eq. 9: a token's position is its
// depth in tokens along the root-to-token path, so sibling branches restart at their parent's end).
// Rotate-half convention: pair (x[i], x[i + d/2]) turns by pos * base^(-2i/d); `inverse` turns the
// other way, which undoes the rotation and is also its backward pass.
//
// HBM-bound: every element is read once and written once with 16-byte accesses.  The d/2 (cos, sin)
// pairs of a token are computed once per token and shared by all its heads through LDS; the angle
// pos * inv_freq is formed and reduced modulo 2 pi in fp64 (positions reach 10^5..10^6, where an fp32
// product would already be wrong in the second decimal), the sine and cosine of the reduced angle in
// fp32.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include "tt_kernels.h"

namespace tt {
namespace {

constexpr int ROPE_THREADS = 256;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8r __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8r __attribute__((ext_vector_type(8)));

template <int EPV> struct Vec;
template <> struct Vec<8> {          // bf16
  static __device__ __forceinline__ void unpack(const u32x4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; i++) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
  }
  static __device__ __forceinline__ u32x4 pack(const float (&f)[8]) {
    f32x8r g;
#pragma unroll
    for (int e = 0; e < 8; e++) g[e] = f[e];
    return __builtin_bit_cast(u32x4, __builtin_convertvector(g, bf16x8r));      // round to nearest even
  }
};
template <> struct Vec<4> {          // fp32
  static __device__ __forceinline__ void unpack(const u32x4& v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ u32x4 pack(const float (&f)[4]) {
    u32x4 o;
    o.x = __float_as_uint(f[0]); o.y = __float_as_uint(f[1]); o.z = __float_as_uint(f[2]); o.w = __float_as_uint(f[3]);
    return o;
  }
};

// A workgroup handles `tpb` consecutive tokens (as many as give its 256 threads one vector pair each,
// at least one).  esz = element size; strides in elements.
template <int ESZ>
__global__ void __launch_bounds__(ROPE_THREADS)
rope_kernel(int64_t n_tokens, int n_heads, int d, const char* x, int64_t x_stride, const int32_t* __restrict__ pos,
            double log2_base, int inverse, char* y, int64_t y_stride, int tpb) {
  constexpr int EPV = 16 / ESZ;
  extern __shared__ float2 cs[];                    // [tpb][d/2] (cos, sin)
  const int half = d / 2;
  const int64_t tok0 = (int64_t)blockIdx.x * tpb;
  const int ntok = (int)min((int64_t)tpb, n_tokens - tok0);
  const int vph = half / EPV;                       // vectors per half head
  const int per_tok = n_heads * vph;
  const int n_work = ntok * per_tok;
  // element offset of work item wk (one vector pair) inside x / y, and where its (cos, sin) pairs start
  auto locate = [&](int wk, int64_t& x_off, int64_t& y_off, int& cs_off) {
    const int tk = wk / per_tok, rem = wk % per_tok;
    const int h = rem / vph, vi = rem % vph;
    const int64_t off = (int64_t)h * d + (int64_t)vi * EPV;
    x_off = ((tok0 + tk) * x_stride + off) * ESZ;
    y_off = ((tok0 + tk) * y_stride + off) * ESZ;
    cs_off = tk * half + vi * EPV;
  };
  // the first vector pair of every thread is requested before the angles are worked out, so that the memory
  // round trip runs under the fp64 arithmetic; streaming (non-temporal) loads: nothing is read twice (the stores
  // are ordinary ones: measured 2-3 % faster than non-temporal stores here, and the next kernel reads what they wrote)
  u32x4 vlo = {0, 0, 0, 0}, vhi = {0, 0, 0, 0};
  if ((int)threadIdx.x < n_work) {
    int64_t xo, yo; int co;
    locate(threadIdx.x, xo, yo, co);
    vlo = __builtin_nontemporal_load((const u32x4*)(x + xo));
    vhi = __builtin_nontemporal_load((const u32x4*)(x + xo + (int64_t)half * ESZ));
  }
  for (int idx = threadIdx.x; idx < ntok * half; idx += ROPE_THREADS) {
    const int tk = idx / half, i = idx % half;
    const double inv_freq = exp2(-(2.0 * i / d) * log2_base);
    const double ang = (double)pos[tok0 + tk] * inv_freq;
    const double two_pi = 6.283185307179586476925286766559;
    const float r = (float)(ang - two_pi * rint(ang / two_pi));                 // |r| <= pi
    float s, c;
    sincosf(r, &s, &c);
    cs[idx] = make_float2(c, inverse ? -s : s);
  }
  __syncthreads();
  for (int wk = threadIdx.x; wk < n_work; wk += ROPE_THREADS) {
    int64_t xo, yo; int co;
    locate(wk, xo, yo, co);
    if (wk != (int)threadIdx.x) {
      vlo = __builtin_nontemporal_load((const u32x4*)(x + xo));
      vhi = __builtin_nontemporal_load((const u32x4*)(x + xo + (int64_t)half * ESZ));
    }
    float lo[EPV], hi[EPV], olo[EPV], ohi[EPV];
    Vec<EPV>::unpack(vlo, lo);
    Vec<EPV>::unpack(vhi, hi);
    const float2* t = cs + co;
#pragma unroll
    for (int e = 0; e < EPV; e++) {
      const float2 q = t[e];
      olo[e] = lo[e] * q.x - hi[e] * q.y;
      ohi[e] = hi[e] * q.x + lo[e] * q.y;
    }
    *(u32x4*)(y + yo) = Vec<EPV>::pack(olo);
    *(u32x4*)(y + yo + (int64_t)half * ESZ) = Vec<EPV>::pack(ohi);
  }
}

}  // namespace

hipError_t rope(int64_t n_tokens, int n_heads, int d, bool bf16, const void* x, int64_t x_stride, const int32_t* pos,
                float theta_base, bool inverse, void* y, int64_t y_stride, hipStream_t st) {
  if (n_tokens == 0) return hipSuccess;
  const int epv = bf16 ? 8 : 4;
  const int per_tok = n_heads * (d / 2 / epv);
  const int tpb = std::max(1, ROPE_THREADS / per_tok);
  const int64_t blocks = (n_tokens + tpb - 1) / tpb;
  const size_t lds = (size_t)tpb * (d / 2) * sizeof(float2);
  const double log2_base = log2((double)theta_base);
  KernelTimer timer(TT_KERNEL_ROPE, st);
  if (bf16)
    rope_kernel<2><<<(unsigned)blocks, ROPE_THREADS, lds, st>>>(n_tokens, n_heads, d, (const char*)x, x_stride, pos, log2_base,
                                                              inverse ? 1 : 0, (char*)y, y_stride, tpb);
  else
    rope_kernel<4><<<(unsigned)blocks, ROPE_THREADS, lds, st>>>(n_tokens, n_heads, d, (const char*)x, x_stride, pos, log2_base,
                                                              inverse ? 1 : 0, (char*)y, y_stride, tpb);
  return hipGetLastError();
}

}  // namespace tt
