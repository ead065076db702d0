// Building blocks shared by the bf16 MFMA attention kernels (gfx950, 64-wide wavefronts).
//
// MFMA 32x32x16 bf16 register layouts (lane l, half hf = l / 32, c = l % 32):
//   A operand [32 x 16]: row c, k = 8*hf .. 8*hf+7            (8 bf16 per lane)
//   B operand [16 x 32]: column c, k = 8*hf .. 8*hf+7
//   C/D       [32 x 32]: column c, rows (r/4)*8 + 4*hf + r%4 for r = 0..15
// An accumulator can be fed back as a B operand of a following MFMA without moving data between
// lanes: registers 8t..8t+7 of the accumulator become the 8 k-values of k-step t, which fixes the
// correspondence  k-index (hf, e)  <->  row 16t + (e/4)*8 + 4*hf + e%4  of the accumulator; the A
// operand of that MFMA must enumerate its k dimension in the same permuted order.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace tt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr float LOG2E_F = 1.4426950408889634f;
constexpr float LN2_F = 0.6931471805599453f;

#define TT_LDS(T) __attribute__((address_space(3))) T

// 2^x as the bare hardware instruction (no denormal-range fix-up): the arguments here are <= 0 up to
// rounding and results below 2^-126 may flush to zero, which is what a softmax weight wants.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Makes the compiler treat a register-resident fragment as consumed here, so that the wait for the
// global load that produced it is placed at this point and not inside the main loop (where a
// vmcnt wait would also stall on the prefetch of the next tile).
__device__ __forceinline__ void pin(const bf16x8& f) { asm volatile("" ::"v"(f)); }

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; r++) z[r] = 0.f;
  return z;
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Transposed LDS read: inside each group of 16 lanes, lane i passes the address of 4 consecutive
// bf16 of row i/4 (columns 4*(i%4) .. +3) of a 4 x 16 block and receives column i of that block
// (rows 0..3).
__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((TT_LDS(s16x4)*)(p));
  return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ bf16x8 cat4(bf16x4 a, bf16x4 b) {
  return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// max / sum of a value with the lane 32 positions away (the other half of the same column)
__device__ __forceinline__ float half_swap_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 8 fp32 -> 8 bf16, round to nearest even
__device__ __forceinline__ bf16x8 cvt8(float a0, float a1, float a2, float a3, float a4, float a5, float a6, float a7) {
  typedef float f32x8 __attribute__((ext_vector_type(8)));
  f32x8 v = {a0, a1, a2, a3, a4, a5, a6, a7};
  return __builtin_convertvector(v, bf16x8);
}
__device__ __forceinline__ bf16x4 cvt4(float a0, float a1, float a2, float a3) {
  f32x4 v = {a0, a1, a2, a3};
  return __builtin_convertvector(v, bf16x4);
}

// Iterates over the key tiles (TT_KTILE keys each, prefix tiles first, then own tiles) that can hold
// a key visible to some query of the range [gi_first, gi_last] (unified indices): tiles up to the
// diagonal whose largest visibility bound exceeds gi_first.  64 tiles are tested per step with one
// wavefront-wide load + ballot; every wavefront of the workgroup walks the same sequence.
struct KTileIter {
  const int32_t *kt_max, *kt_min;
  int u_end;        // one past the last candidate tile
  int gi_first;
  int base;         // next window start
  uint64_t mask;    // unvisited candidates of the current window [base-64, base)
  int kmin_lane;    // kt_min of tile base-64+lane (the window's values, one per lane)
  int kmin;         // kt_min of the tile returned by the last next()
  __device__ __forceinline__ void init(const int32_t* kt_max_, const int32_t* kt_min_, int u_end_, int gi_first_) {
    kt_max = kt_max_; kt_min = kt_min_; u_end = u_end_; gi_first = gi_first_; base = 0; mask = 0;
    kmin_lane = 0; kmin = 0;
  }
  __device__ __forceinline__ int next() {
    while (mask == 0) {
      if (base >= u_end) return -1;
      const int u = base + (int)(threadIdx.x & 63);
      const bool in = u < u_end;
      const bool cand = in && kt_max[u] > gi_first;
      kmin_lane = in ? kt_min[u] : 0;
      mask = __ballot(cand);
      base += 64;
    }
    const int b = __builtin_ctzll(mask);
    mask &= mask - 1;
    kmin = __builtin_amdgcn_readlane(kmin_lane, b);
    return base - 64 + b;
  }
};

}  // namespace tt
