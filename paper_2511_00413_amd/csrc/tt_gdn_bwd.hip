// Gated delta rule with tree state routing, backward (Section "Implementation", paragraph "SSM Layers
// (GDN)" (i): gradients accumulate at the shared parent state; Appendix "Tree-Aware SSM State
// Routing").  Chunked like the forward (64 tokens, chunks never cross a node boundary).  With
//     Vn = U - W S0,   O = Qg S0 + P Vn,   S1 = EL S0 + Kd^T Vn
// (Qg = scale exp(gamma) Q, Kd = exp(gamma_last - gamma) K, EL = exp(gamma_last), U = (I+A)^-1 beta V,
// W = (I+A)^-1 beta exp(gamma) K, A = beta_i A0_ij, A0 = strictly-lower((k_i.k_j) D_ij),
// P = scale tril((q_i.k_j) D_ij), D_ij = exp(gamma_i - gamma_j)) the chain rule gives, per chunk,
//     dVn = P^T dO + Kd dS1                      dS0 = EL dS1 + Qg^T dO - W^T dVn          (serial part)
//     dQg = dO S0^T    dKd = Vn dS1^T    dW = -dVn S0^T    dP = tril(dO Vn^T)
//     [dVb | dKb] = (I+A)^-T [dVn | dW]          dA = strictly-lower(-dVb U^T - dKb W^T)
// and from there dq, dk, dv, dbeta and dgamma by the product rule; dg is the reverse running sum of
// dgamma inside the chunk.  State routing backwards: dS1 of a chunk is the dS0 of the chunk that
// continued from it on chip plus the gradient collected in its saved-state slot (every chunk that
// started from the slot added its dS0 there; they all come later in DFS order, so a reverse walk over
// the chunks has seen them), plus the upstream gradient of a captured state.
//
// Kernels (the first three live in tt_gdn.hip with the forward's):
//   gdn_prepare_kernel<true>   per (chunk, head): the forward walk's bf16 record, the reverse walk's bf16 record
//                              (Kd, -W^T, Qg^T, P^T, dO^T) and gamma, A0, P unrounded
//   gdn_scan_kernel<true>      (32 value columns, head): the forward scan without its output; saves S0 and Vn
//                              of every chunk (bf16)
//   gdn_rscan_kernel           (32 value columns, head): reverse walk in the forward scan's form (bf16 matrix
//                              instruction, fp32 state gradient in accumulators); saves dS1 and dVn (bf16)
//   gdn_bwd_finish_kernel      per (chunk, head): everything else: products on the bf16 matrix instruction (fp32
//                              accumulation) through LDS slabs, the transposed solve with one lane per column
//                              and all element-wise work in fp32; dq / dk per value head in fp32
//   gdn_bwd_group_sum_kernel   sums dq / dk over the value heads that share a key head, rounds to bf16
#include <hip/hip_runtime.h>
#include <algorithm>
#include "tt_internal.h"
#include "tt_kernels.h"
#include "tt_mfma.h"

namespace tt {
namespace {

constexpr int GC = TT_GDN_CHUNK;     // 64
constexpr int GD = 128;
constexpr int BT = 256;
constexpr int KS = 64;               // k-values per LDS slab of the finish kernel's products

struct BwdWs {
  GdnChunkOps ops;
  GdnBwdSaved sv;
  __bf16* x;         // per (head, chunk) [64][256]: [dW] on the way in, [dVb | dKb] after the transposed solve
  float* dqh;        // [N][hv_n][128] per-value-head dq, dk (the heads of the pass)
  float* dkh;
};
struct KArgs {
  GdnBwdArgs b;
  BwdWs w;
};

__device__ __forceinline__ float4 ld4(const float* p) { return *(const float4*)p; }

// Register r of a 32 x 32 accumulator tile holds row (r / 4) * 8 + 4 hf + r % 4 of column lane % 32.
__device__ __forceinline__ int tile_row(int r, int hf) { return (r >> 2) * 8 + 4 * hf + (r & 3); }

// ---- per-chunk finish ----------------------------------------------------------------------------------
// Products C (64 x N) += A (64 x K) B (K x N) of a workgroup on the bf16 matrix instruction, fp32 accumulation
// (slab_product below).  Nearly every operand is bf16 in memory already; only the two 64 x 64 matrices that the
// kernel forms itself (dP scale D and dA beta D) are rounded here.  The operands go through LDS slabs of KS
// k-values, brought in by the loaders that follow.  Wave w holds, in accumulator layout, N = 128: tiles (row
// block t, column block w), t = 0, 1;  N = 64: the tile (row block w & 1, column block w >> 1).
template <int N>
struct TileMap {
  static constexpr int TPW = N / 64;                     // tiles per wave
  __device__ static int ib(int w, int t) { return N == 128 ? t : (w & 1); }
  __device__ static int jb(int w) { return N == 128 ? w : (w >> 1); }
};

// LDS slab layouts (bf16).  "k-major": [k][row or column], the orientation in which most operands arrive (a
// 16-byte piece of memory holds 8 rows / columns of one k); fragments come out of it through the transposing LDS
// read.  "row-major": [row][k] for A operands whose memory has k contiguous; fragments are plain 16-byte reads.
// Pitches (elements): rows 16-byte aligned, 8 elements of padding against bank conflicts.
constexpr int PK_A = GC + 8;                              // k-major A slab: KS rows of 64 (+8)
constexpr int PR_A = KS + 8;                              // row-major A slab: 64 rows of KS (+8)
template <int N> constexpr int pitch_b() { return N + 8; } // k-major B slab: KS rows of N (+8)
constexpr int AS_ELEMS = KS * PK_A > GC * PR_A ? KS * PK_A : GC * PR_A;

// ---- operand loaders ---------------------------------------------------------------------------------------
// A loader brings one KS-wide slab of an operand from memory into registers (load) and from there into the LDS
// slab (store).  Memory is read in 16-byte pieces.  KMAJOR tells the layout of an A loader's slab.

// Vn / dVn in fragment order, element (token, value column).  As A (k-major): (i = token, k = column).  As B:
// (k = column, j = token).  One piece = 8 tokens of one column: tokens base .. base + 3 and base + 8 .. base + 11.
template <int PITCH>
struct FragLoader {
  static constexpr bool KMAJOR = true;
  const __bf16* p;
  struct Regs { bf16x8 v[KS * GC / 8 / BT]; };
  __device__ __forceinline__ void load(int k0, int tid, Regs& r) const {
#pragma unroll
    for (int q = 0; q < KS * GC / 8 / BT; q++) {
      const int piece = tid + q * BT, cl = piece % KS, g = piece / KS;     // column inside the slab; (half, t, hf)
      const int col = k0 + cl;
      r.v[q] = *(const bf16x8*)(p + ((((size_t)(col >> 5) * 4 + (g >> 1)) * 64 + (g & 1) * 32 + (col & 31)) << 3));
    }
  }
  __device__ __forceinline__ void store(__bf16* lds, int tid, const Regs& r, int = 0) const {
#pragma unroll
    for (int q = 0; q < KS * GC / 8 / BT; q++) {
      const int piece = tid + q * BT, cl = piece % KS, g = piece / KS;
      const int base = 32 * (g >> 2) + 16 * ((g >> 1) & 1) + 4 * (g & 1);
      __bf16* d = lds + cl * PITCH + base;
      *(bf16x4*)d = __builtin_shufflevector(r.v[q], r.v[q], 0, 1, 2, 3);
      *(bf16x4*)(d + 8) = __builtin_shufflevector(r.v[q], r.v[q], 4, 5, 6, 7);
    }
  }
};
// bf16 rows with the contraction index contiguous, as A (row-major): (i, k) = p[i * pitch + k]; rows >= len are zero
struct RowsKLoaderA {
  static constexpr bool KMAJOR = false;
  const __bf16* p;
  int pitch, len;
  struct Regs { bf16x8 v[GC * KS / 8 / BT]; };
  __device__ __forceinline__ void load(int k0, int tid, Regs& r) const {
#pragma unroll
    for (int q = 0; q < GC * KS / 8 / BT; q++) {
      const int piece = tid + q * BT, i = piece / (KS / 8), k8 = (piece % (KS / 8)) * 8;
      r.v[q] = *(const bf16x8*)(p + (size_t)min(i, len - 1) * pitch + k0 + k8);
    }
  }
  __device__ __forceinline__ void store(__bf16* lds, int tid, const Regs& r) const {
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; e++) zero[e] = (__bf16)0.f;
#pragma unroll
    for (int q = 0; q < GC * KS / 8 / BT; q++) {
      const int piece = tid + q * BT, i = piece / (KS / 8), k8 = (piece % (KS / 8)) * 8;
      *(bf16x8*)(lds + i * PR_A + k8) = i < len ? r.v[q] : zero;
    }
  }
};
// any A given element by element as fp32 (the LDS-resident 64 x 64 matrices), row-major slab; a thread takes 8
// consecutive k of one row
template <class F>
struct FnLoaderA {
  static constexpr bool KMAJOR = false;
  F f;
  struct Regs { bf16x8 v[GC * KS / 8 / BT]; };
  __device__ __forceinline__ void load(int k0, int tid, Regs& r) const {
#pragma unroll
    for (int q = 0; q < GC * KS / 8 / BT; q++) {
      const int piece = tid + q * BT, i = piece % GC, k8 = (piece / GC) * 8;
      r.v[q] = cvt8(f(i, k0 + k8), f(i, k0 + k8 + 1), f(i, k0 + k8 + 2), f(i, k0 + k8 + 3), f(i, k0 + k8 + 4), f(i, k0 + k8 + 5),
                    f(i, k0 + k8 + 6), f(i, k0 + k8 + 7));
    }
  }
  __device__ __forceinline__ void store(__bf16* lds, int tid, const Regs& r) const {
#pragma unroll
    for (int q = 0; q < GC * KS / 8 / BT; q++) {
      const int piece = tid + q * BT, i = piece % GC, k8 = (piece / GC) * 8;
      *(bf16x8*)(lds + i * PR_A + k8) = r.v[q];
    }
  }
};
template <class F> __device__ __forceinline__ FnLoaderA<F> fn_loader_a(F f) { return FnLoaderA<F>{f}; }
// bf16 rows of 128 with the output index contiguous, as B (N = 128): (k, j) = p[k * pitch + j]; rows >= len are zero
struct RowsJLoaderB {
  const __bf16* p;
  int pitch, len;
  struct Regs { bf16x8 v[KS * GD / 8 / BT]; };
  __device__ __forceinline__ void load(int k0, int tid, Regs& r) const {
#pragma unroll
    for (int q = 0; q < KS * GD / 8 / BT; q++) {
      const int piece = tid + q * BT, kk = piece >> 4, j8 = (piece & 15) * 8;
      r.v[q] = *(const bf16x8*)(p + (size_t)min(k0 + kk, len - 1) * pitch + j8);
    }
  }
  __device__ __forceinline__ void store(__bf16* lds, int tid, const Regs& r, int k0) const {
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; e++) zero[e] = (__bf16)0.f;
#pragma unroll
    for (int q = 0; q < KS * GD / 8 / BT; q++) {
      const int piece = tid + q * BT, kk = piece >> 4, j8 = (piece & 15) * 8;
      *(bf16x8*)(lds + kk * pitch_b<GD>() + j8) = k0 + kk < len ? r.v[q] : zero;
    }
  }
};
// [U | W]^T from the walks' bf16 records, as B (N = 64): (k, j) = k < 128 ? U^T[k][j] : -(-W^T)[k - 128][j]
struct UwLoaderB {
  const __bf16 *ut, *wtn;
  struct Regs { bf16x8 v[KS * GC / 8 / BT]; };
  __device__ __forceinline__ void load(int k0, int tid, Regs& r) const {
    const __bf16* src = k0 < GD ? ut + (size_t)k0 * GC : wtn + (size_t)(k0 - GD) * GC;     // a slab lies in one half
#pragma unroll
    for (int q = 0; q < KS * GC / 8 / BT; q++) {
      const int piece = tid + q * BT, kk = piece >> 3, j8 = (piece & 7) * 8;
      r.v[q] = *(const bf16x8*)(src + (size_t)kk * GC + j8);
    }
  }
  __device__ __forceinline__ void store(__bf16* lds, int tid, const Regs& r, int k0) const {
#pragma unroll
    for (int q = 0; q < KS * GC / 8 / BT; q++) {
      const int piece = tid + q * BT, kk = piece >> 3, j8 = (piece & 7) * 8;
      typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
      const u16x8 flipped = __builtin_bit_cast(u16x8, r.v[q]) ^ (unsigned short)0x8000;      // -x: the sign bit
      *(bf16x8*)(lds + kk * pitch_b<GC>() + j8) = k0 < GD ? r.v[q] : __builtin_bit_cast(bf16x8, flipped);
    }
  }
};
typedef FragLoader<pitch_b<GC>()> FragLoaderB;             // Vn as B (N = 64)

// Barrier that waits for this wave's LDS traffic only (a __syncthreads also waits for every global load in flight,
// i.e. for the slabs that were requested ahead).  Not for global data written by other threads of the workgroup.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int N, int K, class LA, class LB>
__device__ __forceinline__ void slab_product(const LA& la, const LB& lb, f32x16 (&acc)[N / 64], __bf16* as, __bf16* bs, int tid_in) {
  constexpr int PB = pitch_b<N>(), NS = K / KS;
  // The fetch offsets are functions of the thread id alone.  Hidden behind an opaque copy they are computed at each
  // call; otherwise the compiler computes those of all calls at the top of the kernel and keeps them in registers
  // throughout (measured: 174 spilled registers at two waves per SIMD).
  int tid = tid_in;
  asm volatile("" : "+v"(tid));
  typedef TileMap<N> TM;
  const int lane = tid & 63, c = lane & 31, hf = lane >> 5, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  auto multiply = [&]() {
#pragma unroll
    for (int s = 0; s < KS / 16; s++) {
      const bf16x8 b = kmajor_frag(bs, PB, 16 * s + 8 * hf, 32 * TM::jb(w) + 16 * (c >> 4), lane);
#pragma unroll
      for (int t = 0; t < TM::TPW; t++) {
        const int ib = TM::ib(w, t);
        const bf16x8 a = LA::KMAJOR ? kmajor_frag(as, PK_A, 16 * s + 8 * hf, 32 * ib + 16 * (c >> 4), lane)
                                    : *(const bf16x8*)(as + (32 * ib + c) * PR_A + 16 * s + 8 * hf);
        acc[t] = mfma32(a, b, acc[t]);
      }
    }
  };
  // Up to two slabs are in flight: while slab s is multiplied, s + 1 is on its way and s + 2 has just been
  // requested.  Two register sets take turns; the last steps request nothing (a branch around loads would put
  // their wait at its end, so the steps are peeled).
  typename LA::Regs ra[2];
  typename LB::Regs rb[2];
  static_assert(NS == 1 || NS % 2 == 0, "one slab or an even number of slabs");
  la.load(0, tid, ra[0]);
  lb.load(0, tid, rb[0]);
  if constexpr (NS > 1) {
    la.load(KS, tid, ra[1]);
    lb.load(KS, tid, rb[1]);
#pragma unroll 1
    for (int k0 = 0; k0 < K - 2 * KS; k0 += 2 * KS) {
#pragma unroll
      for (int set = 0; set < 2; set++) {
        lds_barrier();                 // the previous slab (or whatever used the slab arrays before) has been read
        la.store(as, tid, ra[set]);
        lb.store(bs, tid, rb[set], k0 + set * KS);
        lds_barrier();
        la.load(k0 + (2 + set) * KS, tid, ra[set]);
        lb.load(k0 + (2 + set) * KS, tid, rb[set]);
        multiply();
      }
    }
  }
#pragma unroll
  for (int set = 0; set < (NS > 1 ? 2 : 1); set++) {
    lds_barrier();
    la.store(as, tid, ra[set]);
    lb.store(bs, tid, rb[set], K - ((NS > 1 ? 2 : 1) - set) * KS);
    lds_barrier();
    multiply();
  }
}

// Sum over the 32 lanes of a half wave (the lanes that hold one row of an accumulator tile), with data-parallel
// lane moves instead of LDS-routed shuffles (the kernel forms 96 such sums per lane).  The total arrives in the
// upper 16 lanes of the half (lanes 16 .. 31 and 48 .. 63).
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ float dpp_move(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float half_wave_sum(float x) {
  x += dpp_move<0xb1>(x);          // quad_perm [1,0,3,2]: lane ^ 1
  x += dpp_move<0x4e>(x);          // quad_perm [2,3,0,1]: lane ^ 2
  x += dpp_move<0x141>(x);         // row_half_mirror: the other quad of each group of 8
  x += dpp_move<0x140>(x);         // row_mirror: the other group of 8 of each row of 16
  x += dpp_move<0x142, 0xa>(x);    // row_bcast15 into rows 1 and 3: adds the total of the row below
  return x;
}
constexpr int HALF_SUM_LANE = 16;  // a lane position (inside its half wave) that holds half_wave_sum's result

constexpr int AP = GC + 1;     // row pitch of the 64 x 64 LDS matrices that are read along rows and columns
constexpr int TP = GC + 4;     // pitch of the transposed A during the solve (rows read as float4)

__global__ __launch_bounds__(BT, 2) void gdn_bwd_finish_kernel(KArgs a) {
  __shared__ __attribute__((aligned(16))) __bf16 as[AS_ELEMS];
  constexpr int BS_FLOATS = GC * AP > KS * pitch_b<GD>() / 2 ? GC * AP : KS * pitch_b<GD>() / 2;
  __shared__ __attribute__((aligned(16))) float bs_f[BS_FLOATS];  // B slabs (bf16); between products also dA o A0 (fp32)
  __bf16* bs = (__bf16*)bs_f;
  __shared__ __attribute__((aligned(16))) float dam[GC * TP];     // A^T during the solve, then dA, then dA beta D
  __shared__ float dpm[GC * AP];                                  // dP, then dP scale D
  __shared__ float gm[GC * AP];                                   // dP o P + dA o A
  __shared__ float gam[GC], bet[GC], eg[GC], el[GC];
  __shared__ float dg_row[GC], dg_col[GC], db_a[GC], db_v[GC], dgam[GC];
  // per-wave parts of row dot products: they live in gm, which is dead by the time they are formed
  float(*dot_q)[GC] = (float(*)[GC])gm;
  float(*dot_kd)[GC] = (float(*)[GC])(gm + 4 * GC);
  float(*dot_kb)[GC] = (float(*)[GC])(gm + 8 * GC);
  float* red = (float*)as;                                        // [BT], after the last product

  int chunk, h;
  if (!gdn_group_order(blockIdx.x, a.b.n_chunks, a.b.hv_n, a.b.hv / a.b.hk, chunk, h)) return;
  const int tid = threadIdx.x & (BT - 1), lane = tid & 63, c = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nc = a.b.n_chunks, hv = a.b.hv, kh = h / (hv / a.b.hk);
  const size_t op = (size_t)h * nc + chunk;
  const int tok0 = a.b.chunk_tok0[chunk], len = a.b.chunk_len[chunk];
  const float scale = a.b.scale;
  const __bf16* ut = (const __bf16*)a.w.sv.fwd_rec + op * GDN_REC_ELEMS + GDN_REC_UT;
  const __bf16* wtn = (const __bf16*)a.w.sv.rev_rec + op * GDN_REC_ELEMS + GDN_REV_WTN;
  const float* A0 = a.w.ops.a0 + op * (GC * GC);
  const float* Pm = a.w.ops.p + op * (GC * GC);
  // saved by the walks (bf16): S0 and dS1 transposed [value col][key dim], Vn and dVn in fragment order
  const __bf16* s0t = (const __bf16*)a.w.sv.s0t + op * (GD * GD);
  const __bf16* ds1t = (const __bf16*)a.w.sv.ds1t + op * (GD * GD);
  const __bf16* vns = (const __bf16*)a.w.sv.vns + op * (GC * GD);
  const __bf16* dvns = (const __bf16*)a.w.sv.dvns + op * (GC * GD);
  __bf16* X = a.w.x + op * (GC * 2 * GD);
  const size_t qrow = (size_t)a.b.hk * GD, vrow = (size_t)hv * GD;
  const __bf16* qb = (const __bf16*)a.b.q + (size_t)tok0 * qrow + (size_t)kh * GD;
  const __bf16* kb = (const __bf16*)a.b.k + (size_t)tok0 * qrow + (size_t)kh * GD;
  const __bf16* vb = (const __bf16*)a.b.v + (size_t)tok0 * vrow + (size_t)h * GD;
  const __bf16* dob = (const __bf16*)a.b.d_o + (size_t)tok0 * vrow + (size_t)h * GD;
  // rows past the chunk's length read a valid row and are then zeroed (no load sits inside a branch)
  // (32-bit offsets: a chunk spans at most 64 rows of at most 65535 * 128 elements)
  const int qrow32 = (int)qrow, vrow32 = (int)vrow;
  auto q_at = [&](int i, int d) { const float x = (float)qb[min(i, len - 1) * qrow32 + d]; return i < len ? x : 0.f; };
  auto k_at = [&](int i, int d) { const float x = (float)kb[min(i, len - 1) * qrow32 + d]; return i < len ? x : 0.f; };

  const float glast = a.w.ops.gam[op * GC + GC - 1];
  const float el_last = __expf(glast);
  if (tid < GC) {
    const float gv = a.w.ops.gam[op * GC + tid];
    gam[tid] = gv;
    bet[tid] = tid < len ? a.b.beta[(size_t)(tok0 + tid) * hv + h] : 0.f;
    eg[tid] = __expf(gv);
    el[tid] = __expf(glast - gv);
  }
  typedef TileMap<GD> T128;
  typedef TileMap<GC> T64;

  // dW = -dVn S0^T, kept in fragment order (the registers of an accumulator tile, eight at a time, are exactly the
  // fragment of its column) in the first 16 KB of X: it is the second half of the right-hand side below
  {
    f32x16 acc[2] = {zero16(), zero16()};
    slab_product<GD, GD>(FragLoader<PK_A>{dvns}, RowsJLoaderB{s0t, GD, GD}, acc, as, bs, tid);
#pragma unroll
    for (int t = 0; t < 2; t++)                        // tile (row block t, column block w)
#pragma unroll
      for (int tt = 0; tt < 2; tt++)
        ((bf16x8*)X)[(((w * 2 + T128::ib(w, t)) * 2 + tt) * 64 + lane)] =
            cvt8(-acc[t][8 * tt], -acc[t][8 * tt + 1], -acc[t][8 * tt + 2], -acc[t][8 * tt + 3], -acc[t][8 * tt + 4],
                 -acc[t][8 * tt + 5], -acc[t][8 * tt + 6], -acc[t][8 * tt + 7]);
  }
  // (I + A)^T x = rhs for the 256 columns of [dVn | dW]: x = T^T rhs with T = (I + A)^-1 from the prepare kernel,
  // computed transposed, X^T = rhs^T T, on the matrix cores.  rhs^T comes straight from the fragment-ordered
  // arrays (a fragment is the A operand of its column block for one k-step, its 8 tokens in accumulator order);
  // T is split into two bf16 halves (hi + lo) in LDS, k-major, read in the same token order.
  {
    __bf16* th = as;                                   // [token][i], pitch PK_A
    __bf16* tl = (__bf16*)dam;
    const float* Tg = a.w.ops.t + op * (GC * GC);
    lds_barrier();                                     // the last slab of the product above has been read
#pragma unroll
    for (int p = 0; p < GC * GC / 4 / BT; p++) {
      const int e4 = tid + p * BT, k = e4 >> 4, i4 = (e4 & 15) * 4;
      const float4 v = ld4(Tg + e4 * 4);
      const bf16x4 h4 = cvt4(v.x, v.y, v.z, v.w);
      *(bf16x4*)(th + k * PK_A + i4) = h4;
      *(bf16x4*)(tl + k * PK_A + i4) = cvt4(v.x - (float)h4[0], v.y - (float)h4[1], v.z - (float)h4[2], v.w - (float)h4[3]);
    }
    // wave w: right-hand-side column blocks 2 w and 2 w + 1 (blocks 0 .. 3: dVn, 4 .. 7: dW)
    bf16x8 af[2][GC / 16];
    __syncthreads();                                   // T in LDS; the dW fragments written above are visible
#pragma unroll
    for (int rbi = 0; rbi < 2; rbi++) {
      const int rb = 2 * w + rbi;
      const bf16x8* src = rb < 4 ? (const bf16x8*)dvns + (size_t)rb * 4 * 64 : (const bf16x8*)X + (size_t)(rb - 4) * 4 * 64;
#pragma unroll
      for (int s4 = 0; s4 < GC / 16; s4++) af[rbi][s4] = src[s4 * 64 + lane];      // (half, t) = (s4 / 2, s4 % 2)
    }
    f32x16 xa[2][2] = {{zero16(), zero16()}, {zero16(), zero16()}};
#pragma unroll
    for (int s4 = 0; s4 < GC / 16; s4++)
#pragma unroll
      for (int cb = 0; cb < 2; cb++) {
        const bf16x8 bh = kmajor_frag_acc_order(th, PK_A, 16 * s4 + 4 * hf, 32 * cb + 16 * (c >> 4), lane);
        const bf16x8 bl = kmajor_frag_acc_order(tl, PK_A, 16 * s4 + 4 * hf, 32 * cb + 16 * (c >> 4), lane);
#pragma unroll
        for (int rbi = 0; rbi < 2; rbi++) {
          xa[rbi][cb] = mfma32(af[rbi][s4], bh, xa[rbi][cb]);
          xa[rbi][cb] = mfma32(af[rbi][s4], bl, xa[rbi][cb]);
        }
      }
    __syncthreads();                                   // every wave holds its dW fragments: X may be overwritten
    // X[i][column]: a lane holds row i = 32 cb + c and, per register group, 4 consecutive columns
#pragma unroll
    for (int rbi = 0; rbi < 2; rbi++)
#pragma unroll
      for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++)
          *(bf16x4*)(X + (size_t)(32 * cb + c) * (2 * GD) + 32 * (2 * w + rbi) + r4 * 8 + 4 * hf) =
              cvt4(xa[rbi][cb][4 * r4], xa[rbi][cb][4 * r4 + 1], xa[rbi][cb][4 * r4 + 2], xa[rbi][cb][4 * r4 + 3]);
  }
  __syncthreads();

  // dA = strictly-lower( -[dVb | dKb] [U | W]^T ),  dP = tril( dO Vn^T )
  {
    f32x16 acc[1] = {zero16()};
    slab_product<GC, 2 * GD>(RowsKLoaderA{X, 2 * GD, GC}, UwLoaderB{ut, wtn}, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int i = 32 * T64::ib(w, 0) + tile_row(r, hf), j = 32 * T64::jb(w) + c;
      dam[i * AP + j] = i > j ? -acc[0][r] : 0.f;
    }
    acc[0] = zero16();
    slab_product<GC, GD>(RowsKLoaderA{dob, vrow32, len}, FragLoaderB{vns}, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int i = 32 * T64::ib(w, 0) + tile_row(r, hf), j = 32 * T64::jb(w) + c;
      dpm[i * AP + j] = i >= j ? acc[0][r] : 0.f;
    }
  }
  __syncthreads();

  // G = dP o P + dA o A: its row sums minus its column sums are the part of dgamma that comes through D
#pragma unroll
  for (int p = 0; p < GC * GC / BT; p++) {
    const int e = tid + p * BT, i = e / GC, j = e % GC;
    const float ga = dam[i * AP + j] * A0[e];
    bs_f[i * AP + j] = ga;                   // its row sums are the part of dbeta that comes through A
    gm[i * AP + j] = dpm[i * AP + j] * Pm[e] + bet[i] * ga;
  }
  __syncthreads();
  {
    // row sums and column sums of G, row sums of dA o A0: four threads per row / column, 16 independent LDS reads
    // each (a single thread walking all 64 waits for every read in turn), then two lane exchanges
    const int n = tid >> 2, part = (tid & 3) * 16;
    float s_row = 0.f, s_col = 0.f, s_a = 0.f;
#pragma unroll
    for (int e = 0; e < 16; e++) {
      s_row += gm[n * AP + part + e];
      s_col += gm[(part + e) * AP + n];
      s_a += bs_f[n * AP + part + e];
    }
    s_row += __shfl_xor(s_row, 1); s_row += __shfl_xor(s_row, 2);
    s_col += __shfl_xor(s_col, 1); s_col += __shfl_xor(s_col, 2);
    s_a += __shfl_xor(s_a, 1); s_a += __shfl_xor(s_a, 2);
    if ((tid & 3) == 0) {
      dg_row[n] = s_row;
      dg_col[n] = s_col;
      db_a[n] = s_a;
    }
  }
  __syncthreads();
  // dP -> dP scale D,  dA -> dA beta_i D   (the factors that multiply k_j, q_i, k_i in the products below)
#pragma unroll
  for (int p = 0; p < GC * GC / BT; p++) {
    const int e = tid + p * BT, i = e / GC, j = e % GC;
    const float dec = i >= j ? __expf(gam[i] - gam[j]) : 0.f;
    dpm[i * AP + j] *= scale * dec;
    dam[i * AP + j] *= bet[i] * dec;
  }
  // (the first slab_product below starts with a barrier)

  // dq_i = scale exp(gamma_i) (dO S0^T)_i + sum_j (dP scale D)_ij k_j
  {
    f32x16 acc[2] = {zero16(), zero16()};
    slab_product<GD, GD>(RowsKLoaderA{dob, vrow32, len}, RowsJLoaderB{s0t, GD, GD}, acc, as, bs, tid);
    const int j = 32 * T128::jb(w) + c;
#pragma unroll
    for (int t = 0; t < 2; t++) {
      // One tile at a time (register pressure); its 16 loads in one straight-line block in front of the sums: the
      // conditional LDS write below ends a basic block per row, and a load left inside would be waited for there,
      // one memory latency per row (measured: a quarter of the kernel's time).
      __builtin_amdgcn_sched_barrier(0);
      float qv[16];
#pragma unroll
      for (int r = 0; r < 16; r++) qv[r] = q_at(32 * T128::ib(w, t) + tile_row(r, hf), j);
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int i = 32 * T128::ib(w, t) + tile_row(r, hf);
        acc[t][r] *= scale * eg[i];                                 // scale eg dQg_i: its contribution to dq_i
        const float dot = half_wave_sum(acc[t][r] * qv[r]);         // dQg_i . Qg_i = (scale eg dQg_i) . q_i
        if (c == HALF_SUM_LANE) dot_q[w][i] = dot;
      }
    }
    slab_product<GD, GC>(fn_loader_a([&](int i, int k) { return dpm[i * AP + k]; }), RowsJLoaderB{kb, qrow32, len}, acc, as, bs, tid);
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int i = 32 * T128::ib(w, t) + tile_row(r, hf);
        if (i < len) a.w.dqh[((size_t)(tok0 + i) * a.b.hv_n + h) * GD + j] = acc[t][r];
      }
  }
  __builtin_amdgcn_sched_barrier(0);
  // dk_j = el_j (Vn dS1^T)_j + beta_j eg_j dKb_j + sum_i (dP scale D)_ij q_i + sum_i (MA_ij + MA_ji) k_i
  {
    f32x16 acc[2] = {zero16(), zero16()};
    slab_product<GD, GD>(FragLoader<PK_A>{vns}, RowsJLoaderB{ds1t, GD, GD}, acc, as, bs, tid);
    int zz = 0;
    asm volatile("" : "+v"(zz));          // row offsets are recomputed here, not kept in registers since the dq block
    const int d = 32 * T128::jb(w) + c + zz;
#pragma unroll
    for (int t = 0; t < 2; t++) {
      __builtin_amdgcn_sched_barrier(0);
      float kvs[16], dkbs[16];              // loads first, as above
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int i = 32 * T128::ib(w, t) + tile_row(r, hf);
        kvs[r] = k_at(i, d);
        dkbs[r] = (float)X[i * (2 * GD) + GD + d];
      }
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int i = 32 * T128::ib(w, t) + tile_row(r, hf);
        const float fe = el[i], fkb = bet[i] * eg[i];
        const float kv = kvs[r], dkb = dkbs[r];
        const float s_kd = half_wave_sum(acc[t][r] * kv), s_kb = half_wave_sum(dkb * kv);
        if (c == HALF_SUM_LANE) {
          dot_kd[w][i] = s_kd;
          dot_kb[w][i] = s_kb;
        }
        acc[t][r] = fe * acc[t][r] + fkb * dkb;
      }
    }
    slab_product<GD, GC>(fn_loader_a([&](int i, int k) { return dpm[k * AP + i]; }), RowsJLoaderB{qb, qrow32, len}, acc, as, bs, tid);
    slab_product<GD, GC>(fn_loader_a([&](int i, int k) { return dam[i * AP + k] + dam[k * AP + i]; }), RowsJLoaderB{kb, qrow32, len}, acc, as, bs,
                         tid);
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int i = 32 * T128::ib(w, t) + tile_row(r, hf);
        if (i < len) a.w.dkh[((size_t)(tok0 + i) * a.b.hv_n + h) * GD + d] = acc[t][r];
      }
  }
  // dv_i = beta_i dVb_i,  dbeta_i += dVb_i . v_i
  {
    const int i = tid >> 2, c0 = (tid & 3) * 32;
    float dot = 0.f;
    bf16x8 xb[4], vv[4];
#pragma unroll
    for (int q = 0; q < 4; q++) {
      xb[q] = *(const bf16x8*)(X + i * (2 * GD) + c0 + 8 * q);
      vv[q] = *(const bf16x8*)(vb + (size_t)min(i, len - 1) * vrow + c0 + 8 * q);
    }
    const float b = bet[i];
#pragma unroll
    for (int q = 0; q < 4; q++) {
      float xv[8];
#pragma unroll
      for (int e = 0; e < 8; e++) {
        xv[e] = (float)xb[q][e];
        dot += xv[e] * (float)vv[q][e];
      }
      if (i < len)
        *(bf16x8*)((__bf16*)a.b.dv + ((size_t)(tok0 + i) * hv + h) * GD + c0 + 8 * q) =
            cvt8(b * xv[0], b * xv[1], b * xv[2], b * xv[3], b * xv[4], b * xv[5], b * xv[6], b * xv[7]);
    }
    dot += __shfl_xor(dot, 1);
    dot += __shfl_xor(dot, 2);
    if ((tid & 3) == 0) db_v[i] = i < len ? dot : 0.f;
  }
  // <dS1, S0>: gamma_last also scales the state that is carried over
  __syncthreads();                     // every wave is done with the slab arrays (red lives there)
  {
    float s = 0.f;
#pragma unroll
    for (int p = 0; p < (GD * GD / 8) / BT; p++) {
      const bf16x8 x = *(const bf16x8*)(ds1t + 8 * (tid + p * BT)), y = *(const bf16x8*)(s0t + 8 * (tid + p * BT));
#pragma unroll
      for (int e = 0; e < 8; e++) s += (float)x[e] * (float)y[e];
    }
    red[tid] = s;
  }
  __syncthreads();
  if (tid < GC) {
    // state inner product: 256 partial sums -> 64 (fixed order), the rest below
    red[tid] = (red[tid] + red[tid + 64]) + (red[tid + 128] + red[tid + 192]);
  }
  __syncthreads();
  if (tid < GC) {
    // row dot products: the four waves hold a quarter of the columns each
    const float dq_ = dot_q[0][tid] + dot_q[1][tid] + dot_q[2][tid] + dot_q[3][tid];
    const float dkd = el[tid] * (dot_kd[0][tid] + dot_kd[1][tid] + dot_kd[2][tid] + dot_kd[3][tid]);      // dKd_i . Kd_i
    const float dkb = dot_kb[0][tid] + dot_kb[1][tid] + dot_kb[2][tid] + dot_kb[3][tid];                  // dKb_i . k_i
    dgam[tid] = dg_row[tid] - dg_col[tid] + dq_ - dkd + bet[tid] * eg[tid] * dkb;
    red[64 + tid] = dkd + el_last * red[tid];             // what reaches every g through gamma_last, 64 parts
    red[128 + tid] = db_a[tid] + eg[tid] * dkb + db_v[tid];
  }
  __syncthreads();
  if (tid < len) {
    float s = 0.f, last = 0.f;
#pragma unroll
    for (int i = 0; i < GC; i++) {                        // independent reads, fixed order
      s += i >= tid ? dgam[i] : 0.f;                      // gamma_i = sum of g_j over j <= i
      last += red[64 + i];
    }
    a.b.dg[(size_t)(tok0 + tid) * hv + h] = s + last;
    a.b.dbeta[(size_t)(tok0 + tid) * hv + h] = red[128 + tid];
  }
}

// dq, dk [N][hk][128] bf16 = sum over the value heads of a group of the per-head fp32 gradients
__global__ __launch_bounds__(BT) void gdn_bwd_group_sum_kernel(KArgs a) {
  const int rep = a.b.hv / a.b.hk, hk_n = a.b.hv_n / rep;          // key heads of this pass
  const size_t n4 = (size_t)a.b.n_tokens * hk_n * (GD / 4);
  for (size_t e = (size_t)blockIdx.x * BT + threadIdx.x; e < n4; e += (size_t)gridDim.x * BT) {
    const size_t t = e / ((size_t)hk_n * (GD / 4));
    const int rem = (int)(e % ((size_t)hk_n * (GD / 4))), kh = rem / (GD / 4), d4 = (rem % (GD / 4)) * 4;
    float4 sq = make_float4(0.f, 0.f, 0.f, 0.f), sk = sq;
    for (int r = 0; r < rep; r++) {
      const size_t src = ((size_t)t * a.b.hv_n + kh * rep + r) * GD + d4;
      const float4 x = ld4(a.w.dqh + src), y = ld4(a.w.dkh + src);
      sq.x += x.x; sq.y += x.y; sq.z += x.z; sq.w += x.w;
      sk.x += y.x; sk.y += y.y; sk.z += y.z; sk.w += y.w;
    }
    const size_t dst = ((size_t)t * a.b.hk + kh) * GD + d4;
    *(bf16x4*)((__bf16*)a.b.dq + dst) = cvt4(sq.x, sq.y, sq.z, sq.w);
    *(bf16x4*)((__bf16*)a.b.dk + dst) = cvt4(sk.x, sk.y, sk.z, sk.w);
  }
}

__global__ __launch_bounds__(BT) void gdn_bwd_fill_zero_kernel(float4* p, size_t n4) {
  for (size_t e = (size_t)blockIdx.x * BT + threadIdx.x; e < n4; e += (size_t)gridDim.x * BT) p[e] = make_float4(0.f, 0.f, 0.f, 0.f);
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// carves the workspace; returns the total size (with p == nullptr: only the size)
// (hv_n: value heads of one pass; the saved states and their gradients keep the tensors' head stride hv)
size_t carve(char* p, int64_t n_tokens, int n_chunks, int n_slots, int n_segments, int hv, int hv_n, BwdWs* w) {
  const size_t per = (size_t)n_chunks * hv_n;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char* r = p ? p + off : nullptr;
    off += align256(bytes);
    return r;
  };
  BwdWs t{};
  t.ops.gam = (float*)take(per * GC * 4);
  t.ops.a0 = (float*)take(per * GC * GC * 4);
  t.ops.p = (float*)take(per * GC * GC * 4);
  t.ops.t = (float*)take(per * GC * GC * 4);
  t.sv.fwd_rec = take(per * GDN_REC_ELEMS * 2);
  t.sv.rev_rec = take(per * GDN_REC_ELEMS * 2);
  t.sv.glast = (float*)take(per * 4);
  t.sv.s0t = take(per * GD * GD * 2);
  t.sv.ds1t = take(per * GD * GD * 2);
  t.sv.vns = take(per * GC * GD * 2);
  t.sv.dvns = take(per * GC * GD * 2);
  t.sv.slots = (float*)take((size_t)n_slots * hv * GD * GD * 4);
  t.sv.slot_grad = (float*)take((size_t)n_slots * hv * GD * GD * 4);
  t.sv.seg_grad = (float*)take((size_t)n_segments * hv * GD * GD * 4);
  t.x = (__bf16*)take(per * GC * 2 * GD * 2);
  t.dqh = (float*)take((size_t)n_tokens * hv_n * GD * 4);
  t.dkh = (float*)take((size_t)n_tokens * hv_n * GD * 4);
  if (w) *w = t;
  return off + 256;
}

}  // namespace

size_t gdn_bwd_workspace(int64_t n_tokens, int n_chunks, int n_slots, int n_segments, int hk, int hv, int key_heads_per_pass) {
  return carve(nullptr, n_tokens, n_chunks, n_slots, n_segments, hv, key_heads_per_pass * (hv / hk), nullptr);
}

// The value heads are independent of each other up to the final sum over the value heads of a key head, so the
// pass can be cut into batches of whole key-head groups: as many per batch as the workspace holds.  A batch sees
// the tensors through pointers moved to its first head (the head counts stay the strides).
hipError_t gdn_bwd(const GdnBwdArgs& b0, hipStream_t st) {
  if (b0.n_chunks == 0 || b0.n_tokens == 0) return hipSuccess;
  const int rep = b0.hv / b0.hk, n_seg = b0.sched ? b0.sched->n_segments : 0;
  int per_pass = b0.hk;
  while (per_pass > 1 && gdn_bwd_workspace(b0.n_tokens, b0.n_chunks, b0.n_slots, n_seg, b0.hk, b0.hv, per_pass) > b0.workspace_bytes)
    per_pass--;
  if (gdn_bwd_workspace(b0.n_tokens, b0.n_chunks, b0.n_slots, n_seg, b0.hk, b0.hv, per_pass) > b0.workspace_bytes)
    return hipErrorInvalidValue;
  auto zero = [&](float* p, size_t floats) {
    if (floats == 0) return;
    const size_t n4 = floats / 4;
    gdn_bwd_fill_zero_kernel<<<dim3((unsigned)std::min<size_t>((n4 + BT - 1) / BT, 4096)), BT, 0, st>>>((float4*)p, n4);
  };
  for (int kh0 = 0; kh0 < b0.hk; kh0 += per_pass) {
    const int hk_n = std::min(per_pass, b0.hk - kh0), h0 = kh0 * rep;
    GdnBwdArgs b = b0;
    b.hv_n = hk_n * rep;
    const size_t ko = (size_t)kh0 * GD, vo = (size_t)h0 * GD, so = (size_t)h0 * GD * GD;
    b.q = (const __bf16*)b0.q + ko; b.k = (const __bf16*)b0.k + ko; b.v = (const __bf16*)b0.v + vo; b.d_o = (const __bf16*)b0.d_o + vo;
    b.g = b0.g + h0; b.beta = b0.beta + h0;
    b.dq = (__bf16*)b0.dq + ko; b.dk = (__bf16*)b0.dk + ko; b.dv = (__bf16*)b0.dv + vo;
    b.dg = b0.dg + h0; b.dbeta = b0.dbeta + h0;
    if (b0.initial_state) b.initial_state = b0.initial_state + so;
    if (b0.d_state_out) b.d_state_out = b0.d_state_out + so;
    if (b0.d_initial_state) b.d_initial_state = b0.d_initial_state + so;
    KArgs a{};
    a.b = b;
    carve((char*)b.workspace, b.n_tokens, b.n_chunks, b.n_slots, n_seg, b.hv, b.hv_n, &a.w);
    // walking all chunks in sequence order, readers add into the slot gradients and into d_initial_state; with a
    // schedule every segment stores its own gradient and nothing has to start from zero
    if (!b.sched) {
      zero(a.w.sv.slot_grad, (size_t)b.n_slots * b.hv * GD * GD);
      if (b.d_initial_state) {
        // the rows of this pass's heads (one contiguous piece: heads are the outer index)
        zero(b.d_initial_state, (size_t)b.hv_n * GD * GD);
      }
    }
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    if (hipError_t e = gdn_bwd_prepare_and_walks(b, a.w.ops, a.w.sv, st); e != hipSuccess) return e;
    {
      KernelTimer t(TT_KERNEL_GDN_BWD_FINISH, st);
      gdn_bwd_finish_kernel<<<gdn_group_order_grid(b.n_chunks, b.hv_n, b.hv / b.hk), BT, 0, st>>>(a);
    }
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    {
      const size_t n4 = (size_t)b.n_tokens * hk_n * (GD / 4);
      gdn_bwd_group_sum_kernel<<<dim3((unsigned)std::min<size_t>((n4 + BT - 1) / BT, 8192)), BT, 0, st>>>(a);
    }
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace tt
