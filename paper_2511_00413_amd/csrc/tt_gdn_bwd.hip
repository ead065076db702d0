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
//                              (Kd, -W^T, Qg^T, P^T, dO^T) and gamma, A0, P, U, W unrounded
//   gdn_scan_kernel<true>      (32 value columns, head): the forward scan without its output; saves S0 and Vn
//                              of every chunk (bf16)
//   gdn_rscan_kernel           (32 value columns, head): reverse walk in the forward scan's form (bf16 matrix
//                              instruction, fp32 state gradient in accumulators); saves dS1 and dVn (bf16)
//   gdn_bwd_finish_kernel      per (chunk, head): everything else, fp32 vector arithmetic with LDS-tiled
//                              products; dq / dk per value head in fp32
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
constexpr int DVB = 32;              // value columns per scan workgroup
constexpr int KS = 32;               // k-slab of the LDS-tiled products of the finish kernel

struct BwdWs {
  GdnChunkOps ops;
  GdnBwdSaved sv;
  float* x;          // per (head, chunk) [64][256]: [dW] on the way in, [dVb | dKb] after the transposed solve
  float* dqh;        // [N][hv][128] per-value-head dq, dk
  float* dkh;
};
struct KArgs {
  GdnBwdArgs b;
  BwdWs w;
};

__device__ __forceinline__ float4 ld4(const float* p) { return *(const float4*)p; }
__device__ __forceinline__ void st4(float* p, const float (&v)[4]) { *(float4*)p = make_float4(v[0], v[1], v[2], v[3]); }

// ---- per-chunk finish ----------------------------------------------------------------------------------
// acc[r][c] += sum_k fa(i, k) fb(k, j) for i = 4 ty + r, j = tile_col(tx, c), over K (a multiple of KS), through
// LDS slabs of KS k-values.  AKF / BKF: consecutive threads fetch consecutive k (operand stored with k
// contiguous) rather than consecutive i / j.  Every thread of the workgroup must call it.
// Output tile of thread (ty, tx): rows 4 ty .. 4 ty + 3; columns tile_col<N, TN>(tx, c), c = 0 .. TN - 1: groups of four
// consecutive columns, the groups N / (TN / 4) apart -- every LDS read of the inner loop is one 16-byte read and
// neighbouring threads read neighbouring 16-byte pieces.
template <int N, int TN>
__device__ __forceinline__ int tile_col(int tx, int c) { return (c >> 2) * (N / (TN / 4)) + tx * 4 + (c & 3); }

template <int M, int N, int TM, int TN, bool AKF, bool BKF, class FA, class FB>
__device__ __forceinline__ void slab_product(int K, FA fa, FB fb, float (&acc)[TM][TN], float* as, float* bs, int tid) {
  constexpr int NT = N / TN, PA = M + 4, PB = N + 4;      // row pitches: 16-byte aligned rows
  static_assert((M / TM) * NT == BT && TM == 4 && TN % 4 == 0, "one 4 x TN output tile per thread");
  const int tx = tid % NT, ty = tid / NT;
  for (int k0 = 0; k0 < K; k0 += KS) {
    __syncthreads();
    float av[M * KS / BT], bv[N * KS / BT];
#pragma unroll
    for (int p = 0; p < M * KS / BT; p++) {
      const int e = tid + p * BT;
      const int kk = AKF ? e % KS : e / M, i = AKF ? e / KS : e % M;
      av[p] = fa(i, k0 + kk);
    }
#pragma unroll
    for (int p = 0; p < N * KS / BT; p++) {
      const int e = tid + p * BT;
      const int kk = BKF ? e % KS : e / N, j = BKF ? e / KS : e % N;
      bv[p] = fb(k0 + kk, j);
    }
#pragma unroll
    for (int p = 0; p < M * KS / BT; p++) {
      const int e = tid + p * BT;
      const int kk = AKF ? e % KS : e / M, i = AKF ? e / KS : e % M;
      as[kk * PA + i] = av[p];
    }
#pragma unroll
    for (int p = 0; p < N * KS / BT; p++) {
      const int e = tid + p * BT;
      const int kk = BKF ? e % KS : e / N, j = BKF ? e / KS : e % N;
      bs[kk * PB + j] = bv[p];
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < KS; kk++) {
      const float4 a4 = *(const float4*)&as[kk * PA + ty * 4];
      const float ar[4] = {a4.x, a4.y, a4.z, a4.w};
      float bc[TN];
#pragma unroll
      for (int c4 = 0; c4 < TN / 4; c4++) {
        const float4 b4 = *(const float4*)&bs[kk * PB + tile_col<N, TN>(tx, 4 * c4)];
        bc[4 * c4] = b4.x; bc[4 * c4 + 1] = b4.y; bc[4 * c4 + 2] = b4.z; bc[4 * c4 + 3] = b4.w;
      }
#pragma unroll
      for (int r = 0; r < TM; r++)
#pragma unroll
        for (int c = 0; c < TN; c++) acc[r][c] = fmaf(ar[r], bc[c], acc[r][c]);
    }
  }
}

// sum over the 16 consecutive lanes that share a row of a [64][128] tile
__device__ __forceinline__ float row16_sum(float x) {
  x += __shfl_xor(x, 1); x += __shfl_xor(x, 2); x += __shfl_xor(x, 4); x += __shfl_xor(x, 8);
  return x;
}

constexpr int AP = GC + 1;     // row pitch of the 64 x 64 LDS matrices that are read along rows and columns
constexpr int TP = GC + 4;     // pitch of the transposed A during the solve (rows read as float4)

__global__ __launch_bounds__(BT) void gdn_bwd_finish_kernel(KArgs a) {
  __shared__ __attribute__((aligned(16))) float as[KS * (GC + 4)];
  __shared__ __attribute__((aligned(16))) float bs[GC * AP > KS * (GD + 4) ? GC * AP : KS * (GD + 4)];   // between products also: dA o A0
  __shared__ __attribute__((aligned(16))) float dam[GC * TP];     // A^T during the solve, then dA, then dA beta D
  __shared__ float dpm[GC * AP];                                  // dP, then dP scale D
  __shared__ float gm[GC * AP];                                   // dP o P + dA o A
  __shared__ float gam[GC], bet[GC], eg[GC], el[GC];
  __shared__ float dg_row[GC], dg_col[GC], dg_q[GC], dg_kd[GC], dg_kb[GC], db_a[GC], db_kb[GC], db_v[GC], dgam[GC];
  __shared__ float red[BT];

  const int chunk = blockIdx.x, h = blockIdx.y;
  const int tid = threadIdx.x & (BT - 1);
  const int nc = a.b.n_chunks, hv = a.b.hv, kh = h / (hv / a.b.hk);
  const size_t op = (size_t)h * nc + chunk;
  const int tok0 = a.b.chunk_tok0[chunk], len = a.b.chunk_len[chunk];
  const float scale = a.b.scale;
  const float* U = a.w.ops.u + op * (GC * GD);
  const float* Wm = a.w.ops.w + op * (GC * GD);
  const float* A0 = a.w.ops.a0 + op * (GC * GC);
  const float* Pm = a.w.ops.p + op * (GC * GC);
  // saved by the walks (bf16): S0 and dS1 transposed [value col][key dim], Vn and dVn in fragment order
  const __bf16* s0t = (const __bf16*)a.w.sv.s0t + op * (GD * GD);
  const __bf16* ds1t = (const __bf16*)a.w.sv.ds1t + op * (GD * GD);
  const __bf16* vns = (const __bf16*)a.w.sv.vns + op * (GC * GD);
  const __bf16* dvns = (const __bf16*)a.w.sv.dvns + op * (GC * GD);
  auto s0_at = [&](int d, int cc) { return (float)s0t[cc * GD + d]; };
  auto ds1_at = [&](int d, int cc) { return (float)ds1t[cc * GD + d]; };
  auto vn_at = [&](int i, int cc) { return (float)vns[gdn_frag_index(i, cc)]; };
  auto dvn_at = [&](int i, int cc) { return (float)dvns[gdn_frag_index(i, cc)]; };
  float* X = a.w.x + op * (GC * 2 * GD);
  const size_t qrow = (size_t)a.b.hk * GD, vrow = (size_t)hv * GD;
  const __bf16* qb = (const __bf16*)a.b.q + (size_t)tok0 * qrow + (size_t)kh * GD;
  const __bf16* kb = (const __bf16*)a.b.k + (size_t)tok0 * qrow + (size_t)kh * GD;
  const __bf16* vb = (const __bf16*)a.b.v + (size_t)tok0 * vrow + (size_t)h * GD;
  const __bf16* dob = (const __bf16*)a.b.d_o + (size_t)tok0 * vrow + (size_t)h * GD;
  // rows past the chunk's length read a valid row and are then zeroed (no load sits inside a branch)
  auto q_at = [&](int i, int d) { const float x = (float)qb[(size_t)min(i, len - 1) * qrow + d]; return i < len ? x : 0.f; };
  auto k_at = [&](int i, int d) { const float x = (float)kb[(size_t)min(i, len - 1) * qrow + d]; return i < len ? x : 0.f; };
  auto do_at = [&](int i, int c) { const float x = (float)dob[(size_t)min(i, len - 1) * vrow + c]; return i < len ? x : 0.f; };

  const float glast = a.w.ops.gam[op * GC + GC - 1];
  const float el_last = __expf(glast);
  if (tid < GC) {
    const float gv = a.w.ops.gam[op * GC + tid];
    gam[tid] = gv;
    bet[tid] = tid < len ? a.b.beta[(size_t)(tok0 + tid) * hv + h] : 0.f;
    eg[tid] = __expf(gv);
    el[tid] = __expf(glast - gv);
  }

  // dW = -dVn S0^T  -> right half of X
  {
    float acc[4][8];
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 8; c++) acc[r][c] = 0.f;
    slab_product<GC, GD, 4, 8, true, false>(GD, dvn_at, [&](int k, int j) { return s0_at(j, k); }, acc, as, bs, tid);
    const int tx = tid & 15, ty = tid >> 4;
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 8; c++) X[(ty * 4 + r) * (2 * GD) + GD + tile_col<GD, 8>(tx, c)] = -acc[r][c];
  }
  // A^T into LDS: dam[i][j] = A_ji = beta_j A0_ji  (zero for j <= i)
#pragma unroll
  for (int p = 0; p < GC * GC / BT; p++) {
    const int e = tid + p * BT, j = e / GC, i = e % GC;
    dam[i * TP + j] = bet[j] * A0[e];
  }
  __syncthreads();

  // (I + A)^T x = rhs by back substitution, one lane per column of [dVn | dW]:  x_i = rhs_i - sum_{j>i} A_ji x_j
  {
    const int c = tid;
    float x[GC];
    // right-hand sides: 64 independent loads per lane in one straight-line block
    if (c < GD) {
#pragma unroll
      for (int i = 0; i < GC; i++) x[i] = dvn_at(i, c);
    } else {
#pragma unroll
      for (int i = 0; i < GC; i++) x[i] = X[i * (2 * GD) + c];
    }
#pragma unroll
    for (int i = GC - 2; i >= 0; i--) {
      float v = x[i];
#pragma unroll
      for (int j4 = (i + 1) / 4; j4 < GC / 4; j4++) {
        const float4 av = *(const float4*)&dam[i * TP + j4 * 4];
        const float ae[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
        for (int e = 0; e < 4; e++)
          if (j4 * 4 + e > i) v -= ae[e] * x[j4 * 4 + e];
      }
      x[i] = v;
    }
#pragma unroll
    for (int i = 0; i < GC; i++) X[i * (2 * GD) + c] = x[i];
  }
  __syncthreads();

  // dA = strictly-lower( -[dVb | dKb] [U | W]^T ),  dP = tril( dO Vn^T )
  {
    float acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 4; c++) acc[r][c] = 0.f;
    slab_product<GC, GC, 4, 4, true, true>(2 * GD, [&](int i, int k) { return X[i * (2 * GD) + k]; },
                                           [&](int k, int j) { return *(k < GD ? U + j * GD + k : Wm + j * GD + (k - GD)); }, acc, as, bs,
                                           tid);
    const int tx = tid & 15, ty = tid >> 4;
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 4; c++) {
        const int i = ty * 4 + r, j = tile_col<GC, 4>(tx, c);
        dam[i * AP + j] = i > j ? -acc[r][c] : 0.f;
      }
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 4; c++) acc[r][c] = 0.f;
    slab_product<GC, GC, 4, 4, true, true>(GD, do_at, [&](int k, int j) { return vn_at(j, k); }, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 4; c++) {
        const int i = ty * 4 + r, j = tile_col<GC, 4>(tx, c);
        dpm[i * AP + j] = i >= j ? acc[r][c] : 0.f;
      }
  }
  __syncthreads();

  // G = dP o P + dA o A: its row sums minus its column sums are the part of dgamma that comes through D
#pragma unroll
  for (int p = 0; p < GC * GC / BT; p++) {
    const int e = tid + p * BT, i = e / GC, j = e % GC;
    const float ga = dam[i * AP + j] * A0[e];
    bs[i * AP + j] = ga;                     // its row sums are the part of dbeta that comes through A
    gm[i * AP + j] = dpm[i * AP + j] * Pm[e] + bet[i] * ga;
  }
  __syncthreads();
  if (tid < GC) {
    float s = 0.f;
    for (int i = 0; i < GC; i++) s += gm[i * AP + tid];
    dg_col[tid] = s;
  } else if (tid < 2 * GC) {
    const int i = tid - GC;
    float s = 0.f;
    for (int j = 0; j < GC; j++) s += gm[i * AP + j];
    dg_row[i] = s;
  } else if (tid < 3 * GC) {
    const int i = tid - 2 * GC;
    float s = 0.f;
    for (int j = 0; j < GC; j++) s += bs[i * AP + j];
    db_a[i] = s;
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

  const int tx = tid & 15, ty = tid >> 4;
  // dq_i = scale exp(gamma_i) (dO S0^T)_i + sum_j (dP scale D)_ij k_j
  {
    float acc[4][8];
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 8; c++) acc[r][c] = 0.f;
    slab_product<GC, GD, 4, 8, true, false>(GD, do_at, [&](int k, int j) { return s0_at(j, k); }, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int i = ty * 4 + r;
      const float f = scale * eg[i];
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < 8; c++) {
        acc[r][c] *= f;                               // dQg_i scaled = its contribution to dq_i
        dot += acc[r][c] * q_at(i, tile_col<GD, 8>(tx, c));      // dQg_i . Qg_i = (scale eg dQg_i) . q_i
      }
      dot = row16_sum(dot);
      if (tx == 0) dg_q[i] = dot;
    }
    slab_product<GC, GD, 4, 8, true, false>(GC, [&](int i, int k) { return dpm[i * AP + k]; }, k_at, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int i = ty * 4 + r;
      if (i < len) {
        float* dst = a.w.dqh + ((size_t)(tok0 + i) * hv + h) * GD;
#pragma unroll
        for (int c4 = 0; c4 < 2; c4++)
          *(float4*)(dst + tile_col<GD, 8>(tx, 4 * c4)) = make_float4(acc[r][4 * c4], acc[r][4 * c4 + 1], acc[r][4 * c4 + 2], acc[r][4 * c4 + 3]);
      }
    }
  }
  // dk_j = el_j (Vn dS1^T)_j + beta_j eg_j dKb_j + sum_i (dP scale D)_ij q_i + sum_i (MA_ij + MA_ji) k_i
  {
    float acc[4][8];
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 8; c++) acc[r][c] = 0.f;
    slab_product<GC, GD, 4, 8, true, false>(GD, vn_at, [&](int k, int j) { return ds1_at(j, k); }, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int i = ty * 4 + r;
      const float fe = el[i], fb_ = bet[i] * eg[i];
      float dot_kd = 0.f, dot_kb = 0.f;
#pragma unroll
      for (int c = 0; c < 8; c++) {
        const int d = tile_col<GD, 8>(tx, c);
        const float kv = k_at(i, d), dkb = X[i * (2 * GD) + GD + d];
        dot_kd += acc[r][c] * kv;
        dot_kb += dkb * kv;
        acc[r][c] = fe * acc[r][c] + fb_ * dkb;
      }
      dot_kd = row16_sum(dot_kd);
      dot_kb = row16_sum(dot_kb);
      if (tx == 0) {
        dg_kd[i] = fe * dot_kd;                 // dKd_i . Kd_i
        db_kb[i] = eg[i] * dot_kb;
        dg_kb[i] = fb_ * dot_kb;                // dKb_i . (beta eg K)_i
      }
    }
    slab_product<GC, GD, 4, 8, false, false>(GC, [&](int i, int k) { return dpm[k * AP + i]; }, q_at, acc, as, bs, tid);
    slab_product<GC, GD, 4, 8, false, false>(GC, [&](int i, int k) { return dam[i * AP + k] + dam[k * AP + i]; }, k_at, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int i = ty * 4 + r;
      if (i < len) {
        float* dst = a.w.dkh + ((size_t)(tok0 + i) * hv + h) * GD;
#pragma unroll
        for (int c4 = 0; c4 < 2; c4++)
          *(float4*)(dst + tile_col<GD, 8>(tx, 4 * c4)) = make_float4(acc[r][4 * c4], acc[r][4 * c4 + 1], acc[r][4 * c4 + 2], acc[r][4 * c4 + 3]);
      }
    }
  }
  // dv_i = beta_i dVb_i,  dbeta_i += dVb_i . v_i
  {
    const int i = tid >> 2, c0 = (tid & 3) * 32;
    float dot = 0.f;
#pragma unroll
    for (int c8 = 0; c8 < 32; c8 += 8) {
      const float4 x0 = ld4(X + i * (2 * GD) + c0 + c8), x1 = ld4(X + i * (2 * GD) + c0 + c8 + 4);
      const bf16x8 vv = *(const bf16x8*)(vb + (size_t)min(i, len - 1) * vrow + c0 + c8);
      const float xv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
      for (int e = 0; e < 8; e++) dot += xv[e] * (float)vv[e];
      const float b = bet[i];
      if (i < len)
        *(bf16x8*)((__bf16*)a.b.dv + ((size_t)(tok0 + i) * hv + h) * GD + c0 + c8) =
            cvt8(b * xv[0], b * xv[1], b * xv[2], b * xv[3], b * xv[4], b * xv[5], b * xv[6], b * xv[7]);
    }
    dot += __shfl_xor(dot, 1);
    dot += __shfl_xor(dot, 2);
    if ((tid & 3) == 0) db_v[i] = i < len ? dot : 0.f;
  }
  // <dS1, S0>: gamma_last also scales the state that is carried over
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
  for (int stride = BT / 2; stride > 0; stride >>= 1) {
    if (tid < stride) red[tid] += red[tid + stride];
    __syncthreads();
  }
  if (tid < GC) {
    float v = dg_row[tid] - dg_col[tid] + dg_q[tid] - dg_kd[tid] + dg_kb[tid];
    if (tid == GC - 1) {
      float s = el_last * red[0];
      for (int i = 0; i < GC; i++) s += dg_kd[i];
      v += s;
    }
    dgam[tid] = v;
  }
  __syncthreads();
  if (tid < len) {
    float s = 0.f;
    for (int i = tid; i < GC; i++) s += dgam[i];        // gamma_i = sum of g_j over j <= i
    a.b.dg[(size_t)(tok0 + tid) * hv + h] = s;
    a.b.dbeta[(size_t)(tok0 + tid) * hv + h] = db_a[tid] + db_kb[tid] + db_v[tid];
  }
}

// dq, dk [N][hk][128] bf16 = sum over the value heads of a group of the per-head fp32 gradients
__global__ __launch_bounds__(BT) void gdn_bwd_group_sum_kernel(KArgs a) {
  const int rep = a.b.hv / a.b.hk;
  const size_t n4 = (size_t)a.b.n_tokens * a.b.hk * (GD / 4);
  for (size_t e = (size_t)blockIdx.x * BT + threadIdx.x; e < n4; e += (size_t)gridDim.x * BT) {
    const size_t t = e / ((size_t)a.b.hk * (GD / 4));
    const int rem = (int)(e % ((size_t)a.b.hk * (GD / 4))), kh = rem / (GD / 4), d4 = (rem % (GD / 4)) * 4;
    float4 sq = make_float4(0.f, 0.f, 0.f, 0.f), sk = sq;
    for (int r = 0; r < rep; r++) {
      const size_t src = ((size_t)t * a.b.hv + kh * rep + r) * GD + d4;
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
size_t carve(char* p, int64_t n_tokens, int n_chunks, int n_slots, int hv, BwdWs* w) {
  const size_t per = (size_t)n_chunks * hv;
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
  t.ops.u = (float*)take(per * GC * GD * 4);
  t.ops.w = (float*)take(per * GC * GD * 4);
  t.sv.fwd_rec = take(per * GDN_REC_ELEMS * 2);
  t.sv.rev_rec = take(per * GDN_REC_ELEMS * 2);
  t.sv.glast = (float*)take(per * 4);
  t.sv.s0t = take(per * GD * GD * 2);
  t.sv.ds1t = take(per * GD * GD * 2);
  t.sv.vns = take(per * GC * GD * 2);
  t.sv.dvns = take(per * GC * GD * 2);
  t.sv.slots = (float*)take((size_t)n_slots * hv * GD * GD * 4);
  t.sv.slot_grad = (float*)take((size_t)n_slots * hv * GD * GD * 4);
  t.x = (float*)take(per * GC * 2 * GD * 4);
  t.dqh = (float*)take((size_t)n_tokens * hv * GD * 4);
  t.dkh = (float*)take((size_t)n_tokens * hv * GD * 4);
  if (w) *w = t;
  return off + 256;
}

}  // namespace

size_t gdn_bwd_workspace(int64_t n_tokens, int n_chunks, int n_slots, int hk, int hv) {
  (void)hk;
  return carve(nullptr, n_tokens, n_chunks, n_slots, hv, nullptr);
}

hipError_t gdn_bwd(const GdnBwdArgs& b, hipStream_t st) {
  if (b.n_chunks == 0 || b.n_tokens == 0) return hipSuccess;
  KArgs a{};
  a.b = b;
  carve((char*)b.workspace, b.n_tokens, b.n_chunks, b.n_slots, b.hv, &a.w);
  auto zero = [&](float* p, size_t floats) {
    if (floats == 0) return;
    const size_t n4 = floats / 4;
    gdn_bwd_fill_zero_kernel<<<dim3((unsigned)std::min<size_t>((n4 + BT - 1) / BT, 4096)), BT, 0, st>>>((float4*)p, n4);
  };
  zero(a.w.sv.slot_grad, (size_t)b.n_slots * b.hv * GD * GD);
  if (b.d_initial_state) zero(b.d_initial_state, (size_t)b.hv * GD * GD);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  if (hipError_t e = gdn_bwd_prepare_and_walks(b, a.w.ops, a.w.sv, st); e != hipSuccess) return e;
  {
    KernelTimer t(TT_KERNEL_GDN_BWD_FINISH, st);
    gdn_bwd_finish_kernel<<<dim3(b.n_chunks, b.hv), BT, 0, st>>>(a);
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  {
    const size_t n4 = (size_t)b.n_tokens * b.hk * (GD / 4);
    gdn_bwd_group_sum_kernel<<<dim3((unsigned)std::min<size_t>((n4 + BT - 1) / BT, 8192)), BT, 0, st>>>(a);
  }
  return hipGetLastError();
}

}  // namespace tt
