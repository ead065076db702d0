// Tree attention backward on bf16 MFMA (gfx950), head dim 128.
//
//   D_i = <dO_i, O_i>;  P = exp(S - LSE);  dP = dO V^T;  dS = P o (dP - D);
//   dQ = scale dS K;    dK = scale dS^T Q;  dV = P^T dO
// dK/dV of a key sum over every visible query, i.e. over all branches through the key (paper
// Eq. 5), and over the query heads of the kv group.  Gradients of cached prefix keys are added
// in fp32 to caller-owned accumulators (Appendix "Float32 Gradient Accumulation").
//
// Kernels, no atomics (results are bit-reproducible); the dK/dV pass lives in tt_attn_dkdv.hip and runs
// after the dQ pass, whose prologue also produces the per-row terms D_i and LSE_i log2 e:
//   dkdv      column-parallel: one work item = a key tile of up to 256 keys x one kv head, 8 wavefronts
//             x 32 keys; loops over the query heads of the group and over the 64-query steps that can
//             see the keys -- a contiguous range [first key, max kend) because in DFS order a subtree
//             is contiguous.  S[q,key] = Q K^T and dP[q,key] = dO V^T come out with one key per lane,
//             already in B-operand layout for dV^T[d,key] += dO^T[d,q] P[q,key] and
//             dK^T[d,key] += Q^T[d,q] dS[q,key]; Q^T / dO^T come from transposed LDS reads.
//   dq        row-parallel, same structure as the forward: S^T = K Q^T, dP^T = V dO^T with one
//             query per lane, dQ^T[d,q] += K^T[d,key] dS^T[key,q].
#include <hip/hip_runtime.h>
#include <algorithm>
#include "tt_kernels.h"
#include "tt_mfma.h"

namespace tt {
namespace {

constexpr int D = 128;
constexpr int NTHREADS = 256;

// ------------------------------------------------------------------------------------------------
// dQ
// ------------------------------------------------------------------------------------------------
constexpr int Q_BM = 128;          // queries per workgroup
constexpr int Q_BN = 64;           // keys per tile (= TT_KTILE)
constexpr int Q_TILE_ELEMS = Q_BN * TILE_ROW;

struct QSmem {
  __bf16 k[2][Q_TILE_ELEMS];       // swizzled tiles, filled by asynchronous global -> LDS copies
  __bf16 v[2][Q_TILE_ELEMS];
  int32_t kend[2][Q_BN];
  KTileMasks masks;
};

struct QCtx {
  const AttnArgs& a;
  int kvh, P, N, npt;
};

// Starts the copy of key tile u (K, V rows and visibility bounds) into stage `buf`, all through the
// asynchronous global -> LDS path (a load into a register would make the compiler wait for every
// outstanding memory operation, the tile copies included, at its first use).  Rows past the end of
// the region repeat the last valid row; dq_tile keeps them invisible.
__device__ __forceinline__ void q_issue_tile(const QCtx& c, QSmem& sm, int buf, int u, int w, int lane) {
  const AttnArgs& a = c.a;
  const __bf16 *kp, *vp;
  const int32_t* ke;
  uint32_t ks, vs;
  int rows;
  if (u < c.npt) {
    const int k0 = u * Q_BN;
    kp = (const __bf16*)a.k_prefix + ((int64_t)k0 * a.hkv + c.kvh) * D;
    vp = (const __bf16*)a.v_prefix + ((int64_t)k0 * a.hkv + c.kvh) * D;
    ks = vs = (uint32_t)a.hkv * D * 2;
    rows = min(Q_BN, c.P - k0);
    ke = a.kend + k0;
  } else {
    const int k0 = (u - c.npt) * Q_BN;
    kp = (const __bf16*)a.k_own + (int64_t)k0 * a.k_stride + (int64_t)c.kvh * D;
    vp = (const __bf16*)a.v_own + (int64_t)k0 * a.v_stride + (int64_t)c.kvh * D;
    ks = (uint32_t)a.k_stride * 2;
    vs = (uint32_t)a.v_stride * 2;
    rows = min(Q_BN, c.N - k0);
    ke = a.kend + c.P + k0;
  }
  dma_tile64(kp, ks, rows, sm.k[buf], w, lane);
  dma_tile64(vp, vs, rows, sm.v[buf], w, lane);
  if (w == 0) dma4(uniform_ptr(ke), (uint32_t)min(lane, rows - 1) * 4u, lds_addr_uniform(sm.kend[buf]));
}

constexpr int Q_STAGE_B = Q_TILE_ELEMS * 2;     // bytes of one staged tile
constexpr int Q_V_OFF = 2 * Q_STAGE_B;          // k[b] -> v[b]
constexpr int Q_RING = 3;                       // operand fragments requested ahead of their MFMA

// One key tile of the dQ pass.  FULL: no per-element visibility test.  ra / ta are this lane's
// fragment addresses in the K tile of the current stage, ka the address of kend[stage][4 hf].
// Each 32-key block is a sequence of slots -- one MFMA, the LDS read for the MFMA Q_RING slots
// ahead, a share of the arithmetic -- closed by scheduling fences.
template <bool FULL>
__device__ __forceinline__ void dq_tile(const uint32_t (&ra)[8], const uint32_t (&ta)[8], uint32_t ka,
                                        const bf16x8 (&qf)[8], const bf16x8 (&gf)[8],
                                        f32x16 (&dq_acc)[4], const f32x16& neg_lse2, const f32x16& neg_delta,
                                        int j0, int j_last, int gi, int hf, int cls) {
  const int gi_c = min(gi, j_last);       // causal bound that also hides the rows past the last key
  bf16x8 fk[Q_RING], fv[Q_RING], fc[Q_RING];
  // transposed K fragments of the dQ phase: slot n: k-step t = n / 4 (16 keys), column block db = n % 4
  auto read_c = [&](int kb, int n) {
    const int db = n & 3, t = n >> 2;
    return lds_tr2(ta[2 * db], ta[2 * db + 1], (kb * 32 + 16 * t) * TILE_ROW * 2);
  };
#pragma unroll
  for (int i = 0; i < Q_RING; i++) fk[i] = lds_b128(ra[i], 0);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int kb = 0; kb < 2; kb++) {
    const int ko = kb * 32 * TILE_ROW * 2;
    f32x16 s_acc, p_acc;
    // The accumulators start from -LSE and -delta of the lane's query (and Q carries the softmax
    // scale), so the MFMA chains deliver the exponent and dP - delta directly.
#pragma unroll
    for (int ss = 0; ss < 8; ss++) {
      s_acc = mfma32(fk[ss % Q_RING], qf[ss], ss == 0 ? neg_lse2 : s_acc);
      const int nx = ss + Q_RING;
      if (nx < 8) fk[nx % Q_RING] = lds_b128(ra[nx], ko);
      else fv[nx - 8] = lds_b128(ra[nx - 8], Q_V_OFF + ko);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int ss = 0; ss < 8; ss++) {
      p_acc = mfma32(fv[ss % Q_RING], gf[ss], ss == 0 ? neg_delta : p_acc);
      const int nx = ss + Q_RING;
      if (nx < 8) fv[nx % Q_RING] = lds_b128(ra[nx], Q_V_OFF + ko);
      else fc[nx - 8] = read_c(kb, nx - 8);
      // P^T (rows = keys: (r/4)*8 + 4*hf + r%4 inside the 32-key block), two registers per slot
      s_acc[2 * ss] = fast_exp2(s_acc[2 * ss]);
      s_acc[2 * ss + 1] = fast_exp2(s_acc[2 * ss + 1]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (!FULL) {
      // cls (wave-uniform) says which of the two tests the tile needs; most boundary tiles need one
      asm volatile("" ::: "memory");
      if (cls == KT_NEED_KEND) {
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
          const i32x4 ke = *(TT_LDS(const i32x4)*)(ka + kb * 128 + r4 * 32);
#pragma unroll
          for (int e = 0; e < 4; e++) s_acc[r4 * 4 + e] = gi < ke[e] ? s_acc[r4 * 4 + e] : 0.f;
        }
      } else if (cls == KT_NEED_CAUSAL) {
        const int rel = gi_c - j0;        // keys 0 .. rel of the tile are visible
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++)
#pragma unroll
          for (int e = 0; e < 4; e++)
            s_acc[r4 * 4 + e] = kb * 32 + r4 * 8 + 4 * hf + e <= rel ? s_acc[r4 * 4 + e] : 0.f;
      } else {
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
          const int jl = kb * 32 + r4 * 8 + 4 * hf;
          const i32x4 ke = *(TT_LDS(const i32x4)*)(ka + kb * 128 + r4 * 32);
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const int j = j0 + jl + e;
            s_acc[r4 * 4 + e] = (j <= gi_c && gi < ke[e]) ? s_acc[r4 * 4 + e] : 0.f;
          }
        }
      }
    }
    // dS^T = P^T (dP^T - delta), then dQ^T[d, q] += K^T[d, key] dS^T[key, q]
    bf16x8 df[2];
#pragma unroll
    for (int r = 0; r < 8; r++) p_acc[r] = s_acc[r] * p_acc[r];
    df[0] = cvt8(p_acc[0], p_acc[1], p_acc[2], p_acc[3], p_acc[4], p_acc[5], p_acc[6], p_acc[7]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int n = 0; n < 8; n++) {
      dq_acc[n & 3] = mfma32(fc[n % Q_RING], df[n >> 2], dq_acc[n & 3]);
      const int nx = n + Q_RING;
      if (nx < 8) fc[nx % Q_RING] = read_c(kb, nx);
      else if (kb == 0) fk[nx - 8] = lds_b128(ra[nx - 8], 32 * TILE_ROW * 2);     // first K fragments of block 1
      if (n < 2) {
#pragma unroll
        for (int r = 8 + 4 * n; r < 12 + 4 * n; r++) p_acc[r] = s_acc[r] * p_acc[r];
      }
      if (n == 2) df[1] = cvt8(p_acc[8], p_acc[9], p_acc[10], p_acc[11], p_acc[12], p_acc[13], p_acc[14], p_acc[15]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

__global__ void __launch_bounds__(NTHREADS, 2)
tree_attn_dq_kernel(AttnArgs a, int n_qtiles) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  QSmem& sm = *reinterpret_cast<QSmem*>(smem_raw);
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c32 = lane & 31, hf = lane >> 5;
  const int G = a.hq / a.hkv;
  const int bid = blockIdx.x;
  const int kvh = bid % a.hkv;
  const int rest = bid / a.hkv;
  const int h = kvh * G + rest % G;
  const int qt = n_qtiles - 1 - rest / G;
  const int q0 = qt * Q_BM;
  const int P = a.n_prefix, N = a.n_q;
  const int q_hi = min(q0 + Q_BM, N);
  const int gi_first = P + q0, gi_last = P + q_hi - 1;
  const int npt = (P + Q_BN - 1) / Q_BN;
  const int u_end = npt + (q_hi - 1) / Q_BN + 1;
  const QCtx ctx{a, kvh, P, N, npt};

  const int q = q0 + 32 * w + c32;
  const int my_q = min(q, N - 1);
  const int gi = P + q;
  bf16x8 qf[8], gf[8];
  {
    const __bf16* qp = (const __bf16*)a.q + (int64_t)my_q * a.q_stride + (int64_t)h * D + 8 * hf;
    const __bf16* gp = (const __bf16*)a.d_o + ((int64_t)my_q * a.hq + h) * D + 8 * hf;
#pragma unroll
    for (int s = 0; s < 8; s++) { qf[s] = *(const bf16x8*)(qp + 16 * s); gf[s] = *(const bf16x8*)(gp + 16 * s); }
  }
  // Per-row terms, stored negated so that the MFMA accumulators can start from them:
  //   -D_i = -sum_d dO[i][h][d] O[i][h][d]   and   -LSE_i log2 e.
  // This lane holds half of its query's dO row (the d values of its operand fragments), so D_i is the sum of
  // the two half-lanes' dot products with the matching half of O.  The terms are also written out for the
  // dK/dV pass, which runs after this kernel.
  float ndelta, nlse2;
  {
    const __bf16* op = (const __bf16*)a.o + ((int64_t)my_q * a.hq + h) * D + 8 * hf;
    bf16x8 of[8];
#pragma unroll
    for (int s = 0; s < 8; s++) of[s] = *(const bf16x8*)(op + 16 * s);
    nlse2 = -a.lse[(int64_t)h * N + my_q] * LOG2E_F;
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < 8; s++)
#pragma unroll
      for (int e = 0; e < 8; e++) acc = fmaf((float)gf[s][e], (float)of[s][e], acc);
    ndelta = -half_swap_sum(acc);
    if (q < N && hf == 0) {
      a.delta[(int64_t)h * N + q] = ndelta;
      a.neg_lse2[(int64_t)h * N + q] = nlse2;
    }
  }

  f32x16 dq_acc[4];
#pragma unroll
  for (int db = 0; db < 4; db++) dq_acc[db] = zero16();

  auto tile_j0 = [&](int u) { return u < npt ? u * Q_BN : P + (u - npt) * Q_BN; };
  auto tile_j_last = [&](int u) {
    return u < npt ? min(u * Q_BN + Q_BN, P) - 1 : P + min((u - npt) * Q_BN + Q_BN, N) - 1;
  };

  // LDS byte addresses of this lane's fragments in stage `buf` of the K tile; V, the 32-key block and
  // the k-step rows are immediate offsets, and the addresses move by +-one stage when the stage flips
  uint32_t ra[8], ta[8];
  const uint32_t sm_base = (uint32_t)(uintptr_t)&sm;
  frag_addresses(sm_base, lane, ra, ta);
  uint32_t ka = sm_base + (uint32_t)offsetof(QSmem, kend) + 16u * hf;
  int stage_step = Q_STAGE_B, kend_step = Q_BN * 4;
  int buf = 0;

#define TT_DQ_STEP(FULLFLAG)                                                                            \
  {                                                                                                     \
    int cls_next = KT_FULL;                                                                             \
    const int u_next = it.next(cls_next);                                                               \
    if (u_next >= 0) q_issue_tile(ctx, sm, buf ^ 1, u_next, w, lane);                                   \
    dq_tile<FULLFLAG>(ra, ta, ka, qf, gf, dq_acc, neg_lse2, neg_delta, tile_j0(u_cur), tile_j_last(u_cur), gi, hf, cls_cur); \
    dma_wait_all();                                                                                     \
    __syncthreads();                                                                                    \
    _Pragma("unroll") for (int i = 0; i < 8; i++) { ra[i] += stage_step; ta[i] += stage_step; }          \
    ka += kend_step;                                                                                    \
    stage_step = -stage_step;                                                                           \
    kend_step = -kend_step;                                                                             \
    buf ^= 1;                                                                                           \
    u_cur = u_next;                                                                                     \
    cls_cur = cls_next;                                                                                 \
  }
  // candidate tiles are classified in chunks of 64 * KT_MAX_WIN (one chunk unless the sequence is
  // longer than 262144 keys)
  KTileIter it;
  // as in the forward kernel: tile 0 is nearly always the first tile delivered, so its copy is started before
  // the classification and runs beside it (a wrong guess costs one wasted tile copy)
  q_issue_tile(ctx, sm, buf, 0, w, lane);
  it.fill(&sm.masks, a.kt_max, a.kt_min, 0, u_end, gi_first, gi_last, npt, P, N, w, NTHREADS / 64);
  int cls_cur = KT_FULL;
  int u_cur = it.next(cls_cur);
  if (u_cur > 0) {
    dma_wait_all();
    q_issue_tile(ctx, sm, buf, u_cur, w, lane);
  }
  // Q is multiplied by scale * log2(e) once (rounded to bf16 again), so that S comes out of the MFMAs
  // as the base-2 exponent
  {
    const float c_scale = a.scale * LOG2E_F;
#pragma unroll
    for (int s = 0; s < 8; s++) qf[s] = scale_frag(qf[s], c_scale);
  }
  f32x16 neg_lse2, neg_delta;
#pragma unroll
  for (int r = 0; r < 16; r++) { neg_lse2[r] = nlse2; neg_delta[r] = ndelta; }
#pragma unroll
  for (int s = 0; s < 8; s++) { pin(qf[s]); pin(gf[s]); }
  pin(neg_lse2);
  pin(neg_delta);
  for (int tile0 = 0;;) {
    dma_wait_all();
    __syncthreads();
    while (u_cur >= 0 && cls_cur == KT_FULL) TT_DQ_STEP(true)
    while (u_cur >= 0) TT_DQ_STEP(false)
    tile0 += 64 * KT_MAX_WIN;
    if (tile0 >= u_end) break;
    it.fill(&sm.masks, a.kt_max, a.kt_min, tile0, u_end, gi_first, gi_last, npt, P, N, w, NTHREADS / 64);
    u_cur = it.next(cls_cur);
    if (u_cur >= 0) q_issue_tile(ctx, sm, buf, u_cur, w, lane);
  }
#undef TT_DQ_STEP

  if (q < N) {
    __bf16* dqp = (__bf16*)a.dq + ((int64_t)q * a.hq + h) * D;
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int r4 = 0; r4 < 4; r4++) {
        const int d0 = db * 32 + r4 * 8 + 4 * hf;
        *(bf16x4*)(dqp + d0) = cvt4(a.scale * dq_acc[db][r4 * 4 + 0], a.scale * dq_acc[db][r4 * 4 + 1],
                                    a.scale * dq_acc[db][r4 * 4 + 2], a.scale * dq_acc[db][r4 * 4 + 3]);
      }
  }
}

}  // namespace

static size_t row_stat_bytes(int n_q, int hq) { return ((size_t)hq * (size_t)n_q * sizeof(float) + 255) & ~(size_t)255; }

size_t mfma_attn_workspace(int n_q, int n_prefix, int hq, int hkv, int d, bool backward) {
  if (!backward) return 0;
  return row_stat_bytes(n_q, hq) + mfma_attn_dkdv_workspace(n_q, n_prefix, hkv);
}

hipError_t mfma_attn_bwd(const AttnArgs& args, hipStream_t st) {
  if (args.n_q == 0) return hipSuccess;
  // the front of the workspace holds -lse * log2(e) (a.delta, before it, holds -D); the rest goes to the dK/dV pass
  AttnArgs a = args;
  const size_t stat = row_stat_bytes(a.n_q, a.hq);
  if (a.workspace_bytes < stat) return hipErrorInvalidValue;
  a.neg_lse2 = (float*)a.workspace;
  a.workspace = (char*)a.workspace + stat;
  a.workspace_bytes -= stat;
  // dQ first: its prologue writes the per-row terms the dK/dV pass streams
  {
    const int n_qtiles = (a.n_q + Q_BM - 1) / Q_BM;
    if (hipError_t e = hipFuncSetAttribute((const void*)tree_attn_dq_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(QSmem)))
      return e;
    KernelTimer timer(TT_KERNEL_ATTN_DQ, st);
    tree_attn_dq_kernel<<<(unsigned)((int64_t)n_qtiles * a.hq), NTHREADS, sizeof(QSmem), st>>>(a, n_qtiles);
    if (hipError_t e = hipGetLastError()) return e;
  }
  return mfma_attn_dkdv(a, st);
}

}  // namespace tt
