// Tree attention forward on bf16 MFMA (gfx950), head dim 128.
//
// Mask (paper, Section "Attention Mask"; Appendix "Tree Attention Mask via FlashMask"): key j is
// visible to query i  <=>  j <= i + P < kend[j].  Per 64-key tile the host supplies min/max of
// kend, which is all that is needed to skip a tile (nothing visible), run it unmasked (everything
// visible) or apply the per-element test (boundary tile).
//
// One workgroup = 128 queries x one query head, 4 wavefronts x 32 queries.  Scores are produced
// transposed, S^T[key, query] = K Q^T, so that a lane owns one query: the softmax statistics are
// per-lane scalars (plus one exchange with the lane holding the other half of the column), and
// P^T is already in B-operand layout for O^T[d, query] += V^T[d, key] P^T[key, query].  K and V
// tiles are staged through LDS (double buffered); V^T fragments come from transposed LDS reads.
#include <hip/hip_runtime.h>
#include "tt_kernels.h"
#include "tt_mfma.h"

namespace tt {
namespace {

constexpr int D = 128;
constexpr int BM = 128;            // queries per workgroup
constexpr int BN = 64;             // keys per tile (= TT_KTILE)
constexpr int NTHREADS = 256;
constexpr int KP = D + 8;          // K row pitch in LDS (elements): 272 B -> conflict-free b128 reads
constexpr int VP = D + 32;         // V row pitch: 320 B -> conflict-free transposed b64 reads
constexpr int K_TILE_ELEMS = BN * KP;
constexpr int V_TILE_ELEMS = BN * VP;

struct Smem {
  __bf16 k[2][K_TILE_ELEMS];
  __bf16 v[2][V_TILE_ELEMS];
  int32_t kend[2][BN];
};

// Registers holding one K/V tile in flight from global memory to LDS.
struct Staging {
  i32x4 k[4], v[4];
  int32_t kend;
};

struct TileSrc {
  const __bf16* k;     // first row of the tile, already offset to the kv head
  const __bf16* v;
  int64_t k_stride, v_stride;
  int rows;            // valid rows in the tile (1..64)
  const int32_t* kend; // kend of the tile's first key
};

__device__ __forceinline__ void load_tile(const TileSrc& s, Staging& st) {
  const int t = threadIdx.x;
#pragma unroll
  for (int u = 0; u < 4; u++) {
    const int c = t + NTHREADS * u;
    const int row = c >> 4, col = (c & 15) * 8;
    i32x4 zk = {0, 0, 0, 0}, zv = {0, 0, 0, 0};
    if (row < s.rows) {
      zk = *(const i32x4*)(s.k + (int64_t)row * s.k_stride + col);
      zv = *(const i32x4*)(s.v + (int64_t)row * s.v_stride + col);
    }
    st.k[u] = zk;
    st.v[u] = zv;
  }
  // keys past the end of the region get bound 0: visible to nobody
  st.kend = (t < BN) ? (t < s.rows ? s.kend[t] : 0) : 0;
}

__device__ __forceinline__ void store_tile(Smem& sm, int buf, const Staging& st) {
  const int t = threadIdx.x;
#pragma unroll
  for (int u = 0; u < 4; u++) {
    const int c = t + NTHREADS * u;
    const int row = c >> 4, col = (c & 15) * 8;
    *(i32x4*)(&sm.k[buf][row * KP + col]) = st.k[u];
    *(i32x4*)(&sm.v[buf][row * VP + col]) = st.v[u];
  }
  if (t < BN) sm.kend[buf][t] = st.kend;
}

__global__ void __launch_bounds__(NTHREADS, 2)
tree_attn_fwd_kernel(AttnArgs a, int n_qtiles) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c32 = lane & 31, hf = lane >> 5;
  const int G = a.hq / a.hkv;
  // consecutive workgroups take different kv heads (they land on different XCDs, so each XCD's L2
  // keeps serving the same K/V head); heavy (late) query tiles are issued first
  const int bid = blockIdx.x;
  const int kvh = bid % a.hkv;
  const int rest = bid / a.hkv;
  const int h = kvh * G + rest % G;
  const int qt = n_qtiles - 1 - rest / G;
  const int q0 = qt * BM;
  const int P = a.n_prefix, N = a.n_q;
  const int q_hi = min(q0 + BM, N);                  // one past the last valid query
  const int gi_first = P + q0, gi_last = P + q_hi - 1;
  const int npt = (P + BN - 1) / BN;                 // prefix tiles
  const int u_end = npt + (q_hi - 1) / BN + 1;       // own tiles up to the diagonal

  // ---- Q fragments (B operand: column = query, k = d) straight from global memory ----
  const int my_q = min(q0 + 32 * w + c32, N - 1);
  const int gi = P + q0 + 32 * w + c32;              // unified index of this lane's query
  bf16x8 qf[8];
  {
    const __bf16* qp = (const __bf16*)a.q + (int64_t)my_q * a.q_stride + (int64_t)h * D + 8 * hf;
#pragma unroll
    for (int s = 0; s < 8; s++) qf[s] = *(const bf16x8*)(qp + 16 * s);
  }

  f32x16 o_acc[4];
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int r = 0; r < 16; r++) o_acc[db][r] = 0.f;
  float m_run = -INFINITY;      // running max of scale*log2(e)*s  (shared by the two half-lanes)
  float l_run = 0.f;            // this lane's part of the running sum (own keys only)
  const float c_scale = a.scale * LOG2E_F;

  KTileIter it;
  it.init(a.kt_max, a.kt_min, u_end, gi_first);

  auto tile_src = [&](int u) {
    TileSrc s;
    if (u < npt) {
      const int k0 = u * BN;
      s.k = (const __bf16*)a.k_prefix + ((int64_t)k0 * a.hkv + kvh) * D;
      s.v = (const __bf16*)a.v_prefix + ((int64_t)k0 * a.hkv + kvh) * D;
      s.k_stride = s.v_stride = (int64_t)a.hkv * D;
      s.rows = min(BN, P - k0);
      s.kend = a.kend + k0;
    } else {
      const int k0 = (u - npt) * BN;
      s.k = (const __bf16*)a.k_own + (int64_t)k0 * a.k_stride + (int64_t)kvh * D;
      s.v = (const __bf16*)a.v_own + (int64_t)k0 * a.v_stride + (int64_t)kvh * D;
      s.k_stride = a.k_stride; s.v_stride = a.v_stride;
      s.rows = min(BN, N - k0);
      s.kend = a.kend + P + k0;
    }
    return s;
  };
  // unified index of the first key of tile u
  auto tile_j0 = [&](int u) { return u < npt ? u * BN : P + (u - npt) * BN; };

#pragma unroll
  for (int s = 0; s < 8; s++) pin(qf[s]);

  Staging st;
  int u_cur = it.next();
  int kmin_cur = it.kmin;
  if (u_cur >= 0) {
    load_tile(tile_src(u_cur), st);
    store_tile(sm, 0, st);
  }
  __syncthreads();
  int buf = 0;

  // per-lane LDS offsets
  const int k_rd = c32 * KP + 8 * hf;                                   // + kb*32*KP + 16*s
  const int i16 = lane & 15, gidx = (lane >> 4) & 1;
  const int v_rd = (4 * hf + (i16 >> 2)) * VP + 16 * gidx + 4 * (i16 & 3);  // + (16*ks + 8*x)*VP + 32*db

  while (u_cur >= 0) {
    const int u_next = it.next();
    const int kmin_next = it.kmin;
    if (u_next >= 0) load_tile(tile_src(u_next), st);

    const int j0 = tile_j0(u_cur);
    const int rows = u_cur < npt ? min(BN, P - u_cur * BN) : min(BN, N - (u_cur - npt) * BN);
    // everything visible: all keys exist, all are at or before the first query, and every bound
    // lies beyond the last query
    const bool full = rows == BN && j0 + BN - 1 <= gi_first && kmin_cur > gi_last;

    // ---- S^T = K Q^T ----
    f32x16 s_acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
#pragma unroll
      for (int s = 0; s < 8; s++) {
        const bf16x8 kf = *(const bf16x8*)(&sm.k[buf][k_rd + kb * 32 * KP + 16 * s]);
        s_acc[kb] = mfma32(kf, qf[s], s == 0 ? zero16() : s_acc[kb]);
      }
    }

    // ---- mask (boundary tiles only) ----
    if (!full) {
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
          const int jl = kb * 32 + r4 * 8 + 4 * hf;
          const i32x4 ke = *(const i32x4*)(&sm.kend[buf][jl]);
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const int j = j0 + jl + e;
            const bool vis = j <= gi && gi < ke[e];
            s_acc[kb][r4 * 4 + e] = vis ? s_acc[kb][r4 * 4 + e] : -INFINITY;
          }
        }
      }
    }

    // ---- online softmax (base 2) ----
    float tmax = s_acc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) tmax = fmaxf(tmax, s_acc[kb][r]);
    tmax = half_swap_max(tmax) * c_scale;               // c_scale > 0
    const float m_new = fmaxf(m_run, tmax);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;   // nothing visible yet: keep everything at 0
    const float alpha = fast_exp2(m_run - m_use);
    m_run = m_new;
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const float p = fast_exp2(fmaf(s_acc[kb][r], c_scale, -m_use));
        s_acc[kb][r] = p;
        psum += p;
      }
    l_run = l_run * alpha + psum;
    // the running max rarely moves after the first tiles: rescale only when some lane needs it
    if (__ballot(alpha != 1.f) != 0) {
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) o_acc[db][r] *= alpha;
    }

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {
      const int kb = ks >> 1, t8 = (ks & 1) * 8;
      const bf16x8 pf = cvt8(s_acc[kb][t8 + 0], s_acc[kb][t8 + 1], s_acc[kb][t8 + 2], s_acc[kb][t8 + 3],
                             s_acc[kb][t8 + 4], s_acc[kb][t8 + 5], s_acc[kb][t8 + 6], s_acc[kb][t8 + 7]);
#pragma unroll
      for (int db = 0; db < 4; db++) {
        const __bf16* vp = &sm.v[buf][v_rd + 16 * ks * VP + 32 * db];
        const bf16x8 vf = cat4(lds_read_tr(vp), lds_read_tr(vp + 8 * VP));
        o_acc[db] = mfma32(vf, pf, o_acc[db]);
      }
    }

    if (u_next >= 0) store_tile(sm, buf ^ 1, st);
    __syncthreads();
    buf ^= 1;
    u_cur = u_next;
    kmin_cur = kmin_next;
  }

  // ---- epilogue ----
  const float l_tot = half_swap_sum(l_run);
  const float inv_l = 1.f / l_tot;
  const int q = q0 + 32 * w + c32;
  if (q < N) {
    __bf16* op = (__bf16*)a.o + ((int64_t)q * a.hq + h) * D;
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int r4 = 0; r4 < 4; r4++) {
        const bf16x4 ov = cvt4(o_acc[db][r4 * 4 + 0] * inv_l, o_acc[db][r4 * 4 + 1] * inv_l,
                               o_acc[db][r4 * 4 + 2] * inv_l, o_acc[db][r4 * 4 + 3] * inv_l);
        *(bf16x4*)(op + db * 32 + r4 * 8 + 4 * hf) = ov;
      }
    if (hf == 0) a.lse[(int64_t)h * N + q] = (m_run + log2f(l_tot)) * LN2_F;
  }
}

}  // namespace

hipError_t mfma_attn_fwd(const AttnArgs& a, hipStream_t st) {
  if (a.n_q == 0) return hipSuccess;
  const int n_qtiles = (a.n_q + BM - 1) / BM;
  const int64_t blocks = (int64_t)n_qtiles * a.hq;
  if (hipError_t e = hipFuncSetAttribute((const void*)tree_attn_fwd_kernel,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Smem)))
    return e;
  KernelTimer timer(TT_KERNEL_ATTN_FWD, st);
  tree_attn_fwd_kernel<<<(unsigned)blocks, NTHREADS, sizeof(Smem), st>>>(a, n_qtiles);
  return hipGetLastError();
}

}  // namespace tt
