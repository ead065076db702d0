// Tree attention forward on bf16 MFMA (gfx950), head dim 128.
//
// Mask (paper, Section "Attention Mask"; Appendix "Tree Attention Mask via FlashMask"): key j is
// visible to query i  <=>  j <= i + P < kend[j].  Per 64-key tile the host supplies min/max of
// kend, which is all that is needed to skip a tile (nothing visible), run it unmasked (everything
// visible) or apply the per-element test (boundary tile).
//
// One workgroup = 128 queries x one query head, 4 wavefronts x 32 queries, two workgroups per
// compute unit.  Scores are produced transposed, S^T[key, query] = K Q^T, so that a lane owns one
// query: the softmax statistics are per-lane scalars (plus one exchange with the lane holding the
// other half of the column), and P^T is already in B-operand layout for
// O^T[d, query] += V^T[d, key] P^T[key, query].  K and V tiles go from global memory straight into
// swizzled LDS tiles (asynchronous, double buffered); V^T fragments come from transposed LDS reads.
#include <hip/hip_runtime.h>
#include "tt_kernels.h"
#include "tt_mfma.h"

namespace tt {
namespace {

constexpr int D = 128;
constexpr int BM = 128;            // queries per workgroup
constexpr int BN = 64;             // keys per tile (= TT_KTILE)
constexpr int NTHREADS = 256;
constexpr int TILE_ELEMS = BN * TILE_ROW;
constexpr float RESCALE_SLACK = 8.f;   // log2 units

struct Smem {
  __bf16 k[2][TILE_ELEMS];
  __bf16 v[2][TILE_ELEMS];
  int32_t kend[2][BN];
  KTileMasks masks;
};

struct Ctx {
  const AttnArgs& a;
  int kvh, P, N, npt;
};

// Starts the copy of key tile u (K, V rows and visibility bounds) into stage `buf`.  Everything goes
// through the asynchronous global -> LDS path: an ordinary load into a register would make the
// compiler wait for all outstanding memory operations -- the tile copies included -- at its first use.
// Rows past the end of the region repeat the last valid row; process_tile keeps them invisible.
__device__ __forceinline__ void issue_tile(const Ctx& c, Smem& sm, int buf, int u, int w, int lane) {
  const AttnArgs& a = c.a;
  const __bf16 *kp, *vp;
  const int32_t* ke;
  uint32_t ks, vs;
  int rows;
  if (u < c.npt) {
    const int k0 = u * BN;
    kp = (const __bf16*)a.k_prefix + ((int64_t)k0 * a.hkv + c.kvh) * D;
    vp = (const __bf16*)a.v_prefix + ((int64_t)k0 * a.hkv + c.kvh) * D;
    ks = vs = (uint32_t)a.hkv * D * 2;
    rows = min(BN, c.P - k0);
    ke = a.kend + k0;
  } else {
    const int k0 = (u - c.npt) * BN;
    kp = (const __bf16*)a.k_own + (int64_t)k0 * a.k_stride + (int64_t)c.kvh * D;
    vp = (const __bf16*)a.v_own + (int64_t)k0 * a.v_stride + (int64_t)c.kvh * D;
    ks = (uint32_t)a.k_stride * 2;
    vs = (uint32_t)a.v_stride * 2;
    rows = min(BN, c.N - k0);
    ke = a.kend + c.P + k0;
  }
  dma_tile64(kp, ks, rows, sm.k[buf], w, lane);
  dma_tile64(vp, vs, rows, sm.v[buf], w, lane);
  if (w == 0) dma4(uniform_ptr(ke), (uint32_t)min(lane, rows - 1) * 4u, lds_addr_uniform(sm.kend[buf]));
}

constexpr int STAGE_B = TILE_ELEMS * 2;       // bytes of one staged tile
constexpr int V_OFF = 2 * STAGE_B;            // k[b] -> v[b]
constexpr int RING = 3;                       // operand fragments requested ahead of their MFMA

// One key tile: S^T = K Q^T, online softmax, O^T += V^T P^T.  FULL = every (query, key) pair of the
// tile is visible: no per-element test.  ra / ta are this lane's fragment addresses in the K tile of
// the current stage, ka the address of kend[stage][4 hf].  The tile is a sequence of slots -- one
// MFMA, the LDS read for the MFMA RING slots ahead, a share of the softmax arithmetic -- closed by
// scheduling fences; the exponentials of key step ks + 1 are computed under the MFMAs of step ks.
template <bool FULL>
__device__ __forceinline__ void process_tile(const uint32_t (&ra)[8], const uint32_t (&ta)[8], uint32_t ka,
                                             const bf16x8 (&qf)[8], f32x16 (&o_acc)[4],
                                             float& m_run, float& l_run, f32x16& neg_m, int j0, int j_last, int gi,
                                             int hf, int cls) {
  f32x16 s_acc[2];
  bf16x8 fk[RING], fvt[RING];
  // K fragment of slot i: key block i % 2, k-step i / 2; V^T fragment of slot n: key step n / 4
  // (16 keys), column block n % 4
  auto read_k = [&](int i) { return lds_b128(ra[i >> 1], (i & 1) * 32 * TILE_ROW * 2); };
  auto read_vt = [&](int n) {
    const int db = n & 3, ks = n >> 2;
    return lds_tr2(ta[2 * db], ta[2 * db + 1], V_OFF + 16 * ks * TILE_ROW * 2);
  };
#pragma unroll
  for (int i = 0; i < RING; i++) fk[i] = read_k(i);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < 16; i++) {
    const int kb = i & 1, ss = i >> 1;
    s_acc[kb] = mfma32(fk[i % RING], qf[ss], ss == 0 ? neg_m : s_acc[kb]);
    const int nx = i + RING;
    if (nx < 16) fk[nx % RING] = read_k(nx);
    else fvt[nx - 16] = read_vt(nx - 16);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (!FULL) {
    // cls (wave-uniform) says which of the two tests the tile needs; most boundary tiles need one
    asm volatile("" ::: "memory");
    const int gi_c = min(gi, j_last);     // causal bound that also hides the rows past the last key
    if (cls == KT_NEED_KEND) {
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
          const i32x4 ke = *(TT_LDS(const i32x4)*)(ka + kb * 128 + r4 * 32);
#pragma unroll
          for (int e = 0; e < 4; e++) s_acc[kb][r4 * 4 + e] = gi < ke[e] ? s_acc[kb][r4 * 4 + e] : -INFINITY;
        }
    } else if (cls == KT_NEED_CAUSAL) {
      const int rel = gi_c - j0;          // keys 0 .. rel of the tile are visible
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++)
#pragma unroll
          for (int e = 0; e < 4; e++)
            s_acc[kb][r4 * 4 + e] = kb * 32 + r4 * 8 + 4 * hf + e <= rel ? s_acc[kb][r4 * 4 + e] : -INFINITY;
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
          const int jl = kb * 32 + r4 * 8 + 4 * hf;
          const i32x4 ke = *(TT_LDS(const i32x4)*)(ka + kb * 128 + r4 * 32);
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const int j = j0 + jl + e;
            const bool vis = j <= gi_c && gi < ke[e];
            s_acc[kb][r4 * 4 + e] = vis ? s_acc[kb][r4 * 4 + e] : -INFINITY;
          }
        }
    }
  }

  // ---- online softmax (base 2) ----
  // Q carries scale * log2(e) and the accumulators started from -m_ref (neg_m), so s_acc already is
  // the exponent relative to the reference m_ref = m_run (0 while nothing has been seen).  The
  // reference follows the running maximum lazily: probabilities may exceed 1 by up to
  // 2^RESCALE_SLACK (harmless in bf16 / fp32), and only when some lane's maximum has grown past that
  // slack -- or the lane sees its first key -- are reference, scores and output accumulators moved;
  // after the first few tiles that almost never happens.
  float tmax = s_acc[0][0];
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int r = 0; r < 16; r++) tmax = fmaxf(tmax, s_acc[kb][r]);
  tmax = half_swap_max(tmax);
  {
    const bool unset = m_run == -INFINITY;
    const bool move = tmax > (unset ? -INFINITY : RESCALE_SLACK);
    if (__ballot(move) != 0) {
      const float shift = move ? tmax : 0.f;
      const float alpha = unset ? 1.f : fast_exp2(-shift);      // nothing accumulated yet: nothing to scale
      if (move) m_run = (unset ? 0.f : m_run) + shift;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) o_acc[db][r] *= alpha;
      const float nm = m_run == -INFINITY ? 0.f : -m_run;
#pragma unroll
      for (int r = 0; r < 16; r++) { s_acc[0][r] -= shift; s_acc[1][r] -= shift; neg_m[r] = nm; }
    }
  }

  // ---- P = exp2(s), O^T += V^T P^T ----
  // key step ks covers accumulator registers 8 (ks % 2) .. + 7 of key block ks / 2
  float psum = 0.f;
  bf16x8 pf[2];
  auto exps = [&](int ks, int r0, int cnt) {
#pragma unroll
    for (int r = 8 * (ks & 1) + r0; r < 8 * (ks & 1) + r0 + cnt; r++) {
      const float pv = fast_exp2(s_acc[ks >> 1][r]);
      s_acc[ks >> 1][r] = pv;
      psum += pv;
    }
  };
  auto pack = [&](int ks) {
    const int kb = ks >> 1, t8 = (ks & 1) * 8;
    return cvt8(s_acc[kb][t8 + 0], s_acc[kb][t8 + 1], s_acc[kb][t8 + 2], s_acc[kb][t8 + 3],
                s_acc[kb][t8 + 4], s_acc[kb][t8 + 5], s_acc[kb][t8 + 6], s_acc[kb][t8 + 7]);
  };
  exps(0, 0, 8);
  pf[0] = pack(0);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int n = 0; n < 16; n++) {
    const int ks = n >> 2, db = n & 3;
    o_acc[db] = mfma32(fvt[n % RING], pf[ks & 1], o_acc[db]);
    if (n + RING < 16) fvt[(n + RING) % RING] = read_vt(n + RING);
    if (ks < 3) {
      exps(ks + 1, 2 * db, 2);
      if (db == 3) pf[(ks + 1) & 1] = pack(ks + 1);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  l_run += psum;
}

__global__ void __launch_bounds__(NTHREADS, 2)
tree_attn_fwd_kernel(AttnArgs a, int n_qtiles) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  Smem& sm = *reinterpret_cast<Smem*>(smem_raw);
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
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
  const Ctx ctx{a, kvh, P, N, npt};

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
  for (int db = 0; db < 4; db++) o_acc[db] = zero16();
  float m_run = -INFINITY;      // softmax reference in log2 units (shared by the two half-lanes); -inf: no key seen yet
  float l_run = 0.f;            // this lane's part of the running sum (own keys only)
  f32x16 neg_m = zero16();      // -(reference), the value every score accumulator starts from

  auto tile_j0 = [&](int u) { return u < npt ? u * BN : P + (u - npt) * BN; };
  auto tile_j_last = [&](int u) { return u < npt ? min(u * BN + BN, P) - 1 : P + min((u - npt) * BN + BN, N) - 1; };

  // LDS byte addresses of this lane's fragments in stage `buf` of the K tile; V, the 32-key block and
  // the k-step rows are immediate offsets, and the addresses move by +-one stage when the stage flips
  uint32_t ra[8], ta[8];
  const uint32_t sm_base = (uint32_t)(uintptr_t)&sm;
  frag_addresses(sm_base, lane, ra, ta);
  uint32_t ka = sm_base + (uint32_t)offsetof(Smem, kend) + 16u * hf;
  int stage_step = STAGE_B, kend_step = BN * 4;
  int buf = 0;

  // One pipeline step: start the copy of the next tile, do this tile's math, publish the next tile.
#define TT_FWD_STEP(FULLFLAG)                                                                          \
  {                                                                                                    \
    int cls_next = KT_FULL;                                                                            \
    const int u_next = it.next(cls_next);                                                              \
    if (u_next >= 0) issue_tile(ctx, sm, buf ^ 1, u_next, w, lane);                                    \
    process_tile<FULLFLAG>(ra, ta, ka, qf, o_acc, m_run, l_run, neg_m, tile_j0(u_cur), tile_j_last(u_cur), gi, hf, cls_cur); \
    dma_wait_all();                                                                                    \
    __syncthreads();                                                                                   \
    _Pragma("unroll") for (int i = 0; i < 8; i++) { ra[i] += stage_step; ta[i] += stage_step; }         \
    ka += kend_step;                                                                                   \
    stage_step = -stage_step;                                                                          \
    kend_step = -kend_step;                                                                            \
    buf ^= 1;                                                                                          \
    u_cur = u_next;                                                                                    \
    cls_cur = cls_next;                                                                                \
  }
  // candidate tiles are classified in chunks of 64 * KT_MAX_WIN (one chunk unless the sequence is
  // longer than 262144 keys)
  KTileIter it;
  // The copy of tile 0 is started before the tile summaries have even been requested: a root's first keys are
  // visible to every later query, so tile 0 is nearly always the first tile delivered, and its round trip then runs
  // beside the classification's instead of behind it (and beside the Q fragments').  A wrong guess (several roots,
  // a prefix whose first tile is hidden) costs one wasted tile copy: the right tile is fetched over it.
  issue_tile(ctx, sm, buf, 0, w, lane);
  it.fill(&sm.masks, a.kt_max, a.kt_min, 0, u_end, gi_first, gi_last, npt, P, N, w, NTHREADS / 64);
  int cls_cur = KT_FULL;
  int u_cur = it.next(cls_cur);
  if (u_cur > 0) {
    dma_wait_all();                        // this wave's rows of the guessed tile have landed; they are overwritten
    issue_tile(ctx, sm, buf, u_cur, w, lane);
  }
  {
    // Q is multiplied by scale * log2(e) once (rounded to bf16 again), so that S comes out of the
    // MFMAs as a base-2 exponent
    const float c_scale = a.scale * LOG2E_F;
#pragma unroll
    for (int s = 0; s < 8; s++) qf[s] = scale_frag(qf[s], c_scale);
#pragma unroll
    for (int s = 0; s < 8; s++) pin(qf[s]);
  }
  for (int tile0 = 0;;) {
    dma_wait_all();
    __syncthreads();
    while (u_cur >= 0 && cls_cur == KT_FULL) TT_FWD_STEP(true)
    while (u_cur >= 0) TT_FWD_STEP(false)
    tile0 += 64 * KT_MAX_WIN;
    if (tile0 >= u_end) break;
    it.fill(&sm.masks, a.kt_max, a.kt_min, tile0, u_end, gi_first, gi_last, npt, P, N, w, NTHREADS / 64);
    u_cur = it.next(cls_cur);
    if (u_cur >= 0) issue_tile(ctx, sm, buf, u_cur, w, lane);
  }
#undef TT_FWD_STEP

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
