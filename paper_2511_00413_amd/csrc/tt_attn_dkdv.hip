// Tree attention backward, dK/dV pass, on bf16 MFMA (gfx950), head dim 128.
//
// Column-parallel: one work item = 128 keys x one kv head (4 wavefronts x 32 keys) x a chunk of the
// (query head, query tile) steps that can see those keys.  In DFS order a subtree is contiguous, so
// the queries that see a key tile form the contiguous range [first key, max kend).
// S[q,key] = Q K^T and dP[q,key] = dO V^T come out with one key per lane, already in B-operand
// layout for dV^T[d,key] += dO^T[d,q] P[q,key] and dK^T[d,key] += Q^T[d,q] dS[q,key]; Q / dO tiles
// are copied asynchronously into swizzled LDS tiles, and Q^T / dO^T fragments come from transposed
// LDS reads.  dK/dV sum over every visible query, i.e. over all branches through the key (paper
// Eq. 5), and over the query heads of the kv group; gradients of cached prefix keys are added in
// fp32 to caller-owned accumulators (Appendix "Float32 Gradient Accumulation").
#include <hip/hip_runtime.h>
#include <algorithm>
#include "tt_kernels.h"
#include "tt_mfma.h"

namespace tt {
namespace {

constexpr int D = 128;
constexpr int NTHREADS = 256;

// ------------------------------------------------------------------------------------------------
// dK / dV
// ------------------------------------------------------------------------------------------------
constexpr int KV_BN = 128;         // keys per workgroup (two TT_KTILE summaries)
constexpr int KV_BM = 64;          // queries per staged tile (one pipeline step)
constexpr int KV_NQB = KV_BM / 32;  // 32-query blocks per step

struct KvSmem {
  __bf16 q[2][KV_BM * TILE_ROW];   // swizzled tiles, filled by asynchronous global -> LDS copies
  __bf16 g[2][KV_BM * TILE_ROW];   // dO
  float lse[2][KV_BM];             // natural-log LSE of the tile's queries
  float delta[2][KV_BM];
};

// Starts the copy of one (head, query tile) step into stage `buf`.
__device__ __forceinline__ void kv_issue(const AttnArgs& a, KvSmem& sm, int buf, int h, int q0, int w, int lane) {
  const int rows = min(KV_BM, a.n_q - q0);
  const __bf16* qsrc = (const __bf16*)a.q + (int64_t)q0 * a.q_stride + (int64_t)h * D;
  const __bf16* gsrc = (const __bf16*)a.d_o + ((int64_t)q0 * a.hq + h) * D;
#pragma unroll
  for (int c = 0; c < KV_BM / 64; c++) {
    dma_tile64(qsrc, (uint32_t)a.q_stride * 2, rows, sm.q[buf] + c * 64 * TILE_ROW, w, lane, 64 * c);
    dma_tile64(gsrc, (uint32_t)a.hq * D * 2, rows, sm.g[buf] + c * 64 * TILE_ROW, w, lane, 64 * c);
  }
  // per-query scalars, 64 per wave: LSE then delta, spread over the waves (rows past the end repeat
  // the last one; such rows are masked by the boundary test)
  constexpr int PARTS = KV_BM / 64;                 // 64-float pieces per array
  static_assert(2 * PARTS <= 4, "at most one scalar piece per wave");
  if (w < 2 * PARTS) {
    const bool is_lse = w < PARTS;
    const int part = is_lse ? w : w - PARTS;
    const float* src = (is_lse ? a.lse : a.delta) + (int64_t)h * a.n_q + q0;
    float* dst = (is_lse ? sm.lse[buf] : sm.delta[buf]) + 64 * part;
    dma4(uniform_ptr(src), (uint32_t)min(64 * part + lane, rows - 1) * 4u, lds_addr_uniform(dst));
  }
}

// ---- work decomposition -------------------------------------------------------------------------
// A key tile's work is its list of (query head, query tile) steps.  Tiles near the root of the tree
// are seen by almost every query while leaf tiles are seen by few, so a tile's steps are cut into
// chunks of at most `chunk` steps; a planner kernel sizes the chunks so that the launch has about
// KV_TARGET_WORK work items, workgroups pull items from a counter, and tiles that were cut have
// their fp32 partial results summed in chunk order by a reduce kernel (bit-reproducible).
constexpr int KV_TARGET_WORK = 1024;     // work items (tile chunk x kv head) aimed for
constexpr int KV_MIN_CHUNK = 32;         // steps
constexpr int PLAN_THREADS = 1024;

struct KvPlanHeader {
  int n_work;        // work items = n_items * hkv
  int counter;       // next work item to hand out
  int chunk;         // steps per chunk
  int n_split_items; // items [0, n_split_items) write partial slots (slot index = item index)
};

struct KvPlan {                // device pointers into the workspace
  KvPlanHeader* hdr;
  int *tile_nq, *tile_qtlo, *tile_nchunks, *tile_item0;   // [n_tiles]
  int *item_tile, *item_chunk;                            // [max_items]
  float* slots;                                           // [max_slots][hkv][2][KV_BN][D]
  int n_tiles, n_ptiles, max_items, max_slots;
};

__host__ __device__ inline int kv_target_items(int hkv) { return (KV_TARGET_WORK + hkv - 1) / hkv; }

__host__ inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Carves the plan out of `base`; with base == nullptr only the size is computed.
__host__ inline size_t kv_plan_layout(void* base, int n_q, int n_prefix, int hkv, KvPlan* out) {
  const int n_ptiles = (n_prefix + KV_BN - 1) / KV_BN, n_otiles = (n_q + KV_BN - 1) / KV_BN;
  const int n_tiles = n_ptiles + n_otiles;
  const int max_items = n_tiles + kv_target_items(hkv);
  const int max_slots = 2 * kv_target_items(hkv);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return base ? (char*)base + o : (char*)nullptr; };
  char* hdr = take(sizeof(KvPlanHeader));
  char* t0 = take(sizeof(int) * n_tiles);
  char* t1 = take(sizeof(int) * n_tiles);
  char* t2 = take(sizeof(int) * n_tiles);
  char* t3 = take(sizeof(int) * n_tiles);
  char* i0 = take(sizeof(int) * max_items);
  char* i1 = take(sizeof(int) * max_items);
  char* sl = take(sizeof(float) * (size_t)max_slots * hkv * 2 * KV_BN * D);
  if (out) {
    out->hdr = (KvPlanHeader*)hdr;
    out->tile_nq = (int*)t0; out->tile_qtlo = (int*)t1; out->tile_nchunks = (int*)t2; out->tile_item0 = (int*)t3;
    out->item_tile = (int*)i0; out->item_chunk = (int*)i1; out->slots = (float*)sl;
    out->n_tiles = n_tiles; out->n_ptiles = n_ptiles; out->max_items = max_items; out->max_slots = max_slots;
  }
  return off;
}

// exclusive prefix sum of one int per thread over the workgroup; returns the total through *total
__device__ inline int block_exclusive_scan(int v, int* scratch /*[PLAN_THREADS]*/, int* total) {
  const int t = threadIdx.x;
  scratch[t] = v;
  __syncthreads();
  for (int off = 1; off < PLAN_THREADS; off <<= 1) {
    const int add = t >= off ? scratch[t - off] : 0;
    __syncthreads();
    scratch[t] += add;
    __syncthreads();
  }
  const int incl = scratch[t];
  *total = scratch[PLAN_THREADS - 1];
  __syncthreads();
  return incl - v;
}

__global__ void __launch_bounds__(PLAN_THREADS)
kv_plan_kernel(KvPlan pl, const int32_t* __restrict__ kt_max, int n_q, int n_prefix, int G, int hkv) {
  __shared__ int scratch[PLAN_THREADS];
  const int t = threadIdx.x;
  const int per = (pl.n_tiles + PLAN_THREADS - 1) / PLAN_THREADS;    // consecutive tiles per thread
  const int lo = min(t * per, pl.n_tiles), hi = min(lo + per, pl.n_tiles);
  const int np64 = (n_prefix + 63) / 64, no64 = (n_q + 63) / 64;
  // pass 1: visible query tiles of every key tile
  int my_steps = 0;
  for (int tl = lo; tl < hi; tl++) {
    int kmax, i_lo;
    if (tl < pl.n_ptiles) {
      const int e0 = 2 * tl, e1 = e0 + 1;
      kmax = max(kt_max[e0], e1 < np64 ? kt_max[e1] : 0);
      i_lo = 0;
    } else {
      const int to = tl - pl.n_ptiles;
      const int e0 = np64 + 2 * to, e1 = e0 + 1;
      kmax = max(kt_max[e0], e1 < np64 + no64 ? kt_max[e1] : 0);
      i_lo = to * KV_BN;
    }
    const int i_hi = (int)min((int64_t)n_q, (int64_t)kmax - n_prefix);
    const int qt_lo = i_lo / KV_BM;
    const int nq = i_hi > i_lo ? (i_hi + KV_BM - 1) / KV_BM - qt_lo : 0;
    pl.tile_nq[tl] = nq;
    pl.tile_qtlo[tl] = qt_lo;
    my_steps += nq * G;
  }
  int total_steps;
  block_exclusive_scan(my_steps, scratch, &total_steps);
  const int64_t all = (int64_t)total_steps * hkv;
  const int chunk = (int)max((int64_t)KV_MIN_CHUNK, (all + KV_TARGET_WORK - 1) / KV_TARGET_WORK);
  // pass 2: chunks per tile; cut tiles are numbered first (their item index is also their slot)
  int my_split = 0, my_whole = 0;
  for (int tl = lo; tl < hi; tl++) {
    const int steps = pl.tile_nq[tl] * G;
    const int nc = (steps + chunk - 1) / chunk;
    pl.tile_nchunks[tl] = nc;
    if (nc > 1) my_split += nc; else my_whole += nc;
  }
  int n_split, n_whole;
  int split0 = block_exclusive_scan(my_split, scratch, &n_split);
  int whole0 = block_exclusive_scan(my_whole, scratch, &n_whole) + n_split;
  for (int tl = lo; tl < hi; tl++) {
    const int nc = pl.tile_nchunks[tl];
    int& cursor = nc > 1 ? split0 : whole0;
    pl.tile_item0[tl] = cursor;
    for (int c = 0; c < nc; c++) { pl.item_tile[cursor + c] = tl; pl.item_chunk[cursor + c] = c; }
    cursor += nc;
  }
  if (t == 0) {
    pl.hdr->n_work = (n_split + n_whole) * hkv;
    pl.hdr->counter = 0;
    pl.hdr->chunk = chunk;
    pl.hdr->n_split_items = n_split;
  }
}

// One (head, 64-query tile) step for a wavefront whose 32 keys are visible to all 64 queries: no
// visibility test and no branch.  The step is written as 64 "slots" of one MFMA each; every slot
// also issues the LDS reads for an MFMA a few slots ahead and a slice of the exp / dS arithmetic of
// the other 32-query block, and ends with a scheduling fence so that the emitted order is the
// written order:
//   slots  0..15  S, dP of query block 0
//   slots 16..31  S, dP of block 1      + P, dS arithmetic of block 0 (one element per slot)
//   slots 32..47  dV, dK from block 0   + P, dS arithmetic of block 1
//   slots 48..63  dV, dK from block 1
__device__ __forceinline__ void kv_step_full(const KvSmem& sm, int buf, const bf16x8 (&kf)[8], const bf16x8 (&vf)[8],
                                             f32x16 (&dk_acc)[4], f32x16 (&dv_acc)[4], float c_scale,
                                             int a_rd, TrBase t_rd, int hf, int qb0) {
  constexpr int AHEAD_A = 6;      // operand-row reads in flight (one b128 read per MFMA)
  constexpr int AHEAD_C = 3;      // transposed fragments in flight (two b64 reads per MFMA)
  f32x16 s_acc[2], p_acc[2];
  f32x4 l2[2][4], dl[2][4];
  bf16x8 fa[AHEAD_A], fc[AHEAD_C];
  bf16x8 pf[2], df[2];            // P / dS of the block being consumed, per 16-query k-step

  // operand of score slot i: i>>4 = query block, (i>>3)&1 = 0: Q rows (S), 1: dO rows (dP), i&7 = d-step
  auto read_a = [&](int i) {
    return lds_row_frag(((i >> 3) & 1) ? sm.g[buf] : sm.q[buf], a_rd, qb0 + (i >> 4), i & 7);
  };
  // operand of gradient slot j: j>>4 = query block, (j>>3)&1 = k-step t, (j>>1)&3 = d block,
  // j&1 = 0: dO^T (feeds dV with P), 1: Q^T (feeds dK with dS)
  auto read_c = [&](int j) {
    return lds_tr_frag((j & 1) ? sm.q[buf] : sm.g[buf], t_rd, (qb0 + (j >> 4)) * 32 + 16 * ((j >> 3) & 1), (j >> 1) & 3);
  };
  auto scalars = [&](int b) {
#pragma unroll
    for (int r4 = 0; r4 < 4; r4++) {
      l2[b][r4] = *(const f32x4*)(&sm.lse[buf][(qb0 + b) * 32 + r4 * 8 + 4 * hf]) * LOG2E_F;
      dl[b][r4] = *(const f32x4*)(&sm.delta[buf][(qb0 + b) * 32 + r4 * 8 + 4 * hf]);
    }
  };
  auto element = [&](int b, int e) {       // P and dS of accumulator register e of block b
    const float p = fast_exp2(fmaf(s_acc[b][e], c_scale, -l2[b][e >> 2][e & 3]));
    s_acc[b][e] = p;
    p_acc[b][e] = p * (p_acc[b][e] - dl[b][e >> 2][e & 3]);
  };
  auto convert = [&](int b, int t) {
    pf[t] = cvt8(s_acc[b][8 * t + 0], s_acc[b][8 * t + 1], s_acc[b][8 * t + 2], s_acc[b][8 * t + 3],
                 s_acc[b][8 * t + 4], s_acc[b][8 * t + 5], s_acc[b][8 * t + 6], s_acc[b][8 * t + 7]);
    df[t] = cvt8(p_acc[b][8 * t + 0], p_acc[b][8 * t + 1], p_acc[b][8 * t + 2], p_acc[b][8 * t + 3],
                 p_acc[b][8 * t + 4], p_acc[b][8 * t + 5], p_acc[b][8 * t + 6], p_acc[b][8 * t + 7]);
  };

#pragma unroll
  for (int i = 0; i < AHEAD_A; i++) fa[i] = read_a(i);
  scalars(0);
  __builtin_amdgcn_sched_barrier(0);

  // ---- score slots ----
#pragma unroll
  for (int i = 0; i < 32; i++) {
    const int b = i >> 4, ss = i & 7;
    if ((i >> 3) & 1) p_acc[b] = mfma32(fa[i % AHEAD_A], vf[ss], ss == 0 ? zero16() : p_acc[b]);
    else s_acc[b] = mfma32(fa[i % AHEAD_A], kf[ss], ss == 0 ? zero16() : s_acc[b]);
    if (i + AHEAD_A < 32) fa[i % AHEAD_A] = read_a(i + AHEAD_A);
    if (i == 8) scalars(1);
    if (i >= 32 - AHEAD_C) fc[i - (32 - AHEAD_C)] = read_c(i - (32 - AHEAD_C));   // first gradient fragments
    if (i >= 16) element(0, i - 16);
    __builtin_amdgcn_sched_barrier(0);
  }
  convert(0, 0);
  convert(0, 1);
  __builtin_amdgcn_sched_barrier(0);

  // ---- gradient slots ----
#pragma unroll
  for (int j = 0; j < 32; j++) {
    const int t = (j >> 3) & 1, db = (j >> 1) & 3;
    if (j == 16) { convert(1, 0); convert(1, 1); }
    if (j & 1) dk_acc[db] = mfma32(fc[j % AHEAD_C], df[t], dk_acc[db]);
    else dv_acc[db] = mfma32(fc[j % AHEAD_C], pf[t], dv_acc[db]);
    if (j + AHEAD_C < 32) fc[j % AHEAD_C] = read_c(j + AHEAD_C);
    if (j < 16) element(1, j);
    __builtin_amdgcn_sched_barrier(0);
  }
}

__global__ void __launch_bounds__(NTHREADS, 1)
tree_attn_dkdv_kernel(AttnArgs a, KvPlan pl) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  KvSmem& sm = *reinterpret_cast<KvSmem*>(smem_raw);
  __shared__ int s_work;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c32 = lane & 31, hf = lane >> 5;
  const int G = a.hq / a.hkv;
  const int P = a.n_prefix, N = a.n_q;
  const float c_scale = a.scale * LOG2E_F;
  const int a_rd = row_frag_base(lane);        // operand-row reads
  const TrBase t_rd = tr_frag_base(lane);      // transposed reads
  const int n_work = pl.hdr->n_work;
  const int chunk = pl.hdr->chunk;

  for (;;) {
    if (threadIdx.x == 0) s_work = atomicAdd(&pl.hdr->counter, 1);
    __syncthreads();
    const int work = s_work;
    __syncthreads();                         // everyone has read s_work before it is rewritten
    if (work >= n_work) break;               // the counter only grows: every wave gets here
    const int kvh = work % a.hkv;            // neighbouring items differ in kv head (XCD locality)
    const int item = work / a.hkv;
    const int tile = pl.item_tile[item];
    const int nq = pl.tile_nq[tile], qt_lo = pl.tile_qtlo[tile];
    const int s_lo = pl.item_chunk[item] * chunk;
    const int s_hi = min(s_lo + chunk, nq * G);
    const bool partial = pl.tile_nchunks[tile] > 1;

    const bool is_prefix = tile < pl.n_ptiles;
    const int k0 = is_prefix ? tile * KV_BN : (tile - pl.n_ptiles) * KV_BN;   // region-local first key
    const int region = is_prefix ? P : N;
    const int j0 = is_prefix ? k0 : P + k0;          // unified index of the first key
    // this lane's key
    const int kl = k0 + 32 * w + c32;
    const bool key_ok = kl < region;
    const int j = j0 + 32 * w + c32;
    const int my_kend = key_ok ? a.kend[j] : 0;
    int kmax_w = my_kend, kmin_w = key_ok ? my_kend : INT32_MAX;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      kmax_w = max(kmax_w, __shfl_xor(kmax_w, off));
      kmin_w = min(kmin_w, __shfl_xor(kmin_w, off));
    }

    // ---- K / V fragments of this wave's 32 keys (B operands: column = key, k = d) ----
    bf16x8 kf[8], vf[8];
    {
      const int krow = min(kl, region - 1);
      const __bf16* kp = is_prefix ? (const __bf16*)a.k_prefix + ((int64_t)krow * a.hkv + kvh) * D
                                   : (const __bf16*)a.k_own + (int64_t)krow * a.k_stride + (int64_t)kvh * D;
      const __bf16* vp = is_prefix ? (const __bf16*)a.v_prefix + ((int64_t)krow * a.hkv + kvh) * D
                                   : (const __bf16*)a.v_own + (int64_t)krow * a.v_stride + (int64_t)kvh * D;
#pragma unroll
      for (int s = 0; s < 8; s++) {
        kf[s] = *(const bf16x8*)(kp + 16 * s + 8 * hf);
        vf[s] = *(const bf16x8*)(vp + 16 * s + 8 * hf);
      }
    }
    f32x16 dk_acc[4], dv_acc[4];
#pragma unroll
    for (int db = 0; db < 4; db++) { dk_acc[db] = zero16(); dv_acc[db] = zero16(); }

    auto step_head = [&](int s) { return kvh * G + s / nq; };      // steps are head-major
    auto step_q0 = [&](int s) { return (qt_lo + s % nq) * KV_BM; };

#pragma unroll
    for (int s = 0; s < 8; s++) { pin(kf[s]); pin(vf[s]); }

    kv_issue(a, sm, 0, step_head(s_lo), step_q0(s_lo), w, lane);
    dma_wait_all();
    __syncthreads();

    // first / last key of this wave's block, unified
    const int jw_first = j0 + 32 * w;
    const int jw_last = jw_first + 31;

    for (int s = s_lo; s < s_hi; s++) {
      const int buf = (s - s_lo) & 1;
      if (s + 1 < s_hi) kv_issue(a, sm, buf ^ 1, step_head(s + 1), step_q0(s + 1), w, lane);   // lands during this step
      const int q0 = step_q0(s);

      // all 32 keys of this wave visible to all queries of the tile?
      if (jw_last <= P + q0 && kmin_w > P + q0 + KV_BM - 1 && q0 + KV_BM <= N) {
#pragma unroll
        for (int half = 0; half < KV_NQB / 2; half++)
          kv_step_full(sm, buf, kf, vf, dk_acc, dv_acc, c_scale, a_rd, t_rd, hf, 2 * half);
      } else
#pragma unroll
      for (int qb = 0; qb < KV_NQB; qb++) {
        const int gq_first = P + q0 + 32 * qb;                 // unified index of the block's first query
        const int gq_last = min(gq_first + 31, P + N - 1);
        // block-level skip: every key is after the last query, or no key's range reaches the block
        if (jw_first > gq_last || kmax_w <= gq_first) continue;
        const bool full = jw_last <= gq_first && kmin_w > gq_last && q0 + 32 * qb + 31 < N;

        f32x16 s_acc, p_acc;
        f32x4 l2[4], dl[4];
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
          l2[r4] = *(const f32x4*)(&sm.lse[buf][qb * 32 + r4 * 8 + 4 * hf]) * LOG2E_F;
          dl[r4] = *(const f32x4*)(&sm.delta[buf][qb * 32 + r4 * 8 + 4 * hf]);
        }
#pragma unroll
        for (int ss = 0; ss < 8; ss++) s_acc = mfma32(lds_row_frag(sm.q[buf], a_rd, qb, ss), kf[ss], ss == 0 ? zero16() : s_acc);
#pragma unroll
        for (int ss = 0; ss < 8; ss++) p_acc = mfma32(lds_row_frag(sm.g[buf], a_rd, qb, ss), vf[ss], ss == 0 ? zero16() : p_acc);
        // P and dS (rows = queries: (r/4)*8 + 4*hf + r%4 inside the block)
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++)
#pragma unroll
          for (int e = 0; e < 4; e++)
            s_acc[r4 * 4 + e] = fast_exp2(fmaf(s_acc[r4 * 4 + e], c_scale, -l2[r4][e]));
        if (!full) {
          const int q_lim = min(my_kend, P + N);           // queries at or beyond this see nothing
#pragma unroll
          for (int r4 = 0; r4 < 4; r4++)
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const int gq = gq_first + r4 * 8 + 4 * hf + e;
              s_acc[r4 * 4 + e] = (j <= gq && gq < q_lim) ? s_acc[r4 * 4 + e] : 0.f;
            }
        }
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++)
#pragma unroll
          for (int e = 0; e < 4; e++)
            p_acc[r4 * 4 + e] = s_acc[r4 * 4 + e] * (p_acc[r4 * 4 + e] - dl[r4][e]);
        // dV^T += dO^T P ; dK^T += Q^T dS
#pragma unroll
        for (int t = 0; t < 2; t++) {
          const bf16x8 pf = cvt8(s_acc[8 * t + 0], s_acc[8 * t + 1], s_acc[8 * t + 2], s_acc[8 * t + 3],
                                 s_acc[8 * t + 4], s_acc[8 * t + 5], s_acc[8 * t + 6], s_acc[8 * t + 7]);
          const bf16x8 df = cvt8(p_acc[8 * t + 0], p_acc[8 * t + 1], p_acc[8 * t + 2], p_acc[8 * t + 3],
                                 p_acc[8 * t + 4], p_acc[8 * t + 5], p_acc[8 * t + 6], p_acc[8 * t + 7]);
#pragma unroll
          for (int db = 0; db < 4; db++) {
            dv_acc[db] = mfma32(lds_tr_frag(sm.g[buf], t_rd, qb * 32 + 16 * t, db), pf, dv_acc[db]);
            dk_acc[db] = mfma32(lds_tr_frag(sm.q[buf], t_rd, qb * 32 + 16 * t, db), df, dk_acc[db]);
          }
        }
      }

      dma_wait_all();
      __syncthreads();
    }

    // ---- epilogue: accumulators hold dK^T / dV^T: column = key, rows d = db*32 + (r/4)*8 + 4*hf + r%4 ----
    if (partial) {
      // raw fp32 partial sums of this chunk; the reduce kernel adds the chunks in order
      float* base = pl.slots + (((int64_t)item * a.hkv + kvh) * 2) * KV_BN * D + (int64_t)(32 * w + c32) * D;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
          const int d0 = db * 32 + r4 * 8 + 4 * hf;
          f32x4 ck, cv;
#pragma unroll
          for (int e = 0; e < 4; e++) { ck[e] = dk_acc[db][r4 * 4 + e]; cv[e] = dv_acc[db][r4 * 4 + e]; }
          *(f32x4*)(base + d0) = ck;
          *(f32x4*)(base + KV_BN * D + d0) = cv;
        }
    } else if (key_ok) {
      if (is_prefix) {
        if (my_kend > P) {       // a visible prefix key; others receive nothing
          float* dkp = a.dk_prefix_acc + ((int64_t)kl * a.hkv + kvh) * D;
          float* dvp = a.dv_prefix_acc + ((int64_t)kl * a.hkv + kvh) * D;
#pragma unroll
          for (int db = 0; db < 4; db++)
#pragma unroll
            for (int r4 = 0; r4 < 4; r4++) {
              const int d0 = db * 32 + r4 * 8 + 4 * hf;
              f32x4 ck = *(f32x4*)(dkp + d0), cv = *(f32x4*)(dvp + d0);
#pragma unroll
              for (int e = 0; e < 4; e++) { ck[e] += a.scale * dk_acc[db][r4 * 4 + e]; cv[e] += dv_acc[db][r4 * 4 + e]; }
              *(f32x4*)(dkp + d0) = ck;
              *(f32x4*)(dvp + d0) = cv;
            }
        }
      } else {
        __bf16* dkp = (__bf16*)a.dk_own + ((int64_t)kl * a.hkv + kvh) * D;
        __bf16* dvp = (__bf16*)a.dv_own + ((int64_t)kl * a.hkv + kvh) * D;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
          for (int r4 = 0; r4 < 4; r4++) {
            const int d0 = db * 32 + r4 * 8 + 4 * hf;
            *(bf16x4*)(dkp + d0) = cvt4(a.scale * dk_acc[db][r4 * 4 + 0], a.scale * dk_acc[db][r4 * 4 + 1],
                                        a.scale * dk_acc[db][r4 * 4 + 2], a.scale * dk_acc[db][r4 * 4 + 3]);
            *(bf16x4*)(dvp + d0) = cvt4(dv_acc[db][r4 * 4 + 0], dv_acc[db][r4 * 4 + 1],
                                        dv_acc[db][r4 * 4 + 2], dv_acc[db][r4 * 4 + 3]);
          }
      }
    }
  }
}

// Sums the partial slots of every key tile that was cut into chunks, in chunk order, and writes the
// final gradients (own keys: bf16; prefix keys: added to the fp32 accumulators).
__global__ void __launch_bounds__(NTHREADS)
kv_reduce_kernel(AttnArgs a, KvPlan pl) {
  const int tile = blockIdx.x, kvh = blockIdx.y;
  const int nc = pl.tile_nchunks[tile];
  if (nc <= 1) return;
  const int item0 = pl.tile_item0[tile];
  const bool is_prefix = tile < pl.n_ptiles;
  const int k0 = is_prefix ? tile * KV_BN : (tile - pl.n_ptiles) * KV_BN;
  const int region = is_prefix ? a.n_prefix : a.n_q;
  for (int u = 0; u < KV_BN * D / 4 / NTHREADS; u++) {
    const int e = (threadIdx.x + NTHREADS * u) * 4;
    const int key = e / D, d0 = e % D;
    if (k0 + key >= region) continue;
    f32x4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < nc; c++) {
      const float* base = pl.slots + (((int64_t)(item0 + c) * a.hkv + kvh) * 2) * KV_BN * D + e;
      sk += *(const f32x4*)base;
      sv += *(const f32x4*)(base + KV_BN * D);
    }
    if (is_prefix) {
      if (a.kend[k0 + key] > a.n_prefix) {
        float* dkp = a.dk_prefix_acc + ((int64_t)(k0 + key) * a.hkv + kvh) * D + d0;
        float* dvp = a.dv_prefix_acc + ((int64_t)(k0 + key) * a.hkv + kvh) * D + d0;
        f32x4 ck = *(f32x4*)dkp, cv = *(f32x4*)dvp;
        ck += a.scale * sk;
        cv += sv;
        *(f32x4*)dkp = ck;
        *(f32x4*)dvp = cv;
      }
    } else {
      __bf16* dkp = (__bf16*)a.dk_own + ((int64_t)(k0 + key) * a.hkv + kvh) * D + d0;
      __bf16* dvp = (__bf16*)a.dv_own + ((int64_t)(k0 + key) * a.hkv + kvh) * D + d0;
      *(bf16x4*)dkp = cvt4(a.scale * sk[0], a.scale * sk[1], a.scale * sk[2], a.scale * sk[3]);
      *(bf16x4*)dvp = cvt4(sv[0], sv[1], sv[2], sv[3]);
    }
  }
}

}  // namespace

size_t mfma_attn_dkdv_workspace(int n_q, int n_prefix, int hkv) { return kv_plan_layout(nullptr, n_q, n_prefix, hkv, nullptr); }

hipError_t mfma_attn_dkdv(const AttnArgs& a, hipStream_t st) {
  KvPlan pl;
  const size_t need = kv_plan_layout(a.workspace, a.n_q, a.n_prefix, a.hkv, &pl);
  if (need > a.workspace_bytes) return hipErrorInvalidValue;
  {
    KernelTimer timer(TT_KERNEL_ATTN_PLAN, st);
    kv_plan_kernel<<<1, PLAN_THREADS, 0, st>>>(pl, a.kt_max, a.n_q, a.n_prefix, a.hq / a.hkv, a.hkv);
    if (hipError_t e = hipGetLastError()) return e;
  }
  if (hipError_t e = hipFuncSetAttribute((const void*)tree_attn_dkdv_kernel,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(KvSmem)))
    return e;
  int dev = 0, n_cu = 256;
  if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  // one resident workgroup per compute unit pulls work items until the counter runs out
  const int64_t max_work = (int64_t)pl.max_items * a.hkv;
  const unsigned grid = (unsigned)std::min<int64_t>(n_cu, max_work);
  {
    KernelTimer timer(TT_KERNEL_ATTN_DKDV, st);
    tree_attn_dkdv_kernel<<<grid, NTHREADS, sizeof(KvSmem), st>>>(a, pl);
    if (hipError_t e = hipGetLastError()) return e;
  }
  {
    KernelTimer timer(TT_KERNEL_ATTN_REDUCE, st);
    kv_reduce_kernel<<<dim3(pl.n_tiles, a.hkv), NTHREADS, 0, st>>>(a, pl);
    if (hipError_t e = hipGetLastError()) return e;
  }
  return hipSuccess;
}

}  // namespace tt
