// Tree attention backward, dK/dV pass, on bf16 MFMA (gfx950), head dim 128.
//
// Column-parallel: one work item = 256 keys x one kv head (8 wavefronts x 32 keys, two per SIMD) x a chunk of the
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
constexpr int KV_NW = 8;                 // wavefronts per workgroup, 32 keys each
constexpr int NTHREADS = 64 * KV_NW;

// ------------------------------------------------------------------------------------------------
// dK / dV
// ------------------------------------------------------------------------------------------------
constexpr int KV_BN = 32 * KV_NW;  // keys per workgroup
constexpr int KV_BM = 64;          // queries per staged tile (one pipeline step)
constexpr int KV_NQB = KV_BM / 32;  // 32-query blocks per step

constexpr int KV_KREG = 6;                 // K fragments (k-steps) held in registers; the rest sit in LDS
constexpr int KV_NFRAG = 8 + (8 - KV_KREG);
struct KvSmem {
  __bf16 q[2][KV_BM * TILE_ROW];   // swizzled tiles, filled by asynchronous global -> LDS copies
  __bf16 g[2][KV_BM * TILE_ROW];   // dO
  float lse[2][KV_BM];             // -LSE * log2(e) of the tile's queries
  float delta[2][KV_BM];           // -delta
  // B-operand fragments of this wave's keys that do not fit in registers, private to each lane
  // (lane l of wave w keeps fragment f at [w][f][8 l]): the 8 k-steps of V (dP = dO V^T), then
  // k-steps KV_KREG .. 7 of K
  __bf16 frag[KV_NW][KV_NFRAG][64 * 8];
  int work, queue, exhausted;
};
// byte offsets between the LDS arrays, used as immediate offsets of the LDS reads
constexpr int KV_STAGE_B = KV_BM * TILE_ROW * 2;        // one staged tile
constexpr int KV_G_OFF = 2 * KV_STAGE_B;                // q[b] -> g[b]
constexpr int KV_SCALAR_STAGE_B = KV_BM * 4;            // lse[b] -> lse[b ^ 1]
constexpr int KV_DELTA_OFF = 2 * KV_SCALAR_STAGE_B;     // lse[b] -> delta[b]
constexpr int KV_RING = 2;                              // operand fragments requested ahead of their MFMA


// Starts the copy of one (head, query tile) step into stage `buf`.  `lane` should be a value the
// compiler cannot trace back to the thread index, so that the per-lane source offsets are
// recomputed here instead of being kept in registers across the whole item.
__device__ __forceinline__ void kv_issue(const AttnArgs& a, KvSmem& sm, int buf, int h, int q0, int w, int lane) {
  const int rows = min(KV_BM, a.n_q - q0);
  const __bf16* qsrc = (const __bf16*)a.q + (int64_t)q0 * a.q_stride + (int64_t)h * D;
  const __bf16* gsrc = (const __bf16*)a.d_o + ((int64_t)q0 * a.hq + h) * D;
  dma_tile64<KV_NW>(qsrc, (uint32_t)a.q_stride * 2, rows, sm.q[buf], w, lane);
  dma_tile64<KV_NW>(gsrc, (uint32_t)a.hq * D * 2, rows, sm.g[buf], w, lane);
  // per-query terms (-LSE log2 e by wave 0, -delta by wave 1; rows past the end repeat the last one,
  // such rows are masked by the boundary test)
  if (w < 2) {
    const float* src = (w == 0 ? a.neg_lse2 : a.delta) + (int64_t)h * a.n_q + q0;
    float* dst = w == 0 ? sm.lse[buf] : sm.delta[buf];
    dma4(uniform_ptr(src), (uint32_t)min(lane, rows - 1) * 4u, lds_addr_uniform(dst));
  }
}

// ---- work decomposition -------------------------------------------------------------------------
// Key tiles.  A workgroup works on up to KV_BN consecutive keys and walks the (query head, query
// tile) steps of every query tile that can see one of them, so keys with different visibility ranges
// in one tile leave wavefronts idle.  In DFS order the keys of a tree node are consecutive and share
// their range; the planner therefore forms tiles from runs of consecutive 64-key summary entries with
// the same largest bound (kt_max), at most KV_BN / 64 entries per tile, instead of cutting the key
// axis at fixed multiples of KV_BN.
//
// Work items.  A tile's work is its list of steps.  Tiles near the root of the tree are seen by
// almost every query while leaf tiles are seen by few, so a tile's steps are cut into chunks of at
// most `chunk` steps; the planner sizes the chunks so that the launch has about KV_ITEMS_PER_WG work
// items per resident workgroup, workgroups pull items from a counter (longest items first), and tiles that were cut have their fp32 partial
// results summed in chunk order by a reduce kernel (bit-reproducible).
constexpr int KV_TARGET_WORK = 768;      // work items (tile chunk x kv head) aimed for, at most (sizes the plan tables)
constexpr int KV_ITEMS_PER_WG = 2;       // ... and per resident workgroup: with the longest items handed out first two
                                         // per workgroup balance as well as three did in plain order, with 40 % fewer
                                         // partial slots to write and reduce
constexpr int KV_MIN_CHUNK = 32;         // steps
constexpr int KV_SORT_BELOW = 16;        // items per workgroup below which the items are handed out longest first
constexpr int PLAN_THREADS = 1024;
constexpr int KV_EPT = KV_BN / 64;       // summary entries per key tile, at most

constexpr int KV_MAX_QUEUES = 64;
struct KvPlanHeader {
  int n_work;        // work items = n_items * hkv
  // Work queues.  With hkv <= KV_MAX_QUEUES there is one queue per kv head (entry w of queue q = item
  // item_order[w] for kv head q) and a workgroup starts on the queue of its XCD: the workgroups of one XCD then
  // work on neighbouring key tiles of one kv head, which stream the same Q / dO tiles at about the same time, so
  // the XCD's L2 serves part of those reads (at a 131 K-token tree: 348 GB fetched per launch with one shared
  // queue, 229 GB with one per head, the pass 5 % faster).  A workgroup whose queue is empty moves on to the next
  // one.  Used when every workgroup gets many items (the plain hand-out order); with few items per workgroup (the
  // longest-first order) one shared queue balances better and is what the planner sets up.
  int n_queues, per_queue;
  int counter[KV_MAX_QUEUES];   // next entry of every queue
  int chunk;         // steps per chunk
  int n_split_items; // items [0, n_split_items) write partial slots (slot index = item index)
  int n_tiles;       // key tiles formed
  int n_split_tiles; // tiles cut into more than one chunk (listed in split_tile)
};

struct KvPlan {                // device pointers into the workspace
  KvPlanHeader* hdr;
  int *tile_e0, *tile_ne;                                 // [max_tiles] first summary entry, entries (64 keys each)
  int *tile_nq, *tile_qtlo, *tile_nchunks, *tile_item0;   // [max_tiles]
  int *item_tile, *item_chunk;                            // [max_items]
  int* item_order;                                        // [max_items] items in the order they are handed out (longest first)
  int* split_tile;                                        // [max_split_tiles]
  float* slots;                                           // [max_slots][hkv][2][KV_BN][D]
  int np64, no64;                                         // summary entries of the prefix / own region
  int max_tiles, max_items, max_slots, max_split_tiles;
};

__host__ __device__ inline int kv_target_items(int hkv) { return (KV_TARGET_WORK + hkv - 1) / hkv; }

__host__ inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Carves the plan out of `base`; with base == nullptr only the size is computed.
// Bounds: every tile holds at least one summary entry, so there are at most np64 + no64 tiles; a
// tile that is cut has more than `chunk` steps and the steps of one kv head sum to at most
// chunk * kv_target_items, so at most kv_target_items tiles are cut, into at most
// 2 * kv_target_items chunks.
__host__ inline size_t kv_plan_layout(void* base, int n_q, int n_prefix, int hkv, KvPlan* out) {
  const int np64 = (n_prefix + 63) / 64, no64 = (n_q + 63) / 64;
  const int max_tiles = np64 + no64;
  const int max_items = max_tiles + kv_target_items(hkv);
  const int max_slots = 2 * kv_target_items(hkv);
  const int max_split_tiles = kv_target_items(hkv);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return base ? (char*)base + o : (char*)nullptr; };
  char* hdr = take(sizeof(KvPlanHeader));
  char* t[6];
  for (int i = 0; i < 6; i++) t[i] = take(sizeof(int) * max_tiles);
  char* i0 = take(sizeof(int) * max_items);
  char* i1 = take(sizeof(int) * max_items);
  char* i2 = take(sizeof(int) * max_items);
  char* st = take(sizeof(int) * max_split_tiles);
  char* sl = take(sizeof(float) * (size_t)max_slots * hkv * 2 * KV_BN * D);
  if (out) {
    out->hdr = (KvPlanHeader*)hdr;
    out->tile_e0 = (int*)t[0]; out->tile_ne = (int*)t[1];
    out->tile_nq = (int*)t[2]; out->tile_qtlo = (int*)t[3]; out->tile_nchunks = (int*)t[4]; out->tile_item0 = (int*)t[5];
    out->item_tile = (int*)i0; out->item_chunk = (int*)i1; out->item_order = (int*)i2; out->split_tile = (int*)st; out->slots = (float*)sl;
    out->np64 = np64; out->no64 = no64;
    out->max_tiles = max_tiles; out->max_items = max_items; out->max_slots = max_slots; out->max_split_tiles = max_split_tiles;
  }
  return off;
}

// exclusive prefix sum / prefix maximum of one int per thread over the workgroup; the reduction over
// all threads is returned through *total
template <bool MAX>
__device__ inline int block_exclusive_scan(int v, int* scratch /*[PLAN_THREADS]*/, int* total, int identity = 0) {
  const int t = threadIdx.x;
  scratch[t] = v;
  __syncthreads();
  for (int off = 1; off < PLAN_THREADS; off <<= 1) {
    const int other = t >= off ? scratch[t - off] : identity;
    __syncthreads();
    scratch[t] = MAX ? max(scratch[t], other) : scratch[t] + other;
    __syncthreads();
  }
  const int excl = t > 0 ? scratch[t - 1] : identity;
  *total = scratch[PLAN_THREADS - 1];
  __syncthreads();
  return excl;
}

__global__ void __launch_bounds__(PLAN_THREADS)
kv_plan_kernel(KvPlan pl, const int32_t* __restrict__ kt_max, int n_q, int n_prefix, int G, int hkv, int n_workgroups) {
  __shared__ int scratch[PLAN_THREADS];
  const int t = threadIdx.x;
  const int np64 = pl.np64, n_ent = pl.np64 + pl.no64;
  // a run starts at the first entry of a region and wherever the largest bound changes
  auto run_break = [&](int e) { return e == 0 || e == np64 || kt_max[e] != kt_max[e - 1]; };

  // ---- pass 1: tiles = runs cut every KV_EPT entries; each thread owns consecutive entries ----
  const int per = (n_ent + PLAN_THREADS - 1) / PLAN_THREADS;
  const int lo = min(t * per, n_ent), hi = min(lo + per, n_ent);
  int last_break = -1;
  for (int e = lo; e < hi; e++)
    if (run_break(e)) last_break = e;
  int unused;
  const int carry = block_exclusive_scan<true>(last_break, scratch, &unused, -1);    // start of the run my first entry is in
  int my_tiles = 0;
  {
    int run_start = carry;
    for (int e = lo; e < hi; e++) {
      if (run_break(e)) run_start = e;
      if (((e - run_start) % KV_EPT) == 0) my_tiles++;
    }
  }
  int n_tiles;
  int tl = block_exclusive_scan<false>(my_tiles, scratch, &n_tiles);
  int my_steps = 0;
  {
    int run_start = carry;
    for (int e = lo; e < hi; e++) {
      if (run_break(e)) run_start = e;
      if (((e - run_start) % KV_EPT) != 0) continue;
      // the tile runs to the next break, region end or KV_EPT entries
      const int e_end = e < np64 ? np64 : n_ent;
      int ne = 1;
      while (ne < KV_EPT && e + ne < e_end && kt_max[e + ne] == kt_max[e]) ne++;
      const int kmax = kt_max[e];
      const int i_lo = e < np64 ? 0 : (e - np64) * 64;                 // first query that can see a key of the tile
      const int i_hi = (int)min((int64_t)n_q, (int64_t)kmax - n_prefix);
      const int qt_lo = i_lo / KV_BM;
      const int nq = i_hi > i_lo ? (i_hi + KV_BM - 1) / KV_BM - qt_lo : 0;
      pl.tile_e0[tl] = e;
      pl.tile_ne[tl] = ne;
      pl.tile_nq[tl] = nq;
      pl.tile_qtlo[tl] = qt_lo;
      my_steps += nq * G;
      tl++;
    }
  }
  int total_steps;
  block_exclusive_scan<false>(my_steps, scratch, &total_steps);       // (its barriers also publish the tile tables)
  const int64_t all = (int64_t)total_steps * hkv;
  const int target = max(1, min(KV_TARGET_WORK, KV_ITEMS_PER_WG * n_workgroups));
  const int chunk = (int)max((int64_t)KV_MIN_CHUNK, (all + target - 1) / target);

  // ---- pass 2: chunks per tile; cut tiles are numbered first (their item index is also their slot);
  //      each thread owns consecutive tiles ----
  const int per_t = (n_tiles + PLAN_THREADS - 1) / PLAN_THREADS;
  const int tlo = min(t * per_t, n_tiles), thi = min(tlo + per_t, n_tiles);
  int my_split = 0, my_whole = 0, my_split_tiles = 0;
  for (int i = tlo; i < thi; i++) {
    const int steps = pl.tile_nq[i] * G;
    const int nc = (steps + chunk - 1) / chunk;
    pl.tile_nchunks[i] = nc;
    if (nc > 1) { my_split += nc; my_split_tiles++; } else my_whole += nc;
  }
  int n_split, n_whole, n_split_tiles;
  int split0 = block_exclusive_scan<false>(my_split, scratch, &n_split);
  int whole0 = block_exclusive_scan<false>(my_whole, scratch, &n_whole) + n_split;
  int st0 = block_exclusive_scan<false>(my_split_tiles, scratch, &n_split_tiles);
  for (int i = tlo; i < thi; i++) {
    const int nc = pl.tile_nchunks[i];
    int& cursor = nc > 1 ? split0 : whole0;
    pl.tile_item0[i] = cursor;
    for (int c = 0; c < nc; c++) { pl.item_tile[cursor + c] = i; pl.item_chunk[cursor + c] = c; }
    cursor += nc;
    if (nc > 1) pl.split_tile[st0++] = i;
  }
  // ---- pass 3: hand-out order.  Workgroups pull items from a counter, so the launch ends when the item that
  //      was started last finishes: long items go first and short ones fill the end.  A stable counting sort
  //      of the items by their number of steps into 64 classes: inside a class the items keep their order
  //      (neighbouring key tiles stream the same query tiles at about the same time, which the L2 likes).
  //      Results do not depend on the order: every item has its own output rows or partial slot.
  //      With many items per workgroup the end effect is small and the plain order (key tiles in sequence order)
  //      measured 1-2 % faster, so the sort is applied only below KV_SORT_BELOW items per workgroup. ----
  constexpr int NCLS = 64, PLAN_WAVES = PLAN_THREADS / 64;      // NCLS = wavefront size (see the placement loop)
  __shared__ int cls_base[NCLS];
  __shared__ int wave_cnt[PLAN_WAVES][NCLS];
  const int n_items = n_split + n_whole;
  if ((int64_t)n_items * hkv >= (int64_t)KV_SORT_BELOW * n_workgroups) {
    for (int i = t; i < n_items; i += PLAN_THREADS) pl.item_order[i] = i;
    if (t == 0) {
      pl.hdr->n_work = (n_split + n_whole) * hkv;
      pl.hdr->n_queues = hkv <= KV_MAX_QUEUES ? hkv : 1;
      pl.hdr->per_queue = hkv <= KV_MAX_QUEUES ? n_split + n_whole : (n_split + n_whole) * hkv;
      for (int q = 0; q < KV_MAX_QUEUES; q++) pl.hdr->counter[q] = 0;
      pl.hdr->chunk = chunk;
      pl.hdr->n_split_items = n_split;
      pl.hdr->n_tiles = n_tiles;
      pl.hdr->n_split_tiles = n_split_tiles;
    }
    return;
  }
  auto item_class = [&](int i) {
    const int tile = pl.item_tile[i];
    const int steps = min(chunk, pl.tile_nq[tile] * G - pl.item_chunk[i] * chunk);
    return NCLS - 1 - min(NCLS - 1, (int)(((int64_t)steps * NCLS) / (chunk + 1)));       // class 0 = longest
  };
  const int lane = t & 63, wv = t >> 6;
  if (t < NCLS) cls_base[t] = 0;
  __syncthreads();                       // (also publishes the item tables written above)
  // class sizes -> first position of every class
  for (int i = t; i < n_items; i += PLAN_THREADS) atomicAdd(&cls_base[item_class(i)], 1);      // integer counts: order-independent
  __syncthreads();
  if (t == 0) {
    int run = 0;
    for (int c = 0; c < NCLS; c++) { const int n = cls_base[c]; cls_base[c] = run; run += n; }
  }
  __syncthreads();
  // placement, 1024 items at a time in item order.  Inside a wavefront the rank of an item among the items of
  // its class comes from one ballot per class that actually occurs in the wavefront (a few: neighbouring
  // items are chunks of the same tile).
  for (int i0 = 0; i0 < n_items; i0 += PLAN_THREADS) {
    const int i = i0 + t;
    const int c = i < n_items ? item_class(i) : -1;
    wave_cnt[wv][lane] = 0;                            // NCLS == wavefront size: one class count per lane
    int rank_in_wave = 0;
    uint64_t todo = __ballot(c >= 0);
    while (todo) {
      const int leader = __builtin_ctzll(todo);
      const int lc = __builtin_amdgcn_readlane(c, leader);
      const uint64_t m = __ballot(c == lc);
      if (c == lc) rank_in_wave = __popcll(m & ((1ull << lane) - 1ull));
      if (lane == 0) wave_cnt[wv][lc] = __popcll(m);
      todo &= ~m;
    }
    __syncthreads();
    if (c >= 0) {
      int before = 0;
      for (int ww = 0; ww < wv; ww++) before += wave_cnt[ww][c];
      pl.item_order[cls_base[c] + before + rank_in_wave] = i;
    }
    __syncthreads();
    if (t < NCLS) {
      int n = 0;
      for (int ww = 0; ww < PLAN_WAVES; ww++) n += wave_cnt[ww][t];
      cls_base[t] += n;
    }
    __syncthreads();
  }
  if (t == 0) {
    pl.hdr->n_work = (n_split + n_whole) * hkv;
    pl.hdr->n_queues = 1;                      // few items per workgroup: one shared queue balances best (measured)
    pl.hdr->per_queue = (n_split + n_whole) * hkv;
    for (int q = 0; q < KV_MAX_QUEUES; q++) pl.hdr->counter[q] = 0;
    pl.hdr->chunk = chunk;
    pl.hdr->n_split_items = n_split;
    pl.hdr->n_tiles = n_tiles;
    pl.hdr->n_split_tiles = n_split_tiles;
  }
}

__global__ void __launch_bounds__(NTHREADS, 2)
tree_attn_dkdv_kernel(AttnArgs a, KvPlan pl) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  KvSmem& sm = *reinterpret_cast<KvSmem*>(smem_raw);
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // wave-uniform: lives in a scalar register
  const int c32 = lane & 31, hf = lane >> 5;
  const int G = a.hq / a.hkv;
  const int P = a.n_prefix, N = a.n_q;
  const float c_scale = a.scale * LOG2E_F;     // folded into K: S comes out of the MFMAs as a base-2 exponent
  const int chunk = pl.hdr->chunk;

  // LDS byte addresses of this lane's operand fragments in stage `buf` of the Q tile.  The dO tile,
  // the 32-query block, the k-step rows and the per-query scalars are reached through immediate
  // offsets; when the stage flips the addresses move by +-one stage.  (A swizzled tile needs one
  // address per k-step / column block: the permutation is an exclusive-or, not an offset.)
  const uint32_t sm_base = (uint32_t)(uintptr_t)&sm;
  uint32_t ra[8], ta[8];
  frag_addresses(sm_base, lane, ra, ta);
  uint32_t la = sm_base + (uint32_t)offsetof(KvSmem, lse) + 16u * hf;      // lse[buf][4 hf]
  const uint32_t va = sm_base + (uint32_t)offsetof(KvSmem, frag) + (uint32_t)(KV_NFRAG * 1024) * w + 16u * lane;
  int buf = 0;                                  // stage of the next step; carried across work items
  int stage_step = KV_STAGE_B, scalar_step = KV_SCALAR_STAGE_B;   // signed distance to the other stage

  const int n_queues = pl.hdr->n_queues, per_queue = pl.hdr->per_queue;
  int queue, exhausted = 0;                  // current queue; queues this workgroup has found empty
  {
    unsigned xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    queue = (int)(xcc & 0xf) % n_queues;
  }
  for (;;) {
    if (threadIdx.x == 0) {
      // next entry of the current queue; an empty queue is left for good (the counters only grow), and once all
      // queues have been found empty the workgroup is done -- every wave reaches that point
      int wk = -1, q = queue, ex = exhausted;
      while (ex < n_queues) {
        const int t = atomicAdd(&pl.hdr->counter[q], 1);
        if (t < per_queue) { wk = t; break; }
        ex++;
        q = q + 1 == n_queues ? 0 : q + 1;
      }
      sm.work = wk; sm.queue = q; sm.exhausted = ex;
    }
    __syncthreads();
    const int work = sm.work;
    queue = sm.queue; exhausted = sm.exhausted;
    __syncthreads();                         // everyone has read the slots before they are rewritten
    if (work < 0) break;
    const int kvh = n_queues == a.hkv ? queue : work % a.hkv;
    const int item = pl.item_order[n_queues == a.hkv ? work : work / a.hkv];
    const int tile = pl.item_tile[item];
    const int nq = pl.tile_nq[tile], qt_lo = pl.tile_qtlo[tile];
    const int s_lo = pl.item_chunk[item] * chunk;
    const int s_hi = min(s_lo + chunk, nq * G);
    const bool partial = pl.tile_nchunks[tile] > 1;

    // steps are head-major: step s = (head kvh*G + s / nq, query tile qt_lo + s % nq)
    int head = kvh * G + s_lo / nq;
    int qi = s_lo % nq;
    // the first step's tiles are requested first, so that their round trip runs beside those of the visibility bounds and the K / V fragments
    // (both stages are free: every wave has passed the barrier behind the previous item's last step)
    {
      int lane_o = lane;
      asm volatile("" : "+v"(lane_o));
      kv_issue(a, sm, buf, head, (qt_lo + qi) * KV_BM, w, lane_o);
    }

    const int e0 = pl.tile_e0[tile];
    const int n_keys = pl.tile_ne[tile] * 64;        // keys of the tile (the last entry of a region may be ragged)
    const bool is_prefix = e0 < pl.np64;
    const int k0 = (is_prefix ? e0 : e0 - pl.np64) * 64;                      // region-local first key
    const int region = is_prefix ? P : N;
    const int j0 = is_prefix ? k0 : P + k0;          // unified index of the first key
    // this lane's key; wavefronts beyond the tile's keys have nothing to do
    const int kl = k0 + 32 * w + c32;
    const bool key_ok = 32 * w + c32 < n_keys && kl < region;
    const int j = j0 + 32 * w + c32;
    const int my_kend = key_ok ? a.kend[j] : 0;
    int kmax_w = my_kend, kmin_w = key_ok ? my_kend : INT32_MAX;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      kmax_w = max(kmax_w, __shfl_xor(kmax_w, off));
      kmin_w = min(kmin_w, __shfl_xor(kmin_w, off));
    }
    kmax_w = __builtin_amdgcn_readfirstlane(kmax_w);
    kmin_w = __builtin_amdgcn_readfirstlane(kmin_w);
    const int q_lim = min(my_kend, P + N);           // queries at or beyond this do not see the key

    // ---- K fragments of this wave's 32 keys stay in registers (B operands: column = key, k = d);
    //      the V fragments go to this lane's private LDS slots ----
    bf16x8 kf[KV_KREG];
    {
      const int krow = min(kl, region - 1);
      const __bf16* kp = is_prefix ? (const __bf16*)a.k_prefix + ((int64_t)krow * a.hkv + kvh) * D
                                   : (const __bf16*)a.k_own + (int64_t)krow * a.k_stride + (int64_t)kvh * D;
      const __bf16* vp = is_prefix ? (const __bf16*)a.v_prefix + ((int64_t)krow * a.hkv + kvh) * D
                                   : (const __bf16*)a.v_own + (int64_t)krow * a.v_stride + (int64_t)kvh * D;
#pragma unroll
      for (int s = 0; s < KV_KREG; s++) kf[s] = scale_frag(*(const bf16x8*)(kp + 16 * s + 8 * hf), c_scale);
#pragma unroll
      for (int s = 0; s < 8; s++) {
        const bf16x8 vf = *(const bf16x8*)(vp + 16 * s + 8 * hf);
        *(TT_LDS(bf16x8)*)(va + 1024 * s) = vf;
      }
#pragma unroll
      for (int s = KV_KREG; s < 8; s++) {
        const bf16x8 kx = scale_frag(*(const bf16x8*)(kp + 16 * s + 8 * hf), c_scale);
        *(TT_LDS(bf16x8)*)(va + 1024 * (8 + s - KV_KREG)) = kx;
      }
    }
    f32x16 dk_acc[4], dv_acc[4];
#pragma unroll
    for (int db = 0; db < 4; db++) { dk_acc[db] = zero16(); dv_acc[db] = zero16(); }

    // every register loaded from global memory is consumed here, so that no wait for it (which would
    // also wait for the tile copies in flight) lands inside the step loop
#pragma unroll
    for (int s = 0; s < KV_KREG; s++) pin(kf[s]);
    pin(q_lim);
    dma_wait_all();
    __syncthreads();

    // first / last key of this wave's block, unified
    const int jw_first = j0 + 32 * w;
    const int jw_last = jw_first + 31;

    for (int s = s_lo; s < s_hi; s++) {
      const int q0 = (qt_lo + qi) * KV_BM;
      if (++qi == nq) { qi = 0; head++; }
      if (s + 1 < s_hi) {                      // the next step's tiles land during this step
        int lane_o = lane;
        asm volatile("" : "+v"(lane_o));
        kv_issue(a, sm, buf ^ 1, head, (qt_lo + qi) * KV_BM, w, lane_o);
      }

#pragma unroll
      for (int qb = 0; qb < KV_NQB; qb++) {
        const int gq_first = P + q0 + 32 * qb;                 // unified index of the block's first query
        const int gq_last = min(gq_first + 31, P + N - 1);
        // block-level skip: every key is after the last query, or no key's range reaches the block
        if (jw_first > gq_last || kmax_w <= gq_first) continue;
        const bool full = jw_last <= gq_first && kmin_w > gq_last && q0 + 32 * qb + 31 < N;
        const int qo = qb * 32 * TILE_ROW * 2;                 // byte offset of the block's rows

        // The block is written as a sequence of slots -- one MFMA, the LDS reads for the MFMA
        // KV_RING slots ahead, a share of the softmax arithmetic -- each closed by a scheduling
        // fence, so that operand fragments live only briefly (the accumulators and K fragments
        // already take 160 of the 256 registers per lane).
        f32x16 s_acc, p_acc;
        bf16x8 fc[KV_RING];
        // transposed fragments of the output phase: slot n < 8: dO^T for dV, k-step t = n / 4, column
        // block db = n % 4; n >= 8: Q^T for dK
        auto read_c = [&](int n) {
          const int db = n & 3, t = (n >> 2) & 1;
          const int off = (n < 8 ? KV_G_OFF : 0) + qo + 16 * t * TILE_ROW * 2;
          return lds_tr2(ta[2 * db], ta[2 * db + 1], off);
        };
        {
          bf16x8 fq[KV_RING], fg[KV_RING], fv[KV_RING];   // fv doubles as the ring of LDS-resident K fragments
          // the accumulators start from -LSE log2 e and -delta of their rows' queries, so the MFMA
          // chains deliver the exponent of P and dP - delta
#pragma unroll
          for (int r4 = 0; r4 < 4; r4++) {
            const f32x4 t = *(TT_LDS(const f32x4)*)(la + qb * 128 + r4 * 32);
#pragma unroll
            for (int e = 0; e < 4; e++) s_acc[r4 * 4 + e] = t[e];
          }
#pragma unroll
          for (int i = 0; i < KV_RING; i++) fq[i] = lds_b128(ra[i], qo);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int ss = 0; ss < 8; ss++) {
            s_acc = mfma32(fq[ss % KV_RING], ss < KV_KREG ? kf[ss < KV_KREG ? ss : 0] : fv[ss % KV_RING], s_acc);
            if (ss >= 4) {
              const int r4 = ss - 4;
              const f32x4 t = *(TT_LDS(const f32x4)*)(la + KV_DELTA_OFF + qb * 128 + r4 * 32);
#pragma unroll
              for (int e = 0; e < 4; e++) p_acc[r4 * 4 + e] = t[e];
            }
            if (ss + KV_RING < 8) {
              fq[ss % KV_RING] = lds_b128(ra[ss + KV_RING], qo);
              if (ss + KV_RING >= KV_KREG) fv[(ss + KV_RING) % KV_RING] = lds_b128(va, 1024 * (8 + ss + KV_RING - KV_KREG));
            } else {
              const int i = ss + KV_RING - 8;
              fg[i] = lds_b128(ra[i], KV_G_OFF + qo);
              fv[i] = lds_b128(va, 1024 * i);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int ss = 0; ss < 8; ss++) {
            p_acc = mfma32(fg[ss % KV_RING], fv[ss % KV_RING], p_acc);
            if (ss + KV_RING < 8) {
              fg[ss % KV_RING] = lds_b128(ra[ss + KV_RING], KV_G_OFF + qo);
              fv[ss % KV_RING] = lds_b128(va, 1024 * (ss + KV_RING));
            } else {
              fc[ss + KV_RING - 8] = read_c(ss + KV_RING - 8);
            }
            // P = exp2(exponent) for two accumulator registers per slot, in the MFMA's shadow
            s_acc[2 * ss] = fast_exp2(s_acc[2 * ss]);
            s_acc[2 * ss + 1] = fast_exp2(s_acc[2 * ss + 1]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        if (!full) {
          asm volatile("" ::: "memory");                   // keep this a real branch (no if-conversion)
          const int jm = jw_first + (lane & 31);           // this lane's key, unified
#pragma unroll
          for (int r4 = 0; r4 < 4; r4++)
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const int gq = gq_first + r4 * 8 + 4 * hf + e;
              s_acc[r4 * 4 + e] = (jm <= gq && gq < q_lim) ? s_acc[r4 * 4 + e] : 0.f;
            }
        }
        // dV^T += dO^T P  (8 slots, with dS = P (dP - delta) = P * p_acc computed in their shadow), then
        // dK^T += Q^T dS  (8 slots); rows = queries (r/4)*8 + 4*hf + r%4 inside the block
        {
          bf16x8 pf[2], df[2];
          pf[0] = cvt8(s_acc[0], s_acc[1], s_acc[2], s_acc[3], s_acc[4], s_acc[5], s_acc[6], s_acc[7]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int n = 0; n < 16; n++) {
            const int t = (n >> 2) & 1, db = n & 3;
            if (n < 8) dv_acc[db] = mfma32(fc[n % KV_RING], pf[t], dv_acc[db]);
            else dk_acc[db] = mfma32(fc[n % KV_RING], df[t], dk_acc[db]);
            if (n + KV_RING < 16) fc[n % KV_RING] = read_c(n + KV_RING);
            if (n < 8) {
              const int e0 = 2 * n;
              p_acc[e0] = s_acc[e0] * p_acc[e0];
              p_acc[e0 + 1] = s_acc[e0 + 1] * p_acc[e0 + 1];
              if (n == 2) pf[1] = cvt8(s_acc[8], s_acc[9], s_acc[10], s_acc[11], s_acc[12], s_acc[13], s_acc[14], s_acc[15]);
              if (n == 4) df[0] = cvt8(p_acc[0], p_acc[1], p_acc[2], p_acc[3], p_acc[4], p_acc[5], p_acc[6], p_acc[7]);
            }
            if (n == 8) df[1] = cvt8(p_acc[8], p_acc[9], p_acc[10], p_acc[11], p_acc[12], p_acc[13], p_acc[14], p_acc[15]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }

      dma_wait_all();
      __syncthreads();
      // the next step reads the other stage
#pragma unroll
      for (int i = 0; i < 8; i++) { ra[i] += stage_step; ta[i] += stage_step; }
      la += scalar_step;
      stage_step = -stage_step;
      scalar_step = -scalar_step;
      buf ^= 1;
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
// final gradients (own keys: bf16; prefix keys: added to the fp32 accumulators).  One workgroup
// handles RED_KEYS keys of one (tile, kv head); a thread owns 4 consecutive d of one key.
constexpr int RED_THREADS = 256;
constexpr int RED_KEYS = RED_THREADS * 4 / D;        // 8 keys per pass
constexpr int RED_PASSES = 4;                        // passes per workgroup
constexpr int RED_PARTS = KV_BN / (RED_KEYS * RED_PASSES);
__global__ void __launch_bounds__(RED_THREADS)
kv_reduce_kernel(AttnArgs a, KvPlan pl) {
  const int si = blockIdx.x / RED_PARTS, part = blockIdx.x % RED_PARTS, kvh = blockIdx.y;
  if (si >= pl.hdr->n_split_tiles) return;
  const int tile = pl.split_tile[si];
  const int nc = pl.tile_nchunks[tile];
  const int item0 = pl.tile_item0[tile];
  const int e0 = pl.tile_e0[tile];
  const int n_keys = pl.tile_ne[tile] * 64;
  const bool is_prefix = e0 < pl.np64;
  const int k0 = (is_prefix ? e0 : e0 - pl.np64) * 64;
  const int region = is_prefix ? a.n_prefix : a.n_q;
  const int64_t slot_stride = (int64_t)a.hkv * 2 * KV_BN * D;             // floats between consecutive chunks
  const float* slot0 = pl.slots + ((int64_t)item0 * a.hkv + kvh) * 2 * KV_BN * D;
#pragma unroll
  for (int u = 0; u < RED_PASSES; u++) {
    const int e = ((part * RED_PASSES + u) * RED_THREADS + threadIdx.x) * 4;
    const int key = e / D, d0 = e % D;
    if (key >= n_keys || k0 + key >= region) continue;
    f32x4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
    const float* base = slot0 + e;
    int c = 0;
    for (; c + 4 <= nc; c += 4) {                      // four chunks in flight; summed in chunk order
      f32x4 tk[4], tv[4];
#pragma unroll
      for (int i = 0; i < 4; i++) {
        tk[i] = __builtin_nontemporal_load((const f32x4*)(base + (c + i) * slot_stride));
        tv[i] = __builtin_nontemporal_load((const f32x4*)(base + (c + i) * slot_stride + KV_BN * D));
      }
#pragma unroll
      for (int i = 0; i < 4; i++) { sk += tk[i]; sv += tv[i]; }
    }
    for (; c < nc; c++) {
      sk += __builtin_nontemporal_load((const f32x4*)(base + c * slot_stride));
      sv += __builtin_nontemporal_load((const f32x4*)(base + c * slot_stride + KV_BN * D));
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
  int dev = 0, n_cu = 256;
  if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  // one resident workgroup per compute unit pulls work items until the counter runs out
  const int64_t max_work = (int64_t)pl.max_items * a.hkv;
  const unsigned grid = (unsigned)std::min<int64_t>(n_cu, max_work);
  {
    KernelTimer timer(TT_KERNEL_ATTN_PLAN, st);
    kv_plan_kernel<<<1, PLAN_THREADS, 0, st>>>(pl, a.kt_max, a.n_q, a.n_prefix, a.hq / a.hkv, a.hkv, (int)grid);
    if (hipError_t e = hipGetLastError()) return e;
  }
  if (hipError_t e = hipFuncSetAttribute((const void*)tree_attn_dkdv_kernel,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(KvSmem)))
    return e;
  {
    KernelTimer timer(TT_KERNEL_ATTN_DKDV, st);
    tree_attn_dkdv_kernel<<<grid, NTHREADS, sizeof(KvSmem), st>>>(a, pl);
    if (hipError_t e = hipGetLastError()) return e;
  }
  {
    KernelTimer timer(TT_KERNEL_ATTN_REDUCE, st);
    kv_reduce_kernel<<<dim3(pl.max_split_tiles * RED_PARTS, a.hkv), RED_THREADS, 0, st>>>(a, pl);
    if (hipError_t e = hipGetLastError()) return e;
  }
  return hipSuccess;
}

}  // namespace tt
