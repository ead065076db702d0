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
// All arithmetic here is plain fp32 (vector ALU, LDS-tiled products): a first, correct form of this pass.
//   gdn_prepare_kernel<true>   (tt_gdn.hip)  per (chunk, head): gamma, A0, P, U, W in fp32
//   gdn_bwd_fscan_kernel       (32 value columns, head): forward walk, saves S0 and Vn of every chunk
//   gdn_bwd_rscan_kernel       (32 value columns, head): reverse walk, saves dS1 and dVn of every chunk
//   gdn_bwd_finish_kernel      per (chunk, head): everything else; dq / dk per value head in fp32
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
  // per (head, chunk)
  float* s0;         // [128][128] state entering the chunk
  float* vn;         // [64][128]
  float* dvn;        // [64][128]
  float* ds1;        // [128][128] gradient of the state leaving the chunk
  float* x;          // [64][256]  [dW] on the way in, [dVb | dKb] after the transposed solve
  float* slots;      // [n_slots][hv][128][128] saved node-end states
  float* slot_grad;  // [n_slots][hv][128][128]
  float* dqh;        // [N][hv][128] per-value-head dq, dk
  float* dkh;
};
struct KArgs {
  GdnBwdArgs b;
  BwdWs w;
};

__device__ __forceinline__ void scan_ids(int id, int hv, int& h, int& dvb) {
  // consecutive ids go round-robin over the 8 XCDs; the four column blocks of a head share one
  if (hv % 8 == 0) { h = (id >> 5) * 8 + (id & 7); dvb = (id >> 3) & 3; }
  else             { h = id >> 2; dvb = id & 3; }
}

__device__ __forceinline__ float4 ld4(const float* p) { return *(const float4*)p; }
__device__ __forceinline__ void st4(float* p, const float (&v)[4]) { *(float4*)p = make_float4(v[0], v[1], v[2], v[3]); }

// fp32 matrix instruction: D (32 x 32) += A (32 x 2) B (2 x 32).  Lane l = 32 hf + c supplies A[row c][k = hf] and
// B[k = hf][column c] and holds D[(r / 4) * 8 + 4 hf + r % 4][c] in register r.
__device__ __forceinline__ f32x16 mfma_f32(float a, float b, f32x16 acc) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0); }
__device__ __forceinline__ int tile_row(int r, int hf) { return (r >> 2) * 8 + 4 * hf + (r & 3); }

// acc += sign A B over LK consecutive k (LK even).  `at` points at element (k = 0, this lane's row) of A stored
// [k][row] with pitch pa, `bm` at element (k = 0, this lane's column) of B stored [k][column] with pitch pb.  The
// instruction's two k-slots take k = s and k = LK / 2 + s.
template <int LK, bool NEG = false>
__device__ __forceinline__ void mfma_range(const float* at, int pa, const float* bm, int pb, int hf, f32x16& acc) {
#pragma unroll 8
  for (int s = 0; s < LK / 2; s++) {
    const int k = hf * (LK / 2) + s;
    const float av = at[k * pa];
    acc = mfma_f32(NEG ? -av : av, bm[k * pb], acc);
  }
}

// Barrier that waits for this wave's LDS traffic only: global stores (nobody in the workgroup reads them back)
// and the prefetch loads of the next chunk stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// The walks are software-pipelined: the operands of chunk i + 1 are fetched into registers while chunk i is
// computed and go to LDS at the top of the next step; the chunk's scalars are fetched per lane one step ahead as
// well (`z` is a per-lane zero the compiler cannot see through, which keeps them in vector registers until they
// are needed instead of waiting for them right behind the load).
struct WalkMeta {
  int tok0, len, src, dst, cap;
};
__device__ __forceinline__ WalkMeta load_walk_meta(const GdnBwdArgs& b, int chunk, int z, bool want_cap) {
  WalkMeta m;
  m.tok0 = b.chunk_tok0[chunk + z]; m.len = b.chunk_len[chunk + z]; m.src = b.chunk_src[chunk + z]; m.dst = b.chunk_dst[chunk + z];
  m.cap = want_cap ? b.chunk_cap[chunk + z] : -1;
  return m;
}
__device__ __forceinline__ WalkMeta uniform(const WalkMeta& m) {
  WalkMeta u;
  u.tok0 = __builtin_amdgcn_readfirstlane(m.tok0); u.len = __builtin_amdgcn_readfirstlane(m.len);
  u.src = __builtin_amdgcn_readfirstlane(m.src); u.dst = __builtin_amdgcn_readfirstlane(m.dst);
  u.cap = __builtin_amdgcn_readfirstlane(m.cap);
  return u;
}

// ---- forward walk ------------------------------------------------------------------------------------
// Wave w owns rows 32 w .. 32 w + 31 of the 128 x 32 state slice (accumulator layout).  The two 32 x 32 blocks of
// Vn are each computed by two waves, one per half of the contraction over the key dimension.
struct FwdStage {                 // one chunk's operands on their way to LDS
  f32x4 wt[(GD * GC / 4) / BT];      // native vector types: they stay in registers
  bf16x8 k[(GC * GD / 8) / BT];
  float gam[(GC * GD / 8) / BT];
  f32x4 u[(GC * DVB / 4) / BT];
  float glast;
};
__device__ __forceinline__ void fwd_fetch(const KArgs& a, int chunk, int h, int dvb, const __bf16* kb, size_t krow, int tid, int z,
                                          FwdStage& st) {
  const size_t op = (size_t)h * a.b.n_chunks + chunk;
  const int tok0 = a.b.chunk_tok0[chunk + z], len = a.b.chunk_len[chunk + z];
  const float* gam = a.w.ops.gam + op * GC;
  const f32x4* wsrc = (const f32x4*)(a.w.ops.wt + op * (GD * GC));
#pragma unroll
  for (int p = 0; p < (GD * GC / 4) / BT; p++) st.wt[p] = wsrc[tid + p * BT];
#pragma unroll
  for (int p = 0; p < (GC * GD / 8) / BT; p++) {
    const int piece = tid + p * BT, i = piece >> 4, c8 = (piece & 15) * 8;
    st.k[p] = *(const bf16x8*)(kb + (size_t)(tok0 + min(i, len - 1)) * krow + c8);
    st.gam[p] = i < len ? gam[i] : 1e30f;                  // exp(glast - 1e30) = 0: rows past the chunk's length
  }
  const float* u = a.w.ops.u + op * (GC * GD) + dvb * DVB;
#pragma unroll
  for (int p = 0; p < (GC * DVB / 4) / BT; p++) {
    const int piece = tid + p * BT, i = piece >> 3, c4 = (piece & 7) * 4;
    st.u[p] = *(const f32x4*)(u + (size_t)i * GD + c4);
  }
  st.glast = gam[GC - 1 + z];
}

__global__ __launch_bounds__(BT, 1) void gdn_bwd_fscan_kernel(KArgs a) {
  __shared__ __attribute__((aligned(16))) float wt[GD * GC];      // W^T [d][i]
  __shared__ __attribute__((aligned(16))) float kd[GC * GD];      // Kd  [i][d]
  __shared__ __attribute__((aligned(16))) float us[GC * DVB];     // U   [i][c]
  __shared__ __attribute__((aligned(16))) float ss[GD * DVB];     // S0  [d][c]
  __shared__ __attribute__((aligned(16))) float vs[GC * DVB];     // Vn  [i][c]
  __shared__ float half2nd[2][32 * DVB];                          // W S0 over the second half of the key dims
  int h, dvb;
  scan_ids(blockIdx.x, a.b.hv, h, dvb);
  const int tid = threadIdx.x & (BT - 1), lane = tid & 63, c = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), ib = w & 1, kq = w >> 1;
  const int nc = a.b.n_chunks, hv = a.b.hv, kh = h / (hv / a.b.hk);
  const __bf16* kb = (const __bf16*)a.b.k + (size_t)kh * GD;
  const size_t krow = (size_t)a.b.hk * GD;
  const size_t col = (size_t)dvb * DVB + c;                   // this lane's column inside a [128][128] state
  f32x16 s = zero16();
  int z = 0;
  asm volatile("" : "+v"(z));

  FwdStage st;
  fwd_fetch(a, 0, h, dvb, kb, krow, tid, z, st);
  WalkMeta next = load_walk_meta(a.b, 0, z, false);
  for (int chunk = 0; chunk < nc; chunk++) {
    const WalkMeta m = uniform(next);
    const size_t op = (size_t)h * nc + chunk;
    if (m.src != -2) {
      const float* sp = m.src >= 0 ? a.w.slots + ((size_t)m.src * hv + h) * (GD * GD) : a.b.initial_state ? a.b.initial_state + (size_t)h * (GD * GD) : nullptr;
#pragma unroll
      for (int r = 0; r < 16; r++) s[r] = sp ? sp[(size_t)(32 * w + tile_row(r, hf)) * GD + col] : 0.f;
    }
#pragma unroll
    for (int r = 0; r < 16; r++) ss[(32 * w + tile_row(r, hf)) * DVB + c] = s[r];
    const float glast = st.glast;
#pragma unroll
    for (int p = 0; p < (GD * GC / 4) / BT; p++) ((f32x4*)wt)[tid + p * BT] = st.wt[p];
#pragma unroll
    for (int p = 0; p < (GC * GD / 8) / BT; p++) {
      const int piece = tid + p * BT, i = piece >> 4, c8 = (piece & 15) * 8;
      const float f = __expf(glast - st.gam[p]);
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] = (float)st.k[p][e] * f;
      *(float4*)&kd[i * GD + c8] = make_float4(o[0], o[1], o[2], o[3]);
      *(float4*)&kd[i * GD + c8 + 4] = make_float4(o[4], o[5], o[6], o[7]);
    }
#pragma unroll
    for (int p = 0; p < (GC * DVB / 4) / BT; p++) ((f32x4*)us)[tid + p * BT] = st.u[p];
    lds_barrier();

    // next chunk's operands and scalars on their way (the last step re-fetches its own: no branch around loads)
    const int nxt = min(chunk + 1, nc - 1);
    fwd_fetch(a, nxt, h, dvb, kb, krow, tid, z, st);
    next = load_walk_meta(a.b, nxt, z, false);
    {   // the entering state, for the finish kernel: 16-byte stores from the LDS copy
      float* s0 = a.w.s0 + op * (GD * GD) + dvb * DVB;
#pragma unroll
      for (int p = 0; p < (GD * DVB / 4) / BT; p++) {
        const int piece = tid + p * BT, d = piece >> 3, c4 = (piece & 7) * 4;
        *(float4*)(s0 + (size_t)d * GD + c4) = *(const float4*)&ss[d * DVB + c4];
      }
    }

    // Vn = U - W S0: rows 32 ib .., key dims 64 kq .. 64 kq + 63
    f32x16 part = zero16();
    mfma_range<64>(wt + (64 * kq) * GC + 32 * ib + c, GC, ss + (64 * kq) * DVB + c, DVB, hf, part);
    if (kq == 1) {
#pragma unroll
      for (int r = 0; r < 16; r++) half2nd[ib][tile_row(r, hf) * DVB + c] = part[r];
    }
    lds_barrier();
    if (kq == 0) {
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int i = 32 * ib + tile_row(r, hf);
        vs[i * DVB + c] = us[i * DVB + c] - (part[r] + half2nd[ib][tile_row(r, hf) * DVB + c]);
      }
    }
    lds_barrier();
    {
      float* vout = a.w.vn + op * (GC * GD) + dvb * DVB;
#pragma unroll
      for (int p = 0; p < (GC * DVB / 4) / BT; p++) {
        const int piece = tid + p * BT, i = piece >> 3, c4 = (piece & 7) * 4;
        *(float4*)(vout + (size_t)i * GD + c4) = *(const float4*)&vs[i * DVB + c4];
      }
    }

    // S1 = EL S0 + Kd^T Vn
    const float el_last = __expf(glast);
#pragma unroll
    for (int r = 0; r < 16; r++) s[r] *= el_last;
    mfma_range<GC>(kd + 32 * w + c, GD, vs + c, DVB, hf, s);
    if (m.dst >= 0) {
      float* sp = a.w.slots + ((size_t)m.dst * hv + h) * (GD * GD) + col;
#pragma unroll
      for (int r = 0; r < 16; r++) sp[(size_t)(32 * w + tile_row(r, hf)) * GD] = s[r];
    }
    lds_barrier();         // the LDS arrays are rewritten by the next chunk
  }
}

// ---- reverse walk ------------------------------------------------------------------------------------
struct RevStage {
  f32x4 kdt[(GD * GC / 4) / BT], w[(GC * GD / 4) / BT], p[(GC * GC / 4) / BT];
  bf16x8 q[(GC * GD / 8) / BT];
  float gam[(GC * GD / 8) / BT];
  bf16x8 d_o;
  float glast;
};
__device__ __forceinline__ void rev_fetch(const KArgs& a, int chunk, int h, const __bf16* qb, size_t qrow, const __bf16* dob, size_t vrow,
                                          int tid, int z, RevStage& st) {
  const size_t op = (size_t)h * a.b.n_chunks + chunk;
  const int tok0 = a.b.chunk_tok0[chunk + z], len = a.b.chunk_len[chunk + z];
  const float* gam = a.w.ops.gam + op * GC;
  const f32x4* ksrc = (const f32x4*)(a.w.ops.kdt + op * (GD * GC));
  const f32x4* wsrc = (const f32x4*)(a.w.ops.w + op * (GC * GD));
  const f32x4* psrc = (const f32x4*)(a.w.ops.p + op * (GC * GC));
#pragma unroll
  for (int p = 0; p < (GD * GC / 4) / BT; p++) {
    st.kdt[p] = ksrc[tid + p * BT];
    st.w[p] = wsrc[tid + p * BT];
  }
#pragma unroll
  for (int p = 0; p < (GC * GC / 4) / BT; p++) st.p[p] = psrc[tid + p * BT];
#pragma unroll
  for (int p = 0; p < (GC * GD / 8) / BT; p++) {
    const int piece = tid + p * BT, i = piece >> 4, c8 = (piece & 15) * 8;
    st.q[p] = *(const bf16x8*)(qb + (size_t)(tok0 + min(i, len - 1)) * qrow + c8);
    st.gam[p] = i < len ? gam[i] : -1e30f;                 // exp(-1e30) = 0: rows past the chunk's length
  }
  {
    const int i = tid >> 2, c8 = (tid & 3) * 8;            // 64 rows x 4 pieces of 8 columns
    const bf16x8 dv = *(const bf16x8*)(dob + (size_t)(tok0 + min(i, len - 1)) * vrow + c8);
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; e++) zero[e] = (__bf16)0.f;
    st.d_o = i < len ? dv : zero;
  }
  st.glast = gam[GC - 1 + z];
}

__global__ __launch_bounds__(BT, 1) void gdn_bwd_rscan_kernel(KArgs a) {
  __shared__ __attribute__((aligned(16))) float kdt[GD * GC];     // Kd^T [d][i]
  __shared__ __attribute__((aligned(16))) float qg[GC * GD];      // Qg   [i][d]
  __shared__ __attribute__((aligned(16))) float wr[GC * GD];      // W    [i][d]
  __shared__ __attribute__((aligned(16))) float pm[GC * GC];      // P    [j][i]
  __shared__ __attribute__((aligned(16))) float dos[GC * DVB];    // dO   [i][c]
  __shared__ __attribute__((aligned(16))) float dvs[GC * DVB];    // dVn  [i][c]
  __shared__ __attribute__((aligned(16))) float dss[GD * DVB];    // dS1  [d][c]
  __shared__ float half2nd[2][32 * DVB];
  int h, dvb;
  scan_ids(blockIdx.x, a.b.hv, h, dvb);
  const int tid = threadIdx.x & (BT - 1), lane = tid & 63, c = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), ib = w & 1, kq = w >> 1;
  const int nc = a.b.n_chunks, hv = a.b.hv, kh = h / (hv / a.b.hk);
  const __bf16* qb = (const __bf16*)a.b.q + (size_t)kh * GD;
  const size_t qrow = (size_t)a.b.hk * GD;
  const __bf16* dob = (const __bf16*)a.b.d_o + (size_t)h * GD + dvb * DVB;
  const size_t vrow = (size_t)hv * GD;
  const size_t col = (size_t)dvb * DVB + c;
  const bool want_cap = a.b.chunk_cap && a.b.d_state_out;
  f32x16 ds = zero16();
  int z = 0;
  asm volatile("" : "+v"(z));

  RevStage st;
  rev_fetch(a, nc - 1, h, qb, qrow, dob, vrow, tid, z, st);
  WalkMeta next = load_walk_meta(a.b, nc - 1, z, want_cap);
  int later_src = -1;                       // source of the chunk after this one in DFS order (handled one step earlier)
  for (int chunk = nc - 1; chunk >= 0; chunk--) {
    const WalkMeta m = uniform(next);
    const size_t op = (size_t)h * nc + chunk;

    // gradient of the state leaving this chunk
    if (later_src != -2) ds = zero16();     // nobody took this chunk's end state on chip
    later_src = m.src;
    if (m.dst >= 0) {
      float* sg = a.w.slot_grad + ((size_t)m.dst * hv + h) * (GD * GD) + col;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        float* e = sg + (size_t)(32 * w + tile_row(r, hf)) * GD;
        ds[r] += *e;
        *e = 0.f;                                   // the slot is reused by an earlier node
      }
    }
    if (m.cap >= 0) {
      const float* up = a.b.d_state_out + ((size_t)m.cap * hv + h) * (GD * GD) + col;
#pragma unroll
      for (int r = 0; r < 16; r++) ds[r] += up[(size_t)(32 * w + tile_row(r, hf)) * GD];
    }
#pragma unroll
    for (int r = 0; r < 16; r++) dss[(32 * w + tile_row(r, hf)) * DVB + c] = ds[r];
    const float glast = st.glast;
#pragma unroll
    for (int p = 0; p < (GD * GC / 4) / BT; p++) {
      ((f32x4*)kdt)[tid + p * BT] = st.kdt[p];
      ((f32x4*)wr)[tid + p * BT] = st.w[p];
    }
#pragma unroll
    for (int p = 0; p < (GC * GC / 4) / BT; p++) ((f32x4*)pm)[tid + p * BT] = st.p[p];
#pragma unroll
    for (int p = 0; p < (GC * GD / 8) / BT; p++) {
      const int piece = tid + p * BT, i = piece >> 4, c8 = (piece & 15) * 8;
      const float f = a.b.scale * __expf(st.gam[p]);
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] = (float)st.q[p][e] * f;
      *(float4*)&qg[i * GD + c8] = make_float4(o[0], o[1], o[2], o[3]);
      *(float4*)&qg[i * GD + c8 + 4] = make_float4(o[4], o[5], o[6], o[7]);
    }
    {
      const int i = tid >> 2, c8 = (tid & 3) * 8;
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] = (float)st.d_o[e];
      *(float4*)&dos[i * DVB + c8] = make_float4(o[0], o[1], o[2], o[3]);
      *(float4*)&dos[i * DVB + c8 + 4] = make_float4(o[4], o[5], o[6], o[7]);
    }
    lds_barrier();

    const int nxt = max(chunk - 1, 0);
    rev_fetch(a, nxt, h, qb, qrow, dob, vrow, tid, z, st);
    next = load_walk_meta(a.b, nxt, z, want_cap);
    {
      float* ds1 = a.w.ds1 + op * (GD * GD) + dvb * DVB;
#pragma unroll
      for (int p = 0; p < (GD * DVB / 4) / BT; p++) {
        const int piece = tid + p * BT, d = piece >> 3, c4 = (piece & 7) * 4;
        *(float4*)(ds1 + (size_t)d * GD + c4) = *(const float4*)&dss[d * DVB + c4];
      }
    }

    // dVn = P^T dO + Kd dS1, rows 32 ib ..; the contraction (64 tokens + 128 key dims) is split in two halves of 96
    f32x16 part = zero16();
    if (kq == 0) {
      mfma_range<GC>(pm + 32 * ib + c, GC, dos + c, DVB, hf, part);
      mfma_range<32>(kdt + 32 * ib + c, GC, dss + c, DVB, hf, part);
    } else {
      mfma_range<96>(kdt + 32 * GC + 32 * ib + c, GC, dss + 32 * DVB + c, DVB, hf, part);
#pragma unroll
      for (int r = 0; r < 16; r++) half2nd[ib][tile_row(r, hf) * DVB + c] = part[r];
    }
    lds_barrier();
    if (kq == 0) {
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int i = 32 * ib + tile_row(r, hf);
        dvs[i * DVB + c] = part[r] + half2nd[ib][tile_row(r, hf) * DVB + c];
      }
    }
    lds_barrier();
    {
      float* dvout = a.w.dvn + op * (GC * GD) + dvb * DVB;
#pragma unroll
      for (int p = 0; p < (GC * DVB / 4) / BT; p++) {
        const int piece = tid + p * BT, i = piece >> 3, c4 = (piece & 7) * 4;
        *(float4*)(dvout + (size_t)i * GD + c4) = *(const float4*)&dvs[i * DVB + c4];
      }
    }

    // dS0 = EL dS1 + Qg^T dO - W^T dVn
    const float el_last = __expf(glast);
#pragma unroll
    for (int r = 0; r < 16; r++) ds[r] *= el_last;
    mfma_range<GC>(qg + 32 * w + c, GD, dos + c, DVB, hf, ds);
    mfma_range<GC, true>(wr + 32 * w + c, GD, dvs + c, DVB, hf, ds);
    if (m.src >= 0 || (m.src == -1 && a.b.d_initial_state)) {
      float* sg = (m.src >= 0 ? a.w.slot_grad + ((size_t)m.src * hv + h) * (GD * GD) : a.b.d_initial_state + (size_t)h * (GD * GD)) + col;
#pragma unroll
      for (int r = 0; r < 16; r++) sg[(size_t)(32 * w + tile_row(r, hf)) * GD] += ds[r];
    }
    lds_barrier();
  }
}

// ---- per-chunk finish ----------------------------------------------------------------------------------
// acc[r][c] += sum_k fa(i, k) fb(k, j) for i = ty TM + r, j = tx + c (N / TN), over K (a multiple of KS), through
// LDS slabs of KS k-values.  AKF / BKF: consecutive threads fetch consecutive k (operand stored with k
// contiguous) rather than consecutive i / j.  Every thread of the workgroup must call it.
template <int M, int N, int TM, int TN, bool AKF, bool BKF, class FA, class FB>
__device__ __forceinline__ void slab_product(int K, FA fa, FB fb, float (&acc)[TM][TN], float* as, float* bs, int tid) {
  constexpr int NT = N / TN;
  static_assert((M / TM) * NT == BT, "one output tile per thread");
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
      as[kk * (M + 1) + i] = av[p];
    }
#pragma unroll
    for (int p = 0; p < N * KS / BT; p++) {
      const int e = tid + p * BT;
      const int kk = BKF ? e % KS : e / N, j = BKF ? e / KS : e % N;
      bs[kk * (N + 1) + j] = bv[p];
    }
    __syncthreads();
#pragma unroll 8
    for (int kk = 0; kk < KS; kk++) {
      float ar[TM], bc[TN];
#pragma unroll
      for (int r = 0; r < TM; r++) ar[r] = as[kk * (M + 1) + ty * TM + r];
#pragma unroll
      for (int c = 0; c < TN; c++) bc[c] = bs[kk * (N + 1) + tx + c * NT];
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
  __shared__ float as[KS * (GC + 1)];
  __shared__ float bs[GC * AP > KS * (GD + 1) ? GC * AP : KS * (GD + 1)];   // between products also: dA o A0
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
  const float* S0 = a.w.s0 + op * (GD * GD);
  const float* Vn = a.w.vn + op * (GC * GD);
  const float* dVn = a.w.dvn + op * (GC * GD);
  const float* dS1 = a.w.ds1 + op * (GD * GD);
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
    slab_product<GC, GD, 4, 8, true, true>(GD, [&](int i, int k) { return dVn[i * GD + k]; },
                                           [&](int k, int j) { return S0[j * GD + k]; }, acc, as, bs, tid);
    const int tx = tid & 15, ty = tid >> 4;
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 8; c++) X[(ty * 4 + r) * (2 * GD) + GD + tx + c * 16] = -acc[r][c];
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
    const float* rhs = c < GD ? dVn + c : X + c;
    const int pitch = c < GD ? GD : 2 * GD;
#pragma unroll
    for (int i = 0; i < GC; i++) x[i] = rhs[(size_t)i * pitch];
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
        const int i = ty * 4 + r, j = tx + c * 16;
        dam[i * AP + j] = i > j ? -acc[r][c] : 0.f;
      }
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 4; c++) acc[r][c] = 0.f;
    slab_product<GC, GC, 4, 4, true, true>(GD, do_at, [&](int k, int j) { return Vn[j * GD + k]; }, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int c = 0; c < 4; c++) {
        const int i = ty * 4 + r, j = tx + c * 16;
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
    slab_product<GC, GD, 4, 8, true, true>(GD, do_at, [&](int k, int j) { return S0[j * GD + k]; }, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int i = ty * 4 + r;
      const float f = scale * eg[i];
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < 8; c++) {
        acc[r][c] *= f;                               // dQg_i scaled = its contribution to dq_i
        dot += acc[r][c] * q_at(i, tx + c * 16);      // dQg_i . Qg_i = (scale eg dQg_i) . q_i
      }
      dot = row16_sum(dot);
      if (tx == 0) dg_q[i] = dot;
    }
    slab_product<GC, GD, 4, 8, true, false>(GC, [&](int i, int k) { return dpm[i * AP + k]; }, k_at, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int i = ty * 4 + r;
      if (i < len) {
        float* dst = a.w.dqh + ((size_t)(tok0 + i) * hv + h) * GD + tx;
#pragma unroll
        for (int c = 0; c < 8; c++) dst[c * 16] = acc[r][c];
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
    slab_product<GC, GD, 4, 8, true, true>(GD, [&](int i, int k) { return Vn[i * GD + k]; },
                                           [&](int k, int j) { return dS1[j * GD + k]; }, acc, as, bs, tid);
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int i = ty * 4 + r;
      const float fe = el[i], fb_ = bet[i] * eg[i];
      float dot_kd = 0.f, dot_kb = 0.f;
#pragma unroll
      for (int c = 0; c < 8; c++) {
        const int d = tx + c * 16;
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
        float* dst = a.w.dkh + ((size_t)(tok0 + i) * hv + h) * GD + tx;
#pragma unroll
        for (int c = 0; c < 8; c++) dst[c * 16] = acc[r][c];
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
    for (int p = 0; p < (GD * GD / 4) / BT; p++) {
      const float4 x = ld4(dS1 + 4 * (tid + p * BT)), y = ld4(S0 + 4 * (tid + p * BT));
      s += x.x * y.x + x.y * y.y + x.z * y.z + x.w * y.w;
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
  auto take = [&](size_t floats) {
    float* r = p ? (float*)(p + off) : nullptr;
    off += align256(floats * 4);
    return r;
  };
  BwdWs t{};
  t.ops.gam = take(per * GC);
  t.ops.a0 = take(per * GC * GC);
  t.ops.p = take(per * GC * GC);
  t.ops.u = take(per * GC * GD);
  t.ops.w = take(per * GC * GD);
  t.ops.wt = take(per * GC * GD);
  t.ops.kdt = take(per * GC * GD);
  t.s0 = take(per * GD * GD);
  t.vn = take(per * GC * GD);
  t.dvn = take(per * GC * GD);
  t.ds1 = take(per * GD * GD);
  t.x = take(per * GC * 2 * GD);
  t.slots = take((size_t)n_slots * hv * GD * GD);
  t.slot_grad = take((size_t)n_slots * hv * GD * GD);
  t.dqh = take((size_t)n_tokens * hv * GD);
  t.dkh = take((size_t)n_tokens * hv * GD);
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
  zero(a.w.slot_grad, (size_t)b.n_slots * b.hv * GD * GD);
  if (b.d_initial_state) zero(b.d_initial_state, (size_t)b.hv * GD * GD);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  if (hipError_t e = gdn_prepare_f32(b.n_tokens, b.hk, b.hv, b.scale, b.q, b.k, b.v, b.g, b.beta, b.n_chunks, b.chunk_tok0, b.chunk_len,
                                     a.w.ops, st);
      e != hipSuccess)
    return e;
  {
    KernelTimer t(TT_KERNEL_GDN_BWD_FSCAN, st);
    gdn_bwd_fscan_kernel<<<dim3((GD / DVB) * b.hv), BT, 0, st>>>(a);
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  {
    KernelTimer t(TT_KERNEL_GDN_BWD_RSCAN, st);
    gdn_bwd_rscan_kernel<<<dim3((GD / DVB) * b.hv), BT, 0, st>>>(a);
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
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
