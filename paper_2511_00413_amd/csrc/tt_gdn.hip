// Gated delta rule with tree state routing, forward (Section "Implementation", paragraph "SSM Layers
// (GDN)" (i); Appendix "Tree-Aware SSM State Routing"): the recurrent state at a node's first token
// is the end state of its parent node, not of the previous node in DFS order.
//
// Chunked form, 64 tokens per chunk, chunks never cross a node boundary.  With gamma_i the running
// sum of the log-decays inside a chunk, beta the write strengths and S0 the state entering the chunk:
//     A  = strictly-lower( beta_i (k_i . k_j) exp(gamma_i - gamma_j) )
//     U  = (I + A)^-1 (beta * V)                 W = (I + A)^-1 (beta * exp(gamma) * K)
//     Vn = U - W S0
//     O  = scale (Q * exp(gamma)) S0 + scale tril( (Q K^T) * exp(gamma_i - gamma_j) ) Vn
//     S1 = exp(gamma_last) S0 + (K * exp(gamma_last - gamma))^T Vn
// which is the token recurrence  S <- e^g S + beta k (v - (e^g S)^T k)^T,  o = scale S^T q  written
// per chunk.  Two kernels:
//   gdn_prepare_kernel  (chunk, value head): everything that does not depend on S0 -- K K^T and
//       Q K^T on MFMA, the inverse T = (I + A)^-1 by forward substitution on the identity (one wave, one
//       lane per column, no synchronisation inside), U and W as products with T on MFMA, operands
//       written in the layouts the second kernel's MFMA fragments want;
//   gdn_scan_kernel  (64 value columns, value head): walks the chunks in DFS order with the state
//       in MFMA accumulators (the columns of S evolve independently, so a head is cut into four
//       independent blocks of 32 columns, four wavefronts each; two blocks form a workgroup and share
//       the LDS copy of the chunk's operands); state routing = where a chunk takes S0 from (registers when it
//       continues the previous chunk's sequence, a saved node-end state, or zero).
// The backward pass (tt_gdn_bwd.hip) reuses both: the prepare kernel in a form that also writes the reverse walk's
// operands, the scan in a form that saves every chunk's entering state and Vn instead of writing the output, and
// gdn_rscan_kernel, the reverse walk, built like the scan.
#include <hip/hip_runtime.h>
#include "tt_internal.h"
#include "tt_kernels.h"
#include "tt_mfma.h"

namespace tt {
namespace {

constexpr int GC = TT_GDN_CHUNK;     // tokens per chunk (64)
constexpr int GD = 128;              // head dim of keys and values
constexpr int GROW = GD + 8;         // padded LDS row (elements) for [*][128] bf16 tiles
constexpr int G_THREADS = 256;
constexpr int T_PITCH = GC + 8;      // padded LDS row (elements) of the 64 x 64 bf16 halves of the triangular inverse
constexpr int AM_PITCH = GC + 4;     // LDS row (floats) of A: rows 16-byte aligned, a column of 32 rows spreads over 16 banks
static_assert(2 * GC * T_PITCH * 2 >= GC * AM_PITCH * 4, "the inverse's halves take the place of A");
constexpr int G_DVB = 32;            // value columns per column block of the scan (one 32 x 32 accumulator tile per wave)
constexpr int SCAN_NB = 2;           // column blocks per scan workgroup: 4 wavefronts each, sharing the chunk's operands in LDS
constexpr int SCAN_NW = 4 * SCAN_NB; // wavefronts per scan workgroup (two per SIMD)
constexpr int SCAN_THREADS = 64 * SCAN_NW;

struct GdnArgs {
  int n_tokens, hk, hv, n_chunks;    // hk, hv: heads of the tensors (their strides)
  int hv_n;                          // value heads this launch works on (h = 0 .. hv_n - 1 relative to the pointers below)
  float scale;
  const __bf16 *q, *k, *v;           // [N][hk][128], [N][hk][128], [N][hv][128]
  const float *g, *beta;             // [N][hv]
  const int32_t *chunk_tok0, *chunk_len, *chunk_src, *chunk_dst;
  const int32_t* chunk_cap;          // nullptr, or per chunk: -1 / index into state_out
  const int32_t *seg_chunk0, *seg_chunk1;   // nullptr (one segment: all chunks), or the chunk ranges of the segments
  int seg_base;                      // first segment of the level this launch walks (blockIdx.y counts from it)
  const float* initial_state;        // nullptr (zero) or [hv][128][128]: the state roots start from
  float* state_out;                  // [n_capture][hv][128][128]
  __bf16* o;                         // [N][hv][128]
  // per (chunk, value head) operands
  __bf16* rec;                       // records of REC_ELEMS: -W [64][128], U^T [128][64], scale Q exp(gamma) [64][128],
                                     // (K exp(gamma_last - gamma))^T [128][64], scale tril((Q K^T) exp(gamma_i - gamma_j)) [64][64]
  float* glast;                      // exp(gamma_last)
  float* slots;                      // [n_slots][hv][128][128] saved node-end states
  // backward pass only
  GdnChunkOps f32;                   // unrounded per-chunk quantities for the finish kernel
  const __bf16* d_o;                 // [N][hv][128]
  __bf16* rev;                       // records of REV_ELEMS for the reverse walk (see REV_*)
  __bf16* s0t;                       // per (head, chunk): entering state transposed [128 value cols][128 key dims]
  __bf16* vns;                       // per (head, chunk): Vn as B-operand fragments [4 col blocks][2 row blocks][2][64 lanes][8]
  __bf16* ds1t;                      // gradient of the leaving state, transposed like s0t
  __bf16* dvns;                      // dVn, fragments like vns
  float* slot_grad;                  // [n_slots][hv][128][128] gradients of the saved states (walk in sequence order)
  float* seg_grad;                   // [n_segments][hv][128][128] gradient of the state a segment started from (scheduled walk)
  const int32_t *slot_cons_off, *slot_cons;   // scheduled walk: the segments that start from every slot
  const float* d_state_out;          // nullptr or [n_capture][hv][128][128]
  float* d_initial_state;            // nullptr or [hv][128][128] (zeroed by the caller)
};

// The operands of one (head, chunk) form one contiguous record, records ordered head-major: a scan
// workgroup (one head) then streams through memory front to back -- consecutive chunks are
// adjacent, so address translation and DRAM pages are reused instead of missed on every step.
constexpr size_t REC_WN = 0, REC_UT = GC * GD, REC_QG = 2 * GC * GD, REC_KDT = 3 * GC * GD, REC_P = 4 * GC * GD;
constexpr size_t REC_ELEMS = 4 * GC * GD + GC * GC;      // bf16 elements per record (72 KB)
// Record of the reverse walk: Kd = K exp(gamma_last - gamma) [64][128], -W^T [128][64], (scale Q exp(gamma))^T
// [128][64], P^T [64][64], dO^T [128 value cols][64]
constexpr size_t REV_KD = 0, REV_WTN = GC * GD, REV_QGT = 2 * GC * GD, REV_PT = 3 * GC * GD, REV_DOT = 3 * GC * GD + GC * GC;
constexpr size_t REV_ELEMS = 4 * GC * GD + GC * GC;
static_assert(REC_ELEMS == GDN_REC_ELEMS && REV_ELEMS == GDN_REC_ELEMS && REC_UT == GDN_REC_UT && REV_WTN == GDN_REV_WTN,
              "record layout shared with the finish kernel");
__device__ __forceinline__ size_t op_index(const GdnArgs& a, int chunk, int h) { return (size_t)h * a.n_chunks + chunk; }

// BWD: additionally the unrounded quantities the backward's finish kernel reads (GdnChunkOps) and the reverse
// walk's record.
template <bool BWD>
__global__ __launch_bounds__(G_THREADS) void gdn_prepare_kernel(GdnArgs a) {
  __shared__ __attribute__((aligned(16))) __bf16 ksm[GC][GROW];
  __shared__ __attribute__((aligned(16))) __bf16 qsm[GC][GROW];
  // A (fp32) until the triangular inverse has been formed from it, then the two bf16 halves of the scaled inverse
  __shared__ __attribute__((aligned(16))) float am_raw[2 * GC * T_PITCH / 2];
  float(*am)[AM_PITCH] = (float(*)[AM_PITCH])am_raw;
  __bf16(*t_hi)[T_PITCH] = (__bf16(*)[T_PITCH])am_raw;
  __bf16(*t_lo)[T_PITCH] = t_hi + GC;
  __shared__ float gam[GC], bet[GC];

  int chunk, h;
  if (!gdn_group_order(blockIdx.x, a.n_chunks, a.hv_n, a.hv / a.hk, chunk, h)) return;
  const int hkv = h / (a.hv / a.hk);
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int tok0 = a.chunk_tok0[chunk], len = a.chunk_len[chunk];
  const size_t op = op_index(a, chunk, h);

  // Every row load of the chunk is issued here, in one straight-line block (K, Q, V -- and dO in the backward
  // form -- as four 16-byte pieces per thread each), so that the trips to memory overlap each other and the scan
  // below.  Rows past the chunk's length read the last valid row and are zeroed on their way into LDS.  (Loaded
  // piece by piece inside the staging loops, behind a row-in-range branch, every piece is waited for in turn.)
  constexpr int NPIECE = GC * (GD / 8) / G_THREADS;
  bf16x8 kreg[NPIECE], qreg[NPIECE], vreg[NPIECE];
  [[maybe_unused]] bf16x8 doreg[NPIECE];
#pragma unroll
  for (int p = 0; p < NPIECE; p++) {
    const int piece = tid + p * G_THREADS, i = piece >> 4, c8 = (piece & 15) * 8;
    const size_t row = (size_t)(tok0 + min(i, len - 1));
    kreg[p] = *(const bf16x8*)(a.k + (row * a.hk + hkv) * GD + c8);
    qreg[p] = *(const bf16x8*)(a.q + (row * a.hk + hkv) * GD + c8);
    vreg[p] = *(const bf16x8*)(a.v + (row * a.hv + h) * GD + c8);
    if constexpr (BWD) doreg[p] = *(const bf16x8*)(a.d_o + (row * a.hv + h) * GD + c8);
  }
  bf16x8 zero8;
#pragma unroll
  for (int e = 0; e < 8; e++) zero8[e] = (__bf16)0.f;

  if (tid < GC) {
    // running sum of the log-decays over the chunk: a parallel scan inside the first wave
    const bool in = tid < len;
    float run = in ? a.g[(size_t)(tok0 + tid) * a.hv + h] : 0.f;
    bet[tid] = in ? a.beta[(size_t)(tok0 + tid) * a.hv + h] : 0.f;
#pragma unroll
    for (int d = 1; d < GC; d <<= 1) {
      const float up = __shfl_up(run, d);
      if (tid >= d) run += up;
    }
    gam[tid] = run;
    if (tid == GC - 1) a.glast[op] = __expf(run);
  }
  __syncthreads();
  const float g_last = gam[GC - 1];
  if constexpr (BWD) {
    if (tid < GC) a.f32.gam[op * GC + tid] = gam[tid];
  }

  // K and Q rows into LDS (zero rows past the chunk's length); Qg written on the way
#pragma unroll
  for (int p = 0; p < NPIECE; p++) {
    const int piece = tid + p * G_THREADS, i = piece >> 4, c8 = (piece & 15) * 8;
    const bf16x8 kv = i < len ? kreg[p] : zero8, qv = i < len ? qreg[p] : zero8;
    *(bf16x8*)&ksm[i][c8] = kv;
    *(bf16x8*)&qsm[i][c8] = qv;
    if constexpr (!BWD) *(bf16x8*)(a.rec + op * REC_ELEMS + REC_QG + i * GD + c8) = scale_frag(qv, a.scale * __expf(gam[i]));
    if constexpr (BWD) *(bf16x8*)(a.rev + op * REV_ELEMS + REV_KD + i * GD + c8) = scale_frag(kv, __expf(g_last - gam[i]));
  }
  __syncthreads();

  // K K^T and Q K^T, one 32x32 tile per wave; the tile above the diagonal is not needed
  {
    const int ib = w >> 1, jb = w & 1;
    const int c = lane & 31, hf = lane >> 5;
    if (jb <= ib) {
      f32x16 kk = zero16(), qk = zero16();
      [[maybe_unused]] f32x16 kq = zero16();      // BWD: (Q K^T)^T formed as K Q^T, so that P^T too is stored along its rows
#pragma unroll
      for (int ks = 0; ks < GD / 16; ks++) {
        const bf16x8 kj = *(const bf16x8*)&ksm[jb * 32 + c][ks * 16 + hf * 8];
        const bf16x8 ki = *(const bf16x8*)&ksm[ib * 32 + c][ks * 16 + hf * 8];
        const bf16x8 qi = *(const bf16x8*)&qsm[ib * 32 + c][ks * 16 + hf * 8];
        kk = mfma32(ki, kj, kk);
        qk = mfma32(qi, kj, qk);
        if constexpr (BWD) kq = mfma32(kj, qi, kq);
      }
      const int j = jb * 32 + c;
      __bf16* pout = a.rec + op * REC_ELEMS + REC_P;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int i = ib * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
        const float dec = j <= i ? __expf(gam[i] - gam[j]) : 0.f;
        const float a0 = j < i ? kk[r] * dec : 0.f;
        am[i][j] = bet[i] * a0;
        if constexpr (BWD) {
          a.f32.a0[op * (GC * GC) + i * GC + j] = a0;
          a.f32.p[op * (GC * GC) + i * GC + j] = a.scale * qk[r] * dec;
          // element (row jt, column it) of the transposed tile: key token jt, query token it
          const int jt = jb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3), it = ib * 32 + c;
          a.rev[op * REV_ELEMS + REV_PT + jt * GC + it] = (__bf16)(jt <= it ? a.scale * kq[r] * __expf(gam[it] - gam[jt]) : 0.f);
        } else {
          pout[i * GC + j] = (__bf16)(a.scale * qk[r] * dec);
        }
      }
    } else {
      const int j = jb * 32 + c;
      __bf16* pout = a.rec + op * REC_ELEMS + REC_P;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int i = ib * 32 + (r >> 2) * 8 + hf * 4 + (r & 3);
        am[i][j] = 0.f;
        if constexpr (BWD) {
          a.f32.a0[op * (GC * GC) + i * GC + j] = 0.f;
          a.f32.p[op * (GC * GC) + i * GC + j] = 0.f;
          a.rev[op * REV_ELEMS + REV_PT + (jb * 32 + (r >> 2) * 8 + hf * 4 + (r & 3)) * GC + ib * 32 + c] = (__bf16)0.f;
        } else {
          pout[i * GC + j] = (__bf16)0.f;
        }
      }
    }
  }

  // (scale Q exp(gamma)) transposed: one 16-byte piece = 8 consecutive tokens of one dim.  (The same of K exp(gamma_last
  // - gamma) is written further down, by the waves that would otherwise wait for the triangular inverse.)
  if constexpr (BWD) {
    for (int piece = tid; piece < GD * (GC / 8); piece += G_THREADS) {
      const int d = piece >> 3, i0 = (piece & 7) * 8;
      float f[8];
#pragma unroll
      for (int e = 0; e < 8; e++) f[e] = (float)qsm[i0 + e][d] * a.scale * __expf(gam[i0 + e]);
      *(bf16x8*)(a.rev + op * REV_ELEMS + REV_QGT + d * GC + i0) = cvt8(f[0], f[1], f[2], f[3], f[4], f[5], f[6], f[7]);
    }
  }
  __syncthreads();
  if constexpr (BWD) {
    // dO^T: the rows of dO go through the Q tile's LDS (free now) and leave transposed (further down, beside the
    // triangular inverse)
#pragma unroll
    for (int p = 0; p < NPIECE; p++) {
      const int piece = tid + p * G_THREADS, i = piece >> 4, c8 = (piece & 15) * 8;
      *(bf16x8*)&qsm[i][c8] = i < len ? doreg[p] : zero8;
    }
    __syncthreads();
  }
  // V rows into the Q tile's LDS (once that is free), for the first product: every thread its own pieces, the wave that
  // forms the inverse after it has done so (the barrier in front of the product covers both)
  auto stage_v_rows = [&]() {
#pragma unroll
    for (int p = 0; p < NPIECE; p++) {
      const int piece = tid + p * G_THREADS, i = piece >> 4, c8 = (piece & 15) * 8;
      *(bf16x8*)&qsm[i][c8] = i < len ? vreg[p] : zero8;
    }
  };

  // U = (I + A)^-1 (beta V),  W = (I + A)^-1 (beta exp(gamma) K) as products with the explicit inverse
  // T = (I + A)^-1 (unit lower triangular, like I + A), formed by one wave (a quarter of the multiply-adds that
  // substitution on the 256 columns of [V | K] took, which kept all four waves busy for most of this kernel's time);
  // the products (T diag(beta)) V and (T diag(beta exp(gamma))) K then run on the matrix cores.  V and K are bf16 as
  // they stand; the scaled T is split into two bf16 halves (hi + lo, relative error 2^-17), so the products carry
  // fp32-grade operands, and U, W are rounded to bf16 once, as before.
  // The inverse by 32 x 32 blocks, T = [T11 0; T21 T22]: the diagonal blocks by forward substitution on the identity,
  // one lane per column, both blocks at once in the two halves of the wave (31 steps instead of 63); then
  // T21 = -T22 (A21 T11) as two products on the fp32 matrix instruction.
  // (the wave that does it differs from workgroup to workgroup: the waves of a workgroup sit on different SIMDs, and
  // with always the same one the inverses of the compute unit's resident workgroups would queue up on one SIMD)
  const int tw = (int)((blockIdx.x >> 3) & 3);
  const int c = lane & 31, hf = lane >> 5;
  float x[32];                          // wave tw: column c of T11 (lanes 0 .. 31) / of T22 (lanes 32 .. 63)
  f32x16 t21;                           // wave tw: T21 as an accumulator tile (rows 32 + tile row, column c)
  if (w == tw) {
    const float* ablk = &am[32 * hf][32 * hf];
#pragma unroll
    for (int i = 0; i < 32; i++) x[i] = i == c ? 1.f : 0.f;
#pragma unroll
    for (int i = 1; i < 32; i++) {
      // x_i = delta_ij - sum_{k<i} A_ik x_k, four partial sums (the chain of one sum would leave the wave waiting)
      float s0 = x[i], s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
      for (int j4 = 0; j4 < (i + 3) / 4; j4++) {
        const float4 av = *(const float4*)(ablk + i * AM_PITCH + j4 * 4);   // entries at k >= i are zero; rows past the chunk too
        s0 -= av.x * x[j4 * 4];
        s1 -= av.y * x[j4 * 4 + 1];
        s2 -= av.z * x[j4 * 4 + 2];
        s3 -= av.w * x[j4 * 4 + 3];
      }
      x[i] = (s0 + s1) + (s2 + s3);
    }
    // Y = A21 T11: step s contracts k = 2 s (lower half of the wave) and 2 s + 1 (upper half); the upper half takes
    // its T11 row from the lower half's registers
    f32x16 y = zero16();
#pragma unroll
    for (int s2 = 0; s2 < 16; s2++) {
      const float from_lower = __shfl(x[2 * s2 + 1], c);
      y = __builtin_amdgcn_mfma_f32_32x32x2f32(am[32 + c][2 * s2 + hf], hf ? from_lower : x[2 * s2], y, 0, 0, 0);
    }
    // T21 = -T22 Y: Y's registers are the B operand as they stand when step s contracts the rows that register s
    // holds (8 (s / 4) + 4 hf + s % 4); T22 goes through LDS to become the A operand (row c, that k) -- into the upper
    // right block of A, which nothing reads
    if (hf) {
#pragma unroll
      for (int i = 0; i < 32; i++) am[i][32 + c] = x[i];
    }
    t21 = zero16();
#pragma unroll
    for (int s2 = 0; s2 < 16; s2++)
      t21 = __builtin_amdgcn_mfma_f32_32x32x2f32(am[c][32 + 8 * (s2 >> 2) + 4 * hf + (s2 & 3)], y[s2], t21, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 16; r++) t21[r] = -t21[r];
    if constexpr (BWD) {
      // T itself, for the finish kernel's transposed solve: the diagonal blocks (row 32 hf + i, column lane), T21, and
      // the zero block
      float* tg = a.f32.t + op * (GC * GC);
#pragma unroll
      for (int i = 0; i < 32; i++) tg[(32 * hf + i) * GC + lane] = x[i];
#pragma unroll
      for (int r = 0; r < 16; r++) {
        tg[(32 + (r >> 2) * 8 + 4 * hf + (r & 3)) * GC + c] = t21[r];
        tg[(2 * r + hf) * GC + 32 + c] = 0.f;
      }
    }
    if constexpr (!BWD) stage_v_rows();
  } else {
    // meanwhile the other three waves write (K exp(gamma_last - gamma)) transposed (K stays in LDS until the second
    // product) and, in the backward form, dO^T: 8 consecutive tokens of one dim per piece
    const int t3 = 64 * (w - (w > tw ? 1 : 0)) + lane;
    if constexpr (BWD) {
      for (int piece = t3; piece < GD * (GC / 8); piece += G_THREADS - 64) {
        const int d = piece >> 3, i0 = (piece & 7) * 8;
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = qsm[i0 + e][d];
        *(bf16x8*)(a.rev + op * REV_ELEMS + REV_DOT + d * GC + i0) = o;
      }
    } else {
      stage_v_rows();
    }
    for (int piece = t3; piece < GD * (GC / 8); piece += G_THREADS - 64) {
      const int d = piece >> 3, i0 = (piece & 7) * 8;
      float f[8];
#pragma unroll
      for (int e = 0; e < 8; e++) f[e] = (float)ksm[i0 + e][d] * __expf(g_last - gam[i0 + e]);
      *(bf16x8*)(a.rec + op * REC_ELEMS + REC_KDT + d * GC + i0) = cvt8(f[0], f[1], f[2], f[3], f[4], f[5], f[6], f[7]);
    }
  }
  if constexpr (BWD) {
    __syncthreads();                    // dO has been read: V may take its place
    stage_v_rows();
  }
  // one product: C (64 x 128) = (hi + lo) (64 x 64) B (64 tokens x 128, row-major in LDS); wave w takes the column
  // block w, both row blocks
  auto product = [&](const __bf16 (*bsm)[GROW], f32x16 (&acc)[2]) {
    acc[0] = zero16(); acc[1] = zero16();
#pragma unroll
    for (int ks = 0; ks < GC / 16; ks++) {
      const bf16x8 b = kmajor_frag(&bsm[0][0], GROW, 16 * ks + 8 * hf, 32 * w + 16 * (c >> 4), lane);
#pragma unroll
      for (int t = ks < GC / 32 ? 0 : 1; t < 2; t++) {   // (rows 0 .. 31 of T are zero from column 32 on)
        const bf16x8 ah = *(const bf16x8*)&t_hi[32 * t + c][16 * ks + 8 * hf];
        const bf16x8 al = *(const bf16x8*)&t_lo[32 * t + c][16 * ks + 8 * hf];
        acc[t] = mfma32(ah, b, acc[t]);
        acc[t] = mfma32(al, b, acc[t]);
      }
    }
  };
  // the inverse with column j scaled by f(j), as hi + lo (its upper right block is zero and is neither written nor read)
  auto put_scaled = [&](auto f) {
    auto put = [&](int i, int j, float v) {
      const __bf16 h = (__bf16)v;
      t_hi[i][j] = h;
      t_lo[i][j] = (__bf16)(v - (float)h);
    };
    const float fd = f(lane), fo = f(c);
#pragma unroll
    for (int i = 0; i < 32; i++) put(32 * hf + i, lane, x[i] * fd);
#pragma unroll
    for (int r = 0; r < 16; r++) put(32 + (r >> 2) * 8 + 4 * hf + (r & 3), c, t21[r] * fo);
  };
  // The results leave through LDS, so that memory sees whole 16-byte pieces from consecutive lanes (stored straight
  // from the accumulators, U^T goes out as 8-byte pieces 128 bytes apart and W as 2-byte elements: most of this
  // part's time).  The V tile's LDS holds U^T once the first product has read it, the K tile's LDS holds -W after the
  // second.  [column][token] arrays: 8-byte piece p of column col sits at position p ^ 2 (col % 8) (keeps the two
  // halves of a 16-byte piece together; without it the 32 columns of a wave would start in two banks).
  __bf16* stage_v = &qsm[0][0];
  __bf16* stage_k = &ksm[0][0];
  auto stage_transposed = [&](__bf16* st, const f32x16 (&ac)[2], float sign) {     // [128 columns][64 tokens]
    const int col = 32 * w + c, sw = (col & 7) << 1;
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int r4 = 0; r4 < 4; r4++)
        *(bf16x4*)(st + col * GC + (((8 * t + 2 * r4 + hf) ^ sw) << 2)) =
            cvt4(sign * ac[t][4 * r4], sign * ac[t][4 * r4 + 1], sign * ac[t][4 * r4 + 2], sign * ac[t][4 * r4 + 3]);
  };
  auto copy_out_transposed = [&](const __bf16* st, __bf16* dst) {                  // dst [128][64], contiguous
#pragma unroll
    for (int p = 0; p < GD * GC / 8 / G_THREADS; p++) {
      const int piece = tid + p * G_THREADS, col = piece >> 3, q = piece & 7;
      *(bf16x8*)(dst + (size_t)piece * 8) = *(const bf16x8*)(st + col * GC + (((2 * q) ^ ((col & 7) << 1)) << 2));
    }
  };
  f32x16 acc[2];
  if (w == tw) put_scaled([&](int j) { return bet[j]; });    // (behind that wave's own reads of A: LDS operations of a wave are ordered)
  __syncthreads();
  product(qsm, acc);                    // U: rows = tokens, columns = value dims 32 w .. 32 w + 31
  __syncthreads();                      // every wave has read the halves and V
  stage_transposed(stage_v, acc, 1.f);
  if (w == tw) put_scaled([&](int j) { return bet[j] * __expf(gam[j]); });
  __syncthreads();
  copy_out_transposed(stage_v, a.rec + op * REC_ELEMS + REC_UT);
  product(ksm, acc);                    // W: columns = key dims
  __syncthreads();                      // K has been read, U^T has left
  {
    // -W [token][key dim]: 2-byte elements, consecutive lanes = consecutive columns of a row
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int r = 0; r < 16; r++) stage_k[(32 * t + (r >> 2) * 8 + 4 * hf + (r & 3)) * GD + 32 * w + c] = (__bf16)(-acc[t][r]);
    if constexpr (BWD) stage_transposed(stage_v, acc, -1.f);      // -W^T for the reverse walk and the finish kernel
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < GC * GD / 8 / G_THREADS; p++) {
    const int piece = tid + p * G_THREADS;
    *(bf16x8*)(a.rec + op * REC_ELEMS + REC_WN + (size_t)piece * 8) = *(const bf16x8*)(stage_k + piece * 8);
  }
  if constexpr (BWD) copy_out_transposed(stage_v, a.rev + op * REV_ELEMS + REV_WTN);
}

typedef unsigned u32x4n __attribute__((ext_vector_type(4)));      // native vector type (stays in registers)

// ---- scan kernel ------------------------------------------------------------------------------------
// LDS image of one chunk's operands, filled by direct global->LDS copies (no registers, no store
// instructions; the copy engine's time overlaps the MFMA phases of the previous chunk).  A copy
// instruction writes 1 KB contiguous, so rows cannot be padded; 16-byte pieces are permuted instead:
// the [64][128] tiles use the attention kernels' swizzle (dma_tile64 / lds_row_frag), the arrays with
// 64-element rows store piece q of row r at position q ^ (r & 7).
struct ScanImage {
  __bf16 wn[GC * GD];           // -W, swizzled tile
  __bf16 qg[GC * GD];           // scale Q exp(gamma), swizzled tile
  __bf16 kd[GD * GC];           // (K decayed)^T, rows of 64
  __bf16 ut[SCAN_NB * G_DVB * GC];   // U^T, this workgroup's value columns (block after block), rows of 64
  __bf16 p[GC * GC];            // scale tril(Q K^T decay), rows of 64
};
// Per column block: st, vx.  The output tiles of waves 2 and 3 of a block, on their way to 16-byte stores, reuse
// the current image's qg tile (OT_ELEMS elements per wave): qg is only read before the step's second barrier, the
// tiles are written after it, and the next copy into that image is issued behind the next step's first barrier.
struct ScanSmem {
  ScanImage img[2];
  __bf16 st[SCAN_NB][G_DVB][GROW];   // S0^T
  bf16x8 vx[SCAN_NB][2][2][64];      // Vn as per-lane B-operand fragments, written by waves 0 and 1, read by the block
};
constexpr int OT_ROW = G_DVB + 8, OT_ELEMS = 32 * OT_ROW;
static_assert(2 * SCAN_NB * OT_ELEMS <= GC * GD, "output tiles fit into the qg tile");
static_assert(sizeof(ScanSmem) <= 160 * 1024, "LDS of one compute unit");

// 4 consecutive elements e0 .. e0+3 (e0 a multiple of 4) of row r of a rows-of-64 array
__device__ __forceinline__ bf16x4 row64_read4(const __bf16* arr, int r, int e0) {
  return *(const bf16x4*)(arr + r * GC + ((((e0 >> 3) ^ (r & 7)) << 3) | (e0 & 7)));
}
// 8 k-values in the order in which an accumulator's registers enumerate rows: elements e = 0..3 are
// columns base + 4 hf .. +3, e = 4..7 columns base + 8 + 4 hf .. +3 of row r.
__device__ __forceinline__ bf16x8 row64_perm_k(const __bf16* arr, int r, int base, int hf) {
  return cat4(row64_read4(arr, r, base + 4 * hf), row64_read4(arr, r, base + 8 + 4 * hf));
}

// Copies `rows` rows of 64 elements (contiguous in memory) into a rows-of-64 array; 8 rows per
// instruction, instructions dealt round-robin to the workgroup's waves (w8 = 0 .. SCAN_NW - 1).
__device__ __forceinline__ void dma_rows64(const __bf16* src, int rows, __bf16* dst, int w8, int lane) {
  const void* gb = uniform_ptr(src);
  const int rr = lane >> 3, pos = lane & 7;
  for (int g = w8; g < rows / 8; g += SCAN_NW)
    dma16(gb, (uint32_t)((8 * g + rr) * 128 + ((pos ^ rr) << 4)), lds_addr_uniform(dst + g * 8 * GC));
}

// Starts the copy of one chunk's operands into `im` (8 instructions per wave; TRAIN: without the output's
// operands, 5).  dvb0: the workgroup's first column block; the U^T rows of its blocks are adjacent in the record.
template <bool TRAIN>
__device__ __forceinline__ void issue_chunk(const GdnArgs& a, int chunk, int h, int dvb0, ScanImage& im, int w8, int lane) {
  const __bf16* rec = a.rec + op_index(a, chunk, h) * REC_ELEMS;
  dma_tile64<SCAN_NW>(rec + REC_WN, GD * 2, GC, im.wn, w8, lane);
  if constexpr (!TRAIN) dma_tile64<SCAN_NW>(rec + REC_QG, GD * 2, GC, im.qg, w8, lane);
  dma_rows64(rec + REC_KDT, GD, im.kd, w8, lane);
  dma_rows64(rec + REC_UT + (size_t)dvb0 * G_DVB * GC, SCAN_NB * G_DVB, im.ut, w8, lane);
  if constexpr (!TRAIN) dma_rows64(rec + REC_P, GC, im.p, w8, lane);
}

// The scalars of a chunk.  `z` is a per-lane zero the compiler cannot see through: they are loaded per
// lane and stay in vector registers (a value proven uniform is moved to a scalar register right behind
// its load, which would stall for a full memory latency).
struct ChunkMeta {
  int tok0, len, src, dst, cap;
  float glast;
};
__device__ __forceinline__ void load_meta(const GdnArgs& a, int chunk, int h, int z, ChunkMeta& r) {
  r.tok0 = a.chunk_tok0[chunk + z]; r.len = a.chunk_len[chunk + z]; r.src = a.chunk_src[chunk + z]; r.dst = a.chunk_dst[chunk + z];
  r.cap = a.chunk_cap ? a.chunk_cap[chunk + z] : -1;
  r.glast = a.glast[op_index(a, chunk, h) + z];
}

// One chunk of the scan.  On entry the copy of this chunk's operands into `im` is in flight (issued one
// step earlier) and `meta` holds its scalars; the step waits for them, starts the next chunk's copy
// into `im_next` and reloads `meta` for the next step.  Two barriers per step.
// TRAIN (first pass of the backward): no output; the entering state (bf16, transposed, as it stands in LDS) and
// Vn (as the B-operand fragments) of every chunk are saved instead.
template <bool TRAIN>
__device__ __forceinline__ void scan_step(const GdnArgs& a, ScanSmem& sm, ScanImage& im, ScanImage& im_next, ChunkMeta& meta, int chunk,
                                          int c_end, int h, int dvb0, int blk, int lane, int z, int w8, int w, int c, int hf, f32x16& s) {
  const int dvb = dvb0 + blk;                     // this wave's column block; w = its wave index inside the block
  const int tok0 = meta.tok0, len = meta.len, src = meta.src, dst = meta.dst, cap = meta.cap;
  const float glast = meta.glast;

  if (src == -1 && !a.initial_state) {
    s = zero16();
  } else if (src != -2) {
    // a saved node-end state, or the state handed in for the roots
    const float* sp = (src >= 0 ? a.slots + ((size_t)src * a.hv + h) * (GD * GD) : a.initial_state + (size_t)h * (GD * GD)) +
                      dvb * G_DVB + c;
#pragma unroll
    for (int r = 0; r < 16; r++) s[r] = sp[(size_t)(32 * w + (r >> 2) * 8 + hf * 4 + (r & 3)) * GD];
    pin(s);       // the wait for these loads belongs inside this (rare) branch, not at the merge point
  }
  // S0 -> bf16, transposed into LDS
#pragma unroll
  for (int r4 = 0; r4 < 4; r4++)
    *(bf16x4*)&sm.st[blk][c][32 * w + r4 * 8 + hf * 4] = cvt4(s[4 * r4], s[4 * r4 + 1], s[4 * r4 + 2], s[4 * r4 + 3]);
  dma_wait_all();                     // this wave's share of the chunk's operands has landed ...
  __syncthreads();                    // ... and so has everybody else's; every wave has also left the previous step,
                                      // so the other image, st and vx may be overwritten
  if (chunk + 1 < c_end) issue_chunk<TRAIN>(a, chunk + 1, h, dvb0, im_next, w8, lane);
  load_meta(a, min(chunk + 1, c_end - 1), h, z, meta);
  [[maybe_unused]] const size_t op = op_index(a, chunk, h);

  // Waves 0 and 1 compute one 32-row block of Vn = U - W S0 each; waves 2 and 3 meanwhile compute their
  // 32 rows of Q S0, the part of the output that does not need Vn.  Vn then goes through LDS as per-lane
  // B-operand fragments (k = tokens, in the order the accumulator registers enumerate rows), and every
  // wave updates its 32 rows of the state.  All LDS reads of a phase are issued before its first MFMA:
  // with one wave per SIMD nothing else hides an LDS round trip.
  bf16x8 sfrag[GD / 16];              // B operand: column c of S0, k = key dims
  bf16x8 afrag[GD / 16];              // A operands: rows of -W (waves 0, 1) or of Q exp(gamma) (waves 2, 3)
  bf16x8 kfrag[2][2];                 // A operands of the state update
  bf16x8 pfrag[2][2];                 // waves 2, 3: A operands of P Vn
  const int half = w & 1;             // which 32-row block this wave works on
  if (!TRAIN || w < 2) {
    const __bf16* atile = w < 2 ? im.wn : im.qg;
    const int abase = row_frag_base(lane);
#pragma unroll
    for (int ks = 0; ks < GD / 16; ks++) {
      sfrag[ks] = *(const bf16x8*)&sm.st[blk][c][ks * 16 + hf * 8];
      afrag[ks] = lds_row_frag(atile, abase, half, ks);
    }
  }
  if constexpr (TRAIN) {
    if (w >= 2) {
      // 32 rows of 256 bytes: 512 pieces of 16 bytes over the 128 lanes of waves 2 and 3
      const int t128 = half * 64 + lane;
      u32x4n* sdst = (u32x4n*)(a.s0t + op * (GD * GD) + (size_t)dvb * G_DVB * GD);
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int piece = i * 128 + t128, row = piece >> 4, c8 = (piece & 15) * 8;
        sdst[piece] = *(const u32x4n*)&sm.st[blk][row][c8];
      }
    }
  }
  f32x16 acc;
  if (w < 2) {
#pragma unroll
    for (int r4 = 0; r4 < 4; r4++) {
      const bf16x4 u4 = row64_read4(im.ut + blk * (G_DVB * GC), c, half * 32 + r4 * 8 + hf * 4);
#pragma unroll
      for (int e = 0; e < 4; e++) acc[4 * r4 + e] = (float)u4[e];
    }
  } else {
    acc = zero16();
  }
#pragma unroll
  for (int jb = 0; jb < 2; jb++)
#pragma unroll
    for (int t = 0; t < 2; t++) {
      kfrag[jb][t] = row64_perm_k(im.kd, 32 * w + c, jb * 32 + t * 16, hf);
      if constexpr (!TRAIN) pfrag[jb][t] = row64_perm_k(im.p, half * 32 + c, jb * 32 + t * 16, hf);     // used by waves 2, 3 only
    }
  __builtin_amdgcn_sched_barrier(0);
  if (!TRAIN || w < 2) {
#pragma unroll
    for (int ks = 0; ks < GD / 16; ks++) acc = mfma32(afrag[ks], sfrag[ks], acc);
  }
  if (w < 2) {
#pragma unroll
    for (int t = 0; t < 2; t++) {
      const bf16x8 f = cvt8(acc[8 * t], acc[8 * t + 1], acc[8 * t + 2], acc[8 * t + 3], acc[8 * t + 4], acc[8 * t + 5],
                            acc[8 * t + 6], acc[8 * t + 7]);
      sm.vx[blk][half][t][lane] = f;
      if constexpr (TRAIN) ((bf16x8*)a.vns)[(((op * 4 + dvb) * 2 + half) * 2 + t) * 64 + lane] = f;
    }
  }
  __syncthreads();
  bf16x8 vfrag[2][2];
#pragma unroll
  for (int rb = 0; rb < 2; rb++)
#pragma unroll
    for (int t = 0; t < 2; t++) vfrag[rb][t] = sm.vx[blk][rb][t][lane];

  // S1 = exp(gamma_last) S0 + (K decayed)^T Vn, rows 32 w .. 32 w + 31 of the state
#pragma unroll
  for (int r = 0; r < 16; r++) s[r] *= glast;
#pragma unroll
  for (int jb = 0; jb < 2; jb++)
#pragma unroll
    for (int t = 0; t < 2; t++) s = mfma32(kfrag[jb][t], vfrag[jb][t], s);
  if (dst >= 0) {
    float* sp = a.slots + ((size_t)dst * a.hv + h) * (GD * GD) + dvb * G_DVB + c;
#pragma unroll
    for (int r = 0; r < 16; r++) sp[(size_t)(32 * w + (r >> 2) * 8 + hf * 4 + (r & 3)) * GD] = s[r];
  }
  if (cap >= 0) {
    float* sp = a.state_out + ((size_t)cap * a.hv + h) * (GD * GD) + dvb * G_DVB + c;
#pragma unroll
    for (int r = 0; r < 16; r++) sp[(size_t)(32 * w + (r >> 2) * 8 + hf * 4 + (r & 3)) * GD] = s[r];
  }

  // O rows 32 half .. 32 half + 31 (waves 2 and 3): add P Vn to the Q S0 they already hold
  if (!TRAIN && w >= 2) {
#pragma unroll
    for (int jb = 0; jb < 2; jb++) {
      if (jb > half) continue;          // P is lower triangular
#pragma unroll
      for (int t = 0; t < 2; t++) acc = mfma32(pfrag[jb][t], vfrag[jb][t], acc);
    }
    // through LDS so that the tile leaves as two 16-byte stores per lane (a row of the tile is 64
    // contiguous bytes of o); only this wave touches its tile, LDS operations of a wave are ordered
    __bf16(*ot)[OT_ROW] = (__bf16(*)[OT_ROW])(im.qg + (blk * 2 + half) * OT_ELEMS);
#pragma unroll
    for (int r = 0; r < 16; r++) ot[(r >> 2) * 8 + hf * 4 + (r & 3)][c] = (__bf16)acc[r];
#pragma unroll
    for (int part = 0; part < 2; part++) {
      const int row = part * 16 + (lane >> 2), q8 = (lane & 3) * 8;
      const u32x4n val = *(const u32x4n*)&ot[row][q8];
      const int i = half * 32 + row;
      if (i < len) *(u32x4n*)(a.o + ((size_t)(tok0 + i) * a.hv + h) * GD + dvb * G_DVB + q8) = val;
    }
  }
}

// (head, first column block) of a scan workgroup from its id.  Consecutive ids go round-robin over the 8 XCDs;
// the workgroups of a head read the same operands, so they are given ids 8 apart and share one XCD's L2.
__device__ __forceinline__ void scan_workgroup(const GdnArgs& a, int id, int& h, int& dvb0) {
  constexpr int PER_HEAD = GD / G_DVB / SCAN_NB;        // workgroups per head
  int part;
  if (a.hv_n % 8 == 0) { h = (id / (8 * PER_HEAD)) * 8 + (id & 7); part = (id >> 3) % PER_HEAD; }
  else               { h = id / PER_HEAD; part = id % PER_HEAD; }
  dvb0 = part * SCAN_NB;
}

template <bool TRAIN>
__global__ __launch_bounds__(SCAN_THREADS, 1) void gdn_scan_kernel(GdnArgs a) {
  __shared__ __attribute__((aligned(1024))) ScanSmem sm;
  int h, dvb0;
  scan_workgroup(a, blockIdx.x, h, dvb0);
  const int tid = threadIdx.x & (SCAN_THREADS - 1);
  const int lane = tid & 63;
  const int w8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = w8 >> 2, w = w8 & 3;
  const int c = lane & 31, hf = lane >> 5;
  f32x16 s = zero16();                  // S[32 w + rows(r)][dvb*32 + c]

  int z = 0;
  asm volatile("" : "+v"(z));
  // this workgroup's segment of the chunk program (blockIdx.y-th segment of the level being walked); the first
  // chunk of a segment never continues a previous chunk, so the state starts from its own source
  const int seg = a.seg_base + blockIdx.y;
  const int c_begin = a.seg_chunk0 ? a.seg_chunk0[seg] : 0;
  const int c_end = a.seg_chunk1 ? a.seg_chunk1[seg] : a.n_chunks;
  ChunkMeta meta;
  issue_chunk<TRAIN>(a, c_begin, h, dvb0, sm.img[0], w8, lane);
  load_meta(a, c_begin, h, z, meta);
  for (int chunk = c_begin; chunk < c_end; chunk += 2) {
    scan_step<TRAIN>(a, sm, sm.img[0], sm.img[1], meta, chunk, c_end, h, dvb0, blk, lane, z, w8, w, c, hf, s);
    if (chunk + 1 < c_end) scan_step<TRAIN>(a, sm, sm.img[1], sm.img[0], meta, chunk + 1, c_end, h, dvb0, blk, lane, z, w8, w, c, hf, s);
  }
}

// ---- reverse walk of the backward ---------------------------------------------------------------------
// Per chunk, last to first:  dVn = P^T dO + Kd dS1,  dS0 = EL dS1 + Qg^T dO - W^T dVn  -- the forward step's
// structure with (-W, S0, U) <-> (Kd, dS1, P^T dO) and (Kd^T, Vn) <-> (-W^T, dVn), plus the Qg^T dO term.  The
// LDS image is reused with other contents: wn <- Kd (swizzled tile), kd <- -W^T, qg <- Qg^T (rows of 64),
// p <- P^T, ut <- this workgroup's 32 rows of dO^T.  Saved for the finish kernel: dS1 (bf16, transposed) and dVn
// (fragments), like the forward walk's S0 and Vn.
// 8 consecutive elements e0 .. e0+7 (e0 a multiple of 8) of row r of a rows-of-64 array
__device__ __forceinline__ bf16x8 row64_read8(const __bf16* arr, int r, int e0) {
  return *(const bf16x8*)(arr + r * GC + (((e0 >> 3) ^ (r & 7)) << 3));
}
__device__ __forceinline__ void issue_rev_chunk(const GdnArgs& a, int chunk, int h, int dvb0, ScanImage& im, int w8, int lane) {
  const __bf16* rec = a.rev + op_index(a, chunk, h) * REV_ELEMS;
  dma_tile64<SCAN_NW>(rec + REV_KD, GD * 2, GC, im.wn, w8, lane);
  dma_rows64(rec + REV_WTN, GD, im.kd, w8, lane);
  dma_rows64(rec + REV_QGT, GD, im.qg, w8, lane);
  dma_rows64(rec + REV_PT, GC, im.p, w8, lane);
  dma_rows64(rec + REV_DOT + (size_t)dvb0 * G_DVB * GC, SCAN_NB * G_DVB, im.ut, w8, lane);
}

// `later_src`: the source of the chunk that follows in DFS order (handled one step earlier); -2 means that chunk
// continued from this one on chip, so `s` holds the gradient of this chunk's leaving state.
__device__ __forceinline__ void rscan_step(const GdnArgs& a, ScanSmem& sm, ScanImage& im, ScanImage& im_next, ChunkMeta& meta, int chunk,
                                           int c_begin, int seg, int h, int dvb0, int blk, int lane, int z, int w8, int w, int c, int hf,
                                           f32x16& s, int& later_src) {
  const int dvb = dvb0 + blk;
  const int src = meta.src, dst = meta.dst, cap = meta.cap;
  const float glast = meta.glast;
  const size_t op = op_index(a, chunk, h);

  if (later_src != -2) s = zero16();
  later_src = src;
  if (dst >= 0) {
    if (a.seg_chunk0) {
      // scheduled walk: every segment that started from this slot (all of later levels, hence done) has stored
      // the gradient of its entering state; they are added in the order of the slot's reader list
      const int k0 = a.slot_cons_off[dst + z], k1 = a.slot_cons_off[dst + 1 + z];
      for (int kk = k0; kk < k1; kk++) {
        const float* sp = a.seg_grad + ((size_t)a.slot_cons[kk + z] * a.hv + h) * (GD * GD) + dvb * G_DVB + c;
#pragma unroll
        for (int r = 0; r < 16; r++) s[r] += sp[(size_t)(32 * w + (r >> 2) * 8 + hf * 4 + (r & 3)) * GD];
        pin(s);
      }
    } else {
      float* sp = a.slot_grad + ((size_t)dst * a.hv + h) * (GD * GD) + dvb * G_DVB + c;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        float* e = sp + (size_t)(32 * w + (r >> 2) * 8 + hf * 4 + (r & 3)) * GD;
        s[r] += *e;
        *e = 0.f;                        // the slot is reused by an earlier node
      }
      pin(s);
    }
  }
  if (cap >= 0) {
    const float* sp = a.d_state_out + ((size_t)cap * a.hv + h) * (GD * GD) + dvb * G_DVB + c;
#pragma unroll
    for (int r = 0; r < 16; r++) s[r] += sp[(size_t)(32 * w + (r >> 2) * 8 + hf * 4 + (r & 3)) * GD];
    pin(s);
  }
  // dS1 -> bf16, transposed into LDS
#pragma unroll
  for (int r4 = 0; r4 < 4; r4++)
    *(bf16x4*)&sm.st[blk][c][32 * w + r4 * 8 + hf * 4] = cvt4(s[4 * r4], s[4 * r4 + 1], s[4 * r4 + 2], s[4 * r4 + 3]);
  dma_wait_all();
  __syncthreads();
  if (chunk > c_begin) issue_rev_chunk(a, chunk - 1, h, dvb0, im_next, w8, lane);
  load_meta(a, max(chunk - 1, c_begin), h, z, meta);

  const int half = w & 1;
  bf16x8 ofrag[GC / 16];              // B operand: column c of dO, k = tokens in plain order
#pragma unroll
  for (int js = 0; js < GC / 16; js++) ofrag[js] = row64_read8(im.ut + blk * (G_DVB * GC), c, js * 16 + hf * 8);
  bf16x8 wfrag[2][2], qfrag[GC / 16];
#pragma unroll
  for (int jb = 0; jb < 2; jb++)
#pragma unroll
    for (int t = 0; t < 2; t++) wfrag[jb][t] = row64_perm_k(im.kd, 32 * w + c, jb * 32 + t * 16, hf);
  if (w < 2) {
    // rows 32 half .. of dVn
    bf16x8 sfrag[GD / 16], afrag[GD / 16], pfrag[GC / 16];
    const int abase = row_frag_base(lane);
#pragma unroll
    for (int ks = 0; ks < GD / 16; ks++) {
      sfrag[ks] = *(const bf16x8*)&sm.st[blk][c][ks * 16 + hf * 8];
      afrag[ks] = lds_row_frag(im.wn, abase, half, ks);
    }
#pragma unroll
    for (int js = 0; js < GC / 16; js++) pfrag[js] = row64_read8(im.p, half * 32 + c, js * 16 + hf * 8);
    f32x16 acc = zero16();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < GD / 16; ks++) acc = mfma32(afrag[ks], sfrag[ks], acc);
#pragma unroll
    for (int js = 0; js < GC / 16; js++) acc = mfma32(pfrag[js], ofrag[js], acc);
#pragma unroll
    for (int t = 0; t < 2; t++) {
      const bf16x8 f = cvt8(acc[8 * t], acc[8 * t + 1], acc[8 * t + 2], acc[8 * t + 3], acc[8 * t + 4], acc[8 * t + 5],
                            acc[8 * t + 6], acc[8 * t + 7]);
      sm.vx[blk][half][t][lane] = f;
      ((bf16x8*)a.dvns)[(((op * 4 + dvb) * 2 + half) * 2 + t) * 64 + lane] = f;
    }
  } else {
    // the gradient of the leaving state, for the finish kernel: 32 rows of 256 bytes over waves 2 and 3
    const int t128 = half * 64 + lane;
    u32x4n* sdst = (u32x4n*)(a.ds1t + op * (GD * GD) + (size_t)dvb * G_DVB * GD);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int piece = i * 128 + t128, row = piece >> 4, c8 = (piece & 15) * 8;
      sdst[piece] = *(const u32x4n*)&sm.st[blk][row][c8];
    }
  }
  __syncthreads();
  bf16x8 vfrag[2][2];
#pragma unroll
  for (int rb = 0; rb < 2; rb++)
#pragma unroll
    for (int t = 0; t < 2; t++) vfrag[rb][t] = sm.vx[blk][rb][t][lane];
  // (Qg^T fragments only now: fetched with the others in front of the first product they would push the wave past
  // its register budget at two waves per SIMD; the image is not overwritten before the next step's first barrier)
#pragma unroll
  for (int js = 0; js < GC / 16; js++) qfrag[js] = row64_read8(im.qg, 32 * w + c, js * 16 + hf * 8);

  // dS0 = exp(gamma_last) dS1 - W^T dVn + Qg^T dO, rows 32 w .. 32 w + 31
#pragma unroll
  for (int r = 0; r < 16; r++) s[r] *= glast;
#pragma unroll
  for (int jb = 0; jb < 2; jb++)
#pragma unroll
    for (int t = 0; t < 2; t++) s = mfma32(wfrag[jb][t], vfrag[jb][t], s);
#pragma unroll
  for (int js = 0; js < GC / 16; js++) s = mfma32(qfrag[js], ofrag[js], s);
  if (src >= 0 || (src == -1 && a.d_initial_state)) {
    if (a.seg_chunk0) {
      // scheduled walk: this is the first chunk of segment `seg`; its entering-state gradient is stored (not
      // added) in the segment's own array -- the slot's saver, or the sum over the roots, picks it up later
      float* sp = a.seg_grad + ((size_t)seg * a.hv + h) * (GD * GD) + dvb * G_DVB + c;
#pragma unroll
      for (int r = 0; r < 16; r++) sp[(size_t)(32 * w + (r >> 2) * 8 + hf * 4 + (r & 3)) * GD] = s[r];
    } else {
      float* sp = (src >= 0 ? a.slot_grad + ((size_t)src * a.hv + h) * (GD * GD) : a.d_initial_state + (size_t)h * (GD * GD)) +
                  dvb * G_DVB + c;
#pragma unroll
      for (int r = 0; r < 16; r++) sp[(size_t)(32 * w + (r >> 2) * 8 + hf * 4 + (r & 3)) * GD] += s[r];
    }
  }
}

__global__ __launch_bounds__(SCAN_THREADS, 1) void gdn_rscan_kernel(GdnArgs a) {
  __shared__ __attribute__((aligned(1024))) ScanSmem sm;
  int h, dvb0;
  scan_workgroup(a, blockIdx.x, h, dvb0);
  const int tid = threadIdx.x & (SCAN_THREADS - 1);
  const int lane = tid & 63;
  const int w8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int blk = w8 >> 2, w = w8 & 3;
  const int c = lane & 31, hf = lane >> 5;
  f32x16 s = zero16();                  // gradient of S[32 w + rows(r)][dvb*32 + c]
  int z = 0;
  asm volatile("" : "+v"(z));
  ChunkMeta meta;
  int later_src = -1;
  // this workgroup's segment, walked from its last chunk to its first (nothing continues from a segment's last
  // chunk on chip, so the state gradient starts from zero)
  const int seg = a.seg_base + blockIdx.y;
  const int c_begin = a.seg_chunk0 ? a.seg_chunk0[seg] : 0;
  const int last = (a.seg_chunk1 ? a.seg_chunk1[seg] : a.n_chunks) - 1;
  issue_rev_chunk(a, last, h, dvb0, sm.img[0], w8, lane);
  load_meta(a, last, h, z, meta);
  for (int chunk = last; chunk >= c_begin; chunk -= 2) {
    rscan_step(a, sm, sm.img[0], sm.img[1], meta, chunk, c_begin, seg, h, dvb0, blk, lane, z, w8, w, c, hf, s, later_src);
    if (chunk > c_begin)
      rscan_step(a, sm, sm.img[1], sm.img[0], meta, chunk - 1, c_begin, seg, h, dvb0, blk, lane, z, w8, w, c, hf, s, later_src);
  }
}

// d_initial_state = sum over the root segments (level 0, in order) of the gradients they stored
__global__ __launch_bounds__(G_THREADS) void gdn_root_grad_kernel(const float* __restrict__ seg_grad, int n_roots, int hv, int hv_n,
                                                                  float* __restrict__ d_initial_state) {
  const size_t n = (size_t)hv_n * GD * GD, seg_stride = (size_t)hv * GD * GD;
  for (size_t e = (size_t)blockIdx.x * G_THREADS + threadIdx.x; e < n; e += (size_t)gridDim.x * G_THREADS) {
    float acc = 0.f;
    for (int r = 0; r < n_roots; r++) acc += seg_grad[(size_t)r * seg_stride + e];
    d_initial_state[e] = acc;
  }
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

}  // namespace

size_t gdn_workspace(int n_chunks, int n_slots, int hv) {
  const size_t per = (size_t)n_chunks * hv;
  return align256(per * REC_ELEMS * 2) + align256(per * 4) + align256((size_t)n_slots * hv * GD * GD * 4) + 256;
}

// Walks the chunk program forward: one launch for everything without a schedule, else one launch per dependency
// level with the level's segments side by side (blockIdx.y).
template <bool TRAIN>
static hipError_t launch_scan(GdnArgs& a, const tt_gdn_schedule* sched, hipStream_t st) {
  const unsigned gx = (unsigned)((GD / G_DVB / SCAN_NB) * a.hv_n);
  if (!sched) {
    a.seg_chunk0 = a.seg_chunk1 = nullptr; a.seg_base = 0;
    gdn_scan_kernel<TRAIN><<<dim3(gx, 1), SCAN_THREADS, 0, st>>>(a);
    return hipGetLastError();
  }
  a.seg_chunk0 = sched->seg_chunk0; a.seg_chunk1 = sched->seg_chunk1;
  for (int l = 0; l < sched->n_levels; l++) {
    a.seg_base = sched->level_off[l];
    gdn_scan_kernel<TRAIN><<<dim3(gx, (unsigned)(sched->level_off[l + 1] - sched->level_off[l])), SCAN_THREADS, 0, st>>>(a);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t gdn_fwd(int64_t n_tokens, int hk, int hv, float scale, const void* q, const void* k, const void* v, const float* g,
                   const float* beta, int n_chunks, const int32_t* chunk_tok0, const int32_t* chunk_len, const int32_t* chunk_src,
                   const int32_t* chunk_dst, int n_slots, const int32_t* chunk_cap, const tt_gdn_schedule* sched,
                   const float* initial_state, float* state_out, void* o, void* workspace, hipStream_t st) {
  if (n_chunks == 0) return hipSuccess;
  GdnArgs a{};
  a.n_tokens = (int)n_tokens; a.hk = hk; a.hv = hv; a.hv_n = hv; a.n_chunks = n_chunks; a.scale = scale;
  a.q = (const __bf16*)q; a.k = (const __bf16*)k; a.v = (const __bf16*)v; a.g = g; a.beta = beta;
  a.chunk_tok0 = chunk_tok0; a.chunk_len = chunk_len; a.chunk_src = chunk_src; a.chunk_dst = chunk_dst;
  a.chunk_cap = chunk_cap; a.initial_state = initial_state; a.state_out = state_out;
  a.o = (__bf16*)o;
  const size_t per = (size_t)n_chunks * hv;
  char* p = (char*)workspace;
  a.rec = (__bf16*)p; p += align256(per * REC_ELEMS * 2);
  a.glast = (float*)p; p += align256(per * 4);
  a.slots = (float*)p;
  {
    KernelTimer t(TT_KERNEL_GDN_PREPARE, st);
    gdn_prepare_kernel<false><<<gdn_group_order_grid(n_chunks, hv, hv / hk), G_THREADS, 0, st>>>(a);
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  KernelTimer t(TT_KERNEL_GDN_SCAN, st);
  return launch_scan<false>(a, sched, st);
}

hipError_t gdn_bwd_prepare_and_walks(const GdnBwdArgs& b, const GdnChunkOps& ops, const GdnBwdSaved& sv, hipStream_t st) {
  if (b.n_chunks == 0) return hipSuccess;
  GdnArgs a{};
  a.n_tokens = (int)b.n_tokens; a.hk = b.hk; a.hv = b.hv; a.hv_n = b.hv_n; a.n_chunks = b.n_chunks; a.scale = b.scale;
  a.q = (const __bf16*)b.q; a.k = (const __bf16*)b.k; a.v = (const __bf16*)b.v; a.g = b.g; a.beta = b.beta;
  a.chunk_tok0 = b.chunk_tok0; a.chunk_len = b.chunk_len; a.chunk_src = b.chunk_src; a.chunk_dst = b.chunk_dst;
  a.initial_state = b.initial_state;
  a.rec = (__bf16*)sv.fwd_rec; a.glast = sv.glast; a.slots = sv.slots;
  a.f32 = ops; a.d_o = (const __bf16*)b.d_o; a.rev = (__bf16*)sv.rev_rec;
  a.s0t = (__bf16*)sv.s0t; a.vns = (__bf16*)sv.vns; a.ds1t = (__bf16*)sv.ds1t; a.dvns = (__bf16*)sv.dvns;
  a.slot_grad = sv.slot_grad; a.d_state_out = b.d_state_out; a.d_initial_state = b.d_initial_state;
  {
    KernelTimer t(TT_KERNEL_GDN_PREPARE, st);
    gdn_prepare_kernel<true><<<gdn_group_order_grid(b.n_chunks, b.hv_n, b.hv / b.hk), G_THREADS, 0, st>>>(a);
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  {
    KernelTimer t(TT_KERNEL_GDN_BWD_FSCAN, st);         // chunk_cap stays null: nothing is captured here
    if (hipError_t e = launch_scan<true>(a, b.sched, st); e != hipSuccess) return e;
  }
  a.chunk_cap = b.d_state_out ? b.chunk_cap : nullptr;
  {
    KernelTimer t(TT_KERNEL_GDN_BWD_RSCAN, st);
    const unsigned gx = (unsigned)((GD / G_DVB / SCAN_NB) * b.hv_n);
    if (!b.sched) {
      a.seg_chunk0 = a.seg_chunk1 = nullptr; a.seg_base = 0;
      gdn_rscan_kernel<<<dim3(gx, 1), SCAN_THREADS, 0, st>>>(a);
    } else {
      // last level first: a level's segments only need the gradients stored by later levels
      a.seg_grad = sv.seg_grad; a.slot_cons_off = b.sched->slot_cons_off; a.slot_cons = b.sched->slot_cons;
      for (int l = b.sched->n_levels - 1; l >= 0; l--) {
        a.seg_base = b.sched->level_off[l];
        gdn_rscan_kernel<<<dim3(gx, (unsigned)(b.sched->level_off[l + 1] - b.sched->level_off[l])), SCAN_THREADS, 0, st>>>(a);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
      }
      if (b.d_initial_state && b.sched->n_levels > 0)
        gdn_root_grad_kernel<<<256, G_THREADS, 0, st>>>(sv.seg_grad, b.sched->level_off[1], b.hv, b.hv_n, b.d_initial_state);
    }
  }
  return hipGetLastError();
}

}  // namespace tt
