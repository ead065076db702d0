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
__device__ __forceinline__ void pin(float f) { asm volatile("" ::"v"(f)); }
__device__ __forceinline__ void pin(const float __attribute__((ext_vector_type(16)))& f) { asm volatile("" ::"v"(f)); }
__device__ __forceinline__ void pin(int f) { asm volatile("" ::"v"(f)); }

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

// 8 consecutive k (k0 .. k0 + 7) of row / column n0 + (lane % 16) from a k-major LDS array ([k][n], `pitch`
// elements per k): two transposing reads of a 4 (k) x 16 (n) block each; inside a group of 16 lanes, lane i supplies
// the address of 4 consecutive elements of block row i / 4 and receives block column i.
__device__ __forceinline__ bf16x8 kmajor_frag(const __bf16* slab, int pitch, int k0, int n0, int lane) {
  const int i = lane & 15;
  const __bf16* p = slab + (k0 + (i >> 2)) * pitch + n0 + 4 * (i & 3);
  return cat4(lds_read_tr(p), lds_read_tr(p + 4 * pitch));
}

// The same for 8 k in the order in which an accumulator's registers enumerate rows: k0 .. k0 + 3 and k0 + 8 .. k0 + 11
// (k0 = 16 s + 4 hf of k-step s) -- the B operand that matches an A operand taken straight from accumulator registers.
__device__ __forceinline__ bf16x8 kmajor_frag_acc_order(const __bf16* slab, int pitch, int k0, int n0, int lane) {
  const int i = lane & 15;
  const __bf16* p = slab + (k0 + (i >> 2)) * pitch + n0 + 4 * (i & 3);
  return cat4(lds_read_tr(p), lds_read_tr(p + 8 * pitch));
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
// fragment * c, rounded to bf16 (nearest even)
__device__ __forceinline__ bf16x8 scale_frag(bf16x8 f, float c) {
  typedef float f32x8 __attribute__((ext_vector_type(8)));
  return __builtin_convertvector(__builtin_convertvector(f, f32x8) * c, bf16x8);
}
__device__ __forceinline__ bf16x4 cvt4(float a0, float a1, float a2, float a3) {
  f32x4 v = {a0, a1, a2, a3};
  return __builtin_convertvector(v, bf16x4);
}

// ---- LDS tiles: rows of 128 bf16 = 16 chunks of 16 bytes, no padding ---------------------------------
// Chunk c of row r is stored at chunk position c ^ swz(r).  With this permutation both access
// patterns of the kernels are bank-conflict free: 16 lanes reading the same chunk of 16 consecutive
// rows (A/B operand rows) and the 4-row x 64-byte blocks of a transposed read.
constexpr int TILE_ROW = 128;                       // elements per row
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// Per-lane base offset (elements) for operand-row reads: lane reads row (blk*32 + c32), d-step s,
// at  row_frag_base(lane) ^ (s << 4)  + blk * 32 * TILE_ROW.
__device__ __forceinline__ int row_frag_base(int lane) {
  const int c32 = lane & 31, hf = lane >> 5;
  return c32 * TILE_ROW + ((hf ^ swz(c32)) << 3);   // bit 0 of the chunk index carries hf
}
__device__ __forceinline__ bf16x8 lds_row_frag(const __bf16* tile, int base, int blk, int s) {
  return *(const bf16x8*)(tile + blk * 32 * TILE_ROW + (base ^ (s << 4)));
}

// Per-lane base offsets (elements) for transposed reads.  The fragment for MFMA k-step with rows
// R .. R+15 (R a multiple of 16) and column block db (32 columns) is
//   cat4( tr(tile + R*TILE_ROW + (tr_base[0] ^ (db << 5))), tr(tile + R*TILE_ROW + (tr_base[1] ^ (db << 5))) )
// and enumerates the rows in the accumulator-as-B-operand order (see the top of this file).
struct TrBase { int x0, x1; };
__device__ __forceinline__ TrBase tr_frag_base(int lane) {
  const int hf = lane >> 5, i16 = lane & 15, gidx = (lane >> 4) & 1;
  const int q2 = i16 >> 2, cc = (i16 & 3) >> 1, half = (i16 & 1) * 4;
  TrBase b;
  // row = R + 8x + 4hf + q2; chunk = 4db + 2gidx + cc; swz(row) = (q2 << 2) | (hf + 2x)
  b.x0 = ((4 * hf + q2) << 7) | (q2 << 5) | ((((2 * gidx + cc) ^ hf) & 3) << 3) | half;
  b.x1 = ((8 + 4 * hf + q2) << 7) | (q2 << 5) | ((((2 * gidx + cc) ^ (hf + 2)) & 3) << 3) | half;
  return b;
}
__device__ __forceinline__ bf16x8 lds_tr_frag(const __bf16* tile, TrBase b, int R, int db) {
  const __bf16* p = tile + R * TILE_ROW;
  return cat4(lds_read_tr(p + (b.x0 ^ (db << 5))), lds_read_tr(p + (b.x1 ^ (db << 5))));
}

// Reads through explicit LDS byte addresses.  A kernel keeps one address per swizzle variant in a
// register (the swizzle is an exclusive-or, so it cannot be expressed as an offset) and reaches the
// tile, the row block and the pipeline stage through the immediate offset of the instruction.
__device__ __forceinline__ bf16x8 lds_b128(uint32_t addr, int off) { return *(TT_LDS(const bf16x8)*)(addr + off); }
__device__ __forceinline__ bf16x8 lds_tr2(uint32_t a0, uint32_t a1, int off) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((TT_LDS(s16x4)*)(a0 + off));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((TT_LDS(s16x4)*)(a1 + off));
  return cat4(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi));
}
// Byte addresses of a lane's operand-row fragments (k-step ss) and transposed fragments (column block
// db, halves x = 0, 1) inside a swizzled tile that starts at LDS byte address `tile`.
__device__ __forceinline__ void frag_addresses(uint32_t tile, int lane, uint32_t (&ra)[8], uint32_t (&ta)[8]) {
  const int a_rd = row_frag_base(lane);
  const TrBase t_rd = tr_frag_base(lane);
#pragma unroll
  for (int ss = 0; ss < 8; ss++) ra[ss] = tile + 2u * (uint32_t)(a_rd ^ (ss << 4));
#pragma unroll
  for (int db = 0; db < 4; db++) {
    ta[2 * db] = tile + 2u * (uint32_t)(t_rd.x0 ^ (db << 5));
    ta[2 * db + 1] = tile + 2u * (uint32_t)(t_rd.x1 ^ (db << 5));
  }
}

// Asynchronous 16-byte-per-lane copy global -> LDS that bypasses the registers: lane l's 16 bytes
// land at lds_dst + 16*l (lds_dst is wave-uniform), read from gbase + voff (gbase wave-uniform).
// Completion is tracked by vmcnt; the data is visible to other waves after a wait + barrier.
__device__ __forceinline__ void dma16(const void* gbase, uint32_t voff, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_dst), "v"(voff), "s"(gbase) : "memory", "m0");
}
// 4-byte-per-lane variant: lane l's dword lands at lds_dst + 4*l
__device__ __forceinline__ void dma4(const void* gbase, uint32_t voff, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_dst), "v"(voff), "s"(gbase) : "memory", "m0");
}
__device__ __forceinline__ void dma_wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ uint32_t lds_addr_uniform(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)p);
}
__device__ __forceinline__ const void* uniform_ptr(const void* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const void*)(((uint64_t)hi << 32) | lo);
}

// Loads 64 rows x 128 bf16 into a swizzled LDS tile: tile row r comes from source row
// min(row0 + r, rows - 1) of a matrix with row stride `stride_b` bytes (so rows past the end repeat the
// last valid row); each of the NW waves moves 64/NW rows with 16/NW dma16 instructions.
template <int NW = 4>
__device__ __forceinline__ void dma_tile64(const void* gbase, uint32_t stride_b, int rows, __bf16* tile, int w, int lane,
                                           int row0 = 0) {
  constexpr int PER = 16 / NW;                       // instructions per wave (4 rows each)
  const int lr = lane >> 4, pc = lane & 15;
  const void* gb = uniform_ptr(gbase);
#pragma unroll
  for (int u = 0; u < PER; u++) {
    const int r4 = PER * w + u;                      // group of 4 rows
    const int row = 4 * r4 + lr;
    const int rc = min(row0 + row, rows - 1);
    const int c = pc ^ ((lr << 2) | (r4 & 3));        // = pc ^ swz(row)
    dma16(gb, (uint32_t)rc * stride_b + (uint32_t)c * 16u, lds_addr_uniform(tile + 4 * r4 * TILE_ROW));
  }
}

// Iterates over the key tiles (TT_KTILE keys each, prefix tiles first, then own tiles) that can hold
// a key visible to some query of the range [gi_first, gi_last] (unified indices): tiles up to the
// diagonal whose largest visibility bound exceeds gi_first.  Tiles in which every (query, key) pair
// is visible ("full": all 64 keys exist, all lie at or before the first query, and the smallest
// bound lies beyond the last query) are delivered first, then the tiles that need the per-element
// test -- softmax accumulation does not care about the order, and the two kinds run in separate
// branch-free loops.
//
// The classification is done up front, once per chunk of KT_MAX_WIN * 64 tiles: the waves of the
// workgroup share the windows of 64 tiles, classify each with one wavefront-wide pair of loads + two
// ballots, and leave the two bit masks in LDS; next() only reads those masks, so the tile loops hold
// no global load.  Every wavefront walks the same sequence.
constexpr int KT_MAX_WIN = 64;
// Class of a candidate tile: which per-element tests it needs (0 = none: a full tile).
enum : int { KT_FULL = 0, KT_NEED_KEND = 1, KT_NEED_CAUSAL = 2 };
struct KTileMasks { uint64_t m[4][KT_MAX_WIN]; };       // [0] full, [1] boundary, [2] boundary needing the kend test, [3] ... the causal test
struct KTileIter {
  const KTileMasks* masks;
  int tile0;        // first tile of the chunk
  int n_win;        // windows in the chunk
  int win;          // next window
  int phase;        // 0: full tiles, 1: boundary tiles
  uint64_t mask;    // undelivered tiles of the current window
  uint64_t m_kend, m_causal;   // test bits of the current window (boundary phase)
  // Classifies tiles [tile0, min(u_end, tile0 + 64 KT_MAX_WIN)); all waves of the workgroup call it
  // (it contains a barrier); nw = waves per workgroup, w = this wave.
  __device__ __forceinline__ void fill(KTileMasks* lds, const int32_t* kt_max, const int32_t* kt_min, int tile0_,
                                       int u_end, int gi_first, int gi_last, int npt, int P, int N, int w, int nw) {
    masks = lds; tile0 = tile0_; win = 0; phase = 0; mask = 0; m_kend = 0; m_causal = 0;
    n_win = min(KT_MAX_WIN, (u_end - tile0 + 63) >> 6);
    const int lane = (int)(threadIdx.x & 63);
    for (int wi = w; wi < n_win; wi += nw) {
      const int u = tile0 + wi * 64 + lane;
      const bool in = u < u_end;
      const int kmx = kt_max[in ? u : 0], kmn = kt_min[in ? u : 0];     // both loads in flight together
      const int j0 = u < npt ? u * 64 : P + (u - npt) * 64;
      const int rows = u < npt ? P - u * 64 : N - (u - npt) * 64;
      const bool cand = in && kmx > gi_first;
      // the causal test also hides the rows past the last key of a ragged tile
      const bool need_causal = cand && !(rows >= 64 && j0 + 63 <= gi_first);
      const bool need_kend = cand && !(kmn > gi_last);
      const bool full = cand && !need_causal && !need_kend;
      const uint64_t mf = __ballot(full), mb = __ballot(cand && !full), mk = __ballot(need_kend), mc = __ballot(need_causal);
      if (lane == 0) { lds->m[0][wi] = mf; lds->m[1][wi] = mb; lds->m[2][wi] = mk; lds->m[3][wi] = mc; }
    }
    __syncthreads();
  }
  __device__ static __forceinline__ uint64_t uniform64(uint64_t m) {
    // (the builtin returns a signed int: without the casts the low half would be sign-extended)
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)m);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(m >> 32));
    return ((uint64_t)hi << 32) | lo;
  }
  // returns the next tile or -1; cls tells which tests it needs (KT_FULL: none)
  __device__ __forceinline__ int next(int& cls) {
    while (mask == 0) {
      if (win >= n_win) {
        if (phase == 1) return -1;
        phase = 1; win = 0;
      }
      mask = uniform64(masks->m[phase][win]);
      if (phase == 1) {
        m_kend = uniform64(masks->m[2][win]);
        m_causal = uniform64(masks->m[3][win]);
      }
      win++;
    }
    const int b = __builtin_ctzll(mask);
    mask &= mask - 1;
    cls = phase == 0 ? KT_FULL : (int)((m_kend >> b) & 1) * KT_NEED_KEND + (int)((m_causal >> b) & 1) * KT_NEED_CAUSAL;
    return tile0 + (win - 1) * 64 + b;
  }
};

// Workgroup order of the gated delta rule's per-(chunk, value head) kernels.  The value heads of one key head read the
// same q and k rows; workgroups are dealt to the chip's 8 XCDs (each with its own L2) round-robin by their linear id,
// so the `group` members of a (chunk, key head) pair get ids that differ by multiples of 8 and follow each other
// directly on their XCD: they run at the same time behind the same L2.  The grid is padded to whole rounds of 8
// pairs; a workgroup past the last pair gets `false` and returns.
constexpr unsigned GDN_XCDS = 8;
inline unsigned gdn_group_order_grid(int n_chunks, int hv_n, int group) {
  const unsigned pairs = (unsigned)n_chunks * (unsigned)(hv_n / group);
  return (pairs + GDN_XCDS - 1) / GDN_XCDS * GDN_XCDS * (unsigned)group;
}
__device__ __forceinline__ bool gdn_group_order(unsigned id, int n_chunks, int hv_n, int group, int& chunk, int& h) {
  const unsigned xcd = id % GDN_XCDS, t = id / GDN_XCDS;
  const unsigned member = t % (unsigned)group, pair = t / (unsigned)group * GDN_XCDS + xcd;
  if (pair >= (unsigned)n_chunks * (unsigned)(hv_n / group)) return false;
  chunk = (int)(pair % (unsigned)n_chunks);
  h = (int)(pair / (unsigned)n_chunks) * group + (int)member;
  return true;
}

}  // namespace tt
