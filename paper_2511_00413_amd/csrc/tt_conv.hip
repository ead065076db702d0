// Tree-correct depthwise causal convolution (Section "Implementation", paragraph "SSM Layers (GDN)",
// item (ii); Appendix "Tree-Correct Causal Convolution"): every token's window holds the K-1 tokens
// that precede it on its own root-to-token sequence, found through tok_pred, not the K-1 tokens that
// precede it in DFS order.  HBM-bound: one lane owns one 16-byte channel vector and walks a tile of
// consecutive tokens with the window in registers; the window is rebuilt from the predecessor chain
// only where the sequence jumps (first token of a node that does not directly follow its parent's
// last token) and at the start of a tile.
#include <hip/hip_runtime.h>
#include "tt_internal.h"
#include "tt_kernels.h"

namespace tt {
namespace {

constexpr int CONV_THREADS = 256;

template <bool BF16> struct Chan { static constexpr int NV = BF16 ? 8 : 4; };

// one 16-byte channel vector of a row, as loaded (8 bf16 or 4 fp32); STREAM: a non-temporal access, for rows
// that this kernel touches once
typedef unsigned int u32x4c __attribute__((ext_vector_type(4)));
template <bool STREAM = false>
__device__ __forceinline__ uint4 load_raw(const void* base, int64_t row, int64_t stride_bytes, int cv) {
  const char* p = (const char*)base + row * stride_bytes + (int64_t)cv * 16;
  if (STREAM) {
    const u32x4c v = __builtin_nontemporal_load(reinterpret_cast<const u32x4c*>(p));
    return uint4{v.x, v.y, v.z, v.w};
  }
  return *reinterpret_cast<const uint4*>(p);
}
template <bool BF16>
__device__ __forceinline__ void unpack_raw(const uint4& u, float (&v)[Chan<BF16>::NV]) {
  if (BF16) {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  } else {
    v[0] = __uint_as_float(u.x); v[1] = __uint_as_float(u.y); v[2] = __uint_as_float(u.z); v[3] = __uint_as_float(u.w);
  }
}
template <bool BF16>
__device__ __forceinline__ void load_row(const void* base, int64_t row, int64_t stride_bytes, int cv, float (&v)[Chan<BF16>::NV]) {
  unpack_raw<BF16>(load_raw(base, row, stride_bytes, cv), v);
}

typedef float f32x8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));

template <bool BF16, bool STREAM = false>
__device__ __forceinline__ void store_row(void* base, int64_t row, int64_t stride_bytes, int cv, const float (&v)[Chan<BF16>::NV]) {
  char* p = (char*)base + row * stride_bytes + (int64_t)cv * 16;
  u32x4c out;
  if (BF16) {
    f32x8v f;
#pragma unroll
    for (int i = 0; i < 8; i++) f[i] = v[i];
    out = __builtin_bit_cast(u32x4c, __builtin_convertvector(f, bf16x8v));       // round to nearest even
  } else {
    out = u32x4c{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
  }
  if (STREAM) __builtin_nontemporal_store(out, reinterpret_cast<u32x4c*>(p));
  else *reinterpret_cast<u32x4c*>(p) = out;
}

struct ConvArgs {
  int n_tokens, channels, tok_tile, n_tiles;
  int silu;
  const void* x; int64_t x_stride;       // strides in bytes
  const float* weight;                   // [C][K]
  const float* bias;                     // [C] or nullptr
  const int32_t* tok_pred;
  void* y; int64_t y_stride;             // forward output / backward: dx
  const void* dy; int64_t dy_stride;
  float* partial;                        // [n_tiles][K+1][C]: per-tile dweight (K rows) and dbias
  int n_fix;
  const int32_t *fix_tok, *fix_off, *fix_t, *fix_r;
};

// sigmoid through the bare exp2 / reciprocal instructions (1 ulp each; the results are rounded to
// bf16 or meet fp32 sums of comparable error)
__device__ __forceinline__ float sigmoid_f(float z) {
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * z));
}
__device__ __forceinline__ float silu_f(float z) { return z * sigmoid_f(z); }
__device__ __forceinline__ float dsilu_f(float z) {
  const float s = sigmoid_f(z);
  return s * (1.f + z * (1.f - s));
}

template <bool BF16, int K>
struct Weights {
  static constexpr int NV = Chan<BF16>::NV;
  float w[K][NV], b[NV];
  __device__ __forceinline__ void load(const ConvArgs& a, int c0) {
#pragma unroll
    for (int i = 0; i < NV; i++) {
#pragma unroll
      for (int j = 0; j < K; j++) w[j][i] = a.weight[(int64_t)(c0 + i) * K + j];
      b[i] = a.bias ? a.bias[c0 + i] : 0.f;
    }
  }
};

// win[m-1] = x[pred^m(t)] for m = 1..K-1, zero past the start of the branch
template <bool BF16, int K>
__device__ __forceinline__ void rebuild_window(const ConvArgs& a, int pred, int cv, float (&win)[K > 1 ? K - 1 : 1][Chan<BF16>::NV]) {
  constexpr int NV = Chan<BF16>::NV;
  int q = pred;
#pragma unroll
  for (int m = 1; m < K; m++) {
    if (q >= 0) {
      load_row<BF16>(a.x, q, a.x_stride, cv, win[m - 1]);
      q = a.tok_pred[q];
    } else {
#pragma unroll
      for (int i = 0; i < NV; i++) win[m - 1][i] = 0.f;
    }
  }
}

template <bool BF16, int K>
__device__ __forceinline__ void pre_activation(const Weights<BF16, K>& wt, const float (&xt)[Chan<BF16>::NV],
                                               const float (&win)[K > 1 ? K - 1 : 1][Chan<BF16>::NV], float (&pre)[Chan<BF16>::NV]) {
  constexpr int NV = Chan<BF16>::NV;
#pragma unroll
  for (int i = 0; i < NV; i++) {
    float acc = wt.b[i] + wt.w[K - 1][i] * xt[i];
#pragma unroll
    for (int m = 1; m < K; m++) acc += wt.w[K - 1 - m][i] * win[m - 1][i];
    pre[i] = acc;
  }
}

// Tokens whose loads are issued together.  A multiple of K: the kernels keep the last K inputs (and, backward,
// the last K gradients) in rings of K register slots, token t0 + i in slot i % K, and with batches that are
// multiples of K every slot index is a compile-time constant after unrolling -- the rings never move.
template <int K> struct ConvBatch { static constexpr int U = K == 3 ? 3 : 4; };

// ring slot m places before slot `slot`
template <int K> __device__ __forceinline__ constexpr int ring_back(int slot, int m) { return (slot - m + 2 * K) % K; }

// xr[ring_back(slot, m)] = x[pred^m(t)] for m = 1..K-1, zero past the start of the branch
template <bool BF16, int K>
__device__ __forceinline__ void rebuild_ring(const ConvArgs& a, int pred, int cv, int slot, float (&xr)[K][Chan<BF16>::NV]) {
  constexpr int NV = Chan<BF16>::NV;
  int q = pred;
#pragma unroll
  for (int m = 1; m < K; m++) {
    if (q >= 0) {
      load_row<BF16>(a.x, q, a.x_stride, cv, xr[ring_back<K>(slot, m)]);
      q = a.tok_pred[q];
    } else {
#pragma unroll
      for (int i = 0; i < NV; i++) xr[ring_back<K>(slot, m)][i] = 0.f;
    }
  }
}

template <bool BF16, int K>
__global__ __launch_bounds__(CONV_THREADS) void tree_conv_fwd_kernel(ConvArgs a) {
  constexpr int NV = Chan<BF16>::NV;
  constexpr int U = ConvBatch<K>::U;
  // consecutive workgroups cover one token tile's channel vectors (a row is read in full by neighbours)
  const int64_t gid = (int64_t)blockIdx.x * CONV_THREADS + threadIdx.x;
  const int vpr = a.channels / NV;
  const int tile = (int)(gid / vpr);
  const int cv = (int)(gid - (int64_t)tile * vpr);
  if (tile >= a.n_tiles) return;
  Weights<BF16, K> wt;
  wt.load(a, cv * NV);
  float xr[K][NV];                                  // ring of the last K inputs
  const int t0 = (int)tile * a.tok_tile;
  const int t1 = min(t0 + a.tok_tile, a.n_tokens);
  // Two batches of U tokens are in flight: the loads of the next batch are issued before the current one is
  // worked on, so the memory round trip of a batch runs under the arithmetic of the one before.
  struct Batch { int p[U]; uint4 x[U]; };
  auto load_batch = [&](int tb, Batch& b) {
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int t = min(tb + u, t1 - 1);
      b.p[u] = a.tok_pred[t];
      b.x[u] = load_raw<true>(a.x, t, a.x_stride, cv);
    }
  };
  auto work_batch = [&](int tb, const Batch& b) {       // (tb - t0) is a multiple of U, hence of K
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int t = tb + u;
      const int slot = u % K;
      if (t < t1) {
        unpack_raw<BF16>(b.x[u], xr[slot]);
        if (t == t0 || b.p[u] != t - 1) rebuild_ring<BF16, K>(a, b.p[u], cv, slot, xr);
        float pre[NV];
#pragma unroll
        for (int i = 0; i < NV; i++) {
          float acc = wt.b[i] + wt.w[K - 1][i] * xr[slot][i];
#pragma unroll
          for (int m = 1; m < K; m++) acc += wt.w[K - 1 - m][i] * xr[ring_back<K>(slot, m)][i];
          pre[i] = a.silu ? silu_f(acc) : acc;
        }
        store_row<BF16>(a.y, t, a.y_stride, cv, pre);
      }
    }
  };
  Batch ba, bb;
  load_batch(t0, ba);
  for (int tb = t0; tb < t1; tb += 2 * U) {
    load_batch(tb + U, bb);
    work_batch(tb, ba);
    load_batch(tb + 2 * U, ba);
    work_batch(tb + U, bb);
  }
}

// g[t] = dy[t] * act'(pre[t]) for one token, everything recomputed from x (used off the fast path)
template <bool BF16, int K>
__device__ __forceinline__ void grad_pre_at(const ConvArgs& a, const Weights<BF16, K>& wt, int t, int cv, float (&g)[Chan<BF16>::NV]) {
  constexpr int NV = Chan<BF16>::NV;
  float xt[NV], pre[NV], win[K > 1 ? K - 1 : 1][NV];
  load_row<BF16>(a.x, t, a.x_stride, cv, xt);
  rebuild_window<BF16, K>(a, a.tok_pred[t], cv, win);
  pre_activation<BF16, K>(wt, xt, win, pre);
  load_row<BF16>(a.dy, t, a.dy_stride, cv, g);
  if (a.silu) {
#pragma unroll
    for (int i = 0; i < NV; i++) g[i] *= dsilu_f(pre[i]);
  }
}

// Backward, fast path.  Walks the tile plus K-1 tokens of look-ahead; g of the last K tokens and
// their "directly follows its predecessor" flags stay in registers.  dx[s] takes the successors
// s+1 .. s+K-1 for as long as each directly follows the one before (successors that sit elsewhere
// in DFS order -- later children of a branch point -- are added by the fix-up kernel, which
// recomputes those few dx rows completely).  dweight / dbias partial sums per tile go to `partial`.
template <bool BF16, int K>
__global__ __launch_bounds__(CONV_THREADS) void tree_conv_bwd_kernel(ConvArgs a) {
  constexpr int NV = Chan<BF16>::NV;
  constexpr int U = ConvBatch<K>::U;
  const int64_t gid = (int64_t)blockIdx.x * CONV_THREADS + threadIdx.x;
  const int vpr = a.channels / NV;
  const int tile = (int)(gid / vpr);
  const int cv = (int)(gid - (int64_t)tile * vpr);
  if (tile >= a.n_tiles) return;
  Weights<BF16, K> wt;
  wt.load(a, cv * NV);
  // rings of K slots, token t0 + i in slot i % K: inputs, g = dy * act'(pre), and the "directly follows its
  // predecessor" flags
  float xr[K][NV], gq[K][NV];
  bool lk[K];
  float dw[K][NV], db[NV];
#pragma unroll
  for (int i = 0; i < NV; i++) {
    db[i] = 0.f;
#pragma unroll
    for (int j = 0; j < K; j++) { dw[j][i] = 0.f; gq[j][i] = 0.f; xr[j][i] = 0.f; }
  }
#pragma unroll
  for (int j = 0; j < K; j++) lk[j] = false;
  const int t0 = (int)tile * a.tok_tile;
  const int t1 = min(t0 + a.tok_tile, a.n_tokens);
  const int t_end = t1 + K - 1;                     // look-ahead: g of the K-1 tokens after the tile
  // two batches of U tokens in flight, as in the forward
  struct Batch { int p[U]; uint4 x[U], dy[U]; };
  auto load_batch = [&](int tb, Batch& b) {
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int t = min(tb + u, a.n_tokens - 1);
      b.p[u] = a.tok_pred[t];
      b.x[u] = load_raw<true>(a.x, t, a.x_stride, cv);
      b.dy[u] = load_raw<true>(a.dy, t, a.dy_stride, cv);
    }
  };
  auto work_batch = [&](int tb, const Batch& b) {       // (tb - t0) is a multiple of U, hence of K
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int t = tb + u;
      const int slot = u % K;
      if (t < t_end) {
        if (t < a.n_tokens) {
          float dyt[NV];
          unpack_raw<BF16>(b.x[u], xr[slot]);
          unpack_raw<BF16>(b.dy[u], dyt);
          if (t == t0 || b.p[u] != t - 1) rebuild_ring<BF16, K>(a, b.p[u], cv, slot, xr);
#pragma unroll
          for (int i = 0; i < NV; i++) {
            float pre = wt.b[i] + wt.w[K - 1][i] * xr[slot][i];
#pragma unroll
            for (int m = 1; m < K; m++) pre += wt.w[K - 1 - m][i] * xr[ring_back<K>(slot, m)][i];
            gq[slot][i] = a.silu ? dyt[i] * dsilu_f(pre) : dyt[i];
          }
          lk[slot] = b.p[u] == t - 1;
          if (t < t1) {
#pragma unroll
            for (int i = 0; i < NV; i++) {
              db[i] += gq[slot][i];
#pragma unroll
              for (int m = 0; m < K; m++) dw[K - 1 - m][i] += gq[slot][i] * xr[ring_back<K>(slot, m)][i];
            }
          }
        } else {
          lk[slot] = false;
#pragma unroll
          for (int i = 0; i < NV; i++) gq[slot][i] = 0.f;
        }
        const int s = t - (K - 1);                // its g sits K-1 slots back; successor m one slot further on each
        if (s >= t0) {                            // s < t1 by the loop bound
          float dx[NV];
#pragma unroll
          for (int i = 0; i < NV; i++) dx[i] = wt.w[K - 1][i] * gq[ring_back<K>(slot, K - 1)][i];
          bool valid = true;
#pragma unroll
          for (int m = 1; m < K; m++) {
            valid = valid && lk[ring_back<K>(slot, K - 1 - m)];
            if (valid) {
#pragma unroll
              for (int i = 0; i < NV; i++) dx[i] += wt.w[K - 1 - m][i] * gq[ring_back<K>(slot, K - 1 - m)][i];
            }
          }
          store_row<BF16, true>(a.y, s, a.y_stride, cv, dx);
        }
      }
    }
  };
  Batch ba, bb;
  load_batch(t0, ba);
  for (int tb = t0; tb < t_end; tb += 2 * U) {
    load_batch(tb + U, bb);
    work_batch(tb, ba);
    load_batch(tb + 2 * U, ba);
    work_batch(tb + U, bb);
  }
  float* part = a.partial + (int64_t)tile * (K + 1) * a.channels + cv * NV;
#pragma unroll
  for (int j = 0; j < K; j++)
#pragma unroll
    for (int i = 0; i < NV; i++) part[(int64_t)j * a.channels + i] = dw[j][i];
#pragma unroll
  for (int i = 0; i < NV; i++) part[(int64_t)K * a.channels + i] = db[i];
}

// Backward, fix-up: dx of the tokens that have a successor outside the "directly follows" chain.
// Each listed token is recomputed completely (chain part + listed extra successors) and overwrites
// what the fast path stored, so every dx row has one writer last and one rounding.
template <bool BF16, int K>
__device__ __forceinline__ void conv_fix_block(const ConvArgs& a, int64_t block) {
  constexpr int NV = Chan<BF16>::NV;
  const int64_t gid = block * CONV_THREADS + threadIdx.x;
  const int vpr = a.channels / NV;
  const int64_t f = gid / vpr;
  const int cv = (int)(gid - f * vpr);
  if (f >= a.n_fix) return;
  Weights<BF16, K> wt;
  wt.load(a, cv * NV);
  const int s = a.fix_tok[f];
  float dx[NV], g[NV];
#pragma unroll
  for (int i = 0; i < NV; i++) dx[i] = 0.f;
  // successors along a run of directly-following tokens that starts at `first`, whose distance
  // from s is `r`
  auto add_run = [&](int first, int r) {
    for (int m1 = 0; r + m1 < K; m1++) {
      const int t = first + m1;
      if (m1 > 0 && (t >= a.n_tokens || a.tok_pred[t] != t - 1)) break;
      grad_pre_at<BF16, K>(a, wt, t, cv, g);
      const int j = K - 1 - (r + m1);
      // weight row j selected without dynamic register indexing
#pragma unroll
      for (int jj = 0; jj < K; jj++)
        if (jj == j) {
#pragma unroll
          for (int i = 0; i < NV; i++) dx[i] += wt.w[jj][i] * g[i];
        }
    }
  };
  add_run(s, 0);
  for (int e = a.fix_off[f]; e < a.fix_off[f + 1]; e++) add_run(a.fix_t[e], a.fix_r[e]);
  store_row<BF16>(a.y, s, a.y_stride, cv, dx);
}

// dweight[c][j] = sum over tiles of partial[tile][j][c]; dbias[c] = same for j = K.  Fixed order: the tiles are
// cut into RED_SEG consecutive segments, one thread sums one segment of one output in tile order (16 loads in
// flight), and the segment sums are added in segment order -- the same association on every run.  A workgroup
// covers RED_OUT consecutive outputs x RED_SEG segments, so a wavefront reads 256 contiguous bytes per tile.
constexpr int RED_SEG = 4, RED_OUT = CONV_THREADS / RED_SEG;
__device__ __forceinline__ void conv_reduce_block(const float* __restrict__ partial, int n_tiles, int K, int channels,
                                                  float* __restrict__ dweight, float* __restrict__ dbias, int64_t block) {
  __shared__ float seg_sum[RED_SEG][RED_OUT];
  const int o = threadIdx.x % RED_OUT, sg = threadIdx.x / RED_OUT;
  const int64_t n_out = (int64_t)(K + 1) * channels;
  const int64_t gid = block * RED_OUT + o;
  const int per = (n_tiles + RED_SEG - 1) / RED_SEG;
  const int t_lo = min(sg * per, n_tiles), t_hi = min(t_lo + per, n_tiles);
  float acc = 0.f;
  if (gid < n_out) {
    const float* src = partial + gid;
    int t = t_lo;
    for (; t + 16 <= t_hi; t += 16) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; u++) v[u] = src[(int64_t)(t + u) * n_out];
#pragma unroll
      for (int u = 0; u < 16; u++) acc += v[u];
    }
    for (; t < t_hi; t++) acc += src[(int64_t)t * n_out];
  }
  seg_sum[sg][o] = acc;
  __syncthreads();
  if (sg == 0 && gid < n_out) {
    float tot = seg_sum[0][o];
#pragma unroll
    for (int q = 1; q < RED_SEG; q++) tot += seg_sum[q][o];
    const int j = (int)(gid / channels), c = (int)(gid - (int64_t)j * channels);
    if (j < K) dweight[(int64_t)c * K + j] = tot;
    else if (dbias) dbias[c] = tot;
  }
}

// What follows the fast path of the backward, in one launch: the first n_reduce_blocks workgroups sum the
// weight-gradient partials, the others recompute the dx rows of the listed branch-point tokens (the two jobs touch
// different outputs and both only need the fast path to have finished).
template <bool BF16, int K>
__global__ __launch_bounds__(CONV_THREADS) void tree_conv_finish_kernel(ConvArgs a, float* dweight, float* dbias, int n_reduce_blocks) {
  if ((int)blockIdx.x < n_reduce_blocks) conv_reduce_block(a.partial, a.n_tiles, K, a.channels, dweight, dbias, blockIdx.x);
  else conv_fix_block<BF16, K>(a, (int64_t)blockIdx.x - n_reduce_blocks);
}

int pick_tile(int64_t n_tokens, int vpr, int lo, int hi) {
  // enough lanes for the chip (about 1024 workgroups) without making tiles shorter than `lo` tokens
  int tile = hi;
  while (tile > lo && tt::ceil_div(n_tokens, tile) * vpr < (int64_t)1024 * CONV_THREADS) tile >>= 1;
  return tile;
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + CONV_THREADS - 1) / CONV_THREADS); }

template <bool BF16, int K>
hipError_t launch_fwd(const ConvArgs& a, hipStream_t st) {
  tree_conv_fwd_kernel<BF16, K><<<blocks_for((int64_t)a.n_tiles * (a.channels / Chan<BF16>::NV)), CONV_THREADS, 0, st>>>(a);
  return hipGetLastError();
}

template <bool BF16, int K>
hipError_t launch_bwd(const ConvArgs& a, float* dweight, float* dbias, hipStream_t st) {
  const int vpr = a.channels / Chan<BF16>::NV;
  if (a.n_tiles > 0) {
    KernelTimer t(TT_KERNEL_CONV_BWD, st);
    tree_conv_bwd_kernel<BF16, K><<<blocks_for((int64_t)a.n_tiles * vpr), CONV_THREADS, 0, st>>>(a);
  }
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  {
    KernelTimer t(TT_KERNEL_CONV_FIX, st);
    const int64_t n_out = (int64_t)(K + 1) * a.channels;
    const int n_reduce_blocks = (int)((n_out + RED_OUT - 1) / RED_OUT);
    const unsigned n_fix_blocks = a.n_fix > 0 ? blocks_for((int64_t)a.n_fix * vpr) : 0;
    tree_conv_finish_kernel<BF16, K><<<(unsigned)n_reduce_blocks + n_fix_blocks, CONV_THREADS, 0, st>>>(a, dweight, dbias, n_reduce_blocks);
  }
  return hipGetLastError();
}

#define TT_CONV_DISPATCH(FN, ...)                                            \
  switch (kernel_size) {                                                     \
    case 2: return bf16 ? FN<true, 2>(__VA_ARGS__) : FN<false, 2>(__VA_ARGS__); \
    case 3: return bf16 ? FN<true, 3>(__VA_ARGS__) : FN<false, 3>(__VA_ARGS__); \
    case 4: return bf16 ? FN<true, 4>(__VA_ARGS__) : FN<false, 4>(__VA_ARGS__); \
    default: return hipErrorInvalidValue;                                    \
  }

}  // namespace

int conv_bwd_tile(int64_t n_tokens, int channels, bool bf16) { return pick_tile(n_tokens, channels / (bf16 ? 8 : 4), 32, 256); }

size_t conv_bwd_workspace(int64_t n_tokens, int channels, int kernel_size, bool bf16) {
  const int tile = conv_bwd_tile(n_tokens, channels, bf16);
  return (size_t)tt::ceil_div(n_tokens, tile) * (size_t)(kernel_size + 1) * (size_t)channels * sizeof(float) + 256;
}

hipError_t conv_fwd(int64_t n_tokens, int channels, int kernel_size, bool bf16, bool silu, const void* x, int64_t x_stride_bytes,
                    const float* weight, const float* bias, const int32_t* tok_pred, void* y, int64_t y_stride_bytes,
                    hipStream_t st) {
  if (n_tokens == 0) return hipSuccess;
  ConvArgs a{};
  a.n_tokens = (int)n_tokens; a.channels = channels; a.silu = silu ? 1 : 0;
  a.tok_tile = pick_tile(n_tokens, channels / (bf16 ? 8 : 4), 16, 64);
  a.n_tiles = (int)tt::ceil_div(n_tokens, a.tok_tile);
  a.x = x; a.x_stride = x_stride_bytes; a.weight = weight; a.bias = bias; a.tok_pred = tok_pred;
  a.y = y; a.y_stride = y_stride_bytes;
  KernelTimer t(TT_KERNEL_CONV_FWD, st);
  TT_CONV_DISPATCH(launch_fwd, a, st)
}

hipError_t conv_bwd(int64_t n_tokens, int channels, int kernel_size, bool bf16, bool silu, const void* x, int64_t x_stride_bytes,
                    const float* weight, const float* bias, const int32_t* tok_pred, const void* dy, int64_t dy_stride_bytes,
                    int n_fix, const int32_t* fix_tok, const int32_t* fix_off, const int32_t* fix_t, const int32_t* fix_r,
                    void* dx, int64_t dx_stride_bytes, float* dweight, float* dbias, void* workspace, hipStream_t st) {
  ConvArgs a{};
  a.n_tokens = (int)n_tokens; a.channels = channels; a.silu = silu ? 1 : 0;
  a.tok_tile = conv_bwd_tile(n_tokens, channels, bf16);
  a.n_tiles = (int)tt::ceil_div(n_tokens, a.tok_tile);
  a.x = x; a.x_stride = x_stride_bytes; a.weight = weight; a.bias = bias; a.tok_pred = tok_pred;
  a.y = dx; a.y_stride = dx_stride_bytes; a.dy = dy; a.dy_stride = dy_stride_bytes;
  a.partial = (float*)workspace;
  a.n_fix = n_fix; a.fix_tok = fix_tok; a.fix_off = fix_off; a.fix_t = fix_t; a.fix_r = fix_r;
  TT_CONV_DISPATCH(launch_bwd, a, dweight, dbias, st)
}

}  // namespace tt
