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

template <bool BF16>
__device__ __forceinline__ void load_row(const void* base, int64_t row, int64_t stride_bytes, int cv, float (&v)[Chan<BF16>::NV]) {
  const char* p = (const char*)base + row * stride_bytes + (int64_t)cv * 16;
  if (BF16) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      v[2 * i] = __uint_as_float(w[i] << 16);
      v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  } else {
    const float4 f = *reinterpret_cast<const float4*>(p);
    v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
  }
}

typedef float f32x8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));

template <bool BF16>
__device__ __forceinline__ void store_row(void* base, int64_t row, int64_t stride_bytes, int cv, const float (&v)[Chan<BF16>::NV]) {
  char* p = (char*)base + row * stride_bytes + (int64_t)cv * 16;
  if (BF16) {
    f32x8v f;
#pragma unroll
    for (int i = 0; i < 8; i++) f[i] = v[i];
    const bf16x8v b = __builtin_convertvector(f, bf16x8v);       // round to nearest even
    *reinterpret_cast<uint4*>(p) = __builtin_bit_cast(uint4, b);
  } else {
    *reinterpret_cast<float4*>(p) = float4{v[0], v[1], v[2], v[3]};
  }
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

template <bool BF16, int K>
__device__ __forceinline__ void shift_window(float (&win)[K > 1 ? K - 1 : 1][Chan<BF16>::NV], const float (&xt)[Chan<BF16>::NV]) {
  constexpr int NV = Chan<BF16>::NV;
#pragma unroll
  for (int m = K - 2; m >= 1; m--)
#pragma unroll
    for (int i = 0; i < NV; i++) win[m][i] = win[m - 1][i];
  if (K > 1)
#pragma unroll
    for (int i = 0; i < NV; i++) win[0][i] = xt[i];
}

constexpr int CONV_U = 4;      // tokens whose loads are issued together

template <bool BF16, int K>
__global__ __launch_bounds__(CONV_THREADS) void tree_conv_fwd_kernel(ConvArgs a) {
  constexpr int NV = Chan<BF16>::NV;
  const int64_t gid = (int64_t)blockIdx.x * CONV_THREADS + threadIdx.x;
  const int vpr = a.channels / NV;
  const int64_t tile = gid / vpr;
  const int cv = (int)(gid - tile * vpr);
  if (tile >= a.n_tiles) return;
  Weights<BF16, K> wt;
  wt.load(a, cv * NV);
  float win[K > 1 ? K - 1 : 1][NV];
  const int t0 = (int)tile * a.tok_tile;
  const int t1 = min(t0 + a.tok_tile, a.n_tokens);
  for (int tb = t0; tb < t1; tb += CONV_U) {
    int p[CONV_U];
    float xt[CONV_U][NV];
#pragma unroll
    for (int u = 0; u < CONV_U; u++) {
      const int t = min(tb + u, t1 - 1);
      p[u] = a.tok_pred[t];
      load_row<BF16>(a.x, t, a.x_stride, cv, xt[u]);
    }
#pragma unroll
    for (int u = 0; u < CONV_U; u++) {
      const int t = tb + u;
      if (t < t1) {
        float pre[NV];
        if (t == t0 || p[u] != t - 1) rebuild_window<BF16, K>(a, p[u], cv, win);
        pre_activation<BF16, K>(wt, xt[u], win, pre);
        if (a.silu) {
#pragma unroll
          for (int i = 0; i < NV; i++) pre[i] = silu_f(pre[i]);
        }
        store_row<BF16>(a.y, t, a.y_stride, cv, pre);
        shift_window<BF16, K>(win, xt[u]);
      }
    }
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
  const int64_t gid = (int64_t)blockIdx.x * CONV_THREADS + threadIdx.x;
  const int vpr = a.channels / NV;
  const int64_t tile = gid / vpr;
  const int cv = (int)(gid - tile * vpr);
  if (tile >= a.n_tiles) return;
  Weights<BF16, K> wt;
  wt.load(a, cv * NV);
  float win[K > 1 ? K - 1 : 1][NV];
  float gq[K][NV];          // gq[j] = g[t - j]
  bool lk[K];               // lk[j] = token t-j directly follows token t-j-1 on its sequence
  float dw[K][NV], db[NV];
#pragma unroll
  for (int i = 0; i < NV; i++) {
    db[i] = 0.f;
#pragma unroll
    for (int j = 0; j < K; j++) { dw[j][i] = 0.f; gq[j][i] = 0.f; }
  }
#pragma unroll
  for (int j = 0; j < K; j++) lk[j] = false;
  const int t0 = (int)tile * a.tok_tile;
  const int t1 = min(t0 + a.tok_tile, a.n_tokens);
  const int t_end = t1 + K - 1;                     // look-ahead: g of the K-1 tokens after the tile
  for (int tb = t0; tb < t_end; tb += CONV_U) {
    int p[CONV_U];
    float xt[CONV_U][NV], dyt[CONV_U][NV];
#pragma unroll
    for (int u = 0; u < CONV_U; u++) {
      const int t = min(tb + u, a.n_tokens - 1);
      p[u] = a.tok_pred[t];
      load_row<BF16>(a.x, t, a.x_stride, cv, xt[u]);
      load_row<BF16>(a.dy, t, a.dy_stride, cv, dyt[u]);
    }
#pragma unroll
    for (int u = 0; u < CONV_U; u++) {
      const int t = tb + u;
      if (t >= t_end) break;
      // shift the ring
#pragma unroll
      for (int j = K - 1; j >= 1; j--) {
        lk[j] = lk[j - 1];
#pragma unroll
        for (int i = 0; i < NV; i++) gq[j][i] = gq[j - 1][i];
      }
      if (t < a.n_tokens) {
        float pre[NV];
        if (t == t0 || p[u] != t - 1) rebuild_window<BF16, K>(a, p[u], cv, win);
        pre_activation<BF16, K>(wt, xt[u], win, pre);
#pragma unroll
        for (int i = 0; i < NV; i++) gq[0][i] = a.silu ? dyt[u][i] * dsilu_f(pre[i]) : dyt[u][i];
        lk[0] = p[u] == t - 1;
        if (t < t1) {
#pragma unroll
          for (int i = 0; i < NV; i++) {
            db[i] += gq[0][i];
            dw[K - 1][i] += gq[0][i] * xt[u][i];
#pragma unroll
            for (int m = 1; m < K; m++) dw[K - 1 - m][i] += gq[0][i] * win[m - 1][i];
          }
        }
        shift_window<BF16, K>(win, xt[u]);
      } else {
        lk[0] = false;
#pragma unroll
        for (int i = 0; i < NV; i++) gq[0][i] = 0.f;
      }
      const int s = t - (K - 1);
      if (s >= t0) {          // s < t1 by the loop bound
        float dx[NV];
#pragma unroll
        for (int i = 0; i < NV; i++) dx[i] = wt.w[K - 1][i] * gq[K - 1][i];
        bool valid = true;
#pragma unroll
        for (int m = 1; m < K; m++) {
          valid = valid && lk[K - 1 - m];
          if (valid) {
#pragma unroll
            for (int i = 0; i < NV; i++) dx[i] += wt.w[K - 1 - m][i] * gq[K - 1 - m][i];
          }
        }
        store_row<BF16>(a.y, s, a.y_stride, cv, dx);
      }
    }
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
__global__ __launch_bounds__(CONV_THREADS) void tree_conv_fix_kernel(ConvArgs a) {
  constexpr int NV = Chan<BF16>::NV;
  const int64_t gid = (int64_t)blockIdx.x * CONV_THREADS + threadIdx.x;
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

// dweight[c][j] = sum over tiles of partial[tile][j][c]; dbias[c] = same for j = K.  Fixed order.
__global__ __launch_bounds__(CONV_THREADS) void tree_conv_reduce_kernel(const float* __restrict__ partial, int n_tiles, int K,
                                                                        int channels, float* __restrict__ dweight,
                                                                        float* __restrict__ dbias) {
  const int64_t gid = (int64_t)blockIdx.x * CONV_THREADS + threadIdx.x;
  if (gid >= (int64_t)(K + 1) * channels) return;
  const int j = (int)(gid / channels), c = (int)(gid - (int64_t)j * channels);
  const float* src = partial + (int64_t)j * channels + c;
  const int64_t step = (int64_t)(K + 1) * channels;
  float acc = 0.f;
  int t = 0;
  for (; t + 8 <= n_tiles; t += 8) {               // eight loads in flight, added in tile order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; u++) v[u] = src[(t + u) * step];
#pragma unroll
    for (int u = 0; u < 8; u++) acc += v[u];
  }
  for (; t < n_tiles; t++) acc += src[t * step];
  if (j < K) dweight[(int64_t)c * K + j] = acc;
  else if (dbias) dbias[c] = acc;
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
  const int64_t lanes = (int64_t)a.n_tiles * (a.channels / Chan<BF16>::NV);
  tree_conv_fwd_kernel<BF16, K><<<blocks_for(lanes), CONV_THREADS, 0, st>>>(a);
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
  if (a.n_fix > 0) {
    KernelTimer t(TT_KERNEL_CONV_FIX, st);
    tree_conv_fix_kernel<BF16, K><<<blocks_for((int64_t)a.n_fix * vpr), CONV_THREADS, 0, st>>>(a);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  }
  {
    KernelTimer t(TT_KERNEL_CONV_FIX, st);
    tree_conv_reduce_kernel<<<blocks_for((int64_t)(K + 1) * a.channels), CONV_THREADS, 0, st>>>(a.partial, a.n_tiles, K, a.channels,
                                                                                                 dweight, dbias);
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
