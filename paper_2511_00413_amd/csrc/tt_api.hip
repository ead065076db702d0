// C ABI entry points of the device calls: argument validation on the host, then dispatch to the
// kernels.  Nothing is launched unless every check passes.
#include <hip/hip_runtime.h>
#include <climits>
#include <cmath>
#include <mutex>
#include "tt_internal.h"
#include "tt_kernels.h"

namespace {

using tt::fail;

struct Checked {
  tt::AttnArgs a;
  bool bf16;
  bool use_mfma;
};

size_t delta_bytes(const tt_attn_desc* d) {
  return ((size_t)d->hq * (size_t)d->n_q * sizeof(float) + 255) & ~(size_t)255;
}

tt_status check_desc(const tt_attn_desc* d) { return tt::check_attn_desc(d); }

}  // namespace

tt_status tt::check_attn_desc(const tt_attn_desc* d) {
  if (!d) return fail(TT_ERR_NULL, "desc is NULL");
  if (d->dtype != TT_DTYPE_BF16 && d->dtype != TT_DTYPE_FP32) return fail(TT_ERR_DTYPE, "unknown dtype %d", d->dtype);
  if (d->n_q < 0 || d->n_prefix < 0 || (int64_t)d->n_q + d->n_prefix >= INT32_MAX)
    return fail(TT_ERR_SHAPE, "n_q=%d n_prefix=%d out of range", d->n_q, d->n_prefix);
  if (d->hq <= 0 || d->hkv <= 0 || d->hq % d->hkv != 0 || d->hq > 65535)
    return fail(TT_ERR_SHAPE, "hq=%d must be a positive multiple of hkv=%d (and <= 65535)", d->hq, d->hkv);
  if (d->d <= 0 || d->d > 256 || d->d % 8 != 0) return fail(TT_ERR_SHAPE, "d=%d must be a multiple of 8 in [8, 256]", d->d);
  if (!(d->scale > 0.f) || !std::isfinite(d->scale)) return fail(TT_ERR_SHAPE, "scale must be positive and finite");
  if (d->flags & ~TT_FLAG_REFERENCE_KERNELS) return fail(TT_ERR_UNSUPPORTED, "unknown flags 0x%x", d->flags);
  const int64_t qs = d->q_stride_tok ? d->q_stride_tok : (int64_t)d->hq * d->d;
  const int64_t ks = d->k_stride_tok ? d->k_stride_tok : (int64_t)d->hkv * d->d;
  const int64_t vs = d->v_stride_tok ? d->v_stride_tok : (int64_t)d->hkv * d->d;
  if (qs < (int64_t)d->hq * d->d || ks < (int64_t)d->hkv * d->d || vs < (int64_t)d->hkv * d->d)
    return fail(TT_ERR_SHAPE, "a token stride is smaller than heads*d");
  if (qs % 8 || ks % 8 || vs % 8) return fail(TT_ERR_ALIGN, "token strides must be multiples of 8 elements");
  return TT_OK;
}

namespace {

bool mfma_supported(const tt_attn_desc* d) {
  return d->dtype == TT_DTYPE_BF16 && d->d == 128 && !(d->flags & TT_FLAG_REFERENCE_KERNELS);
}

tt_status check_common(const tt_attn_desc* d, const void* q, const void* k_own, const void* v_own,
                       const void* k_prefix, const void* v_prefix, const int32_t* kend,
                       const int32_t* kt_min, const int32_t* kt_max, Checked& c) {
  if (tt_status s = check_desc(d)) return s;
  if (d->n_q > 0 && (!q || !k_own || !v_own)) return fail(TT_ERR_NULL, "q / k_own / v_own is NULL");
  if ((int64_t)d->n_q + d->n_prefix > 0 && (!kend || !kt_min || !kt_max)) return fail(TT_ERR_NULL, "kend / kt_min / kt_max is NULL");
  if ((d->n_prefix > 0) != (k_prefix != nullptr) || (d->n_prefix > 0) != (v_prefix != nullptr))
    return fail(TT_ERR_NULL, "k_prefix / v_prefix must be given exactly when n_prefix > 0");
  const void* ptrs[] = {q, k_own, v_own, k_prefix, v_prefix};
  for (const void* p : ptrs)
    if (!tt::aligned16(p)) return fail(TT_ERR_ALIGN, "device pointer %p is not 16-byte aligned", p);
  tt::AttnArgs& a = c.a;
  a = tt::AttnArgs{};
  a.n_q = d->n_q; a.n_prefix = d->n_prefix; a.hq = d->hq; a.hkv = d->hkv; a.d = d->d;
  a.scale = d->scale;
  a.q_stride = d->q_stride_tok ? d->q_stride_tok : (int64_t)d->hq * d->d;
  a.k_stride = d->k_stride_tok ? d->k_stride_tok : (int64_t)d->hkv * d->d;
  a.v_stride = d->v_stride_tok ? d->v_stride_tok : (int64_t)d->hkv * d->d;
  a.q = q; a.k_own = k_own; a.v_own = v_own; a.k_prefix = k_prefix; a.v_prefix = v_prefix;
  a.kend = kend; a.kt_min = kt_min; a.kt_max = kt_max;
  c.bf16 = d->dtype == TT_DTYPE_BF16;
  c.use_mfma = mfma_supported(d);
  return TT_OK;
}

tt_status hip_result(hipError_t e, const char* what) {
  if (e == hipSuccess) return TT_OK;
  return fail(TT_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

extern "C" size_t tt_tree_attn_workspace(const tt_attn_desc* desc, int32_t backward) {
  tt::clear_error();
  if (check_desc(desc) != TT_OK) return 0;
  size_t bytes = 256;                         // never 0 for a valid descriptor
  if (backward) bytes += delta_bytes(desc);
  if (mfma_supported(desc)) bytes += tt::mfma_attn_workspace(desc->n_q, desc->n_prefix, desc->hq, desc->hkv, desc->d, backward != 0);
  return bytes;
}

extern "C" tt_status tt_tree_attn_fwd(const tt_attn_desc* desc, const void* q, const void* k_own, const void* v_own,
                                      const void* k_prefix, const void* v_prefix,
                                      const int32_t* kend, const int32_t* kt_min, const int32_t* kt_max,
                                      void* o, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  tt::clear_error();
  Checked c;
  if (tt_status s = check_common(desc, q, k_own, v_own, k_prefix, v_prefix, kend, kt_min, kt_max, c)) return s;
  if (desc->n_q > 0 && (!o || !lse)) return fail(TT_ERR_NULL, "o / lse is NULL");
  if (!tt::aligned16(o)) return fail(TT_ERR_ALIGN, "o is not 16-byte aligned");
  const size_t need = tt_tree_attn_workspace(desc, 0);
  if (!workspace || workspace_bytes < need || !tt::aligned16(workspace))
    return fail(TT_ERR_WORKSPACE, "forward needs %zu bytes of 16-byte aligned workspace, got %zu", need, workspace_bytes);
  c.a.o = o; c.a.lse = lse;
  c.a.workspace = workspace; c.a.workspace_bytes = workspace_bytes;
  hipStream_t st = (hipStream_t)stream;
  if (c.use_mfma) return hip_result(tt::mfma_attn_fwd(c.a, st), "tree_attn_fwd");
  return hip_result(tt::ref_attn_fwd(c.a, c.bf16, st), "tree_attn_fwd (reference kernels)");
}

extern "C" tt_status tt_tree_attn_bwd(const tt_attn_desc* desc, const void* q, const void* k_own, const void* v_own,
                                      const void* k_prefix, const void* v_prefix,
                                      const int32_t* kend, const int32_t* kt_min, const int32_t* kt_max,
                                      const void* o, const void* d_o, const float* lse,
                                      void* dq, void* dk_own, void* dv_own,
                                      float* dk_prefix_acc, float* dv_prefix_acc,
                                      void* workspace, size_t workspace_bytes, void* stream) {
  tt::clear_error();
  Checked c;
  if (tt_status s = check_common(desc, q, k_own, v_own, k_prefix, v_prefix, kend, kt_min, kt_max, c)) return s;
  if (desc->n_q > 0 && (!o || !d_o || !lse || !dq || !dk_own || !dv_own)) return fail(TT_ERR_NULL, "o / d_o / lse / dq / dk_own / dv_own is NULL");
  if ((desc->n_prefix > 0) != (dk_prefix_acc != nullptr) || (desc->n_prefix > 0) != (dv_prefix_acc != nullptr))
    return fail(TT_ERR_NULL, "dk_prefix_acc / dv_prefix_acc must be given exactly when n_prefix > 0");
  const void* ptrs[] = {o, d_o, dq, dk_own, dv_own, dk_prefix_acc, dv_prefix_acc};
  for (const void* p : ptrs)
    if (!tt::aligned16(p)) return fail(TT_ERR_ALIGN, "device pointer %p is not 16-byte aligned", p);
  const size_t need = tt_tree_attn_workspace(desc, 1);
  if (!workspace || workspace_bytes < need || !tt::aligned16(workspace))
    return fail(TT_ERR_WORKSPACE, "backward needs %zu bytes of 16-byte aligned workspace, got %zu", need, workspace_bytes);
  c.a.o = const_cast<void*>(o); c.a.lse = const_cast<float*>(lse); c.a.d_o = d_o;
  c.a.dq = dq; c.a.dk_own = dk_own; c.a.dv_own = dv_own;
  c.a.dk_prefix_acc = dk_prefix_acc; c.a.dv_prefix_acc = dv_prefix_acc;
  c.a.delta = (float*)workspace;
  c.a.neg_lse2 = nullptr;                      // carved out of the remaining workspace by the MFMA path
  c.a.workspace = (char*)workspace + delta_bytes(desc);
  c.a.workspace_bytes = workspace_bytes - delta_bytes(desc);
  hipStream_t st = (hipStream_t)stream;
  if (c.use_mfma) return hip_result(tt::mfma_attn_bwd(c.a, st), "tree_attn_bwd");
  return hip_result(tt::ref_attn_bwd(c.a, c.bf16, st), "tree_attn_bwd (reference kernels)");
}

extern "C" tt_status tt_tree_weighted_logprob(int64_t n_rows, int32_t vocab, int32_t dtype, const void* logits,
                                              int64_t row_stride, const int32_t* target, const float* weight,
                                              float* logp, float* lse, float* loss_acc, void* stream) {
  tt::clear_error();
  if (dtype != TT_DTYPE_BF16 && dtype != TT_DTYPE_FP32) return fail(TT_ERR_DTYPE, "unknown dtype %d", dtype);
  if (n_rows < 0 || n_rows > 0x7fffffffLL) return fail(TT_ERR_SHAPE, "n_rows=%lld out of range", (long long)n_rows);
  if (vocab <= 0) return fail(TT_ERR_SHAPE, "vocab=%d must be positive", vocab);
  if (row_stride == 0) row_stride = vocab;
  if (row_stride < vocab) return fail(TT_ERR_SHAPE, "row_stride=%lld is smaller than vocab=%d", (long long)row_stride, vocab);
  if (n_rows > 0 && (!logits || !target || !logp)) return fail(TT_ERR_NULL, "logits / target / logp is NULL");
  const size_t es = dtype == TT_DTYPE_BF16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(logits) % es) return fail(TT_ERR_ALIGN, "logits is not aligned to its element size");
  return hip_result(tt::weighted_logprob(n_rows, vocab, dtype == TT_DTYPE_BF16, logits, row_stride, target, weight,
                                         logp, lse, loss_acc, (hipStream_t)stream),
                    "tree_weighted_logprob");
}

extern "C" tt_status tt_tree_weighted_logprob_bwd(int64_t n_rows, int32_t vocab, int32_t dtype, const void* logits,
                                                  int64_t row_stride, const int32_t* target, const float* weight,
                                                  const float* lse, float grad_scale, void* dlogits,
                                                  int64_t dlogits_row_stride, void* stream) {
  tt::clear_error();
  if (dtype != TT_DTYPE_BF16 && dtype != TT_DTYPE_FP32) return fail(TT_ERR_DTYPE, "unknown dtype %d", dtype);
  if (n_rows < 0 || n_rows > 0x7fffffffLL) return fail(TT_ERR_SHAPE, "n_rows=%lld out of range", (long long)n_rows);
  if (vocab <= 0) return fail(TT_ERR_SHAPE, "vocab=%d must be positive", vocab);
  if (row_stride == 0) row_stride = vocab;
  if (dlogits_row_stride == 0) dlogits_row_stride = vocab;
  if (row_stride < vocab || dlogits_row_stride < vocab)
    return fail(TT_ERR_SHAPE, "row strides %lld / %lld are smaller than vocab=%d", (long long)row_stride,
                (long long)dlogits_row_stride, vocab);
  if (!std::isfinite(grad_scale)) return fail(TT_ERR_SHAPE, "grad_scale must be finite");
  if (n_rows > 0 && (!logits || !target || !lse || !dlogits)) return fail(TT_ERR_NULL, "logits / target / lse / dlogits is NULL");
  if (dlogits == logits && dlogits_row_stride != row_stride)
    return fail(TT_ERR_SHAPE, "dlogits may alias logits only with equal row strides");
  const size_t es = dtype == TT_DTYPE_BF16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(logits) % es || reinterpret_cast<uintptr_t>(dlogits) % es)
    return fail(TT_ERR_ALIGN, "logits / dlogits is not aligned to its element size");
  return hip_result(tt::weighted_logprob_bwd(n_rows, vocab, dtype == TT_DTYPE_BF16, logits, row_stride, target, weight,
                                             lse, grad_scale, dlogits, dlogits_row_stride, (hipStream_t)stream),
                    "tree_weighted_logprob_bwd");
}

extern "C" tt_status tt_tree_weighted_logprob_fwd_bwd(int64_t n_rows, int32_t vocab, int32_t dtype, const void* logits,
                                                      int64_t row_stride, const int32_t* target, const float* weight,
                                                      float grad_scale, float* logp, float* lse, float* loss_acc,
                                                      void* dlogits, int64_t dlogits_row_stride, void* stream) {
  tt::clear_error();
  if (dtype != TT_DTYPE_BF16 && dtype != TT_DTYPE_FP32) return fail(TT_ERR_DTYPE, "unknown dtype %d", dtype);
  if (n_rows < 0 || n_rows > 0x7fffffffLL) return fail(TT_ERR_SHAPE, "n_rows=%lld out of range", (long long)n_rows);
  if (vocab <= 0) return fail(TT_ERR_SHAPE, "vocab=%d must be positive", vocab);
  if (row_stride == 0) row_stride = vocab;
  if (dlogits_row_stride == 0) dlogits_row_stride = vocab;
  if (row_stride < vocab || dlogits_row_stride < vocab)
    return fail(TT_ERR_SHAPE, "row strides %lld / %lld are smaller than vocab=%d", (long long)row_stride,
                (long long)dlogits_row_stride, vocab);
  if (!std::isfinite(grad_scale)) return fail(TT_ERR_SHAPE, "grad_scale must be finite");
  if (n_rows > 0 && (!logits || !target || !logp || !lse || !dlogits))
    return fail(TT_ERR_NULL, "logits / target / logp / lse / dlogits is NULL");
  if (dlogits == logits && dlogits_row_stride != row_stride)
    return fail(TT_ERR_SHAPE, "dlogits may alias logits only with equal row strides");
  const size_t es = dtype == TT_DTYPE_BF16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(logits) % es || reinterpret_cast<uintptr_t>(dlogits) % es)
    return fail(TT_ERR_ALIGN, "logits / dlogits is not aligned to its element size");
  const bool bf16 = dtype == TT_DTYPE_BF16;
  hipStream_t st = (hipStream_t)stream;
  if (tt::weighted_logprob_fused_ok(bf16, logits, row_stride, dlogits, dlogits_row_stride))
    return hip_result(tt::weighted_logprob_fused(n_rows, vocab, bf16, logits, row_stride, target, weight, grad_scale, logp, lse,
                                                 loss_acc, dlogits, dlogits_row_stride, st),
                      "tree_weighted_logprob_fwd_bwd");
  // rows off the 16-byte grid: the two passes one after the other
  if (tt_status s = hip_result(tt::weighted_logprob(n_rows, vocab, bf16, logits, row_stride, target, weight, logp, lse, loss_acc, st),
                               "tree_weighted_logprob_fwd_bwd (forward pass)"))
    return s;
  return hip_result(tt::weighted_logprob_bwd(n_rows, vocab, bf16, logits, row_stride, target, weight, lse, grad_scale, dlogits,
                                             dlogits_row_stride, st),
                    "tree_weighted_logprob_fwd_bwd (backward pass)");
}

extern "C" tt_status tt_tree_rope(int64_t n_tokens, int32_t n_heads, int32_t d, int32_t dtype, const void* x,
                                  int64_t x_stride_tok, const int32_t* tok_pos, float theta_base, int32_t inverse,
                                  void* y, int64_t y_stride_tok, void* stream) {
  tt::clear_error();
  if (dtype != TT_DTYPE_BF16 && dtype != TT_DTYPE_FP32) return fail(TT_ERR_DTYPE, "unknown dtype %d", dtype);
  if (n_tokens < 0 || n_tokens > 0x7fffffffLL) return fail(TT_ERR_SHAPE, "n_tokens=%lld out of range", (long long)n_tokens);
  const int epv = dtype == TT_DTYPE_BF16 ? 8 : 4;
  if (n_heads <= 0 || d <= 0 || d > 1024 || d % (2 * epv) != 0 || (int64_t)n_heads * d > 65536)
    return fail(TT_ERR_SHAPE, "n_heads=%d, d=%d: d must be a multiple of %d in [%d, 1024] and n_heads * d <= 65536", n_heads, d,
                2 * epv, 2 * epv);
  if (!(theta_base > 1.f) || !std::isfinite(theta_base)) return fail(TT_ERR_SHAPE, "theta_base must be finite and > 1");
  if (x_stride_tok == 0) x_stride_tok = (int64_t)n_heads * d;
  if (y_stride_tok == 0) y_stride_tok = (int64_t)n_heads * d;
  if (x_stride_tok < (int64_t)n_heads * d || y_stride_tok < (int64_t)n_heads * d || x_stride_tok % epv || y_stride_tok % epv)
    return fail(TT_ERR_SHAPE, "token strides %lld / %lld must be >= n_heads * d and a multiple of %d elements",
                (long long)x_stride_tok, (long long)y_stride_tok, epv);
  if (n_tokens > 0 && (!x || !y || !tok_pos)) return fail(TT_ERR_NULL, "x / y / tok_pos is NULL");
  if (!tt::aligned16(x) || !tt::aligned16(y)) return fail(TT_ERR_ALIGN, "x / y is not 16-byte aligned");
  if (x == y && x_stride_tok != y_stride_tok) return fail(TT_ERR_SHAPE, "y may alias x only with equal token strides");
  return hip_result(tt::rope(n_tokens, n_heads, d, dtype == TT_DTYPE_BF16, x, x_stride_tok, tok_pos, theta_base, inverse != 0,
                             y, y_stride_tok, (hipStream_t)stream),
                    "tree_rope");
}

namespace {

struct ConvChecked { bool bf16; int64_t xs, ys; };

// Common validation of the convolution calls; strides come back in bytes.
tt_status check_conv(int64_t n_tokens, int32_t channels, int32_t kernel_size, int32_t dtype, int32_t activation,
                     const void* x, int64_t x_stride, const float* weight, const int32_t* tok_pred, const void* y,
                     int64_t y_stride, ConvChecked& c) {
  if (dtype != TT_DTYPE_BF16 && dtype != TT_DTYPE_FP32) return fail(TT_ERR_DTYPE, "unknown dtype %d", dtype);
  if (n_tokens < 0 || n_tokens >= INT32_MAX) return fail(TT_ERR_SHAPE, "n_tokens=%lld out of range", (long long)n_tokens);
  if (kernel_size < 2 || kernel_size > 4) return fail(TT_ERR_UNSUPPORTED, "kernel_size=%d: only 2, 3, 4 are built", kernel_size);
  if (activation != 0 && activation != 1) return fail(TT_ERR_UNSUPPORTED, "activation=%d: 0 (none) or 1 (SiLU)", activation);
  const int epv = dtype == TT_DTYPE_BF16 ? 8 : 4;
  if (channels <= 0 || channels % epv) return fail(TT_ERR_SHAPE, "channels=%d must be a positive multiple of %d", channels, epv);
  if (x_stride == 0) x_stride = channels;
  if (y_stride == 0) y_stride = channels;
  if (x_stride < channels || y_stride < channels || x_stride % epv || y_stride % epv)
    return fail(TT_ERR_ALIGN, "token strides %lld / %lld must be >= channels and a multiple of %d elements", (long long)x_stride,
                (long long)y_stride, epv);
  if (!weight) return fail(TT_ERR_NULL, "weight is NULL");
  if (n_tokens > 0 && (!x || !y || !tok_pred)) return fail(TT_ERR_NULL, "x / output / tok_pred is NULL");
  if (!tt::aligned16(x) || !tt::aligned16(y)) return fail(TT_ERR_ALIGN, "a tensor pointer is not 16-byte aligned");
  c.bf16 = dtype == TT_DTYPE_BF16;
  const int64_t esz = c.bf16 ? 2 : 4;
  c.xs = x_stride * esz; c.ys = y_stride * esz;
  return TT_OK;
}

}  // namespace

extern "C" tt_status tt_tree_conv_fwd(int64_t n_tokens, int32_t channels, int32_t kernel_size, int32_t dtype, int32_t activation,
                                      const void* x, int64_t x_stride_tok, const float* weight, const float* bias,
                                      const int32_t* tok_pred, void* y, int64_t y_stride_tok, void* stream) {
  tt::clear_error();
  ConvChecked c;
  if (tt_status s = check_conv(n_tokens, channels, kernel_size, dtype, activation, x, x_stride_tok, weight, tok_pred, y, y_stride_tok, c))
    return s;
  if (n_tokens > 0 && x == y) return fail(TT_ERR_SHAPE, "y may not alias x (later tokens read earlier rows of x)");
  return hip_result(tt::conv_fwd(n_tokens, channels, kernel_size, c.bf16, activation == 1, x, c.xs, weight, bias, tok_pred, y, c.ys,
                                 (hipStream_t)stream),
                    "tree_conv_fwd");
}

extern "C" size_t tt_tree_conv_bwd_workspace(int64_t n_tokens, int32_t channels, int32_t kernel_size, int32_t dtype) {
  tt::clear_error();
  if ((dtype != TT_DTYPE_BF16 && dtype != TT_DTYPE_FP32) || n_tokens < 0 || n_tokens >= INT32_MAX || channels <= 0 ||
      kernel_size < 2 || kernel_size > 4)
    return 0;
  return tt::conv_bwd_workspace(n_tokens, channels, kernel_size, dtype == TT_DTYPE_BF16);
}

namespace {

// Arguments of a convolution backward call (tt_tree_conv_bwd and tt_tree_conv_bwd_static share validation and launch).
struct ConvBwdCall {
  int64_t n_tokens; int32_t channels, kernel_size, dtype, activation;
  const void* x; int64_t x_stride_tok; const float *weight, *bias; const int32_t* tok_pred;
  const void* dy; int64_t dy_stride_tok;
  int32_t n_fix; const int32_t *fix_tok, *fix_off, *fix_t, *fix_r;
  void* dx; int64_t dx_stride_tok; float *dweight, *dbias;
};

// Host-side checks; on success `need` is the scratch the kernels use for this shape.
tt_status conv_bwd_validate(const ConvBwdCall& k, ConvChecked& c, ConvChecked& cd, size_t& need) {
  if (tt_status s = check_conv(k.n_tokens, k.channels, k.kernel_size, k.dtype, k.activation, k.x, k.x_stride_tok, k.weight,
                               k.tok_pred, k.dx, k.dx_stride_tok, c))
    return s;
  if (tt_status s = check_conv(k.n_tokens, k.channels, k.kernel_size, k.dtype, k.activation, k.dy, k.dy_stride_tok, k.weight,
                               k.tok_pred, k.dx, k.dx_stride_tok, cd))
    return s;
  if (!k.dweight) return fail(TT_ERR_NULL, "dweight is NULL");
  if (k.n_fix < 0 || (k.n_fix > 0 && (!k.fix_tok || !k.fix_off || !k.fix_t || !k.fix_r)))
    return fail(TT_ERR_NULL, "n_fix=%d with a NULL list", k.n_fix);
  if (k.n_tokens > 0 && (k.dx == k.x || k.dx == k.dy)) return fail(TT_ERR_SHAPE, "dx may not alias x or dy");
  need = tt::conv_bwd_workspace(k.n_tokens, k.channels, k.kernel_size, c.bf16);
  return TT_OK;
}

tt_status conv_bwd_launch(const ConvBwdCall& k, const ConvChecked& c, const ConvChecked& cd, void* workspace, void* stream,
                          const char* what) {
  return hip_result(tt::conv_bwd(k.n_tokens, k.channels, k.kernel_size, c.bf16, k.activation == 1, k.x, c.xs, k.weight, k.bias,
                                 k.tok_pred, k.dy, cd.xs, k.n_fix, k.fix_tok, k.fix_off, k.fix_t, k.fix_r, k.dx, c.ys, k.dweight,
                                 k.dbias, workspace, (hipStream_t)stream),
                    what);
}

// ---- static scratch of the allocation-free variant ---------------------------------------------------------
// One array per GPU, part of the code object: the loader places it when the library is loaded on a device and
// it lives until the process ends.  In host code the array's name is only a handle; its device address is
// looked up once per device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[TT_CONV_BWD_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES];

// Device address of the scratch array on the current device, looked up on the first call per device.
tt_status static_scratch(void** out) {
  int dev = -1;
  if (hipError_t e = hipGetDevice(&dev); e != hipSuccess || dev < 0 || dev >= MAX_DEVICES)
    return fail(TT_ERR_HIP, "tree_conv_bwd_static: no usable current device (%s)", hipGetErrorString(e));
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess || !p)
      return fail(TT_ERR_HIP, "tree_conv_bwd_static: address of the scratch array on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return TT_OK;
}

}  // namespace

extern "C" tt_status tt_tree_conv_bwd(int64_t n_tokens, int32_t channels, int32_t kernel_size, int32_t dtype, int32_t activation,
                                      const void* x, int64_t x_stride_tok, const float* weight, const float* bias,
                                      const int32_t* tok_pred, const void* dy, int64_t dy_stride_tok, int32_t n_fix,
                                      const int32_t* fix_tok, const int32_t* fix_off, const int32_t* fix_t, const int32_t* fix_r,
                                      void* dx, int64_t dx_stride_tok, float* dweight, float* dbias, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  tt::clear_error();
  const ConvBwdCall k{n_tokens, channels, kernel_size, dtype, activation, x, x_stride_tok, weight, bias, tok_pred, dy, dy_stride_tok,
                      n_fix, fix_tok, fix_off, fix_t, fix_r, dx, dx_stride_tok, dweight, dbias};
  ConvChecked c, cd;
  size_t need = 0;
  if (tt_status s = conv_bwd_validate(k, c, cd, need)) return s;
  if (!workspace || workspace_bytes < need || !tt::aligned16(workspace))
    return fail(TT_ERR_WORKSPACE, "conv backward needs %zu bytes of 16-byte aligned workspace, got %zu", need, workspace_bytes);
  return conv_bwd_launch(k, c, cd, workspace, stream, "tree_conv_bwd");
}

extern "C" tt_status tt_tree_conv_bwd_static(int64_t n_tokens, int32_t channels, int32_t kernel_size, int32_t dtype,
                                             int32_t activation, const void* x, int64_t x_stride_tok, const float* weight,
                                             const float* bias, const int32_t* tok_pred, const void* dy, int64_t dy_stride_tok,
                                             int32_t n_fix, const int32_t* fix_tok, const int32_t* fix_off, const int32_t* fix_t,
                                             const int32_t* fix_r, void* dx, int64_t dx_stride_tok, float* dweight, float* dbias,
                                             void* stream) {
  tt::clear_error();
  const ConvBwdCall k{n_tokens, channels, kernel_size, dtype, activation, x, x_stride_tok, weight, bias, tok_pred, dy, dy_stride_tok,
                      n_fix, fix_tok, fix_off, fix_t, fix_r, dx, dx_stride_tok, dweight, dbias};
  ConvChecked c, cd;
  size_t need = 0;
  if (tt_status s = conv_bwd_validate(k, c, cd, need)) return s;
  if (need > (size_t)TT_CONV_BWD_STATIC_SCRATCH_BYTES)
    return fail(TT_ERR_WORKSPACE,
                "conv backward of this shape needs %zu bytes of scratch, the static array of tt_tree_conv_bwd_static holds %zu; "
                "use tt_tree_conv_bwd with a caller workspace",
                need, (size_t)TT_CONV_BWD_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  if (tt_status s = static_scratch(&ws)) return s;
  return conv_bwd_launch(k, c, cd, ws, stream, "tree_conv_bwd_static");
}

namespace {
// Host-checkable part of a schedule: counts, the level table (a host array) and the presence of the device arrays.
tt_status check_gdn_schedule(const tt_gdn_schedule* sc, int32_t n_chunks, bool backward) {
  if (!sc) return TT_OK;
  if (sc->n_segments < 0 || sc->n_levels < 0 || sc->n_segments > n_chunks || sc->n_levels > sc->n_segments)
    return fail(TT_ERR_SHAPE, "schedule: %d segments in %d levels for %d chunks", sc->n_segments, sc->n_levels, n_chunks);
  if ((n_chunks > 0) != (sc->n_segments > 0)) return fail(TT_ERR_SHAPE, "schedule: %d segments for %d chunks", sc->n_segments, n_chunks);
  if (!sc->level_off || (sc->n_segments > 0 && (!sc->seg_chunk0 || !sc->seg_chunk1))) return fail(TT_ERR_NULL, "schedule: an array is NULL");
  if (backward && !sc->slot_cons_off) return fail(TT_ERR_NULL, "schedule: the backward needs slot_cons_off / slot_cons");
  if (sc->level_off[0] != 0 || sc->level_off[sc->n_levels] != sc->n_segments) return fail(TT_ERR_SHAPE, "schedule: level_off does not cover the segments");
  for (int32_t l = 0; l < sc->n_levels; l++) {
    const int32_t n = sc->level_off[l + 1] - sc->level_off[l];
    if (n <= 0 || n > 65535) return fail(TT_ERR_SHAPE, "schedule: level %d has %d segments (1..65535)", l, n);
  }
  return TT_OK;
}
}  // namespace

extern "C" size_t tt_tree_gdn_workspace(int32_t n_chunks, int32_t n_slots, int32_t hv) {
  tt::clear_error();
  if (n_chunks < 0 || n_slots < 0 || hv <= 0) return 0;
  return tt::gdn_workspace(n_chunks, n_slots, hv);
}

extern "C" tt_status tt_tree_gdn_fwd(int64_t n_tokens, int32_t hk, int32_t hv, int32_t dk, int32_t dv, float scale,
                                     const void* q, const void* k, const void* v, const float* g, const float* beta,
                                     int32_t n_chunks, const int32_t* chunk_tok0, const int32_t* chunk_len,
                                     const int32_t* chunk_src, const int32_t* chunk_dst, int32_t n_slots,
                                     const int32_t* chunk_cap, const tt_gdn_schedule* schedule, const float* initial_state,
                                     float* state_out, void* o, void* workspace, size_t workspace_bytes, void* stream) {
  tt::clear_error();
  if (n_tokens < 0 || n_tokens >= INT32_MAX) return fail(TT_ERR_SHAPE, "n_tokens=%lld out of range", (long long)n_tokens);
  if (dk != 128 || dv != 128) return fail(TT_ERR_UNSUPPORTED, "dk=%d, dv=%d: only 128 x 128 states are built", dk, dv);
  if (hk <= 0 || hv <= 0 || hv % hk != 0 || hv > 65535) return fail(TT_ERR_SHAPE, "hv=%d must be a positive multiple of hk=%d", hv, hk);
  if (!(scale > 0.f) || !std::isfinite(scale)) return fail(TT_ERR_SHAPE, "scale must be positive and finite");
  if (n_chunks < 0 || n_slots < 0 || n_chunks > 65535 * 16) return fail(TT_ERR_SHAPE, "n_chunks=%d, n_slots=%d out of range", n_chunks, n_slots);
  if ((n_tokens > 0) != (n_chunks > 0)) return fail(TT_ERR_SHAPE, "n_tokens=%lld with %d chunks", (long long)n_tokens, n_chunks);
  if (n_chunks > 0 && (!q || !k || !v || !g || !beta || !o || !chunk_tok0 || !chunk_len || !chunk_src || !chunk_dst))
    return fail(TT_ERR_NULL, "a tensor or plan pointer is NULL");
  if ((chunk_cap != nullptr) != (state_out != nullptr)) return fail(TT_ERR_NULL, "chunk_cap and state_out must be given together");
  if (tt_status sst = check_gdn_schedule(schedule, n_chunks, false)) return sst;
  const void* ptrs[] = {q, k, v, o, initial_state, state_out};
  for (const void* p : ptrs)
    if (!tt::aligned16(p)) return fail(TT_ERR_ALIGN, "device pointer %p is not 16-byte aligned", p);
  const size_t need = tt::gdn_workspace(n_chunks, n_slots, hv);
  if (!workspace || workspace_bytes < need || !tt::aligned16(workspace))
    return fail(TT_ERR_WORKSPACE, "gdn forward needs %zu bytes of 16-byte aligned workspace, got %zu", need, workspace_bytes);
  return hip_result(tt::gdn_fwd(n_tokens, hk, hv, scale, q, k, v, g, beta, n_chunks, chunk_tok0, chunk_len, chunk_src, chunk_dst,
                                n_slots, chunk_cap, schedule, initial_state, state_out, o, workspace, (hipStream_t)stream),
                    "tree_gdn_fwd");
}

extern "C" size_t tt_tree_gdn_bwd_workspace(int64_t n_tokens, int32_t n_chunks, int32_t n_slots, int32_t n_segments, int32_t hk,
                                            int32_t hv) {
  tt::clear_error();
  if (n_tokens < 0 || n_chunks < 0 || n_slots < 0 || n_segments < 0 || hk <= 0 || hv <= 0 || hv % hk != 0) return 0;
  return tt::gdn_bwd_workspace(n_tokens, n_chunks, n_slots, n_segments, hk, hv, hk);
}

extern "C" size_t tt_tree_gdn_bwd_workspace_min(int64_t n_tokens, int32_t n_chunks, int32_t n_slots, int32_t n_segments, int32_t hk,
                                                int32_t hv) {
  tt::clear_error();
  if (n_tokens < 0 || n_chunks < 0 || n_slots < 0 || n_segments < 0 || hk <= 0 || hv <= 0 || hv % hk != 0) return 0;
  return tt::gdn_bwd_workspace(n_tokens, n_chunks, n_slots, n_segments, hk, hv, 1);
}

extern "C" tt_status tt_tree_gdn_bwd(int64_t n_tokens, int32_t hk, int32_t hv, int32_t dk, int32_t dv, float scale,
                                     const void* q, const void* k, const void* v, const float* g, const float* beta,
                                     const void* d_o, int32_t n_chunks, const int32_t* chunk_tok0, const int32_t* chunk_len,
                                     const int32_t* chunk_src, const int32_t* chunk_dst, int32_t n_slots,
                                     const int32_t* chunk_cap, const tt_gdn_schedule* schedule, const float* initial_state,
                                     const float* d_state_out, void* dq, void* dk_out, void* dv_out, float* dg, float* dbeta,
                                     float* d_initial_state, void* workspace, size_t workspace_bytes, void* stream) {
  tt::clear_error();
  if (n_tokens < 0 || n_tokens >= INT32_MAX) return fail(TT_ERR_SHAPE, "n_tokens=%lld out of range", (long long)n_tokens);
  if (dk != 128 || dv != 128) return fail(TT_ERR_UNSUPPORTED, "dk=%d, dv=%d: only 128 x 128 states are built", dk, dv);
  if (hk <= 0 || hv <= 0 || hv % hk != 0 || hv > 65535) return fail(TT_ERR_SHAPE, "hv=%d must be a positive multiple of hk=%d", hv, hk);
  if (!(scale > 0.f) || !std::isfinite(scale)) return fail(TT_ERR_SHAPE, "scale must be positive and finite");
  if (n_chunks < 0 || n_slots < 0 || n_chunks > 65535 * 16) return fail(TT_ERR_SHAPE, "n_chunks=%d, n_slots=%d out of range", n_chunks, n_slots);
  if ((n_tokens > 0) != (n_chunks > 0)) return fail(TT_ERR_SHAPE, "n_tokens=%lld with %d chunks", (long long)n_tokens, n_chunks);
  if (n_chunks > 0 && (!q || !k || !v || !g || !beta || !d_o || !dq || !dk_out || !dv_out || !dg || !dbeta || !chunk_tok0 || !chunk_len ||
                       !chunk_src || !chunk_dst))
    return fail(TT_ERR_NULL, "a tensor or plan pointer is NULL");
  if (d_state_out && !chunk_cap) return fail(TT_ERR_NULL, "d_state_out needs chunk_cap");
  if (tt_status sst = check_gdn_schedule(schedule, n_chunks, true)) return sst;
  const void* ptrs[] = {q, k, v, d_o, dq, dk_out, dv_out, initial_state, d_state_out, d_initial_state};
  for (const void* p : ptrs)
    if (!tt::aligned16(p)) return fail(TT_ERR_ALIGN, "device pointer %p is not 16-byte aligned", p);
  if (n_tokens > 0) {
    const void* outs[] = {dq, dk_out, dv_out, dg, dbeta, d_initial_state};
    const void* ins[] = {q, k, v, g, beta, d_o, initial_state, d_state_out};
    for (const void* o : outs)
      for (const void* i : ins)
        if (o && o == i) return fail(TT_ERR_SHAPE, "an output aliases an input");
  }
  const size_t need = tt::gdn_bwd_workspace(n_tokens, n_chunks, n_slots, schedule ? schedule->n_segments : 0, hk, hv, 1);
  if (!workspace || workspace_bytes < need || !tt::aligned16(workspace))
    return fail(TT_ERR_WORKSPACE, "gdn backward needs at least %zu bytes of 16-byte aligned workspace, got %zu", need, workspace_bytes);
  tt::GdnBwdArgs a{};
  a.n_tokens = n_tokens; a.hk = hk; a.hv = hv; a.n_chunks = n_chunks; a.n_slots = n_slots; a.scale = scale;
  a.q = q; a.k = k; a.v = v; a.d_o = d_o; a.g = g; a.beta = beta;
  a.chunk_tok0 = chunk_tok0; a.chunk_len = chunk_len; a.chunk_src = chunk_src; a.chunk_dst = chunk_dst; a.chunk_cap = chunk_cap;
  a.sched = schedule;
  a.initial_state = initial_state; a.d_state_out = d_state_out;
  a.dq = dq; a.dk = dk_out; a.dv = dv_out; a.dg = dg; a.dbeta = dbeta; a.d_initial_state = d_initial_state;
  a.workspace = workspace; a.workspace_bytes = workspace_bytes;
  return hip_result(tt::gdn_bwd(a, (hipStream_t)stream), "tree_gdn_bwd");
}
