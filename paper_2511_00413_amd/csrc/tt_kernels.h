// Kernel launch interfaces shared by the API layer and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "treetrain.h"

namespace tt {

// Brackets one kernel launch with HIP events on its stream when kernel timing is enabled
// (tt_kernel_timing_enable); does nothing otherwise.
class KernelTimer {
 public:
  KernelTimer(int id, hipStream_t st);
  ~KernelTimer();
  KernelTimer(const KernelTimer&) = delete;
  KernelTimer& operator=(const KernelTimer&) = delete;
 private:
  int id_;
  hipStream_t st_;
  bool active_;
  hipEvent_t start_, stop_;
};

// Arguments of one attention call, after validation; strides are in elements.
struct RefArgs {
  int n_q, n_prefix, hq, hkv, d;
  float scale;
  int64_t q_stride, k_stride, v_stride;
  const void *q, *k_own, *v_own, *k_prefix, *v_prefix;
  const int32_t *kend, *kt_min, *kt_max;
  void* o;
  float* lse;
  // backward only
  const void* d_o;
  float* delta;                 // [hq][n_q] workspace: rowsum(dO o O); the MFMA path stores its negation here
  float* neg_lse2;              // [hq][n_q] MFMA path only: -lse * log2(e)
  void *dq, *dk_own, *dv_own;
  float *dk_prefix_acc, *dv_prefix_acc;
  void* workspace;              // remaining workspace after delta (MFMA path scratch)
  size_t workspace_bytes;
};
typedef RefArgs AttnArgs;

// fp32-arithmetic reference-grade kernels (tt_attn_ref.hip)
hipError_t ref_attn_fwd(const RefArgs& a, bool bf16, hipStream_t st);
hipError_t ref_attn_bwd(const RefArgs& a, bool bf16, hipStream_t st);

// bf16 MFMA kernels, d = 128 (tt_attn_fwd.hip / tt_attn_bwd.hip)
hipError_t mfma_attn_fwd(const AttnArgs& a, hipStream_t st);
hipError_t mfma_attn_bwd(const AttnArgs& a, hipStream_t st);
size_t mfma_attn_workspace(int n_q, int n_prefix, int hq, int hkv, int d, bool backward);
// dK/dV pass of the backward (tt_attn_dkdv.hip); a.workspace must hold mfma_attn_dkdv_workspace bytes
hipError_t mfma_attn_dkdv(const AttnArgs& a, hipStream_t st);
size_t mfma_attn_dkdv_workspace(int n_q, int n_prefix, int hkv);

// fused log-softmax / gather / weighting (tt_loss.hip)
hipError_t weighted_logprob(int64_t n_rows, int vocab, bool bf16, const void* logits, int64_t row_stride,
                            const int32_t* target, const float* weight, float* logp, float* lse,
                            float* loss_acc, hipStream_t st);
hipError_t weighted_logprob_bwd(int64_t n_rows, int vocab, bool bf16, const void* logits, int64_t row_stride,
                                const int32_t* target, const float* weight, const float* lse, float grad_scale,
                                void* dlogits, int64_t out_stride, hipStream_t st);

// both in one pass over the logits; weighted_logprob_fused_ok tells whether the pointers and strides allow it (rows of
// the logits and of the gradient on 16-byte boundaries)
bool weighted_logprob_fused_ok(bool bf16, const void* logits, int64_t row_stride, const void* dlogits, int64_t out_stride);
hipError_t weighted_logprob_fused(int64_t n_rows, int vocab, bool bf16, const void* logits, int64_t row_stride,
                                  const int32_t* target, const float* weight, float grad_scale, float* logp, float* lse,
                                  float* loss_acc, void* dlogits, int64_t out_stride, hipStream_t st);

// rotary position embedding (tt_rope.hip); strides in elements
hipError_t rope(int64_t n_tokens, int n_heads, int d, bool bf16, const void* x, int64_t x_stride, const int32_t* pos,
                float theta_base, bool inverse, void* y, int64_t y_stride, hipStream_t st);

// tree-correct causal convolution (tt_conv.hip); strides in bytes
hipError_t conv_fwd(int64_t n_tokens, int channels, int kernel_size, bool bf16, bool silu, const void* x, int64_t x_stride_bytes,
                    const float* weight, const float* bias, const int32_t* tok_pred, void* y, int64_t y_stride_bytes,
                    hipStream_t st);
hipError_t conv_bwd(int64_t n_tokens, int channels, int kernel_size, bool bf16, bool silu, const void* x, int64_t x_stride_bytes,
                    const float* weight, const float* bias, const int32_t* tok_pred, const void* dy, int64_t dy_stride_bytes,
                    int n_fix, const int32_t* fix_tok, const int32_t* fix_off, const int32_t* fix_t, const int32_t* fix_r,
                    void* dx, int64_t dx_stride_bytes, float* dweight, float* dbias, void* workspace, hipStream_t st);
size_t conv_bwd_workspace(int64_t n_tokens, int channels, int kernel_size, bool bf16);

// gated delta rule with tree state routing, forward (tt_gdn.hip); dk = dv = 128, bf16
// `sched` (nullable): the segments of the chunk program by dependency level; see tt_gdn_schedule
hipError_t gdn_fwd(int64_t n_tokens, int hk, int hv, float scale, const void* q, const void* k, const void* v, const float* g,
                   const float* beta, int n_chunks, const int32_t* chunk_tok0, const int32_t* chunk_len, const int32_t* chunk_src,
                   const int32_t* chunk_dst, int n_slots, const int32_t* chunk_cap, const tt_gdn_schedule* sched,
                   const float* initial_state, float* state_out, void* o, void* workspace, hipStream_t st);
size_t gdn_workspace(int n_chunks, int n_slots, int hv);

// Backward of the gated delta rule.  Every per-chunk array is indexed by (head * n_chunks + chunk).
// Unrounded per-chunk quantities that do not depend on the state (written by the prepare kernel, read by the
// finish kernel):
struct GdnChunkOps {
  float* gam;      // [64]       running sum of the log-decays inside the chunk
  float* a0;       // [64][64]   strictly-lower (k_i . k_j) exp(gamma_i - gamma_j)   (A without beta_i)
  float* p;        // [64][64]   scale tril((q_i . k_j) exp(gamma_i - gamma_j))
  float* t;        // [64][64]   (I + A)^-1, A = diag(beta) a0: the inverse both triangular solves are products with
};
// bf16 operands of the two walks and what they save for the finish kernel:
constexpr size_t GDN_REC_ELEMS = 4 * 64 * 128 + 64 * 64;     // elements of one walk record (forward and reverse alike)
constexpr size_t GDN_REC_UT = 64 * 128;      // forward record: U^T [128 value cols][64 tokens], U = (I + A)^-1 (beta V)
constexpr size_t GDN_REV_WTN = 64 * 128;     // reverse record: -W^T [128 key dims][64 tokens], W = (I + A)^-1 (beta exp(gamma) K)
struct GdnBwdSaved {
  void* fwd_rec;     // forward walk records
  void* rev_rec;     // reverse walk records
  float* glast;      // exp(gamma_last)
  void* s0t;         // [128 value cols][128 key dims] bf16: state entering the chunk, transposed
  void* ds1t;        // same layout: gradient of the state leaving the chunk
  void* vns;         // Vn  [64][128] bf16 in matrix-instruction fragment order (gdn_frag_index)
  void* dvns;        // dVn, same order
  float* slots;      // [n_slots][hv][128][128] saved node-end states
  float* slot_grad;  // their gradients (zeroed by the caller); walk in sequence order only
  float* seg_grad;   // [n_segments][hv][128][128] gradient of the state every segment starts from; scheduled walk only
};
// position of element (token i, value column col) inside a chunk's fragment-ordered [64][128] array
__host__ __device__ inline int gdn_frag_index(int i, int col) {
  const int dvb = col >> 5, c = col & 31, half = i >> 5, t = (i >> 4) & 1, i16 = i & 15;
  const int hf = (i16 >> 2) & 1, e = ((i16 >> 3) << 2) | (i16 & 3);
  return ((((dvb * 2 + half) * 2 + t) * 64 + hf * 32 + c) << 3) | e;
}

// backward of the gated delta rule (tt_gdn_bwd.hip)
struct GdnBwdArgs {
  int64_t n_tokens;
  int hk, hv, n_chunks, n_slots;
  int hv_n;                          // value heads this pass works on (set by gdn_bwd: a batch of whole key-head groups;
                                     // the tensor pointers are moved to the batch's first head, hk / hv stay the strides)
  float scale;
  const void *q, *k, *v, *d_o;       // bf16
  const float *g, *beta;
  const int32_t *chunk_tok0, *chunk_len, *chunk_src, *chunk_dst, *chunk_cap;
  const tt_gdn_schedule* sched;      // nullptr: all chunks in one sequence
  const float* initial_state;        // nullptr or [hv][128][128]
  const float* d_state_out;          // nullptr or [n_capture][hv][128][128]: upstream gradient of the captured states
  void *dq, *dk, *dv;                // bf16
  float *dg, *dbeta;                 // [N][hv]
  float* d_initial_state;            // nullptr or [hv][128][128], overwritten
  void* workspace;
  size_t workspace_bytes;            // decides how many key-head groups one pass takes
};
// prepare kernel (backward form) + forward walk + reverse walk (tt_gdn.hip)
hipError_t gdn_bwd_prepare_and_walks(const GdnBwdArgs& b, const GdnChunkOps& ops, const GdnBwdSaved& sv, hipStream_t st);
hipError_t gdn_bwd(const GdnBwdArgs& a, hipStream_t st);
// workspace for passes of key_heads_per_pass key heads (with their hv / hk value heads) at a time
size_t gdn_bwd_workspace(int64_t n_tokens, int n_chunks, int n_slots, int n_segments, int hk, int hv, int key_heads_per_pass);

}  // namespace tt
