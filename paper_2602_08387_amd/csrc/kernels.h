// Internal launch interface between the C-ABI layer (api.hip) and the kernel files.
// Every launcher validates nothing (the C-ABI layer did), enqueues on `st` and returns 0 or a
// DLAYER_ERR_LAUNCH code with the thread-local message set.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace dl {

// ---- elementwise.hip
int launch_rmsnorm_fwd(const void* x, const void* gamma, int64_t T, int64_t D, float eps, void* h,
                       float* rstd, hipStream_t st);
size_t rmsnorm_bwd_workspace(int64_t T, int64_t D);
int launch_rmsnorm_bwd(const void* x, const void* gamma, const float* rstd, const void* dh,
                       const void* dres, int64_t T, int64_t D, void* dx, void* dgamma,
                       int accumulate, void* workspace, hipStream_t st);
int launch_rope(void* z, int64_t batch, int64_t seq, int64_t n_heads, int64_t head_dim, float base,
                int layout, int inverse, hipStream_t st);
// q and k of a layer in one launch (same positions and angles)
int launch_rope_pair(void* q, void* k, int64_t batch, int64_t seq, int64_t n_q_heads, int64_t n_kv_heads,
                     int64_t head_dim, float base, int layout, int inverse, hipStream_t st);
// cos and sin of angle(p, i) = p * base^(-2 i / head_dim) for p < seq, i < head_dim / 2, evaluated in
// fp64 and stored as fp32 [seq][head_dim / 2]
int launch_rope_table(float* cos, float* sin, int64_t seq, int64_t head_dim, float base, hipStream_t st);
int launch_swiglu_fwd(const void* g, const void* u, int64_t n, void* a, hipStream_t st);
int launch_swiglu_bwd(const void* g, const void* u, const void* da, int64_t n, void* dg, void* du,
                      hipStream_t st);
// g, u: [rows, cols] with leading dimension ld_gu; a / da / dg / du with their own (padded) one
int launch_swiglu_fwd_rows(const void* g, const void* u, int64_t rows, int64_t cols, int64_t ld_gu, void* a,
                           int64_t ld_a, hipStream_t st);
int launch_swiglu_bwd_rows(const void* g, const void* u, const void* da, int64_t rows, int64_t cols, int64_t ld_gu,
                           int64_t ld_p, void* dg, void* du, hipStream_t st);
// out[c][r] = in[r][c]; out has leading dimension ld_out >= R
int launch_transpose(const void* in, void* out, int64_t R, int64_t C, int64_t ld_out, hipStream_t st);
// up to 8 transposes (each R, C multiples of 64) in one launch
constexpr int kMaxTransposeGroup = 8;
struct TransposeJob { const void* in; void* out; int64_t R, C, ld_out; };
int launch_transpose_group(const TransposeJob* jobs, int n, hipStream_t st);
int launch_embed_fwd(const void* table, const int64_t* ids, int64_t T, int64_t V, int64_t D,
                     void* x0, hipStream_t st);
size_t embed_bwd_workspace(int64_t T, int64_t V);
int launch_embed_bwd(const void* dx0, const int64_t* ids, int64_t T, int64_t V, int64_t D,
                     void* dtable, void* workspace, hipStream_t st);

// ---- gemm.hip
// C[M,N] (bf16, row-major, leading dimension ldc) = sum over segments s of opA_s * opB_s
//        (+ R[M,N] if R) (+ C if accumulate), fp32 accumulation.
// Segment operands are bf16 row-major.  a_kmajor: A_s is [M, K_s] (lda >= K_s) else [K_s, M]
// (lda >= M).  b_kmajor: B_s is [N, K_s] else [K_s, N].  K_s % 64 == 0, N % 8 == 0.
struct GemmSeg {
  const void* a;
  const void* b;
  int64_t lda, ldb;
  int K;
};
struct GemmArgs {
  GemmSeg seg[3];
  int nseg;
  int M, N;
  void* c;
  int64_t ldc;
  const void* r;  // optional residual, same leading dimension as c
  int accumulate;
  bool a_kmajor, b_kmajor;
};
int launch_gemm(const GemmArgs& g, hipStream_t st);
// Up to 8 independent problems with the same a_kmajor/b_kmajor in one launch (built for both operands
// mn-major, the weight-gradient products, and both k-major, the forward projections).
int launch_gemm_group(const GemmArgs* gs, int n, hipStream_t st);
// The same for k-major products whose outputs are [tokens][heads][head_dim], with the rotary embedding
// applied in the epilogue (on the fp32 accumulators) to the problems whose bit is set in rotate_mask.
// cos, sin: [seq][head_dim / 2] fp32 (launch_rope_table); position of a row = row % seq.
struct RopeEpilogue { const float *cos, *sin; int seq, head_dim, layout; unsigned rotate_mask; };
int launch_gemm_group_rope(const GemmArgs* gs, int n, const RopeEpilogue* rope, hipStream_t st);
// g = x Wg^T, u = x Wu^T and a = silu(g) * u (from the rounded g, u) in one launch.  x [T, K] with
// leading dimension ldx, wg and wu [F, K] with ldw, g and u with ldgu, a with lda.  Only shapes
// gemm_swiglu_applies() accepts (enough 256 x 256 tiles to fill the chip).
bool gemm_swiglu_applies(int64_t T, int64_t F);
int launch_gemm_swiglu(const void* x, int64_t ldx, const void* wg, const void* wu, int64_t ldw, int64_t T, int64_t K,
                       int64_t F, void* g, void* u, int64_t ldgu, void* a, int64_t lda, hipStream_t st);
// da = dy W^T for dy [T, K] (lddy) and wt = W [F, K] (ldw), then (dg, du) = gradient of silu(g) * u for
// the rounded da, without da ever being stored.  g, u with ldgu; dg, du with ldd.
bool gemm_swiglu_grad_applies(int64_t T, int64_t F);
int launch_gemm_swiglu_grad(const void* dy, int64_t lddy, const void* wt, int64_t ldw, int64_t T, int64_t K, int64_t F,
                            const void* g, const void* u, int64_t ldgu, void* dg, void* du, int64_t ldd,
                            hipStream_t st);

// ---- attention.hip
int launch_attention_fwd(const void* q, const void* k, const void* v, int64_t B, int64_t S,
                         int64_t Hq, int64_t Hkv, int64_t dh, void* o, float* lse, hipStream_t st);
size_t attention_bwd_workspace(int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t dh);
int launch_attention_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                         const float* lse, int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t dh,
                         void* dq, void* dk, void* dv, void* workspace, hipStream_t st);

// The same for q and k that were rotated (rotary embedding) after their projections: dq and dk are
// the gradients of the UNROTATED q and k, the inverse rotation being applied to the fp32 sums before
// they are rounded.  rope_cos, rope_sin: [S][dh / 2] fp32 (launch_rope_table), or null for no rotation.
int launch_attention_bwd_rope(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                              const float* lse, int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t dh,
                              void* dq, void* dk, void* dv, void* workspace, const float* rope_cos,
                              const float* rope_sin, int rope_layout, hipStream_t st);

// ---- ce.hip
size_t ce_workspace(int64_t T, int64_t V);
int launch_ce(const void* logits, const int64_t* targets, int64_t T, int64_t V, float grad_scale,
              float* loss, void* dlogits, void* workspace, hipStream_t st);
// the two halves of launch_ce, for callers that walk the rows in chunks
int launch_ce_rows(const void* logits, const int64_t* targets, int64_t rows, int64_t V, float scale, float* row_loss,
                   void* dlogits, hipStream_t st);
int launch_ce_mean(const float* row_loss, int64_t T, float* loss, hipStream_t st);
// launch_ce for at most ce_static_max_rows() rows, with the per-row losses in a static device array
int64_t ce_static_max_rows();
int launch_ce_static(const void* logits, const int64_t* targets, int64_t T, int64_t V, float grad_scale,
                     float* loss, void* dlogits, hipStream_t st);

// ---- optimizer.hip
constexpr int kOptMaxTensors = 16;
// number of 16384-element chunks the tensors of a call split into (= floats of workspace the norm needs)
int64_t opt_chunks(int n, const int64_t* numel);
// *sq_norm (+)= sum over all elements of all n gradient tensors of g^2 (fp32, fixed summation order)
int launch_grad_sq_norm(int n, const void* const* g, const int64_t* numel, float* sq_norm, float* partial,
                        int accumulate, hipStream_t st);
// AdamW on n tensors; sq_norm (device, may be null): gradients are scaled by min(1, max_norm / (sqrt(*sq_norm) + 1e-6))
int launch_adamw(int n, void* const* p, const void* const* g, float* const* m, float* const* v, const int64_t* numel,
                 int64_t step, float lr, float beta1, float beta2, float eps, float weight_decay, float max_norm,
                 const float* sq_norm, hipStream_t st);

// probes.hip: synthetic issue-rate measurements (see the file's header for families and variants);
// result[4] = cycles per block per SIMD, milliseconds, shader clock in GHz, second role's cycles per op
int launch_probe(int family, int variant, int waves_per_simd, double* result, hipStream_t st);

}  // namespace dl
