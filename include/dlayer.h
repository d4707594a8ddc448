/*
 * dlayer.h - C ABI of the MI355X (gfx950) decoder-layer training-step library.
 *
 * The library computes one bf16 training step (forward + backward) of the model the paper
 * benchmarks (Fig. 2: an 8B Llama-3-style decoder stack; the "transformer block" of its
 * Training Pipeline paragraph): pre-norm RMSNorm, Q/K/V projections, rotary position
 * embedding, causal softmax attention with grouped KV heads, output projection with residual,
 * and a SwiGLU MLP with residual; plus token embedding, final norm, LM head and mean softmax
 * cross-entropy (the training loss of Fig. 2a).  The paper gives no equations; the definitions
 * are the standard ones and are restated at each entry point.
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, 16-byte aligned, dense
 *     row-major.  bf16 = upper 16 bits of an IEEE fp32 (1-8-7).  "f32" = IEEE fp32.
 *   - Activations are [T, features] with T = batch * seq tokens (equivalently [B, S, features]);
 *     head tensors are [T, H, head_dim] (the projection output viewed as heads, no transpose);
 *     weights are [out_features, in_features] (y = x W^T); norm gains are [D].
 *   - Contractions take bf16 operands and accumulate in fp32; reductions (norm statistics,
 *     softmax, gain gradients, loss) are fp32; stored results are bf16 unless stated.
 *   - The library never allocates, frees or keeps device memory.  Scratch is passed in by the
 *     caller (`workspace`, sized by the matching *_workspace_bytes query; contents are
 *     undefined on entry and on return and may be reused by the next call on the same stream).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work on it and return without synchronising; outputs are valid once the stream has been
 *     synchronised by the caller.
 *   - Return value: 0 on success; DLAYER_ERR_INVALID for a rejected argument (null or
 *     misaligned pointer, unsupported shape) - nothing has been launched and outputs are
 *     untouched; DLAYER_ERR_DEVICE if the current device is not gfx950; DLAYER_ERR_LAUNCH if
 *     HIP reported an error while enqueueing.  dlayer_last_error() returns a thread-local,
 *     statically stored message for the last failing call on the calling thread.
 *   - Shape granularity: head_dim in {32, 64, 128}; n_q_heads % n_kv_heads == 0; seq a
 *     multiple of 128; every contraction (inner) dimension a multiple of 64 (for a layer:
 *     d_model, d_ff, n_q_heads*head_dim, n_kv_heads*head_dim and batch*seq) and every output
 *     feature dimension a multiple of 8; d_model <= 16384; feature counts of the element-wise
 *     kernels a multiple of 8; every tensor, activation or weight, smaller than 4 GiB.
 */
#ifndef DLAYER_H
#define DLAYER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DLAYER_OK 0
#define DLAYER_ERR_INVALID (-1)
#define DLAYER_ERR_DEVICE (-2)
#define DLAYER_ERR_LAUNCH (-3)

/* Host-side description of one decoder layer call. */
typedef struct dlayer_cfg {
  int32_t batch, seq, d_model, n_q_heads, n_kv_heads, head_dim, d_ff;
  float rms_eps;       /* added to the mean square inside the square root          */
  float rope_base;     /* rotary base: angle(p, i) = p * rope_base^(-2 i / head_dim) */
  int32_t rope_layout; /* 0: element i pairs with i + head_dim/2; 1: 2i pairs with 2i+1 */
  int32_t recompute;   /* 0, or an OR of DLAYER_RECOMPUTE_*: activations dlayer_forward does not keep in
                          `saved` and dlayer_backward rebuilds (they are operands of the weight gradients
                          only).  Same cfg in the forward, the backward and the size queries.           */
} dlayer_cfg;
/* the two RMSNorm outputs h1, h2 [T, D]: rebuilt from x, y1 and the saved statistics                 */
#define DLAYER_RECOMPUTE_NORMS 1
/* the SwiGLU output a [T, d_ff]: rebuilt from the saved g and u (from their bf16 values, where the
 * forward's fused kernel used the fp32 sums: the down-projection weight gradient sees a rounded once
 * more)                                                                                              */
#define DLAYER_RECOMPUTE_SWIGLU 2

/* Device pointers to the nine parameter tensors of a layer (bf16):
 * g_attn [D], wq [Hq*dh, D], wk [Hkv*dh, D], wv [Hkv*dh, D], wo [D, Hq*dh],
 * g_mlp [D], w_gate [F, D], w_up [F, D], w_down [D, F].                                   */
typedef struct dlayer_weights {
  const void *g_attn, *wq, *wk, *wv, *wo, *g_mlp, *w_gate, *w_up, *w_down;
} dlayer_weights;
/* Same shapes, written by dlayer_backward (bf16). */
typedef struct dlayer_wgrads {
  void *g_attn, *wq, *wk, *wv, *wo, *g_mlp, *w_gate, *w_up, *w_down;
} dlayer_wgrads;

int dlayer_version(void);
const char* dlayer_last_error(void);

/* Bytes of the `saved` buffer that carries activations from dlayer_forward to
 * dlayer_backward, and of the scratch `workspace` either call needs.  Return 0 for a
 * configuration the library rejects (see shape granularity above).                          */
size_t dlayer_saved_bytes(const dlayer_cfg* cfg);
size_t dlayer_workspace_bytes(const dlayer_cfg* cfg);

/*
 * Forward of one decoder layer (the transformer block of the paper's benchmark model):
 *   h1 = RMSNorm(x; g_attn);  q,k,v = h1 Wq^T, h1 Wk^T, h1 Wv^T;  q,k <- RoPE(q), RoPE(k)
 *   o_h = softmax(q_h k_j^T / sqrt(head_dim) + causal mask) v_j,  j = h / (Hq/Hkv)
 *   y1 = x + o Wo^T;  h2 = RMSNorm(y1; g_mlp);  y = y1 + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T
 * RMSNorm(t; g) = t * (mean_d t^2 + rms_eps)^(-1/2) * g.  Positions restart at 0 for every
 * batch row.  x [T, D] bf16 (read only) -> y [T, D] bf16.  `saved` receives everything the
 * backward needs.  x and y must not overlap.
 */
int dlayer_forward(const dlayer_cfg* cfg, const void* x, const dlayer_weights* w, void* y,
                   void* saved, void* workspace, void* stream);

/*
 * Backward of dlayer_forward for upstream gradient dy [T, D] bf16: writes dx [T, D] bf16 and
 * the nine parameter gradients (each summed over all T tokens; fp32 accumulation, bf16
 * result).  x, w and saved must be those of the matching forward call.  flags (0 or an OR of):
 *   DLAYER_ACCUMULATE_WGRADS         add to the current contents of the gradient tensors instead of
 *                                    overwriting them;
 *   DLAYER_REUSE_TRANSPOSED_WEIGHTS  the input-gradient products read transposed copies of the seven
 *                                    weight matrices, written into `workspace` at the start of every
 *                                    call; with this flag the call trusts that the copies a previous
 *                                    dlayer_backward left there - same cfg, same weight VALUES, same
 *                                    workspace, nothing else having written to it since
 *                                    (dlayer_forward leaves that part alone) - are still valid and skips rewriting
 *                                    them: for several micro-batches between two optimizer steps.
 */
#define DLAYER_ACCUMULATE_WGRADS 1
#define DLAYER_REUSE_TRANSPOSED_WEIGHTS 2
int dlayer_backward(const dlayer_cfg* cfg, const void* x, const dlayer_weights* w,
                    const void* dy, const void* saved, void* dx, const dlayer_wgrads* dw,
                    int flags, void* workspace, void* stream);

/*
 * Mean softmax cross-entropy over T rows of V logits and its gradient (training loss of the
 * paper's Fig. 2a, next-token objective):
 *   loss = (1/T) sum_t ( logsumexp(logits[t, :]) - logits[t, targets[t]] )     -> *loss (device f32)
 *   dlogits[t, v] = (softmax(logits[t, :])[v] - [v == targets[t]]) * grad_scale / T   (bf16)
 * logits [T, V] bf16, targets [T] int64 with 0 <= target < V (out-of-range targets contribute
 * only the logsumexp term and no -1).  dlogits may alias logits.  V % 8 == 0.
 * workspace: ce_loss_workspace_bytes(T, V).
 */
size_t ce_loss_workspace_bytes(int64_t T, int64_t V);
int ce_loss_fwd_bwd(const void* logits, const int64_t* targets, int64_t T, int64_t V,
                    float grad_scale, float* loss, void* dlogits, void* workspace, void* stream);

/*
 * ce_loss_fwd_bwd for callers that cannot allocate or pass scratch memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the
 * workspace, same results bit for bit.  The per-row losses live in a static device array inside the
 * library (CE_LOSS_STATIC_MAX_ROWS floats = 256 KiB on every GPU the library runs on, held until the
 * process ends); T above that limit is rejected with DLAYER_ERR_INVALID.  The call allocates and
 * frees nothing.  All calls on one GPU share that array: calls that overlap on one GPU (two streams,
 * two threads) race and must be serialised by the caller.  The first call on a device looks up the
 * array's address and should be made outside graph capture.
 */
#define CE_LOSS_STATIC_MAX_ROWS 65536
int ce_loss_fwd_bwd_static(const void* logits, const int64_t* targets, int64_t T, int64_t V,
                           float grad_scale, float* loss, void* dlogits, void* stream);

/*
 * The LM head and its loss in one call, without ever holding all T x V logits (same training loss):
 *   logits = h w_lm^T;  loss, dlogits as in ce_loss_fwd_bwd;  dh = dlogits w_lm;  dw_lm (+)= dlogits^T h
 * The rows are walked in chunks of chunk_rows (0 = chosen by the library: about 1 GiB of logits):
 * each chunk's logits are formed, turned into their gradient in place and consumed by the two
 * gradient products before the next chunk overwrites them.  dw_lm is accumulated in bf16 from chunk
 * to chunk (fp32 within a chunk), so it is rounded once per chunk instead of once.
 * h, dh [T, D], w_lm, dw_lm [V, D] bf16, targets [T] int64, *loss device f32.  T, D, V multiples of
 * 64; chunk_rows 0 or a multiple of 64; one chunk of logits and every operand below 4 GiB (T * V
 * itself may exceed it).  accumulate_dw as in dlayer_backward.
 * workspace: lm_head_ce_workspace_bytes(T, D, V, chunk_rows) - one chunk of logits, a transposed
 * copy of w_lm and T floats.
 */
size_t lm_head_ce_workspace_bytes(int64_t T, int64_t D, int64_t V, int64_t chunk_rows);
int lm_head_ce_fwd_bwd(const void* h, const void* w_lm, const int64_t* targets, int64_t T, int64_t D,
                       int64_t V, float grad_scale, int64_t chunk_rows, float* loss, void* dh,
                       void* dw_lm, int accumulate_dw, void* workspace, void* stream);

/* ------------------------------------------------------------------------------------------
 * Building blocks (the steps of the layer, exposed for the model stack around it: embedding,
 * final norm, LM head - and for step-by-step verification).
 * ------------------------------------------------------------------------------------------ */

/* h[t,:] = x[t,:] * rstd[t] * gamma,  rstd[t] = (mean_d x[t,d]^2 + eps)^(-1/2).
 * x, h [T, D] bf16; gamma [D] bf16; rstd [T] f32 (written).  D % 8 == 0, D <= 16384.        */
int rmsnorm_forward(const void* x, const void* gamma, int64_t T, int64_t D, float eps, void* h,
                    float* rstd, void* stream);

/* Gradient of rmsnorm_forward given dh [T, D] bf16 and the saved rstd:
 *   xhat = x*rstd; dgamma = sum_t dh*xhat; dxhat = dh*gamma;
 *   dx = rstd*(dxhat - xhat*mean_d(dxhat*xhat)) + (dres ? dres : 0)
 * dres [T, D] bf16 is an optional gradient arriving through a residual connection (may be
 * NULL; may alias dx).  dgamma [D] bf16; accumulate_dgamma as in dlayer_backward.
 * workspace: rmsnorm_backward_workspace_bytes(T, D).                                        */
size_t rmsnorm_backward_workspace_bytes(int64_t T, int64_t D);
int rmsnorm_backward(const void* x, const void* gamma, const float* rstd, const void* dh,
                     const void* dres, int64_t T, int64_t D, void* dx, void* dgamma,
                     int accumulate_dgamma, void* workspace, void* stream);

/* y = x W^T (+ residual).  x [T, K], w [N, K], residual [T, N] or NULL, y [T, N]; all bf16.
 * K % 64 == 0, N % 8 == 0.  y may alias residual.                                           */
int linear_forward(const void* x, const void* w, const void* residual, int64_t T, int64_t K,
                   int64_t N, void* y, void* stream);

/* The three head projections of the transformer block (Fig. 2; Training Pipeline paragraph) in one
 * launch, q and k leaving it rotated: q = RoPE(h Wq^T), k = RoPE(h Wk^T), v = h Wv^T.  The rotation
 * (dlayer_cfg: angle and the two pairings; position = token index within its batch row) is applied
 * in the product's epilogue to the fp32 sums, so q and k are rounded to bf16 once.
 * h [B*S, D], wq [Hq*dh, D], wk and wv [Hkv*dh, D], q [B*S, Hq*dh], k and v [B*S, Hkv*dh]; all bf16.
 * D % 64 == 0.  workspace (device): qkv_rope_workspace_bytes(seq, head_dim), receives the fp32 cos and
 * sin of every (position, pair), evaluated in fp64.                                              */
size_t qkv_rope_workspace_bytes(int64_t seq, int64_t head_dim);
int qkv_rope_forward(const void* h, const void* wq, const void* wk, const void* wv, int64_t batch,
                     int64_t seq, int64_t d_model, int64_t n_q_heads, int64_t n_kv_heads,
                     int64_t head_dim, float rope_base, int32_t rope_layout, void* q, void* k, void* v,
                     void* workspace, void* stream);

/* The gated pair of the SwiGLU MLP of the transformer block (Fig. 2; Training Pipeline paragraph):
 * g = x Wg^T, u = x Wu^T, a = silu(g) * u.  x [T, K], w_gate and w_up [F, K], g, u, a [T, F] dense;
 * all bf16.  K % 64 == 0, F % 8 == 0.  Large problems run as one kernel whose epilogue applies the
 * activation to the fp32 sums (a is rounded once); small ones as two products and the activation
 * kernel, which reads g and u as stored.                                                       */
int linear_swiglu_forward(const void* x, const void* w_gate, const void* w_up, int64_t T, int64_t K,
                          int64_t F, void* g, void* u, void* a, void* stream);

/* Backward of y = a W_down^T with a = silu(g) * u, as far as g and u: da = dy W_down, then
 * (dg, du) = swiglu_backward(g, u, da); large problems run as one kernel that applies the gradient to
 * the fp32 sums of da and never stores it, small ones as the product (da rounded to bf16) and the
 * activation-gradient kernel.  dy [T, D], w_down [D, F], g, u, dg, du [T, F] dense; all bf16.
 * T, D, F multiples of 64.  workspace (device; receives a transposed copy of w_down):
 * linear_swiglu_backward_workspace_bytes(T, D, F).                                             */
size_t linear_swiglu_backward_workspace_bytes(int64_t T, int64_t D, int64_t F);
int linear_swiglu_backward(const void* dy, const void* w_down, const void* g, const void* u,
                           int64_t T, int64_t D, int64_t F, void* dg, void* du, void* workspace,
                           void* stream);

/* Gradients of y = x W^T: dx = dy W ([T, K], skipped if dx == NULL) and dw = dy^T x ([N, K],
 * skipped if dw == NULL).  T, K, N multiples of 64.  workspace (device, needed when dx is
 * asked for: it receives a transposed copy of w): linear_backward_workspace_bytes(T, K, N).   */
size_t linear_backward_workspace_bytes(int64_t T, int64_t K, int64_t N);
int linear_backward(const void* x, const void* w, const void* dy, int64_t T, int64_t K,
                    int64_t N, void* dx, void* dw, int accumulate_dw, void* workspace,
                    void* stream);

/* Weight gradients of n (1..8) linear layers over the same T tokens in ONE launch:
 * dw[i] [N[i], K[i]] (+)= dy[i]^T x[i] with dy[i] [T, N[i]], x[i] [T, K[i]], all bf16 row-major device
 * pointers; dy, x, dw, N, K are host arrays of length n.  T, N[i], K[i] multiples of 64.  The tile
 * sequences of the n products are laid end to end, so a product that leaves the last round of
 * workgroups partly filled (or is too small to fill the chip) runs alongside the next one;
 * dlayer_backward computes the seven weight gradients of the transformer block (Fig. 2) this way.
 * Results are bitwise those of n linear_backward calls with dx == NULL.                      */
int linear_wgrad_group(int32_t n, const void* const* dy, const void* const* x, const int64_t* N,
                       const int64_t* K, int64_t T, void* const* dw, int accumulate_dw, void* stream);

/* Rotary embedding applied in place to z [B*S, H, head_dim] bf16 (see dlayer_cfg for the angle
 * and the two pairings); inverse != 0 rotates by the negative angle, which is the gradient
 * map of the forward rotation.                                                              */
int rope_apply(void* z, int64_t batch, int64_t seq, int64_t n_heads, int64_t head_dim,
               float rope_base, int32_t rope_layout, int32_t inverse, void* stream);

/* Causal softmax attention (definition at dlayer_forward).  q, o [B*S, Hq, dh]; k, v
 * [B*S, Hkv, dh] bf16; lse [B, Hq, S] f32 = log-sum-exp of the scaled, masked score rows.   */
int attention_forward(const void* q, const void* k, const void* v, int64_t batch, int64_t seq,
                      int64_t n_q_heads, int64_t n_kv_heads, int64_t head_dim, void* o,
                      float* lse, void* stream);

/* Gradient of attention_forward: with P = exp(s - lse), dP = dO V^T, delta = rowsum(dO * O),
 * dS = P * (dP - delta):  dV_j = sum_h P_h^T dO_h, dQ_h = dS_h K_j / sqrt(dh),
 * dK_j = sum_h dS_h^T Q_h / sqrt(dh), sums over the query heads h of KV group j.
 * workspace (device): attention_backward_workspace_bytes(...) - two f32 per (head, position)
 * and, for head_dim 128 and seq >= 2048, the causal half of dS in bf16 (seq * (seq + 128)
 * bytes per (batch, query head): 4.4 GB at batch 2, seq 8192, 32 heads), which the dK/dV
 * pass writes and the dQ pass reads back instead of forming S and dP a second time.        */
size_t attention_backward_workspace_bytes(int64_t batch, int64_t seq, int64_t n_q_heads,
                                          int64_t n_kv_heads, int64_t head_dim);
int attention_backward(const void* q, const void* k, const void* v, const void* o,
                       const void* d_o, const float* lse, int64_t batch, int64_t seq,
                       int64_t n_q_heads, int64_t n_kv_heads, int64_t head_dim, void* dq,
                       void* dk, void* dv, void* workspace, void* stream);

/* a = silu(g) * u, silu(z) = z / (1 + exp(-z)); g, u, a [n] bf16, n % 8 == 0.                */
int swiglu_forward(const void* g, const void* u, int64_t n, void* a, void* stream);
/* dg = da * u * s * (1 + g * (1 - s)), du = da * g * s, s = 1/(1+exp(-g)).  dg may alias g,
 * du may alias u.                                                                           */
int swiglu_backward(const void* g, const void* u, const void* da, int64_t n, void* dg, void* du,
                    void* stream);

/* x0[t, :] = table[ids[t], :].  table [V, D] bf16, ids [T] int64 in [0, V), x0 [T, D] bf16.  */
int embed_forward(const void* table, const int64_t* ids, int64_t T, int64_t V, int64_t D,
                  void* x0, void* stream);
/* dtable[v, :] = sum over t with ids[t] == v of dx0[t, :] (rows of absent ids are zero; ids outside
 * [0, V) are skipped).  Deterministic: the tokens of an id are listed, sorted and summed in fp32 in
 * ascending token order (interleaved partial sums, combined in a fixed order), bf16 result; no
 * floating-point atomics, bitwise reproducible.  An id with more than four tokens is summed by one
 * workgroup per 128 columns, whatever its frequency.  dtable [V, D] bf16 is overwritten.
 * workspace (device): embed_backward_workspace_bytes(T, V), about (3 V + 2.2 T) ints.         */
size_t embed_backward_workspace_bytes(int64_t T, int64_t V);
int embed_backward(const void* dx0, const int64_t* ids, int64_t T, int64_t V, int64_t D,
                   void* dtable, void* workspace, void* stream);

/* ------------------------------------------------------------------------------------------
 * Optimizer step.  The paper's Training Pipeline paragraph speaks of training steps and names no
 * optimizer; the reading taken is the usual one for this model family: clipping of the gradients by
 * their global norm, then AdamW (Adam with decoupled weight decay).  Parameters and gradients are
 * bf16, the two moment tensors fp32, the arithmetic fp32.  Up to 16 tensors per call; all lists are
 * host arrays of length n holding device pointers / element counts (each a multiple of 8).
 * ------------------------------------------------------------------------------------------ */

/* *sq_norm (device f32) = sum over every element of the n gradient tensors of g^2, or that sum added
 * to the value already there when accumulate != 0 (a model with more than 16 tensors takes several
 * calls).  Summed in a fixed order: the result is bitwise reproducible.
 * workspace (device): grad_sq_norm_workspace_bytes(n, numel).                                      */
size_t grad_sq_norm_workspace_bytes(int32_t n, const int64_t* numel);
int grad_sq_norm(int32_t n, const void* const* grads, const int64_t* numel, float* sq_norm,
                 int accumulate, void* workspace, void* stream);

/* One AdamW update of n tensors, in place (step counts from 1):
 *   g' = g * min(1, max_grad_norm / (sqrt(*sq_norm) + 1e-6))      (g' = g when sq_norm is NULL)
 *   p <- p (1 - lr weight_decay);  m <- beta1 m + (1 - beta1) g';  v <- beta2 v + (1 - beta2) g'^2
 *   p <- p - lr / (1 - beta1^step) * m / (sqrt(v) / sqrt(1 - beta2^step) + eps)
 * sq_norm is read on the device (the value grad_sq_norm left there): no host synchronisation between
 * the two calls.  params bf16 (updated), grads bf16 (read only), exp_avg = m and exp_avg_sq = v fp32
 * (updated).                                                                                      */
int adamw_step(int32_t n, void* const* params, const void* const* grads, float* const* exp_avg,
               float* const* exp_avg_sq, const int64_t* numel, int64_t step, float lr, float beta1,
               float beta2, float eps, float weight_decay, float max_grad_norm, const float* sq_norm,
               void* stream);

/* ------------------------------------------------------------------------------------------
 * Measurement aid, not a step of the path: synthetic kernels that time the matrix pipe next to a set
 * amount of other work on this GPU (one workgroup per compute unit, fixed trip counts, no inputs).
 * They back the design notes on what bounds the GEMM and attention kernels; bench.py --probes
 * prints the table.
 *   family 0  32x32x16 MFMAs and softmax-like VALU work, one block = 16 MFMAs + 16 exp + 64 fma:
 *             variant 0 MFMAs alone, 1 VALU alone, 2 evenly interleaved, 3 in two regions
 *             (8 MFMAs with 1 fma each, then 8 with 2 exp + 7 fma each)
 *   family 1  16x16x32 MFMAs fed from LDS, one block = 8 MFMAs: variant 0 no reads, 1 two and 2 three
 *             16-byte fragment reads per block, 3 three pairs of transposing 8-byte reads
 *   family 2  four waves issue MFMAs only, their four SIMD partners v_fma_f32 only (waves_per_simd is
 *             ignored): variant 0 the MFMA waves alone, 1 the VALU waves alone, 2 both
 *   family 3  family 1's variants 0, 1, 2 with pseudo-random operands in (-1, 1) instead of constants,
 *             2500 launches back to back (about a second): the rate the matrix pipes hold at the clock
 *             the power management settles on under a long load; the milliseconds are the mean launch;
 *             variant 3: the 32x32x16 MFMAs of family 0, variant 0, the same way (block = 16 MFMAs)
 * waves_per_simd: 1 or 2.  result (host, 4 doubles): shader-clock cycles per block per SIMD (family 2:
 * per MFMA of an MFMA wave), milliseconds of the launch, shader clock in GHz during it, and for family
 * 2 the cycles per fma of a VALU wave (else 0).  Allocates and frees a few KB of device memory and
 * synchronises with the stream.                                                                   */
int issue_rate_probe(int family, int variant, int waves_per_simd, double* result, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DLAYER_H */
