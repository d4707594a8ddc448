// C-ABI entry points declared in include/dlayer.h: argument validation, buffer carving and the
// order of kernel launches.  No arithmetic of the layer lives here.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "../../include/dlayer.h"
#include "common.h"
#include "kernels.h"

namespace dl {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(DLAYER_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
  return 0;
}

static int check_device() {
  static thread_local int cached_dev = -1;
  static thread_local int cached_ok = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return fail(DLAYER_ERR_DEVICE, "no HIP device is current");
  if (dev != cached_dev) {
    hipDeviceProp_t p;
    if (hipGetDeviceProperties(&p, dev) != hipSuccess) return fail(DLAYER_ERR_DEVICE, "cannot query device %d", dev);
    cached_dev = dev;
    cached_ok = strncmp(p.gcnArchName, "gfx950", 6) == 0;
    if (!cached_ok) return fail(DLAYER_ERR_DEVICE, "device %d is %s; this library is built for gfx950 only", dev, p.gcnArchName);
  }
  if (!cached_ok) return fail(DLAYER_ERR_DEVICE, "device %d is not gfx950", dev);
  return 0;
}

#define REQUIRE(cond, ...) \
  do { if (!(cond)) return dl::fail(DLAYER_ERR_INVALID, __VA_ARGS__); } while (0)
#define REQUIRE_PTR(p) REQUIRE((p) != nullptr && dl::aligned16(p), "%s: pointer %s is null or not 16-byte aligned", __func__, #p)
#define TRY(x) do { int rc_ = (x); if (rc_) return rc_; } while (0)

static inline size_t up256(size_t n) { return (n + 255) & ~(size_t)255; }

// rows * cols bf16 elements stay below 4 GiB (what a buffer descriptor's 32-bit byte count and the kernels'
// 32-bit byte offsets can address); the dimensions are bounded first so that the product cannot wrap
static inline bool under_4gib(int64_t rows, int64_t cols) {
  return rows >= 0 && cols >= 0 && rows < ((int64_t)1 << 31) && cols < ((int64_t)1 << 31) && rows * cols * 2 < ((int64_t)1 << 32);
}

struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* p) : base((char*)p) {}
  void* take(size_t bytes) { void* r = base ? base + off : nullptr; off += up256(bytes); return r; }
};

// Leading dimension of the layer's own [*, d_ff] buffers (a, da/dg, du, the transposed gate/up
// weights).  Rows 2*d_ff bytes apart are a multiple of 4 KiB apart for the usual widths, and a GEMM
// whose tile rows all sit at such a stride runs 7 % (K = 14336) to 23 % (K = 28672) slower than with
// rows 128 bytes further apart (measured): the tile's loads then pile onto few memory channels.
static int64_t padded_ff(const dlayer_cfg* c) { return (int64_t)c->d_ff + 64; }

static const char* cfg_problem(const dlayer_cfg* c) {
  if (!c) return "cfg is null";
  if (c->batch <= 0 || c->seq <= 0 || c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->d_ff <= 0)
    return "non-positive dimension";
  if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) return "head_dim must be 32, 64 or 128";
  if (c->n_q_heads % c->n_kv_heads) return "n_q_heads must be a multiple of n_kv_heads";
  if (c->seq % 128) return "seq must be a multiple of 128";
  if (c->d_model % 64 || c->d_ff % 64) return "d_model and d_ff must be multiples of 64";
  if ((c->n_q_heads * c->head_dim) % 64 || (c->n_kv_heads * c->head_dim) % 64)
    return "n_q_heads*head_dim and n_kv_heads*head_dim must be multiples of 64";
  if (c->d_model > 16384) return "d_model above 16384 is not supported";
  if (c->rope_layout != 0 && c->rope_layout != 1) return "rope_layout must be 0 or 1";
  if (c->recompute & ~(DLAYER_RECOMPUTE_NORMS | DLAYER_RECOMPUTE_SWIGLU)) return "unknown recompute bits";
  if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return "rms_eps must be >= 0 and rope_base > 0";
  const int64_t T = (int64_t)c->batch * c->seq;
  const int64_t widest = padded_ff(c) > (int64_t)c->n_q_heads * c->head_dim ? padded_ff(c) : (int64_t)c->n_q_heads * c->head_dim;
  if (!under_4gib(T, widest) || !under_4gib(T, c->d_model))
    return "an activation tensor reaches 4 GiB";
  // the weights (and their transposed copies, whose d_ff rows are padded) are addressed with 32-bit byte offsets too
  const int64_t D = c->d_model, QD = (int64_t)c->n_q_heads * c->head_dim;
  if (!under_4gib(padded_ff(c), D) || !under_4gib(QD, D))
    return "a weight tensor reaches 4 GiB";
  return nullptr;
}

struct Saved {
  float *rstd1, *rstd2, *lse, *rope_cos, *rope_sin;
  void *h1, *q, *k, *v, *o, *y1, *h2, *g, *u, *a;
  size_t bytes;
};
static Saved carve_saved(const dlayer_cfg* c, void* p) {
  const size_t T = (size_t)c->batch * c->seq, D = c->d_model, F = c->d_ff;
  const size_t QD = (size_t)c->n_q_heads * c->head_dim, KD = (size_t)c->n_kv_heads * c->head_dim;
  Carver cv(p);
  Saved s;
  s.rstd1 = (float*)cv.take(T * 4);
  s.rstd2 = (float*)cv.take(T * 4);
  s.lse = (float*)cv.take(T * c->n_q_heads * 4);
  s.rope_cos = (float*)cv.take((size_t)c->seq * (c->head_dim / 2) * 4);
  s.rope_sin = (float*)cv.take((size_t)c->seq * (c->head_dim / 2) * 4);
  s.h1 = (c->recompute & DLAYER_RECOMPUTE_NORMS) ? nullptr : cv.take(T * D * 2);
  s.q = cv.take(T * QD * 2);
  s.k = cv.take(T * KD * 2);
  s.v = cv.take(T * KD * 2);
  s.o = cv.take(T * QD * 2);
  s.y1 = cv.take(T * D * 2);
  s.h2 = (c->recompute & DLAYER_RECOMPUTE_NORMS) ? nullptr : cv.take(T * D * 2);
  s.g = cv.take(T * F * 2);
  s.u = cv.take(T * F * 2);
  s.a = (c->recompute & DLAYER_RECOMPUTE_SWIGLU) ? nullptr : cv.take(T * padded_ff(c) * 2);
  s.bytes = cv.off;
  return s;
}

struct Work {
  void *da_dg, *du, *dh2, *dy1, *d_o, *dq, *dk, *dv, *dh1, *attn_ws, *rms_ws;
  void *h1, *h2, *a;   // the activations a recomputing configuration does not keep in `saved` (null otherwise)
  void *wqT, *wkT, *wvT, *woT, *wgT, *wuT, *wdT;   // W^T copies: the input-gradient products then read both operands k-major
  size_t bytes;
};
static Work carve_work(const dlayer_cfg* c, void* p) {
  const size_t T = (size_t)c->batch * c->seq, D = c->d_model, F = c->d_ff;
  const size_t QD = (size_t)c->n_q_heads * c->head_dim, KD = (size_t)c->n_kv_heads * c->head_dim;
  Carver cv(p);
  Work w;
  w.da_dg = cv.take(T * padded_ff(c) * 2);
  w.du = cv.take(T * padded_ff(c) * 2);
  w.dh2 = cv.take(T * D * 2);
  w.dy1 = cv.take(T * D * 2);
  w.d_o = cv.take(T * QD * 2);
  w.dq = cv.take(T * QD * 2);
  w.dk = cv.take(T * KD * 2);
  w.dv = cv.take(T * KD * 2);
  w.dh1 = cv.take(T * D * 2);
  w.attn_ws = cv.take(attention_bwd_workspace(c->batch, c->seq, c->n_q_heads, c->n_kv_heads, c->head_dim));
  w.rms_ws = cv.take(rmsnorm_bwd_workspace(T, D));
  w.wqT = cv.take(QD * D * 2); w.wkT = cv.take(KD * D * 2); w.wvT = cv.take(KD * D * 2); w.woT = cv.take(D * QD * 2);
  w.wgT = cv.take(D * padded_ff(c) * 2); w.wuT = cv.take(D * padded_ff(c) * 2); w.wdT = cv.take(D * F * 2);
  w.h1 = (c->recompute & DLAYER_RECOMPUTE_NORMS) ? cv.take(T * D * 2) : nullptr;
  w.h2 = (c->recompute & DLAYER_RECOMPUTE_NORMS) ? cv.take(T * D * 2) : nullptr;
  w.a = (c->recompute & DLAYER_RECOMPUTE_SWIGLU) ? cv.take(T * padded_ff(c) * 2) : nullptr;
  w.bytes = cv.off;
  return w;
}

// y[T,N] = x[T,K] W[N,K]^T (+ residual); ldx: leading dimension of x
static GemmArgs nt_args(const void* x, int64_t ldx, const void* w, const void* res, int64_t T, int64_t K, int64_t N,
                        void* y) {
  GemmArgs g{};
  g.nseg = 1;
  g.seg[0] = {x, w, ldx, K, (int)K};
  g.M = (int)T; g.N = (int)N; g.c = y; g.ldc = N; g.r = res; g.accumulate = 0;
  g.a_kmajor = true; g.b_kmajor = true;
  return g;
}
static int gemm_nt(const void* x, int64_t ldx, const void* w, const void* res, int64_t T, int64_t K, int64_t N, void* y,
                   hipStream_t st) {
  return launch_gemm(nt_args(x, ldx, w, res, T, K, N, y), st);
}

// g = x Wg^T, u = x Wu^T, a = silu(g) * u (a with leading dimension lda): one fused launch when the
// problem fills the chip with 256 x 256 tiles, otherwise two products and the activation kernel.
// Both routes give the same bits (the fused epilogue applies the activation to the rounded g, u).
static int gate_up_swiglu(const void* x, const void* wg, const void* wu, int64_t T, int64_t K, int64_t F, void* g,
                          void* u, void* a, int64_t lda, hipStream_t st) {
  if (gemm_swiglu_applies(T, F)) return launch_gemm_swiglu(x, K, wg, wu, K, T, K, F, g, u, F, a, lda, st);
  TRY(gemm_nt(x, K, wg, nullptr, T, K, F, g, st));
  TRY(gemm_nt(x, K, wu, nullptr, T, K, F, u, st));
  return launch_swiglu_fwd_rows(g, u, T, F, F, a, lda, st);
}

// dx[T,K] = sum_s dy_s[T,N_s] WT_s[K,N_s]^T with the transposed weights WT_s = W_s^T; ld: leading
// dimension of every dy_s and WT_s, lddx: that of dx
static int gemm_dgrad_t(int nseg, const void* const* dy, const void* const* wt, const int64_t* Ns, int64_t ld,
                        int64_t T, int64_t K, void* dx, int64_t lddx, hipStream_t st) {
  GemmArgs g{};
  g.nseg = nseg;
  for (int s = 0; s < nseg; ++s) g.seg[s] = {dy[s], wt[s], ld ? ld : Ns[s], ld ? ld : Ns[s], (int)Ns[s]};
  g.M = (int)T; g.N = (int)K; g.c = dx; g.ldc = lddx; g.r = nullptr; g.accumulate = 0;
  g.a_kmajor = true; g.b_kmajor = true;
  return launch_gemm(g, st);
}

// da = dy Wd for the transposed copy wdT [F, D], then (dg, du) = SwiGLU gradient; dg, du with leading
// dimension ldd.  One fused launch when the problem fills the chip, otherwise the product into dg
// followed by the activation-gradient kernel in place; same bits either way.
static int down_dgrad_swiglu(const void* dy, const void* wdT, int64_t T, int64_t D, int64_t F, const void* g,
                             const void* u, void* dg, void* du, int64_t ldd, hipStream_t st) {
  if (gemm_swiglu_grad_applies(T, F)) return launch_gemm_swiglu_grad(dy, D, wdT, D, T, D, F, g, u, F, dg, du, ldd, st);
  const void* dys[1] = {dy}; const void* ws[1] = {wdT}; const int64_t ns[1] = {D};
  TRY(gemm_dgrad_t(1, dys, ws, ns, 0, T, F, dg, ldd, st));
  return launch_swiglu_bwd_rows(g, u, dg, T, F, F, ldd, dg, du, st);
}

// dw[N,K] (+)= dy[T,N]^T x[T,K]; lddy, ldx: leading dimensions of dy and x
static GemmArgs wgrad_args(const void* dy, int64_t lddy, const void* x, int64_t ldx, int64_t T, int64_t N, int64_t K,
                           void* dw, int accumulate) {
  GemmArgs g{};
  g.nseg = 1;
  g.seg[0] = {dy, x, lddy, ldx, (int)T};
  g.M = (int)N; g.N = (int)K; g.c = dw; g.ldc = K; g.r = nullptr; g.accumulate = accumulate;
  g.a_kmajor = false; g.b_kmajor = false;
  return g;
}
static int gemm_wgrad(const void* dy, const void* x, int64_t T, int64_t N, int64_t K, void* dw, int accumulate,
                      hipStream_t st) {
  return launch_gemm(wgrad_args(dy, N, x, K, T, N, K, dw, accumulate), st);
}

}  // namespace dl

using namespace dl;

extern "C" {

int dlayer_version(void) { return 1; }
const char* dlayer_last_error(void) { return g_err; }

size_t dlayer_saved_bytes(const dlayer_cfg* cfg) {
  if (cfg_problem(cfg)) return 0;
  return carve_saved(cfg, nullptr).bytes;
}
size_t dlayer_workspace_bytes(const dlayer_cfg* cfg) {
  if (cfg_problem(cfg)) return 0;
  return carve_work(cfg, nullptr).bytes;
}

int dlayer_forward(const dlayer_cfg* cfg, const void* x, const dlayer_weights* w, void* y, void* saved,
                   void* workspace, void* stream) {
  const char* prob = cfg_problem(cfg);
  REQUIRE(!prob, "dlayer_forward: %s", prob);
  REQUIRE(w != nullptr, "dlayer_forward: weights struct is null");
  REQUIRE_PTR(x); REQUIRE_PTR(y); REQUIRE_PTR(saved); REQUIRE_PTR(workspace);
  REQUIRE_PTR(w->g_attn); REQUIRE_PTR(w->wq); REQUIRE_PTR(w->wk); REQUIRE_PTR(w->wv); REQUIRE_PTR(w->wo);
  REQUIRE_PTR(w->g_mlp); REQUIRE_PTR(w->w_gate); REQUIRE_PTR(w->w_up); REQUIRE_PTR(w->w_down);
  REQUIRE(x != y, "dlayer_forward: x and y must not overlap");
  TRY(check_device());
  hipStream_t st = (hipStream_t)stream;
  const int64_t B = cfg->batch, S = cfg->seq, T = B * S, D = cfg->d_model, F = cfg->d_ff;
  const int64_t Hq = cfg->n_q_heads, Hkv = cfg->n_kv_heads, dh = cfg->head_dim, QD = Hq * dh, KD = Hkv * dh;
  Saved s = carve_saved(cfg, saved);
  {
    // what a recomputing configuration does not keep for the backward lives in the workspace for the
    // length of this call
    const Work k = carve_work(cfg, workspace);
    if (!s.h1) { s.h1 = k.h1; s.h2 = k.h2; }
    if (!s.a) s.a = k.a;
  }
  TRY(launch_rmsnorm_fwd(x, w->g_attn, T, D, cfg->rms_eps, s.h1, s.rstd1, st));
  TRY(launch_rope_table(s.rope_cos, s.rope_sin, S, dh, cfg->rope_base, st));
  {
    // q, k and v in one launch: their tile sequences run end to end (k and v alone do not fill the chip
    // for small layers); q and k leave the epilogue rotated, from the fp32 sums
    const GemmArgs qkv[3] = {nt_args(s.h1, D, w->wq, nullptr, T, D, QD, s.q), nt_args(s.h1, D, w->wk, nullptr, T, D, KD, s.k),
                             nt_args(s.h1, D, w->wv, nullptr, T, D, KD, s.v)};
    const RopeEpilogue rope = {s.rope_cos, s.rope_sin, (int)S, (int)dh, cfg->rope_layout, 0x3u};
    TRY(launch_gemm_group_rope(qkv, 3, &rope, st));
  }
  TRY(launch_attention_fwd(s.q, s.k, s.v, B, S, Hq, Hkv, dh, s.o, s.lse, st));
  TRY(gemm_nt(s.o, QD, w->wo, x, T, QD, D, s.y1, st));
  TRY(launch_rmsnorm_fwd(s.y1, w->g_mlp, T, D, cfg->rms_eps, s.h2, s.rstd2, st));
  const int64_t Fp = padded_ff(cfg);
  TRY(gate_up_swiglu(s.h2, w->w_gate, w->w_up, T, D, F, s.g, s.u, s.a, Fp, st));
  TRY(gemm_nt(s.a, Fp, w->w_down, s.y1, T, F, D, y, st));
  return DLAYER_OK;
}

int dlayer_backward(const dlayer_cfg* cfg, const void* x, const dlayer_weights* w, const void* dy,
                    const void* saved, void* dx, const dlayer_wgrads* dw, int flags,
                    void* workspace, void* stream) {
  const char* prob = cfg_problem(cfg);
  REQUIRE(!prob, "dlayer_backward: %s", prob);
  REQUIRE(w != nullptr && dw != nullptr, "dlayer_backward: weights or gradient struct is null");
  REQUIRE((flags & ~(DLAYER_ACCUMULATE_WGRADS | DLAYER_REUSE_TRANSPOSED_WEIGHTS)) == 0, "dlayer_backward: unknown flag bits 0x%x", flags);
  REQUIRE_PTR(x); REQUIRE_PTR(dy); REQUIRE_PTR(saved); REQUIRE_PTR(dx); REQUIRE_PTR(workspace);
  REQUIRE_PTR(w->g_attn); REQUIRE_PTR(w->wq); REQUIRE_PTR(w->wk); REQUIRE_PTR(w->wv); REQUIRE_PTR(w->wo);
  REQUIRE_PTR(w->g_mlp); REQUIRE_PTR(w->w_gate); REQUIRE_PTR(w->w_up); REQUIRE_PTR(w->w_down);
  REQUIRE_PTR(dw->g_attn); REQUIRE_PTR(dw->wq); REQUIRE_PTR(dw->wk); REQUIRE_PTR(dw->wv); REQUIRE_PTR(dw->wo);
  REQUIRE_PTR(dw->g_mlp); REQUIRE_PTR(dw->w_gate); REQUIRE_PTR(dw->w_up); REQUIRE_PTR(dw->w_down);
  TRY(check_device());
  hipStream_t st = (hipStream_t)stream;
  const int acc = (flags & DLAYER_ACCUMULATE_WGRADS) ? 1 : 0;
  const int64_t B = cfg->batch, S = cfg->seq, T = B * S, D = cfg->d_model, F = cfg->d_ff;
  const int64_t Hq = cfg->n_q_heads, Hkv = cfg->n_kv_heads, dh = cfg->head_dim, QD = Hq * dh, KD = Hkv * dh;
  Saved s = carve_saved(cfg, const_cast<void*>(saved));
  Work k = carve_work(cfg, workspace);
  const int64_t Fp = padded_ff(cfg);
  if (!(flags & DLAYER_REUSE_TRANSPOSED_WEIGHTS)) {
    const TransposeJob jobs[7] = {{w->w_down, k.wdT, D, F, D},  {w->w_gate, k.wgT, F, D, Fp}, {w->w_up, k.wuT, F, D, Fp},
                                  {w->wo, k.woT, D, QD, D},     {w->wq, k.wqT, QD, D, QD},    {w->wk, k.wkT, KD, D, KD},
                                  {w->wv, k.wvT, KD, D, KD}};
    TRY(launch_transpose_group(jobs, 7, st));
  }
  // y = y1 + a Wd^T
  TRY(down_dgrad_swiglu(dy, k.wdT, T, D, F, s.g, s.u, k.da_dg, k.du, Fp, st));
  {
    const void* dys[2] = {k.da_dg, k.du}; const void* ws[2] = {k.wgT, k.wuT}; const int64_t ns[2] = {F, F};
    TRY(gemm_dgrad_t(2, dys, ws, ns, Fp, T, D, k.dh2, D, st));
  }
  TRY(launch_rmsnorm_bwd(s.y1, w->g_mlp, s.rstd2, k.dh2, dy, T, D, k.dy1, dw->g_mlp, acc, k.rms_ws, st));
  // y1 = x + o Wo^T
  {
    const void* dys[1] = {k.dy1}; const void* ws[1] = {k.woT}; const int64_t ns[1] = {D};
    TRY(gemm_dgrad_t(1, dys, ws, ns, 0, T, QD, k.d_o, QD, st));
  }
  // dq and dk come back as gradients of the unrotated q and k (inverse rotation inside the kernels' stores)
  TRY(launch_attention_bwd_rope(s.q, s.k, s.v, s.o, k.d_o, s.lse, B, S, Hq, Hkv, dh, k.dq, k.dk, k.dv, k.attn_ws,
                                s.rope_cos, s.rope_sin, cfg->rope_layout, st));
  {
    const void* dys[3] = {k.dq, k.dk, k.dv}; const void* ws[3] = {k.wqT, k.wkT, k.wvT};
    const int64_t ns[3] = {QD, KD, KD};
    TRY(gemm_dgrad_t(3, dys, ws, ns, 0, T, D, k.dh1, D, st));
  }
  TRY(launch_rmsnorm_bwd(x, w->g_attn, s.rstd1, k.dh1, k.dy1, T, D, dx, dw->g_attn, acc, k.rms_ws, st));
  // Recomputing configurations: the normalised activations and the SwiGLU output are only operands of
  // the weight gradients; they are rebuilt here from x, y1 (with the saved statistics) and from g, u.
  if (!s.h1) {
    s.h1 = k.h1; s.h2 = k.h2;
    TRY(launch_rmsnorm_fwd(x, w->g_attn, T, D, cfg->rms_eps, s.h1, s.rstd1, st));
    TRY(launch_rmsnorm_fwd(s.y1, w->g_mlp, T, D, cfg->rms_eps, s.h2, s.rstd2, st));
  }
  if (!s.a) {
    s.a = k.a;
    TRY(launch_swiglu_fwd_rows(s.g, s.u, T, F, F, s.a, Fp, st));
  }
  // All seven weight gradients in one grid: every operand (saved activations, the gradient buffers
  // of the workspace, dy) is still alive here, and one launch fills the chip evenly where the
  // separate products leave partly filled rounds (and two of them are too small to fill it at all).
  const GemmArgs wg[7] = {
      wgrad_args(dy, D, s.a, Fp, T, D, F, dw->w_down, acc),      wgrad_args(k.da_dg, Fp, s.h2, D, T, F, D, dw->w_gate, acc),
      wgrad_args(k.du, Fp, s.h2, D, T, F, D, dw->w_up, acc),     wgrad_args(k.dy1, D, s.o, QD, T, D, QD, dw->wo, acc),
      wgrad_args(k.dq, QD, s.h1, D, T, QD, D, dw->wq, acc),      wgrad_args(k.dk, KD, s.h1, D, T, KD, D, dw->wk, acc),
      wgrad_args(k.dv, KD, s.h1, D, T, KD, D, dw->wv, acc)};
  TRY(launch_gemm_group(wg, 7, st));
  return DLAYER_OK;
}

size_t ce_loss_workspace_bytes(int64_t T, int64_t V) { return T > 0 && V > 0 ? ce_workspace(T, V) : 0; }

int ce_loss_fwd_bwd(const void* logits, const int64_t* targets, int64_t T, int64_t V, float grad_scale,
                    float* loss, void* dlogits, void* workspace, void* stream) {
  REQUIRE(T > 0 && V > 0 && V % 8 == 0, "ce_loss_fwd_bwd: need T > 0, V > 0, V %% 8 == 0 (T=%lld V=%lld)", (long long)T, (long long)V);
  REQUIRE(T < ((int64_t)1 << 31), "ce_loss_fwd_bwd: T too large");
  REQUIRE_PTR(logits); REQUIRE_PTR(dlogits); REQUIRE_PTR(workspace);
  REQUIRE(targets != nullptr && loss != nullptr, "ce_loss_fwd_bwd: targets or loss is null");
  TRY(check_device());
  return launch_ce(logits, targets, T, V, grad_scale, loss, dlogits, workspace, (hipStream_t)stream);
}

int ce_loss_fwd_bwd_static(const void* logits, const int64_t* targets, int64_t T, int64_t V, float grad_scale,
                           float* loss, void* dlogits, void* stream) {
  REQUIRE(T > 0 && V > 0 && V % 8 == 0, "ce_loss_fwd_bwd_static: need T > 0, V > 0, V %% 8 == 0 (T=%lld V=%lld)", (long long)T, (long long)V);
  REQUIRE(T <= ce_static_max_rows(), "ce_loss_fwd_bwd_static: T=%lld exceeds the %lld rows the static scratch holds; use ce_loss_fwd_bwd",
          (long long)T, (long long)ce_static_max_rows());
  REQUIRE_PTR(logits); REQUIRE_PTR(dlogits);
  REQUIRE(targets != nullptr && loss != nullptr, "ce_loss_fwd_bwd_static: targets or loss is null");
  TRY(check_device());
  return launch_ce_static(logits, targets, T, V, grad_scale, loss, dlogits, (hipStream_t)stream);
}

// rows of logits held at a time by lm_head_ce_fwd_bwd
static int64_t lm_head_chunk(int64_t T, int64_t V, int64_t chunk_rows) {
  int64_t c = chunk_rows;
  if (c <= 0) {
    // about 1 GiB of logits: at V = 128256 that is 4096 rows, where the call costs what the unchunked
    // route does (21 ms at T = 8192, D = 4096); with 2048 rows it is 20 % slower, the weight gradient
    // being re-read and re-rounded once per chunk and its products having a shorter contraction
    c = (((int64_t)1 << 30) / (V * 2)) / 256 * 256;
    if (c < 256) c = 256;
  }
  return c < T ? c : T;
}

size_t lm_head_ce_workspace_bytes(int64_t T, int64_t D, int64_t V, int64_t chunk_rows) {
  if (T <= 0 || D <= 0 || V <= 0 || chunk_rows < 0 || chunk_rows % 64) return 0;
  return up256((size_t)lm_head_chunk(T, V, chunk_rows) * V * 2) + up256((size_t)V * D * 2) + up256((size_t)T * 4);
}

int lm_head_ce_fwd_bwd(const void* h, const void* w_lm, const int64_t* targets, int64_t T, int64_t D, int64_t V,
                       float grad_scale, int64_t chunk_rows, float* loss, void* dh, void* dw_lm, int accumulate_dw,
                       void* workspace, void* stream) {
  REQUIRE(T > 0 && D > 0 && V > 0 && T % 64 == 0 && D % 64 == 0 && V % 64 == 0,
          "lm_head_ce_fwd_bwd: T, D and V must be positive multiples of 64");
  REQUIRE(chunk_rows >= 0 && chunk_rows % 64 == 0, "lm_head_ce_fwd_bwd: chunk_rows must be 0 or a multiple of 64");
  const int64_t Tc = lm_head_chunk(T, V, chunk_rows);
  REQUIRE(under_4gib(T, D) && under_4gib(V, D) && under_4gib(Tc, V) &&
              T < ((int64_t)1 << 31),
          "lm_head_ce_fwd_bwd: an operand (or a chunk of logits) reaches 4 GiB");
  REQUIRE_PTR(h); REQUIRE_PTR(w_lm); REQUIRE_PTR(dh); REQUIRE_PTR(dw_lm); REQUIRE_PTR(workspace);
  REQUIRE(targets != nullptr && loss != nullptr, "lm_head_ce_fwd_bwd: targets or loss is null");
  TRY(check_device());
  hipStream_t st = (hipStream_t)stream;
  Carver cv(workspace);
  void* logits = cv.take((size_t)Tc * V * 2);
  void* wT = cv.take((size_t)V * D * 2);
  float* row_loss = (float*)cv.take((size_t)T * 4);
  TRY(launch_transpose(w_lm, wT, V, D, V, st));
  const float scale = grad_scale / (float)T;
  for (int64_t r0 = 0; r0 < T; r0 += Tc) {
    const int64_t rows = T - r0 < Tc ? T - r0 : Tc;
    const bf16_t* hc = (const bf16_t*)h + r0 * D;
    TRY(gemm_nt(hc, D, w_lm, nullptr, rows, D, V, logits, st));
    TRY(launch_ce_rows(logits, targets + r0, rows, V, scale, row_loss + r0, logits, st));
    const void* dys[1] = {logits}; const void* ws[1] = {wT}; const int64_t ns[1] = {V};
    TRY(gemm_dgrad_t(1, dys, ws, ns, 0, rows, D, (bf16_t*)dh + r0 * D, D, st));
    TRY(gemm_wgrad(logits, hc, rows, V, D, dw_lm, (accumulate_dw || r0 > 0) ? 1 : 0, st));
  }
  return launch_ce_mean(row_loss, T, loss, st);
}

int rmsnorm_forward(const void* x, const void* gamma, int64_t T, int64_t D, float eps, void* h, float* rstd,
                    void* stream) {
  REQUIRE(T > 0 && D > 0 && D % 8 == 0 && D <= 16384, "rmsnorm_forward: need T > 0, D %% 8 == 0, D <= 16384");
  REQUIRE_PTR(x); REQUIRE_PTR(gamma); REQUIRE_PTR(h);
  REQUIRE(rstd != nullptr, "rmsnorm_forward: rstd is null");
  TRY(check_device());
  return launch_rmsnorm_fwd(x, gamma, T, D, eps, h, rstd, (hipStream_t)stream);
}

size_t rmsnorm_backward_workspace_bytes(int64_t T, int64_t D) { return T > 0 && D > 0 ? rmsnorm_bwd_workspace(T, D) : 0; }

int rmsnorm_backward(const void* x, const void* gamma, const float* rstd, const void* dh, const void* dres,
                     int64_t T, int64_t D, void* dx, void* dgamma, int accumulate_dgamma, void* workspace,
                     void* stream) {
  REQUIRE(T > 0 && D > 0 && D % 8 == 0 && D <= 16384, "rmsnorm_backward: need T > 0, D %% 8 == 0, D <= 16384");
  REQUIRE_PTR(x); REQUIRE_PTR(gamma); REQUIRE_PTR(dh); REQUIRE_PTR(dx); REQUIRE_PTR(workspace);
  REQUIRE(dgamma != nullptr && rstd != nullptr, "rmsnorm_backward: dgamma or rstd is null");
  REQUIRE(dres == nullptr || aligned16(dres), "rmsnorm_backward: dres is misaligned");
  TRY(check_device());
  return launch_rmsnorm_bwd(x, gamma, rstd, dh, dres, T, D, dx, dgamma, accumulate_dgamma ? 1 : 0, workspace,
                            (hipStream_t)stream);
}

int linear_forward(const void* x, const void* w, const void* residual, int64_t T, int64_t K, int64_t N, void* y,
                   void* stream) {
  REQUIRE(T > 0 && K > 0 && N > 0 && K % 64 == 0 && N % 8 == 0, "linear_forward: need K %% 64 == 0 and N %% 8 == 0");
  REQUIRE(under_4gib(T, K) && under_4gib(N, K) && T < (1 << 30) && N < (1 << 30),
          "linear_forward: an operand reaches 4 GiB");
  REQUIRE_PTR(x); REQUIRE_PTR(w); REQUIRE_PTR(y);
  REQUIRE(residual == nullptr || aligned16(residual), "linear_forward: residual is misaligned");
  TRY(check_device());
  return gemm_nt(x, K, w, residual, T, K, N, y, (hipStream_t)stream);
}

size_t qkv_rope_workspace_bytes(int64_t seq, int64_t head_dim) {
  if (seq <= 0 || (head_dim != 32 && head_dim != 64 && head_dim != 128)) return 0;
  return 2 * up256((size_t)seq * (head_dim / 2) * 4);   // cos and sin tables
}

int qkv_rope_forward(const void* h, const void* wq, const void* wk, const void* wv, int64_t batch, int64_t seq,
                     int64_t d_model, int64_t n_q_heads, int64_t n_kv_heads, int64_t head_dim, float rope_base,
                     int32_t rope_layout, void* q, void* k, void* v, void* workspace, void* stream) {
  REQUIRE(batch > 0 && seq > 0 && d_model > 0 && n_q_heads > 0 && n_kv_heads > 0, "qkv_rope_forward: non-positive dimension");
  REQUIRE(head_dim == 32 || head_dim == 64 || head_dim == 128, "qkv_rope_forward: head_dim must be 32, 64 or 128");
  REQUIRE(d_model % 64 == 0, "qkv_rope_forward: d_model must be a multiple of 64");
  REQUIRE(rope_layout == 0 || rope_layout == 1, "qkv_rope_forward: rope_layout must be 0 or 1");
  REQUIRE(rope_base > 0.f, "qkv_rope_forward: rope_base must be positive");
  const int64_t T = batch * seq, QD = n_q_heads * head_dim, KD = n_kv_heads * head_dim;
  REQUIRE(under_4gib(T, d_model) && under_4gib(QD, d_model) && under_4gib(T, QD) &&
              under_4gib(KD, d_model) && under_4gib(T, KD),
          "qkv_rope_forward: an operand reaches 4 GiB");
  REQUIRE_PTR(h); REQUIRE_PTR(wq); REQUIRE_PTR(wk); REQUIRE_PTR(wv); REQUIRE_PTR(q); REQUIRE_PTR(k); REQUIRE_PTR(v);
  REQUIRE_PTR(workspace);
  TRY(check_device());
  hipStream_t st = (hipStream_t)stream;
  Carver cv(workspace);
  float* cs = (float*)cv.take((size_t)seq * (head_dim / 2) * 4);
  float* sn = (float*)cv.take((size_t)seq * (head_dim / 2) * 4);
  TRY(launch_rope_table(cs, sn, seq, head_dim, rope_base, st));
  const GemmArgs qkv[3] = {nt_args(h, d_model, wq, nullptr, T, d_model, QD, q), nt_args(h, d_model, wk, nullptr, T, d_model, KD, k),
                           nt_args(h, d_model, wv, nullptr, T, d_model, KD, v)};
  const RopeEpilogue rope = {cs, sn, (int)seq, (int)head_dim, rope_layout, 0x3u};
  return launch_gemm_group_rope(qkv, 3, &rope, st);
}

int linear_swiglu_forward(const void* x, const void* w_gate, const void* w_up, int64_t T, int64_t K, int64_t F,
                          void* g, void* u, void* a, void* stream) {
  REQUIRE(T > 0 && K > 0 && F > 0 && K % 64 == 0 && F % 8 == 0,
          "linear_swiglu_forward: need K %% 64 == 0 and F %% 8 == 0");
  REQUIRE(under_4gib(T, K) && under_4gib(F, K) && T < (1 << 30) && F < (1 << 29),
          "linear_swiglu_forward: an operand reaches 4 GiB");
  REQUIRE_PTR(x); REQUIRE_PTR(w_gate); REQUIRE_PTR(w_up); REQUIRE_PTR(g); REQUIRE_PTR(u); REQUIRE_PTR(a);
  TRY(check_device());
  return gate_up_swiglu(x, w_gate, w_up, T, K, F, g, u, a, F, (hipStream_t)stream);
}

size_t linear_backward_workspace_bytes(int64_t T, int64_t K, int64_t N) {
  return T > 0 && K > 0 && N > 0 ? (size_t)N * K * 2 : 0;   // W^T for the input-gradient product
}

int linear_backward(const void* x, const void* w, const void* dy, int64_t T, int64_t K, int64_t N, void* dx,
                    void* dw, int accumulate_dw, void* workspace, void* stream) {
  REQUIRE(T > 0 && K > 0 && N > 0 && T % 64 == 0 && K % 64 == 0 && N % 64 == 0,
          "linear_backward: T, K and N must be multiples of 64");
  REQUIRE(under_4gib(T, K) && under_4gib(N, K) && under_4gib(T, N),
          "linear_backward: an operand reaches 4 GiB");
  REQUIRE_PTR(x); REQUIRE_PTR(w); REQUIRE_PTR(dy);
  REQUIRE((dx == nullptr || aligned16(dx)) && (dw == nullptr || aligned16(dw)), "linear_backward: misaligned output");
  TRY(check_device());
  hipStream_t st = (hipStream_t)stream;
  if (dx) {
    REQUIRE_PTR(workspace);
    TRY(launch_transpose(w, workspace, N, K, N, st));
    const void* dys[1] = {dy}; const void* ws[1] = {workspace}; const int64_t ns[1] = {N};
    TRY(gemm_dgrad_t(1, dys, ws, ns, 0, T, K, dx, K, st));
  }
  if (dw) TRY(gemm_wgrad(dy, x, T, N, K, dw, accumulate_dw ? 1 : 0, st));
  return DLAYER_OK;
}

size_t linear_swiglu_backward_workspace_bytes(int64_t T, int64_t D, int64_t F) {
  return T > 0 && D > 0 && F > 0 ? (size_t)D * F * 2 : 0;   // W_down^T
}

int linear_swiglu_backward(const void* dy, const void* w_down, const void* g, const void* u, int64_t T, int64_t D,
                           int64_t F, void* dg, void* du, void* workspace, void* stream) {
  REQUIRE(T > 0 && D > 0 && F > 0 && T % 64 == 0 && D % 64 == 0 && F % 64 == 0,
          "linear_swiglu_backward: T, D and F must be multiples of 64");
  REQUIRE(under_4gib(T, D) && under_4gib(D, F) && under_4gib(T, F),
          "linear_swiglu_backward: an operand reaches 4 GiB");
  REQUIRE_PTR(dy); REQUIRE_PTR(w_down); REQUIRE_PTR(g); REQUIRE_PTR(u); REQUIRE_PTR(dg); REQUIRE_PTR(du);
  REQUIRE_PTR(workspace);
  TRY(check_device());
  hipStream_t st = (hipStream_t)stream;
  TRY(launch_transpose(w_down, workspace, D, F, D, st));
  return down_dgrad_swiglu(dy, workspace, T, D, F, g, u, dg, du, F, st);
}

int linear_wgrad_group(int32_t n, const void* const* dy, const void* const* x, const int64_t* N, const int64_t* K,
                       int64_t T, void* const* dw, int accumulate_dw, void* stream) {
  REQUIRE(n >= 1 && n <= 8, "linear_wgrad_group: 1..8 products, got %d", (int)n);
  REQUIRE(dy && x && N && K && dw, "linear_wgrad_group: null argument array");
  REQUIRE(T > 0 && T % 64 == 0, "linear_wgrad_group: T must be a positive multiple of 64");
  GemmArgs gs[8];
  for (int i = 0; i < n; ++i) {
    REQUIRE(N[i] > 0 && K[i] > 0 && N[i] % 64 == 0 && K[i] % 64 == 0,
            "linear_wgrad_group: N[%d] and K[%d] must be positive multiples of 64", i, i);
    REQUIRE(under_4gib(T, K[i]) && under_4gib(N[i], K[i]) && under_4gib(T, N[i]),
            "linear_wgrad_group: an operand of product %d reaches 4 GiB", i);
    REQUIRE(dy[i] && x[i] && dw[i] && aligned16(dy[i]) && aligned16(x[i]) && aligned16(dw[i]),
            "linear_wgrad_group: a pointer of product %d is null or not 16-byte aligned", i);
    gs[i] = wgrad_args(dy[i], N[i], x[i], K[i], T, N[i], K[i], dw[i], accumulate_dw ? 1 : 0);
  }
  TRY(check_device());
  return launch_gemm_group(gs, n, (hipStream_t)stream);
}

int rope_apply(void* z, int64_t batch, int64_t seq, int64_t n_heads, int64_t head_dim, float rope_base,
               int32_t rope_layout, int32_t inverse, void* stream) {
  REQUIRE(batch > 0 && seq > 0 && n_heads > 0, "rope_apply: non-positive dimension");
  REQUIRE(head_dim == 32 || head_dim == 64 || head_dim == 128, "rope_apply: head_dim must be 32, 64 or 128");
  REQUIRE(rope_layout == 0 || rope_layout == 1, "rope_apply: rope_layout must be 0 or 1");
  REQUIRE(rope_base > 0.f, "rope_apply: rope_base must be positive");
  REQUIRE_PTR(z);
  TRY(check_device());
  return launch_rope(z, batch, seq, n_heads, head_dim, rope_base, rope_layout, inverse ? 1 : 0, (hipStream_t)stream);
}

static int attn_shape_ok(int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t dh, const char* who) {
  REQUIRE(B > 0 && S > 0 && Hq > 0 && Hkv > 0, "%s: non-positive dimension", who);
  REQUIRE(dh == 32 || dh == 64 || dh == 128, "%s: head_dim must be 32, 64 or 128", who);
  REQUIRE(Hq % Hkv == 0, "%s: n_q_heads must be a multiple of n_kv_heads", who);
  REQUIRE(S % 128 == 0, "%s: seq must be a multiple of 128", who);
  REQUIRE(under_4gib(B, S) && under_4gib(Hq, dh) && under_4gib(B * S, Hq * dh), "%s: q reaches 4 GiB", who);
  REQUIRE(B < 65536 && Hq < 65536, "%s: batch or head count too large", who);
  return 0;
}

int attention_forward(const void* q, const void* k, const void* v, int64_t batch, int64_t seq, int64_t n_q_heads,
                      int64_t n_kv_heads, int64_t head_dim, void* o, float* lse, void* stream) {
  TRY(attn_shape_ok(batch, seq, n_q_heads, n_kv_heads, head_dim, "attention_forward"));
  REQUIRE_PTR(q); REQUIRE_PTR(k); REQUIRE_PTR(v); REQUIRE_PTR(o);
  REQUIRE(lse != nullptr, "attention_forward: lse is null");
  TRY(check_device());
  return launch_attention_fwd(q, k, v, batch, seq, n_q_heads, n_kv_heads, head_dim, o, lse, (hipStream_t)stream);
}

size_t attention_backward_workspace_bytes(int64_t batch, int64_t seq, int64_t n_q_heads, int64_t n_kv_heads,
                                          int64_t head_dim) {
  if (batch <= 0 || seq <= 0 || n_q_heads <= 0) return 0;
  return attention_bwd_workspace(batch, seq, n_q_heads, n_kv_heads, head_dim);
}

int attention_backward(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                       const float* lse, int64_t batch, int64_t seq, int64_t n_q_heads, int64_t n_kv_heads,
                       int64_t head_dim, void* dq, void* dk, void* dv, void* workspace, void* stream) {
  TRY(attn_shape_ok(batch, seq, n_q_heads, n_kv_heads, head_dim, "attention_backward"));
  REQUIRE_PTR(q); REQUIRE_PTR(k); REQUIRE_PTR(v); REQUIRE_PTR(o); REQUIRE_PTR(d_o);
  REQUIRE_PTR(dq); REQUIRE_PTR(dk); REQUIRE_PTR(dv); REQUIRE_PTR(workspace);
  REQUIRE(lse != nullptr, "attention_backward: lse is null");
  TRY(check_device());
  return launch_attention_bwd(q, k, v, o, d_o, lse, batch, seq, n_q_heads, n_kv_heads, head_dim, dq, dk, dv,
                              workspace, (hipStream_t)stream);
}

static int opt_args_ok(const char* who, int32_t n, const int64_t* numel) {
  REQUIRE(n >= 1 && n <= kOptMaxTensors, "%s: 1..%d tensors per call, got %d", who, kOptMaxTensors, (int)n);
  REQUIRE(numel != nullptr, "%s: numel is null", who);
  int64_t chunks = 0;
  for (int i = 0; i < n; ++i) {
    REQUIRE(numel[i] > 0 && numel[i] % 8 == 0, "%s: numel[%d] must be a positive multiple of 8", who, i);
    chunks += (numel[i] + 16383) / 16384;
  }
  REQUIRE(chunks < ((int64_t)1 << 31), "%s: too many elements for one call", who);
  return 0;
}

size_t grad_sq_norm_workspace_bytes(int32_t n, const int64_t* numel) {
  if (n < 1 || n > kOptMaxTensors || !numel) return 0;
  for (int i = 0; i < n; ++i) if (numel[i] <= 0) return 0;
  return up256((size_t)opt_chunks(n, numel) * sizeof(float));
}

int grad_sq_norm(int32_t n, const void* const* grads, const int64_t* numel, float* sq_norm, int accumulate,
                 void* workspace, void* stream) {
  TRY(opt_args_ok("grad_sq_norm", n, numel));
  REQUIRE(grads != nullptr && sq_norm != nullptr, "grad_sq_norm: grads or sq_norm is null");
  REQUIRE_PTR(workspace);
  for (int i = 0; i < n; ++i)
    REQUIRE(grads[i] != nullptr && aligned16(grads[i]), "grad_sq_norm: grads[%d] is null or not 16-byte aligned", i);
  TRY(check_device());
  return launch_grad_sq_norm(n, grads, numel, sq_norm, (float*)workspace, accumulate ? 1 : 0, (hipStream_t)stream);
}

int adamw_step(int32_t n, void* const* params, const void* const* grads, float* const* exp_avg, float* const* exp_avg_sq,
               const int64_t* numel, int64_t step, float lr, float beta1, float beta2, float eps, float weight_decay,
               float max_grad_norm, const float* sq_norm, void* stream) {
  TRY(opt_args_ok("adamw_step", n, numel));
  REQUIRE(params && grads && exp_avg && exp_avg_sq, "adamw_step: null tensor list");
  REQUIRE(step >= 1, "adamw_step: the step counter starts at 1");
  REQUIRE(lr >= 0.f && beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f && eps >= 0.f && weight_decay >= 0.f,
          "adamw_step: need lr >= 0, 0 <= beta < 1, eps >= 0, weight_decay >= 0");
  REQUIRE(sq_norm == nullptr || max_grad_norm > 0.f, "adamw_step: max_grad_norm must be positive when sq_norm is given");
  for (int i = 0; i < n; ++i)
    REQUIRE(params[i] && grads[i] && exp_avg[i] && exp_avg_sq[i] && aligned16(params[i]) && aligned16(grads[i]) &&
                aligned16(exp_avg[i]) && aligned16(exp_avg_sq[i]),
            "adamw_step: a pointer of tensor %d is null or not 16-byte aligned", i);
  TRY(check_device());
  return launch_adamw(n, params, grads, exp_avg, exp_avg_sq, numel, step, lr, beta1, beta2, eps, weight_decay,
                      max_grad_norm, sq_norm, (hipStream_t)stream);
}

int swiglu_forward(const void* g, const void* u, int64_t n, void* a, void* stream) {
  REQUIRE(n > 0 && n % 8 == 0, "swiglu_forward: n must be a positive multiple of 8");
  REQUIRE_PTR(g); REQUIRE_PTR(u); REQUIRE_PTR(a);
  TRY(check_device());
  return launch_swiglu_fwd(g, u, n, a, (hipStream_t)stream);
}

int swiglu_backward(const void* g, const void* u, const void* da, int64_t n, void* dg, void* du, void* stream) {
  REQUIRE(n > 0 && n % 8 == 0, "swiglu_backward: n must be a positive multiple of 8");
  REQUIRE_PTR(g); REQUIRE_PTR(u); REQUIRE_PTR(da); REQUIRE_PTR(dg); REQUIRE_PTR(du);
  TRY(check_device());
  return launch_swiglu_bwd(g, u, da, n, dg, du, (hipStream_t)stream);
}

int embed_forward(const void* table, const int64_t* ids, int64_t T, int64_t V, int64_t D, void* x0, void* stream) {
  REQUIRE(T > 0 && V > 0 && D > 0 && D % 8 == 0 && T < ((int64_t)1 << 31), "embed_forward: need T, V > 0 and D %% 8 == 0");
  REQUIRE_PTR(table); REQUIRE_PTR(x0);
  REQUIRE(ids != nullptr, "embed_forward: ids is null");
  TRY(check_device());
  return launch_embed_fwd(table, ids, T, V, D, x0, (hipStream_t)stream);
}

size_t embed_backward_workspace_bytes(int64_t T, int64_t V) { return T > 0 && V > 0 ? embed_bwd_workspace(T, V) : 0; }

int embed_backward(const void* dx0, const int64_t* ids, int64_t T, int64_t V, int64_t D, void* dtable,
                   void* workspace, void* stream) {
  REQUIRE(T > 0 && V > 0 && D > 0 && D % 8 == 0 && T < ((int64_t)1 << 30) && V < ((int64_t)1 << 30),
          "embed_backward: need 0 < T, V < 2^30 and D %% 8 == 0");
  REQUIRE_PTR(dx0); REQUIRE_PTR(dtable); REQUIRE_PTR(workspace);
  REQUIRE(ids != nullptr, "embed_backward: ids is null");
  TRY(check_device());
  return launch_embed_bwd(dx0, ids, T, V, D, dtable, workspace, (hipStream_t)stream);
}

int issue_rate_probe(int family, int variant, int waves_per_simd, double* result, void* stream) {
  REQUIRE(result != nullptr, "issue_rate_probe: result is null");
  REQUIRE(family >= 0 && family <= 3 && variant >= 0 && variant <= 3, "issue_rate_probe: family 0..3, variant 0..3");
  TRY(check_device());
  return launch_probe(family, variant, waves_per_simd, result, (hipStream_t)stream);
}

}  // extern "C"
