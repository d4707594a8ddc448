// Memory-bound kernels of the decoder layer: RMSNorm forward/backward, rotary embedding,
// SwiGLU forward/backward, bf16 matrix transpose, embedding gather and its gradient.
// All of them move 16 bytes per lane per access (8 bf16) with consecutive lanes on
// consecutive addresses, keep a row in registers between the reduction and the write, and
// reduce with wavefront shuffles.
#include "common.h"
#include "kernels.h"

namespace dl {

// ------------------------------------------------------------------------------------------
// RMSNorm forward: one wavefront per token row, the row stays in registers.
// ------------------------------------------------------------------------------------------
template <int NV>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const bf16_t* __restrict__ x,
                                                          const bf16_t* __restrict__ gamma,
                                                          bf16_t* __restrict__ h,
                                                          float* __restrict__ rstd, int64_t T,
                                                          int D, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T) return;
  const int nvec = D >> 3;
  const bf16x8* xr = reinterpret_cast<const bf16x8*>(x + row * D);
  bf16x8 v[NV];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = i * 64 + lane;
    if (c < nvec) {
      v[i] = xr[c];
#pragma unroll
      for (int e = 0; e < 8; ++e) { float f = (float)v[i][e]; ss += f * f; }
    }
  }
  ss = wave_sum(ss);
  const float r = 1.0f / sqrtf(ss / (float)D + eps);
  if (lane == 0) rstd[row] = r;
  bf16x8* hr = reinterpret_cast<bf16x8*>(h + row * D);
  const bf16x8* gr = reinterpret_cast<const bf16x8*>(gamma);
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = i * 64 + lane;
    if (c < nvec) {
      bf16x8 g = gr[c], o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (bf16_t)((float)v[i][e] * r * (float)g[e]);
      hr[c] = o;
    }
  }
}

int launch_rmsnorm_fwd(const void* x, const void* gamma, int64_t T, int64_t D, float eps, void* h,
                       float* rstd, hipStream_t st) {
  const int nv = (int)((D / 8 + 63) / 64);
  dim3 grid((unsigned)((T + 3) / 4)), block(256);
#define RMS_FWD(NV)                                                                             \
  hipLaunchKernelGGL(rmsnorm_fwd_kernel<NV>, grid, block, 0, st, (const bf16_t*)x,              \
                     (const bf16_t*)gamma, (bf16_t*)h, rstd, T, (int)D, eps)
  if (nv <= 1) RMS_FWD(1);
  else if (nv <= 2) RMS_FWD(2);
  else if (nv <= 4) RMS_FWD(4);
  else if (nv <= 8) RMS_FWD(8);
  else if (nv <= 16) RMS_FWD(16);
  else RMS_FWD(32);
#undef RMS_FWD
  return check_launch("rmsnorm_forward");
}

// ------------------------------------------------------------------------------------------
// RMSNorm backward.  Each wavefront walks rows with a grid stride, writes dx for its rows and
// keeps the gain-gradient partial sums of its columns in registers; the block then folds its
// waves through LDS and writes one fp32 partial row; a second kernel sums the partial rows.
// ------------------------------------------------------------------------------------------
constexpr int kRmsBwdWaves = 8;
constexpr int kRmsBwdChunk = 4096;   // columns a wave keeps gain-gradient sums for (8 vectors of 8 per lane)

// mean_d(dh * gamma * xhat) per row, for rows wider than one chunk: one wave per row at a time
__global__ __launch_bounds__(256) void rms_dot_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ gamma,
                                                      const float* __restrict__ rstd, const bf16_t* __restrict__ dh,
                                                      float* __restrict__ dot, int64_t T, int D) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nvec = D >> 3;
  for (int64_t row = (int64_t)blockIdx.x * 4 + wave; row < T; row += (int64_t)gridDim.x * 4) {
    const bf16x8* xr = reinterpret_cast<const bf16x8*>(x + row * D);
    const bf16x8* dr = reinterpret_cast<const bf16x8*>(dh + row * D);
    const bf16x8* gr = reinterpret_cast<const bf16x8*>(gamma);
    const float r = rstd[row];
    float s = 0.f;
    for (int c = lane; c < nvec; c += 64) {
      const bf16x8 xv = xr[c], dv = dr[c], gv = gr[c];
#pragma unroll
      for (int e = 0; e < 8; ++e) s += (float)dv[e] * (float)gv[e] * ((float)xv[e] * r);
    }
    s = wave_sum(s);
    if (lane == 0) dot[row] = s / (float)D;
  }
}

template <int NV>
__global__ __launch_bounds__(64 * kRmsBwdWaves) void rmsnorm_bwd_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ gamma, const float* __restrict__ rstd,
    const bf16_t* __restrict__ dh, const bf16_t* dres, bf16_t* dx, float* __restrict__ partial,
    int64_t T, int D, const float* __restrict__ dot_in) {
  // Rows wider than 4096 are handled in column chunks of 4096, one per blockIdx.y, with the row's
  // mean_d(dxhat * xhat) taken from dot_in (a kernel of its own computes it first); gridDim.y == 1 and
  // dot_in == nullptr is the one-pass case.
  extern __shared__ float red[];  // [kRmsBwdWaves][Dc]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int base = blockIdx.y * kRmsBwdChunk;
  const int Dc = gridDim.y == 1 ? D : min(kRmsBwdChunk, D - base);
  x += base; dh += base; dx += base; gamma += base;
  if (dres) dres += base;
  const int nvec = Dc >> 3;
  float dg[NV][8];
  bf16x8 gv[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = i * 64 + lane;
    if (c < nvec) gv[i] = reinterpret_cast<const bf16x8*>(gamma)[c];
#pragma unroll
    for (int e = 0; e < 8; ++e) dg[i][e] = 0.f;
  }
  const int64_t wstride = (int64_t)gridDim.x * kRmsBwdWaves;
  for (int64_t row = (int64_t)blockIdx.x * kRmsBwdWaves + wave; row < T; row += wstride) {
    const bf16x8* xr = reinterpret_cast<const bf16x8*>(x + row * D);
    const bf16x8* dr = reinterpret_cast<const bf16x8*>(dh + row * D);
    const float r = rstd[row];
    bf16x8 xv[NV], dv[NV];
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = i * 64 + lane;
      if (c < nvec) {
        xv[i] = xr[c];
        dv[i] = dr[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (float)xv[i][e] * r, d = (float)dv[i][e];
          dg[i][e] += d * xh;
          dot += d * (float)gv[i][e] * xh;
        }
      }
    }
    dot = dot_in ? dot_in[row] : wave_sum(dot) / (float)D;
    bf16x8* oxr = reinterpret_cast<bf16x8*>(dx + row * D);
    const bf16x8* rr = dres ? reinterpret_cast<const bf16x8*>(dres + row * D) : nullptr;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = i * 64 + lane;
      if (c < nvec) {
        bf16x8 o, rs;
        if (rr) rs = rr[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xh = (float)xv[i][e] * r;
          float g = r * ((float)dv[i][e] * (float)gv[i][e] - xh * dot);
          if (rr) g += (float)rs[e];
          o[e] = (bf16_t)g;
        }
        oxr[c] = o;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = i * 64 + lane;
    if (c < nvec) {
#pragma unroll
      for (int e = 0; e < 8; ++e) red[wave * Dc + c * 8 + e] = dg[i][e];
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < Dc; c += blockDim.x) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kRmsBwdWaves; ++w) s += red[w * Dc + c];
    partial[(int64_t)blockIdx.x * D + base + c] = s;
  }
}

// Column sums of the per-block partial rows: 256 threads = 32 columns x 8 row groups, folded through LDS.
__global__ __launch_bounds__(256) void colsum_partials_kernel(const float* __restrict__ partial, int nrows, int D,
                                                              bf16_t* out, int accumulate) {
  __shared__ float red[8][33];
  const int cl = threadIdx.x & 31, rg = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cl;
  // four loads in flight per thread: the loop is latency-bound otherwise (20 us for 512 rows)
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (c < D) {
    int r = rg;
    for (; r + 24 < nrows; r += 32) {
      s0 += partial[(int64_t)r * D + c];
      s1 += partial[(int64_t)(r + 8) * D + c];
      s2 += partial[(int64_t)(r + 16) * D + c];
      s3 += partial[(int64_t)(r + 24) * D + c];
    }
    for (; r < nrows; r += 8) s0 += partial[(int64_t)r * D + c];
  }
  red[rg][cl] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (rg == 0 && c < D) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < 8; ++g) t += red[g][cl];
    if (accumulate) t += (float)out[c];
    out[c] = (bf16_t)t;
  }
}

static int rms_bwd_blocks(int64_t T) {
  int64_t b = (T + kRmsBwdWaves - 1) / kRmsBwdWaves;
  return (int)(b < 512 ? b : 512);
}
size_t rmsnorm_bwd_workspace(int64_t T, int64_t D) {
  return (size_t)rms_bwd_blocks(T) * D * sizeof(float) + (D > kRmsBwdChunk ? (size_t)T * sizeof(float) : 0);
}

int launch_rmsnorm_bwd(const void* x, const void* gamma, const float* rstd, const void* dh,
                       const void* dres, int64_t T, int64_t D, void* dx, void* dgamma,
                       int accumulate, void* workspace, hipStream_t st) {
  const int nchunk = (int)((D + kRmsBwdChunk - 1) / kRmsBwdChunk);
  const int64_t Dc = nchunk == 1 ? D : kRmsBwdChunk;       // widest chunk
  const int nv = (int)((Dc / 8 + 63) / 64);
  const int nb = rms_bwd_blocks(T);
  const size_t lds = (size_t)kRmsBwdWaves * Dc * sizeof(float);
  float* partial = (float*)workspace;
  float* dot = nullptr;
  if (nchunk > 1) {
    dot = partial + (size_t)nb * D;
    hipLaunchKernelGGL(rms_dot_kernel, dim3((unsigned)(T < 4096 ? (T + 3) / 4 : 1024)), dim3(256), 0, st, (const bf16_t*)x,
                       (const bf16_t*)gamma, rstd, (const bf16_t*)dh, dot, T, (int)D);
    if (int rc = check_launch("rmsnorm_backward(dot)")) return rc;
  }
  dim3 grid(nb, nchunk), block(64 * kRmsBwdWaves);
#define RMS_BWD(NV)                                                                             \
  do {                                                                                          \
    static std::atomic<unsigned long long> lds_done{0};                                                     \
    if (int rc_ = reserve_lds(rmsnorm_bwd_kernel<NV>, (size_t)kRmsBwdWaves * NV * 512 * sizeof(float), lds_done,        \
                              "rmsnorm_backward")) return rc_;                                  \
    hipLaunchKernelGGL(rmsnorm_bwd_kernel<NV>, grid, block, lds, st, (const bf16_t*)x,          \
                       (const bf16_t*)gamma, rstd, (const bf16_t*)dh, (const bf16_t*)dres,      \
                       (bf16_t*)dx, partial, T, (int)D, (const float*)dot);                     \
  } while (0)
  if (nv <= 1) RMS_BWD(1);
  else if (nv <= 2) RMS_BWD(2);
  else if (nv <= 4) RMS_BWD(4);
  else RMS_BWD(8);
#undef RMS_BWD
  int rc = check_launch("rmsnorm_backward");
  if (rc) return rc;
  hipLaunchKernelGGL(colsum_partials_kernel, dim3((unsigned)((D + 31) / 32)), dim3(256), 0, st,
                     (const float*)workspace, nb, (int)D, (bf16_t*)dgamma, accumulate);
  return check_launch("rmsnorm_backward(dgamma)");
}

// ------------------------------------------------------------------------------------------
// Rotary embedding, in place.  One block per token: the first head_dim/2 threads evaluate the
// angle p * base^(-2i/dh) and its sine/cosine in fp64 (positions reach 8191 rad, where fp32
// range reduction is not accurate enough), park them in LDS as fp32, then every thread rotates
// pairs of all heads of that token.
// ------------------------------------------------------------------------------------------
// rotates all heads of one token row zt ([n_heads, head_dim]) with the angles parked in cs / sn
__device__ __forceinline__ void rope_rotate_row(bf16_t* zt, const float* cs, const float* sn, int n_heads,
                                                int head_dim, int layout) {
  const int half = head_dim >> 1;
  if (layout == 0) {
    // pairs (i, i + half): handle 8 consecutive i per thread
    const int groups = half >> 3;  // per head
    for (int w = threadIdx.x; w < n_heads * groups; w += blockDim.x) {
      const int hd = w / groups, i0 = (w % groups) << 3;
      bf16x8* pa = reinterpret_cast<bf16x8*>(zt + hd * head_dim + i0);
      bf16x8* pb = reinterpret_cast<bf16x8*>(zt + hd * head_dim + half + i0);
      bf16x8 a = *pa, b = *pb, oa, ob;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float c = cs[i0 + e], s = sn[i0 + e], fa = (float)a[e], fb = (float)b[e];
        oa[e] = (bf16_t)(fa * c - fb * s);
        ob[e] = (bf16_t)(fa * s + fb * c);
      }
      *pa = oa;
      *pb = ob;
    }
  } else {
    const int groups = head_dim >> 3;
    for (int w = threadIdx.x; w < n_heads * groups; w += blockDim.x) {
      const int hd = w / groups, e0 = (w % groups) << 3;
      bf16x8* pz = reinterpret_cast<bf16x8*>(zt + hd * head_dim + e0);
      bf16x8 v = *pz, o;
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const int i = (e0 + e) >> 1;
        const float c = cs[i], s = sn[i], fa = (float)v[e], fb = (float)v[e + 1];
        o[e] = (bf16_t)(fa * c - fb * s);
        o[e + 1] = (bf16_t)(fa * s + fb * c);
      }
      *pz = o;
    }
  }
}

// z2 (n_heads2 heads per token) is an optional second tensor rotated by the same angles: q and k of
// a layer in one launch, with the fp64 trigonometry done once.
__global__ __launch_bounds__(256) void rope_kernel(bf16_t* z, bf16_t* z2, int seq, int n_heads, int n_heads2,
                                                   int head_dim, double log2_base, int layout, int inverse) {
  __shared__ float cs[64], sn[64];
  const int64_t tok = blockIdx.x;
  const int p = (int)(tok % seq);
  const int half = head_dim >> 1;
  if ((int)threadIdx.x < half) {
    const double theta = exp2(-2.0 * (double)threadIdx.x / (double)head_dim * log2_base);
    double s, c;
    sincos((double)p * theta, &s, &c);
    cs[threadIdx.x] = (float)c;
    sn[threadIdx.x] = inverse ? -(float)s : (float)s;
  }
  __syncthreads();
  rope_rotate_row(z + tok * (int64_t)n_heads * head_dim, cs, sn, n_heads, head_dim, layout);
  if (z2) rope_rotate_row(z2 + tok * (int64_t)n_heads2 * head_dim, cs, sn, n_heads2, head_dim, layout);
}

int launch_rope(void* z, int64_t batch, int64_t seq, int64_t n_heads, int64_t head_dim,
                float base, int layout, int inverse, hipStream_t st) {
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)(batch * seq)), dim3(256), 0, st, (bf16_t*)z, (bf16_t*)nullptr,
                     (int)seq, (int)n_heads, 0, (int)head_dim, log2((double)base), layout, inverse);
  return check_launch("rope_apply");
}

int launch_rope_pair(void* q, void* k, int64_t batch, int64_t seq, int64_t n_q_heads, int64_t n_kv_heads,
                     int64_t head_dim, float base, int layout, int inverse, hipStream_t st) {
  hipLaunchKernelGGL(rope_kernel, dim3((unsigned)(batch * seq)), dim3(256), 0, st, (bf16_t*)q, (bf16_t*)k, (int)seq,
                     (int)n_q_heads, (int)n_kv_heads, (int)head_dim, log2((double)base), layout, inverse);
  return check_launch("rope_apply(q, k)");
}

// The angles as a table for the kernels that rotate inside another pass (the q/k projection epilogue,
// the attention backward stores): one thread per (position, pair).
__global__ __launch_bounds__(256) void rope_table_kernel(float* __restrict__ cs, float* __restrict__ sn, int seq, int half,
                                                         double log2_base) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= seq * half) return;
  const int p = idx / half, i = idx % half;
  const double theta = exp2(-(double)i / (double)half * log2_base);
  double s, c;
  sincos((double)p * theta, &s, &c);
  cs[idx] = (float)c;
  sn[idx] = (float)s;
}

int launch_rope_table(float* cos, float* sin, int64_t seq, int64_t head_dim, float base, hipStream_t st) {
  const int64_t n = seq * (head_dim / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, cos, sin, (int)seq,
                     (int)(head_dim / 2), log2((double)base));
  return check_launch("rope table");
}

// ------------------------------------------------------------------------------------------
// SwiGLU
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const bf16x8* __restrict__ g,
                                                         const bf16x8* __restrict__ u,
                                                         bf16x8* __restrict__ a, int64_t nvec) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec;
       i += (int64_t)gridDim.x * blockDim.x) {
    bf16x8 gv = g[i], uv = u[i], o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float z = (float)gv[e];
      o[e] = (bf16_t)(z * logistic(z) * (float)uv[e]);
    }
    a[i] = o;
  }
}

__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const bf16x8* g, const bf16x8* u,
                                                         const bf16x8* __restrict__ da, bf16x8* dg,
                                                         bf16x8* du, int64_t nvec) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec;
       i += (int64_t)gridDim.x * blockDim.x) {
    bf16x8 gv = g[i], uv = u[i], dv = da[i], og, ou;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float z = (float)gv[e], d = (float)dv[e];
      const float s = logistic(z);
      og[e] = (bf16_t)(d * (float)uv[e] * s * (1.0f + z * (1.0f - s)));
      ou[e] = (bf16_t)(d * z * s);
    }
    dg[i] = og;
    du[i] = ou;
  }
}

// Row variants: g, u are [rows, cols] with leading dimension ld_gu, the other arrays with ld_p
// (the layer keeps a, da/dg and du with padded rows).  One row per workgroup at a time.
constexpr int SW_U = 4;   // 16-byte vectors per thread in flight
__device__ __forceinline__ bf16x8 swiglu_vec(bf16x8 gv, bf16x8 uv) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float z = (float)gv[e];
    o[e] = (bf16_t)(z * logistic(z) * (float)uv[e]);
  }
  return o;
}
__device__ __forceinline__ void swiglu_grad_vec(bf16x8 gv, bf16x8 uv, bf16x8 dv, bf16x8& og, bf16x8& ou) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float z = (float)gv[e], d = (float)dv[e];
    const float sg = logistic(z);
    og[e] = (bf16_t)(d * (float)uv[e] * sg * (1.0f + z * (1.0f - sg)));
    ou[e] = (bf16_t)(d * z * sg);
  }
}

__global__ __launch_bounds__(256) void swiglu_fwd_rows_kernel(const bf16_t* __restrict__ g, const bf16_t* __restrict__ u,
                                                              bf16_t* __restrict__ a, int rows, int cols_vec,
                                                              int64_t ld_gu, int64_t ld_p) {
  for (int r = blockIdx.x; r < rows; r += gridDim.x) {
    const bf16x8* gr = reinterpret_cast<const bf16x8*>(g + r * ld_gu);
    const bf16x8* ur = reinterpret_cast<const bf16x8*>(u + r * ld_gu);
    bf16x8* ar = reinterpret_cast<bf16x8*>(a + r * ld_p);
    for (int i0 = threadIdx.x; i0 < cols_vec; i0 += 256 * SW_U) {
      bf16x8 gv[SW_U], uv[SW_U];
#pragma unroll
      for (int q = 0; q < SW_U; ++q) {
        const int i = i0 + q * 256;
        if (i < cols_vec) { gv[q] = __builtin_nontemporal_load(gr + i); uv[q] = __builtin_nontemporal_load(ur + i); }
      }
#pragma unroll
      for (int q = 0; q < SW_U; ++q) {
        const int i = i0 + q * 256;
        if (i < cols_vec) ar[i] = swiglu_vec(gv[q], uv[q]);
      }
    }
  }
}

__global__ __launch_bounds__(256) void swiglu_bwd_rows_kernel(const bf16_t* __restrict__ g, const bf16_t* __restrict__ u,
                                                              const bf16_t* da, bf16_t* dg, bf16_t* __restrict__ du,
                                                              int rows, int cols_vec, int64_t ld_gu, int64_t ld_p) {
  for (int r = blockIdx.x; r < rows; r += gridDim.x) {
    const bf16x8* gr = reinterpret_cast<const bf16x8*>(g + r * ld_gu);
    const bf16x8* ur = reinterpret_cast<const bf16x8*>(u + r * ld_gu);
    const bf16x8* dr = reinterpret_cast<const bf16x8*>(da + r * ld_p);
    bf16x8* ogr = reinterpret_cast<bf16x8*>(dg + r * ld_p);
    bf16x8* our = reinterpret_cast<bf16x8*>(du + r * ld_p);
    for (int i0 = threadIdx.x; i0 < cols_vec; i0 += 256 * SW_U) {
      bf16x8 gv[SW_U], uv[SW_U], dv[SW_U];
#pragma unroll
      for (int q = 0; q < SW_U; ++q) {
        const int i = i0 + q * 256;
        if (i < cols_vec) {
          gv[q] = __builtin_nontemporal_load(gr + i); uv[q] = __builtin_nontemporal_load(ur + i); dv[q] = dr[i];
        }
      }
#pragma unroll
      for (int q = 0; q < SW_U; ++q) {
        const int i = i0 + q * 256;
        if (i < cols_vec) {
          bf16x8 og, ou;
          swiglu_grad_vec(gv[q], uv[q], dv[q], og, ou);
          ogr[i] = og;
          our[i] = ou;
        }
      }
    }
  }
}

static unsigned ew_blocks(int64_t nvec) {
  int64_t b = (nvec + 255) / 256;
  return (unsigned)(b < 256 * 16 ? (b > 0 ? b : 1) : 256 * 16);
}

int launch_swiglu_fwd(const void* g, const void* u, int64_t n, void* a, hipStream_t st) {
  hipLaunchKernelGGL(swiglu_fwd_kernel, dim3(ew_blocks(n / 8)), dim3(256), 0, st, (const bf16x8*)g,
                     (const bf16x8*)u, (bf16x8*)a, n / 8);
  return check_launch("swiglu_forward");
}
int launch_swiglu_bwd(const void* g, const void* u, const void* da, int64_t n, void* dg, void* du,
                      hipStream_t st) {
  hipLaunchKernelGGL(swiglu_bwd_kernel, dim3(ew_blocks(n / 8)), dim3(256), 0, st, (const bf16x8*)g,
                     (const bf16x8*)u, (const bf16x8*)da, (bf16x8*)dg, (bf16x8*)du, n / 8);
  return check_launch("swiglu_backward");
}

int launch_swiglu_fwd_rows(const void* g, const void* u, int64_t rows, int64_t cols, int64_t ld_gu, void* a,
                           int64_t ld_a, hipStream_t st) {
  hipLaunchKernelGGL(swiglu_fwd_rows_kernel, dim3((unsigned)(rows < 8192 ? rows : 8192)), dim3(256), 0, st,
                     (const bf16_t*)g, (const bf16_t*)u, (bf16_t*)a, (int)rows, (int)(cols / 8), ld_gu, ld_a);
  return check_launch("swiglu_forward(rows)");
}
int launch_swiglu_bwd_rows(const void* g, const void* u, const void* da, int64_t rows, int64_t cols, int64_t ld_gu,
                           int64_t ld_p, void* dg, void* du, hipStream_t st) {
  hipLaunchKernelGGL(swiglu_bwd_rows_kernel, dim3((unsigned)(rows < 8192 ? rows : 8192)), dim3(256), 0, st,
                     (const bf16_t*)g, (const bf16_t*)u, (const bf16_t*)da, (bf16_t*)dg, (bf16_t*)du, (int)rows,
                     (int)(cols / 8), ld_gu, ld_p);
  return check_launch("swiglu_backward(rows)");
}

// ------------------------------------------------------------------------------------------
// bf16 transpose: out[c][r] = in[r][c], 64x64 tiles through LDS (16-byte global accesses on
// both sides).  R and C are multiples of 64.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void transpose_tile(const bf16_t* __restrict__ in, bf16_t* __restrict__ out, int64_t C,
                                               int64_t ld_out, int64_t r0, int64_t c0) {
  __shared__ bf16_t tile[64][66];
  const int t = threadIdx.x;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int idx = it * 256 + t;         // 512 vectors of 8
    const int r = idx >> 3, cv = (idx & 7) << 3;
    bf16x8 v = *reinterpret_cast<const bf16x8*>(in + (r0 + r) * C + c0 + cv);
#pragma unroll
    for (int e = 0; e < 8; ++e) tile[r][cv + e] = v[e];
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int idx = it * 256 + t;
    const int c = idx >> 3, rv = (idx & 7) << 3;
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = tile[rv + e][c];
    *reinterpret_cast<bf16x8*>(out + (c0 + c) * ld_out + r0 + rv) = v;
  }
}

__global__ __launch_bounds__(256) void transpose_kernel(const bf16_t* __restrict__ in,
                                                        bf16_t* __restrict__ out, int64_t R,
                                                        int64_t C, int64_t ld_out) {
  transpose_tile(in, out, C, ld_out, (int64_t)blockIdx.y * 64, (int64_t)blockIdx.x * 64);
}

// Several transposes in one launch (the seven weights of a layer: for small layers each launch costs
// more than its copy).  The argument block is only read with compile-time indices.
struct TransposeGroup {
  const bf16_t* in[kMaxTransposeGroup];
  bf16_t* out[kMaxTransposeGroup];
  int R[kMaxTransposeGroup], C[kMaxTransposeGroup];
  int64_t ld_out[kMaxTransposeGroup];
  int tile_start[kMaxTransposeGroup + 1];
  int n;
};
__global__ __launch_bounds__(256) void transpose_group_kernel(const TransposeGroup g) {
  const int id = blockIdx.x;
  const bf16_t* in = g.in[0];
  bf16_t* out = g.out[0];
  int C = g.C[0], start = 0;
  int64_t ld_out = g.ld_out[0];
#pragma unroll
  for (int i = 1; i < kMaxTransposeGroup; ++i)
    if (i < g.n && id >= g.tile_start[i]) { in = g.in[i]; out = g.out[i]; C = g.C[i]; ld_out = g.ld_out[i]; start = g.tile_start[i]; }
  const int tiles_x = C / 64, tl = id - start;
  transpose_tile(in, out, C, ld_out, (int64_t)(tl / tiles_x) * 64, (int64_t)(tl % tiles_x) * 64);
}

int launch_transpose_group(const TransposeJob* jobs, int n, hipStream_t st) {
  if (n < 1 || n > kMaxTransposeGroup) return fail(-1, "transpose group: 1..%d matrices, got %d", kMaxTransposeGroup, n);
  TransposeGroup g{};
  g.n = n;
  for (int i = 0; i < n; ++i) {
    g.in[i] = (const bf16_t*)jobs[i].in;
    g.out[i] = (bf16_t*)jobs[i].out;
    g.R[i] = (int)jobs[i].R;
    g.C[i] = (int)jobs[i].C;
    g.ld_out[i] = jobs[i].ld_out;
    g.tile_start[i + 1] = g.tile_start[i] + (int)((jobs[i].R / 64) * (jobs[i].C / 64));
  }
  hipLaunchKernelGGL(transpose_group_kernel, dim3((unsigned)g.tile_start[n]), dim3(256), 0, st, g);
  return check_launch("transpose group");
}

int launch_transpose(const void* in, void* out, int64_t R, int64_t C, int64_t ld_out, hipStream_t st) {
  hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)(C / 64), (unsigned)(R / 64)), dim3(256), 0,
                     st, (const bf16_t*)in, (bf16_t*)out, R, C, ld_out);
  return check_launch("transpose");
}

// ------------------------------------------------------------------------------------------
// Embedding gather and its gradient.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void embed_fwd_kernel(const bf16_t* __restrict__ table,
                                                        const int64_t* __restrict__ ids,
                                                        bf16_t* __restrict__ x0, int64_t V, int D) {
  const int64_t t = blockIdx.x;
  int64_t id = ids[t];
  const bool ok = id >= 0 && id < V;
  const bf16x8* src = reinterpret_cast<const bf16x8*>(table + (ok ? id : 0) * D);
  bf16x8* dst = reinterpret_cast<bf16x8*>(x0 + t * D);
  bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int c = threadIdx.x; c < (D >> 3); c += blockDim.x) dst[c] = ok ? src[c] : zero;
}

int launch_embed_fwd(const void* table, const int64_t* ids, int64_t T, int64_t V, int64_t D,
                     void* x0, hipStream_t st) {
  hipLaunchKernelGGL(embed_fwd_kernel, dim3((unsigned)T), dim3(256), 0, st, (const bf16_t*)table,
                     ids, (bf16_t*)x0, V, (int)D);
  return check_launch("embed_forward");
}

// ------------------------------------------------------------------------------------------
// Embedding gradient dtable[v] = sum of the rows dx0[t] with ids[t] == v, deterministic and without
// floating-point atomics.  The tokens of every id are gathered into a list (integer atomics: which slot
// a token gets depends on scheduling, the SET of tokens in a list does not), the list is sorted, and
// the rows are summed in ascending token order by a fixed assignment of rows to partial sums.  So the
// result is bitwise reproducible.  Ids with up to four tokens (one workgroup each) and ids with more (a
// sorting pass, then one workgroup per 128 columns) take different kernels; which one depends on the
// count alone.
//   count[v]   tokens with id v                       (embed_count_kernel)
//   start[v]   first slot of id v's segment of list   (embed_segments_kernel)
//   list[...]  token indices grouped by id, slot[t] = position of t in list    (embed_fill_kernel)
//   owner of an id = the token that drew the first slot of its group: its workgroups sum the rows
// ------------------------------------------------------------------------------------------
constexpr int kEmbSortMax = 8192;   // tokens of one id that are sorted in LDS (ids beyond that are walked)
constexpr int kEmbVecPerBlock = 16; // 16-byte column vectors per workgroup (128 columns) of the heavy kernel
constexpr int kEmbLight = 4;        // ids with at most this many tokens: one workgroup sums the whole row, no LDS

__global__ __launch_bounds__(256) void embed_zero_ints_kernel(int* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0;
}

__global__ __launch_bounds__(256) void embed_count_kernel(const int64_t* __restrict__ ids, int T, int64_t V, int* count) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const int64_t id = ids[t];
  if (id >= 0 && id < V) atomicAdd(&count[id], 1);
}

// start[v] = first slot of id v's segment of `list`.  The segments only have to be disjoint, not in id
// order, so they are handed out from a running cursor: one atomic per wavefront (the lanes' counts are
// prefix-summed with shuffles).  Where a segment lands depends on scheduling; what it holds does not.
__global__ __launch_bounds__(256) void embed_segments_kernel(const int* __restrict__ count, int* __restrict__ start, int V,
                                                             int* cursor) {
  const int v = blockIdx.x * 256 + threadIdx.x, lane = threadIdx.x & 63;
  const int c = v < V ? count[v] : 0;
  int incl = c;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int x = __shfl_up(incl, off, 64);
    if (lane >= off) incl += x;
  }
  const int total = __shfl(incl, 63, 64);
  int base = 0;
  if (lane == 63 && total > 0) base = atomicAdd(cursor, total);
  base = __shfl(base, 63, 64);
  if (v < V) start[v] = base + incl - c;
}

__global__ __launch_bounds__(256) void embed_fill_kernel(const int64_t* __restrict__ ids, int T, int64_t V,
                                                         const int* __restrict__ count, const int* __restrict__ start, int* fill,
                                                         int* __restrict__ list, int* __restrict__ slot, int* heavy,
                                                         int* n_heavy) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  const int64_t id = ids[t];
  if (id < 0 || id >= V) { slot[t] = -1; return; }
  const int first = start[id], s = first + atomicAdd(&fill[id], 1);
  list[s] = t;
  slot[t] = s;
  // ids with more than kEmbLight tokens are summed by the heavy kernel; the order of this list does not
  // matter (every entry is worked on independently)
  if (s == first && count[id] > kEmbLight) heavy[atomicAdd(n_heavy, 1)] = (int)id;
}

// rows of dtable no token points at
__global__ __launch_bounds__(256) void embed_zero_rows_kernel(const int* __restrict__ count, u32x4* __restrict__ dtable, int64_t V,
                                                              int row_vec) {
  const u32x4 z = {0, 0, 0, 0};
  for (int64_t v = blockIdx.x; v < V; v += gridDim.x) {
    if (count[v] != 0) continue;
    u32x4* row = dtable + v * row_vec;
    for (int c = threadIdx.x; c < row_vec; c += 256) row[c] = z;
  }
}

// Ids with at most kEmbLight tokens (nearly all of them unless the ids are very skewed).  One workgroup
// per token; the token that owns its id sorts the id's few tokens in registers and sums their rows with the
// same rule as the heavy kernel: row of rank r to partial sum r % 4, then (s0 + s1) + (s2 + s3).
__global__ __launch_bounds__(256) void embed_sum_light_kernel(const bf16_t* __restrict__ dx0, const int64_t* __restrict__ ids,
                                                              const int* __restrict__ count, const int* __restrict__ start,
                                                              const int* __restrict__ list, const int* __restrict__ slot,
                                                              bf16_t* __restrict__ dtable, int T, int64_t V, int D) {
  const int t = blockIdx.x;
  const int64_t id = ids[t];
  if (id < 0 || id >= V) return;
  const int first = start[id], L = count[id];
  if (slot[t] != first || L > kEmbLight) return;
  int r[kEmbLight];
#pragma unroll
  for (int i = 0; i < kEmbLight; ++i) r[i] = i < L ? list[first + i] : T;
#pragma unroll
  for (int i = 0; i < kEmbLight; ++i)       // sorting network for four keys (padding sorts last)
#pragma unroll
    for (int j = 0; j + 1 < kEmbLight - i; ++j)
      if (r[j] > r[j + 1]) { const int x = r[j]; r[j] = r[j + 1]; r[j + 1] = x; }
  static_assert(kEmbLight == 4, "one row per partial sum");
  for (int c = threadIdx.x; c < (D >> 3); c += 256) {
    float a[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (i < L) v = *reinterpret_cast<const bf16x8*>(dx0 + (int64_t)r[i] * D + c * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) a[i][e] = (float)v[e];
    }
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16_t)((a[0][e] + a[1][e]) + (a[2][e] + a[3][e]));
    *reinterpret_cast<bf16x8*>(dtable + id * D + c * 8) = o;
  }
}

// Sorts the token list of every id on the heavy list, in place: one workgroup per id at a time.  Lists
// of up to kEmbSortMax tokens go through a bitonic network in LDS; a longer one is rebuilt in order by
// walking all ids (a bitmap per piece of kEmbSortMax tokens, positions from prefix sums of its words).
__global__ __launch_bounds__(1024) void embed_sort_kernel(const int64_t* __restrict__ ids, const int* __restrict__ count,
                                                         const int* __restrict__ start, int* list,
                                                         const int* __restrict__ heavy, const int* __restrict__ n_heavy, int T) {
  __shared__ int lst[kEmbSortMax];
  __shared__ unsigned bits[kEmbSortMax / 32];
  __shared__ int wpre[kEmbSortMax / 32 + 1];
  const int nh = *n_heavy;
  for (int hi = blockIdx.x; hi < nh; hi += gridDim.x) {
    const int64_t id = heavy[hi];
    const int first = start[id], L = count[id];
    __syncthreads();   // the previous id's list has been written back
    if (L <= kEmbSortMax) {
      int n2 = 1;
      while (n2 < L) n2 <<= 1;
      for (int i = threadIdx.x; i < n2; i += 1024) lst[i] = i < L ? list[first + i] : T;
      __syncthreads();
      for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
          for (int i = threadIdx.x; i < n2; i += 1024) {
            const int p = i ^ j;
            if (p > i) {
              const int x = lst[i], y = lst[p];
              const bool up = (i & k) == 0;
              if ((x > y) == up) { lst[i] = y; lst[p] = x; }
            }
          }
          __syncthreads();
        }
      for (int i = threadIdx.x; i < L; i += 1024) list[first + i] = lst[i];
    } else {
      int rank = 0;
      for (int base = 0; base < T; base += kEmbSortMax) {
        __syncthreads();
        for (int w = threadIdx.x; w < kEmbSortMax / 32; w += 1024) bits[w] = 0u;
        __syncthreads();
        for (int k = threadIdx.x; k < kEmbSortMax; k += 1024)
          if (base + k < T && ids[base + k] == id) atomicOr(&bits[k >> 5], 1u << (k & 31));
        __syncthreads();
        if (threadIdx.x == 0) {
          int run = 0;
          for (int w = 0; w < kEmbSortMax / 32; ++w) { wpre[w] = run; run += __builtin_popcount(bits[w]); }
          wpre[kEmbSortMax / 32] = run;
        }
        __syncthreads();
        for (int w = threadIdx.x; w < kEmbSortMax / 32; w += 1024) {
          unsigned m = bits[w];
          int o = first + rank + wpre[w];
          while (m) { list[o++] = base + w * 32 + __builtin_ctz(m); m &= m - 1; }
        }
        rank += wpre[kEmbSortMax / 32];
      }
    }
  }
}

// Sums the rows of every id on the heavy list, whose token lists are sorted by now.  grid (workgroups,
// column splits of 128 columns); a workgroup is 16 column vectors x 16 row groups: the row of rank r goes
// to partial sum r % 16 (each summed in ascending token order), and the 16 partial sums are combined
// pairwise in a fixed order.
__global__ __launch_bounds__(256) void embed_sum_kernel(const bf16_t* __restrict__ dx0, const int* __restrict__ count,
                                                        const int* __restrict__ start, const int* __restrict__ list,
                                                        const int* __restrict__ heavy, const int* __restrict__ n_heavy,
                                                        bf16_t* __restrict__ dtable, int D) {
  __shared__ float part[16][kEmbVecPerBlock][8];
  const int vec = threadIdx.x & (kEmbVecPerBlock - 1), grp = threadIdx.x / kEmbVecPerBlock;
  const int cvec = blockIdx.y * kEmbVecPerBlock + vec;
  const bool col_ok = cvec < (D >> 3);
  const int nh = *n_heavy;
  for (int hi = blockIdx.x; hi < nh; hi += gridDim.x) {
    const int64_t id = heavy[hi];
    const int* lst = list + start[id];
    const int L = count[id];
    float a[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = 0.f;
    if (col_ok) {
      const bf16_t* col = dx0 + cvec * 8;
      int j = grp;
      for (; j + 112 < L; j += 128) {   // eight rows in flight
        bf16x8 r[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) r[q] = *reinterpret_cast<const bf16x8*>(col + (int64_t)lst[j + 16 * q] * D);
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
          for (int e = 0; e < 8; ++e) a[e] += (float)r[q][e];
      }
      for (; j < L; j += 16) {
        const bf16x8 r0 = *reinterpret_cast<const bf16x8*>(col + (int64_t)lst[j] * D);
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] += (float)r0[e];
      }
    }
    __syncthreads();   // the previous id's partial sums have been read
#pragma unroll
    for (int e = 0; e < 8; ++e) part[grp][vec][e] = a[e];
    __syncthreads();
    if (grp == 0 && col_ok) {
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float q[16];
#pragma unroll
        for (int g = 0; g < 16; ++g) q[g] = part[g][vec][e];
#pragma unroll
        for (int w = 1; w < 16; w <<= 1)
#pragma unroll
          for (int g = 0; g < 16; g += 2 * w) q[g] += q[g + w];
        o[e] = (bf16_t)q[0];
      }
      *reinterpret_cast<bf16x8*>(dtable + id * D + cvec * 8) = o;
    }
  }
}

// count[V], fill[V], the heavy-id counter and the segment cursor (padded to 4 ints), start[V], list[T], slot[T],
// heavy[T / 5 + 1]
size_t embed_bwd_workspace(int64_t T, int64_t V) { return (size_t)(3 * V + 4 + 2 * T + T / (kEmbLight + 1) + 1) * sizeof(int); }

int launch_embed_bwd(const void* dx0, const int64_t* ids, int64_t T, int64_t V, int64_t D,
                     void* dtable, void* workspace, hipStream_t st) {
  int* count = (int*)workspace;
  int* fill = count + V;
  int* n_heavy = fill + V;
  int* start = n_heavy + 4;
  int* list = start + V;
  int* slot = list + T;
  int* heavy = slot + T;
  const unsigned tb = (unsigned)((T + 255) / 256);
  const int64_t zn = 2 * V + 4, zb = (zn + 255) / 256;
  hipLaunchKernelGGL(embed_zero_ints_kernel, dim3((unsigned)(zb < 2048 ? zb : 2048)), dim3(256), 0, st, count, zn);
  if (int rc = check_launch("embed_backward(clear)")) return rc;
  hipLaunchKernelGGL(embed_count_kernel, dim3(tb), dim3(256), 0, st, ids, (int)T, V, count);
  if (int rc = check_launch("embed_backward(count)")) return rc;
  hipLaunchKernelGGL(embed_segments_kernel, dim3((unsigned)((V + 255) / 256)), dim3(256), 0, st, (const int*)count, start, (int)V,
                     n_heavy + 1);
  if (int rc = check_launch("embed_backward(segments)")) return rc;
  hipLaunchKernelGGL(embed_fill_kernel, dim3(tb), dim3(256), 0, st, ids, (int)T, V, (const int*)count, (const int*)start, fill,
                     list, slot, heavy, n_heavy);
  if (int rc = check_launch("embed_backward(fill)")) return rc;
  hipLaunchKernelGGL(embed_zero_rows_kernel, dim3((unsigned)(V < 16384 ? V : 16384)), dim3(256), 0, st, (const int*)count,
                     (u32x4*)dtable, V, (int)(D / 8));
  if (int rc = check_launch("embed_backward(zero)")) return rc;
  hipLaunchKernelGGL(embed_sum_light_kernel, dim3((unsigned)T), dim3(256), 0, st, (const bf16_t*)dx0, ids, (const int*)count,
                     (const int*)start, (const int*)list, (const int*)slot, (bf16_t*)dtable, (int)T, V, (int)D);
  if (int rc = check_launch("embed_backward(light)")) return rc;
  const unsigned cs = (unsigned)((D / 8 + kEmbVecPerBlock - 1) / kEmbVecPerBlock);
  const int64_t max_heavy = T / (kEmbLight + 1) + 1;
  hipLaunchKernelGGL(embed_sort_kernel, dim3((unsigned)(max_heavy < 1024 ? max_heavy : 1024)), dim3(1024), 0, st, ids,
                     (const int*)count, (const int*)start, list, (const int*)heavy, (const int*)n_heavy, (int)T);
  if (int rc = check_launch("embed_backward(sort)")) return rc;
  hipLaunchKernelGGL(embed_sum_kernel, dim3((unsigned)(max_heavy < 256 ? max_heavy : 256), cs), dim3(256), 0, st,
                     (const bf16_t*)dx0, (const int*)count, (const int*)start, (const int*)list, (const int*)heavy,
                     (const int*)n_heavy, (bf16_t*)dtable, (int)D);
  return check_launch("embed_backward");
}

}  // namespace dl
