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
      o[e] = (bf16_t)(z / (1.0f + __expf(-z)) * (float)uv[e]);
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
      const float s = 1.0f / (1.0f + __expf(-z));
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
    o[e] = (bf16_t)(z / (1.0f + __expf(-z)) * (float)uv[e]);
  }
  return o;
}
__device__ __forceinline__ void swiglu_grad_vec(bf16x8 gv, bf16x8 uv, bf16x8 dv, bf16x8& og, bf16x8& ou) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float z = (float)gv[e], d = (float)dv[e];
    const float sg = 1.0f / (1.0f + __expf(-z));
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

__global__ __launch_bounds__(256) void zero_kernel(u32x4* p, int64_t nvec) {
  const u32x4 z = {0, 0, 0, 0};
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec;
       i += (int64_t)gridDim.x * blockDim.x)
    p[i] = z;
}

// One block per token t.  The block owns row ids[t] iff no earlier token has the same id; it then
// sums (fp32, ascending token order: the result does not depend on scheduling) the gradient rows of
// every token with that id.  The tokens are scanned in segments of kEmbSeg: all threads mark the
// matches of a segment in an LDS bitmap (atomic OR, so the bitmap is the same however the threads are
// scheduled), then every thread walks the set bits in order for its columns.
constexpr int kEmbSeg = 8192;
__global__ __launch_bounds__(256) void embed_bwd_kernel(const bf16_t* __restrict__ dx0,
                                                        const int64_t* __restrict__ ids,
                                                        bf16_t* __restrict__ dtable, int64_t T,
                                                        int64_t V, int D) {
  __shared__ int earlier;
  __shared__ unsigned bits[kEmbSeg / 32];
  const int64_t t = blockIdx.x;
  const int64_t id = ids[t];
  if (id < 0 || id >= V) return;  // uniform over the block
  if (threadIdx.x == 0) earlier = 0;
  __syncthreads();
  for (int64_t s = threadIdx.x; s < t; s += blockDim.x)
    if (ids[s] == id) earlier = 1;
  __syncthreads();
  if (earlier) return;            // uniform over the block
  const int nv = D >> 3;
  constexpr int NC = 2;           // column vectors per thread and pass: D up to 4096 in one pass
  bf16x8* out = reinterpret_cast<bf16x8*>(dtable + id * D);
  for (int c0 = 0; c0 < nv; c0 += NC * 256) {
    float a[NC][8];
#pragma unroll
    for (int q = 0; q < NC; ++q)
#pragma unroll
      for (int e = 0; e < 8; ++e) a[q][e] = 0.f;
    for (int64_t base = t - t % kEmbSeg; base < T; base += kEmbSeg) {
      __syncthreads();
      for (int w = threadIdx.x; w < kEmbSeg / 32; w += 256) bits[w] = 0u;
      __syncthreads();
      for (int k = threadIdx.x; k < kEmbSeg; k += 256) {
        const int64_t s = base + k;
        if (s >= t && s < T && ids[s] == id) atomicOr(&bits[k >> 5], 1u << (k & 31));
      }
      __syncthreads();
      // one row ahead: the loads of the next matching row go out before the current one is summed
      // (a frequent token has thousands of rows, all summed by this one workgroup)
      bf16x8 cur[NC], nxt[NC];
      bool have = false;
      auto add_cur = [&]() {
#pragma unroll
        for (int q = 0; q < NC; ++q) {
          const int c = c0 + q * 256 + threadIdx.x;
          if (c < nv) {
#pragma unroll
            for (int e = 0; e < 8; ++e) a[q][e] += (float)cur[q][e];
          }
        }
      };
      for (int w = 0; w < kEmbSeg / 32; ++w) {
        unsigned m = bits[w];
        while (m) {
          const int k = w * 32 + __builtin_ctz(m);
          m &= m - 1;
          const bf16x8* row = reinterpret_cast<const bf16x8*>(dx0 + (base + k) * D);
#pragma unroll
          for (int q = 0; q < NC; ++q) {
            const int c = c0 + q * 256 + threadIdx.x;
            if (c < nv) nxt[q] = row[c];
          }
          if (have) add_cur();
#pragma unroll
          for (int q = 0; q < NC; ++q) cur[q] = nxt[q];
          have = true;
        }
      }
      if (have) add_cur();
    }
#pragma unroll
    for (int q = 0; q < NC; ++q) {
      const int c = c0 + q * 256 + threadIdx.x;
      if (c < nv) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (bf16_t)a[q][e];
        out[c] = o;
      }
    }
  }
}

int launch_embed_bwd(const void* dx0, const int64_t* ids, int64_t T, int64_t V, int64_t D,
                     void* dtable, hipStream_t st) {
  const int64_t nvec = V * D / 8;
  hipLaunchKernelGGL(zero_kernel, dim3(ew_blocks(nvec)), dim3(256), 0, st, (u32x4*)dtable, nvec);
  int rc = check_launch("embed_backward(zero)");
  if (rc) return rc;
  hipLaunchKernelGGL(embed_bwd_kernel, dim3((unsigned)T), dim3(256), 0, st, (const bf16_t*)dx0, ids,
                     (bf16_t*)dtable, T, V, (int)D);
  return check_launch("embed_backward");
}

}  // namespace dl
