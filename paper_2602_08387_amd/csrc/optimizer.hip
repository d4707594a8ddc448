// Optimizer step of the training loop: global-norm gradient clipping and AdamW over a list of tensors.
// bf16 parameters and gradients, fp32 moments.  Both kernels are bound by HBM: the norm reads 2 bytes
// per element, the update reads 12 and writes 10.  A launch covers up to kOptMaxTensors tensors; block
// b works on one 16384-element chunk of one tensor (the table is only read with compile-time indices: a
// run-time index into kernel arguments makes the compiler copy them to scratch memory).
#include "common.h"
#include "kernels.h"

namespace dl {

constexpr int kOptChunk = 16384;   // elements per workgroup: 256 threads x 8 vectors of 8

struct OptTable {
  bf16_t* p[kOptMaxTensors];
  const bf16_t* g[kOptMaxTensors];
  float* m[kOptMaxTensors];
  float* v[kOptMaxTensors];
  int64_t n[kOptMaxTensors];
  int blk_start[kOptMaxTensors + 1];
  int count;
};

struct OptSlot { bf16_t* p; const bf16_t* g; float *m, *v; int64_t n; int chunk; };
__device__ __forceinline__ OptSlot opt_locate(const OptTable& t, int blk) {
  OptSlot s{t.p[0], t.g[0], t.m[0], t.v[0], t.n[0], blk};
#pragma unroll
  for (int i = 1; i < kOptMaxTensors; ++i)
    if (i < t.count && blk >= t.blk_start[i]) s = OptSlot{t.p[i], t.g[i], t.m[i], t.v[i], t.n[i], blk - t.blk_start[i]};
  return s;
}

// Sum over a workgroup in a fixed order (wave shuffles, then the waves' sums one after the other): the
// result does not depend on scheduling.
__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// partial[b] = sum of squares of chunk b
__global__ __launch_bounds__(256) void grad_sq_partial_kernel(const OptTable t, float* __restrict__ partial) {
  __shared__ float red[4];
  const OptSlot s = opt_locate(t, blockIdx.x);
  const int64_t base = (int64_t)s.chunk * kOptChunk;
  float a0 = 0.f, a1 = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int64_t e = base + ((int64_t)i * 256 + threadIdx.x) * 8;
    if (e < s.n) {
      const bf16x8 g = *reinterpret_cast<const bf16x8*>(s.g + e);
#pragma unroll
      for (int k = 0; k < 8; k += 2) {
        const float x = (float)g[k], y = (float)g[k + 1];
        a0 += x * x;
        a1 += y * y;
      }
    }
  }
  const float r = block_sum_256(a0 + a1, red);
  if (threadIdx.x == 0) partial[blockIdx.x] = r;
}

// out = sum of the partials, one workgroup, fixed order
__global__ __launch_bounds__(256) void grad_sq_final_kernel(const float* __restrict__ partial, int n, float* out,
                                                            int accumulate) {
  __shared__ float red[4];
  float a = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) a += partial[i];
  const float r = block_sum_256(a, red);
  if (threadIdx.x == 0) *out = accumulate ? *out + r : r;
}

struct AdamwScalars {
  float decay;          // 1 - lr * weight_decay
  float beta1, beta2, one_minus_beta1, one_minus_beta2;
  float step_size;      // lr / (1 - beta1^t)
  float inv_sqrt_bc2;   // 1 / sqrt(1 - beta2^t)
  float eps, max_norm;
};

__global__ __launch_bounds__(256) void adamw_kernel(const OptTable t, const AdamwScalars h, const float* __restrict__ sq_norm) {
  const OptSlot s = opt_locate(t, blockIdx.x);
  float coef = 1.0f;
  if (sq_norm) coef = fminf(1.0f, h.max_norm / (sqrtf(*sq_norm) + 1e-6f));
  const int64_t base = (int64_t)s.chunk * kOptChunk;
#pragma unroll 2
  for (int i = 0; i < 8; ++i) {
    const int64_t e = base + ((int64_t)i * 256 + threadIdx.x) * 8;
    if (e < s.n) {
      const bf16x8 p = *reinterpret_cast<const bf16x8*>(s.p + e), g = *reinterpret_cast<const bf16x8*>(s.g + e);
      f32x4 m[2] = {*reinterpret_cast<const f32x4*>(s.m + e), *reinterpret_cast<const f32x4*>(s.m + e + 4)};
      f32x4 v[2] = {*reinterpret_cast<const f32x4*>(s.v + e), *reinterpret_cast<const f32x4*>(s.v + e + 4)};
      bf16x8 po;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float gk = (float)g[k] * coef;
        const float mk = h.beta1 * m[k >> 2][k & 3] + h.one_minus_beta1 * gk;
        const float vk = h.beta2 * v[k >> 2][k & 3] + h.one_minus_beta2 * gk * gk;
        m[k >> 2][k & 3] = mk;
        v[k >> 2][k & 3] = vk;
        po[k] = (bf16_t)((float)p[k] * h.decay - h.step_size * mk / (sqrtf(vk) * h.inv_sqrt_bc2 + h.eps));
      }
      *reinterpret_cast<bf16x8*>(s.p + e) = po;
      *reinterpret_cast<f32x4*>(s.m + e) = m[0];
      *reinterpret_cast<f32x4*>(s.m + e + 4) = m[1];
      *reinterpret_cast<f32x4*>(s.v + e) = v[0];
      *reinterpret_cast<f32x4*>(s.v + e + 4) = v[1];
    }
  }
}

static int fill_table(OptTable& t, int n, void* const* p, const void* const* g, float* const* m, float* const* v,
                      const int64_t* numel) {
  t.count = n;
  t.blk_start[0] = 0;
  for (int i = 0; i < n; ++i) {
    t.p[i] = p ? (bf16_t*)p[i] : nullptr;
    t.g[i] = (const bf16_t*)g[i];
    t.m[i] = m ? m[i] : nullptr;
    t.v[i] = v ? v[i] : nullptr;
    t.n[i] = numel[i];
    t.blk_start[i + 1] = t.blk_start[i] + (int)((numel[i] + kOptChunk - 1) / kOptChunk);
  }
  return t.blk_start[n];
}

int64_t opt_chunks(int n, const int64_t* numel) {
  int64_t c = 0;
  for (int i = 0; i < n; ++i) c += (numel[i] + kOptChunk - 1) / kOptChunk;
  return c;
}

int launch_grad_sq_norm(int n, const void* const* g, const int64_t* numel, float* sq_norm, float* partial, int accumulate,
                        hipStream_t st) {
  OptTable t{};
  const int blocks = fill_table(t, n, nullptr, g, nullptr, nullptr, numel);
  hipLaunchKernelGGL(grad_sq_partial_kernel, dim3((unsigned)blocks), dim3(256), 0, st, t, partial);
  if (int rc = check_launch("grad_sq_norm(partials)")) return rc;
  hipLaunchKernelGGL(grad_sq_final_kernel, dim3(1), dim3(256), 0, st, (const float*)partial, blocks, sq_norm, accumulate);
  return check_launch("grad_sq_norm");
}

int launch_adamw(int n, void* const* p, const void* const* g, float* const* m, float* const* v, const int64_t* numel,
                 int64_t step, float lr, float beta1, float beta2, float eps, float weight_decay, float max_norm,
                 const float* sq_norm, hipStream_t st) {
  OptTable t{};
  const int blocks = fill_table(t, n, p, g, m, v, numel);
  AdamwScalars h;
  const double bc1 = 1.0 - pow((double)beta1, (double)step), bc2 = 1.0 - pow((double)beta2, (double)step);
  h.decay = (float)(1.0 - (double)lr * (double)weight_decay);
  h.beta1 = beta1; h.beta2 = beta2;
  h.one_minus_beta1 = (float)(1.0 - (double)beta1); h.one_minus_beta2 = (float)(1.0 - (double)beta2);
  h.step_size = (float)((double)lr / bc1);
  h.inv_sqrt_bc2 = (float)(1.0 / sqrt(bc2));
  h.eps = eps; h.max_norm = max_norm;
  hipLaunchKernelGGL(adamw_kernel, dim3((unsigned)blocks), dim3(256), 0, st, t, h, sq_norm);
  return check_launch("adamw_step");
}

}  // namespace dl
