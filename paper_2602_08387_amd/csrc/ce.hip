// Fused softmax cross-entropy forward + backward over rows of bf16 logits.
// One 1024-thread workgroup per row.  Short rows (V <= 65536) are read from HBM once and kept in
// registers (up to 16 x 8 bf16 per thread) between the max/sum reductions and the gradient write.
// Long rows take two passes with 30 registers per thread: maximum and sum together in one pass
// (each thread keeps its sum relative to its own running maximum), then a second read for the
// gradient.  At V = 128256 that is 5 % faster than the register-cached form (0.94 against 0.99 ms for
// 8192 rows): two workgroups fit a CU and overlap their phases, and the second read of a row is
// served by the L2 and the memory-side cache, so HBM still sees 2 bytes in + 2 bytes out per logit.
#include "common.h"
#include "kernels.h"
#include <atomic>

namespace dl {

// Per-row losses of the allocation-free entry point: one float per row, at most kCeStaticMaxRows rows
// (256 KiB, held by every GPU the library runs on until the process ends).  In host code this name
// is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
constexpr int64_t kCeStaticMaxRows = 65536;
static __device__ __align__(256) float scratch[kCeStaticMaxRows];

constexpr int kCeThreads = 1024;
constexpr float kCeLog2e = 1.4426950408889634f;
// exp(x - m) as one FMA and one v_exp_f32: 2^(x * log2(e) - m * log2(e)); results below 2^-126 flush to
// zero, which is what a softmax weight that small should be anyway.  The kernel is bound by its vector
// arithmetic (two exponentials and three conversions per logit), so instructions per element count.
__device__ __forceinline__ float exp_shifted(float x, float m_log2e) {
  return __builtin_amdgcn_exp2f(__builtin_fmaf(x, kCeLog2e, -m_log2e));
}

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = is_max ? wave_max(v) : wave_sum(v);
  __syncthreads();  // protect red[] from the previous use
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < kCeThreads / 64; ++w) r = is_max ? fmaxf(r, red[w]) : r + red[w];
  return r;
}

template <bool CACHED>
__global__ __launch_bounds__(kCeThreads) void ce_kernel(const bf16_t* logits,
                                                        const int64_t* __restrict__ targets,
                                                        int64_t V, float scale,
                                                        float* __restrict__ row_loss,
                                                        bf16_t* dlogits) {
  __shared__ float red[kCeThreads / 64];
  __shared__ float picked_s;
  constexpr int NV = 16;
  const int64_t row = blockIdx.x;
  const int nvec = (int)(V >> 3);
  const bf16x8* in = reinterpret_cast<const bf16x8*>(logits + row * V);
  bf16x8* out = reinterpret_cast<bf16x8*>(dlogits + row * V);
  const int64_t tgt = targets[row];
  const bool tgt_ok = tgt >= 0 && tgt < V;
  if (threadIdx.x == 0) picked_s = tgt_ok ? (float)logits[row * V + tgt] : 0.f;

  bf16x8 v[CACHED ? NV : 1];
  float mx = -INFINITY, lsum = 0.f;
  if constexpr (CACHED) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = i * kCeThreads + threadIdx.x;
      if (c < nvec) {
        v[i] = in[c];
#pragma unroll
        for (int e = 0; e < 8; ++e) mx = fmaxf(mx, (float)v[i][e]);
      }
    }
  } else {
    // one pass for maximum and sum: the sum is kept relative to the running maximum of this thread
    // and rescaled when that rises
#pragma unroll 4
    for (int c = threadIdx.x; c < nvec; c += kCeThreads) {
      const bf16x8 t = in[c];
      float vm = (float)t[0];
#pragma unroll
      for (int e = 1; e < 8; ++e) vm = fmaxf(vm, (float)t[e]);
      if (vm > mx) {
        lsum *= exp_shifted(mx, vm * kCeLog2e);   // exp(mx - vm); 0 while mx is still -inf
        mx = vm;
      }
      const float m2 = mx * kCeLog2e;
#pragma unroll
      for (int e = 0; e < 8; ++e) lsum += exp_shifted((float)t[e], m2);
    }
  }
  const float mx_own = mx;
  mx = block_reduce(mx, true, red);
  const float mx2 = mx * kCeLog2e;
  float sum = 0.f;
  if constexpr (CACHED) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = i * kCeThreads + threadIdx.x;
      if (c < nvec) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sum += exp_shifted((float)v[i][e], mx2);
      }
    }
  } else {
    sum = lsum > 0.f ? lsum * exp_shifted(mx_own, mx2) : 0.f;
  }
  sum = block_reduce(sum, false, red);  // its barriers also order every read before any write
  const float lse = mx + __logf(sum);
  if (threadIdx.x == 0) row_loss[row] = tgt_ok ? lse - picked_s : lse;
  const int tc = tgt_ok ? (int)(tgt >> 3) : -1, te = (int)(tgt & 7);
  const float lse2 = lse * kCeLog2e;
  // gradient of one 8-vector, without the -1 of the target: the thread that owns the target's vector
  // stores that one element again after its vector (same thread, same address: in order), from the
  // logit saved at the start - a store under a rarely taken branch instead of a select per element
  auto grad_vec = [&](const bf16x8& x) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16_t)(exp_shifted((float)x[e], lse2) * scale);
    return o;
  };
  auto fix_target = [&](int c) {
    if (c == tc) dlogits[row * V + tgt] = (bf16_t)((exp_shifted(picked_s, lse2) - 1.0f) * scale);
  };
  if constexpr (CACHED) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = i * kCeThreads + threadIdx.x;
      if (c < nvec) {
        out[c] = grad_vec(v[i]);
        fix_target(c);
      }
    }
  } else {
    for (int c = threadIdx.x; c < nvec; c += kCeThreads) {
      out[c] = grad_vec(in[c]);
      fix_target(c);
    }
  }
}

// Mean of the per-row losses, summed in a fixed order by one workgroup.
__global__ __launch_bounds__(1024) void mean_kernel(const float* __restrict__ v, int64_t n,
                                                    float* out) {
  __shared__ float red[16];
  float s = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += 1024) s += v[i];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int w = 0; w < 16; ++w) t += red[w];
    *out = t / (float)n;
  }
}

size_t ce_workspace(int64_t T, int64_t) { return (size_t)T * sizeof(float); }

// rows [0, rows) of a larger problem: per-row losses into row_loss, gradient scaled by `scale`
int launch_ce_rows(const void* logits, const int64_t* targets, int64_t rows, int64_t V, float scale, float* row_loss,
                   void* dlogits, hipStream_t st) {
  if (V <= 65536)
    hipLaunchKernelGGL(ce_kernel<true>, dim3((unsigned)rows), dim3(kCeThreads), 0, st,
                       (const bf16_t*)logits, targets, V, scale, row_loss, (bf16_t*)dlogits);
  else
    hipLaunchKernelGGL(ce_kernel<false>, dim3((unsigned)rows), dim3(kCeThreads), 0, st,
                       (const bf16_t*)logits, targets, V, scale, row_loss, (bf16_t*)dlogits);
  return check_launch("ce_loss_fwd_bwd");
}

int launch_ce_mean(const float* row_loss, int64_t T, float* loss, hipStream_t st) {
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(1024), 0, st, row_loss, T, loss);
  return check_launch("ce_loss_fwd_bwd(mean)");
}

int launch_ce(const void* logits, const int64_t* targets, int64_t T, int64_t V, float grad_scale,
              float* loss, void* dlogits, void* workspace, hipStream_t st) {
  float* row_loss = (float*)workspace;
  int rc = launch_ce_rows(logits, targets, T, V, grad_scale / (float)T, row_loss, dlogits, st);
  if (rc) return rc;
  return launch_ce_mean(row_loss, T, loss, st);
}

// Device address of `scratch` on the current device, looked up once per device (each GPU holds its
// own copy of the array at its own address).
static int ce_static_rows(float** out) {
  static std::atomic<float*> ptrs[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(-3, "ce_loss_fwd_bwd_static: no current device");
  float* p = ptrs[dev].load(std::memory_order_acquire);
  if (!p) {
    hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(-3, "ce_loss_fwd_bwd_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    ptrs[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return 0;
}

int64_t ce_static_max_rows() { return kCeStaticMaxRows; }

// launch_ce with the per-row losses in the library's own static device array: every row < T is
// written by the row kernel before the mean kernel reads it, so nothing needs clearing between calls.
int launch_ce_static(const void* logits, const int64_t* targets, int64_t T, int64_t V, float grad_scale,
                     float* loss, void* dlogits, hipStream_t st) {
  float* row_loss = nullptr;
  if (int rc = ce_static_rows(&row_loss)) return rc;
  return launch_ce(logits, targets, T, V, grad_scale, loss, dlogits, row_loss, st);
}

}  // namespace dl
