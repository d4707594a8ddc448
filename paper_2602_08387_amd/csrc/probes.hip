// Issue-rate probes for gfx950: small synthetic kernels that answer "how fast can the matrix pipe run
// next to this much other work", used to put numbers behind the design notes of the GEMM and attention
// kernels.  They compute nothing useful; every loop has a fixed trip count and every LDS access stays
// inside the workgroup's 64 KB allocation (offsets are masked).  Timing: s_memtime inside the kernel
// (shader clock cycles per wave) and HIP events around the launch, which together also give the shader
// clock the chip settled at.
//
//   family 0, "arrangement" (32x32x16 MFMAs, one block = 16 MFMAs, 16 exponentials, 64 plain VALU ops):
//     variant 0  the MFMAs alone
//     variant 1  the VALU work alone
//     variant 2  uniform: every MFMA followed by 1 v_exp_f32 and 4 v_fma_f32
//     variant 3  two regions: 8 x (MFMA, 1 fma) then 8 x (MFMA, 2 exp, 7 fma) - the shape of a softmax
//                that is software-pipelined by key blocks
//   family 1, "operand feed" (16x16x32 MFMAs, one block = 8 MFMAs whose A operand comes from LDS):
//     variant 0  no LDS reads
//     variant 1  2 ds_read_b128 per block   (a 128x128 wave tile)
//     variant 2  3 ds_read_b128 per block   (a 128x64 wave tile)
//     variant 3  3 pairs of ds_read_b64_tr_b16 per block (128x64 wave tile, transposed operands)
//   family 2, "neighbour" (waves 0-3 of the workgroup run MFMAs only, waves 4-7, their SIMD partners, run
//     v_fma_f32 only): variant 0 MFMA waves alone, 1 VALU waves alone, 2 together.  result[0] is then the
//     cycles per MFMA of the MFMA waves and result[3] the cycles per fma of the VALU waves.
//   family 3, "sustained": the operand-feed kernels of family 1 (variants 0, 1, 2) with pseudo-random operands
//     in (-1, 1) instead of constants, launched back to back for about a second, so that the figure is
//     the rate the matrix pipes hold at the clock the power management settles on under a long load with
//     operands that toggle like real data.  result[1] is then the mean over all launches.  Variant 3: the
//     32x32x16 MFMAs of family 0, variant 0, the same way (one block = 16 MFMAs).
#include "common.h"
#include "kernels.h"
#include <type_traits>

namespace dl {
namespace {

__device__ __forceinline__ void probe_valu(float (&x)[8], float (&y)[8], int j, int ne, int nf) {
#pragma unroll
  for (int v = 0; v < ne; ++v) asm volatile("v_exp_f32 %0, %1" : "=v"(y[(2 * j + v) & 7]) : "v"(x[(2 * j + v) & 7]));
#pragma unroll
  for (int v = 0; v < nf; ++v) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x[(j * nf + v) & 7]) : "v"(y[(j * nf + v + 3) & 7]));
}

// pseudo-random bf16 in (-1, 1) from an integer (a multiplicative hash; no statistical claims)
__device__ __forceinline__ bf16_t probe_noise(unsigned i) {
  i = (i + 0x9e3779b9u) * 0x85ebca6bu;
  i ^= i >> 15;
  i *= 0xc2b2ae35u;
  i ^= i >> 13;
  return (bf16_t)((float)(int)(i >> 8) * (1.0f / 8388608.0f) - 1.0f);
}

template <int NW, int VARIANT, bool NOISE = false>
__global__ __launch_bounds__(NW * 64) void probe_arrangement_kernel(float* out, long long* cyc, int iters) {
  const int lane = threadIdx.x & 63;
  f32x16 acc[4];
  for (int i = 0; i < 4; ++i)
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (bf16_t)1.0f; b[e] = (bf16_t)(float)(lane & 1); }
  if (NOISE)
    for (int e = 0; e < 8; ++e) { a[e] = probe_noise(threadIdx.x * 16 + e); b[e] = probe_noise(threadIdx.x * 16 + 8 + e); }
  float x[8], y[8];
  for (int i = 0; i < 8; ++i) { x[i] = (float)(lane + i) * 1e-3f; y[i] = -(float)i; }
  __syncthreads();
  const long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (VARIANT != 1) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[j & 3]) : "v"(a), "v"(b));
      if (VARIANT == 1 || VARIANT == 2) probe_valu(x, y, j, 1, 4);
      if (VARIANT == 3) { if (j < 8) probe_valu(x, y, j, 0, 1); else probe_valu(x, y, j, 2, 7); }
    }
  }
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");   // results of the last MFMAs are read below
  const long long t1 = __builtin_readcyclecounter();
  float sum = 0;
  for (int i = 0; i < 8; ++i) sum += x[i] + y[i];
  for (int i = 0; i < 4; ++i)
    for (int e = 0; e < 16; ++e) sum += acc[i][e];
  out[blockIdx.x * NW * 64 + threadIdx.x] = sum;
  if (lane == 0) cyc[blockIdx.x * NW + (threadIdx.x >> 6)] = t1 - t0;
}

// R fragment reads per block of 8 MFMAs, fetched one block ahead (two register sets); TR: pairs of transposing reads
template <int NW, int R, bool TR, bool NOISE = false>
__global__ __launch_bounds__(NW * 64) void probe_feed_kernel(float* out, long long* cyc, int iters) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  if (NOISE)
    for (int i = threadIdx.x; i < 65536 / 2; i += NW * 64) ((bf16_t*)lds)[i] = probe_noise(blockIdx.x * 32768u + i);
  else
    for (int i = threadIdx.x; i < 65536 / 4; i += NW * 64) ((float*)lds)[i] = 0.0f;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  f32x4 acc[8];
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 4; ++e) acc[i][e] = 0.f;
  bf16x8 b[2];
  for (int e = 0; e < 8; ++e) { b[0][e] = (bf16_t)1.0f; b[1][e] = (bf16_t)0.5f; }
  bf16x8 f[2][4];
  for (int s = 0; s < 2; ++s)
    for (int j = 0; j < 4; ++j)
      for (int e = 0; e < 8; ++e) f[s][j][e] = (bf16_t)0.0f;
  if (NOISE) {
    for (int e = 0; e < 8; ++e) { b[0][e] = probe_noise(threadIdx.x * 16 + e); b[1][e] = probe_noise(threadIdx.x * 16 + 8 + e); }
    for (int s = 0; s < 2; ++s)
      for (int j = 0; j < 4; ++j)
        for (int e = 0; e < 8; ++e) f[s][j][e] = probe_noise(0x10000u + threadIdx.x * 64 + s * 32 + j * 8 + e);
  }
  const unsigned base = (unsigned)(uintptr_t)(LDS_PTR(char))lds + (wave & 7) * 8192 + lane * 16;   // 8 KB window per wave
  const long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (R > 0 && (j == 0 || (j * R) / 8 != ((j - 1) * R) / 8)) {
          const int fi = (j * R) / 8;
          const unsigned addr = base + ((fi * 1024 + it * 64) & 6144);
          if (!TR) asm volatile("ds_read_b128 %0, %1" : "=v"(f[s ^ 1][fi]) : "v"(addr));
          else {
            bf16x4 lo, hi;
            asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(addr));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:512" : "=v"(hi) : "v"(addr));
            f[s ^ 1][fi].lo = lo;
            f[s ^ 1][fi].hi = hi;
          }
        }
        const int fi = R ? (j * R) / 8 : 0;
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(f[s][fi]), "v"(b[j & 1]));
      }
      if (R > 0) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[s ^ 1][0]), "+v"(f[s ^ 1][1]), "+v"(f[s ^ 1][2]), "+v"(f[s ^ 1][3]));
    }
  }
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
  const long long t1 = __builtin_readcyclecounter();
  float sum = 0;
  for (int i = 0; i < 8; ++i)
    for (int e = 0; e < 4; ++e) sum += acc[i][e];
  out[blockIdx.x * NW * 64 + threadIdx.x] = sum;
  if (lane == 0) cyc[blockIdx.x * NW + (threadIdx.x >> 6)] = t1 - t0;
}

// MODE bit 0: the MFMA waves work, bit 1: the VALU waves work
template <int MODE>
__global__ __launch_bounds__(512) void probe_neighbour_kernel(float* out, long long* cyc, int iters) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float sum = 0.f;
  long long t0 = 0, t1 = 0;
  __syncthreads();
  if (wave < 4) {
    if (MODE & 1) {
      f32x16 acc[4];
      for (int i = 0; i < 4; ++i)
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
      bf16x8 a, b;
      for (int e = 0; e < 8; ++e) { a[e] = (bf16_t)1.0f; b[e] = (bf16_t)(float)(lane & 1); }
      t0 = __builtin_readcyclecounter();
      for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[j & 3]) : "v"(a), "v"(b));
      }
      asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
      t1 = __builtin_readcyclecounter();
      for (int i = 0; i < 4; ++i)
        for (int e = 0; e < 16; ++e) sum += acc[i][e];
    }
  } else if (MODE & 2) {
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = (float)(lane + i) * 1e-3f;
    t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int j = 0; j < 64; ++j) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x[j & 7]) : "v"(x[(j + 3) & 7]));
    }
    t1 = __builtin_readcyclecounter();
    for (int i = 0; i < 8; ++i) sum += x[i];
  }
  out[blockIdx.x * 512 + threadIdx.x] = sum;
  if (lane == 0) cyc[blockIdx.x * 8 + wave] = t1 - t0;
}

constexpr int kProbeBlocks = 256, kProbeIters = 2000;

// launches `kern` (NW waves per workgroup, one workgroup per CU; `units_per_iter` blocks per loop iteration and wave)
// and fills result: cycles per block per SIMD,
// milliseconds of the launch, shader clock in GHz (and, for the neighbour probe, the second role's figure)
template <typename K>
int run_probe(K kern, int nw, size_t lds, bool roles, double units_per_iter, double* result, hipStream_t st, int launches = 1) {
  float* out = nullptr;
  long long* cyc = nullptr;
  if (hipMalloc(&out, (size_t)kProbeBlocks * nw * 64 * sizeof(float)) != hipSuccess) return fail(-3, "probe: out of device memory");
  if (hipMalloc(&cyc, (size_t)kProbeBlocks * nw * sizeof(long long)) != hipSuccess) {
    (void)hipFree(out);
    return fail(-3, "probe: out of device memory");
  }
  hipEvent_t e0 = nullptr, e1 = nullptr, e2 = nullptr;
  int rc = 0;
  float ms = 0.f, ms_all = 0.f;
  static long long host[kProbeBlocks * 8];
  if (lds && hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
    rc = fail(-3, "probe: cannot reserve LDS");
  if (!rc && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess || hipEventCreate(&e2) != hipSuccess))
    rc = fail(-3, "probe: no events");
  if (!rc) {
    hipLaunchKernelGGL(kern, dim3(kProbeBlocks), dim3(nw * 64), lds, st, out, cyc, 10);   // warm-up
    (void)hipEventRecord(e2, st);
    for (int l = 1; l < launches; ++l) hipLaunchKernelGGL(kern, dim3(kProbeBlocks), dim3(nw * 64), lds, st, out, cyc, kProbeIters);
    (void)hipEventRecord(e0, st);
    hipLaunchKernelGGL(kern, dim3(kProbeBlocks), dim3(nw * 64), lds, st, out, cyc, kProbeIters);   // the launch the cycle counts are of
    (void)hipEventRecord(e1, st);
    rc = check_launch("probe");
    if (!rc && hipEventSynchronize(e1) != hipSuccess) rc = fail(-3, "probe: synchronisation failed");
    if (!rc && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = fail(-3, "probe: no elapsed time");
    if (!rc && hipEventElapsedTime(&ms_all, e2, e1) != hipSuccess) rc = fail(-3, "probe: no elapsed time");
    if (!rc && hipMemcpy(host, cyc, (size_t)kProbeBlocks * nw * sizeof(long long), hipMemcpyDeviceToHost) != hipSuccess)
      rc = fail(-3, "probe: copy failed");
  }
  if (!rc) {
    // A SIMD's waves share its pipes unevenly (the older wave is served first and finishes early), so the
    // time a SIMD took for the work of all its waves is that of its slowest wave: per workgroup the longest
    // wave of each role, averaged over the workgroups.
    double first = 0, second = 0, longest = 0;
    for (int bl = 0; bl < kProbeBlocks; ++bl) {
      double m1 = 0, m2 = 0;
      for (int w = 0; w < nw; ++w) {
        const double c = (double)host[bl * nw + w];
        if (roles && w >= 4) { if (c > m2) m2 = c; } else if (c > m1) m1 = c;
        if (c > longest) longest = c;
      }
      first += m1;
      second += m2;
    }
    first /= kProbeBlocks;
    second /= kProbeBlocks;
    const double waves_per_simd = roles ? 1.0 : nw / 4.0;
    result[0] = first / (kProbeIters * units_per_iter) / waves_per_simd;
    result[1] = launches > 1 ? ms_all / launches : ms;
    result[2] = longest / (ms * 1e6);
    result[3] = roles ? second / (kProbeIters * 64.0) : 0.0;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (e2) (void)hipEventDestroy(e2);
  (void)hipFree(out);
  (void)hipFree(cyc);
  return rc;
}

template <int NW>
int arrangement(int variant, double* result, hipStream_t st) {
  switch (variant) {
    case 0: return run_probe(probe_arrangement_kernel<NW, 0>, NW, 0, false, 1.0, result, st);
    case 1: return run_probe(probe_arrangement_kernel<NW, 1>, NW, 0, false, 1.0, result, st);
    case 2: return run_probe(probe_arrangement_kernel<NW, 2>, NW, 0, false, 1.0, result, st);
    case 3: return run_probe(probe_arrangement_kernel<NW, 3>, NW, 0, false, 1.0, result, st);
  }
  return fail(-1, "probe: arrangement variant %d", variant);
}
template <int NW>
int feed(int variant, double* result, hipStream_t st) {
  switch (variant) {
    case 0: return run_probe(probe_feed_kernel<NW, 0, false>, NW, 65536, false, 2.0, result, st);
    case 1: return run_probe(probe_feed_kernel<NW, 2, false>, NW, 65536, false, 2.0, result, st);
    case 2: return run_probe(probe_feed_kernel<NW, 3, false>, NW, 65536, false, 2.0, result, st);
    case 3: return run_probe(probe_feed_kernel<NW, 3, true>, NW, 65536, false, 2.0, result, st);
  }
  return fail(-1, "probe: feed variant %d", variant);
}
constexpr int kSustainedLaunches = 2500;   // about a second of back-to-back launches
template <int NW>
int sustained(int variant, double* result, hipStream_t st) {
  switch (variant) {
    case 0: return run_probe(probe_feed_kernel<NW, 0, false, true>, NW, 65536, false, 2.0, result, st, kSustainedLaunches);
    case 1: return run_probe(probe_feed_kernel<NW, 2, false, true>, NW, 65536, false, 2.0, result, st, kSustainedLaunches);
    case 2: return run_probe(probe_feed_kernel<NW, 3, false, true>, NW, 65536, false, 2.0, result, st, kSustainedLaunches);
    case 3: return run_probe(probe_arrangement_kernel<NW, 0, true>, NW, 0, false, 1.0, result, st, kSustainedLaunches / 2);
  }
  return fail(-1, "probe: sustained variant %d", variant);
}

}  // namespace

int launch_probe(int family, int variant, int waves_per_simd, double* result, hipStream_t st) {
  if (!result) return fail(-1, "probe: null result");
  if (family == 2) {
    switch (variant) {
      case 0: return run_probe(probe_neighbour_kernel<1>, 8, 0, true, 16.0, result, st);
      case 1: return run_probe(probe_neighbour_kernel<2>, 8, 0, true, 16.0, result, st);
      case 2: return run_probe(probe_neighbour_kernel<3>, 8, 0, true, 16.0, result, st);
    }
    return fail(-1, "probe: neighbour variant %d", variant);
  }
  if (waves_per_simd != 1 && waves_per_simd != 2) return fail(-1, "probe: 1 or 2 waves per SIMD, got %d", waves_per_simd);
  if (family == 0) return waves_per_simd == 1 ? arrangement<4>(variant, result, st) : arrangement<8>(variant, result, st);
  if (family == 1) return waves_per_simd == 1 ? feed<4>(variant, result, st) : feed<8>(variant, result, st);
  if (family == 3) return waves_per_simd == 1 ? sustained<4>(variant, result, st) : sustained<8>(variant, result, st);
  return fail(-1, "probe: family %d", family);
}

}  // namespace dl
