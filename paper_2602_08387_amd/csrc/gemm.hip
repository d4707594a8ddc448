// bf16 GEMM for gfx950: C[M,N] = sum_s opA_s[M,K_s] * opB_s[K_s,N] (+R) with fp32 accumulation
// on v_mfma_f32_32x32x16_bf16.  One kernel template serves the three products of a linear
// layer (y = x W^T, dx = dy W, dW = dy^T x): each operand may be stored with the contraction
// index contiguous ("k-major") or with its M/N index contiguous ("mn-major").
//
// Data path: global --buffer_load ... lds (16 B per lane, no VGPR staging)--> LDS (two stages
// of BK = 64) --ds_read_b128 (k-major) or ds_read_b64_tr_b16 (mn-major)--> MFMA operands.
// The buffer descriptor's range check zero-fills rows past the end of a matrix, so M and N
// need not be tile multiples; K_s must be a multiple of 64.
//
// LDS layouts (the async load puts lane l's 16 bytes at chunk l of a 1 KiB span, so swizzles
// are applied on the global-address side):
//   k-major tile  [rows][64 k]   : 128 B per row = 8 chunks; chunk c of row r sits at c ^ (r & 7).
//   mn-major tile [64 k][R mn]   : R/8 chunks per k-row; chunk c of k-row k sits at
//                                  c ^ (((k & 3) << 2) & (R/8 - 1)).
// MFMA roles: the N-side operand feeds MFMA "A" (row index i), the M-side operand feeds MFMA
// "B" (column index j), so a lane ends up with 4 consecutive n for one m and the epilogue
// stores 8 bytes per lane into row-major C.
#include "common.h"
#include "kernels.h"

namespace dl {

constexpr int BK = 64;

struct GemmKArgs {
  const bf16_t* a[3];
  const bf16_t* b[3];
  int64_t lda[3], ldb[3];
  int K[3];
  int nseg;
  int M, N;
  bf16_t* c;
  int64_t ldc;
  const bf16_t* r;
  int accumulate;
  int tiles_m, tiles_n;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// Loads one operand tile (R rows of the M/N index, BK of k) for K-step origin k0 into LDS.
template <int R, bool KMAJOR, int NW>
struct TileLoader {
  static constexpr int NINSTR = R * BK * 2 / 1024;  // wave-wide 1 KiB loads per tile
  static constexpr int PER_WAVE = NINSTR / NW;
  static_assert(NINSTR % NW == 0, "tile loads must divide across waves");
  static constexpr int CPR = R / 8;                 // chunks per k-row (mn-major)
  static constexpr int RPI = KMAJOR ? 8 : 1024 / (R * 2);  // tile rows per instruction

  uint32_t voff[KMAJOR ? 1 : (RPI >= 4 ? 1 : 4 / RPI)];

  __device__ __forceinline__ void init(int lane, int64_t ld) {
    if constexpr (KMAJOR) {
      voff[0] = (uint32_t)((lane >> 3) * ld * 2 + (((lane & 7) ^ (lane >> 3)) << 4));
    } else {
      constexpr int NVAR = RPI >= 4 ? 1 : 4 / RPI;
#pragma unroll
      for (int v = 0; v < NVAR; ++v) {
        const int krow = v * RPI + lane / CPR;  // k-row within a group of 4 (only k & 3 matters)
        const int pc = lane % CPR;
        const int c = pc ^ (((krow & 3) << 2) & (CPR - 1));
        voff[v] = (uint32_t)((lane / CPR) * ld * 2 + (c << 4));
      }
    }
  }

  // lds_tile: byte offset of this tile's stage in LDS (uniform).  k0: k origin (uniform).
  __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rs, char* smem, int lds_tile, int wave,
                                        int64_t ld, int k0) const {
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
      const int j = wave * PER_WAVE + i;
      uint32_t soff, vo;
      if constexpr (KMAJOR) {
        soff = (uint32_t)(((int64_t)8 * j * ld + k0) * 2);
        vo = voff[0];
      } else {
        constexpr int NVAR = RPI >= 4 ? 1 : 4 / RPI;
        static_assert(PER_WAVE % NVAR == 0, "swizzle variant must not depend on the wave index");
        soff = (uint32_t)(((int64_t)(k0 + j * RPI) * ld) * 2);
        vo = voff[i % NVAR];
      }
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (LDS_PTR(void))(smem + lds_tile + j * 1024), 16, vo,
                                               soff, 0, 0);
    }
  }
};

// Reads the MFMA operand fragment for 32 rows starting at row0 (tile-local M/N index), k-substep
// kk (16 k), from a tile stored in LDS at `tile`.
template <int R, bool KMAJOR>
__device__ __forceinline__ bf16x8 read_frag(const char* tile, int row0, int kk, int lane) {
  if constexpr (KMAJOR) {
    const int row = row0 + (lane & 31);
    const int c = (kk * 2 + (lane >> 5)) ^ (row & 7);
    return *reinterpret_cast<const bf16x8*>(tile + row * 128 + (c << 4));
  } else {
    constexpr int CPR = R / 8;
    const int grp = lane >> 4, s = lane & 15, e = s >> 2, g = s & 3;
    const int col = row0 + ((grp & 1) << 4) + (g << 2);
    const int krow = kk * 16 + ((grp >> 1) << 3) + e;
    const int f = ((krow & 3) << 2) & (CPR - 1);  // same for krow and krow + 4
    const int byte = (((col >> 3) ^ f) << 4) + ((col & 7) << 1);
    const char* p0 = tile + krow * (R * 2) + byte;
    bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(p0));
    bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(p0 + 4 * R * 2));
    bf16x8 v;
    v.lo = lo;
    v.hi = hi;
    return v;
  }
}

template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__global__ __launch_bounds__(WM* WN * 64) void gemm_kernel(const GemmKArgs p) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int FM = TM / 32, FN = TN / 32;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wave_m = wave % WM, wave_n = wave / WM;

  // Tile order.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: give every
  // XCD a contiguous range of the tile sequence, and walk that sequence in bands of 8 tile-rows so
  // that the ~32 tiles an XCD holds at a time share A and B panels.
  int pid = blockIdx.x;
  const int ntiles = p.tiles_m * p.tiles_n;
  const int per_xcd = ntiles >> 3;
  if (pid < (per_xcd << 3)) pid = (pid & 7) * per_xcd + (pid >> 3);
  constexpr int GM = 8;
  const int band = pid / (GM * p.tiles_n);
  const int first_m = band * GM;
  const int band_h = min(p.tiles_m - first_m, GM);
  const int in_band = pid - band * GM * p.tiles_n;
  const int tile_m = first_m + in_band % band_h;
  const int tile_n = in_band / band_h;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  TileLoader<BM, AK, NW> la;
  TileLoader<BN, BKM, NW> lb;

  f32x16 acc[FN][FM];
#pragma unroll
  for (int i = 0; i < FN; ++i)
#pragma unroll
    for (int j = 0; j < FM; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  int stage = 0;
  bool first = true;
  for (int s = 0; s < p.nseg; ++s) {
    const int K = p.K[s];
    const int64_t lda = p.lda[s], ldb = p.ldb[s];
    const bf16_t* ab = AK ? p.a[s] + (int64_t)m0 * lda : p.a[s] + m0;
    const bf16_t* bb = BKM ? p.b[s] + (int64_t)n0 * ldb : p.b[s] + n0;
    const uint32_t a_bytes =
        AK ? (uint32_t)((((int64_t)(p.M - m0 - 1)) * lda + K) * 2) : (uint32_t)((((int64_t)(K - 1)) * lda + (p.M - m0)) * 2);
    const uint32_t b_bytes =
        BKM ? (uint32_t)((((int64_t)(p.N - n0 - 1)) * ldb + K) * 2) : (uint32_t)((((int64_t)(K - 1)) * ldb + (p.N - n0)) * 2);
    const __amdgpu_buffer_rsrc_t ra = make_rsrc(ab, a_bytes), rb = make_rsrc(bb, b_bytes);
    la.init(lane, lda);
    lb.init(lane, ldb);
    const int KT = K / BK;
    if (first) {
      la.issue(ra, smem, 0, wave, lda, 0);
      lb.issue(rb, smem, A_BYTES, wave, ldb, 0);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      first = false;
    }
    for (int kt = 0; kt < KT; ++kt) {
      const char* ta = smem + stage * STAGE;
      const char* tb = ta + A_BYTES;
      if (kt + 1 < KT) {
        la.issue(ra, smem, (stage ^ 1) * STAGE, wave, lda, (kt + 1) * BK);
        lb.issue(rb, smem, (stage ^ 1) * STAGE + A_BYTES, wave, ldb, (kt + 1) * BK);
      } else if (s + 1 < p.nseg) {
        // first K-step of the next segment
        const int64_t lda2 = p.lda[s + 1], ldb2 = p.ldb[s + 1];
        const int K2 = p.K[s + 1];
        const bf16_t* ab2 = AK ? p.a[s + 1] + (int64_t)m0 * lda2 : p.a[s + 1] + m0;
        const bf16_t* bb2 = BKM ? p.b[s + 1] + (int64_t)n0 * ldb2 : p.b[s + 1] + n0;
        const uint32_t a2 = AK ? (uint32_t)((((int64_t)(p.M - m0 - 1)) * lda2 + K2) * 2)
                               : (uint32_t)((((int64_t)(K2 - 1)) * lda2 + (p.M - m0)) * 2);
        const uint32_t b2 = BKM ? (uint32_t)((((int64_t)(p.N - n0 - 1)) * ldb2 + K2) * 2)
                                : (uint32_t)((((int64_t)(K2 - 1)) * ldb2 + (p.N - n0)) * 2);
        TileLoader<BM, AK, NW> la2;
        TileLoader<BN, BKM, NW> lb2;
        la2.init(lane, lda2);
        lb2.init(lane, ldb2);
        la2.issue(make_rsrc(ab2, a2), smem, (stage ^ 1) * STAGE, wave, lda2, 0);
        lb2.issue(make_rsrc(bb2, b2), smem, (stage ^ 1) * STAGE + A_BYTES, wave, ldb2, 0);
      }
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        bf16x8 fa[FM], fb[FN];
#pragma unroll
        for (int j = 0; j < FM; ++j) fa[j] = read_frag<BM, AK>(ta, wave_m * TM + j * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < FN; ++i) fb[i] = read_frag<BN, BKM>(tb, wave_n * TN + i * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < FN; ++i)
#pragma unroll
          for (int j = 0; j < FM; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i], fa[j], acc[i][j], 0, 0, 0);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      stage ^= 1;
    }
  }

  // Epilogue: lane holds, per 32x32 MFMA tile, column m = lane % 32 and rows
  // n = 8*(r/4) + 4*(lane/32) + r%4 of acc (acc is indexed [n][m]).
  const int lm = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int j = 0; j < FM; ++j) {
    const int m = m0 + wave_m * TM + j * 32 + lm;
    if (m < p.M) {
      bf16_t* crow = p.c + (int64_t)m * p.ldc;
      const bf16_t* rrow = p.r ? p.r + (int64_t)m * p.ldc : nullptr;
#pragma unroll
      for (int i = 0; i < FN; ++i) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = n0 + wave_n * TN + i * 32 + g * 8 + lh * 4;
          if (n < p.N) {
            float v0 = acc[i][j][g * 4 + 0], v1 = acc[i][j][g * 4 + 1], v2 = acc[i][j][g * 4 + 2],
                  v3 = acc[i][j][g * 4 + 3];
            if (rrow) {
              bf16x4 rv = *reinterpret_cast<const bf16x4*>(rrow + n);
              v0 += (float)rv[0]; v1 += (float)rv[1]; v2 += (float)rv[2]; v3 += (float)rv[3];
            }
            if (p.accumulate) {
              bf16x4 cv = *reinterpret_cast<const bf16x4*>(crow + n);
              v0 += (float)cv[0]; v1 += (float)cv[1]; v2 += (float)cv[2]; v3 += (float)cv[3];
            }
            bf16x4 o;
            o[0] = (bf16_t)v0; o[1] = (bf16_t)v1; o[2] = (bf16_t)v2; o[3] = (bf16_t)v3;
            *reinterpret_cast<bf16x4*>(crow + n) = o;
          }
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
static int launch_cfg(const GemmKArgs& k, bool ak, bool bk, hipStream_t st) {
  GemmKArgs a = k;
  a.tiles_m = (k.M + BM - 1) / BM;
  a.tiles_n = (k.N + BN - 1) / BN;
  const dim3 grid((unsigned)(a.tiles_m * a.tiles_n)), block(WM * WN * 64);
  const size_t lds = 2 * (size_t)(BM + BN) * BK * 2;
#define GEMM_LAUNCH(AK_, BK_)                                                                    \
  do {                                                                                           \
    auto kern = gemm_kernel<BM, BN, WM, WN, AK_, BK_>;                                           \
    static bool attr_set = false;                                                                \
    if (!attr_set) {                                                                             \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                    \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
      if (e != hipSuccess) return fail(-3, "gemm: cannot reserve %zu B of LDS: %s", lds, hipGetErrorString(e)); \
      attr_set = true;                                                                           \
    }                                                                                            \
    hipLaunchKernelGGL(kern, grid, block, lds, st, a);                                           \
  } while (0)
  if (ak && bk) GEMM_LAUNCH(true, true);
  else if (ak && !bk) GEMM_LAUNCH(true, false);
  else if (!ak && bk) GEMM_LAUNCH(false, true);
  else GEMM_LAUNCH(false, false);
#undef GEMM_LAUNCH
  return check_launch("gemm");
}

int launch_gemm(const GemmArgs& g, hipStream_t st) {
  GemmKArgs k{};
  k.nseg = g.nseg;
  for (int s = 0; s < g.nseg; ++s) {
    k.a[s] = (const bf16_t*)g.seg[s].a;
    k.b[s] = (const bf16_t*)g.seg[s].b;
    k.lda[s] = g.seg[s].lda;
    k.ldb[s] = g.seg[s].ldb;
    k.K[s] = g.seg[s].K;
  }
  k.M = g.M;
  k.N = g.N;
  k.c = (bf16_t*)g.c;
  k.ldc = g.ldc;
  k.r = (const bf16_t*)g.r;
  k.accumulate = g.accumulate;
  // Large problems: 256x256 tiles, 8 waves (2 per SIMD), 128x64 per wave.  Small ones: 128x128
  // tiles so that the grid still covers the 256 CUs.
  const int64_t tiles256 = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256);
  if (tiles256 >= 192) return launch_cfg<256, 256, 2, 4>(k, g.a_kmajor, g.b_kmajor, st);
  return launch_cfg<128, 128, 2, 2>(k, g.a_kmajor, g.b_kmajor, st);
}

}  // namespace dl
