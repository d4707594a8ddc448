// bf16 GEMM for gfx950: C[M,N] = sum_s opA_s[M,K_s] * opB_s[K_s,N] (+R) with fp32 accumulation
// on v_mfma_f32_16x16x32_bf16.  One kernel template serves the three products of a linear
// layer (y = x W^T, dx = dy W, dW = dy^T x): each operand may be stored with the contraction
// index contiguous ("k-major") or with its M/N index contiguous ("mn-major").
//
// Data path: global --buffer_load ... lds (16 B per lane, no VGPR staging)--> LDS ring of NS
// stages, BK k-values each --ds_read_b128 (k-major) or ds_read_b64_tr_b16 (mn-major)--> MFMA
// operands.  Loads run NS-1 K-steps ahead of the MFMAs.  The buffer descriptor's range check
// zero-fills rows past the end of a matrix, so M and N need not be tile multiples; K_s must be a
// multiple of 64.
//
// LDS layouts (the async load puts lane l's 16 bytes at chunk l of a 1 KiB span, so swizzles
// are applied on the global-address side).  The LDS serves 256 B of banks per clock: a 16-byte
// read is done 16 lanes at a time, an 8-byte transposed read 32 lanes at a time.
//   k-major tile  [rows][BK k]   : BK*2 bytes per row = CPR chunks; chunk c of row r sits at
//                                  c ^ ((r / (16/CPR)) & (CPR-1)), so 16 consecutive rows reading
//                                  one logical chunk touch 16 different 16-byte bank groups.
//   mn-major tile [BK k][R mn]   : R/8 chunks per k-row; chunk c of k-row k sits at
//                                  c ^ ((((k & 3) << 2) | (((k >> 3) & 1) << 1)) & (R/8 - 1)): the
//                                  8 k-rows x 32 B that 32 lanes of a transposed read touch fall in
//                                  8 different 32-byte bank groups.
// MFMA roles: the N-side operand feeds MFMA "A" (row index i), the M-side operand feeds MFMA
// "B" (column index j), so a lane ends up with 4 consecutive n for one m.  The epilogue passes
// the tile through LDS so that global stores (and residual loads) are 16 bytes per lane along
// rows of C.
#include "common.h"
#include "kernels.h"
#include <atomic>
#include <type_traits>

namespace dl {

// Measured on MI355X (M=16384, K=4096, N=14336, normal data): 2 stages of 64 k-values beat 3, 4 and 5
// stages of 32 (the K-step is not latency-bound, a deeper ring only adds barriers); 16x16x32 MFMA
// blocks beat 32x32x16 by 3 % on y = x W^T and 11 % on dx = dy W (half the accumulator traffic per
// flop); 8 waves of 128x64 beat 4 waves of 128x128 under the compiler's schedule.
constexpr int BK = 64;   // k-values per pipeline stage
constexpr int NS = 2;    // ring stages
constexpr int MI = 16;               // MFMA block edge: 32 (32x32x16) or 16 (16x16x32)
constexpr int KSTEP = MI == 32 ? 16 : 32;  // k per MFMA
constexpr int NACC = MI * MI / 64;       // accumulator registers per MFMA block
typedef float acc_t __attribute__((ext_vector_type(NACC)));
__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

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
  int band_rows;   // tile rows per band of the tile sequence (see band_rows_for)
  // gated-pair products only (see gemm_swiglu_kernel): second weight, second and third output
  const bf16_t* b2;
  bf16_t *c2, *c3;
  int64_t ldc3;
  // activation-gradient epilogue only (see EPI_SWIGLU_GRAD)
  const bf16_t *e1, *e2;
  int64_t lde;
  // rotary epilogue only (see EPI_ROPE): rotate this problem's output
  int rope;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// Loads one operand tile (R rows of the M/N index, BK of k) for K-step origin k0 into LDS.
template <int R, bool KMAJOR, int NW>
struct TileLoader {
  static constexpr int NINSTR = R * BK * 2 / 1024;  // wave-wide 1 KiB loads per tile
  static constexpr int PER_WAVE = NINSTR / NW;
  static_assert(NINSTR % NW == 0 && PER_WAVE >= 1, "tile loads must divide across waves");
  static constexpr int CPRK = BK / 8;               // chunks per row of a k-major tile
  static constexpr int RPW = 16 / CPRK;             // k-major rows per 256-byte bank window
  static constexpr int CPR = R / 8;                 // chunks per k-row (mn-major)
  static constexpr int RPI = KMAJOR ? 1024 / (BK * 2) : 1024 / (R * 2);  // tile rows per instruction
  // k-major: swizzle variants a lane needs across its instructions (precomputed offsets);
  // mn-major: the chunk swizzle is applied per instruction from (row part, chunk, k-row in instr).
  static constexpr int NVAR = KMAJOR ? (RPI >= 16 ? 1 : 16 / RPI) : 1;
  static_assert(PER_WAVE % NVAR == 0, "swizzle variant must not depend on the wave index");
  uint32_t voff[NVAR];
  int pc, kq;

  // chunk XOR of k-row k of an mn-major tile: the rows k..k+3 (bits 2-3) and k+8.. (bit 1) that a
  // 32-lane transposed read touches fall in 8 different 32-byte bank groups.
  static __device__ __forceinline__ int mn_swz(int k) {
    return (((k & 3) << 2) | (((k >> 3) & 1) << 1)) & (CPR - 1);
  }

  __device__ __forceinline__ void init(int lane, int64_t ld) {
    if constexpr (KMAJOR) {
      // instruction j covers rows RPI*j ..; the swizzle depends on (row / RPW) & (CPRK - 1)
#pragma unroll
      for (int v = 0; v < NVAR; ++v) {
        const int row = v * RPI + lane / CPRK;   // row modulo 16
        const int c = (lane % CPRK) ^ ((row / RPW) & (CPRK - 1));
        voff[v] = (uint32_t)((lane / CPRK) * ld * 2 + (c << 4));
      }
    } else {
      kq = lane / CPR;
      pc = lane % CPR;
      voff[0] = (uint32_t)(kq * ld * 2);
    }
  }

  __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rs, char* lds_tile, int wave, int64_t ld,
                                        int k0) const {
    issue_range<0, PER_WAVE>(rs, lds_tile, wave, ld, k0);
  }
  // this wave's loads I0 .. I1-1 of the tile
  template <int I0, int I1>
  __device__ __forceinline__ void issue_range(__amdgpu_buffer_rsrc_t rs, char* lds_tile, int wave, int64_t ld,
                                              int k0) const {
#pragma unroll
    for (int i = I0; i < I1; ++i) {
      const int j = wave * PER_WAVE + i;
      const uint32_t soff = KMAJOR ? (uint32_t)(((int64_t)RPI * j * ld + k0) * 2)
                                   : (uint32_t)(((int64_t)(k0 + j * RPI) * ld) * 2);
      uint32_t vo;
      if constexpr (KMAJOR) vo = voff[i % NVAR];
      else vo = voff[0] + (uint32_t)((pc ^ mn_swz(j * RPI + kq)) << 4);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (LDS_PTR(void))(lds_tile + j * 1024), 16, vo, soff, 0, 0);
    }
  }
  // Tile of a k-major matrix whose rows are heads of 128 features, loaded so that a wave whose MFMA
  // tile spans 64 tile rows holds 32 features of a head's first half and, 32 tile rows further, their
  // rotary partners 64 features on: tile row r <- matrix row
  // 128 * (r / 128) + 32 * ((r / 64) & 1) + r % 32 + 64 * ((r / 32) & 1).
  static __device__ __forceinline__ int perm_row(int r) {
    return ((r >> 7) << 7) + (((r >> 6) & 1) << 5) + (r & 31) + (((r >> 5) & 1) << 6);
  }
  template <int I0, int I1>
  __device__ __forceinline__ void issue_perm_range(__amdgpu_buffer_rsrc_t rs, char* lds_tile, int wave, int64_t ld,
                                                   int k0) const {
    static_assert(KMAJOR && 32 % RPI == 0, "an instruction's rows must lie in one run of 32");
#pragma unroll
    for (int i = I0; i < I1; ++i) {
      const int j = wave * PER_WAVE + i;
      const uint32_t soff = (uint32_t)(((int64_t)perm_row(j * RPI) * ld + k0) * 2);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (LDS_PTR(void))(lds_tile + j * 1024), 16, voff[i % NVAR], soff, 0, 0);
    }
  }
  // Tile of a PAIR of k-major matrices: of every 64 tile rows the first 32 are rows of the first
  // matrix and the next 32 the SAME rows of the second (tile row r <- matrix (r / 32) & 1, row
  // (r / 64) * 32 + r % 32), so that a wave whose MFMA tile spans 64 of these rows holds both values
  // of a column pair.  LDS placement and swizzle are those of the plain tile.
  template <int I0, int I1>
  __device__ __forceinline__ void issue_pair_range(__amdgpu_buffer_rsrc_t rs0, __amdgpu_buffer_rsrc_t rs1,
                                                   char* lds_tile, int wave, int64_t ld, int k0) const {
    static_assert(KMAJOR && 32 % RPI == 0, "an instruction's rows must lie in one matrix");
#pragma unroll
    for (int i = I0; i < I1; ++i) {
      const int j = wave * PER_WAVE + i;
      const int r0 = j * RPI;
      const int row = (r0 >> 6) * 32 + (r0 & 31);
      const uint32_t soff = (uint32_t)(((int64_t)row * ld + k0) * 2);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(((r0 >> 5) & 1) ? rs1 : rs0, (LDS_PTR(void))(lds_tile + j * 1024), 16,
                                               voff[i % NVAR], soff, 0, 0);
    }
  }
};

// MFMA operand fragment for MI rows starting at row0 (tile-local M/N index), k-substep kk (KSTEP k).
template <int R, bool KMAJOR>
__device__ __forceinline__ bf16x8 read_frag(const char* tile, int row0, int kk, int lane) {
  if constexpr (KMAJOR) {
    constexpr int CPRK = BK / 8, RPW = 16 / CPRK;
    const int row = row0 + (lane & (MI - 1));
    const int c = (kk * (KSTEP / 8) + lane / MI) ^ ((row / RPW) & (CPRK - 1));
    return *reinterpret_cast<const bf16x8*>(tile + row * (BK * 2) + (c << 4));
  } else {
    constexpr int CPR = R / 8;
    const int grp = lane >> 4, s = lane & 15, e = s >> 2, g = s & 3;
    const int col = MI == 32 ? row0 + ((grp & 1) << 4) + (g << 2) : row0 + (g << 2);
    const int krow = MI == 32 ? kk * 16 + ((grp >> 1) << 3) + e : kk * 32 + (grp << 3) + e;
    const int f = (((krow & 3) << 2) | (((krow >> 3) & 1) << 1)) & (CPR - 1);  // same for krow and krow + 4
    const char* p0 = tile + krow * (R * 2) + ((((col >> 3) ^ f) << 4) | ((col & 7) << 1));
    // Issued as inline assembly: for the builtin the compiler cannot tell that the read does not
    // touch the stage the asynchronous global -> LDS loads are filling and puts an s_waitcnt vmcnt(0)
    // in front of it, which stalls the loading waves for the whole load latency every K-step.  The
    // price: the compiler does not count these reads in lgkmcnt either, so every consumer must sit
    // behind wait_frags().
    bf16x8 v;
    bf16x4 lo, hi;
    const uint32_t a0 = (uint32_t)(uintptr_t)(LDS_PTR(char))(p0);
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(a0));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a0), "n"(4 * R * 2));
    v.lo = lo;
    v.hi = hi;
    return v;
  }
}

// f(integral_constant<int, I>) for I = I0 .. N-1: a loop whose index is a compile-time constant
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Waits for every LDS read of this wave and makes the fragments depend on that wait, so that no
// consumer of a fragment fetched by the inline-assembly transposed read can be scheduled before it.
template <int FM, int FN>
__device__ __forceinline__ void wait_frags(bf16x8 (&fa)[FM], bf16x8 (&fb)[FN]) {
  static_assert(FM == 8 && FN == 4 || FM == 4 && FN == 4, "operand list written out for the two wave tiles in use");
  if constexpr (FM == 8)
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(fa[0]), "+v"(fa[1]), "+v"(fa[2]), "+v"(fa[3]), "+v"(fa[4]), "+v"(fa[5]), "+v"(fa[6]), "+v"(fa[7]),
                   "+v"(fb[0]), "+v"(fb[1]), "+v"(fb[2]), "+v"(fb[3]));
  else
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(fa[0]), "+v"(fa[1]), "+v"(fa[2]), "+v"(fa[3]), "+v"(fb[0]), "+v"(fb[1]), "+v"(fb[2]), "+v"(fb[3]));
}

// Position of the next tile pair to fetch: segment, k offset, and that segment's descriptors.
// PAIR: the B tile interleaves two weight matrices (TileLoader::issue_pair_range); n0 and N then
// count columns of the interleaved product, twice the rows of either matrix.
// PERM: the B tile takes its rows in the rotary-partner order of TileLoader::issue_perm_range.
template <int BM, int BN, int NW, bool AK, bool BKM, bool PAIR = false, bool PERM = false>
struct LoadCursor {
  TileLoader<BM, AK, NW> la;
  TileLoader<BN, BKM, NW> lb;
  __amdgpu_buffer_rsrc_t ra, rb, rb2;
  int64_t lda, ldb;
  int seg = 0, k = 0, kend = 0, nseg = 1;   // kend: K of the open segment (kept in a register: no kernarg read per K-step)
  int left = 0;                             // K-steps of the tile still to fetch; the walk may start anywhere and wraps

  __device__ __forceinline__ void open_raw(const bf16_t* a, const bf16_t* b, int64_t lda_, int64_t ldb_, int K, int M,
                                           int N, int m0, int n0, int lane) {
    kend = K;
    lda = lda_;
    ldb = ldb_;
    const bf16_t* ab = AK ? a + (int64_t)m0 * lda : a + m0;
    const bf16_t* bb = BKM ? b + (int64_t)n0 * ldb : b + n0;
    const uint32_t a_bytes = AK ? (uint32_t)((((int64_t)(M - m0 - 1)) * lda + K) * 2)
                                : (uint32_t)((((int64_t)(K - 1)) * lda + (M - m0)) * 2);
    const uint32_t b_bytes = BKM ? (uint32_t)((((int64_t)(N - n0 - 1)) * ldb + K) * 2)
                                 : (uint32_t)((((int64_t)(K - 1)) * ldb + (N - n0)) * 2);
    ra = make_rsrc(ab, a_bytes);
    rb = make_rsrc(bb, b_bytes);
    la.init(lane, lda);
    lb.init(lane, ldb);
  }
  __device__ __forceinline__ void open_pair(const bf16_t* a, const bf16_t* b, const bf16_t* b2, int64_t lda_,
                                            int64_t ldb_, int K, int M, int N, int m0, int n0, int lane) {
    static_assert(!PAIR || (AK && BKM), "paired weights are k-major");
    open_raw(a, b, lda_, ldb_, K, M, N / 2, m0, n0 / 2, lane);
    rb2 = make_rsrc(b2 + (int64_t)(n0 / 2) * ldb_, (uint32_t)((((int64_t)(N / 2 - n0 / 2 - 1)) * ldb_ + K) * 2));
  }
  __device__ __forceinline__ void open(const GemmKArgs& p, int s, int m0, int n0, int lane) {
    open_raw(p.a[s], p.b[s], p.lda[s], p.ldb[s], p.K[s], p.M, p.N, m0, n0, lane);
  }
  // The same in NC pieces (piece C of the A loads and of the B loads), so that a wave can spread its
  // loads between MFMAs; the cursor moves on with the last piece.
  template <int C, int NC>
  __device__ __forceinline__ void issue_piece(const GemmKArgs& segs, char* stage, int wave, int m0, int n0, int lane) {
    constexpr int PA = TileLoader<BM, AK, NW>::PER_WAVE, PB = TileLoader<BN, BKM, NW>::PER_WAVE;
    if (left > 0) {
      la.template issue_range<C * PA / NC, (C + 1) * PA / NC>(ra, stage, wave, lda, k);
      if constexpr (PAIR)
        lb.template issue_pair_range<C * PB / NC, (C + 1) * PB / NC>(rb, rb2, stage + BM * BK * 2, wave, ldb, k);
      else if constexpr (PERM)
        lb.template issue_perm_range<C * PB / NC, (C + 1) * PB / NC>(rb, stage + BM * BK * 2, wave, ldb, k);
      else
        lb.template issue_range<C * PB / NC, (C + 1) * PB / NC>(rb, stage + BM * BK * 2, wave, ldb, k);
      if constexpr (C + 1 == NC) advance(segs, m0, n0, lane);
    }
  }
  // `segs`: the problem whose further K-segments follow (only read when nseg > 1)
  __device__ __forceinline__ void issue_next(const GemmKArgs& segs, char* stage, int wave, int m0, int n0, int lane) {
    if (left > 0) {
      la.issue(ra, stage, wave, lda, k);
      if constexpr (PAIR)
        lb.template issue_pair_range<0, TileLoader<BN, BKM, NW>::PER_WAVE>(rb, rb2, stage + BM * BK * 2, wave, ldb, k);
      else if constexpr (PERM)
        lb.template issue_perm_range<0, TileLoader<BN, BKM, NW>::PER_WAVE>(rb, stage + BM * BK * 2, wave, ldb, k);
      else
        lb.issue(rb, stage + BM * BK * 2, wave, ldb, k);
      advance(segs, m0, n0, lane);
    }
  }
  // one K-step on: past the end of a segment the walk goes on in the next one, past the last in the first
  __device__ __forceinline__ void advance(const GemmKArgs& segs, int m0, int n0, int lane) {
    --left;
    k += BK;
    if (k == kend) {
      k = 0;
      if (nseg > 1 && left > 0) {
        seg = seg + 1 == nseg ? 0 : seg + 1;
        open(segs, seg, m0, n0, lane);
      }
    }
  }
};

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: give every XCD a contiguous
// range of the tile sequence.
__device__ __forceinline__ int xcd_contiguous(int id, int ntiles) {
  const int per_xcd = ntiles >> 3;
  return id < (per_xcd << 3) ? (id & 7) * per_xcd + (id >> 3) : id;
}

// Several independent problems of one operand layout in one grid: their tile sequences are laid end
// to end, so the last, partly filled round of one problem runs alongside the first of the next.
constexpr int MAX_GROUP = 8;
struct GemmGroupKArgs {
  GemmKArgs prob[MAX_GROUP];
  int tile_start[MAX_GROUP + 1];
  int n;
  // rotary epilogue only (see EPI_ROPE): cos and sin of the angle of (position, pair), [seq][head_dim/2]
  const float *rope_cos, *rope_sin;
  int rope_seq, rope_dh, rope_layout;
};

// Persistent workgroup: one per CU, walking the tile sequence with stride gridDim.x.  Between two
// tiles the first two K-steps of the next tile are already on their way into the LDS ring while the
// epilogue of the current one drains the accumulators through a staging region of its own, and the
// C stores of a tile complete under the next tile's main loop.
//
// The kernel arguments are only ever read with compile-time offsets (a grouped launch picks its
// problem by comparing against each index in turn): a run-time index into the argument block would
// make the compiler copy the whole block to scratch memory and read it back through vector loads.
//
// EPI_SWIGLU: the gated pair of the MLP in one pass.  B interleaves the rows of two weight matrices
// (LoadCursor PAIR) so that every wave holds g = x Wg^T and u = x Wu^T for the same 32 columns; the
// epilogue stores g to c, u to c2 and silu(g) * u, taken from the ROUNDED g and u like the separate
// activation kernel would, to c3.  M x N is the interleaved product: N = twice the columns of g.
//
// EPI_SWIGLU_GRAD: the product is da, the gradient arriving at a = silu(g) * u; the epilogue reads the
// g and u tiles (e1, e2, leading dimension lde) and stores dg to c and du to c2 instead of da,
// again from the rounded da like the separate kernel.
//
// EPI_ROPE (grouped launch of head projections): problems flagged `rope` have the rotary embedding
// applied to their output in the epilogue, on the fp32 accumulators, so that q and k are rounded to
// bf16 once.  Rows of C are tokens (position = row % rope_seq), columns are [head][head_dim].  A wave
// owns 64 columns and needs both members of a pair: with adjacent pairs (2i, 2i+1) a lane holds them
// already; with split pairs (i, i + head_dim/2) a 64-wide head is one wave's strip, a 32-wide head half
// of one, and for 128-wide heads the B tile is loaded in partner order (PERM, every problem of the
// launch) and the epilogue stores the two 32-column runs of a wave where they belong.
enum { EPI_PLAIN = 0, EPI_SWIGLU = 1, EPI_SWIGLU_GRAD = 2, EPI_ROPE = 3 };
template <bool GROUPED, int BM, int BN, int WM, int WN, bool AK, bool BKM, int EPI = EPI_PLAIN, bool PERM = false>
__device__ __forceinline__ void gemm_persistent(const GemmGroupKArgs& grp, const GemmKArgs& one) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int FM = TM / MI, FN = TN / MI;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
  // Only one wave per SIMD issues the global -> LDS loads.  The address unit takes 16 cycles per
  // wave-wide 16-byte load (1024 cycles per K-step for a 256x256x64 tile pair) and a wave blocks
  // while its loads queue up; if both waves of a SIMD do that at the same time the matrix pipe
  // starves, whereas a loading wave next to a computing wave keeps it fed (+3..6 % measured).
  constexpr int NL = NW < 4 ? NW : 4;
  using LoadA = TileLoader<BM, AK, NL>;
  using LoadB = TileLoader<BN, BKM, NL>;
  constexpr int LPW = LoadA::PER_WAVE + LoadB::PER_WAVE;   // loads per wave per stage
  static_assert(NS == 2, "the stage hand-over below is written for a two-stage ring");
  static_assert(TN % 64 == 0 && FM % 4 == 0, "staging layout: 128-byte rows, four row quarters");
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wave_m = wave % WM, wave_n = wave / WM;
  const bool loader = wave < NL;
  int ntiles;
  if constexpr (GROUPED) {
    ntiles = grp.tile_start[1];
#pragma unroll
    for (int i = 2; i <= MAX_GROUP; ++i) if (i <= grp.n) ntiles = grp.tile_start[i];
  } else {
    ntiles = one.tiles_m * one.tiles_n;
  }

  // What the epilogue needs of a tile's problem, by value (the next tile's cursor is opened before the
  // current tile's epilogue runs).
  struct Tile { int m0, n0, total, M, N, accumulate, rope; bf16_t* c; const bf16_t* r; int64_t ldc; };
  constexpr bool SWIGLU = EPI == EPI_SWIGLU;
  LoadCursor<BM, BN, NL, AK, BKM, SWIGLU, PERM> cur;
  static_assert(EPI == EPI_PLAIN || (TN == 64 && MI == 16), "fused epilogues: one 64-column strip per wave");
  static_assert(EPI == EPI_PLAIN || GROUPED == (EPI == EPI_ROPE), "the rotary epilogue is the grouped launch's, the others are not");
  static_assert(!PERM || (EPI == EPI_ROPE && AK && BKM && BN % 128 == 0), "partner-order tiles: rotary epilogue only");

  // tile id -> tile origin, and the load cursor opened on the tile's first K-segment.  The tile
  // sequence of a problem runs in bands of band_rows (8 or 4) tile-rows, so that the ~32 consecutive
  // tiles an XCD holds at a time share A and B panels.
  auto locate = [&](int id) {
    int pid = xcd_contiguous(id, ntiles);
    int tiles_m, tiles_n, K0, GM, start = 0;
    const bf16_t *a0, *b0;
    int64_t lda0, ldb0;
    Tile t;
    auto take = [&](const GemmKArgs& q) {
      tiles_m = q.tiles_m; tiles_n = q.tiles_n; K0 = q.K[0]; GM = q.band_rows > 0 ? q.band_rows : 8;
      a0 = q.a[0]; b0 = q.b[0]; lda0 = q.lda[0]; ldb0 = q.ldb[0];
      t.M = q.M; t.N = q.N; t.accumulate = q.accumulate; t.c = q.c; t.r = q.r; t.ldc = q.ldc;
      t.rope = EPI == EPI_ROPE ? q.rope : 0;
    };
    if constexpr (GROUPED) {
      // problem index: the number of problems whose first tile is not after pid
      take(grp.prob[0]);
#pragma unroll
      for (int i = 1; i < MAX_GROUP; ++i)
        if (i < grp.n && pid >= grp.tile_start[i]) { take(grp.prob[i]); start = grp.tile_start[i]; }
      pid -= start;
      cur.nseg = 1;   // grouped problems have a single K-segment (checked on the host)
      t.total = K0 / BK;
    } else {
      take(one);
      cur.nseg = one.nseg;
      t.total = 0;
      for (int s2 = 0; s2 < one.nseg; ++s2) t.total += one.K[s2] / BK;
    }
    const int band = pid / (GM * tiles_n);
    const int first_m = band * GM;
    const int band_h = min(tiles_m - first_m, GM);
    const int in_band = pid - band * GM * tiles_n;
    t.m0 = (first_m + in_band % band_h) * BM;
    t.n0 = (in_band / band_h) * BN;
    // The contraction of a tile starts (g mod 8) eighths of the way through K and wraps around, g = the
    // tile's group of 8 tile-rows.  The XCDs work on different groups at any one time, and without this
    // they would all stream the same k-range of their operands at once: the requests then crowd the
    // same memory channels (worst with rows a multiple of 4 KiB apart, see the down projection's
    // weight).  The start depends on the tile's rows only - not on the workgroup, the launch or the band
    // height - so a product gives the same bits in whatever launch it is computed.
    cur.left = t.total;
    int first = (((t.m0 / (8 * BM)) & 7) * t.total) >> 3;   // in K-steps from the start of segment 0
    cur.seg = 0;
    if constexpr (!GROUPED) {
      for (int s2 = 0; s2 + 1 < one.nseg; ++s2)
        if (cur.seg == s2 && first >= one.K[s2] / BK) { first -= one.K[s2] / BK; cur.seg = s2 + 1; }
    }
    cur.k = first * BK;
    if (cur.seg == 0) {
      if constexpr (SWIGLU) cur.open_pair(a0, b0, one.b2, lda0, ldb0, K0, t.M, t.N, t.m0, t.n0, lane);
      else cur.open_raw(a0, b0, lda0, ldb0, K0, t.M, t.N, t.m0, t.n0, lane);
    } else {
      cur.open(one, cur.seg, t.m0, t.n0, lane);
    }
    return t;
  };

  // Load cursor: runs two K-steps ahead of the compute cursor, across segment boundaries.
  int id = blockIdx.x;
  if (id >= ntiles) return;
  Tile tl = locate(id);
  if (loader) {
    cur.issue_next(one, smem, wave, tl.m0, tl.n0, lane);
    cur.issue_next(one, smem + STAGE, wave, tl.m0, tl.n0, lane);
  }
  if (tl.total >= 2) wait_vmcnt<LPW>(); else wait_vmcnt<0>();

  // K-step s of a tile lives in ring stage (s + par) & 1: the K-steps of successive tiles form one
  // stream through the ring, so `par` moves on by the tile's number of K-steps.
  int par = 0;
  while (true) {
    const Tile p = tl;   // this tile; `tl` moves on to the next one during its last K-steps
    const int m0 = tl.m0, n0 = tl.n0, total = tl.total;
    bool early = false;
    acc_t acc[FN][FM];
#pragma unroll
    for (int i = 0; i < FN; ++i)
#pragma unroll
      for (int j = 0; j < FM; ++j)
#pragma unroll
        for (int e = 0; e < NACC; ++e) acc[i][j][e] = 0.f;

    // K-step 0 has landed in every loading wave's share (waited for before the first tile, or in the
    // previous tile's epilogue); the barrier makes it visible to all waves
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // Software-pipelined K loop: operand fragments are double-buffered in registers; the barrier that
    // hands over to the next stage sits before the last MFMA group of the current one, so the matrix
    // pipe stays busy while the first fragments of the next stage are fetched from LDS.
    constexpr int KK = BK / KSTEP;
    bf16x8 fa[2][FM], fb[2][FN];
    {
      const char* ta = smem + par * STAGE;
      const char* tb = ta + A_BYTES;
#pragma unroll
      for (int j = 0; j < FM; ++j) fa[0][j] = read_frag<BM, AK>(ta, wave_m * TM + j * MI, 0, lane);
#pragma unroll
      for (int i = 0; i < FN; ++i) fb[0][i] = read_frag<BN, BKM>(tb, wave_n * TN + i * MI, 0, lane);
    }
    if constexpr (!(AK && BKM)) wait_frags<FM, FN>(fa[0], fb[0]);
    for (int t = 0; t < total; ++t) {
      // Every load of this tile is out once its last but one K-step begins.  The cursor moves on to the
      // workgroup's next tile there, and that tile's first two K-steps go out at this tile's last two
      // hand-overs like any other refill: by the time the epilogue runs they have had a K-step to land.
      if (t == total - 2 && id + (int)gridDim.x < ntiles) {
        tl = locate(id + gridDim.x);
        early = true;
      }
      char* st_cur = smem + ((t + par) & 1) * STAGE;
      const char* ta = st_cur;
      const char* tb = ta + A_BYTES;
      static_for<0, KK>([&](auto kk_c) {
        constexpr int kk = decltype(kk_c)::value;
        constexpr int cb = kk & 1, nb = cb ^ 1;
        if constexpr (AK && BKM) {
          if (kk + 1 < KK) {
#pragma unroll
            for (int j = 0; j < FM; ++j) fa[nb][j] = read_frag<BM, AK>(ta, wave_m * TM + j * MI, kk + 1, lane);
#pragma unroll
            for (int i = 0; i < FN; ++i) fb[nb][i] = read_frag<BN, BKM>(tb, wave_n * TN + i * MI, kk + 1, lane);
          } else {
            // all of this wave's reads of stage t are in registers; stage t+1 must have landed
            wait_vmcnt<0>();   // the only loads in flight are those of stage t+1, issued one K-step ago
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            // every wave now holds its last fragments of stage t in registers: refill that stage with
            // step t+2 right away, so the loads get a whole K-step to land (about 2800 cycles at 1.9 GHz
            // under sustained load; cycle counters put the wait for the slowest of them, those that
            // miss the L2, at some 300 cycles per K-step on top of that)
            if (loader) cur.issue_next(one, st_cur, wave, tl.m0, tl.n0, lane);
            // the reads go out unconditionally (after the last K-step they fetch stale bytes nobody
            // uses), which keeps them in one block with this group's MFMAs so that the scheduler
            // interleaves them (+2 %)
            const char* na = smem + ((t + 1 + par) & 1) * STAGE;
            const char* nbp = na + A_BYTES;
#pragma unroll
            for (int j = 0; j < FM; ++j) fa[nb][j] = read_frag<BM, AK>(na, wave_m * TM + j * MI, 0, lane);
#pragma unroll
            for (int i = 0; i < FN; ++i) fb[nb][i] = read_frag<BN, BKM>(nbp, wave_n * TN + i * MI, 0, lane);
          }
#pragma unroll
          for (int i = 0; i < FN; ++i)
#pragma unroll
            for (int j = 0; j < FM; ++j)
              acc[i][j] = mfma(fb[cb][i], fa[cb][j], acc[i][j]);
#pragma unroll
          for (int q = 0; q < FM + FN; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, (FM * FN) / (FM + FN), 0);  // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                      // DS read
          }
        } else {
          // With a transposed operand the fragment reads are inline assembly (see read_frag), which the
          // scheduler neither counts nor places, so the order is fixed by hand: the group's FN rows of
          // MFMAs, each preceded by its share of the next fragments.  In the last group of a K-step the
          // first row runs before the hand-over (it only needs registers), so the matrix pipe has
          // work while the wave sits at the barrier.
          constexpr bool last = kk + 1 == KK;
          // the refill of the drained stage is spread over the rows after the hand-over: a wave is held
          // for some 27 cycles per load instruction, which its own queued MFMAs then cover (-0.15 ms)
          constexpr bool GEMM_SPREAD_LOADS = true;
          constexpr int NF = FM + FN;                       // fragments to fetch: A 0..FM-1, then B
          constexpr int NCH = last ? FN - 1 : FN;           // chunks they are spread over
          const char* ra_ = last ? smem + ((t + 1 + par) & 1) * STAGE : ta;
          const char* rb_ = ra_ + A_BYTES;
          const bool do_reads = !last || t + 1 < total;
          static_for<0, FN>([&](auto i_c) {
            constexpr int i = decltype(i_c)::value;
            if (last && i == 1) {
              wait_vmcnt<0>();   // stage t+1 has landed (loads issued one K-step ago)
              asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
              __builtin_amdgcn_s_barrier();
              asm volatile("" ::: "memory");
              if (!GEMM_SPREAD_LOADS && loader) cur.issue_next(one, st_cur, wave, tl.m0, tl.n0, lane);   // step t+2 into the drained stage
            }
            if constexpr (GEMM_SPREAD_LOADS && last && i >= 1) {
              if (loader) cur.template issue_piece<i - 1, FN - 1>(one, st_cur, wave, tl.m0, tl.n0, lane);
            }
              const int ch = last ? i - 1 : i;
            if (ch >= 0 && do_reads) {
#pragma unroll
              for (int f = ch * NF / NCH; f < (ch + 1) * NF / NCH; ++f) {
                if (f < FM) fa[nb][f] = read_frag<BM, AK>(ra_, wave_m * TM + f * MI, last ? 0 : kk + 1, lane);
                else fb[nb][f - FM] = read_frag<BN, BKM>(rb_, wave_n * TN + (f - FM) * MI, last ? 0 : kk + 1, lane);
              }
            }
#pragma unroll
            for (int j = 0; j < FM; ++j) acc[i][j] = mfma(fb[cb][i], fa[cb][j], acc[i][j]);
            __builtin_amdgcn_sched_barrier(0);
          });
          // the fragments fetched above are complete once this wait has passed; the next group's MFMAs
          // depend on it
          wait_frags<FM, FN>(fa[nb], fb[nb]);
        }
      });
    }
    // Next tile.  Normally its cursor was opened and its first two K-steps sent during the last two
    // K-steps above; a tile of a single K-step sends them here (the last hand-over waited for every
    // load and passed a barrier after every wave's last LDS read: the whole ring is free).
    id += gridDim.x;
    const bool more = id < ntiles;
    par = (par + total) & 1;
    if (more && !early) {
      tl = locate(id);
      if (loader) {
        cur.issue_next(one, smem + par * STAGE, wave, tl.m0, tl.n0, lane);
        cur.issue_next(one, smem + (par ^ 1) * STAGE, wave, tl.m0, tl.n0, lane);
      }
    }

    // Epilogue through LDS (a region behind the ring): each wave owns a [TM/4][64] bf16 staging area
    // (128 bytes per row, chunk c of row m stored at c ^ ((m >> 1) & 7)), filled from the accumulator
    // layout (8 bytes per lane) and drained row-contiguously (16 bytes per lane, 8 lanes per row); a
    // wave's tile goes through it in 4 * TN/64 pieces.
    constexpr int HM = TM / 4, HF = FM / 4;
    char* stg = smem + NS * STAGE + wave * (HM * 128);
    const int lm = lane & (MI - 1), lq = lane / MI;
    const int rrow = lane >> 3, rpc = lane & 7;
    constexpr int TPB = 64 / MI;      // MFMA blocks per 64 staged columns
    constexpr int NG = NACC / 4;      // 4-column groups a lane holds per MFMA block
    // column (within the 64 staged ones) of group g of block i for this lane; jj: block row in the half
    auto stg_off = [&](int jj, int i, int g) {
      const int row = jj * MI + lm;
      const int n = i * MI + (MI == 32 ? g * 8 + lq * 4 : lq * 4);
      return row * 128 + ((((n >> 3) ^ ((row >> 1) & 7)) << 4) | ((n & 4) << 1));
    };
    if constexpr (EPI == EPI_SWIGLU_GRAD) {
      // In steps of one MFMA block row (MI rows x 64 columns per wave), which keeps the registers the
      // step needs next to the accumulators few: a whole row quarter at a time made the compiler
      // spill values the main loop uses.
      const int nbase = n0 + wave_n * TN;
      constexpr int NT = MI / 8;
      // block rows whose g and u are in flight ahead of the one being worked on.  Two or three ahead
      // measure the same (three spills registers of the main loop): all workgroups reach their
      // epilogues together, and what the reads then wait for is HBM bandwidth, not latency.
      constexpr int PF = 1;
      bf16x8 gv[PF + 1][NT], uv[PF + 1][NT];
      // g and u of block row s, 16 bytes per lane along rows (the layout of the drain below)
      auto fetch = [&](int s, bf16x8 (&g8)[NT], bf16x8 (&u8)[NT]) {
        const int mbase = m0 + wave_m * TM + s * MI;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int row = t * 8 + rrow;
          const int m = mbase + row;
          const int n = nbase + ((rpc ^ ((row >> 1) & 7)) << 3);
          const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
          g8[t] = zero;
          u8[t] = zero;
          if (m < p.M && n < p.N) {
            g8[t] = *reinterpret_cast<const bf16x8*>(one.e1 + (int64_t)m * one.lde + n);
            u8[t] = *reinterpret_cast<const bf16x8*>(one.e2 + (int64_t)m * one.lde + n);
          }
        }
      };
      // rows -> accumulator layout through the staging area
      auto to_acc_layout = [&](const bf16x8 (&v8)[NT], bf16x4 (&q)[TPB]) {
#pragma unroll
        for (int t = 0; t < NT; ++t) *reinterpret_cast<bf16x8*>(stg + (t * 8 + rrow) * 128 + (rpc << 4)) = v8[t];
#pragma unroll
        for (int i = 0; i < TPB; ++i) q[i] = *reinterpret_cast<const bf16x4*>(stg + stg_off(0, i, 0));
      };
      auto drain = [&](int s, const bf16x4 (&q)[TPB], bf16_t* dst) {
#pragma unroll
        for (int i = 0; i < TPB; ++i) *reinterpret_cast<bf16x4*>(stg + stg_off(0, i, 0)) = q[i];
        const int mbase = m0 + wave_m * TM + s * MI;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int row = t * 8 + rrow;
          const int m = mbase + row;
          const int n = nbase + ((rpc ^ ((row >> 1) & 7)) << 3);
          const bf16x8 v = *reinterpret_cast<const bf16x8*>(stg + row * 128 + (rpc << 4));
          if (m < p.M && n < p.N) *reinterpret_cast<bf16x8*>(dst + (int64_t)m * p.ldc + n) = v;
        }
      };
      static_for<0, PF>([&](auto s_c) {
        constexpr int s = decltype(s_c)::value;
        fetch(s, gv[s], uv[s]);
      });
      static_for<0, FM>([&](auto s_c) {
        constexpr int s = decltype(s_c)::value;
        bf16x4 gq[TPB], uq[TPB];
        to_acc_layout(gv[s % (PF + 1)], gq);
        to_acc_layout(uv[s % (PF + 1)], uq);
        // each fetch is issued before this row's stores, so waiting for it does not wait for the stores
        if constexpr (s + PF < FM) fetch(s + PF, gv[(s + PF) % (PF + 1)], uv[(s + PF) % (PF + 1)]);
#pragma unroll
        for (int i = 0; i < TPB; ++i)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float z = (float)gq[i][e], d = acc[i][s][e];
            const float sg = logistic(z);
            gq[i][e] = (bf16_t)(d * (float)uq[i][e] * sg * (1.0f + z * (1.0f - sg)));
            uq[i][e] = (bf16_t)(d * z * sg);
          }
        if (s == 0 && more) {
          if (tl.total >= 2) wait_vmcnt<LPW>(); else wait_vmcnt<0>();
        }
        drain(s, gq, p.c);
        drain(s, uq, one.c2);
      });
    } else if constexpr (SWIGLU) {
      // staged columns 0..31 are g, 32..63 are u, both for columns nh .. nh+31 of their matrices
      const int nh = n0 / 2 + wave_n * 32, NH = p.N / 2;
#pragma unroll
      for (int hf = 0; hf < 4; ++hf) {
        const int mbase = m0 + wave_m * TM + hf * HM;
#pragma unroll
        for (int jj = 0; jj < HF; ++jj)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16_t)acc[i][hf * HF + jj][e];
            *reinterpret_cast<bf16x4*>(stg + stg_off(jj, i, 0)) = o;
          }
        if (hf == 0 && more) {
          if (tl.total >= 2) wait_vmcnt<LPW>(); else wait_vmcnt<0>();
        }
#pragma unroll
        for (int t = 0; t < HM / 8; ++t) {
          const int row = t * 8 + rrow;
          const int m = mbase + row;
          const int cl = (rpc ^ ((row >> 1) & 7)) << 3;
          const int n = nh + (cl & 31);
          const bf16x8 v = *reinterpret_cast<const bf16x8*>(stg + row * 128 + (rpc << 4));
          bf16_t* dst = cl >= 32 ? one.c2 : p.c;
          if (m < p.M && n < NH) *reinterpret_cast<bf16x8*>(dst + (int64_t)m * p.ldc + n) = v;
        }
#pragma unroll
        for (int jj = 0; jj < HF; ++jj)
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float z = acc[i][hf * HF + jj][e];
              o[e] = (bf16_t)(z * logistic(z) * acc[i + 2][hf * HF + jj][e]);
            }
            *reinterpret_cast<bf16x4*>(stg + stg_off(jj, i, 0)) = o;
          }
#pragma unroll
        for (int t = 0; t < HM / 8; ++t) {
          const int row = t * 8 + rrow;
          const int m = mbase + row;
          const int cl = (rpc ^ ((row >> 1) & 7)) << 3;
          const int n = nh + cl;
          const bf16x8 v = *reinterpret_cast<const bf16x8*>(stg + row * 128 + (rpc << 4));
          if (cl < 32 && m < p.M && n < NH) *reinterpret_cast<bf16x8*>(one.c3 + (int64_t)m * one.ldc3 + n) = v;
        }
      }
    } else {
#pragma unroll
    for (int nb = 0; nb < TN / 64; ++nb) {
      const int nbase = n0 + wave_n * TN + nb * 64;
#pragma unroll
      for (int hf = 0; hf < 4; ++hf) {
        const int mbase = m0 + wave_m * TM + hf * HM;
        if (p.r || p.accumulate) {
          const bf16_t* src = p.r ? p.r : p.c;
#pragma unroll
          for (int t = 0; t < HM / 8; ++t) {
            const int row = t * 8 + rrow;
            const int m = mbase + row;
            const int n = nbase + ((rpc ^ ((row >> 1) & 7)) << 3);
            bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (m < p.M && n < p.N) v = *reinterpret_cast<const bf16x8*>(src + (int64_t)m * p.ldc + n);
            *reinterpret_cast<bf16x8*>(stg + row * 128 + (rpc << 4)) = v;
          }
#pragma unroll
          for (int jj = 0; jj < HF; ++jj)
#pragma unroll
            for (int i = 0; i < TPB; ++i)
#pragma unroll
              for (int g = 0; g < NG; ++g) {
                const bf16x4 v = *reinterpret_cast<const bf16x4*>(stg + stg_off(jj, i, g));
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[nb * TPB + i][hf * HF + jj][g * 4 + e] += (float)v[e];
              }
        }
        if constexpr (EPI == EPI_ROPE) {
          if (p.rope) {
            const int hd2 = grp.rope_dh >> 1;
#pragma unroll
            for (int jj = 0; jj < HF; ++jj) {
              const int j = hf * HF + jj;
              const int pos = (mbase + jj * MI + lm) % grp.rope_seq;
              const float* cr = grp.rope_cos + (int64_t)pos * hd2;
              const float* sr = grp.rope_sin + (int64_t)pos * hd2;
              if (grp.rope_layout == 0) {
                // block ib holds first-half features idx .. idx+3 of a head for this lane, block pb their partners
                const bool narrow = grp.rope_dh == 32;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                  const int idx = narrow ? lq * 4 : (PERM ? (wave_n & 1) * 32 : 0) + t * 16 + lq * 4;
                  const f32x4 c4 = *reinterpret_cast<const f32x4*>(cr + idx);
                  const f32x4 s4 = *reinterpret_cast<const f32x4*>(sr + idx);
                  auto rot = [&](acc_t& a, acc_t& b) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                      const float fa = a[e], fb = b[e];
                      a[e] = fa * c4[e] - fb * s4[e];
                      b[e] = fa * s4[e] + fb * c4[e];
                    }
                  };
                  if (narrow) rot(acc[2 * t][j], acc[2 * t + 1][j]);
                  else rot(acc[t][j], acc[t + 2][j]);
                }
              } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  const int idx = ((nbase + i * MI + lq * 4) % grp.rope_dh) >> 1;
                  const f32x2 c2 = *reinterpret_cast<const f32x2*>(cr + idx);
                  const f32x2 s2 = *reinterpret_cast<const f32x2*>(sr + idx);
#pragma unroll
                  for (int e = 0; e < 4; e += 2) {
                    const float fa = acc[i][j][e], fb = acc[i][j][e + 1];
                    acc[i][j][e] = fa * c2[e >> 1] - fb * s2[e >> 1];
                    acc[i][j][e + 1] = fa * s2[e >> 1] + fb * c2[e >> 1];
                  }
                }
              }
            }
          }
        }
#pragma unroll
        for (int jj = 0; jj < HF; ++jj)
#pragma unroll
          for (int i = 0; i < TPB; ++i)
#pragma unroll
            for (int g = 0; g < NG; ++g) {
              bf16x4 o;
#pragma unroll
              for (int e = 0; e < 4; ++e) o[e] = (bf16_t)acc[nb * TPB + i][hf * HF + jj][g * 4 + e];
              *reinterpret_cast<bf16x4*>(stg + stg_off(jj, i, g)) = o;
            }
        // Before this tile's first store: the next tile's K-step 0 must have landed, and waiting for
        // it here (nothing younger than K-step 1 is in flight) keeps the stores out of that wait, so
        // they complete under the next main loop.
        if (nb == 0 && hf == 0 && more) {
          if (tl.total >= 2) wait_vmcnt<LPW>(); else wait_vmcnt<0>();
        }
#pragma unroll
        for (int t = 0; t < HM / 8; ++t) {
          const int row = t * 8 + rrow;
          const int m = mbase + row;
          const int cl = (rpc ^ ((row >> 1) & 7)) << 3;   // column among the wave's 64
          // partner-order tiles: staged columns 0..31 are features (wave_n & 1) * 32 + .. of head wave_n / 2 of
          // the tile, columns 32..63 the same features 64 further on
          const int n = PERM ? n0 + (wave_n >> 1) * 128 + (wave_n & 1) * 32 + (cl & 31) + ((cl >> 5) << 6) : nbase + cl;
          const bf16x8 v = *reinterpret_cast<const bf16x8*>(stg + row * 128 + (rpc << 4));
          if (m < p.M && n < p.N) *reinterpret_cast<bf16x8*>(p.c + (int64_t)m * p.ldc + n) = v;
        }
      }
    }
    }
    if (!more) break;
  }
}

template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__global__ __launch_bounds__(WM* WN * 64) void gemm_kernel(const GemmKArgs p) {
  gemm_persistent<false, BM, BN, WM, WN, AK, BKM>(GemmGroupKArgs{}, p);
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM* WN * 64) void gemm_swiglu_kernel(const GemmKArgs p) {
  gemm_persistent<false, BM, BN, WM, WN, true, true, EPI>(GemmGroupKArgs{}, p);
}

template <int BM, int BN, int WM, int WN, bool AK, bool BKM>
__global__ __launch_bounds__(WM* WN * 64) void gemm_group_kernel(const GemmGroupKArgs g) {
  gemm_persistent<true, BM, BN, WM, WN, AK, BKM>(g, g.prob[0]);
}

template <int BM, int BN, int WM, int WN, bool PERM>
__global__ __launch_bounds__(WM* WN * 64, WM* WN == 4 ? 2 : 1) void gemm_group_rope_kernel(const GemmGroupKArgs g) {
  gemm_persistent<true, BM, BN, WM, WN, true, true, EPI_ROPE, PERM>(g, g.prob[0]);
}

// Tile rows per band of the tile sequence.  An XCD runs some 32 consecutive tiles at a time: 8 rows x 4
// columns of tiles with bands of 8, 4 x 8 with bands of 4 - twelve operand panels either way, but the
// wider arrangement touches longer runs of every C row (and of the g, u rows the activation-gradient
// epilogue reads).  Measured at the 8B shape, per launch: bands of 8 are 1-2.5 % faster for k-major
// products with K <= 4096 (q/k/v, o, gate/up forward, o input gradient), bands of 4 are 1-4 % faster for
// the long contractions (down projection, fused input gradients: +6-8 % at K = 8192), the
// activation-gradient epilogue and the weight gradients; bands of 2 or 16 lose everywhere.
static int band_rows_for(bool both_kmajor, int64_t k_total, bool epilogue_reads_tiles) {
  return both_kmajor && !epilogue_reads_tiles && k_total <= 4096 ? 8 : 4;
}

// As many workgroups as the LDS lets a CU hold at once (one for the 256 x 256 tile's 160 KB, two for
// the 128 x 128 tile's 72 KB, which then also gives every SIMD a second wave), fewer if there are fewer
// tiles.
static int persistent_grid(int ntiles, size_t lds) {
  static std::atomic<int> cu_count[64];   // per device; 0 = not asked yet
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return ntiles;
  int cus = cu_count[dev].load(std::memory_order_relaxed);
  if (cus == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return ntiles;
    cus = n > 0 ? n : 256;
    cu_count[dev].store(cus, std::memory_order_relaxed);
  }
  const int per_cu = lds * 2 <= 160 * 1024 ? 2 : 1;
  return ntiles < cus * per_cu ? ntiles : cus * per_cu;
}

template <int BM, int BN>
static size_t lds_bytes(int nwaves, int wm) {
  const size_t ring = (size_t)NS * (BM + BN) * BK * 2, staging = (size_t)nwaves * (BM / wm / 4) * 128;
  return ring + staging;
}

template <int BM, int BN, int WM, int WN>
static int launch_group_cfg(const GemmKArgs* ks, int n, bool ak, bool bk, const RopeEpilogue* rope, hipStream_t st) {
  GemmGroupKArgs g{};
  g.n = n;
  for (int i = 0; i < n; ++i) {
    g.prob[i] = ks[i];
    g.prob[i].tiles_m = (ks[i].M + BM - 1) / BM;
    g.prob[i].band_rows = band_rows_for(ak && bk, ks[i].K[0], false);
    g.prob[i].tiles_n = (ks[i].N + BN - 1) / BN;
    g.tile_start[i + 1] = g.tile_start[i] + g.prob[i].tiles_m * g.prob[i].tiles_n;
  }
  const size_t lds = lds_bytes<BM, BN>(WM * WN, WM);
  const dim3 grid((unsigned)persistent_grid(g.tile_start[n], lds)), block(WM * WN * 64);
  if (rope) {
    g.rope_cos = rope->cos; g.rope_sin = rope->sin;
    g.rope_seq = rope->seq; g.rope_dh = rope->head_dim; g.rope_layout = rope->layout;
    for (int i = 0; i < n; ++i) g.prob[i].rope = (rope->rotate_mask >> i) & 1;
#define GEMM_ROPE_LAUNCH(PERM_)                                                                  \
  do {                                                                                           \
    auto kern = gemm_group_rope_kernel<BM, BN, WM, WN, PERM_>;                                   \
    static std::atomic<unsigned long long> lds_done{0};                                          \
    if (int rc_ = reserve_lds(kern, lds, lds_done, "gemm rope")) return rc_;                     \
    hipLaunchKernelGGL(kern, grid, block, lds, st, g);                                           \
  } while (0)
    if (rope->layout == 0 && rope->head_dim == 128) GEMM_ROPE_LAUNCH(true);
    else GEMM_ROPE_LAUNCH(false);
#undef GEMM_ROPE_LAUNCH
    return check_launch("gemm group (rotary epilogue)");
  }
#define GEMM_GROUP_LAUNCH(AK_, BK_)                                                              \
  do {                                                                                           \
    auto kern = gemm_group_kernel<BM, BN, WM, WN, AK_, BK_>;                                     \
    static std::atomic<unsigned long long> lds_done{0};                                                      \
    if (int rc_ = reserve_lds(kern, lds, lds_done, "gemm")) return rc_;                          \
    hipLaunchKernelGGL(kern, grid, block, lds, st, g);                                           \
  } while (0)
  // only the layouts in use are instantiated: the weight-gradient products (both operands mn-major)
  // and the forward projections (both k-major)
  if (!ak && !bk) GEMM_GROUP_LAUNCH(false, false);
  else if (ak && bk) GEMM_GROUP_LAUNCH(true, true);
  else return fail(-1, "gemm group: operand layout not built");
#undef GEMM_GROUP_LAUNCH
  return check_launch("gemm group");
}

template <int BM, int BN, int WM, int WN>
static int launch_cfg(const GemmKArgs& k, bool ak, bool bk, hipStream_t st) {
  GemmKArgs a = k;
  a.tiles_m = (k.M + BM - 1) / BM;
  int64_t k_total = 0;
  for (int s = 0; s < k.nseg; ++s) k_total += k.K[s];
  a.band_rows = band_rows_for(ak && bk, k_total, false);
  a.tiles_n = (k.N + BN - 1) / BN;
  const size_t lds = lds_bytes<BM, BN>(WM * WN, WM);
  const dim3 grid((unsigned)persistent_grid(a.tiles_m * a.tiles_n, lds)), block(WM * WN * 64);
#define GEMM_LAUNCH(AK_, BK_)                                                                    \
  do {                                                                                           \
    auto kern = gemm_kernel<BM, BN, WM, WN, AK_, BK_>;                                           \
    static std::atomic<unsigned long long> lds_done{0};                                                      \
    if (int rc_ = reserve_lds(kern, lds, lds_done, "gemm")) return rc_;                          \
    hipLaunchKernelGGL(kern, grid, block, lds, st, a);                                           \
  } while (0)
  if (ak && bk) GEMM_LAUNCH(true, true);
  else if (ak && !bk) GEMM_LAUNCH(true, false);
  else if (!ak && bk) GEMM_LAUNCH(false, true);
  else GEMM_LAUNCH(false, false);
#undef GEMM_LAUNCH
  return check_launch("gemm");
}

static GemmKArgs kernel_args(const GemmArgs& g) {
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
  return k;
}

int launch_gemm(const GemmArgs& g, hipStream_t st) {
  const GemmKArgs k = kernel_args(g);
  // Large problems: 256x256 tiles, 8 waves (2 per SIMD), 128x64 per wave.  Small ones: 128x128
  // tiles so that the grid still covers the 256 CUs.
  const int64_t tiles256 = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256);
  if (tiles256 >= 192) return launch_cfg<256, 256, 2, 4>(k, g.a_kmajor, g.b_kmajor, st);
  return launch_cfg<128, 128, 2, 2>(k, g.a_kmajor, g.b_kmajor, st);
}

bool gemm_swiglu_applies(int64_t T, int64_t F) {
  return F % 8 == 0 && ((T + 255) / 256) * ((2 * F + 255) / 256) >= 192;
}
bool gemm_swiglu_grad_applies(int64_t T, int64_t F) {
  return F % 8 == 0 && ((T + 255) / 256) * ((F + 255) / 256) >= 192;
}

template <int EPI>
static int launch_fused(GemmKArgs k, const char* what, hipStream_t st) {
  constexpr int BM = 256, BN = 256, WM = 2, WN = 4;
  k.nseg = 1;
  k.tiles_m = (k.M + BM - 1) / BM;
  k.band_rows = band_rows_for(true, k.K[0], EPI == EPI_SWIGLU_GRAD);
  k.tiles_n = (k.N + BN - 1) / BN;
  const size_t lds = lds_bytes<BM, BN>(WM * WN, WM);
  const dim3 grid((unsigned)persistent_grid(k.tiles_m * k.tiles_n, lds)), block(WM * WN * 64);
  auto kern = gemm_swiglu_kernel<BM, BN, WM, WN, EPI>;
  static std::atomic<unsigned long long> lds_done{0};
  if (int rc = reserve_lds(kern, lds, lds_done, what)) return rc;
  hipLaunchKernelGGL(kern, grid, block, lds, st, k);
  return check_launch(what);
}

int launch_gemm_swiglu(const void* x, int64_t ldx, const void* wg, const void* wu, int64_t ldw, int64_t T, int64_t K,
                       int64_t F, void* g, void* u, int64_t ldgu, void* a, int64_t lda, hipStream_t st) {
  if (!gemm_swiglu_applies(T, F)) return fail(-1, "gemm swiglu: shape T=%lld F=%lld not served by the fused kernel", (long long)T, (long long)F);
  GemmKArgs k{};
  k.a[0] = (const bf16_t*)x;
  k.b[0] = (const bf16_t*)wg;
  k.b2 = (const bf16_t*)wu;
  k.lda[0] = ldx;
  k.ldb[0] = ldw;
  k.K[0] = (int)K;
  k.M = (int)T;
  k.N = (int)(2 * F);
  k.c = (bf16_t*)g;
  k.c2 = (bf16_t*)u;
  k.ldc = ldgu;
  k.c3 = (bf16_t*)a;
  k.ldc3 = lda;
  return launch_fused<EPI_SWIGLU>(k, "gemm swiglu", st);
}

int launch_gemm_swiglu_grad(const void* dy, int64_t lddy, const void* wt, int64_t ldw, int64_t T, int64_t K, int64_t F,
                            const void* g, const void* u, int64_t ldgu, void* dg, void* du, int64_t ldd,
                            hipStream_t st) {
  if (!gemm_swiglu_grad_applies(T, F)) return fail(-1, "gemm swiglu grad: shape T=%lld F=%lld not served by the fused kernel", (long long)T, (long long)F);
  GemmKArgs k{};
  k.a[0] = (const bf16_t*)dy;
  k.b[0] = (const bf16_t*)wt;
  k.lda[0] = lddy;
  k.ldb[0] = ldw;
  k.K[0] = (int)K;
  k.M = (int)T;
  k.N = (int)F;
  k.c = (bf16_t*)dg;
  k.c2 = (bf16_t*)du;
  k.ldc = ldd;
  k.e1 = (const bf16_t*)g;
  k.e2 = (const bf16_t*)u;
  k.lde = ldgu;
  return launch_fused<EPI_SWIGLU_GRAD>(k, "gemm swiglu grad", st);
}

int launch_gemm_group(const GemmArgs* gs, int n, hipStream_t st) { return launch_gemm_group_rope(gs, n, nullptr, st); }

int launch_gemm_group_rope(const GemmArgs* gs, int n, const RopeEpilogue* rope, hipStream_t st) {
  if (n < 1 || n > MAX_GROUP) return fail(-1, "gemm group: 1..%d problems, got %d", MAX_GROUP, n);
  GemmKArgs ks[MAX_GROUP];
  int64_t tiles256 = 0;
  for (int i = 0; i < n; ++i) {
    if (gs[i].a_kmajor != gs[0].a_kmajor || gs[i].b_kmajor != gs[0].b_kmajor)
      return fail(-1, "gemm group: all problems must share one operand layout");
    if (gs[i].nseg != 1) return fail(-1, "gemm group: problems must have a single K-segment");
    ks[i] = kernel_args(gs[i]);
    tiles256 += (int64_t)((gs[i].M + 255) / 256) * ((gs[i].N + 255) / 256);
  }
  if (rope) {
    if (!gs[0].a_kmajor || !gs[0].b_kmajor) return fail(-1, "gemm group: the rotary epilogue needs k-major operands");
    if (rope->head_dim != 32 && rope->head_dim != 64 && rope->head_dim != 128) return fail(-1, "gemm group: head_dim %d", rope->head_dim);
    for (int i = 0; i < n; ++i)
      if (gs[i].r || gs[i].accumulate || gs[i].N % rope->head_dim || gs[i].ldc % 8)
        return fail(-1, "gemm group: rotary epilogue on a product with residual, accumulation or partial heads");
  }
  if (tiles256 >= 192) return launch_group_cfg<256, 256, 2, 4>(ks, n, gs[0].a_kmajor, gs[0].b_kmajor, rope, st);
  return launch_group_cfg<128, 128, 2, 2>(ks, n, gs[0].a_kmajor, gs[0].b_kmajor, rope, st);
}

}  // namespace dl
