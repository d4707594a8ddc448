// Causal softmax attention with grouped KV heads for gfx950: forward and backward, blockwise
// ("flash") so that no S x S matrix is ever stored.  q, o [B*S, Hq, DH]; k, v [B*S, Hkv, DH].
//
// All products run on v_mfma_f32_32x32x16_bf16 and are arranged so that the score tile comes out
// of the MFMA already in the register layout the next product consumes (no LDS round trip for
// P or dS):
//   forward / dQ kernel : S^T[kv][q] = K Q^T   -> lane owns one query column, keys along registers
//                         O^T[d][q] += V^T P^T,  dQ^T[d][q] += K^T dS^T
//   dK/dV kernel        : S[q][kv]  = Q K^T    -> lane owns one key column, queries along registers
//                         dV^T[d][kv] += dO^T P,  dK^T[d][kv] += Q^T dS
// Row statistics (max, sum, LSE, delta) then live one per lane in the first pair of kernels, and
// the row reductions are an in-lane loop plus one exchange between lane l and lane l^32.
// The "transposed" operands (V^T, K^T, dO^T, Q^T) are read from row-major LDS tiles with
// ds_read_b64_tr_b16.  K/V (or Q/dO) tiles stream global -> LDS with buffer_load ... lds,
// double buffered.
//
// An MFMA sums over its 16 k-slots in any order, so the slot -> key assignment is chosen to match
// the accumulator layout of the score tile: for a 16-key step, slot (half = lane / 32, e = 0..7)
// holds key 8*(e/4) + 4*half + e%4.  The transposed loads of the other operand use the same map.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace dl {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// v_exp_f32: 2^x without the denormal-range fix-up (results below 2^-126 flush to zero, which is
// what a softmax weight that small should be anyway).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ __amdgpu_buffer_rsrc_t attn_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// [ROWS][DH] bf16 tile in LDS, DH*2 bytes per row, 16-byte chunk c of row r stored at chunk
// c ^ swz(r).  Loaded by NW waves with 1 KiB wave-wide async loads.  swz is chosen so that both
// access patterns are free of bank conflicts (the LDS serves 256 B of banks per clock):
//   row reads  (ds_read_b128, 16 lanes = 16 consecutive rows, one logical chunk), and
//   transposed reads (ds_read_b64_tr_b16, 32 lanes = 4 consecutive rows x 64 B).
template <int ROWS, int DH, int NW>
struct RowTile {
  static constexpr int ROW_B = DH * 2;
  static constexpr int LPR = DH / 8;          // lanes (16 B chunks) per row
  static constexpr int RPI = 1024 / ROW_B;    // rows per wave-wide load
  static constexpr int NINSTR = ROWS / RPI;
  static constexpr int PER_WAVE = NINSTR / NW;
  static __device__ __forceinline__ int swz(int row) {
    if constexpr (LPR == 16) { const int i = row & 15; return ((i & 3) << 2) | (i >> 2); }
    else if constexpr (LPR == 8) { const int i = (row >> 1) & 7; return ((i & 1) << 2) | (i >> 1); }
    else { return (row >> 2) & 3; }
  }
  static_assert(NINSTR % NW == 0 && ((ROWS / NW) % 16) == 0, "tile split");
  static constexpr int BYTES = ROWS * ROW_B;

  // rs describes memory starting at the tile's first row; ld = row stride in elements.
  // AUX: cache-policy bits of the load (0 = default, 2 = non-temporal)
  template <int AUX = 0>
  static __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rs, char* lds_tile, int wave,
                                               int lane, int64_t ld) {
    const int r = lane / LPR, pc = lane % LPR;
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
      const int j = wave * PER_WAVE + i;
      const int c = pc ^ swz(i * RPI + r);   // rows per wave are a multiple of 16
      const uint32_t vo = (uint32_t)(r * ld * 2 + (c << 4));
      const uint32_t so = (uint32_t)((int64_t)j * RPI * ld * 2);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (LDS_PTR(void))(lds_tile + j * 1024), 16, vo, so, 0, AUX);
    }
  }
  // MFMA operand for rows row0 + lane%32, contraction over the DH index, step kk (16 of DH).
  static __device__ __forceinline__ bf16x8 frag_rows(const char* t, int row0, int kk, int lane) {
    const int row = row0 + (lane & 31);
    const int c = (kk * 2 + (lane >> 5)) ^ swz(row);
    return *reinterpret_cast<const bf16x8*>(t + row * ROW_B + (c << 4));
  }
  // MFMA operand for "rows" = 32 columns of the tile starting at col0 (the DH index), contraction
  // over 16 tile rows starting at krow0, with the slot -> row map described at the top of the file.
  static __device__ __forceinline__ bf16x8 frag_cols(const char* t, int col0, int krow0, int lane) {
    const int grp = lane >> 4, s = lane & 15, e = s >> 2, g = s & 3;
    const int col = col0 + ((grp & 1) << 4) + (g << 2);
    const int row = krow0 + ((grp >> 1) << 2) + e;
    const char* p0 = t + row * ROW_B + ((((col >> 3) ^ swz(row)) << 4) | ((col & 7) << 1));
    const int row2 = row + 8;
    const char* p1 = t + row2 * ROW_B + ((((col >> 3) ^ swz(row2)) << 4) | ((col & 7) << 1));
    bf16x8 v;
    v.lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(p0));
    v.hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((LDS_PTR(bf16x4))(p1));
    return v;
  }
};

__device__ __forceinline__ bf16x8 pack_slots(const f32x16& a, int first) {
  bf16x8 v;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (bf16_t)a[first + e];
  return v;
}


// Value exchange between lane l and lane l ^ 32 without the LDS round trip of a bpermute: after the swap
// `a` holds the low half's values in both halves and `b` the high half's.
__device__ __forceinline__ float max_across_halves(float x) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return __builtin_fmaxf(a, b);
}
__device__ __forceinline__ float sum_across_halves(float x) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return a + b;
}
// max of three as one instruction, without the canonicalising self-maximum the compiler puts in front of
// fmaxf operands (scores are finite or -inf here, never NaN)
__device__ __forceinline__ float max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
}

// Causal mask for a score tile held in the "lane owns one query (or key) column" accumulator
// layout: register r of 32-row block i holds row i*32 + 8*(r/4) + 4*(lane/32) + r%4.  `lim` is the
// largest row offset this lane may keep (computed by the caller with the 4*(lane/32) folded in);
// rows above it get `fill`.  The empty volatile asm keeps the compiler from turning the caller's
// wave-uniform `if (diagonal tile)` into per-element selects executed on every tile.
template <int NBLK>
__device__ __forceinline__ void mask_rows_above(f32x16 (&s)[NBLK], int lim, float fill) {
  asm volatile("" ::: "memory");
#pragma unroll
  for (int i = 0; i < NBLK; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (i * 32 + ((r >> 2) << 3) + (r & 3) > lim) s[i][r] = fill;
}

// ------------------------------------------------------------------------------------------
// Workgroup -> work mapping shared by all kernels here.  Consecutive workgroup ids are dealt to the
// eight XCDs in turn and every XCD has an L2 of its own, so all work on one (batch, kv head) pair is
// given to ONE XCD (ids congruent mod 8) when the number of pairs is a multiple of 8: the K/V tiles
// (forward, dQ) or Q/dO tiles (dK, dV) of that pair are then fetched into one L2 only, and the
// workgroups that share them run side by side and walk them in the same order.  `j` counts the
// position in the pair's own queue (heaviest first is the caller's business).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void split_block_id(int id, int npairs, int& j, int& pair) {
  int per_xcd = npairs, xcd = 0, slot = id;
  if ((npairs & 7) == 0) { per_xcd = npairs >> 3; xcd = id & 7; slot = id >> 3; }
  j = slot / per_xcd;
  pair = xcd * per_xcd + slot % per_xcd;
}

// ------------------------------------------------------------------------------------------
// Forward.  Workgroup = 4 waves = 128 query rows of one (batch, query head); wave = 32 rows.
// The softmax is VALU-bound next to the MFMA work, so the per-tile VALU count is kept minimal:
// the 1/sqrt(dh)*log2(e) scale is folded into the exp2 argument with one FMA, the causal mask runs
// only on diagonal tiles, and the running maximum is only raised (and O and the row sum rescaled)
// when some row's maximum grew by more than 2^8 - P then stays below 256, well inside bf16, and
// the final O / rowsum is unchanged because both carry the same stale reference.
// ------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, 2) void attn_fwd_kernel(const bf16_t* __restrict__ q,
                                                          const bf16_t* __restrict__ k,
                                                          const bf16_t* __restrict__ v,
                                                          bf16_t* __restrict__ o, float* __restrict__ lse,
                                                          int B, int S, int Hq, int Hkv, float scale_log2) {
  using Tile = RowTile<64, DH, 4>;
  constexpr int STAGE = 2 * Tile::BYTES;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int j, pair;
  split_block_id((int)blockIdx.x, B * Hkv, j, pair);
  const int G = Hq / Hkv, b = pair / Hkv, hk = pair % Hkv;
  const int qt = S / 128 - 1 - j / G, h = hk * G + j % G;   // long rows (late query tiles) first
  const int q0 = qt * 128, qw = q0 + wave * 32;
  const int lq = lane & 31, half = lane >> 5;
  const int64_t ldq = (int64_t)Hq * DH, ldk = (int64_t)Hkv * DH;

  bf16x8 qf[DH / 16];
  {
    const bf16_t* qp = q + ((int64_t)b * S + qw + lq) * ldq + (int64_t)h * DH + half * 8;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qp + kk * 16);
  }
  f32x16 oacc[DH / 32];
#pragma unroll
  for (int t = 0; t < DH / 32; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[t][e] = 0.f;
  float m = -INFINITY, lsum = 0.f;   // m: reference exponent in scaled log2 units

  const bf16_t* kb = k + (int64_t)b * S * ldk + (int64_t)hk * DH;
  const bf16_t* vb = v + (int64_t)b * S * ldk + (int64_t)hk * DH;
  const uint32_t kv_bytes = (uint32_t)((((int64_t)S - 1) * ldk + DH) * 2);
  const int nkv = (q0 + 128) / 64;
  // One buffer descriptor per tile: base at the tile's first key row, range to the end of this
  // batch row's keys (rows past it would read as zero).
  auto issue_tile = [&](int t, int stage) {
    const uint32_t skip = (uint32_t)((int64_t)t * 64 * ldk * 2);
    Tile::issue(attn_rsrc(kb + (int64_t)t * 64 * ldk, kv_bytes - skip), smem + stage * STAGE, wave, lane, ldk);
    Tile::issue(attn_rsrc(vb + (int64_t)t * 64 * ldk, kv_bytes - skip), smem + stage * STAGE + Tile::BYTES, wave, lane, ldk);
  };

  issue_tile(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int stage = 0;
  for (int t = 0; t < nkv; ++t) {
    if (t + 1 < nkv) issue_tile(t + 1, stage ^ 1);
    const int kv0 = t * 64;
    const char* tk = smem + stage * STAGE;
    const char* tv = tk + Tile::BYTES;
    f32x16 s[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) s[i][e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk)
#pragma unroll
      for (int i = 0; i < 2; ++i)
        s[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(tk, i * 32, kk, lane), qf[kk], s[i], 0, 0, 0);
    // keys after the query (only on tiles that reach past this wave's first row; a tile that lies
    // entirely after the wave's rows is masked out completely and contributes exact zeros)
    if (kv0 + 63 > qw) mask_rows_above<2>(s, qw + lq - kv0 - (half << 2), -INFINITY);
    float mx = s[0][0];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[i][r]);
    mx = max_across_halves(mx) * scale_log2;
    if (__builtin_amdgcn_ballot_w64(mx > m + 8.0f) != 0) {
      const float m_new = fmaxf(m, mx);
      const float alpha = fast_exp2(m - m_new);
      lsum *= alpha;
      m = m_new;
#pragma unroll
      for (int t2 = 0; t2 < DH / 32; ++t2)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[t2][e] *= alpha;
    }
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pv = fast_exp2(__builtin_fmaf(s[i][r], scale_log2, -m));
        s[i][r] = pv;
        psum += pv;
      }
    lsum += psum;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const bf16x8 pf = pack_slots(s[ks >> 1], (ks & 1) * 8);
#pragma unroll
      for (int t2 = 0; t2 < DH / 32; ++t2)
        oacc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(tv, t2 * 32, ks * 16, lane), pf, oacc[t2], 0, 0, 0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    stage ^= 1;
  }
  lsum = sum_across_halves(lsum);
  const float inv = 1.0f / lsum;
  bf16_t* op = o + ((int64_t)b * S + qw + lq) * ldq + (int64_t)h * DH + half * 4;
#pragma unroll
  for (int t2 = 0; t2 < DH / 32; ++t2)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 ov;
#pragma unroll
      for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(oacc[t2][g * 4 + e] * inv);
      *reinterpret_cast<bf16x4*>(op + t2 * 32 + g * 8) = ov;
    }
  if (half == 0) lse[((int64_t)b * Hq + h) * S + qw + lq] = (m + log2f(lsum)) * kLn2;
}

// ------------------------------------------------------------------------------------------
// delta[b, h, q] = -sum_d dO[q, h, d] * O[q, h, d] (negated: the dQ and dK kernels start their dP
// accumulators from it, so dP - rowsum(dO * O) needs no subtraction), and lse2 = lse * log2(e) (the exponent reference
// in the units the backward kernels' exp2 works in), both [B, Hq, S] fp32.
// ------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void attn_delta_kernel(const bf16_t* __restrict__ o,
                                                         const bf16_t* __restrict__ d_o,
                                                         const float* __restrict__ lse,
                                                         float* __restrict__ delta, float* __restrict__ lse2,
                                                         int64_t rows, int S, int Hq) {
  constexpr int LPR = DH / 8;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = idx / LPR;  // row = (b*S + q)*Hq + h
  float acc = 0.f;
  if (row < rows) {
    const bf16x8 a = reinterpret_cast<const bf16x8*>(o)[idx], d = reinterpret_cast<const bf16x8*>(d_o)[idx];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)d[e];
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (row < rows && (idx % LPR) == 0) {
    const int64_t tok = row / Hq;
    const int h = (int)(row % Hq);
    const int64_t b = tok / S, qi = tok % S;
    delta[(b * Hq + h) * S + qi] = -acc;   // stored negated: the backward products start their dP sums from it
    lse2[(b * Hq + h) * S + qi] = lse[(b * Hq + h) * S + qi] * kLog2e;
  }
}

// Rotary embedding backward on an accumulator tile held as "lane owns one token, features along
// registers" (register g*4+e of block t2 = feature t2*32 + g*8 + 4*half + e): the gradient of a rotation
// by angle phi is the rotation by -phi.  cr, sr: this token's cos / sin row ([DH/2] fp32).  Both
// members of a pair sit in the same lane for either pairing.
template <int DH>
__device__ __forceinline__ void rope_unrotate(f32x16 (&acc)[DH / 32], const float* cr, const float* sr, int layout,
                                              int half) {
  if (layout == 0) {
    constexpr int NT2 = DH >= 64 ? DH / 64 : 1, NG = DH >= 64 ? 4 : 2;
#pragma unroll
    for (int t2 = 0; t2 < NT2; ++t2)
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const int t2p = DH >= 64 ? t2 + DH / 64 : 0, gp = DH >= 64 ? g : g + 2;
        const int idx = t2 * 32 + g * 8 + half * 4;
        const f32x4 c4 = *reinterpret_cast<const f32x4*>(cr + idx), s4 = *reinterpret_cast<const f32x4*>(sr + idx);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float a = acc[t2][g * 4 + e], b = acc[t2p][gp * 4 + e];
          acc[t2][g * 4 + e] = a * c4[e] + b * s4[e];
          acc[t2p][gp * 4 + e] = b * c4[e] - a * s4[e];
        }
      }
  } else {
#pragma unroll
    for (int t2 = 0; t2 < DH / 32; ++t2)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int idx = (t2 * 32 + g * 8 + half * 4) >> 1;
        const f32x2 c2 = *reinterpret_cast<const f32x2*>(cr + idx), s2 = *reinterpret_cast<const f32x2*>(sr + idx);
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
          const float a = acc[t2][g * 4 + e], b = acc[t2][g * 4 + e + 1];
          acc[t2][g * 4 + e] = a * c2[e >> 1] + b * s2[e >> 1];
          acc[t2][g * 4 + e + 1] = b * c2[e >> 1] - a * s2[e >> 1];
        }
      }
  }
}

// ------------------------------------------------------------------------------------------
// dQ.  Same decomposition as the forward: workgroup = 128 query rows of one (batch, head).
// ------------------------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ d_o, const float* __restrict__ lse, const float* __restrict__ delta,
    bf16_t* __restrict__ dq, int B, int S, int Hq, int Hkv, float scale, const float* __restrict__ rope_cos,
    const float* __restrict__ rope_sin, int rope_layout) {
  using Tile = RowTile<64, DH, 4>;
  constexpr int STAGE = 2 * Tile::BYTES;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int j, pair;
  split_block_id((int)blockIdx.x, B * Hkv, j, pair);
  const int G = Hq / Hkv, b = pair / Hkv, hk = pair % Hkv;
  const int qt = S / 128 - 1 - j / G, h = hk * G + j % G;   // long rows (late query tiles) first
  const int q0 = qt * 128, qw = q0 + wave * 32;
  const int lq = lane & 31, half = lane >> 5;
  const int64_t ldq = (int64_t)Hq * DH, ldk = (int64_t)Hkv * DH;
  const float scale_log2 = scale * kLog2e;

  bf16x8 qf[DH / 16], dof[DH / 16];
  {
    const int64_t off = ((int64_t)b * S + qw + lq) * ldq + (int64_t)h * DH + half * 8;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) {
      qf[kk] = *reinterpret_cast<const bf16x8*>(q + off + kk * 16);
      dof[kk] = *reinterpret_cast<const bf16x8*>(d_o + off + kk * 16);
    }
  }
  const int64_t stat = ((int64_t)b * Hq + h) * S + qw + lq;
  const float lse2 = lse[stat] * kLog2e;
  // dP - delta comes out of the product itself: the dP accumulator starts from -delta (this lane's query)
  f32x16 neg_delta;
  {
    const float nd = delta[stat];
#pragma unroll
    for (int e = 0; e < 16; ++e) neg_delta[e] = nd;
  }
  f32x16 acc[DH / 32];
#pragma unroll
  for (int t = 0; t < DH / 32; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  const bf16_t* kb = k + (int64_t)b * S * ldk + (int64_t)hk * DH;
  const bf16_t* vb = v + (int64_t)b * S * ldk + (int64_t)hk * DH;
  const uint32_t kv_bytes = (uint32_t)((((int64_t)S - 1) * ldk + DH) * 2);
  const int nkv = (q0 + 128) / 64;
  auto issue_tile = [&](int t, int stage) {
    const uint32_t skip = (uint32_t)((int64_t)t * 64 * ldk * 2);
    Tile::issue(attn_rsrc(kb + (int64_t)t * 64 * ldk, kv_bytes - skip), smem + stage * STAGE, wave, lane, ldk);
    Tile::issue(attn_rsrc(vb + (int64_t)t * 64 * ldk, kv_bytes - skip), smem + stage * STAGE + Tile::BYTES, wave, lane, ldk);
  };
  issue_tile(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int stage = 0;
  for (int t = 0; t < nkv; ++t) {
    if (t + 1 < nkv) issue_tile(t + 1, stage ^ 1);
    const int kv0 = t * 64;
    const char* tk = smem + stage * STAGE;
    const char* tv = tk + Tile::BYTES;
    // two 32-key halves per tile: keeps the live score registers at 32 so two waves fit per SIMD
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      f32x16 s[1], dp = neg_delta;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[0][e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < DH / 16; ++kk) {
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(tk, i * 32, kk, lane), qf[kk], s[0], 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(tv, i * 32, kk, lane), dof[kk], dp, 0, 0, 0);
      }
      // P^T = exp2(s*c - lse); keys after the query get exp2(-inf) = 0
      if (kv0 + i * 32 + 31 > qw) mask_rows_above<1>(s, qw + lq - kv0 - i * 32 - (half << 2), -INFINITY);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pv = fast_exp2(__builtin_fmaf(s[0][r], scale_log2, -lse2));
        s[0][r] = pv * dp[r];  // dS^T = P^T (dP^T - delta)
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const bf16x8 df = pack_slots(s[0], ks * 8);
#pragma unroll
        for (int t2 = 0; t2 < DH / 32; ++t2)
          acc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(tk, t2 * 32, i * 32 + ks * 16, lane), df, acc[t2], 0, 0, 0);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    stage ^= 1;
  }
  // q was rotated after its projection: hand back the gradient of the unrotated q
  if (rope_cos) rope_unrotate<DH>(acc, rope_cos + (int64_t)(qw + lq) * (DH / 2), rope_sin + (int64_t)(qw + lq) * (DH / 2), rope_layout, half);
  bf16_t* op = dq + ((int64_t)b * S + qw + lq) * ldq + (int64_t)h * DH + half * 4;
#pragma unroll
  for (int t2 = 0; t2 < DH / 32; ++t2)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 ov;
#pragma unroll
      for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(acc[t2][g * 4 + e] * scale);
      *reinterpret_cast<bf16x4*>(op + t2 * 32 + g * 8) = ov;
    }
}

// ------------------------------------------------------------------------------------------
// dK or dV (template flag), the two-launch form kept for head dim 32 (whose 32-row tiles are too small to
// split over four loading waves in attn_bwd_dkdv_kernel).  Workgroup = 4 waves = 128 keys of one (batch,
// kv head); wave = 32 keys.  Streams the Q and dO tiles (64 query rows) of every query head of the group,
// from the last query tile back to the diagonal: dV takes the S and dV^T products, dK the S, dP and dK^T
// products.
// ------------------------------------------------------------------------------------------
template <int DH, bool WANT_DV>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ d_o, const float* __restrict__ lse2, const float* __restrict__ delta,
    bf16_t* __restrict__ dout, int B, int S, int Hq, int Hkv, float scale, const float* __restrict__ rope_cos,
    const float* __restrict__ rope_sin, int rope_layout) {
  using Tile = RowTile<64, DH, 4>;
  constexpr int STAGE = 2 * Tile::BYTES + 512;  // Q tile, dO tile, lse[64], delta[64]
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int kt, pair;   // low key tiles have the most query tiles: first
  split_block_id((int)blockIdx.x, B * Hkv, kt, pair);
  const int G = Hq / Hkv, b = pair / Hkv, hk = pair % Hkv;
  const int kv0 = kt * 128, kvw = kv0 + wave * 32;
  const int lk = lane & 31, half = lane >> 5;
  const int64_t ldq = (int64_t)Hq * DH, ldk = (int64_t)Hkv * DH;
  const float scale_log2 = scale * kLog2e;

  bf16x8 kf[DH / 16], vf[WANT_DV ? 1 : DH / 16];
  {
    const int64_t off = ((int64_t)b * S + kvw + lk) * ldk + (int64_t)hk * DH + half * 8;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) {
      kf[kk] = *reinterpret_cast<const bf16x8*>(k + off + kk * 16);
      if constexpr (!WANT_DV) vf[kk] = *reinterpret_cast<const bf16x8*>(v + off + kk * 16);
    }
  }
  f32x16 acc[DH / 32];
#pragma unroll
  for (int t = 0; t < DH / 32; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  const int first_qt = kv0 / 64, nq = S / 64 - first_qt, niter = G * nq;
  const uint32_t q_bytes = (uint32_t)((((int64_t)S - 1) * ldq + DH) * 2);
  // (query tile, head) of the tile to load next and of the tile being processed, advanced without
  // divisions.  Every workgroup walks the query tiles from the LAST one down to its diagonal, all G
  // heads of a tile in turn: workgroups of one pair that start together then read the same Q/dO
  // tile at the same time, whatever their key tile, and share it in the L2.
  int ld_g = 0, ld_qt = S / 64 - 1, cur_g = 0, cur_qt = S / 64 - 1;
  auto issue_tile = [&](int stage) {
    const int h = hk * G + ld_g, qrow = ld_qt * 64;
    if (++ld_g == G) { ld_g = 0; --ld_qt; }
    const int64_t base = ((int64_t)b * S) * ldq + (int64_t)h * DH;
    const uint32_t skip = (uint32_t)((int64_t)qrow * ldq * 2);
    char* st = smem + stage * STAGE;
    Tile::issue(attn_rsrc(q + base + (int64_t)qrow * ldq, q_bytes - skip), st, wave, lane, ldq);
    Tile::issue(attn_rsrc(d_o + base + (int64_t)qrow * ldq, q_bytes - skip), st + Tile::BYTES, wave, lane, ldq);
    // the 64 lse2 (and delta) values of the tile take the same asynchronous global -> LDS path, 4 bytes
    // per lane: a register round trip here would make the wave wait for the tile loads as well
    const int64_t sidx = ((int64_t)b * Hq + h) * S + qrow;
    if (wave == 0)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(attn_rsrc(lse2 + sidx, 256), (LDS_PTR(void))(st + 2 * Tile::BYTES), 4,
                                               (uint32_t)lane * 4, 0, 0, 0);
    if (!WANT_DV && wave == 1)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(attn_rsrc(delta + sidx, 256), (LDS_PTR(void))(st + 2 * Tile::BYTES + 256),
                                               4, (uint32_t)lane * 4, 0, 0, 0);
  };
  issue_tile(0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int stage = 0;
  for (int it = 0; it < niter; ++it) {
    if (it + 1 < niter) issue_tile(stage ^ 1);
    const int qrow = cur_qt * 64;
    if (++cur_g == G) { cur_g = 0; --cur_qt; }
    const char* tq = smem + stage * STAGE;
    const char* tdo = tq + Tile::BYTES;
    const float* stat = reinterpret_cast<const float*>(tq + 2 * Tile::BYTES);
    // queries before the key are masked: P = 0 for query rows below  kvw + lk - qrow
    const bool diag = qrow < kvw + 31;
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
      // S[q][kv] (and dP[q][kv]) for 32 queries: lane owns key kvw + lk, queries along registers
      f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
      if constexpr (!WANT_DV) {
        // dP - delta comes out of the product itself: the dP accumulator starts from -delta of its query rows
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(stat + 64 + qs * 32 + g * 8 + half * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) dp[g * 4 + e] = d4[e];
        }
      }
#pragma unroll
      for (int kk = 0; kk < DH / 16; ++kk) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(tq, qs * 32, kk, lane), kf[kk], s, 0, 0, 0);
        if constexpr (!WANT_DV)
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(tdo, qs * 32, kk, lane), vf[kk], dp, 0, 0, 0);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ql = qs * 32 + g * 8 + half * 4;
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(stat + ql);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = g * 4 + e;
          const float pv = fast_exp2(__builtin_fmaf(s[r], scale_log2, -l4[e]));
          if constexpr (WANT_DV) s[r] = pv; else s[r] = pv * dp[r];   // P or dS = P (dP - delta)
        }
      }
      if (diag) {
        asm volatile("" ::: "memory");
        const int first_ok = kvw + lk - qrow - (half << 2);   // smallest unmasked row offset for this lane
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (qs * 32 + ((r >> 2) << 3) + (r & 3) < first_ok) s[r] = 0.f;
      }
      // dV^T[d][kv] += dO^T[d][q] P[q][kv]   or   dK^T[d][kv] += Q^T[d][q] dS[q][kv]
      const char* tsrc = WANT_DV ? tdo : tq;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const bf16x8 pf = pack_slots(s, ks * 8);
#pragma unroll
        for (int t2 = 0; t2 < DH / 32; ++t2)
          acc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(tsrc, t2 * 32, qs * 32 + ks * 16, lane), pf, acc[t2], 0, 0, 0);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    stage ^= 1;
  }
  const float oscale = WANT_DV ? 1.0f : scale;
  if constexpr (!WANT_DV) {
    if (rope_cos) rope_unrotate<DH>(acc, rope_cos + (int64_t)(kvw + lk) * (DH / 2), rope_sin + (int64_t)(kvw + lk) * (DH / 2), rope_layout, half);
  }
  const int64_t off = ((int64_t)b * S + kvw + lk) * ldk + (int64_t)hk * DH + half * 4;
#pragma unroll
  for (int t2 = 0; t2 < DH / 32; ++t2)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 ov;
#pragma unroll
      for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(acc[t2][g * 4 + e] * oscale);
      *reinterpret_cast<bf16x4*>(dout + off + t2 * 32 + g * 8) = ov;
    }
}

// ------------------------------------------------------------------------------------------
// dS handed from the dK/dV pass to the dQ pass (128-wide heads, long sequences), so that dQ is one product per tile
// instead of three (S and dP are not formed a second time).  Storage, bf16, lower triangle only:
//   per (batch, query head): query blocks qb of 128 rows, each followed by its 2 (qb + 1) key tiles of 64;
//   one (query block, key tile) unit = 16 KiB = four sub-tiles of 4 KiB, one per 32 query rows of the block;
//   a sub-tile is [2 runs of 32 keys][2 planes][32 keys][16 query slots], 32 bytes per key and plane; slot
//   p = 16 plane + c holds query row 16 plane + 8 ((c >> 2) & 1) + 4 (c >> 3) + (c & 3) of the 32 - plane and c
//   are the 16-key step and the position (lane half, element) at which a lane of the dK/dV kernel holds the
//   packed dS operand, so each of its two 16-byte stores covers 1 KiB without gaps over the wave.
// The dQ pass reads a unit as one contiguous 16 KiB tile per 64 keys.
// ------------------------------------------------------------------------------------------
struct DsLayout {
  static constexpr int64_t UNIT = 16384, SUB = 4096;
  static __host__ __device__ __forceinline__ int64_t block_unit(int64_t qb) { return qb * (qb + 1); }   // units before block qb
  static __host__ __device__ __forceinline__ int64_t head_units(int64_t S) { return block_unit(S / 128); }
  static __device__ __forceinline__ int slot_row(int p) { return (p & 16) | (((p >> 2) & 1) << 3) | (((p >> 3) & 1) << 2) | (p & 3); }
};

// dQ from the stored dS: workgroup = 128 query rows of NH query heads of one KV group (they share the K
// tiles, which the first four waves load), wave = 32 rows of one head (one sub-tile per key tile);
// dQ^T[d][q] += K^T[d][key] dS^T[key][q] with both operands read from LDS tiles through transposing reads.
// Lane l of a wave owns query slot l % 32, i.e. row slot_row(l % 32) of the wave's 32.
template <int DH, int NH>
__global__ __launch_bounds__(256 * NH, 2 / NH) void attn_bwd_dq_from_ds_kernel(
    const bf16_t* __restrict__ k, const bf16_t* __restrict__ ds, bf16_t* __restrict__ dq, int B, int S, int Hq,
    int Hkv, float scale, const float* __restrict__ rope_cos, const float* __restrict__ rope_sin, int rope_layout) {
  using KTile = RowTile<64, DH, 4>;
  constexpr int DSUB = (int)DsLayout::SUB;
  // LDS: two stages of K tiles, then three of dS tiles (one 4 KiB sub-tile per wave): the dS tiles are the
  // kernel's HBM stream and are requested two tiles ahead, the K tiles (L2 hits) one ahead
  static_assert(NH == 1 || NH == 2, "one or two heads per workgroup");
  constexpr int KRING = 2 * KTile::BYTES, DSTAGE = 4 * NH * DSUB;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sub = wave & 3, hsel = wave >> 2;
  int j, pair;
  split_block_id((int)blockIdx.x, B * Hkv, j, pair);
  const int G = Hq / Hkv, GW = G / NH, b = pair / Hkv, hk = pair % Hkv;
  const int qb = S / 128 - 1 - j / GW, h = hk * G + (j % GW) * NH + hsel;   // long rows (late query blocks) first
  const int half = lane >> 5;
  const int qrow = qb * 128 + sub * 32 + DsLayout::slot_row(lane & 31);
  const int64_t ldq = (int64_t)Hq * DH, ldk = (int64_t)Hkv * DH;

  f32x16 acc[DH / 32];
#pragma unroll
  for (int t = 0; t < DH / 32; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  const bf16_t* kb = k + (int64_t)b * S * ldk + (int64_t)hk * DH;
  const uint32_t kv_bytes = (uint32_t)((((int64_t)S - 1) * ldk + DH) * 2);
  const char* dsb = reinterpret_cast<const char*>(ds) +
                    (DsLayout::head_units(S) * ((int64_t)b * Hq + h) + DsLayout::block_unit(qb)) * DsLayout::UNIT + sub * DsLayout::SUB;
  const int nkv = 2 * (qb + 1);
  auto issue_k = [&](int t) {
    if (NH > 1 && hsel != 0) return;
    const uint32_t skip = (uint32_t)((int64_t)t * 64 * ldk * 2);
    KTile::issue(attn_rsrc(kb + (int64_t)t * 64 * ldk, kv_bytes - skip), smem + (t & 1) * KTile::BYTES, sub, lane, ldk);
  };
  auto issue_ds = [&](int t, int dstage) {
    // the wave's sub-tile as it is stored: four wave-wide 1 KiB loads, non-temporal (read once)
    const __amdgpu_buffer_rsrc_t rs = attn_rsrc(dsb + (int64_t)t * DsLayout::UNIT, (uint32_t)DsLayout::SUB);
    char* dst = smem + KRING + dstage * DSTAGE + wave * DSUB;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (LDS_PTR(void))(dst + i * 1024), 16, (uint32_t)lane * 16, i * 1024, 0, 2);
  };
  // LDS addresses of the transposed reads for 16-key step 0 of stage 0 (see RowTile::frag_cols); later steps
  // and the other stage are immediate offsets / one add away because the swizzle repeats every 16 rows.
  constexpr int NT2 = DH / 32;
  uint32_t ka[NT2][2], da[2];
  {
    const int grp = lane >> 4, sl = lane & 15, e = sl >> 2, g = sl & 3;
    const int row = ((grp >> 1) << 2) + e, colq = ((grp & 1) << 4) + (g << 2);
    const uint32_t s0 = (uint32_t)(uintptr_t)(LDS_PTR(char))smem;
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
      const int r = row + rr * 8;
#pragma unroll
      for (int t2 = 0; t2 < NT2; ++t2) {
        const int col = t2 * 32 + colq;
        ka[t2][rr] = s0 + r * KTile::ROW_B + ((((col >> 3) ^ KTile::swz(r)) << 4) | ((col & 7) << 1));
      }
      // dS: plane = the lane's 16-column half, 32-byte rows: the 16 lanes of a transposing read fetch 128
      // contiguous bytes, so the stored layout needs no swizzle
      da[rr] = s0 + KRING + wave * DSUB + (grp & 1) * 1024 + r * 32 + (g << 3);
    }
  }
  issue_k(0);
  issue_ds(0, 0);
  issue_ds(1, 1);            // nkv >= 2
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int dcur = 0;              // dS stage of tile t; tile t + 2 goes to the stage tile t - 1 used
  for (int t = 0; t < nkv; ++t) {
    // K of the next tile first, then dS two tiles ahead: the wait at the bottom leaves the latter in flight
    if (t + 1 < nkv) issue_k(t + 1);
    const bool ahead = t + 2 < nkv;
    if (ahead) issue_ds(t + 2, dcur == 0 ? 2 : dcur - 1);
    const uint32_t sbk = (uint32_t)((t & 1) * KTile::BYTES), sbd = (uint32_t)(dcur * DSTAGE);
    // The reads are inline assembly (the compiler would put a wait for the tile loads just issued in front
    // of the builtin, which it cannot tell apart from the stage being filled) and are neither counted nor
    // moved by the compiler: fragments of step ks + 1 are requested before the products of step ks, and
    // every use sits behind a wait that names the fragments.
    bf16x8 kf[2][NT2], df[2];
    auto request = [&](auto KS) {
      constexpr int ks = decltype(KS)::value, bi = ks & 1;
      bf16x4 lo, hi;
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(da[0] + sbd), "n"((ks >> 1) * 2048 + (ks & 1) * 512));
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(da[1] + sbd), "n"((ks >> 1) * 2048 + (ks & 1) * 512));
      df[bi].lo = lo; df[bi].hi = hi;
#pragma unroll
      for (int t2 = 0; t2 < NT2; ++t2) {
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(ka[t2][0] + sbk), "n"(ks * 16 * KTile::ROW_B));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(ka[t2][1] + sbk), "n"(ks * 16 * KTile::ROW_B));
        kf[bi][t2].lo = lo; kf[bi][t2].hi = hi;
      }
    };
    auto step = [&](auto KS) {
      constexpr int ks = decltype(KS)::value, bi = ks & 1;
      if constexpr (ks < 3) {
        request(std::integral_constant<int, ks + 1>{});
        if constexpr (NT2 == 4)
          asm volatile("s_waitcnt lgkmcnt(10)" : "+v"(df[bi]), "+v"(kf[bi][0]), "+v"(kf[bi][1]), "+v"(kf[bi][2]), "+v"(kf[bi][3]));
        else
          asm volatile("s_waitcnt lgkmcnt(6)" : "+v"(df[bi]), "+v"(kf[bi][0]), "+v"(kf[bi][1]));
      } else {
        if constexpr (NT2 == 4)
          asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(df[bi]), "+v"(kf[bi][0]), "+v"(kf[bi][1]), "+v"(kf[bi][2]), "+v"(kf[bi][3]));
        else
          asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(df[bi]), "+v"(kf[bi][0]), "+v"(kf[bi][1]));
      }
#pragma unroll
      for (int t2 = 0; t2 < NT2; ++t2)
        acc[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[bi][t2], df[bi], acc[t2], 0, 0, 0);
    };
    request(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{});
    step(std::integral_constant<int, 3>{});
    // four dS loads per wave and tile, issued after the K loads: the wait leaves those of tile t + 2 in flight
    if (ahead) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    dcur = dcur == 2 ? 0 : dcur + 1;
  }
  // q was rotated after its projection: hand back the gradient of the unrotated q
  if (rope_cos) rope_unrotate<DH>(acc, rope_cos + (int64_t)qrow * (DH / 2), rope_sin + (int64_t)qrow * (DH / 2), rope_layout, half);
  bf16_t* op = dq + ((int64_t)b * S + qrow) * ldq + (int64_t)h * DH + half * 4;
#pragma unroll
  for (int t2 = 0; t2 < DH / 32; ++t2)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 ov;
#pragma unroll
      for (int e = 0; e < 4; ++e) ov[e] = (bf16_t)(acc[t2][g * 4 + e] * scale);
      *reinterpret_cast<bf16x4*>(op + t2 * 32 + g * 8) = ov;
    }
}

// ------------------------------------------------------------------------------------------
// dK and dV in one pass (head dims 64 and 128).  Workgroup = 4 waves = 128 keys of one (batch, kv head),
// wave = 32 keys; it streams 32-row Q / dO tiles of every query head of the group from the last query
// tile back to the diagonal.  Per tile: S = Q K^T and dP = dO V^T - delta once, P = exp2(..), dS = P dP,
// then dV^T += dO^T P and dK^T += Q^T dS: 4 products where the two separate kernels run 5, one
// exponential pass instead of two, and every Q / dO tile crosses L2 -> LDS once instead of twice.
// To hold both accumulators at two waves per SIMD the wave's V fragments live in LDS (the 128-key V tile
// stays resident), only its K fragments in registers, and the query tile is 32 rows.
// ------------------------------------------------------------------------------------------
template <int DH, bool WRITE_DS>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkdv_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ d_o, const float* __restrict__ lse2, const float* __restrict__ delta,
    bf16_t* __restrict__ dk_out, bf16_t* __restrict__ dv_out, bf16_t* __restrict__ ds_out, int B, int S, int Hq,
    int Hkv, float scale, const float* __restrict__ rope_cos, const float* __restrict__ rope_sin, int rope_layout) {
  using VTile = RowTile<128, DH, 4>;
  using Tile = RowTile<32, DH, 1>;          // addressing of a 32-row tile; loaded by issue32 below
  constexpr int TB = 32 * DH * 2;           // one Q or dO tile
  constexpr int STAGE = 2 * TB + 512;       // Q tile, dO tile, lse2[32] (+ pad), delta[32] (+ pad)
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  char* tv = smem + 2 * STAGE;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int kt, pair;   // low key tiles have the most query tiles: first
  split_block_id((int)blockIdx.x, B * Hkv, kt, pair);
  const int G = Hq / Hkv, b = pair / Hkv, hk = pair % Hkv;
  const int kv0 = kt * 128, kvw = kv0 + wave * 32;
  const int lk = lane & 31, half = lane >> 5;
  const int64_t ldq = (int64_t)Hq * DH, ldk = (int64_t)Hkv * DH;
  const float scale_log2 = scale * kLog2e;

  bf16x8 kf[DH / 16];
  {
    const int64_t off = ((int64_t)b * S + kvw + lk) * ldk + (int64_t)hk * DH + half * 8;
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) kf[kk] = *reinterpret_cast<const bf16x8*>(k + off + kk * 16);
  }
  f32x16 acc_k[DH / 32], acc_v[DH / 32];
#pragma unroll
  for (int t = 0; t < DH / 32; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) { acc_k[t][e] = 0.f; acc_v[t][e] = 0.f; }

  const int nq = (S - kv0) / 32, niter = G * nq;
  const uint32_t q_bytes = (uint32_t)((((int64_t)S - 1) * ldq + DH) * 2);
  // 32 rows x DH*2 bytes = 32*DH*2/1024 wave-wide loads per tile, dealt to the four waves
  constexpr int RPI = 1024 / (DH * 2), NI = 32 / RPI, IPW = NI / 4;
  static_assert(NI % 4 == 0 && IPW >= 1, "a 32-row tile must split over four waves");
  auto issue32 = [&](const bf16_t* base, uint32_t bytes, char* dst) {
    const __amdgpu_buffer_rsrc_t rs = attn_rsrc(base, bytes);
    const int r = lane / Tile::LPR, pc = lane % Tile::LPR;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int j = wave * IPW + i, row = j * RPI + r;
      const int c = pc ^ Tile::swz(row);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (LDS_PTR(void))(dst + j * 1024), 16, (uint32_t)(r * ldq * 2 + (c << 4)),
                                               (uint32_t)((int64_t)j * RPI * ldq * 2), 0, 0);
    }
  };
  int ld_g = 0, ld_qt = S / 32 - 1, cur_g = 0, cur_qt = S / 32 - 1;
  const uint32_t ds_lane = (uint32_t)(lk * 32 + half * 16);
  auto issue_tile = [&](int stage) {
    const int h = hk * G + ld_g, qrow = ld_qt * 32;
    if (++ld_g == G) { ld_g = 0; --ld_qt; }
    const int64_t base = ((int64_t)b * S) * ldq + (int64_t)h * DH;
    const uint32_t skip = (uint32_t)((int64_t)qrow * ldq * 2);
    char* st = smem + stage * STAGE;
    issue32(q + base + (int64_t)qrow * ldq, q_bytes - skip, st);
    issue32(d_o + base + (int64_t)qrow * ldq, q_bytes - skip, st + TB);
    // 32 lse2 and 32 -delta values of the tile, 4 bytes per lane, lanes 32..63 out of range (they store zeros into the pad)
    const int64_t sidx = ((int64_t)b * Hq + h) * S + qrow;
    if (wave == 0)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(attn_rsrc(lse2 + sidx, 128), (LDS_PTR(void))(st + 2 * TB), 4, (uint32_t)lane * 4, 0, 0, 0);
    if (wave == 1)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(attn_rsrc(delta + sidx, 128), (LDS_PTR(void))(st + 2 * TB + 256), 4, (uint32_t)lane * 4, 0, 0, 0);
  };
  {
    // the workgroup's 128 rows of V stay in LDS; wave w loads (and later reads) rows 32 w .. 32 w + 31
    const uint32_t kv_bytes = (uint32_t)((((int64_t)S - 1) * ldk + DH) * 2);
    const bf16_t* vb = v + ((int64_t)b * S + kv0) * ldk + (int64_t)hk * DH;
    VTile::issue(attn_rsrc(vb, kv_bytes - (uint32_t)((int64_t)kv0 * ldk * 2)), tv, wave, lane, ldk);
  }
  issue_tile(0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  int stage = 0;
  for (int it = 0; it < niter; ++it) {
    // The K fragments are pinned in registers across the loads below.  The kernel is a few registers
    // short, and left alone the compiler spills one K fragment and reloads it at the top of the loop:
    // vmcnt counts in order, so the wait for that reload also waits for the tile loads issued just
    // before it, every iteration (-7 % on the backward at S = 2048; at S = 8192, where the kernels run
    // at the power limit, the other workgroup's waves cover the stall and nothing changes).  With the
    // pin the spill moves to values whose reload comes after the first two products.
    static_assert(DH == 128 || DH == 64, "the pin lists the DH / 16 fragments by name");
    if constexpr (DH == 128)
      asm volatile("" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]), "+v"(kf[4]), "+v"(kf[5]), "+v"(kf[6]), "+v"(kf[7]));
    else
      asm volatile("" : "+v"(kf[0]), "+v"(kf[1]), "+v"(kf[2]), "+v"(kf[3]));
    if (it + 1 < niter) issue_tile(stage ^ 1);
    const int qrow = cur_qt * 32;
    // where this wave's 32 keys x 32 queries of dS go (layout: DsLayout above)
    const char* ds_dst = reinterpret_cast<const char*>(ds_out) +
                         (DsLayout::head_units(S) * ((int64_t)b * Hq + hk * G + cur_g) + DsLayout::block_unit(cur_qt >> 2) + 2 * kt + (wave >> 1)) * DsLayout::UNIT +
                         (cur_qt & 3) * DsLayout::SUB + (wave & 1) * 2048;   // wave-uniform; the lane adds ds_lane
    if (++cur_g == G) { cur_g = 0; --cur_qt; }
    const char* tq = smem + stage * STAGE;
    const char* tdo = tq + TB;
    const float* stat = reinterpret_cast<const float*>(tq + 2 * TB);
    // S[q][kv] and dP[q][kv] - delta[q] for the 32 queries: lane owns key kvw + lk, queries along registers
    // (the lane's offset into the statistics is formed anew every iteration: kept across the loop it is the
    // value the register allocator spills, and its reload would sit right behind the tile loads above)
    int half_l = half;
    asm volatile("" : "+v"(half_l));
    f32x16 s, dp;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 d4 = *reinterpret_cast<const f32x4*>(stat + 64 + g * 8 + half_l * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { s[g * 4 + e] = 0.f; dp[g * 4 + e] = d4[e]; }
    }
#pragma unroll
    for (int kk = 0; kk < DH / 16; ++kk) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(tq, 0, kk, lane), kf[kk], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_rows(tdo, 0, kk, lane), VTile::frag_rows(tv, wave * 32, kk, lane), dp, 0, 0, 0);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 l4 = *reinterpret_cast<const f32x4*>(stat + g * 8 + half_l * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = g * 4 + e;
        const float pv = fast_exp2(__builtin_fmaf(s[r], scale_log2, -l4[e]));
        s[r] = pv;            // P
        dp[r] = pv * dp[r];   // dS = P (dP - delta)
      }
    }
    if (qrow < kvw + 31) {
      // queries before the key are masked: P = dS = 0 for query rows below kvw + lk - qrow
      asm volatile("" ::: "memory");
      const int first_ok = kvw + lk - qrow - (half << 2);
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (((r >> 2) << 3) + (r & 3) < first_ok) { s[r] = 0.f; dp[r] = 0.f; }
    }
    // dV^T[d][kv] += dO^T[d][q] P[q][kv]   and   dK^T[d][kv] += Q^T[d][q] dS[q][kv]
    const bf16x8 df0 = pack_slots(dp, 0), df1 = pack_slots(dp, 8);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const bf16x8 pf = pack_slots(s, ks * 8), df = ks ? df1 : df0;
#pragma unroll
      for (int t2 = 0; t2 < DH / 32; ++t2) {
        acc_v[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(tdo, t2 * 32, ks * 16, lane), pf, acc_v[t2], 0, 0, 0);
        acc_k[t2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Tile::frag_cols(tq, t2 * 32, ks * 16, lane), df, acc_k[t2], 0, 0, 0);
      }
    }
    // dS for the dQ pass.  The two stores are the last vector-memory instructions of the iteration and the
    // wait below leaves exactly them in flight (the counter retires in issue order, so every tile load
    // issued before them has landed); their latency is then covered by the next iteration instead of
    // being waited for here.
    if constexpr (WRITE_DS)
      asm volatile("global_store_dwordx4 %0, %1, %3 nt\n\tglobal_store_dwordx4 %0, %2, %3 offset:1024 nt\n\ts_waitcnt vmcnt(2)"
                   :: "v"(ds_lane), "v"(df0), "v"(df1), "s"(ds_dst) : "memory");
    else
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    stage ^= 1;
  }
  if (rope_cos) rope_unrotate<DH>(acc_k, rope_cos + (int64_t)(kvw + lk) * (DH / 2), rope_sin + (int64_t)(kvw + lk) * (DH / 2), rope_layout, half);
  const int64_t off = ((int64_t)b * S + kvw + lk) * ldk + (int64_t)hk * DH + half * 4;
#pragma unroll
  for (int t2 = 0; t2 < DH / 32; ++t2)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 ok, ov;
#pragma unroll
      for (int e = 0; e < 4; ++e) { ok[e] = (bf16_t)(acc_k[t2][g * 4 + e] * scale); ov[e] = (bf16_t)acc_v[t2][g * 4 + e]; }
      *reinterpret_cast<bf16x4*>(dk_out + off + t2 * 32 + g * 8) = ok;
      *reinterpret_cast<bf16x4*>(dv_out + off + t2 * 32 + g * 8) = ov;
    }
}


// ------------------------------------------------------------------------------------------
template <int DH>
static int fwd_dh(const void* q, const void* k, const void* v, int64_t B, int64_t S, int64_t Hq,
                  int64_t Hkv, void* o, float* lse, hipStream_t st) {
  const size_t lds = 2 * 2 * (size_t)RowTile<64, DH, 4>::BYTES;
  static std::atomic<unsigned long long> lds_done{0};
  if (int rc = reserve_lds(attn_fwd_kernel<DH>, lds, lds_done, "attention_forward")) return rc;
  const float scale_log2 = (float)(1.0 / sqrt((double)DH)) * kLog2e;
  hipLaunchKernelGGL(attn_fwd_kernel<DH>, dim3((unsigned)(S / 128 * Hq * B)), dim3(256),
                     lds, st, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)o, lse, (int)B, (int)S,
                     (int)Hq, (int)Hkv, scale_log2);
  return check_launch("attention_forward");
}

int launch_attention_fwd(const void* q, const void* k, const void* v, int64_t B, int64_t S, int64_t Hq,
                         int64_t Hkv, int64_t dh, void* o, float* lse, hipStream_t st) {
  if (dh == 128) return fwd_dh<128>(q, k, v, B, S, Hq, Hkv, o, lse, st);
  if (dh == 64) return fwd_dh<64>(q, k, v, B, S, Hq, Hkv, o, lse, st);
  return fwd_dh<32>(q, k, v, B, S, Hq, Hkv, o, lse, st);
}

// -rowsum(dO * O) and lse * log2(e), then (head dims 64 and 128) the dS tiles of DsLayout
static size_t bwd_stats_bytes(int64_t B, int64_t S, int64_t Hq) {
  return (2 * (size_t)B * Hq * S * sizeof(float) + 4095) / 4096 * 4096;
}
// Handing dS over costs its HBM round trip (2 bytes per causal score, written and read once) and saves two of
// the dQ pass's three products, whose cost grows with the head dim: worth it for 128-wide heads once the
// sequences are long enough for the products to dominate (measured on the backward: -6 % at S = 2048 to
// 16384 with 128-wide heads; with 64-wide heads +4 % at S = 2048, +11 % at 4096 and +29 % at 8192).
static bool ds_handoff(int64_t S, int64_t dh) { return dh == 128 && S >= 2048; }
size_t attention_bwd_workspace(int64_t B, int64_t S, int64_t Hq, int64_t, int64_t dh) {
  const size_t stats = bwd_stats_bytes(B, S, Hq);
  return ds_handoff(S, dh) ? stats + (size_t)B * Hq * DsLayout::head_units(S) * DsLayout::UNIT : stats;
}

template <int DH>
static int bwd_dh(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                  const float* lse, int64_t B, int64_t S, int64_t Hq, int64_t Hkv, void* dq, void* dk,
                  void* dv, void* workspace, const float* rope_cos, const float* rope_sin, int rope_layout,
                  hipStream_t st) {
  float* delta = (float*)workspace;
  float* lse2 = delta + B * Hq * S;
  const int64_t rows = B * S * Hq;
  const int64_t nthreads = rows * (DH / 8);
  hipLaunchKernelGGL(attn_delta_kernel<DH>, dim3((unsigned)((nthreads + 255) / 256)), dim3(256), 0, st,
                     (const bf16_t*)o, (const bf16_t*)d_o, lse, delta, lse2, rows, (int)S, (int)Hq);
  if (int rc = check_launch("attention_backward(delta)")) return rc;
  const float scale = (float)(1.0 / sqrt((double)DH));
  const dim3 kv_grid((unsigned)(S / 128 * Hkv * B)), q_grid((unsigned)(S / 128 * Hq * B));
  if constexpr (DH >= 64) {
    const size_t lds_m = 2 * (2 * (size_t)(32 * DH * 2) + 512) + (size_t)RowTile<128, DH, 4>::BYTES;
    if constexpr (DH == 128) {
      if (ds_handoff(S, DH)) {
        bf16_t* ds = reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(workspace) + bwd_stats_bytes(B, S, Hq));
        static std::atomic<unsigned long long> done_m{0};
        if (int rc = reserve_lds(attn_bwd_dkdv_kernel<DH, true>, lds_m, done_m, "attention_backward")) return rc;
        hipLaunchKernelGGL((attn_bwd_dkdv_kernel<DH, true>), kv_grid, dim3(256), lds_m, st, (const bf16_t*)q, (const bf16_t*)k,
                           (const bf16_t*)v, (const bf16_t*)d_o, (const float*)lse2, (const float*)delta, (bf16_t*)dk, (bf16_t*)dv, ds,
                           (int)B, (int)S, (int)Hq, (int)Hkv, scale, rope_cos, rope_sin, rope_layout);
        if (int rc = check_launch("attention_backward(dk, dv)")) return rc;
        // two query heads of a KV group per workgroup where the group has an even number of them
        if ((Hq / Hkv) % 2 == 0) {
          const size_t lds_q = 2 * (size_t)RowTile<64, DH, 4>::BYTES + 3 * 8 * (size_t)DsLayout::SUB;
          static std::atomic<unsigned long long> done_q{0};
          if (int rc = reserve_lds(attn_bwd_dq_from_ds_kernel<DH, 2>, lds_q, done_q, "attention_backward")) return rc;
          hipLaunchKernelGGL((attn_bwd_dq_from_ds_kernel<DH, 2>), dim3(q_grid.x / 2), dim3(512), lds_q, st, (const bf16_t*)k,
                             (const bf16_t*)ds, (bf16_t*)dq, (int)B, (int)S, (int)Hq, (int)Hkv, scale, rope_cos, rope_sin, rope_layout);
        } else {
          const size_t lds_q = 2 * (size_t)RowTile<64, DH, 4>::BYTES + 3 * 4 * (size_t)DsLayout::SUB;
          static std::atomic<unsigned long long> done_q{0};
          if (int rc = reserve_lds(attn_bwd_dq_from_ds_kernel<DH, 1>, lds_q, done_q, "attention_backward")) return rc;
          hipLaunchKernelGGL((attn_bwd_dq_from_ds_kernel<DH, 1>), q_grid, dim3(256), lds_q, st, (const bf16_t*)k,
                             (const bf16_t*)ds, (bf16_t*)dq, (int)B, (int)S, (int)Hq, (int)Hkv, scale, rope_cos, rope_sin, rope_layout);
        }
        return check_launch("attention_backward(dq)");
      }
    }
    static std::atomic<unsigned long long> done_m{0};
    if (int rc = reserve_lds(attn_bwd_dkdv_kernel<DH, false>, lds_m, done_m, "attention_backward")) return rc;
    hipLaunchKernelGGL((attn_bwd_dkdv_kernel<DH, false>), kv_grid, dim3(256), lds_m, st, (const bf16_t*)q, (const bf16_t*)k,
                       (const bf16_t*)v, (const bf16_t*)d_o, (const float*)lse2, (const float*)delta, (bf16_t*)dk, (bf16_t*)dv,
                       (bf16_t*)nullptr, (int)B, (int)S, (int)Hq, (int)Hkv, scale, rope_cos, rope_sin, rope_layout);
    if (int rc = check_launch("attention_backward(dk, dv)")) return rc;
  } else {
    const size_t lds_kv = 2 * (2 * (size_t)RowTile<64, DH, 4>::BYTES + 512);
    static std::atomic<unsigned long long> done_dv{0}, done_dk{0};
    if (int rc = reserve_lds(attn_bwd_dkv_kernel<DH, true>, lds_kv, done_dv, "attention_backward")) return rc;
    if (int rc = reserve_lds(attn_bwd_dkv_kernel<DH, false>, lds_kv, done_dk, "attention_backward")) return rc;
    hipLaunchKernelGGL((attn_bwd_dkv_kernel<DH, true>), kv_grid, dim3(256), lds_kv, st, (const bf16_t*)q, (const bf16_t*)k,
                       (const bf16_t*)v, (const bf16_t*)d_o, (const float*)lse2, (const float*)delta, (bf16_t*)dv, (int)B, (int)S, (int)Hq,
                       (int)Hkv, scale, rope_cos, rope_sin, rope_layout);
    if (int rc = check_launch("attention_backward(dv)")) return rc;
    hipLaunchKernelGGL((attn_bwd_dkv_kernel<DH, false>), kv_grid, dim3(256), lds_kv, st, (const bf16_t*)q, (const bf16_t*)k,
                       (const bf16_t*)v, (const bf16_t*)d_o, (const float*)lse2, (const float*)delta, (bf16_t*)dk, (int)B, (int)S, (int)Hq,
                       (int)Hkv, scale, rope_cos, rope_sin, rope_layout);
    if (int rc = check_launch("attention_backward(dk)")) return rc;
  }
  const size_t lds_dq = 2 * 2 * (size_t)RowTile<64, DH, 4>::BYTES;
  static std::atomic<unsigned long long> done_dq{0};
  if (int rc = reserve_lds(attn_bwd_dq_kernel<DH>, lds_dq, done_dq, "attention_backward")) return rc;
  hipLaunchKernelGGL(attn_bwd_dq_kernel<DH>, q_grid, dim3(256), lds_dq, st, (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v,
                     (const bf16_t*)d_o, lse, (const float*)delta, (bf16_t*)dq, (int)B, (int)S, (int)Hq, (int)Hkv, scale, rope_cos,
                     rope_sin, rope_layout);
  return check_launch("attention_backward(dq)");
}

int launch_attention_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                         const float* lse, int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t dh,
                         void* dq, void* dk, void* dv, void* workspace, hipStream_t st) {
  return launch_attention_bwd_rope(q, k, v, o, d_o, lse, B, S, Hq, Hkv, dh, dq, dk, dv, workspace, nullptr, nullptr, 0, st);
}

int launch_attention_bwd_rope(const void* q, const void* k, const void* v, const void* o, const void* d_o,
                              const float* lse, int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t dh,
                              void* dq, void* dk, void* dv, void* workspace, const float* rope_cos,
                              const float* rope_sin, int rope_layout, hipStream_t st) {
  if (dh == 128) return bwd_dh<128>(q, k, v, o, d_o, lse, B, S, Hq, Hkv, dq, dk, dv, workspace, rope_cos, rope_sin, rope_layout, st);
  if (dh == 64) return bwd_dh<64>(q, k, v, o, d_o, lse, B, S, Hq, Hkv, dq, dk, dv, workspace, rope_cos, rope_sin, rope_layout, st);
  return bwd_dh<32>(q, k, v, o, d_o, lse, B, S, Hq, Hkv, dq, dk, dv, workspace, rope_cos, rope_sin, rope_layout, st);
}

}  // namespace dl
