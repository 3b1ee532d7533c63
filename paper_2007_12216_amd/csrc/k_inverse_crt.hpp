// K3: inverse transform on the matrix cores, fused with the conversion out of the RNS.
//
// Y_i = A^T_p O_i A_p after the reduction over C (paper section 6, eq. "direct_sum_2"), then the residues
// (Y_0..Y_{n-1}) are converted to the integer result (section 3).  A^T O A = (A^T kron A^T) vec(O): per residue
// an (m*m) x (t*t) matrix applied to the t*t transform points of a (channel k, tile) pair.  MFMA roles: A operand =
// the Kronecker table (rows = 16 outputs), B operand = O (columns = 16 consecutive (k, tile) pairs),
// contraction index = transform point; a lane's 16 operand bytes are four O words (groups q = 16s + 4g + e).
//
// Conversion: the table rows are pre-multiplied by (P/p_i)^-1 mod p_i (P = prod p_i), so the reduced accumulator
// w_i is the CRT coefficient of residue i and
//     y = sum_i (P/p_i) w_i - P * rint(sum_i w_i / p_i)        (computed modulo 2^32)
// is the representative of the result in [-(P-1)/2, (P-1)/2] -- the same value mixed-radix conversion with
// symmetric digits yields; any representative of w_i gives the same y.  sum_i w_i/p_i = y/P + integer with
// |y/P| <= 1/2 - 1/(2P).  The rounding is done in binary64 (error of the sum below 1e-14, while 1/(2P) > 1e-10 for
// every moduli set whose product can matter for a 32-bit result), or in binary32 when the layer's worst case
// 2^14 r^2 C keeps |y/P| below 0.45 (the host decides: KParams::quot32).
//
// Fast conversion (8-bit moduli, KParams::fastcrt): the accumulator a_i is not reduced at all.  a_i is congruent to
// w_i modulo p_i, and (P/p_i) p_i = P, so S = sum_i (P/p_i) a_i is congruent to y modulo P and y = S - P rint(S/P) with
// S/P = sum_i a_i / p_i.  The accumulators start at 2^22 (|a_i| <= t*t * 126 * 128 <= 2^22), so that a_i + 2^22 is an
// unsigned 23-bit number: one 24-bit multiply-add (P/p_i < 2^24) and one binary32 multiply-add per residue and
// output; the constants that undo the offset sit in KParams (crt_sum0, crt_fs0).  The binary32 sum carries an
// error of a few hundredths (bounded on the host from the moduli), so the host enables this path only when the
// layer's worst case keeps |y/P| that far below 1/2 -- true for every layer whose moduli were chosen by the
// range bound with a little room, e.g. all five benchmark workloads.  Otherwise (KParams::fastcrt == 2) the same sum
// is taken in binary64, which is exact enough for every result the moduli can represent.
//
// Block = one unit of 16 consecutive (k, tile) pairs and four 16-output row blocks rb = 4*blockIdx.y + wave; every
// wave loads the O operand itself (the copies hit in L1): a wave-uniform row of O plus a 32-bit lane offset per
// word.  No LDS.
// Grid: x = ceil(K*T/16) rounded up to a multiple of 8, y = ceil(RB3/4); 256 threads.
// 16-bit moduli: table and O are two byte planes each; three accumulators as in the GEMM.
#pragma once
#include "kernels_common.hpp"

namespace rnswino {


// Where the output tile of a (k, tile) pair starts in y (or in the int8 activation plane): computed once per pair,
// the row blocks of the pair only add their own row and column to it.
struct TilePos {
  size_t origin;     // element index of output (oy0, ox0) of channel k of image img
  int oy0, ox0;      // top-left output of the tile
  bool ok;           // false for padding tiles and padding pairs
};

__device__ __forceinline__ TilePos tile_position(const KParams &P, int k, int tau) {
  TilePos tp;
  tp.ok = tau < P.T;
  const int trow = tau / P.tw;
  const int tx = tau - trow * P.tw;
  const int img = trow / P.th;
  const int ty = trow - img * P.th;
  tp.oy0 = ty * P.m;
  tp.ox0 = tx * P.m;
  const size_t plane = (size_t)img * P.K + k;
  if (P.epi == 2) tp.origin = (plane * (P.Ho >> 1) + (tp.oy0 >> 1)) * (P.Wo >> 1) + (tp.ox0 >> 1);
  else tp.origin = (plane * P.Ho + tp.oy0) * P.Wo + tp.ox0;
  return tp;
}

// CRT conversion of the four outputs of one lane (row block rb, lane group g) and their store: int32 y, or, for
// chained layers, int8 clamp(y >> shift) with an optional 2x2 max-pool (the shift is monotone, so it commutes with
// the max).  Must be called by all lanes of a wave (the pooled mode exchanges rows between lanes).
template <int NRES, bool CRT24, bool QUOT32>
__device__ __forceinline__ void crt_convert(const KParams &P, const uint32_t (&w)[NRES][4], int (&val)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t sum = 0;
    int kk;
    if (QUOT32) {
      // |y| <= 0.45 P: the sum is within 0.45 of an integer and binary32 (error below 1e-4) finds that integer
      float fs = 0.0f;
#pragma unroll
      for (int i = 0; i < NRES; ++i) {
        sum += CRT24 ? __umul24(P.crt_c[i], w[i][j]) : P.crt_c[i] * w[i][j];
        fs = __builtin_fmaf((float)w[i][j], P.inv_p[i], fs);
      }
      kk = (int)__builtin_rintf(fs);
    } else {
      double fs = 0.0;
#pragma unroll
      for (int i = 0; i < NRES; ++i) {
        sum += CRT24 ? __umul24(P.crt_c[i], w[i][j]) : P.crt_c[i] * w[i][j];
        fs = __builtin_fma((double)w[i][j], P.inv_pd[i], fs);
      }
      kk = __double2int_rn(fs);
    }
    val[j] = (int)(sum - P.prod_mod32 * (uint32_t)kk);
  }
}

// Fast conversion (see the header): w[i][j] = a_i + 2^22, unreduced.
template <int NRES>
__device__ __forceinline__ void crt_convert_fast(const KParams &P, const uint32_t (&w)[NRES][4], int (&val)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t sum = P.crt_sum0;
    float fs = P.crt_fs0;
#pragma unroll
    for (int i = 0; i < NRES; ++i) {
      sum += __umul24(P.crt_c[i], w[i][j]);
      fs = __builtin_fmaf((float)w[i][j], P.inv_p[i], fs);
    }
    const int kk = (int)__builtin_rintf(fs);
    val[j] = (int)(sum - P.prod_mod32 * (uint32_t)kk);
  }
}

// The same with the quotient in binary64: the sum then carries an error below 1e-10 and finds the quotient for every
// result in [-(P-1)/2, (P-1)/2] (the host checks its bound against 1/(2P)), so layers at the edge of the dynamic
// range and plans with an unchecked range take this form.
template <int NRES>
__device__ __forceinline__ void crt_convert_fast64(const KParams &P, const uint32_t (&w)[NRES][4], int (&val)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    uint32_t sum = P.crt_sum0;
    double fs = P.crt_fs0d;
#pragma unroll
    for (int i = 0; i < NRES; ++i) {
      sum += __umul24(P.crt_c[i], w[i][j]);
      fs = __builtin_fma((double)w[i][j], P.inv_pd[i], fs);
    }
    const int kk = __double2int_rn(fs);
    val[j] = (int)(sum - P.prod_mod32 * (uint32_t)kk);
  }
}

template <int NRES, bool FAST>
__device__ __forceinline__ void k3_convert(const KParams &P, const uint32_t (&w)[NRES][4], int (&val)[4]) {
  if (FAST) {
    if (P.fastcrt == 2) crt_convert_fast64<NRES>(P, w, val);   // uniform
    else crt_convert_fast<NRES>(P, w, val);
  } else if (P.crt24) {               // uniform: one branch per call instead of one per multiply
    if (P.quot32) crt_convert<NRES, true, true>(P, w, val);
    else crt_convert<NRES, true, false>(P, w, val);
  } else {
    crt_convert<NRES, false, false>(P, w, val);
  }
}

// Store of a lane's four outputs for 8 x 8 output tiles (the streaming kernel's unrolled path): the lane's row u
// and first column v (0 or 4) inside the tile and their offset `off` from the tile's origin in the stored plane do
// not depend on the unit and are kept in registers by the caller.  Same modes as k3_convert_and_store; the host
// selects this path for int32 output only when Wo is a multiple of 4.  Must be called by all lanes of a wave.
__device__ __forceinline__ void k3_store_m8(const KParams &P, const int (&val)[4], int u, int v, uint32_t off,
                                            const TilePos &tp, int32_t *__restrict__ y) {
  const bool inside = tp.ok && tp.oy0 + u < P.Ho && tp.ox0 + v < P.Wo;
  if (P.epi == 0) {
    if (inside) *(v4i *)(y + tp.origin + off) = (v4i){val[0], val[1], val[2], val[3]};
  } else if (P.epi == 1) {
    uint32_t packed = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) packed |= ((uint32_t)min(127, max(-128, val[j] >> P.shift)) & 0xFFu) << (8 * j);
    int8_t *dst = P.act + tp.origin + off;
    if ((P.Wo & 3) == 0) {
      if (inside) *(uint32_t *)dst = packed;
    } else {
      if (inside) *(uint16_t *)dst = (uint16_t)packed;
      if (inside && tp.ox0 + v + 2 < P.Wo) *(uint16_t *)(dst + 2) = (uint16_t)(packed >> 16);
    }
  } else {
    // rows u and u + 1 (u even) of the tile sit in lanes l and l ^ 32
    const int h0 = max(val[0], val[1]), h1 = max(val[2], val[3]);
    const int o0p = __shfl_xor(h0, 32), o1p = __shfl_xor(h1, 32);
    const int p0 = min(127, max(-128, max(h0, o0p) >> P.shift)), p1 = min(127, max(-128, max(h1, o1p) >> P.shift));
    if (inside && (u & 1) == 0)
      *(uint16_t *)(P.act + tp.origin + off) = (uint16_t)(((uint32_t)p0 & 0xFFu) | (((uint32_t)p1 & 0xFFu) << 8));
  }
}

template <int NRES, bool FAST>
__device__ __forceinline__ void k3_convert_and_store(const KParams &P, const uint32_t (&w)[NRES][4], int rb, int g,
                                                     const TilePos &tp, int32_t *__restrict__ y) {
  int val[4];
  k3_convert<NRES, FAST>(P, w, val);
  const int m = P.m, mm = m * m;
  const float inv_m = 1.0f / (float)m;
  const int o0 = 16 * rb + 4 * g;
  if (P.epi == 1 && (((m & 3) != 0) || (P.Wo & 1))) {
    // any other tile size or an odd row length: the four outputs may sit in two rows of the tile and at any byte
    // alignment, so each is stored as a byte of its own
    if (!tp.ok) return;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int o = o0 + j;
      const int u = (int)(((float)o + 0.5f) * inv_m);
      const int v = o - u * m;
      if (o < mm && tp.oy0 + u < P.Ho && tp.ox0 + v < P.Wo)
        P.act[tp.origin + (uint32_t)(u * P.Wo + v)] = (int8_t)min(127, max(-128, val[j] >> P.shift));
    }
    return;
  }
  if (P.epi != 0) {
    // here m is 4 or 8 and Wo even (pooling: the host also guarantees Wo % 4 == 0 and an even Ho)
    const int u = (int)(((float)o0 + 0.5f) * inv_m);
    const int v = o0 - u * m;
    const bool inside = tp.ok && o0 < mm && tp.oy0 + u < P.Ho && tp.ox0 + v < P.Wo;
    if (P.epi == 1) {
      uint32_t packed = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) packed |= ((uint32_t)min(127, max(-128, val[j] >> P.shift)) & 0xFFu) << (8 * j);
      int8_t *dst = P.act + tp.origin + (uint32_t)(u * P.Wo + v);
      if ((P.Wo & 3) == 0) {
        if (inside) *(uint32_t *)dst = packed;
      } else {
        // Wo even but not a multiple of 4: rows are only 2-byte aligned, and the second half may hang over the edge
        if (inside) *(uint16_t *)dst = (uint16_t)packed;
        if (inside && tp.ox0 + v + 2 < P.Wo) *(uint16_t *)(dst + 2) = (uint16_t)(packed >> 16);
      }
    } else {
      // rows u and u+1 (u even) of an output tile sit in lanes l and l ^ 4m (m = 8: 32 apart, m = 4: 16 apart)
      const int h0 = max(val[0], val[1]), h1 = max(val[2], val[3]);
      const int delta = 4 * m;
      const int o0p = __shfl_xor(h0, delta), o1p = __shfl_xor(h1, delta);
      const int p0 = min(127, max(-128, max(h0, o0p) >> P.shift)), p1 = min(127, max(-128, max(h1, o1p) >> P.shift));
      if (inside && (u & 1) == 0)
        *(uint16_t *)(P.act + tp.origin + (uint32_t)((u >> 1) * (P.Wo >> 1) + (v >> 1))) =
            (uint16_t)(((uint32_t)p0 & 0xFFu) | (((uint32_t)p1 & 0xFFu) << 8));
    }
    return;
  }
  if (!tp.ok || o0 >= mm) return;
  int32_t *ytile = y + tp.origin;
  if (((m & 3) == 0) && ((P.Wo & 3) == 0)) {   // four consecutive outputs stay in one row, 16-byte aligned
    const int u = (int)(((float)o0 + 0.5f) * inv_m);
    const int v = o0 - u * m;
    if (tp.oy0 + u < P.Ho && tp.ox0 + v < P.Wo) *(v4i *)(ytile + (uint32_t)(u * P.Wo + v)) = (v4i){val[0], val[1], val[2], val[3]};
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int o = o0 + j;
      const int u = (int)(((float)o + 0.5f) * inv_m);
      const int v = o - u * m;
      if (o < mm && tp.oy0 + u < P.Ho && tp.ox0 + v < P.Wo) ytile[(uint32_t)(u * P.Wo + v)] = val[j];
    }
  }
}

// FAST: the conversion with unreduced accumulators (the host launches it when KParams::fastcrt is set).
template <int NRES, int KS3, bool WIDE, bool FAST>
__global__ __launch_bounds__(256) void k3_inverse_crt(KParams P, const uint32_t *__restrict__ O,
                                                       int32_t *__restrict__ y) {
  constexpr int PL = WIDE ? 2 : 1;
  constexpr int NACC = WIDE ? 3 : 1;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: row block and table addresses stay scalar
  const int lane = threadIdx.x & 63, g = lane >> 4;
  const int rb = blockIdx.y * 4 + wave;            // this wave's block of 16 outputs
  if (rb >= P.RB3) return;
  // A unit is 16 consecutive (k, tile) pairs of the flattened K x T index space (no padding tiles: a unit may span
  // several k's).  Workgroups go to the 8 XCDs round-robin by id; neighbouring units share 128-byte lines of O, so
  // each XCD gets one contiguous chunk of the units (grid.x is a multiple of 8).
  // (For layers that pack TL tiles into a channel block, GEMM row kg = k * TL + tile / Tg and GEMM column tile % Tg.)
  const int npairs = P.Kg * P.Tg;                  // below 2^31 (checked when the plan is made)
  const int unit = xcd_chunked(blockIdx.x, gridDim.x, (npairs + 15) >> 4);
  if (unit < 0) return;
  const int pair = unit * 16 + (lane & 15);
  const bool pair_ok = pair < npairs;
  const int kg = pair_ok ? pair / P.Tg : 0;
  const int taug = pair_ok ? pair - kg * P.Tg : P.Tg;   // a padding lane's loads stay inside row 0
  const int k = kg / P.TL;
  const int tau = pair_ok ? (kg % P.TL) * P.Tg + taug : P.T;   // tau >= T marks a lane without output

  // O is [Kp][n][Q][Tp] words (x PL planes) and smaller than 4 GiB: the address of a word is a wave-uniform row
  // (residue, point group 16s + e) plus a 32-bit lane offset (k, lane group 4g, tile).  Point groups >= Q of the
  // last contraction step are clamped to Q - 1: the table is zero there, so whatever is read does not count.
  const uint32_t rowstride = (uint32_t)P.Tp * PL;
  const uint32_t lane_off = (uint32_t)(kg * P.n * P.Q) * rowstride + (uint32_t)taug * PL;
  uint32_t voff[KS3][4];
#pragma unroll
  for (int s = 0; s < KS3; ++s)
#pragma unroll
    for (int e = 0; e < 4; ++e) voff[s][e] = lane_off + (uint32_t)min(16 * s + 4 * g + e, P.Q - 1) * rowstride;
  v4i of[NRES][KS3][PL];
#pragma unroll
  for (int i = 0; i < NRES; ++i) {       // residue by residue, the order in which the products below consume them
    const uint32_t *row = O + (size_t)(i * P.Q) * rowstride;
#pragma unroll
    for (int s = 0; s < KS3; ++s)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (WIDE) {
          const v2i two = *(const v2i *)(row + voff[s][e]);
          of[i][s][0][e] = two[0];
          of[i][s][PL - 1][e] = two[1];
        } else {
          of[i][s][0][e] = (int)row[voff[s][e]];
        }
      }
  }

  {
    uint32_t w[NRES][4];
#pragma unroll
    for (int i = 0; i < NRES; ++i) {
      v4i acc[NACC];
#pragma unroll
      for (int a = 0; a < NACC; ++a) acc[a] = FAST ? (v4i){P.acc0, P.acc0, P.acc0, P.acc0} : (v4i){0, 0, 0, 0};
      const int8_t *ka = P.KA + (((size_t)i * P.RB3 + rb) * KS3) * (1024 * PL) + lane * 16;
#pragma unroll
      for (int s = 0; s < KS3; ++s) {
        const v4i ah = *(const v4i *)(ka + (size_t)s * (1024 * PL));
        if (WIDE) {
          const v4i al = *(const v4i *)(ka + (size_t)s * (1024 * PL) + 1024);
          acc[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ah, of[i][s][0], acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ah, of[i][s][PL - 1], acc[1], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(al, of[i][s][0], acc[1], 0, 0, 0);
          acc[NACC - 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(al, of[i][s][PL - 1], acc[NACC - 1], 0, 0, 0);
        } else {
          acc[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ah, of[i][s][0], acc[0], 0, 0, 0);
        }
      }
      // residue shifted by +p so that it is non-negative
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (WIDE) {
          // per accumulator |sum| <= t*t * 2^15: the combination stays below 2^40
          const long long tot = (long long)acc[0][j] * 65536 + (long long)acc[1][j] * 256 + (long long)acc[NACC - 1][j];
          w[i][j] = (uint32_t)(mod_near64(tot, P.inv_pd[i], P.p[i]) + P.p[i]);
        } else {
          // |acc| <= t*t * 126 * 128 <= 2^22 (plus the 2^22 of the fast conversion, which then takes it as it is)
          w[i][j] = FAST ? (uint32_t)acc[0][j] : mod_near_plus_p(acc[0][j], P.inv_p[i], -P.p[i], P.bias_p[i]);
        }
      }
    }
    k3_convert_and_store<NRES, FAST>(P, w, rb, g, tile_position(P, k, tau), y);
  }
}

// Streaming variant for layers with many tiles (8-bit moduli, table of all residues <= 64 KiB): the table is staged
// once per block in LDS, and every wave walks over units = (k, block of 16 tiles) with a grid stride.  Per unit a wave
// issues only its own O loads (no table reads from global memory, no copies of O in other waves); the table fragments
// come from LDS.  A unit's loads are hidden by the other waves of the SIMD (four resident blocks per CU; a second
// register set that prefetched the next unit's operand cost a block of occupancy and measured 3-10 % slower).
// Grid: min(ceil(units / 4), four blocks per CU) blocks of 256 threads; dynamic LDS = n * RB3 * KS3 KiB.
constexpr int K3_STREAM_BLOCKS = 1024;  // four resident blocks per CU (register budget) on 256 CUs

// M8: 8 x 8 output tiles (four row blocks), the usual case: where a lane's outputs go inside the tile is computed once
// per kernel instead of once per row block, and the table fragments of a row block sit at immediate LDS offsets.
template <int NRES, int KS3, bool FAST, bool M8>
__global__ __launch_bounds__(256) void k3_inverse_crt_stream(KParams P, const uint32_t *__restrict__ O,
                                                              int32_t *__restrict__ y) {
  extern __shared__ __attribute__((aligned(16))) uint8_t ka_lds[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: unit arithmetic stays scalar
  const int lane = threadIdx.x & 63, g = lane >> 4;
  const int ntb = P.Tp >> 4;
  const int nunits = P.Kg * ntb;                   // below 2^31 (checked when the plan is made); rows and columns are the GEMM's
  const int nwaves = gridDim.x * 4;
  {
    const int bytes = NRES * P.RB3 * KS3 * 1024;
    for (int off = threadIdx.x * 16; off < bytes; off += 256 * 16) *(v4i *)(ka_lds + off) = *(const v4i *)(P.KA + off);
  }
  __syncthreads();
  int unit = blockIdx.x * 4 + wave;
  if (unit >= nunits) return;

  // lane part of an O address, the same for every unit: point group (clamped to Q - 1 where the table is zero)
  // and tile within the block of 16; the unit contributes a wave-uniform base
  uint32_t voff[KS3][4];
#pragma unroll
  for (int s = 0; s < KS3; ++s)
#pragma unroll
    for (int e = 0; e < 4; ++e) voff[s][e] = (uint32_t)min(16 * s + 4 * g + e, P.Q - 1) * (uint32_t)P.Tp + (lane & 15);

  auto load_o = [&](int u, v4i (&of)[NRES][KS3]) {
    const int k = u / ntb, tb = u - k * ntb;
    const uint32_t *base = O + (size_t)k * P.n * P.Q * P.Tp + tb * 16;
#pragma unroll
    for (int i = 0; i < NRES; ++i) {
      const uint32_t *row = base + (size_t)(i * P.Q) * P.Tp;
#pragma unroll
      for (int s = 0; s < KS3; ++s)
#pragma unroll
        for (int e = 0; e < 4; ++e) of[i][s][e] = (int)row[voff[s][e]];
    }
  };

  // One unit with its O operand in `o`.
  const int a0 = FAST ? P.acc0 : 0;                 // 2^22 for the fast conversion
  const v4i acc_start = (v4i){a0, a0, a0, a0};
  // 8 x 8 tiles: outputs 16 rb + 4 g .. + 3 are row u = 2 rb + (g >> 1), columns v = 4 (g & 1) .. + 3 of the tile; in the
  // stored plane (pooled: half the rows and columns) row block rb + 1 lies m8_step elements after row block rb
  const int m8_u0 = g >> 1, m8_v = 4 * (g & 1);
  const uint32_t m8_step = P.epi == 2 ? (uint32_t)(P.Wo >> 1) : (uint32_t)(2 * P.Wo);
  const uint32_t m8_off0 = P.epi == 2 ? (uint32_t)(m8_v >> 1) : (uint32_t)(m8_u0 * P.Wo + m8_v);
  auto do_unit = [&](int u, v4i (&o)[NRES][KS3]) {
    const int kg = u / ntb, taug = (u - kg * ntb) * 16 + (lane & 15);
    const int k = kg / P.TL, tau = taug < P.Tg ? (kg % P.TL) * P.Tg + taug : P.T;   // packed layers: see plan.hpp
    const TilePos tp = tile_position(P, k, tau);
    if (M8) {
      // not unrolled: with the four row blocks in one basic block the scheduler requests all their table fragments
      // at once and the kernel needs twice the registers
#pragma clang loop unroll(disable)
      for (int rb = 0; rb < 4; ++rb) {
        uint32_t w[NRES][4];
        const uint8_t *ka_rb = ka_lds + lane * 16 + rb * (KS3 * 1024);
#pragma unroll
        for (int i = 0; i < NRES; ++i) {
          v4i acc = acc_start;
#pragma unroll
          for (int s = 0; s < KS3; ++s) {
            const v4i a = *(const v4i *)(ka_rb + (i * 4 * KS3 + s) * 1024);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, o[i][s], acc, 0, 0, 0);
          }
#pragma unroll
          for (int j = 0; j < 4; ++j)
            w[i][j] = FAST ? (uint32_t)acc[j] : mod_near_plus_p(acc[j], P.inv_p[i], -P.p[i], P.bias_p[i]);
        }
        int val[4];
        k3_convert<NRES, FAST>(P, w, val);
        k3_store_m8(P, val, 2 * rb + m8_u0, m8_v, m8_off0 + rb * m8_step, tp, y);
      }
      return;
    }
    for (int rb = 0; rb < P.RB3; ++rb) {
      uint32_t w[NRES][4];
#pragma unroll
      for (int i = 0; i < NRES; ++i) {
        v4i acc = acc_start;
#pragma unroll
        for (int s = 0; s < KS3; ++s) {
          const v4i a = *(const v4i *)(ka_lds + (((i * P.RB3 + rb) * KS3) + s) * 1024 + lane * 16);
          acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, o[i][s], acc, 0, 0, 0);
        }
        // |acc| <= t*t * 126 * 128 <= 2^22: the fast conversion takes acc + 2^22 as it is, the general one the
        // residue shifted by +p so that it is non-negative
#pragma unroll
        for (int j = 0; j < 4; ++j)
          w[i][j] = FAST ? (uint32_t)acc[j] : mod_near_plus_p(acc[j], P.inv_p[i], -P.p[i], P.bias_p[i]);
      }
      k3_convert_and_store<NRES, FAST>(P, w, rb, g, tp, y);
    }
  };
  v4i oa[NRES][KS3];
  for (; unit < nunits; unit += nwaves) {
    load_o(unit, oa);
    do_unit(unit, oa);
  }
}

}  // namespace rnswino
