// K2: the residue-domain GEMM  O[i][xi,nu][k][tau] = (sum_c U[i][xi,nu][k][c] V[i][xi,nu][tau][c]) mod p_i,
// one GEMM per transform point and residue, the modulo taken after the sum over C (paper section 6, eq. "gemm").
// int8 operands on v_mfma_i32_16x16x64_i8, int32 accumulation.
//
// Block = 4 waves = the 4 transform points of one group q (they end up as the 4 bytes of one O word); every
// wave computes a 16*RM (k) x 16*NTB (tile) block of its point over the whole of C (RM = 2, or 4 on layers large
// enough to fill the chip with the bigger blocks: each V fragment then feeds four MFMAs instead of two).  Operand fragments are read
// straight from global memory in 1 KiB runs (layout.hpp); KS contraction steps are loaded before any is
// consumed.  The four results of a group are exchanged through LDS so that O is written as whole words.
//
// 16-bit moduli: both operands are two byte planes, U = 256 Uh + Ul, V = 256 Vh + Vl, and
//   sum U V = 65536 sum(Uh Vh) + 256 sum(Uh Vl + Ul Vh) + sum(Ul Vl):
// four int8 MFMAs into three accumulators, combined in 64 bits and reduced once at the end.
//
// Grid: x = n*Q rounded up to a multiple of 8, y = ceil(Kp / (16*RM)), z = ceil(Tp / (16*NTB)).  Workgroups are handed to the
// 8 XCDs round-robin by linear id, so with gridDim.x a multiple of 8 all blocks of one x (which read the same V) share an L2.
#pragma once
#include "kernels_common.hpp"

namespace rnswino {

template <int KS, int NTB, int RM, bool WIDE>
__global__ __launch_bounds__(256) void k2_residue_gemm(KParams P, const int8_t *__restrict__ U,
                                                        const int8_t *__restrict__ V, uint32_t *__restrict__ O) {
  constexpr int PL = WIDE ? 2 : 1;
  constexpr int NACC = WIDE ? 3 : 1;
  constexpr int COLS = 16 * NTB;
  constexpr int ROWS = 16 * RM;          // k rows per wave and per block
  __shared__ uint32_t tile[ROWS * COLS * PL];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: slab addresses stay scalar
  const int lane = threadIdx.x & 63;
  if (blockIdx.x >= P.n * P.Q) return;             // grid.x is padded to a multiple of 8 (one XCD per x residue class)
  const int i = blockIdx.x / P.Q, q = blockIdx.x % P.Q;
  const int pt = 4 * q + wave;
  const int nkb = P.Kp >> 4, ntb = P.Tp >> 4, ncb = P.Cp >> 6;
  const int kb0 = blockIdx.y * RM, tb0 = blockIdx.z * NTB;
  const int p = P.p[i];
  const float inv = P.inv_p[i];

  v4i acc[NACC][RM][NTB];
#pragma unroll
  for (int a = 0; a < NACC; ++a)
#pragma unroll
    for (int rm = 0; rm < RM; ++rm)
#pragma unroll
      for (int tb = 0; tb < NTB; ++tb) acc[a][rm][tb] = (v4i){0, 0, 0, 0};

  if (pt < P.P2) {
    const int slab = i * P.P2 + pt;
    const int8_t *Ub = U + (size_t)slab * nkb * ncb * (1024 * PL) + lane * 16;
    const int8_t *Vb = V + (size_t)slab * ncb * (1024 * PL) + (lane & 15) * 64 + (lane >> 4) * 16;   // + tile block * vstride
    const size_t vstride = (size_t)P.n * P.P2 * ncb * (1024 * PL);
    for (int s0 = 0; s0 < ncb; s0 += KS) {
      v4i a[KS][RM][PL], b[KS][NTB][PL];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
#pragma unroll
        for (int rm = 0; rm < RM; ++rm)
#pragma unroll
          for (int pl = 0; pl < PL; ++pl) {
            a[s][rm][pl] = (v4i){0, 0, 0, 0};
            if (kb0 + rm < nkb)
              a[s][rm][pl] = *(const v4i *)(Ub + ((((size_t)(kb0 + rm) * ncb + s0 + s) * PL) + pl) * 1024);
          }
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
          for (int pl = 0; pl < PL; ++pl) {
            b[s][tb][pl] = (v4i){0, 0, 0, 0};
            if (tb0 + tb < ntb)
              b[s][tb][pl] = *(const v4i *)(Vb + (size_t)(tb0 + tb) * vstride + (size_t)((s0 + s) * PL + pl) * 1024);
          }
      }
#pragma unroll
      for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int rm = 0; rm < RM; ++rm)
#pragma unroll
          for (int tb = 0; tb < NTB; ++tb) {
            if (WIDE) {
              acc[0][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][0], b[s][tb][0], acc[0][rm][tb], 0, 0, 0);
              acc[1][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][0], b[s][tb][PL - 1], acc[1][rm][tb], 0, 0, 0);
              acc[1][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][PL - 1], b[s][tb][0], acc[1][rm][tb], 0, 0, 0);
              acc[NACC - 1][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][PL - 1], b[s][tb][PL - 1], acc[NACC - 1][rm][tb], 0, 0, 0);
            } else {
              acc[0][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][0], b[s][tb][0], acc[0][rm][tb], 0, 0, 0);
            }
          }
      // 8-bit residues, |U|,|V| <= 127: 512 channels add at most 8.3e6, so reducing every 8 steps keeps
      // |acc| < 2^24.  (Byte planes need nothing here: a step adds at most 2^21 and C is below 2^14.)
      if (!WIDE && (((s0 + KS) & 7) == 0) && (s0 + KS < ncb)) {
#pragma unroll
        for (int rm = 0; rm < RM; ++rm)
#pragma unroll
          for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[0][rm][tb][j] = mod_near(acc[0][rm][tb][j], inv, p);
      }
    }
  }

  uint8_t *tile8 = (uint8_t *)tile;
#pragma unroll
  for (int rm = 0; rm < RM; ++rm)
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = rm * 16 + 4 * (lane >> 4) + j, col = tb * 16 + (lane & 15);
        if (WIDE) {
          const long long tot = (long long)acc[0][rm][tb][j] * 65536 + (long long)acc[1][rm][tb][j] * 256 +
                                (long long)acc[NACC - 1][rm][tb][j];
          const int v = storable16(mod_near64(tot, P.inv_pd[i], p), p);
          const int lo = (int)(int8_t)(v & 0xFF), hi = (v - lo) >> 8;
          tile8[((row * COLS + col) * PL) * 4 + wave] = (uint8_t)hi;
          tile8[((row * COLS + col) * PL + PL - 1) * 4 + wave] = (uint8_t)lo;
        } else {
          tile8[(row * COLS + col) * 4 + wave] = (uint8_t)mod_lowbyte(acc[0][rm][tb][j], inv, -p);
        }
      }
  __syncthreads();
  // O is [Kp][n][Q][Tp] words (x PL) and smaller than 4 GiB: 32-bit word offsets, advanced by whole rows
  constexpr int ROWW = COLS * PL;         // words per tile row; divides 256
  constexpr int RSTEP = 256 / ROWW;       // rows covered by one pass of the block
  const uint32_t krow = (uint32_t)(P.n * P.Q * P.Tp) * PL;
  const int r0 = threadIdx.x / ROWW, rem = threadIdx.x % ROWW;
  const int tau = tb0 * 16 + rem / PL;
  uint32_t off = (uint32_t)(kb0 * 16 + r0) * krow + (uint32_t)((i * P.Q + q) * P.Tp + tb0 * 16) * PL + rem;
  const bool col_ok = tau < P.T;          // padding tiles are neither written nor read
#pragma unroll
  for (int it = 0; it < (ROWS * ROWW) / 256; ++it) {
    const int k = kb0 * 16 + it * RSTEP + r0;
    if (k < P.Kp && col_ok) O[off] = tile[it * 256 + threadIdx.x];
    off += RSTEP * krow;
  }
}

}  // namespace rnswino
