// K2: the residue-domain GEMM  O[i][xi,nu][k][tau] = (sum_c U[i][xi,nu][k][c] V[i][xi,nu][tau][c]) mod p_i,
// one GEMM per transform point and residue, the modulo taken after the sum over C (paper section 6, eq. "gemm").
// int8 operands on v_mfma_i32_16x16x64_i8, int32 accumulation.
//
// Block = 4 waves = the 4 transform points of one group q (they end up as the 4 bytes of one O word); every
// wave computes a 16*RM (k) x 16*NTB (tile) block of its point over the whole of C (RM = 2, or 4 on layers large
// enough to fill the chip with the bigger blocks: each V fragment then feeds four MFMAs instead of two).  Operand fragments are read
// straight from global memory in 1 KiB runs (layout.hpp); KS contraction steps are loaded before any is
// consumed.  The four results of a group are exchanged through LDS so that O is written as whole words,
// 16 bytes per thread.
//
// 16-bit moduli: both operands are two byte planes, U = 256 Uh + Ul, V = 256 Vh + Vl, and
//   sum U V = 65536 sum(Uh Vh) + 256 sum(Uh Vl + Ul Vh) + sum(Ul Vl):
// four int8 MFMAs into three accumulators, combined in 64 bits and reduced once at the end.
//
// Grid: one-dimensional, 8 * (ceil(n*Q / 8) rounded up to a multiple of xgroup) * ceil(Kp / (16*RM)) * ceil(Tp / (16*NTB)).
#pragma once
#include <type_traits>

#include "kernels_common.hpp"

namespace rnswino {

template <int KS, int NTB, int RM, bool WIDE>
__global__ __launch_bounds__(256) void k2_residue_gemm(KParams P, const int8_t *__restrict__ U,
                                                        const int8_t *__restrict__ V, uint32_t *__restrict__ O, int xgroup) {
  constexpr int PL = WIDE ? 2 : 1;
  constexpr int NACC = WIDE ? 3 : 1;
  constexpr int COLS = 16 * NTB;
  constexpr int ROWS = 16 * RM;          // k rows per wave and per block
  constexpr int ROWW = COLS * PL;        // words per tile row
  constexpr int PITCH = ROWW + 4;        // LDS row pitch: the four row groups of a byte store fall into different banks
  __shared__ __attribute__((aligned(16))) uint32_t tile[ROWS * PITCH];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: slab addresses stay scalar
  const int lane = threadIdx.x & 63;
  const int nkb = P.Kp >> 4, ntb = P.Tp >> 4, ncb = P.Cp >> 6;
  // Work item (x = residue and point group, y = row block, z = tile block) from the linear workgroup id.  Workgroups
  // are handed to the 8 XCDs round-robin by id, so x = 8 * (...) + id % 8 keeps one x on one XCD.  Within an XCD the
  // ids run over `xgroup` values of x first, then y, then z, then the groups of x: the workgroups that share a slice
  // of U (same x and y, along z) or of V (same x and z, along y) follow each other closely enough to find it in the
  // XCD's L2, while `xgroup` different x at a time spread the accesses over the L2's channels.
  const int gy = (nkb + RM - 1) / RM, gz = (ntb + NTB - 1) / NTB;
  int rest = blockIdx.x >> 3;
  const int xi = rest % xgroup;
  rest /= xgroup;
  const int by = rest % gy;
  rest /= gy;
  const int bz = rest % gz;
  const int bx = ((rest / gz) * xgroup + xi) * 8 + (blockIdx.x & 7);
  if (bx >= P.n * P.Q) return;                     // x is padded to a multiple of 8
  const int i = bx / P.Q, q = bx % P.Q;
  const int pt = 4 * q + wave;
  const int kb0 = by * RM, tb0 = bz * NTB;
  const int p = P.p[i];
  const float inv = P.inv_p[i];

  v4i acc[NACC][RM][NTB];
  if (pt < P.P2) {
    const int slab = i * P.P2 + pt;
    // Row blocks and tile blocks past the end are clamped to the last one: what they compute is never stored, and
    // the loads need neither a branch nor a zero fill.
    const int8_t *Ur[RM], *Vt[NTB];
#pragma unroll
    for (int rm = 0; rm < RM; ++rm)
      Ur[rm] = U + ((size_t)slab * nkb + min(kb0 + rm, nkb - 1)) * ncb * (1024 * PL) + lane * 16;
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb)
      Vt[tb] = V + ((size_t)min(tb0 + tb, ntb - 1) * (P.n * P.P2) + slab) * ncb * (1024 * PL) + (lane & 15) * 64 + (lane >> 4) * 16;

    // KS contraction steps from s0 on; the very first step starts the accumulators (no zero fill)
    auto steps = [&](int s0, auto first_tag) {
      constexpr bool FIRST = decltype(first_tag)::value;
      v4i a[KS][RM][PL], b[KS][NTB][PL];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
#pragma unroll
        for (int rm = 0; rm < RM; ++rm)
#pragma unroll
          for (int pl = 0; pl < PL; ++pl) a[s][rm][pl] = *(const v4i *)(Ur[rm] + (size_t)((s0 + s) * PL + pl) * 1024);
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
          for (int pl = 0; pl < PL; ++pl) b[s][tb][pl] = *(const v4i *)(Vt[tb] + (size_t)((s0 + s) * PL + pl) * 1024);
      }
      // every load of the step is issued before its first product (left alone, the scheduler sinks the loads
      // between the products to save registers, and the wave then waits for them one at a time)
      __builtin_amdgcn_sched_barrier(0);
      const v4i zero = (v4i){0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int rm = 0; rm < RM; ++rm)
#pragma unroll
          for (int tb = 0; tb < NTB; ++tb) {
            const bool start = FIRST && s == 0;
            if constexpr (WIDE) {
              acc[0][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][0], b[s][tb][0], start ? zero : acc[0][rm][tb], 0, 0, 0);
              acc[1][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][0], b[s][tb][PL - 1], start ? zero : acc[1][rm][tb], 0, 0, 0);
              acc[1][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][PL - 1], b[s][tb][0], acc[1][rm][tb], 0, 0, 0);
              acc[NACC - 1][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][PL - 1], b[s][tb][PL - 1], start ? zero : acc[NACC - 1][rm][tb], 0, 0, 0);
            } else {
              acc[0][rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm][0], b[s][tb][0], start ? zero : acc[0][rm][tb], 0, 0, 0);
            }
          }
      // 8-bit residues, |U|,|V| <= 127: 512 channels add at most 8.3e6, so reducing every 8 steps keeps
      // |acc| < 2^24.  (Byte planes need nothing here: a step adds at most 2^21 to the middle sum and the plan
      // admits 16-bit moduli only with fewer than 1024 steps.)
      if (!WIDE && (((s0 + KS) & 7) == 0) && (s0 + KS < ncb)) {
#pragma unroll
        for (int rm = 0; rm < RM; ++rm)
#pragma unroll
          for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[0][rm][tb][j] = mod_near(acc[0][rm][tb][j], inv, p);
      }
    };
    steps(0, std::true_type{});
    for (int s0 = KS; s0 < ncb; s0 += KS) steps(s0, std::false_type{});
  } else {
    // a point group's unused byte lanes (t*t not a multiple of 4) are written as zeros
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
      for (int rm = 0; rm < RM; ++rm)
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb) acc[a][rm][tb] = (v4i){0, 0, 0, 0};
  }

  // the four results of a point group become the four bytes of one word, through LDS.  The lane's part of the
  // address is computed once and hidden from the optimiser, so that each byte store carries its (compile-time)
  // row and column as the instruction's immediate offset instead of recomputing the address.
  uint32_t lane_byte = (uint32_t)((4 * (lane >> 4)) * PITCH + (lane & 15) * PL) * 4 + wave;
  asm volatile("" : "+v"(lane_byte));
  uint8_t *tile8 = (uint8_t *)tile + lane_byte;
#pragma unroll
  for (int rm = 0; rm < RM; ++rm)
#pragma unroll
    for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int at = ((rm * 16 + j) * PITCH + tb * 16 * PL) * 4;   // row rm*16 + 4*(lane>>4) + j, column tb*16 + lane%16
        if constexpr (WIDE) {
          const long long tot = (long long)acc[0][rm][tb][j] * 65536 + (long long)acc[1][rm][tb][j] * 256 +
                                (long long)acc[NACC - 1][rm][tb][j];
          const int v = storable16(mod_near64(tot, P.inv_pd[i], p), p);
          const int lo = (int)(int8_t)(v & 0xFF), hi = (v - lo) >> 8;
          tile8[at] = (uint8_t)hi;
          tile8[at + (PL - 1) * 4] = (uint8_t)lo;
        } else {
          tile8[at] = (uint8_t)mod_lowbyte(acc[0][rm][tb][j], inv, -p);
        }
      }
  __syncthreads();
  // O is [Kp][n][Q][Tp] words (x PL) and smaller than 4 GiB: 32-bit word offsets.  16 bytes per thread; whole tile
  // rows are written, padding tiles included (nothing depends on what they hold); only rows >= Kp and tile blocks
  // beyond Tp are left out.
  constexpr int VPR = ROWW / 4;           // 16-byte vectors per tile row
  constexpr int RP = 256 / VPR;           // rows per pass of the block
  const uint32_t krow = (uint32_t)(P.n * P.Q * P.Tp) * PL;
  const int r0 = threadIdx.x / VPR, c4 = threadIdx.x % VPR;
  const int valid_rows = min(ROWS, P.Kp - kb0 * 16);
  const bool vec_ok = tb0 * 16 * PL + 4 * c4 < P.Tp * PL;
  uint32_t off = (uint32_t)(kb0 * 16 + r0) * krow + (uint32_t)((i * P.Q + q) * P.Tp + tb0 * 16) * PL + 4 * c4;
#pragma unroll
  for (int ps = 0; ps < (ROWS + RP - 1) / RP; ++ps) {
    const int row = ps * RP + r0;
    if (vec_ok && row < valid_rows) *(v4i *)(O + off) = *(const v4i *)(tile + row * PITCH + 4 * c4);
    off += RP * krow;
  }
}

}  // namespace rnswino
