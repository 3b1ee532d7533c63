// Memory layouts of the transform-domain tensors U, V, O (device memory).
//
// All three are private to the library: the filter transform writes U, the
// input transform writes V, the residue GEMM reads both and writes O, the
// inverse transform reads O.  They are laid out for the int8 matrix-core
// instruction v_mfma_i32_16x16x64_i8: one operand fragment is 16 rows x 64
// contraction elements = 1 KiB, and lane l of a wavefront holds 16 consecutive
// bytes of row (l % 16), contraction slice g = l / 16.
//
// Contraction (channel) order inside a block of 64 channels: byte b of slice g
// holds channel  16*(b/4) + 4*g + (b%4).  The order of a contraction is free
// as long as both operands agree; this one is what the input-transform kernel
// produces without any cross-lane shuffle (its accumulator rows are channels
// 4*g + j, and four accumulators u = b/4 cover the 64 channels).
//
//   U  [n][t*t][Kp/16][Cp/64][lane = (k%16) + 16*g][16 B]      (fragment-major: a wave reads 1 KiB runs)
//   V  [Tp/16][n][t*t][Cp/64][tile%16][g][16 B]                 (fragment-major: 1 KiB per 16 tiles x 64 channels;
//                               tile block outermost, so that everything one tile produces lies in one region)
//   O  [Kp][n][Q][Tp][4 B]      byte e of the last axis is transform point 4*q + e; k outermost, so that the
//                               n*Q words the inverse transform needs for one (k, tile) lie in one small region
//
// (k, c and tile are the GEMM's row, channel and column: for layers with few channels they are the packed indices
// described in plan.hpp.)
// n moduli, t*t transform points, Cp = C rounded up to 64 (padding channels are
// zero in U), Kp = K rounded up to 16, Tp = T rounded up to 16, Q = ceil(t*t/4).
// For 16-bit moduli a residue is two signed bytes (value = 256*h + l) kept in two
// planes, h first: every U and V fragment becomes 2 KiB ([plane][...]), and every
// O word becomes a pair of words ([..][Tp][plane][4 B]).
#pragma once
#include <cstddef>
#include <cstdint>

#if defined(__HIPCC__)
#define RNSW_HD __host__ __device__ inline
#else
#define RNSW_HD inline
#endif

namespace rnswino {

// position of channel c (0..63) inside its 64-channel block: slice g, byte b
RNSW_HD int chan_pos64(int cc) {
  const int u = cc >> 4, g = (cc >> 2) & 3, j = cc & 3;
  return g * 16 + 4 * u + j;
}

RNSW_HD size_t u_offset(int slab, int k, int c, int Kp, int Cp) {
  const int kb = k >> 4, cb = c >> 6;
  const int pos = chan_pos64(c & 63);            // g*16 + b
  const int g = pos >> 4, b = pos & 15;
  const size_t frag = (size_t)slab * (Kp >> 4) * (Cp >> 6) + (size_t)kb * (Cp >> 6) + cb;
  return frag * 1024 + (size_t)(((k & 15) + 16 * g) * 16 + b);
}

RNSW_HD size_t v_offset(int slab, int nslab, int tau, int c, int Cp) {
  const size_t frag = ((size_t)(tau >> 4) * nslab + slab) * (Cp >> 6) + (c >> 6);
  return frag * 1024 + (size_t)((tau & 15) * 64 + chan_pos64(c & 63));
}

RNSW_HD size_t o_offset(int i, int pt, int k, int tau, int n, int Q, int Kp, int Tp) {
  (void)Kp;
  return ((((size_t)k * n + i) * Q + (pt >> 2)) * Tp + tau) * 4 + (pt & 3);
}

RNSW_HD size_t u_offset_wide(int slab, int k, int c, int Kp, int Cp, int plane) {
  const int kb = k >> 4, cb = c >> 6;
  const int pos = chan_pos64(c & 63);
  const int g = pos >> 4, b = pos & 15;
  const size_t frag = (size_t)slab * (Kp >> 4) * (Cp >> 6) + (size_t)kb * (Cp >> 6) + cb;
  return frag * 2048 + (size_t)plane * 1024 + (size_t)(((k & 15) + 16 * g) * 16 + b);
}

RNSW_HD size_t v_offset_wide(int slab, int nslab, int tau, int c, int Cp, int plane) {
  const size_t frag = ((size_t)(tau >> 4) * nslab + slab) * (Cp >> 6) + (c >> 6);
  return frag * 2048 + (size_t)plane * 1024 + (size_t)((tau & 15) * 64 + chan_pos64(c & 63));
}

RNSW_HD size_t o_offset_wide(int i, int pt, int k, int tau, int n, int Q, int Kp, int Tp, int plane) {
  (void)Kp;
  return (((((size_t)k * n + i) * Q + (pt >> 2)) * Tp + tau) * 2 + plane) * 4 + (pt & 3);
}

}  // namespace rnswino
