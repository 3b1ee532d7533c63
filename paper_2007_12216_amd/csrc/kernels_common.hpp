// Shared device-side definitions of the rnswino kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "layout.hpp"

namespace rnswino {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));

// Everything a kernel needs to know about the layer, passed by value.
struct KParams {
  int N, C, K, H, W, r, m, t, pad;
  int Ho, Wo, th, tw, T, n;
  int TL, Cq, Kg, Tg;         // tile packing of layers with few channels (plan.hpp); TL = 1: none
  int Cp, Kp, Tp, P2, Q;      // GEMM extents (of the packed problem when TL > 1)
  int p[8];
  float inv_p[8];
  double inv_pd[8];           // 1 / p_i
  const int32_t *G;           // device table [n][t*r] for the filter transform
  // transforms on the matrix cores: Kronecker tables in operand-fragment order (see plan_math.cpp)
  int CB1, KS1, RP1, RB3, KS3;
  const int8_t *KB;           // (B^T kron B^T) mod p          [n][CB1][KS1][planes][64 lanes][16]
  const int8_t *KA;           // (A^T kron A^T) crt_inv mod p  [n][RB3][KS3][planes][64 lanes][16]
  uint32_t crt_c[8];          // prod_{l != i} p_l mod 2^32
  uint32_t prod_mod32;        // prod p_i mod 2^32
  int crt24;                  // every prod_{l != i} p_l is below 2^24: 24-bit multiplies suffice
  int quot32;                 // the layer's worst-case |y| is at most 0.45 prod p_i: binary32 finds the CRT quotient
  int bias_p[8];              // p_i * 2^22 + p_i (8-bit moduli), see mod_near_plus_p()
  // fast conversion out of the RNS (k_inverse_crt.hpp): unreduced accumulators that start at acc0 = 2^22
  int fastcrt, acc0;          // fastcrt: 0 = off, 1 = binary32 quotient, 2 = binary64 quotient
  uint32_t crt_sum0;          // -acc0 * sum_i prod_{l != i} p_l mod 2^32
  float crt_fs0;              // -acc0 * sum_i 1/p_i
  double crt_fs0d;            // the same in binary64
  // fused re-quantisation in the inverse-transform kernel (chained layers): 0 = store int32 y,
  // 1 = store int8 clamp(y >> shift), 2 = the same after a 2x2 stride-2 max-pool
  int epi, shift;
  int8_t *act;                // int8 output of modes 1 and 2
};

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by linear workgroup id.  For a grid
// whose x extent is a multiple of 8, this maps block x to a work item such that each XCD gets one contiguous
// chunk of the items: neighbours (which share input lines) then share an L2.  Items >= count are padding.
__device__ __forceinline__ int xcd_chunked(int x, int gx, int count) {
  const int per = gx >> 3;                 // blocks per XCD
  const int item = (x & 7) * per + (x >> 3);
  return item < count ? item : -1;
}

// ---- residues of 8-bit moduli -------------------------------------------------------------------

// Residue of x modulo p for |x| < 2^24 and p <= 253, without division: q = rint(x/p) from one fused
// multiply-add against 1.5*2^23 (whose mantissa then holds q), r = x - q p.  1/p carries a relative error
// of 2^-24, so |x/p - q| <= 1/2 + |x| 2^-24 / p and |r| <= p/2 + 1: a valid representative that fits int8
// (|r| <= 127), not always the canonical one.
__device__ __forceinline__ int mod_near(int x, float inv_p, int p) {
  const float f = __builtin_fmaf((float)x, inv_p, 12582912.0f);
  const int q = __float_as_int(f) - 0x4B400000;
  return x - __mul24(q, p);
}

// Low byte of that residue: the constant term 2^22 * p of the mantissa trick is a multiple of 256 and drops out.
// (Written as the full-rate 24-bit multiply-add itself: since only the low byte is kept, the compiler would
// otherwise swap it for a quarter-rate 64-bit multiply-add.)
__device__ __forceinline__ uint32_t mod_lowbyte(int x, float inv_p, int neg_p) {
  const float f = __builtin_fmaf((float)x, inv_p, 12582912.0f);
  int r;
  asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(__float_as_int(f)), "v"(neg_p), "v"(x));
  return (uint32_t)r;
}

// That residue plus p (so that it is positive), 8-bit p: the low 24 bits of the biased float are 2^22 + q, the
// 24-bit multiply-add gives x - q p - 2^22 p + bias with bias = 2^22 p + p.  Four full-rate instructions.
__device__ __forceinline__ uint32_t mod_near_plus_p(int x, float inv_p, int neg_p, int bias) {
  const float f = __builtin_fmaf((float)x, inv_p, 12582912.0f);
  int r;
  asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(__float_as_int(f)), "v"(neg_p), "v"(x + bias));
  return (uint32_t)r;
}

// byte 0 of a, b, c, d -> one word
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  const uint32_t ab = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);
  const uint32_t cd = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
  return __builtin_amdgcn_perm(cd, ab, 0x05040100u);
}

// ---- residues of 16-bit moduli ------------------------------------------------------------------
// A residue is stored as two signed bytes, value = 256*h + l, which covers [-32896, 32639]; every class
// modulo p <= 65521 has a representative there.

// representative of x modulo p with |r| <= p/2 + 1, |x| < 2^52 (binary64 quotient estimate)
__device__ __forceinline__ int mod_near64(long long x, double inv_pd, int p) {
  const long long q = __double2ll_rn((double)x * inv_pd);
  return (int)(x - q * (long long)p);
}

// move a representative with |r| <= 32761 into the storable range
__device__ __forceinline__ int storable16(int r, int p) { return r > 32639 ? r - p : r; }

__device__ __forceinline__ int sym_mod64(long long v, int p) {   // exact, slow; offline kernels only
  int r = (int)(v % p);
  const int h = (p - 1) >> 1;
  if (r > h) r -= p;
  if (r < -h) r += p;
  return r;
}

}  // namespace rnswino
