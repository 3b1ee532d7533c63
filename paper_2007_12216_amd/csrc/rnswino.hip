// rnswino: C ABI entry points and HIP kernels (gfx950).
//
// Pipeline of one layer (paper section 6):
//   K0  filter transform   U = G g G^T mod p                 (offline, once per weight set)
//   K1  input transform    V = B^T d B mod p                 (per tile, channel, residue)
//   K2  residue GEMM       O = sum_c U V mod p               (per transform point and residue; int8 MFMA)
//   K3  inverse transform  Y = A^T O A mod p, then mixed-radix conversion to int32
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "layout.hpp"
#include "plan.hpp"
#include "rnswino.h"

using namespace rnswino;

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// Everything a kernel needs to know about the layer, passed by value.
struct KParams {
  int N, C, K, H, W, r, m, t, pad;
  int Ho, Wo, th, tw, T, n;
  int Cp, Kp, Tp, P2, Q;
  int p[8];
  float inv_p[8];
  int mrc_inv[8][8];          // mrc_inv[l][j] = p_l^-1 mod p_j  (l < j)
  const int32_t *AT, *G, *BT; // device tables [n][m*t], [n][t*r], [n][t*t]
  // MFMA transforms (8-bit moduli)
  int CB1, KS1, RB3, KS3;
  const int8_t *KB;           // [n][CB1][KS1][64 lanes][16]: (B^T kron B^T) mod p as B-operand fragments
  const int8_t *KA;           // [n][RB3][KS3][64 lanes][16]: (A^T kron A^T) * crt_inv mod p as A-operand fragments
  uint32_t crt_c[8];          // prod_{l != i} p_l mod 2^32
  double inv_pd[8];           // 1 / p_i
  uint32_t prod_mod32;        // prod p_i mod 2^32
  int crt24;                  // every crt_c[i] < 2^24: 24-bit multiplies suffice
};

// ---------------------------------------------------------------------------------------------
// modular helpers
// ---------------------------------------------------------------------------------------------

// exact symmetric residue of a 64-bit value (slow; used off the hot path)
__device__ __forceinline__ int sym_mod64(long long v, int p) {
  int r = (int)(v % p);
  const int h = (p - 1) >> 1;
  if (r > h) r -= p;
  if (r < -h) r += p;
  return r;
}

// Residue of x modulo p for |x| < 2^24 and p <= 253, without division: q = rint(x/p) from one fused
// multiply-add against 1.5*2^23 (whose mantissa then holds q), r = x - q p.  1/p carries a relative error
// of 2^-24, so |x/p - q| <= 1/2 + |x| 2^-24 / p and |r| <= p/2 + 1: a valid representative that fits int8
// (|r| <= 127), not always the canonical one.
__device__ __forceinline__ int mod_near(int x, float inv_p, int p) {
  const float f = __builtin_fmaf((float)x, inv_p, 12582912.0f);
  const int q = __float_as_int(f) - 0x4B400000;
  return x - __mul24(q, p);
}

// low byte of the residue of x (|x| < 2^24): the mantissa trick of mod_near with the constant term dropped,
// because 2^22 * p is a multiple of 256
__device__ __forceinline__ uint32_t mod_lowbyte(int x, float inv_p, int neg_p) {
  const float f = __builtin_fmaf((float)x, inv_p, 12582912.0f);
  return (uint32_t)(__mul24(__float_as_int(f), neg_p) + x);
}

__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  const uint32_t ab = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);
  const uint32_t cd = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
  return __builtin_amdgcn_perm(cd, ab, 0x05040100u);
}

// ---------------------------------------------------------------------------------------------
// K0: filter transform (offline).  One thread per (residue, k, c) of the padded K x C grid.
// ---------------------------------------------------------------------------------------------
template <typename RT>
__global__ void k0_filter_transform(KParams P, const int8_t *__restrict__ w, RT *__restrict__ U) {
  const long long total = (long long)P.n * P.Kp * P.Cp;
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c = (int)(idx % P.Cp); idx /= P.Cp;
  const int k = (int)(idx % P.Kp);
  const int i = (int)(idx / P.Kp);
  const int p = P.p[i], t = P.t, r = P.r;
  const int32_t *G = P.G + (size_t)i * t * r;
  int g[25];
  const bool live = (k < P.K) && (c < P.C);
  for (int e = 0; e < r * r; ++e) g[e] = live ? (int)w[((size_t)k * P.C + c) * r * r + e] : 0;
  for (int xi = 0; xi < t; ++xi) {
    long long row[5];
    for (int b = 0; b < r; ++b) {
      long long s = 0;
      for (int a = 0; a < r; ++a) s += (long long)G[xi * r + a] * g[a * r + b];
      row[b] = s;
    }
    for (int nu = 0; nu < t; ++nu) {
      long long s = 0;
      for (int b = 0; b < r; ++b) s += row[b] * G[nu * r + b];
      U[u_offset(i * P.P2 + xi * t + nu, k, c, P.Kp, P.Cp)] = (RT)sym_mod64(s, p);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// K1 (plain version): one thread per (residue, tile, channel, column nu) computes column nu of B^T d B.
// ---------------------------------------------------------------------------------------------
template <typename RT>
__global__ void k1_input_transform_plain(KParams P, const int8_t *__restrict__ x, RT *__restrict__ V) {
  const int t = P.t;
  const long long total = (long long)P.n * P.T * P.Cp * t;
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int c = (int)(idx % P.Cp); idx /= P.Cp;
  const int nu = (int)(idx % t); idx /= t;
  const int tau = (int)(idx % P.T);
  const int i = (int)(idx / P.T);
  const int p = P.p[i];
  const int32_t *BT = P.BT + (size_t)i * t * t;
  if (c >= P.C) {
    for (int xi = 0; xi < t; ++xi) V[v_offset(i * P.P2 + xi * t + nu, tau, c, P.Tp, P.Cp)] = 0;
    return;
  }
  const int tx = tau % P.tw, ty = (tau / P.tw) % P.th, img = tau / (P.tw * P.th);
  const int y0 = ty * P.m - P.pad, x0 = tx * P.m - P.pad;
  const int8_t *plane = x + ((size_t)img * P.C + c) * P.H * P.W;
  int e[16];
  for (int a = 0; a < t; ++a) {
    long long s = 0;
    const int gy = y0 + a;
    if (gy >= 0 && gy < P.H)
      for (int b = 0; b < t; ++b) {
        const int gx = x0 + b;
        if (gx >= 0 && gx < P.W) s += (long long)plane[(size_t)gy * P.W + gx] * BT[nu * t + b];
      }
    e[a] = sym_mod64(s, p);
  }
  for (int xi = 0; xi < t; ++xi) {
    long long s = 0;
    for (int a = 0; a < t; ++a) s += (long long)BT[xi * t + a] * e[a];
    V[v_offset(i * P.P2 + xi * t + nu, tau, c, P.Tp, P.Cp)] = (RT)sym_mod64(s, p);
  }
}


// ---------------------------------------------------------------------------------------------
// K1, 8-bit moduli, on the matrix cores.  B^T d B = (B^T kron B^T) vec(d): per residue one dense
// (t*t) x (t*t) int8 matrix applied to the t*t pixels of a tile, i.e. a GEMM whose columns are the
// (tile, channel) pairs.  MFMA roles: A operand = pixels (rows = 16 channels of one tile), B operand =
// the Kronecker table (columns = 16 transform points), contraction index = pixel.  A contraction step
// of 64 covers four tile rows of 16 pixels each (lane group g = row 4s+g; columns >= t have weight 0),
// so a lane's 16 operand bytes are 16 consecutive pixels of one image row: one unaligned 16-byte load,
// masked where the tile hangs over the image border.
//
// Block = (tile, block of 64 channels, residue): its 64 x t x 16 pixel patch is gathered once into LDS
// (the gather of 16-byte row segments is what costs; sharing it between the four waves pays), then each
// wave takes every fourth group of K1_CPW column blocks.  Accumulator rows are channels 4g+j, so the four
// channel groups u give one lane exactly the 16 bytes of V it has to store (channel order of layout.hpp).
// Grid: x = T * Cp/64, y = n; 256 threads; 64 * 4*KS1 * 16 bytes of LDS.
// ---------------------------------------------------------------------------------------------
constexpr int K1_CPW = 2;

template <int KS1>
__global__ __launch_bounds__(256) void k1_input_transform_i8(KParams P, const int8_t *__restrict__ x,
                                                              int8_t *__restrict__ V) {
  constexpr int ROWS = 4 * KS1;
  __shared__ __attribute__((aligned(16))) uint8_t xs[64 * ROWS * 16];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, g = lane >> 4;
  const int ncb = P.Cp >> 6;
  const int i = blockIdx.y;
  const int cb = blockIdx.x % ncb, tau = blockIdx.x / ncb;
  const int tx = tau % P.tw, ty = (tau / P.tw) % P.th, img = tau / (P.tw * P.th);
  const int y0 = ty * P.m - P.pad, x0 = tx * P.m - P.pad;
  {
    // columns b of the 16-pixel row segment that lie inside the image and inside the tile: [lo, hi)
    const int lo = x0 < 0 ? -x0 : 0;
    const int hi = min(P.t, P.W - x0);
    uint32_t cmask[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      uint32_t mk = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) mk |= ((4 * d + e) >= lo && (4 * d + e) < hi) ? (0xFFu << (8 * e)) : 0u;
      cmask[d] = mk;
    }
    const long long total = (long long)P.N * P.C * P.H * P.W;
    for (int task = threadIdx.x; task < 64 * ROWS; task += 256) {
      const int c = task / ROWS, a = task - c * ROWS;
      const int gc = cb * 64 + c, gy = y0 + a;
      v4i val = (v4i){0, 0, 0, 0};
      if (gc < P.C && a < P.t && gy >= 0 && gy < P.H) {
        const long long b0 = (((long long)img * P.C + gc) * P.H + gy) * P.W + x0;
        if (b0 >= 0 && b0 + 16 <= total) {
          __builtin_memcpy(&val, x + b0, 16);          // one unaligned 16-byte load
        } else {                                       // first / last bytes of the tensor
          uint32_t wv[4] = {0, 0, 0, 0};
          for (int b = 0; b < 16; ++b) {
            const long long o = b0 + b;
            if (o >= 0 && o < total) wv[b >> 2] |= (uint32_t)(uint8_t)x[o] << (8 * (b & 3));
          }
          val = (v4i){(int)wv[0], (int)wv[1], (int)wv[2], (int)wv[3]};
        }
        val[0] &= cmask[0]; val[1] &= cmask[1]; val[2] &= cmask[2]; val[3] &= cmask[3];
      }
      *(v4i *)(xs + task * 16) = val;
    }
  }
  // table fragments of this wave's first column-block group: issued before the barrier so that their latency
  // overlaps the gather
  const int ncg = (P.CB1 + K1_CPW - 1) / K1_CPW;
  v4i bf[K1_CPW][KS1];
#pragma unroll
  for (int cc = 0; cc < K1_CPW; ++cc)
#pragma unroll
    for (int s = 0; s < KS1; ++s) {
      const int cbk = min(wave * K1_CPW + cc, P.CB1 - 1);
      bf[cc][s] = *(const v4i *)(P.KB + (((size_t)i * P.CB1 + cbk) * KS1 + s) * 1024 + lane * 16);
    }
  __syncthreads();

  v4i af[4][KS1];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int s = 0; s < KS1; ++s) af[u][s] = *(const v4i *)(xs + ((16 * u + (lane & 15)) * ROWS + 4 * s + g) * 16);

  const int neg_p = -P.p[i];
  const float inv = P.inv_p[i];
  for (int cg = wave; cg < ncg; cg += 4) {
    if (cg != wave) {
#pragma unroll
      for (int cc = 0; cc < K1_CPW; ++cc)
#pragma unroll
        for (int s = 0; s < KS1; ++s) {
          const int cbk = min(cg * K1_CPW + cc, P.CB1 - 1);
          bf[cc][s] = *(const v4i *)(P.KB + (((size_t)i * P.CB1 + cbk) * KS1 + s) * 1024 + lane * 16);
        }
    }
#pragma unroll
    for (int cc = 0; cc < K1_CPW; ++cc) {
      const int cbk = cg * K1_CPW + cc;
      if (cbk >= P.CB1) break;
      v4i acc[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] = (v4i){0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KS1; ++s) {
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[u][s], bf[cc][s], acc[u], 0, 0, 0);
      }
      // |acc| <= t*t * 126 * 128 < 2^24
      v4i out;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        out[u] = (int)pack_low_bytes(mod_lowbyte(acc[u][0], inv, neg_p), mod_lowbyte(acc[u][1], inv, neg_p),
                                     mod_lowbyte(acc[u][2], inv, neg_p), mod_lowbyte(acc[u][3], inv, neg_p));
      const int pt = 16 * cbk + (lane & 15);
      if (pt < P.P2)
        *(v4i *)(V + (((size_t)(i * P.P2 + pt) * (P.Tp >> 4) + (tau >> 4)) * ncb + cb) * 1024 + (tau & 15) * 64 + g * 16) = out;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// K3, 8-bit moduli, on the matrix cores, fused with the conversion out of the RNS.
// A^T O A = (A^T kron A^T) vec(O): per residue an (m*m) x (t*t) int8 matrix applied to the t*t transform
// points of a (channel k, tile) pair.  MFMA roles: A operand = the Kronecker table (rows = 16 outputs),
// B operand = O (columns = 16 consecutive tiles of one channel k), contraction index = transform point;
// a lane's 16 operand bytes are four O words (groups q = 16s + 4g + e).
// The table rows are pre-multiplied by (P/p_i)^-1 mod p_i, so that the accumulator w_i is the CRT
// coefficient of residue i and  y = sum_i (P/p_i) w_i - P * rint(sum_i w_i / p_i)  (mod 2^32) is the
// representative of the result in [-(P-1)/2, (P-1)/2]; any representative of w_i gives the same y.
// The rounding is done in binary64: sum_i w_i/p_i = y/P + integer with |y/P| <= 1/2 - 1/(2P), and
// the error of the sum is below 1e-14.
// Block = one (k, block of 16 tiles); its waves take the 16-output row blocks rb = wave, wave+4, ...
// (four waves cover an 8x8 output tile); every wave loads the O operand itself (the copies hit in L1).
// No LDS.  Grid: K * Tp/16 blocks of 256 threads.
// ---------------------------------------------------------------------------------------------
template <int NRES, int KS3>
__global__ __launch_bounds__(256) void k3_inverse_crt_i8(KParams P, const uint32_t *__restrict__ O,
                                                          int32_t *__restrict__ y) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, g = lane >> 4;
  if (wave >= P.RB3) return;
  const int ntb = P.Tp >> 4;
  const int k = blockIdx.x / ntb, tb = blockIdx.x % ntb;
  const int tau = tb * 16 + (lane & 15);

  v4i of[NRES][KS3];
#pragma unroll
  for (int i = 0; i < NRES; ++i)
#pragma unroll
    for (int s = 0; s < KS3; ++s)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int q = 16 * s + 4 * g + e;
        of[i][s][e] = (q < P.Q && tau < P.T) ? (int)O[(((size_t)i * P.Q + q) * P.Kp + k) * P.Tp + tau] : 0;
      }

  const int m = P.m, mm = m * m;
  const bool tile_ok = tau < P.T;
  const int tx = tau % P.tw, ty = (tau / P.tw) % P.th, img = tau / (P.tw * P.th);
  int32_t *yplane = y + ((size_t)img * P.K + k) * P.Ho * P.Wo;
  const float inv_m = 1.0f / (float)m;
  const bool vec4 = ((m & 3) == 0) && ((P.Wo & 3) == 0);   // four consecutive outputs stay in one row, 16-byte aligned

  for (int rb = wave; rb < P.RB3; rb += 4) {
    uint32_t w[NRES][4];
#pragma unroll
    for (int i = 0; i < NRES; ++i) {
      v4i acc = (v4i){0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KS3; ++s) {
        const v4i a = *(const v4i *)(P.KA + (((size_t)i * P.RB3 + rb) * KS3 + s) * 1024 + lane * 16);
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, of[i][s], acc, 0, 0, 0);
      }
      // |acc| <= t*t * 126 * 127 < 2^24; residue shifted by +p so that it is non-negative (0 <= w < 2p + 2)
#pragma unroll
      for (int j = 0; j < 4; ++j) w[i][j] = (uint32_t)(mod_near(acc[j], P.inv_p[i], P.p[i]) + P.p[i]);
    }
    int val[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t sum = 0;
      double fs = 0.0;
#pragma unroll
      for (int i = 0; i < NRES; ++i) {
        sum += P.crt24 ? __umul24(P.crt_c[i], w[i][j]) : P.crt_c[i] * w[i][j];
        fs = __builtin_fma((double)w[i][j], P.inv_pd[i], fs);
      }
      const int kk = __double2int_rn(fs);
      val[j] = (int)(sum - P.prod_mod32 * (uint32_t)kk);
    }
    const int o0 = 16 * rb + 4 * g;
    if (!tile_ok || o0 >= mm) continue;
    if (vec4) {
      const int u = (int)(((float)o0 + 0.5f) * inv_m);
      const int v = o0 - u * m;
      const int oy = ty * m + u, ox = tx * m + v;
      if (oy < P.Ho && ox < P.Wo) *(v4i *)(yplane + (size_t)oy * P.Wo + ox) = (v4i){val[0], val[1], val[2], val[3]};
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int o = o0 + j;
        const int u = (int)(((float)o + 0.5f) * inv_m);
        const int v = o - u * m;
        const int oy = ty * m + u, ox = tx * m + v;
        if (o < mm && oy < P.Ho && ox < P.Wo) yplane[(size_t)oy * P.Wo + ox] = val[j];
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// K2, 8-bit moduli: O = U V^T mod p on v_mfma_i32_16x16x64_i8.
// Block = 4 waves = the 4 transform points of one group q (they end up as the 4 bytes of one O word);
// every wave computes a 32 (k) x 64 (tile) block of its point over the whole of C.
// Grid: x = n*Q, y = ceil(Kp/32), z = ceil(Tp/64).
// KS = contraction steps (of 64 channels) whose operand fragments are loaded before any is consumed.
// ---------------------------------------------------------------------------------------------
template <int KS>
__global__ __launch_bounds__(256) void k2_gemm_i8(KParams P, const int8_t *__restrict__ U,
                                                   const int8_t *__restrict__ V, uint32_t *__restrict__ O) {
  __shared__ uint32_t tile[32 * 64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x / P.Q, q = blockIdx.x % P.Q;
  const int pt = 4 * q + wave;
  const int nkb = P.Kp >> 4, ntb = P.Tp >> 4, ncb = P.Cp >> 6;
  const int kb0 = blockIdx.y * 2, tb0 = blockIdx.z * 4;
  const int p = P.p[i];
  const float inv = P.inv_p[i];

  v4i acc[2][4];
#pragma unroll
  for (int rm = 0; rm < 2; ++rm)
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) acc[rm][tb] = (v4i){0, 0, 0, 0};

  if (pt < P.P2) {
    const int slab = i * P.P2 + pt;
    const int8_t *Ub = U + (size_t)slab * nkb * ncb * 1024 + lane * 16;
    const int8_t *Vb = V + (size_t)slab * ntb * ncb * 1024 + (lane & 15) * 64 + (lane >> 4) * 16;
    for (int s0 = 0; s0 < ncb; s0 += KS) {
      v4i a[KS][2], b[KS][4];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
#pragma unroll
        for (int rm = 0; rm < 2; ++rm) {
          a[s][rm] = (v4i){0, 0, 0, 0};
          if (kb0 + rm < nkb) a[s][rm] = *(const v4i *)(Ub + ((size_t)(kb0 + rm) * ncb + s0 + s) * 1024);
        }
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {
          b[s][tb] = (v4i){0, 0, 0, 0};
          if (tb0 + tb < ntb) b[s][tb] = *(const v4i *)(Vb + ((size_t)(tb0 + tb) * ncb + s0 + s) * 1024);
        }
      }
#pragma unroll
      for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int rm = 0; rm < 2; ++rm)
#pragma unroll
          for (int tb = 0; tb < 4; ++tb)
            acc[rm][tb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s][rm], b[s][tb], acc[rm][tb], 0, 0, 0);
      // |U|,|V| <= 127: 512 channels add at most 8.3e6, so reducing every 8 steps keeps |acc| < 2^24
      if ((((s0 + KS) & 7) == 0) && (s0 + KS < ncb)) {
#pragma unroll
        for (int rm = 0; rm < 2; ++rm)
#pragma unroll
          for (int tb = 0; tb < 4; ++tb)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[rm][tb][j] = mod_near(acc[rm][tb][j], inv, p);
      }
    }
  }

  uint8_t *tile8 = (uint8_t *)tile;
#pragma unroll
  for (int rm = 0; rm < 2; ++rm)
#pragma unroll
    for (int tb = 0; tb < 4; ++tb)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = rm * 16 + 4 * (lane >> 4) + j, col = tb * 16 + (lane & 15);
        tile8[(row * 64 + col) * 4 + wave] = (uint8_t)mod_lowbyte(acc[rm][tb][j], inv, -p);
      }
  __syncthreads();
  uint32_t *Ob = O + ((size_t)i * P.Q + q) * P.Kp * P.Tp;
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int e = it * 256 + threadIdx.x;
    const int row = e >> 6, col = e & 63;
    const int k = kb0 * 16 + row, tau = tb0 * 16 + col;
    if (k < P.Kp && tau < P.T) Ob[(size_t)k * P.Tp + tau] = tile[e];   // padding tiles are neither written nor read
  }
}

// K2 (plain version, any modulus width): one thread per output element, 64-bit accumulation.
template <typename RT>
__global__ void k2_gemm_plain(KParams P, const RT *__restrict__ U, const RT *__restrict__ V, RT *__restrict__ O) {
  const long long total = (long long)P.n * P.P2 * P.K * P.T;
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int tau = (int)(idx % P.T); idx /= P.T;
  const int k = (int)(idx % P.K); idx /= P.K;
  const int pt = (int)(idx % P.P2);
  const int i = (int)(idx / P.P2);
  long long s = 0;
  for (int c = 0; c < P.C; ++c)
    s += (long long)U[u_offset(i * P.P2 + pt, k, c, P.Kp, P.Cp)] * (long long)V[v_offset(i * P.P2 + pt, tau, c, P.Tp, P.Cp)];
  O[o_offset(i, pt, k, tau, P.Q, P.Kp, P.Tp)] = (RT)sym_mod64(s, P.p[i]);
}

// ---------------------------------------------------------------------------------------------
// K3 (plain version): one thread per (k, tile, output column v): column v of A^T O A for every residue,
// then mixed-radix conversion (symmetric digits) and the store of m outputs.
// ---------------------------------------------------------------------------------------------
template <typename RT>
__global__ void k3_inverse_mrc_plain(KParams P, const RT *__restrict__ O, int32_t *__restrict__ y) {
  const int t = P.t, m = P.m;
  const long long total = (long long)P.K * P.T * m;
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int tau = (int)(idx % P.T); idx /= P.T;
  const int v = (int)(idx % m);
  const int k = (int)(idx / m);
  const int tx = tau % P.tw, ty = (tau / P.tw) % P.th, img = tau / (P.tw * P.th);
  const int ox = tx * m + v;
  if (ox >= P.Wo) return;
  int digits[8];
  for (int u = 0; u < m; ++u) {
    const int oy = ty * m + u;
    if (oy >= P.Ho) break;
    for (int i = 0; i < P.n; ++i) {
      const int p = P.p[i];
      const int32_t *AT = P.AT + (size_t)i * m * t;
      long long s = 0;
      for (int xi = 0; xi < t; ++xi) {
        long long e = 0;
        for (int nu = 0; nu < t; ++nu)
          e += (long long)O[o_offset(i, xi * t + nu, k, tau, P.Q, P.Kp, P.Tp)] * AT[v * t + nu];
        s += (long long)AT[u * t + xi] * sym_mod64(e, p);
      }
      long long d = sym_mod64(s, p);
      for (int l = 0; l < i; ++l) d = sym_mod64((d - digits[l]) * (long long)P.mrc_inv[l][i], p);
      digits[i] = (int)d;
    }
    uint32_t val = (uint32_t)digits[P.n - 1];
    for (int j = P.n - 2; j >= 0; --j) val = (uint32_t)digits[j] + (uint32_t)P.p[j] * val;
    y[(((size_t)img * P.K + k) * P.Ho + oy) * P.Wo + ox] = (int32_t)val;
  }
}

// ---------------------------------------------------------------------------------------------
// Layer glue: a = clamp(y >> shift, -128, 127), optional 2x2 max-pool.
// ---------------------------------------------------------------------------------------------
__global__ void k_requant_pool(const int32_t *__restrict__ y, int8_t *__restrict__ a, long long planes, int H, int W,
                               int shift, int pool) {
  const int Hq = pool ? H / 2 : H, Wq = pool ? W / 2 : W;
  const long long total = planes * Hq * Wq;
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int xx = (int)(idx % Wq);
    const int yy = (int)((idx / Wq) % Hq);
    const long long pl = idx / ((long long)Wq * Hq);
    int best;
    if (pool) {
      const int32_t *src = y + (pl * H + 2 * yy) * W + 2 * xx;
      best = max(max(src[0], src[1]), max(src[W], src[W + 1]));
    } else {
      best = y[idx];
    }
    best >>= shift;   // arithmetic shift: floor division; monotone, so it commutes with the max
    best = min(127, max(-128, best));
    a[idx] = (int8_t)best;
  }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------

KParams make_params(const rnswino_plan_t *pl) {
  KParams P;
  std::memset(&P, 0, sizeof(P));
  const Dims &d = pl->dims;
  P.N = d.N; P.C = d.C; P.K = d.K; P.H = d.H; P.W = d.W; P.r = d.r; P.m = d.m; P.t = d.t; P.pad = d.pad;
  P.Ho = d.Ho; P.Wo = d.Wo; P.th = d.th; P.tw = d.tw; P.T = d.T; P.n = d.n;
  P.Cp = d.Cp; P.Kp = d.Kp; P.Tp = d.Tp; P.P2 = d.P2; P.Q = d.Q;
  for (int i = 0; i < d.n; ++i) {
    P.p[i] = (int)pl->desc.moduli[i];
    P.inv_p[i] = 1.0f / (float)pl->desc.moduli[i];
    for (int j = 0; j < d.n; ++j) P.mrc_inv[i][j] = (int)pl->mrc_inv[i][j];
  }
  const char *base = (const char *)pl->d_tables;
  P.AT = (const int32_t *)(base + pl->off_AT);
  P.G = (const int32_t *)(base + pl->off_G);
  P.BT = (const int32_t *)(base + pl->off_BT);
  P.CB1 = d.CB1; P.KS1 = d.KS1; P.RB3 = d.RB3; P.KS3 = d.KS3;
  P.KB = (const int8_t *)(base + pl->off_KB);
  P.KA = (const int8_t *)(base + pl->off_KA);
  for (int i = 0; i < d.n; ++i) {
    P.crt_c[i] = pl->crt_c[i];
    P.inv_pd[i] = 1.0 / (double)pl->desc.moduli[i];
  }
  P.prod_mod32 = pl->prod_mod32;
  P.crt24 = 1;
  for (int i = 0; i < d.n; ++i)
    if (pl->crt_c_exact_small[i] == 0) P.crt24 = 0;
  return P;
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline size_t elem_bytes(const Dims &d) { return d.wide ? 2 : 1; }
inline size_t v_bytes(const Dims &d) { return (size_t)d.n * d.P2 * d.Tp * d.Cp * elem_bytes(d); }
inline size_t o_bytes(const Dims &d) { return (size_t)d.n * d.Q * d.Kp * d.Tp * 4 * elem_bytes(d); }
inline size_t u_bytes(const Dims &d) { return (size_t)d.n * d.P2 * d.Kp * d.Cp * elem_bytes(d); }

inline int launch_status() { return hipGetLastError() == hipSuccess ? RNSWINO_OK : RNSWINO_E_HIP; }

inline unsigned blocks_for(long long total, int bs) { return (unsigned)((total + bs - 1) / bs); }

template <int NRES>
void launch_k3_nres(const Dims &d, const KParams &P, const uint32_t *O, int32_t *y, hipStream_t st) {
  const dim3 grid((unsigned)(d.K * (d.Tp / 16)));
  switch (d.KS3) {
    case 1: hipLaunchKernelGGL((k3_inverse_crt_i8<NRES, 1>), grid, dim3(256), 0, st, P, O, y); break;
    case 2: hipLaunchKernelGGL((k3_inverse_crt_i8<NRES, 2>), grid, dim3(256), 0, st, P, O, y); break;
    case 3: hipLaunchKernelGGL((k3_inverse_crt_i8<NRES, 3>), grid, dim3(256), 0, st, P, O, y); break;
    default: hipLaunchKernelGGL((k3_inverse_crt_i8<NRES, 4>), grid, dim3(256), 0, st, P, O, y); break;
  }
}

void launch_k3_i8(const Dims &d, const KParams &P, const uint32_t *O, int32_t *y, hipStream_t st) {
  switch (d.n) {
    case 1: launch_k3_nres<1>(d, P, O, y, st); break;
    case 2: launch_k3_nres<2>(d, P, O, y, st); break;
    case 3: launch_k3_nres<3>(d, P, O, y, st); break;
    case 4: launch_k3_nres<4>(d, P, O, y, st); break;
    case 5: launch_k3_nres<5>(d, P, O, y, st); break;
    case 6: launch_k3_nres<6>(d, P, O, y, st); break;
    case 7: launch_k3_nres<7>(d, P, O, y, st); break;
    default: launch_k3_nres<8>(d, P, O, y, st); break;
  }
}

}  // namespace

// =============================================================================================
// C ABI
// =============================================================================================

extern "C" {

int rnswino_plan(rnswino_plan_t **out, const rnswino_desc_t *desc) {
  if (out) *out = nullptr;
  if (!out || !desc) return RNSWINO_E_INVALID;
  rnswino_plan_t *pl = new (std::nothrow) rnswino_plan_t();
  if (!pl) return RNSWINO_E_INVALID;
  pl->desc = *desc;
  pl->device = -1;
  pl->d_tables = nullptr;
  pl->d_tables_bytes = 0;
  int rc = validate_desc(*desc, pl->dims);
  if (rc != RNSWINO_OK) { delete pl; return rc; }
  const Dims &d = pl->dims;
  pl->tf.resize(d.n);
  for (int i = 0; i < d.n; ++i) {
    rc = build_transforms(d.m, d.r, desc->moduli[i], pl->tf[i]);
    if (rc != RNSWINO_OK) { delete pl; return rc; }
  }
  // dynamic range (prod - 1)/2, saturated, against the worst case 2^14 r^2 C (sections 3, 5, 8)
  unsigned __int128 prod = 1;
  const unsigned __int128 cap = ((unsigned __int128)1 << 100);
  for (int i = 0; i < d.n; ++i) { prod *= desc->moduli[i]; if (prod > cap) prod = cap; }
  const unsigned __int128 half = (prod - 1) / 2;
  pl->dyn_range = half > (unsigned __int128)INT64_MAX ? INT64_MAX : (int64_t)half;
  const unsigned __int128 worst = (unsigned __int128)16384u * (unsigned)d.r * (unsigned)d.r * (unsigned)d.C;
  if (!(desc->flags & RNSWINO_FLAG_ALLOW_UNCHECKED_RANGE) && worst > half) { delete pl; return RNSWINO_E_RANGE; }
  std::memset(pl->mrc_inv, 0, sizeof(pl->mrc_inv));
  for (int l = 0; l < d.n; ++l)
    for (int j = l + 1; j < d.n; ++j) pl->mrc_inv[l][j] = (uint32_t)mod_inverse(desc->moduli[l], desc->moduli[j]);

  // device tables
  const size_t szAT = (size_t)d.n * d.m * d.t * 4, szG = (size_t)d.n * d.t * d.r * 4, szBT = (size_t)d.n * d.t * d.t * 4;
  pl->off_AT = 0;
  pl->off_G = align256(pl->off_AT + szAT);
  pl->off_BT = align256(pl->off_G + szG);
  // CRT constants: c_i = prod_{l != i} p_l (mod 2^32), its inverse modulo p_i, and P mod 2^32
  pl->prod_mod32 = 1;
  for (int i = 0; i < d.n; ++i) {
    uint32_t c32 = 1;
    int64_t cmod = 1;
    for (int l = 0; l < d.n; ++l)
      if (l != i) { c32 *= desc->moduli[l]; cmod = (cmod * (int64_t)desc->moduli[l]) % (int64_t)desc->moduli[i]; }
    pl->crt_c[i] = c32;
    {
      unsigned __int128 full = 1;
      for (int l = 0; l < d.n; ++l)
        if (l != i) { full *= desc->moduli[l]; if (full > ((unsigned __int128)1 << 40)) full = (unsigned __int128)1 << 40; }
      pl->crt_c_exact_small[i] = full < ((unsigned __int128)1 << 24) ? 1 : 0;
    }
    pl->crt_inv[i] = (uint32_t)mod_inverse(cmod, desc->moduli[i]);
    pl->prod_mod32 *= desc->moduli[i];
  }
  const size_t szKB = d.wide ? 0 : (size_t)d.n * d.CB1 * d.KS1 * 1024;
  const size_t szKA = d.wide ? 0 : (size_t)d.n * d.RB3 * d.KS3 * 1024;
  pl->off_KB = align256(pl->off_BT + szBT);
  pl->off_KA = align256(pl->off_KB + szKB);
  pl->d_tables_bytes = align256(pl->off_KA + szKA);
  if (!(desc->flags & RNSWINO_FLAG_HOST_ONLY)) {
    std::vector<char> host(pl->d_tables_bytes, 0);
    for (int i = 0; i < d.n; ++i) {
      std::memcpy(host.data() + pl->off_AT + (size_t)i * d.m * d.t * 4, pl->tf[i].AT.data(), (size_t)d.m * d.t * 4);
      std::memcpy(host.data() + pl->off_G + (size_t)i * d.t * d.r * 4, pl->tf[i].G.data(), (size_t)d.t * d.r * 4);
      std::memcpy(host.data() + pl->off_BT + (size_t)i * d.t * d.t * 4, pl->tf[i].BT.data(), (size_t)d.t * d.t * 4);
    }
    if (!d.wide) {
      // Kronecker tables in MFMA fragment order: lane = (row or column % 16) + 16*g, 16 bytes per lane
      for (int i = 0; i < d.n; ++i) {
        const int64_t p = desc->moduli[i];
        const std::vector<int32_t> &BT = pl->tf[i].BT, &AT = pl->tf[i].AT;
        int8_t *kb = (int8_t *)host.data() + pl->off_KB + (size_t)i * d.CB1 * d.KS1 * 1024;
        for (int cbk = 0; cbk < d.CB1; ++cbk)
          for (int s = 0; s < d.KS1; ++s)
            for (int lane = 0; lane < 64; ++lane)
              for (int b = 0; b < 16; ++b) {
                const int pt = 16 * cbk + (lane & 15), a = 4 * s + (lane >> 4);
                int32_t v = 0;
                if (pt < d.P2 && a < d.t && b < d.t)
                  v = sym_residue((int64_t)BT[(size_t)(pt / d.t) * d.t + a] * BT[(size_t)(pt % d.t) * d.t + b], p);
                kb[((size_t)(cbk * d.KS1 + s) * 64 + lane) * 16 + b] = (int8_t)v;
              }
        int8_t *ka = (int8_t *)host.data() + pl->off_KA + (size_t)i * d.RB3 * d.KS3 * 1024;
        for (int rb = 0; rb < d.RB3; ++rb)
          for (int s = 0; s < d.KS3; ++s)
            for (int lane = 0; lane < 64; ++lane)
              for (int b = 0; b < 16; ++b) {
                const int o = 16 * rb + (lane & 15), pt = 64 * s + 16 * (lane >> 4) + b;
                int32_t v = 0;
                if (o < d.m * d.m && pt < d.P2) {
                  const int64_t aa = (int64_t)AT[(size_t)(o / d.m) * d.t + pt / d.t] * AT[(size_t)(o % d.m) * d.t + pt % d.t];
                  v = sym_residue((aa % p) * (int64_t)pl->crt_inv[i], p);
                }
                ka[((size_t)(rb * d.KS3 + s) * 64 + lane) * 16 + b] = (int8_t)v;
              }
      }
    }
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); delete pl; return RNSWINO_E_NO_DEVICE; }
    if (hipMalloc(&pl->d_tables, pl->d_tables_bytes) != hipSuccess) { (void)hipGetLastError(); delete pl; return RNSWINO_E_HIP; }
    if (hipMemcpy(pl->d_tables, host.data(), pl->d_tables_bytes, hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipGetLastError(); (void)hipFree(pl->d_tables); delete pl; return RNSWINO_E_HIP;
    }
    pl->device = dev;
  }
  *out = pl;
  return RNSWINO_OK;
}

int rnswino_plan_destroy(rnswino_plan_t *plan) {
  if (!plan) return RNSWINO_E_INVALID;
  int rc = RNSWINO_OK;
  if (plan->d_tables && hipFree(plan->d_tables) != hipSuccess) { (void)hipGetLastError(); rc = RNSWINO_E_HIP; }
  delete plan;
  return rc;
}

int rnswino_output_dims(const rnswino_plan_t *plan, int32_t *Ho, int32_t *Wo) {
  if (!plan || !Ho || !Wo) return RNSWINO_E_INVALID;
  *Ho = plan->dims.Ho; *Wo = plan->dims.Wo;
  return RNSWINO_OK;
}

size_t rnswino_filter_bytes(const rnswino_plan_t *plan) { return plan ? align256(u_bytes(plan->dims)) : 0; }

size_t rnswino_workspace_bytes(const rnswino_plan_t *plan) {
  return plan ? align256(v_bytes(plan->dims)) + align256(o_bytes(plan->dims)) : 0;
}

int rnswino_filter_transform(const rnswino_plan_t *plan, const int8_t *w_dev, void *U_dev, void *stream) {
  if (!plan || !w_dev || !U_dev) return RNSWINO_E_INVALID;
  if (plan->device < 0) return RNSWINO_E_NO_DEVICE;
  const Dims &d = plan->dims;
  const KParams P = make_params(plan);
  const long long total = (long long)d.n * d.Kp * d.Cp;
  hipStream_t st = (hipStream_t)stream;
  if (d.wide)
    hipLaunchKernelGGL(k0_filter_transform<int16_t>, dim3(blocks_for(total, 256)), dim3(256), 0, st, P, w_dev, (int16_t *)U_dev);
  else
    hipLaunchKernelGGL(k0_filter_transform<int8_t>, dim3(blocks_for(total, 256)), dim3(256), 0, st, P, w_dev, (int8_t *)U_dev);
  return launch_status();
}

static int conv2d_impl(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int32_t *y_dev,
                       void *workspace_dev, void *stream, void *const *events) {
  if (!plan || !x_dev || !U_dev || !y_dev || !workspace_dev) return RNSWINO_E_INVALID;
  if (plan->device < 0) return RNSWINO_E_NO_DEVICE;
  const Dims &d = plan->dims;
  const KParams P = make_params(plan);
  hipStream_t st = (hipStream_t)stream;
  char *Vp = (char *)workspace_dev;
  char *Op = Vp + align256(v_bytes(d));
  auto mark = [&](int e) {
    if (events && events[e]) (void)hipEventRecord((hipEvent_t)events[e], st);
  };

  const long long t1 = (long long)d.n * d.T * d.Cp * d.t;
  const long long t3 = (long long)d.K * d.T * d.m;
  mark(0);
  if (d.wide) {
    hipLaunchKernelGGL(k1_input_transform_plain<int16_t>, dim3(blocks_for(t1, 256)), dim3(256), 0, st, P, x_dev, (int16_t *)Vp);
    mark(1);
    const long long t2 = (long long)d.n * d.P2 * d.K * d.T;
    hipLaunchKernelGGL(k2_gemm_plain<int16_t>, dim3(blocks_for(t2, 256)), dim3(256), 0, st, P, (const int16_t *)U_dev,
                       (const int16_t *)Vp, (int16_t *)Op);
    mark(2);
    hipLaunchKernelGGL(k3_inverse_mrc_plain<int16_t>, dim3(blocks_for(t3, 256)), dim3(256), 0, st, P, (const int16_t *)Op, y_dev);
  } else {
    {
      const dim3 g1((unsigned)(d.T * (d.Cp / 64)), (unsigned)d.n);
      switch (d.KS1) {
        case 1: hipLaunchKernelGGL(k1_input_transform_i8<1>, g1, dim3(256), 0, st, P, x_dev, (int8_t *)Vp); break;
        case 2: hipLaunchKernelGGL(k1_input_transform_i8<2>, g1, dim3(256), 0, st, P, x_dev, (int8_t *)Vp); break;
        case 3: hipLaunchKernelGGL(k1_input_transform_i8<3>, g1, dim3(256), 0, st, P, x_dev, (int8_t *)Vp); break;
        default: hipLaunchKernelGGL(k1_input_transform_i8<4>, g1, dim3(256), 0, st, P, x_dev, (int8_t *)Vp); break;
      }
    }
    mark(1);
    const dim3 grid((unsigned)(d.n * d.Q), (unsigned)((d.Kp + 31) / 32), (unsigned)((d.Tp + 63) / 64));
    const int ncb = d.Cp / 64;
    if (ncb % 4 == 0)
      hipLaunchKernelGGL(k2_gemm_i8<4>, grid, dim3(256), 0, st, P, (const int8_t *)U_dev, (const int8_t *)Vp, (uint32_t *)Op);
    else if (ncb % 2 == 0)
      hipLaunchKernelGGL(k2_gemm_i8<2>, grid, dim3(256), 0, st, P, (const int8_t *)U_dev, (const int8_t *)Vp, (uint32_t *)Op);
    else
      hipLaunchKernelGGL(k2_gemm_i8<1>, grid, dim3(256), 0, st, P, (const int8_t *)U_dev, (const int8_t *)Vp, (uint32_t *)Op);
    mark(2);
    launch_k3_i8(d, P, (const uint32_t *)Op, y_dev, st);
  }
  mark(3);
  return launch_status();
}

int rnswino_conv2d(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int32_t *y_dev,
                   void *workspace_dev, void *stream) {
  return conv2d_impl(plan, x_dev, U_dev, y_dev, workspace_dev, stream, nullptr);
}

int rnswino_conv2d_events(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int32_t *y_dev,
                          void *workspace_dev, void *stream, void *const events[4]) {
  if (!events) return RNSWINO_E_INVALID;
  return conv2d_impl(plan, x_dev, U_dev, y_dev, workspace_dev, stream, events);
}

int rnswino_requant_pool(const int32_t *y_dev, int8_t *a_dev, int64_t planes, int32_t H, int32_t W, int32_t shift,
                         int32_t pool, void *stream) {
  if (!y_dev || !a_dev || planes <= 0 || H <= 0 || W <= 0 || shift < 0 || shift > 31) return RNSWINO_E_INVALID;
  if (pool && ((H | W) & 1)) return RNSWINO_E_INVALID;
  const long long total = (long long)planes * (pool ? H / 2 : H) * (pool ? W / 2 : W);
  unsigned blocks = blocks_for(total, 256);
  if (blocks > 65536u * 4u) blocks = 65536u * 4u;
  hipLaunchKernelGGL(k_requant_pool, dim3(blocks), dim3(256), 0, (hipStream_t)stream, y_dev, a_dev, (long long)planes, H, W,
                     shift, pool);
  return launch_status();
}

int rnswino_plan_get_matrix(const rnswino_plan_t *plan, int which, int modulus_idx, int32_t *host_out) {
  if (!plan || !host_out || modulus_idx < 0 || modulus_idx >= plan->dims.n) return RNSWINO_E_INVALID;
  const Transforms &tf = plan->tf[modulus_idx];
  const std::vector<int32_t> *src = which == RNSWINO_MATRIX_AT ? &tf.AT : which == RNSWINO_MATRIX_G ? &tf.G
                                    : which == RNSWINO_MATRIX_BT ? &tf.BT : nullptr;
  if (!src) return RNSWINO_E_INVALID;
  std::memcpy(host_out, src->data(), src->size() * sizeof(int32_t));
  return RNSWINO_OK;
}

int rnswino_plan_get_mrc_inverse(const rnswino_plan_t *plan, int l, int j, uint32_t *host_out) {
  if (!plan || !host_out || l < 0 || j <= l || j >= plan->dims.n) return RNSWINO_E_INVALID;
  *host_out = plan->mrc_inv[l][j];
  return RNSWINO_OK;
}

int64_t rnswino_plan_dynamic_range(const rnswino_plan_t *plan) { return plan ? plan->dyn_range : 0; }

int rnswino_debug_stage(const rnswino_plan_t *plan, int stage, const void *src_dev, int32_t *host_out) {
  if (!plan || !src_dev || !host_out) return RNSWINO_E_INVALID;
  if (plan->device < 0) return RNSWINO_E_NO_DEVICE;
  const Dims &d = plan->dims;
  const size_t es = elem_bytes(d);
  size_t bytes, skip = 0;
  if (stage == RNSWINO_STAGE_U) bytes = u_bytes(d);
  else if (stage == RNSWINO_STAGE_V) bytes = v_bytes(d);
  else if (stage == RNSWINO_STAGE_O) { bytes = o_bytes(d); skip = align256(v_bytes(d)); }
  else return RNSWINO_E_INVALID;
  std::vector<char> raw(bytes);
  if (hipDeviceSynchronize() != hipSuccess ||
      hipMemcpy(raw.data(), (const char *)src_dev + skip, bytes, hipMemcpyDeviceToHost) != hipSuccess) {
    (void)hipGetLastError();
    return RNSWINO_E_HIP;
  }
  auto fetch = [&](size_t off) -> int64_t {
    return es == 1 ? (int64_t)((const int8_t *)raw.data())[off] : (int64_t)((const int16_t *)raw.data())[off];
  };
  for (int i = 0; i < d.n; ++i) {
    const int64_t p = plan->desc.moduli[i];
    for (int pt = 0; pt < d.P2; ++pt) {
      const int slab = i * d.P2 + pt;
      if (stage == RNSWINO_STAGE_U) {
        for (int k = 0; k < d.K; ++k)
          for (int c = 0; c < d.C; ++c)
            host_out[((size_t)slab * d.K + k) * d.C + c] = sym_residue(fetch(u_offset(slab, k, c, d.Kp, d.Cp)), p);
      } else if (stage == RNSWINO_STAGE_V) {
        for (int tau = 0; tau < d.T; ++tau)
          for (int c = 0; c < d.C; ++c)
            host_out[((size_t)slab * d.T + tau) * d.C + c] = sym_residue(fetch(v_offset(slab, tau, c, d.Tp, d.Cp)), p);
      } else {
        for (int k = 0; k < d.K; ++k)
          for (int tau = 0; tau < d.T; ++tau)
            host_out[((size_t)slab * d.K + k) * d.T + tau] = sym_residue(fetch(o_offset(i, pt, k, tau, d.Q, d.Kp, d.Tp)), p);
      }
    }
  }
  return RNSWINO_OK;
}

const char *rnswino_strerror(int code) {
  switch (code) {
    case RNSWINO_OK: return "ok";
    case RNSWINO_E_INVALID: return "invalid argument";
    case RNSWINO_E_UNSUPPORTED: return "unsupported configuration";
    case RNSWINO_E_NOT_COPRIME: return "moduli are not pairwise coprime";
    case RNSWINO_E_POINT_NOT_INVERTIBLE: return "a modulus shares a factor with an interpolation-point difference";
    case RNSWINO_E_RANGE: return "dynamic range of the moduli set is below the worst-case output 2^14 r^2 C";
    case RNSWINO_E_HIP: return "HIP runtime error";
    case RNSWINO_E_NO_DEVICE: return "plan is host-only or no GPU is available";
    default: return "unknown error";
  }
}

}  // extern "C"
