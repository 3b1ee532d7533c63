// Direct int8 convolution as an implicit GEMM on the matrix cores: the baseline the paper measures its method against
// (section 8, Tables 4 and 5: Im2col + INT8 GEMM), written for the same chip so that the two can be timed side by side.
//
//   y[n][k][oy][ox] = sum_{c,i,j} xpad[n][c][oy+i-pad][ox+j-pad] w[k][c][i][j]            (int32, stride 1)
// is a GEMM with rows k, columns = output pixels and contraction index (i, j, c).  No im2col matrix is ever
// written: a column block's operand fragment for filter tap (i, j) and 64 channels is gathered straight from the
// activations, 16 bytes (16 channels of one pixel) per lane.  For that the activations are first copied once into a
// channel-innermost, zero-bordered layout (one pass over x; part of the timed call):
//   xt [N][H + 2 pad][W + 2 pad][Cp]      Cp = C rounded up to 64, padding channels and the border are zero
// and the weights are packed ahead of time into matrix-core fragments (they are constants of the layer):
//   wt [r*r taps][Kp/16][Cp/64][lane = k%16 + 16 g][16 B]     byte b of slice g = channel 64 cb + 16 g + b.
// The GEMM kernel has the structure of the LDS-tiled residue GEMM (k_residue_gemm_lds.hpp): WM x WN waves of
// RM x NT fragments each, operand fragments loaded from global memory straight into LDS S steps deep and shared by
// the waves; a step is one (tap, 64-channel block).  The int32 sums are stored as they are (no modulus anywhere).
#pragma once
#include "k_residue_gemm_lds.hpp"

namespace rnswino {

struct DirectParams {
  int N, C, K, H, W, r, pad;
  int Ho, Wo, Hp, Wp, Cp, Kp;
  int npix;                     // N * Ho * Wo
};

// x [N][C][H][W] -> xt [N][Hp][Wp][Cp], zero border and zero padding channels.  One thread writes 16 channels of one
// padded pixel; a block of 256 threads covers 64 consecutive padded pixels of one row and 64 channels, staged through
// LDS so that both the reads (along W) and the writes (along C) are contiguous.
__global__ __launch_bounds__(256) void k_direct_to_nhwc(DirectParams P, const int8_t *__restrict__ x, int8_t *__restrict__ xt) {
  __shared__ uint8_t tile[64][64 + 4];                 // [channel][pixel], rows padded against bank conflicts
  const int xblocks = (P.Wp + 63) / 64;
  int b = blockIdx.x;
  const int xb = b % xblocks; b /= xblocks;
  const int cb = b % (P.Cp / 64); b /= (P.Cp / 64);
  const int yp = b % P.Hp, n = b / P.Hp;
  const int iy = yp - P.pad;
  {
    // read: thread (c = tid / 4, quarter q = tid % 4) takes 16 pixels of channel c
    const int c = threadIdx.x >> 2, q = threadIdx.x & 3;
    const int ch = cb * 64 + c;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int xp = xb * 64 + q * 16 + e, ix = xp - P.pad;
      uint8_t v = 0;
      if (ch < P.C && iy >= 0 && iy < P.H && ix >= 0 && ix < P.W) v = (uint8_t)x[(((size_t)n * P.C + ch) * P.H + iy) * P.W + ix];
      tile[c][q * 16 + e] = v;
    }
  }
  __syncthreads();
  {
    // write: thread (pixel = tid / 4, slice g = tid % 4) stores channels 16 g .. 16 g + 15 of that pixel
    const int px = threadIdx.x >> 2, g = threadIdx.x & 3;
    const int xp = xb * 64 + px;
    if (xp < P.Wp) {
      uint32_t wv[4] = {0, 0, 0, 0};
#pragma unroll
      for (int e = 0; e < 16; ++e) wv[e >> 2] |= (uint32_t)tile[16 * g + e][px] << (8 * (e & 3));
      *(v4i *)(xt + (((size_t)n * P.Hp + yp) * P.Wp + xp) * P.Cp + cb * 64 + 16 * g) = (v4i){(int)wv[0], (int)wv[1], (int)wv[2], (int)wv[3]};
    }
  }
}

// w [K][C][r][r] -> wt fragments (offline).  One thread per (tap, k, 16-channel slice).
__global__ __launch_bounds__(256) void k_direct_pack_filter(DirectParams P, const int8_t *__restrict__ w, int8_t *__restrict__ wt) {
  const long long total = (long long)P.r * P.r * P.Kp * (P.Cp / 16);
  const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
  if (id >= total) return;
  const int sl = (int)(id % (P.Cp / 16));               // 16-channel slice
  long long rest = id / (P.Cp / 16);
  const int k = (int)(rest % P.Kp);
  const int tap = (int)(rest / P.Kp);
  const int cb = sl >> 2, g = sl & 3;
  uint32_t wv[4] = {0, 0, 0, 0};
  for (int e = 0; e < 16; ++e) {
    const int c = sl * 16 + e;
    if (k < P.K && c < P.C) wv[e >> 2] |= (uint32_t)(uint8_t)w[((size_t)k * P.C + c) * P.r * P.r + tap] << (8 * (e & 3));
  }
  const size_t frag = ((size_t)tap * (P.Kp / 16) + (k >> 4)) * (P.Cp / 64) + cb;
  *(v4i *)(wt + frag * 1024 + ((k & 15) + 16 * g) * 16) = (v4i){(int)wv[0], (int)wv[1], (int)wv[2], (int)wv[3]};
}

// Grid: one-dimensional, 8 * ceil(pixel blocks / 8) * row blocks.  Workgroups go to the 8 XCDs round-robin by id: pixel
// block = 8 * (id / 8 / row blocks) + id % 8, row block = (id / 8) % row blocks, so the workgroups that share a pixel
// block's activations follow each other on one XCD (one L2).  256 threads.
template <int WM, int WN, int RM, int NT, int S>
__global__ __launch_bounds__(256) void k_direct_conv(DirectParams P, const int8_t *__restrict__ xt, const int8_t *__restrict__ wt,
                                                      int32_t *__restrict__ y) {
  static_assert(WM * WN == 4, "four waves per workgroup");
  constexpr int BRF = WM * RM, BTF = WN * NT;
  constexpr int NF = BRF + BTF;
  constexpr int LPW = (NF + 3) / 4;
  constexpr int SLOTS = 4 * LPW;
  __shared__ __attribute__((aligned(16))) uint8_t stage[S * SLOTS * 1024];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int wm = wave / WN, wn = wave % WN;
  const int nkb = P.Kp >> 4, ntb = (P.npix + 15) >> 4, ncb = P.Cp >> 6;
  const int gy = (nkb + BRF - 1) / BRF, gz = (ntb + BTF - 1) / BTF;
  const int pb = ((blockIdx.x >> 3) / gy) * 8 + (blockIdx.x & 7);
  if (pb >= gz) return;                            // block-uniform: the grid is padded to a multiple of 8 pixel blocks
  const int kb0 = ((blockIdx.x >> 3) % gy) * BRF, tb0 = pb * BTF;
  const int taps = P.r * P.r;
  const int total = taps * ncb;

  // where output pixel `pix` (clamped to the last one) starts in xt: the patch origin (oy, ox) of image n
  auto pixel_origin = [&](int pix) -> uint32_t {
    pix = min(pix, P.npix - 1);
    const int n = pix / (P.Ho * P.Wo), rem = pix - n * (P.Ho * P.Wo);
    const int oy = rem / P.Wo, ox = rem - oy * P.Wo;
    return (uint32_t)(((n * P.Hp + oy) * P.Wp + ox) * P.Cp);        // xt is smaller than 4 GiB (checked on the host)
  };
  // this wave's loads of a step: fragment f = wave + 4 j: a weight fragment (contiguous) or a pixel-block fragment
  // (lane = pixel l % 16, channels 16 (l / 16) .. + 15); per step only the wave-uniform part of the address changes
  const int8_t *base[LPW];
  uint32_t lane_off[LPW], tap_stride[LPW];
  bool is_w[LPW];
#pragma unroll
  for (int j = 0; j < LPW; ++j) {
    const int f = min(wave + 4 * j, NF - 1);
    is_w[j] = f < BRF;
    if (is_w[j]) {
      base[j] = wt + (size_t)min(kb0 + f, nkb - 1) * ncb * 1024;
      lane_off[j] = (uint32_t)lane * 16u;
      tap_stride[j] = (uint32_t)(nkb * ncb) * 1024u;
    } else {
      base[j] = xt;
      lane_off[j] = pixel_origin((min(tb0 + f - BRF, ntb - 1)) * 16 + (lane & 15)) + (uint32_t)(lane >> 4) * 16u;
      tap_stride[j] = 0;
    }
  }
  const uint32_t stage_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t *)stage;
  auto issue = [&](int tap, int cb, int slot) {
    const int ti = tap / P.r, tj = tap - ti * P.r;
    const size_t x_off = (size_t)(ti * P.Wp + tj) * P.Cp + (size_t)cb * 64;
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
      const int8_t *src = is_w[j] ? base[j] + (size_t)tap * tap_stride[j] + (size_t)cb * 1024 : base[j] + x_off;
      load_to_lds16(src, lane_off[j], stage_lds + (uint32_t)((slot * SLOTS + wave + 4 * j) * 1024));
    }
  };
  int ptap = 0, pcb = 0;
  auto advance = [&]() {
    if (++pcb == ncb) { pcb = 0; ++ptap; }
  };
#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (ptap < taps) { issue(ptap, pcb, s); advance(); }

  v4i acc[RM][NT];
#pragma unroll
  for (int rm = 0; rm < RM; ++rm)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[rm][nt] = (v4i){0, 0, 0, 0};
  const uint8_t *lds_a = stage + (wm * RM) * 1024 + lane * 16;
  const uint8_t *lds_b = stage + (BRF + wn * NT) * 1024 + lane * 16;
  int slot = 0, fill = S - 1;
  for (int it = 0; it < total; ++it) {
    const int rem = total - 1 - it;
    if (rem >= S - 2) wait_vmcnt<LPW * (S - 2)>();
    else if (S >= 4 && rem == 1) wait_vmcnt<LPW>();
    else wait_vmcnt<0>();
    __syncthreads();
    if (ptap < taps) { issue(ptap, pcb, fill); advance(); }
    v4i a[RM];
#pragma unroll
    for (int rm = 0; rm < RM; ++rm) a[rm] = *(const v4i *)(lds_a + (slot * SLOTS + rm) * 1024);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const v4i b = *(const v4i *)(lds_b + (slot * SLOTS + nt) * 1024);
#pragma unroll
      for (int rm = 0; rm < RM; ++rm) acc[rm][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[rm], b, acc[rm][nt], 0, 0, 0);
    }
    if (++slot == S) slot = 0;
    if (++fill == S) fill = 0;
  }

  // a lane holds rows 16 kb + 4 (lane / 16) + j of pixel 16 tb + lane % 16
  const size_t plane = (size_t)P.Ho * P.Wo;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int pix = (tb0 + wn * NT + nt) * 16 + (lane & 15);
    if (pix >= P.npix) continue;
    const int n = pix / (P.Ho * P.Wo), rem = pix - n * (P.Ho * P.Wo);
    int32_t *ypix = y + (size_t)n * P.K * plane + rem;
#pragma unroll
    for (int rm = 0; rm < RM; ++rm)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = (kb0 + wm * RM + rm) * 16 + 4 * (lane >> 4) + j;
        if (k < P.K) ypix[(size_t)k * plane] = acc[rm][nt][j];
      }
  }
}

}  // namespace rnswino
