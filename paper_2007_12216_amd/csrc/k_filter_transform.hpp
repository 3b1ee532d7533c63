// K0: offline filter transform  U[i][xi,nu][k][c] = (G_p g G_p^T)[xi,nu] mod p_i   (paper section 6: the
// filter transform depends on the weights only and is computed ahead of time).  One thread per (residue, row, channel) of the padded GEMM grid;
// padding rows and channels are written as zeros, which is what lets the GEMM ignore them.
#pragma once
#include "kernels_common.hpp"

namespace rnswino {

template <bool WIDE>
__global__ void k0_filter_transform(KParams P, const int8_t *__restrict__ w, int8_t *__restrict__ U) {
  const long long total = (long long)P.n * P.Kp * P.Cp;
  long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  // GEMM row kg and channel cg; for packed layers (TL > 1) kg = k * TL + tl and cg = tl' * Cq + c, and the entry is
  // the filter's where the tile slots agree (tl = tl') and zero elsewhere
  const int cg = (int)(idx % P.Cp); idx /= P.Cp;
  const int kg = (int)(idx % P.Kp);
  const int i = (int)(idx / P.Kp);
  const int k = kg / P.TL, c = P.TL > 1 ? cg % P.Cq : cg;
  const bool diagonal = P.TL == 1 || (kg % P.TL) == (cg / P.Cq);
  const int p = P.p[i], t = P.t, r = P.r;
  const int32_t *G = P.G + (size_t)i * t * r;
  int g[49];                       // r <= 7 (checked by the plan)
  const bool live = (k < P.K) && (c < P.C) && diagonal;
  for (int e = 0; e < r * r; ++e) g[e] = live ? (int)w[((size_t)k * P.C + c) * r * r + e] : 0;
  for (int xi = 0; xi < t; ++xi) {
    long long row[7];
    for (int b = 0; b < r; ++b) {
      long long s = 0;
      for (int a = 0; a < r; ++a) s += (long long)G[xi * r + a] * g[a * r + b];
      row[b] = s;
    }
    for (int nu = 0; nu < t; ++nu) {
      long long s = 0;
      for (int b = 0; b < r; ++b) s += row[b] * G[nu * r + b];
      const int res = sym_mod64(s, p);
      const int slab = i * P.P2 + xi * t + nu;
      if (WIDE) {
        const int v = storable16(res, p);
        const int lo = (int)(int8_t)(v & 0xFF), hi = (v - lo) >> 8;
        U[u_offset_wide(slab, kg, cg, P.Kp, P.Cp, 0)] = (int8_t)hi;
        U[u_offset_wide(slab, kg, cg, P.Kp, P.Cp, 1)] = (int8_t)lo;
      } else {
        U[u_offset(slab, kg, cg, P.Kp, P.Cp)] = (int8_t)res;
      }
    }
  }
}

}  // namespace rnswino
