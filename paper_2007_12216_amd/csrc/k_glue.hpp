// Layer glue for chained layers: a = clamp(y >> shift, -128, 127), optional 2x2 stride-2 max-pool.
// Not part of the paper's method.
#pragma once
#include "kernels_common.hpp"

namespace rnswino {

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

// A kernel that does nothing: timing it with a stage's grid gives the part of that stage's duration that is dispatch,
// ramp-up and completion rather than work (rnswino_debug_empty_launch).
__global__ __launch_bounds__(256) void k_empty(int unused) { (void)unused; }

}  // namespace rnswino
