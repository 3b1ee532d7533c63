// Host-side driver for the sanitizer test: runs the plan generator (descriptor checks, transform matrices modulo every
// modulus, Kronecker tables in operand-fragment order) over every accepted (r, m) with 8-bit and 16-bit moduli sets.
// Built by tests/test_host_sanitizers.py with -fsanitize=address,undefined; touches no GPU.
#include <cstdio>
#include <cstring>

#include "plan.hpp"

using namespace rnswino;

int main() {
  int bad = 0, plans = 0;
  const uint32_t n8[8] = {251, 241, 239, 233, 229, 227, 223, 211}, n16[3] = {65521, 65519, 65497};
  for (int r = 1; r <= 7; ++r)
    for (int m = 1; m + r - 1 <= 16; ++m) {
      if (m + r - 1 < 2) continue;
      for (int wide = 0; wide < 2; ++wide)
        for (int C : {3, 70}) {
          rnswino_plan_s pl;
          std::memset(&pl.desc, 0, sizeof(pl.desc));
          rnswino_desc_t &d = pl.desc;
          d.N = 2; d.C = C; d.K = 33; d.H = 19; d.W = 23; d.r = r; d.m = m; d.pad = r / 2; d.stride = 1;
          d.n_moduli = wide ? 3 : 8;
          for (int i = 0; i < d.n_moduli; ++i) d.moduli[i] = wide ? n16[i] : n8[i];
          d.flags = RNSWINO_FLAG_ALLOW_UNCHECKED_RANGE;
          int rc = validate_desc(d, pl.dims);
          if (rc) { std::printf("validate_desc rc=%d r=%d m=%d\n", rc, r, m); ++bad; continue; }
          pl.tf.resize(pl.dims.n);
          for (int i = 0; i < pl.dims.n; ++i) {
            rc = build_transforms(m, r, d.moduli[i], pl.tf[i]);
            if (rc) { std::printf("build_transforms rc=%d r=%d m=%d p=%u\n", rc, r, m, d.moduli[i]); ++bad; break; }
          }
          if (rc) continue;
          std::vector<char> blob;
          build_tables(pl, blob);
          if (blob.empty() || blob.size() != pl.d_tables_bytes) { std::printf("tables r=%d m=%d\n", r, m); ++bad; }
          ++plans;
        }
    }
  std::printf("plans=%d bad=%d\n", plans, bad);
  return bad ? 1 : 0;
}
