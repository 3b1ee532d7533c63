// Internal plan structure of the rnswino library (host side).
#pragma once
#include <cstdint>
#include <vector>
#include "rnswino.h"

namespace rnswino {

// Derived sizes of a layer.  Paper notation: t is N = M + R - 1 of section 4.
struct Dims {
  int N, C, K, H, W, r, m, t, pad;
  int Ho, Wo, th, tw, T;     // output plane, tiles per image, tiles in total
  int n;                     // number of moduli
  int wide;                  // 0: moduli < 256 (residues in 8 bits), 1: 16-bit moduli
  // Layers with at most 32 channels pack TL = 2..16 neighbouring tiles into one 64-channel block instead of padding
  // each tile's few channels with zeros.  Tile tau sits in slot tau / Tg of GEMM column tau % Tg (consecutive columns are
  // consecutive tiles): GEMM channel c' = slot * Cq + c, GEMM row k' = k * TL + slot (the transformed filter is
  // block-diagonal in the slot).  Same products, same sums, 1/TL of the transformed-input bytes.  TL = 1, Cq = 64 otherwise.
  int TL, Cq;                // tiles per 64-channel block, channel slots per tile (TL * Cq = 64 when TL > 1)
  int Kg, Tg;                // GEMM rows K * TL and GEMM columns ceil(T / TL)
  int Cp, Kp, Tp;            // GEMM extents of the tiled tensors: channels padded to 64, Kg and Tg padded to 16
  int P2;                    // t*t transform points
  int Q;                     // ceil(t*t / 4): groups of four transform points in the O tensor
  int CB1, KS1, RP1;         // input transform on MFMA: 16-point column blocks ceil(t*t/16); a tile row takes RP1 = 4 ceil(t/4)
                             // contraction slots (its t pixels, then zeros), the tile t * RP1: KS1 = ceil(t * RP1 / 64) steps
  int RB3, KS3;              // inverse transform on MFMA: 16-output row blocks ceil(m*m/16), contraction steps ceil(t*t/64)
};

// Transform matrices modulo one modulus, entries symmetric in [-(p-1)/2, (p-1)/2].
struct Transforms {
  std::vector<int32_t> AT;   // m x t
  std::vector<int32_t> G;    // t x r
  std::vector<int32_t> BT;   // t x t
};

// Exact modular helpers (plan_math.cpp).
int64_t mod_inverse(int64_t a, int64_t p);              // -1 when gcd(a, p) != 1
int32_t sym_residue(int64_t v, int64_t p);              // representative in [-(p-1)/2, (p-1)/2]
std::vector<int> interpolation_points(int t);           // the t-1 finite points 0, 1, -1, 2, -2, ...
int build_transforms(int m, int r, uint32_t p, Transforms &out);   // RNSWINO_OK or an error code
int validate_desc(const rnswino_desc_t &d, Dims &dims);            // fills dims; all host-side checks

}  // namespace rnswino

struct rnswino_plan_s;
namespace rnswino {
// Fills the CRT constants of the plan and lays out every table the kernels read into one host blob
// (offsets are stored in the plan).  Host only.
void build_tables(rnswino_plan_s &plan, std::vector<char> &blob);
}

struct rnswino_plan_s {
  rnswino_desc_t desc;
  rnswino::Dims dims;
  std::vector<rnswino::Transforms> tf;      // one per modulus
  uint32_t mrc_inv[8][8];                   // mrc_inv[l][j] = moduli[l]^-1 mod moduli[j], l < j
  int64_t dyn_range;                        // (prod - 1)/2, saturated
  uint32_t crt_c[8];                        // prod_{l != i} m_l  mod 2^32
  int crt_c_exact_small[8];                 // 1 when prod_{l != i} m_l itself is below 2^24
  uint32_t crt_inv[8];                      // (prod_{l != i} m_l)^-1 mod m_i
  uint32_t prod_mod32;                      // prod m_i mod 2^32
  int device;                               // HIP device the tables live on, -1 for host-only plans
  int n_cus;                                // compute units of that device (0 if unknown)
  void *d_tables;                           // one device allocation holding every table below
  std::vector<char> h_tables;               // the same bytes on the host (query calls)
  size_t d_tables_bytes;
  // offsets (bytes) into d_tables
  size_t off_G;                             // int32 G matrices [n][t*r] (filter transform)
  size_t off_KB, off_KA;                    // int8 Kronecker tables of the input / inverse transform
  void *kparams;                            // the kernels' parameter block (rnswino::KParams), built once with the plan
};
