// Host generator for the Winograd transform matrices modulo each modulus and the
// checks a plan must pass.  Exact integer arithmetic only.
//
// Construction (paper sections 4 and 5).  With t = m + r - 1 interpolation points
// S_0 .. S_{t-2} finite and S_{t-1} = infinity:
//   A^T = V^T restricted to m rows, G = V restricted to r columns, B^T = V^{-T},
// V the Vandermonde matrix of the points.  Instead of inverting V, the rows of
// V^{-T} are written down directly: row j is the coefficient vector of the
// Lagrange basis polynomial  prod_{l != j}(x - S_l) / prod_{l != j}(S_j - S_l),
// and the row of the infinite point is the coefficient vector of
// prod_l (x - S_l) (it carries the leading coefficient).  The paper moves the
// fractions of B^T into G; here row j of B^T keeps sign(N_j) * prod_{l != j}(x - S_l)
// and row j of G is divided by |N_j|, N_j = prod_{l != j}(S_j - S_l), which is the
// split that reproduces the matrices printed in the paper.  Division by |N_j| is a
// multiplication by its inverse modulo p, which exists iff p is coprime to every
// point difference (section 5, after eq. "inverse_vandermonde").
#include "plan.hpp"

#include <cstdlib>
#include <cstring>
#include <numeric>

namespace rnswino {

int64_t mod_inverse(int64_t a, int64_t p) {
  // extended Euclid; p need not be prime (the paper uses 253 = 11*23 and 247 = 13*19)
  a %= p;
  if (a < 0) a += p;
  int64_t r0 = p, r1 = a, s0 = 0, s1 = 1;
  while (r1 != 0) {
    int64_t q = r0 / r1;
    int64_t r2 = r0 - q * r1; r0 = r1; r1 = r2;
    int64_t s2 = s0 - q * s1; s0 = s1; s1 = s2;
  }
  if (r0 != 1) return -1;
  s0 %= p;
  if (s0 < 0) s0 += p;
  return s0;
}

int32_t sym_residue(int64_t v, int64_t p) {
  int64_t h = (p - 1) / 2;
  int64_t w = (v + h) % p;
  if (w < 0) w += p;
  return (int32_t)(w - h);
}

std::vector<int> interpolation_points(int t) {
  std::vector<int> pts;
  pts.push_back(0);
  for (int a = 1; (int)pts.size() < t - 1; ++a) {
    pts.push_back(a);
    if ((int)pts.size() < t - 1) pts.push_back(-a);
  }
  return pts;
}

static int64_t mulmod(int64_t a, int64_t b, int64_t p) {
  a %= p; b %= p;
  if (a < 0) a += p;
  if (b < 0) b += p;
  return (a * b) % p;   // p < 2^17, so the product is below 2^34
}

int build_transforms(int m, int r, uint32_t pu, Transforms &out) {
  const int t = m + r - 1;
  const int64_t p = pu;
  const std::vector<int> S = interpolation_points(t);       // t-1 finite points
  const int f = t - 1;

  // every difference of two finite points must be a unit modulo p
  for (int j = 0; j < f; ++j)
    for (int l = j + 1; l < f; ++l)
      if (std::gcd((int64_t)std::abs(S[j] - S[l]), p) != 1) return RNSWINO_E_POINT_NOT_INVERTIBLE;

  out.AT.assign((size_t)m * t, 0);
  out.G.assign((size_t)t * r, 0);
  out.BT.assign((size_t)t * t, 0);

  // A^T[i][j] = S_j^i ; the infinite point sees the leading coefficient (degree m-1)
  for (int j = 0; j < f; ++j) {
    int64_t pw = 1;
    for (int i = 0; i < m; ++i) {
      out.AT[(size_t)i * t + j] = sym_residue(pw, p);
      pw = mulmod(pw, S[j], p);
    }
  }
  out.AT[(size_t)(m - 1) * t + (t - 1)] = 1;

  // coefficients (ascending) of prod over a subset of the finite points of (x - S_l), modulo p
  auto poly_without = [&](int skip) {
    std::vector<int64_t> c(1, 1);
    for (int l = 0; l < f; ++l) {
      if (l == skip) continue;
      std::vector<int64_t> nx(c.size() + 1, 0);
      for (size_t e = 0; e < c.size(); ++e) {
        nx[e + 1] = (nx[e + 1] + c[e]) % p;                               // * x
        nx[e] = ((nx[e] - mulmod(c[e], S[l], p)) % p + p) % p;            // * (-S_l)
      }
      c.swap(nx);
    }
    return c;
  };

  for (int j = 0; j < f; ++j) {
    // N_j = prod_{l != j}(S_j - S_l): sign exactly, magnitude modulo p
    int sign = 1;
    int64_t mag = 1;
    for (int l = 0; l < f; ++l) {
      if (l == j) continue;
      int dlt = S[j] - S[l];
      if (dlt < 0) { sign = -sign; dlt = -dlt; }
      mag = mulmod(mag, dlt, p);
    }
    const int64_t inv = mod_inverse(mag, p);
    if (inv < 0) return RNSWINO_E_POINT_NOT_INVERTIBLE;
    // G[j][k] = S_j^k / |N_j|
    int64_t pw = 1;
    for (int k = 0; k < r; ++k) {
      out.G[(size_t)j * r + k] = sym_residue(mulmod(pw, inv, p), p);
      pw = mulmod(pw, S[j], p);
    }
    // B^T[j][.] = sign(N_j) * coefficients of prod_{l != j}(x - S_l)   (degree t-2; last column 0)
    std::vector<int64_t> c = poly_without(j);
    for (int e = 0; e < (int)c.size(); ++e)
      out.BT[(size_t)j * t + e] = sym_residue(sign * c[e], p);
  }
  out.G[(size_t)(t - 1) * r + (r - 1)] = 1;                  // infinite point: leading coefficient of g
  std::vector<int64_t> full = poly_without(-1);             // prod over all finite points, degree t-1
  for (int e = 0; e < t; ++e) out.BT[(size_t)(t - 1) * t + e] = sym_residue(full[e], p);
  return RNSWINO_OK;
}

int validate_desc(const rnswino_desc_t &d, Dims &o) {
  if (d.N <= 0 || d.C <= 0 || d.K <= 0 || d.H <= 0 || d.W <= 0 || d.r <= 0 || d.m <= 0 || d.pad < 0)
    return RNSWINO_E_INVALID;
  if (d.n_moduli < 1 || d.n_moduli > 8) return RNSWINO_E_INVALID;
  const int t = d.m + d.r - 1;
  if (t < 2 || t > 16) return RNSWINO_E_INVALID;
  if (d.r > 7) return RNSWINO_E_UNSUPPORTED;   // the filter-transform kernel keeps an r x r filter in registers
  if (d.stride != 0 && d.stride != 1) return RNSWINO_E_UNSUPPORTED;
  const long Ho = (long)d.H + 2L * d.pad - d.r + 1, Wo = (long)d.W + 2L * d.pad - d.r + 1;
  if (Ho <= 0 || Wo <= 0) return RNSWINO_E_INVALID;
  if ((long long)d.H * d.W > (1LL << 24)) return RNSWINO_E_UNSUPPORTED;   // kernels offset 64 image planes in 32 bits
  int n8 = 0, n16 = 0;
  for (int i = 0; i < d.n_moduli; ++i) {
    const uint32_t p = d.moduli[i];
    if (p < 3 || p > 65521 || (p & 1u) == 0) return RNSWINO_E_UNSUPPORTED;
    if (p > 253 && p < 257) return RNSWINO_E_UNSUPPORTED;   // 8-bit class ends at 253 (residue slack must fit int8)
    if (p < 256) ++n8; else ++n16;
  }
  if (n8 && n16) return RNSWINO_E_UNSUPPORTED;
  // 16-bit moduli: the GEMM keeps three unreduced 32-bit byte-plane sums over all channels; the middle one grows by up to
  // 2 * 64 * 2^14 = 2^21 per 64-channel step, so the contraction must have fewer than 1024 steps (only 1 x 1 filters can
  // ask for more within the int32 output bound below)
  if (n16 && ((long long)d.C + 63) / 64 >= 1024) return RNSWINO_E_UNSUPPORTED;
  for (int i = 0; i < d.n_moduli; ++i)
    for (int j = i + 1; j < d.n_moduli; ++j)
      if (std::gcd(d.moduli[i], d.moduli[j]) != 1u) return RNSWINO_E_NOT_COPRIME;
  // int32 output must hold the worst case regardless of the RNS
  const unsigned __int128 worst = (unsigned __int128)16384u * (unsigned)d.r * (unsigned)d.r * (unsigned)d.C;
  if (worst > 2147483647u) return RNSWINO_E_UNSUPPORTED;

  o.N = d.N; o.C = d.C; o.K = d.K; o.H = d.H; o.W = d.W; o.r = d.r; o.m = d.m; o.t = t; o.pad = d.pad;
  o.Ho = (int)Ho; o.Wo = (int)Wo;
  o.th = (o.Ho + d.m - 1) / d.m; o.tw = (o.Wo + d.m - 1) / d.m;
  const long long T = (long long)d.N * o.th * o.tw;
  if (T > (1LL << 24)) return RNSWINO_E_UNSUPPORTED;
  o.T = (int)T;
  o.n = d.n_moduli;
  o.wide = n16 ? 1 : 0;
  o.TL = 1;
  o.Cq = 64;
  if (d.C <= 32) {
    int cq = 4;
    while (cq < d.C) cq *= 2;
    int tl = 64 / cq;
    while (tl > 1 && o.T < 16 * tl) tl /= 2;      // not worth it before the packed tiles fill a 16-column block
    o.TL = tl;
    o.Cq = 64 / tl;
  }
  o.Kg = d.K * o.TL;
  o.Tg = (o.T + o.TL - 1) / o.TL;
  o.Cp = (d.C + 63) / 64 * 64;
  o.Kp = (o.Kg + 15) / 16 * 16;
  o.Tp = (o.Tg + 15) / 16 * 16;
  o.P2 = t * t;
  o.Q = (o.P2 + 3) / 4;
  o.CB1 = (o.P2 + 15) / 16;
  o.RP1 = (t + 3) / 4 * 4;
  o.KS1 = (t * o.RP1 + 63) / 64;
  o.RB3 = (d.m * d.m + 15) / 16;
  o.KS3 = (o.P2 + 63) / 64;
  // the kernels address the GEMM output O = [Kp][n][Q][Tp] words (two planes for 16-bit moduli) with 32-bit byte
  // offsets and count (k, tile) pairs in 32 bits
  const unsigned __int128 o_bytes = (unsigned __int128)o.Kp * o.n * o.Q * o.Tp * 4u * (o.wide ? 2u : 1u);
  if (o_bytes >= ((unsigned __int128)1 << 32) || (long long)o.Kp * o.Tp >= (1LL << 31)) return RNSWINO_E_UNSUPPORTED;
  return RNSWINO_OK;
}


// ---------------------------------------------------------------------------------------------------
// Tables read by the kernels.
//
// The 2-D transforms are applied as Kronecker products on the matrix cores:
//   vec(B^T d B) = (B^T kron B^T) vec(d),      vec(A^T O A) = (A^T kron A^T) vec(O),
// so each residue needs a (t*t) x (t*t) and an (m*m) x (t*t) matrix modulo p.  They are stored in the operand
// fragment order of v_mfma_i32_16x16x64_i8: a fragment is 16 rows (or columns) x 64 contraction elements,
// lane l holds row l%16 and the 16 contraction elements of slice g = l/16.
//   KB (input transform, B operand): fragment (cbk, s): column = transform point 16*cbk + l%16,
//       contraction element (g, b) = slot f = 64s + 16g + b = pixel (row f / RP1, column f % RP1) of the tile, where a
//       tile row takes RP1 = 4 ceil(t/4) slots; zero for column >= t or row >= t.
//   KA (inverse transform, A operand): fragment (rb, s): row = output u*m+v = 16*rb + l%16,
//       contraction element (g, b) = transform point 64s + 16g + b.  Each entry is multiplied by
//       (P/p_i)^-1 mod p_i so that the kernel's accumulator is directly the CRT coefficient of the residue.
// 8-bit moduli: one signed byte per entry (symmetric residue).  16-bit moduli: two byte planes h, l with
// entry = 256 h + l, the representative chosen in [-32896, 32639].
// ---------------------------------------------------------------------------------------------------
static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

static void put_entry(int8_t *frag, int planes, int lane, int b, int32_t sym, int64_t p) {
  if (planes == 1) {
    frag[lane * 16 + b] = (int8_t)sym;
  } else {
    int32_t v = sym > 32639 ? sym - (int32_t)p : sym;
    const int32_t lo = (int32_t)(int8_t)(v & 0xFF), hi = (v - lo) >> 8;
    frag[lane * 16 + b] = (int8_t)hi;
    frag[1024 + lane * 16 + b] = (int8_t)lo;
  }
}

void build_tables(rnswino_plan_s &pl, std::vector<char> &blob) {
  const Dims &d = pl.dims;
  const rnswino_desc_t &desc = pl.desc;
  // CRT constants: c_i = prod_{l != i} p_l (mod 2^32), its inverse modulo p_i, and P mod 2^32
  pl.prod_mod32 = 1;
  for (int i = 0; i < d.n; ++i) {
    uint32_t c32 = 1;
    int64_t cmod = 1;
    unsigned __int128 full = 1;
    for (int l = 0; l < d.n; ++l)
      if (l != i) {
        c32 *= desc.moduli[l];
        cmod = (cmod * (int64_t)desc.moduli[l]) % (int64_t)desc.moduli[i];
        full *= desc.moduli[l];
        if (full > ((unsigned __int128)1 << 40)) full = (unsigned __int128)1 << 40;
      }
    pl.crt_c[i] = c32;
    pl.crt_c_exact_small[i] = full < ((unsigned __int128)1 << 24) ? 1 : 0;
    pl.crt_inv[i] = (uint32_t)mod_inverse(cmod, desc.moduli[i]);
    pl.prod_mod32 *= desc.moduli[i];
  }

  const int planes = d.wide ? 2 : 1;
  const size_t szG = (size_t)d.n * d.t * d.r * 4;
  const size_t szKB = (size_t)d.n * d.CB1 * d.KS1 * planes * 1024;
  const size_t szKA = (size_t)d.n * d.RB3 * d.KS3 * planes * 1024;
  pl.off_G = 0;
  pl.off_KB = align256(pl.off_G + szG);
  pl.off_KA = align256(pl.off_KB + szKB);
  pl.d_tables_bytes = align256(pl.off_KA + szKA);
  blob.assign(pl.d_tables_bytes, 0);

  for (int i = 0; i < d.n; ++i) {
    const int64_t p = desc.moduli[i];
    const std::vector<int32_t> &BT = pl.tf[i].BT, &AT = pl.tf[i].AT;
    std::memcpy(blob.data() + pl.off_G + (size_t)i * d.t * d.r * 4, pl.tf[i].G.data(), (size_t)d.t * d.r * 4);
    int8_t *kb = (int8_t *)blob.data() + pl.off_KB + (size_t)i * d.CB1 * d.KS1 * planes * 1024;
    for (int cbk = 0; cbk < d.CB1; ++cbk)
      for (int s = 0; s < d.KS1; ++s)
        for (int lane = 0; lane < 64; ++lane)
          for (int b = 0; b < 16; ++b) {
            const int pt = 16 * cbk + (lane & 15), slot = 64 * s + 16 * (lane >> 4) + b;
            const int a = slot / d.RP1, col = slot % d.RP1;
            int32_t v = 0;
            if (pt < d.P2 && a < d.t && col < d.t)
              v = sym_residue((int64_t)BT[(size_t)(pt / d.t) * d.t + a] * BT[(size_t)(pt % d.t) * d.t + col], p);
            put_entry(kb + (size_t)(cbk * d.KS1 + s) * planes * 1024, planes, lane, b, v, p);
          }
    int8_t *ka = (int8_t *)blob.data() + pl.off_KA + (size_t)i * d.RB3 * d.KS3 * planes * 1024;
    for (int rb = 0; rb < d.RB3; ++rb)
      for (int s = 0; s < d.KS3; ++s)
        for (int lane = 0; lane < 64; ++lane)
          for (int b = 0; b < 16; ++b) {
            const int o = 16 * rb + (lane & 15), pt = 64 * s + 16 * (lane >> 4) + b;
            int32_t v = 0;
            if (o < d.m * d.m && pt < d.P2) {
              const int64_t aa = (int64_t)AT[(size_t)(o / d.m) * d.t + pt / d.t] * AT[(size_t)(o % d.m) * d.t + pt % d.t];
              v = sym_residue(sym_residue(aa, p) * (int64_t)pl.crt_inv[i], p);
            }
            put_entry(ka + (size_t)(rb * d.KS3 + s) * planes * 1024, planes, lane, b, v, p);
          }
  }
}

}  // namespace rnswino
