// rnswino: C ABI entry points (host side) and kernel dispatch for gfx950.
//
// Pipeline of one layer (paper section 6):
//   K0  filter transform   U = G g G^T mod p                 (offline, once per weight set)   k_filter_transform.hpp
//   K1  input transform    V = B^T d B mod p                 (int8 MFMA, Kronecker form)      k_input_transform.hpp
//   K2  residue GEMM       O = sum_c U V mod p               (int8 MFMA)                      k_residue_gemm.hpp
//   K3  inverse transform  Y = A^T O A mod p, then CRT to int32 (int8 MFMA, Kronecker form)   k_inverse_crt.hpp
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "k_direct_conv.hpp"
#include "k_filter_transform.hpp"
#include "k_glue.hpp"
#include "k_input_transform.hpp"
#include "k_inverse_crt.hpp"
#include "k_residue_gemm.hpp"
#include "k_residue_gemm_lds.hpp"
#include "layout.hpp"
#include "plan.hpp"
#include "rnswino.h"

using namespace rnswino;

// Workspace of rnswino_conv2d_static(): device memory that is part of the loaded code object, so the entry point needs
// no allocation.  Every GPU holds its own copy at its own address; in host code the name below is only a handle for
// hipGetSymbolAddress(), never an address to hand to a kernel.
static __device__ __align__(256) unsigned char scratch[RNSWINO_STATIC_WORKSPACE_BYTES];

namespace {

// Address of `scratch` on each device, looked up once per device (with that device current) when the first plan is
// made there; rnswino_conv2d_static() only reads it.
constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void *scratch_ptr[MAX_DEVICES] = {};

int resolve_scratch(int dev) {          // called with device `dev` current
  if (dev < 0 || dev >= MAX_DEVICES) return RNSWINO_E_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (scratch_ptr[dev]) return RNSWINO_OK;
  void *ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return RNSWINO_E_HIP; }
  scratch_ptr[dev] = ptr;
  return RNSWINO_OK;
}

// The largest |y| the plan has to represent: the worst case 2^14 r^2 C of int8 operands (sections 3, 5, 8), or the
// caller's tighter bound for the layer's actual weights (rnswino_desc_t::output_bound), whichever is smaller.
unsigned __int128 output_bound(const rnswino_desc_t &desc, const Dims &d) {
  const unsigned __int128 worst = (unsigned __int128)16384u * (unsigned)d.r * (unsigned)d.r * (unsigned)d.C;
  return desc.output_bound != 0 && (unsigned __int128)desc.output_bound < worst ? (unsigned __int128)desc.output_bound : worst;
}

KParams make_params(const rnswino_plan_t *pl) {
  KParams P;
  std::memset(&P, 0, sizeof(P));
  const Dims &d = pl->dims;
  P.N = d.N; P.C = d.C; P.K = d.K; P.H = d.H; P.W = d.W; P.r = d.r; P.m = d.m; P.t = d.t; P.pad = d.pad;
  P.Ho = d.Ho; P.Wo = d.Wo; P.th = d.th; P.tw = d.tw; P.T = d.T; P.n = d.n;
  P.TL = d.TL; P.Cq = d.Cq; P.Kg = d.Kg; P.Tg = d.Tg;
  P.Cp = d.Cp; P.Kp = d.Kp; P.Tp = d.Tp; P.P2 = d.P2; P.Q = d.Q;
  P.CB1 = d.CB1; P.KS1 = d.KS1; P.RP1 = d.RP1; P.RB3 = d.RB3; P.KS3 = d.KS3;
  P.crt24 = 1;
  for (int i = 0; i < d.n; ++i) {
    P.p[i] = (int)pl->desc.moduli[i];
    P.inv_p[i] = 1.0f / (float)pl->desc.moduli[i];
    P.inv_pd[i] = 1.0 / (double)pl->desc.moduli[i];
    P.crt_c[i] = pl->crt_c[i];
    if (!pl->crt_c_exact_small[i]) P.crt24 = 0;
    P.bias_p[i] = d.wide ? 0 : (int)(pl->desc.moduli[i] * 4194304u + pl->desc.moduli[i]);
  }
  {
    // binary32 is enough for the CRT quotient when 2 * (worst-case |y|) <= 0.9 * prod p_i
    unsigned __int128 prod = 1;
    const unsigned __int128 cap = ((unsigned __int128)1 << 100);
    for (int i = 0; i < d.n; ++i) { prod *= pl->desc.moduli[i]; if (prod > cap) prod = cap; }
    const unsigned __int128 worst = output_bound(pl->desc, d);
    P.quot32 = (worst * 20 <= prod * 9) ? 1 : 0;
    // Fast conversion: the binary32 sum of (a_i + 2^22) / p_i - B, B = 2^22 sum_i 1/p_i, stays within [-B, B]; it
    // takes n + 1 roundings of at most half an ulp of 2B each, and the rounded 1/p_i add at most 2B 2^-23 in all.
    // Enabled when the layer's worst case leaves twice that error below 0.49 - |y|/P.
    if (!d.wide && P.crt24 && prod < cap) {
      long double Bl = 0.0L;             // extended precision: the one rounding to binary64 is counted below
      uint32_t c32 = 0;
      for (int i = 0; i < d.n; ++i) { Bl += 4194304.0L / (long double)pl->desc.moduli[i]; c32 += pl->crt_c[i]; }
      const double B = (double)Bl;
      int e = 0;
      std::frexp(2.0 * B, &e);                                   // 2B = f * 2^e, f in [0.5, 1)
      const double half_ulp = std::ldexp(1.0, e - 24 - 1);      // binary32: ulp = 2^(e - 24)
      const double err = (d.n + 1) * half_ulp + 2.0 * B * std::ldexp(1.0, -23);
      // The same sum in binary64 (ulp = 2^(e64 - 53)) must find the quotient for every |y| <= (P - 1)/2, i.e. stay
      // within 1/(2P) of the true value: twice its error bound has to fit.
      int e64 = 0;
      std::frexp(B, &e64);                                       // every partial sum lies in [-B, B], B < 2^e64
      const double err64 = (d.n + 1) * std::ldexp(1.0, e64 - 53 - 1) + 2.0 * B * std::ldexp(1.0, -52);
      if ((double)worst / (double)prod + 2.0 * err <= 0.49) P.fastcrt = 1;
      else if (2.0 * err64 <= 0.5 / (double)prod) P.fastcrt = 2;
      if (P.fastcrt) {
        P.acc0 = 4194304;
        P.crt_sum0 = 0u - 4194304u * c32;
        P.crt_fs0 = (float)(-B);
        P.crt_fs0d = -B;
      }
    }
  }
  P.prod_mod32 = pl->prod_mod32;
  if (pl->d_tables) {                   // host-only plans are never executed: their table pointers stay null
    const char *base = (const char *)pl->d_tables;
    P.G = (const int32_t *)(base + pl->off_G);
    P.KB = (const int8_t *)(base + pl->off_KB);
    P.KA = (const int8_t *)(base + pl->off_KA);
  }
  return P;
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline size_t elem_bytes(const Dims &d) { return d.wide ? 2 : 1; }
inline size_t v_bytes(const Dims &d) { return (size_t)d.n * d.P2 * d.Tp * d.Cp * elem_bytes(d); }
inline size_t o_bytes(const Dims &d) { return (size_t)d.n * d.Q * d.Kp * d.Tp * 4 * elem_bytes(d); }
inline size_t u_bytes(const Dims &d) { return (size_t)d.n * d.P2 * d.Kp * d.Cp * elem_bytes(d); }

// The plan's tables live on the device that was current when it was made: executing it from another device would hand
// the kernels pointers of the wrong GPU.
inline bool on_plan_device(const rnswino_plan_t *plan) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return false; }
  return dev == plan->device;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? RNSWINO_OK : RNSWINO_E_HIP; }

inline unsigned blocks_for(long long total, int bs) { return (unsigned)((total + bs - 1) / bs); }

// Optional pair of events that receive the kernel's own start and stop timestamps.
struct Timing {
  hipEvent_t start = nullptr, stop = nullptr;
};

template <typename Kern, typename... Args>
inline void launch(Kern kern, dim3 grid, size_t lds, hipStream_t st, Timing tm, Args... args) {
  if (tm.start || tm.stop)
    hipExtLaunchKernelGGL(kern, grid, dim3(256), lds, st, tm.start, tm.stop, 0, args...);
  else
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, args...);
}

// =============================================================================================
// Kernel selection.  Which instantiation of each kernel a layer runs, and its grid, is decided here from the plan's
// sizes alone (no GPU needed), so that rnswino_plan_describe() can report it and the launches below cannot disagree
// with the report.
// =============================================================================================

struct K1Choice { int KS1; bool wide, pack; unsigned gx, gy; };

K1Choice choose_k1(const Dims &d) {
  K1Choice c;
  c.KS1 = d.KS1 < 4 ? d.KS1 : 4;
  c.wide = d.wide != 0;
  c.pack = d.TL > 1;
  const long long units = (long long)d.Tg * (d.Cp / 64);
  // x: multiple of 8 (see xcd_chunked()); y: one block per residue, or one block for all residues when there are
  // enough units to fill the chip (the pixel gather is then done once instead of n times; measured on the VGG16
  // stack, two blocks per CU are already enough for that to win)
  c.gx = (unsigned)((units + 7) / 8 * 8);
  c.gy = (unsigned)(units >= 512 ? 1 : d.n);
  return c;
}

// NTB = 16-tile column blocks per wave (1, 2 or 4, the smallest that covers Tp up to 64); KS = contraction steps
// in flight, limited by the register budget of the variant; RM = 16-row blocks per wave.
// lds: the LDS-tiled kernel (8-bit moduli): WM x WN waves of RM x NTB fragments each, S steps in flight.
struct K2Choice { int KS, NTB, RM; bool wide; int xgroup; unsigned blocks; bool lds; int WM, WN, S; };

// L2-aware grouping of the x index (see the kernels): brf / btf = row / tile fragments per workgroup
void k2_grid(const Dims &d, int brf, int btf, K2Choice &c) {
  const int ntb = d.Tp / 16;
  const long long pl = c.wide ? 2 : 1;
  const long long nxh = (d.n * d.Q + 7) / 8, gy = (d.Kp / 16 + brf - 1) / brf, gz = (ntb + btf - 1) / btf;
  const long long u_x = 4LL * d.Kp * d.Cp * pl, v_slice = 4LL * 16 * btf * d.Cp * pl;
  long long xgroup = gz == 1 ? 1 : (3LL << 20) / (u_x + 2 * v_slice);
  xgroup = xgroup < 1 ? 1 : (xgroup > nxh ? nxh : xgroup);
  if (xgroup > 1 && xgroup < nxh && (xgroup & 1) == 0) --xgroup;
  c.xgroup = (int)xgroup;
  c.blocks = (unsigned)(8 * ((nxh + xgroup - 1) / xgroup * xgroup) * gy * gz);
}

K2Choice choose_k2(const Dims &d, uint32_t flags) {
  K2Choice c;
  c.wide = d.wide != 0;
  c.lds = false; c.WM = c.WN = c.S = 0;
  const int ntb = d.Tp / 16, ncb = d.Cp / 64;
  c.NTB = ntb == 1 ? 1 : ntb == 2 ? 2 : 4;
  if (!c.wide && (flags & RNSWINO_FLAG_GEMM_BLOCK_64X16)) {
    // measurement only: the GEMM on the block a fused GEMM + inverse transform could hold on chip
    c.lds = true; c.KS = 0; c.NTB = 1; c.WM = 4; c.WN = 1; c.RM = 1; c.S = 4;
    k2_grid(d, 4, 1, c);
    return c;
  }
  if (!c.wide && d.Kp >= 128) {
    // LDS-tiled kernel where it measured faster than the register-direct one (VGG16 stack at batch 8, the 256-channel
    // layer at batch 1): 128 x 64 blocks for 33..64 tiles; 128 x 128 blocks for many tiles and a contraction of two or
    // more steps (with a single step the pipeline over the four points never fills), unless the last tile block would be
    // mostly padding (more than a tenth of the tile blocks wasted)
    const int tb128 = (ntb + 7) / 8;
    const bool few = ntb == 3 || ntb == 4;
    const bool many = ntb >= 5 && ncb >= 2 && tb128 * 80 <= ntb * 11;
    if (few || many) {
      c.lds = true; c.KS = 0; c.NTB = 4;
      if (few) { c.WM = 4; c.WN = 1; c.RM = 2; c.S = 4; }
      else { c.WM = 2; c.WN = 2; c.RM = 4; c.S = 3; }
      k2_grid(d, c.WM * c.RM, c.WN * c.NTB, c);
      return c;
    }
  }
  // 64 rows per wave when K is large (V re-reads dominate), the contraction has more than one step and that still
  // leaves >= 4 blocks per CU; measured on the VGG16 stack this wins for K >= 256 and loses for K <= 128 (8-bit
  // moduli, full-width tiles only: the register budget of the other variants is spent on their extra accumulators)
  const long long big_blocks = (long long)((d.n * d.Q + 7) / 8 * 8) * ((d.Kp + 63) / 64) * ((ntb + c.NTB - 1) / c.NTB);
  if (!c.wide && c.NTB == 4 && d.Kp >= 256 && ncb >= 2 && big_blocks >= 1024) {
    c.RM = 4;
    c.KS = ncb % 2 == 0 ? 2 : 1;
  } else {
    const int ksmax = c.wide ? (c.NTB == 1 ? 4 : c.NTB == 2 ? 2 : 1) : 4;
    c.RM = 2;
    c.KS = (ksmax >= 4 && ncb % 4 == 0) ? 4 : (ksmax >= 2 && ncb % 2 == 0) ? 2 : 1;
  }
  // One-dimensional grid: the kernel derives (x, row block, tile block) from the id in an order that suits the L2s.
  // A slice of U is used again after xgroup * gy workgroups of its XCD, which meanwhile touch xgroup * (U of one x +
  // about two tile-block slices of V): xgroup is the largest count for which that stays within 3 of the L2's 4 MiB.
  // With a single tile block nothing of U is used twice: one x at a time, so that the workgroups in flight on an XCD
  // read neighbouring row blocks of one U slab (measured: 3-7 % faster than walking over all x at once).  Even group
  // sizes measured slower (they run into each other in the L2 channels).
  k2_grid(d, c.RM, c.NTB, c);
  return c;
}

// stream: the streaming variant (8-bit moduli, table of all residues at most 64 KiB, n * KS3 <= 8: O operand in
// registers) for layers with 3072 and more units (measured on the VGG16 stack);
// fast: conversion out of the RNS from unreduced accumulators; m8: the 8 x 8 store path of the streaming variant
// (int32 output: only with rows that keep four outputs 16-byte aligned; int8 output: only with an even row length).
struct K3Choice { bool stream, wide, fast, m8; int NRES, KS3; unsigned gx, gy; size_t lds; };

K3Choice choose_k3(const Dims &d, const KParams &P, int n_cus, int epi) {
  K3Choice c;
  c.wide = d.wide != 0;
  c.NRES = d.n;
  c.KS3 = d.KS3 < 4 ? d.KS3 : 4;
  c.fast = !c.wide && P.fastcrt != 0;
  c.stream = !c.wide && d.n * d.KS3 <= 8 && d.n <= 4 && d.KS3 <= 2 && (size_t)d.n * d.RB3 * d.KS3 * 1024 <= 65536 &&
             (long long)d.Kg * (d.Tp / 16) >= 3072;
  c.m8 = false;
  c.lds = 0;
  if (c.stream) {
    const long long blocks = ((long long)d.Kg * (d.Tp / 16) + 3) / 4;
    const long long max_blocks = n_cus > 0 ? 4LL * n_cus : K3_STREAM_BLOCKS;
    c.gx = (unsigned)(blocks < max_blocks ? blocks : max_blocks);
    c.gy = 1;
    c.lds = (size_t)d.n * d.RB3 * d.KS3 * 1024;
    c.m8 = c.fast && d.m == 8 && (epi == 0 ? (d.Wo & 3) == 0 : (d.Wo & 1) == 0);
  } else {
    const long long units = ((long long)d.Kg * d.Tg + 15) / 16;
    c.gx = (unsigned)((units + 7) / 8 * 8);       // x multiple of 8: see xcd_chunked()
    c.gy = (unsigned)((d.RB3 + 3) / 4);
  }
  return c;
}

// The instantiations that exist, as tables: the launches below and rnswino_kernel_variants() both expand them.
// Inverse transform: 16-bit moduli take the general conversion (any moduli count); with 8-bit moduli the conversion from
// unreduced accumulators needs every P/p_i below 2^24, i.e. at most four moduli, and sets of fewer than four moduli
// always qualify for it (their product leaves the binary64 quotient ample room), so the reduced form exists from four
// moduli on (with exactly four, only up to t = 13: a product large enough to rule the unreduced form out needs 253,
// which 14 or more interpolation points exclude).  The streaming kernel's 8 x 8 store path exists for the unreduced
// form only.  A launch function returns false when the choice has no instantiation; rnswino_plan() refuses such a plan.
#define RNSW_K1_TABLE(X) \
  X(1, false, false) X(1, false, true) X(1, true, false) X(1, true, true) X(2, false, false) X(2, false, true) X(2, true, false) X(2, true, true) \
  X(3, false, false) X(3, false, true) X(3, true, false) X(3, true, true) X(4, false, false) X(4, false, true) X(4, true, false) X(4, true, true)
#define RNSW_K2_TABLE(X) \
  X(1, 1, 2, false) X(2, 1, 2, false) X(4, 1, 2, false) X(1, 2, 2, false) X(2, 2, 2, false) X(4, 2, 2, false) \
  X(1, 4, 2, false) X(2, 4, 2, false) X(4, 4, 2, false) X(1, 4, 4, false) X(2, 4, 4, false) \
  X(1, 1, 2, true) X(2, 1, 2, true) X(4, 1, 2, true) X(1, 2, 2, true) X(2, 2, 2, true) X(1, 4, 2, true)
#define RNSW_K2L_TABLE(X) X(2, 2, 4, 4, 3) X(4, 1, 2, 4, 4) X(4, 1, 1, 1, 4)
#define RNSW_K3_NK(X, nres, wd, fs) X(nres, 1, wd, fs) X(nres, 2, wd, fs) X(nres, 3, wd, fs) X(nres, 4, wd, fs)
#define RNSW_K3_TABLE(X) \
  RNSW_K3_NK(X, 1, true, false) RNSW_K3_NK(X, 2, true, false) RNSW_K3_NK(X, 3, true, false) RNSW_K3_NK(X, 4, true, false) \
  RNSW_K3_NK(X, 5, true, false) RNSW_K3_NK(X, 6, true, false) RNSW_K3_NK(X, 7, true, false) RNSW_K3_NK(X, 8, true, false) \
  RNSW_K3_NK(X, 1, false, true) RNSW_K3_NK(X, 2, false, true) RNSW_K3_NK(X, 3, false, true) RNSW_K3_NK(X, 4, false, true) \
  X(4, 1, false, false) X(4, 2, false, false) X(4, 3, false, false) RNSW_K3_NK(X, 5, false, false) RNSW_K3_NK(X, 6, false, false) RNSW_K3_NK(X, 7, false, false) \
  RNSW_K3_NK(X, 8, false, false)
#define RNSW_K3S_M8(X, nres, ks3, fs) X(nres, ks3, fs, true) X(nres, ks3, fs, false)
#define RNSW_K3S_TABLE(X) \
  RNSW_K3S_M8(X, 1, 1, true) RNSW_K3S_M8(X, 1, 2, true) RNSW_K3S_M8(X, 2, 1, true) RNSW_K3S_M8(X, 2, 2, true) \
  RNSW_K3S_M8(X, 3, 1, true) RNSW_K3S_M8(X, 3, 2, true) RNSW_K3S_M8(X, 4, 1, true) RNSW_K3S_M8(X, 4, 2, true) \
  X(4, 1, false, false) X(4, 2, false, false)

// ---- K1 ----  (dry: only report whether the instantiation exists)
bool launch_k1(const Dims &d, const KParams &P, const int8_t *x, int8_t *V, hipStream_t st, Timing tm, bool dry = false) {
  const K1Choice c = choose_k1(d);
  const dim3 grid(c.gx, c.gy);
#define RNSW_X(ks, wd, pk) \
  if (c.KS1 == ks && c.wide == wd && c.pack == pk) { if (!dry) launch(k1_input_transform<ks, wd, pk>, grid, 0, st, tm, P, x, V); return true; }
  RNSW_K1_TABLE(RNSW_X)
#undef RNSW_X
  return false;
}

// ---- K2 ----
bool launch_k2(const Dims &d, uint32_t flags, const KParams &P, const int8_t *U, const int8_t *V, uint32_t *O, hipStream_t st, Timing tm, bool dry = false) {
  const K2Choice c = choose_k2(d, flags);
  const dim3 grid(c.blocks);
  if (c.lds) {
#define RNSW_X(wm_, wn_, rm, ntb, s_) \
    if (c.WM == wm_ && c.WN == wn_ && c.RM == rm && c.NTB == ntb && c.S == s_) { \
      if (!dry) launch(k2_residue_gemm_lds<wm_, wn_, rm, ntb, s_>, grid, 0, st, tm, P, U, V, O, c.xgroup); return true; }
    RNSW_K2L_TABLE(RNSW_X)
#undef RNSW_X
    return false;
  }
#define RNSW_X(ks, ntb, rm, wd) \
  if (c.KS == ks && c.NTB == ntb && c.RM == rm && c.wide == wd) { if (!dry) launch(k2_residue_gemm<ks, ntb, rm, wd>, grid, 0, st, tm, P, U, V, O, c.xgroup); return true; }
  RNSW_K2_TABLE(RNSW_X)
#undef RNSW_X
  return false;
}

// ---- K3 ----
bool launch_k3(const Dims &d, const KParams &P, int n_cus, const uint32_t *O, int32_t *y, hipStream_t st, Timing tm, bool dry = false) {
  const K3Choice c = choose_k3(d, P, n_cus, P.epi);
  const dim3 grid(c.gx, c.gy);
  if (c.stream) {
#define RNSW_X(nres, ks3, fs, e8) \
    if (c.NRES == nres && c.KS3 == ks3 && c.fast == fs && c.m8 == e8) { \
      if (!dry) launch(k3_inverse_crt_stream<nres, ks3, fs, e8>, grid, c.lds, st, tm, P, O, y); return true; }
    RNSW_K3S_TABLE(RNSW_X)
#undef RNSW_X
    return false;
  }
#define RNSW_X(nres, ks3, wd, fs) \
  if (c.NRES == nres && c.KS3 == ks3 && c.wide == wd && c.fast == fs) { \
    if (!dry) launch(k3_inverse_crt<nres, ks3, wd, fs>, grid, 0, st, tm, P, O, y); return true; }
  RNSW_K3_TABLE(RNSW_X)
#undef RNSW_X
  return false;
}

// Every name of the tables above, one per line, as a profiler prints them.
std::string all_kernel_variants() {
  std::string out;
#define RNSW_X(ks, wd, pk) out += "k1_input_transform<" #ks ", " #wd ", " #pk ">\n";
  RNSW_K1_TABLE(RNSW_X)
#undef RNSW_X
#define RNSW_X(ks, ntb, rm, wd) out += "k2_residue_gemm<" #ks ", " #ntb ", " #rm ", " #wd ">\n";
  RNSW_K2_TABLE(RNSW_X)
#undef RNSW_X
#define RNSW_X(wm_, wn_, rm, ntb, s_) out += "k2_residue_gemm_lds<" #wm_ ", " #wn_ ", " #rm ", " #ntb ", " #s_ ">\n";
  RNSW_K2L_TABLE(RNSW_X)
#undef RNSW_X
#define RNSW_X(nres, ks3, wd, fs) out += "k3_inverse_crt<" #nres ", " #ks3 ", " #wd ", " #fs ">\n";
  RNSW_K3_TABLE(RNSW_X)
#undef RNSW_X
#define RNSW_X(nres, ks3, fs, m8) out += "k3_inverse_crt_stream<" #nres ", " #ks3 ", " #fs ", " #m8 ">\n";
  RNSW_K3S_TABLE(RNSW_X)
#undef RNSW_X
  return out;
}

// epi: 0 = int32 y_dev; 1 / 2 = int8 act_dev after shift/clamp (/ and 2x2 max-pool)
int conv2d_impl(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int32_t *y_dev,
                void *workspace_dev, void *stream, void *const *events, int epi = 0, int shift = 0,
                int8_t *act_dev = nullptr) {
  if (!plan || !x_dev || !U_dev || !workspace_dev) return RNSWINO_E_INVALID;
  if (epi == 0 ? !y_dev : !act_dev) return RNSWINO_E_INVALID;
  if (plan->device < 0) return RNSWINO_E_NO_DEVICE;
  if (!on_plan_device(plan)) return RNSWINO_E_INVALID;
  if (((uintptr_t)U_dev | (uintptr_t)workspace_dev | (uintptr_t)y_dev) & 15) return RNSWINO_E_INVALID;
  if ((uintptr_t)act_dev & 3) return RNSWINO_E_INVALID;
  const Dims &d = plan->dims;
  KParams P = *(const KParams *)plan->kparams;    // per call only the output mode differs
  P.epi = epi; P.shift = shift; P.act = act_dev;
  hipStream_t st = (hipStream_t)stream;
  int8_t *Vp = (int8_t *)workspace_dev;
  uint32_t *Op = (uint32_t *)((char *)workspace_dev + align256(v_bytes(d)));
  Timing t1, t2, t3;
  if (events) {
    t1.start = (hipEvent_t)events[0]; t1.stop = (hipEvent_t)events[1];
    t2.start = (hipEvent_t)events[2]; t2.stop = (hipEvent_t)events[3];
    t3.start = (hipEvent_t)events[4]; t3.stop = (hipEvent_t)events[5];
  }
  // (rnswino_plan() has checked that all three instantiations exist)
  if (!launch_k1(d, P, x_dev, Vp, st, t1) || !launch_k2(d, plan->desc.flags, P, (const int8_t *)U_dev, Vp, Op, st, t2) ||
      !launch_k3(d, P, plan->n_cus, Op, y_dev, st, t3))
    return RNSWINO_E_UNSUPPORTED;
  return launch_status();
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
  pl->n_cus = 0;
  pl->d_tables = nullptr;
  pl->d_tables_bytes = 0;
  pl->kparams = nullptr;
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
  const unsigned __int128 worst = output_bound(*desc, d);
  if (!(desc->flags & RNSWINO_FLAG_ALLOW_UNCHECKED_RANGE) && worst > half) { delete pl; return RNSWINO_E_RANGE; }
  std::memset(pl->mrc_inv, 0, sizeof(pl->mrc_inv));
  for (int l = 0; l < d.n; ++l)
    for (int j = l + 1; j < d.n; ++j) pl->mrc_inv[l][j] = (uint32_t)mod_inverse(desc->moduli[l], desc->moduli[j]);

  std::vector<char> &blob = pl->h_tables;
  build_tables(*pl, blob);
  if (!(desc->flags & RNSWINO_FLAG_HOST_ONLY)) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); delete pl; return RNSWINO_E_NO_DEVICE; }
    if (hipMalloc(&pl->d_tables, pl->d_tables_bytes) != hipSuccess) { (void)hipGetLastError(); delete pl; return RNSWINO_E_HIP; }
    if (hipMemcpy(pl->d_tables, blob.data(), pl->d_tables_bytes, hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipGetLastError(); (void)hipFree(pl->d_tables); delete pl; return RNSWINO_E_HIP;
    }
    pl->device = dev;
    rc = resolve_scratch(dev);
    if (rc != RNSWINO_OK) { (void)hipFree(pl->d_tables); delete pl; return rc; }
    {
      int cus = 0;
      if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess) pl->n_cus = cus;
      else (void)hipGetLastError();
    }
  }
  pl->kparams = new (std::nothrow) KParams(make_params(pl));
  if (!pl->kparams) { (void)rnswino_plan_destroy(pl); return RNSWINO_E_INVALID; }
  {
    // every kernel the layer would launch, in each output mode, must be an instantiation that exists
    KParams P = *(const KParams *)pl->kparams;
    bool ok = launch_k1(d, P, nullptr, nullptr, nullptr, Timing(), true) && launch_k2(d, pl->desc.flags, P, nullptr, nullptr, nullptr, nullptr, Timing(), true);
    for (int epi = 0; epi < 3 && ok; ++epi) {
      P.epi = epi;
      ok = launch_k3(d, P, pl->n_cus, nullptr, nullptr, nullptr, Timing(), true);
    }
    if (!ok) { (void)rnswino_plan_destroy(pl); return RNSWINO_E_UNSUPPORTED; }
  }
  *out = pl;
  return RNSWINO_OK;
}

int rnswino_plan_destroy(rnswino_plan_t *plan) {
  if (!plan) return RNSWINO_E_INVALID;
  int rc = RNSWINO_OK;
  if (plan->d_tables && hipFree(plan->d_tables) != hipSuccess) { (void)hipGetLastError(); rc = RNSWINO_E_HIP; }
  delete (KParams *)plan->kparams;
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
  if (!on_plan_device(plan)) return RNSWINO_E_INVALID;
  const Dims &d = plan->dims;
  const KParams P = *(const KParams *)plan->kparams;
  const long long total = (long long)d.n * d.Kp * d.Cp;
  hipStream_t st = (hipStream_t)stream;
  if (d.wide)
    hipLaunchKernelGGL(k0_filter_transform<true>, dim3(blocks_for(total, 256)), dim3(256), 0, st, P, w_dev, (int8_t *)U_dev);
  else
    hipLaunchKernelGGL(k0_filter_transform<false>, dim3(blocks_for(total, 256)), dim3(256), 0, st, P, w_dev, (int8_t *)U_dev);
  return launch_status();
}

int rnswino_conv2d(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int32_t *y_dev,
                   void *workspace_dev, void *stream) {
  return conv2d_impl(plan, x_dev, U_dev, y_dev, workspace_dev, stream, nullptr);
}

int rnswino_conv2d_requant(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int8_t *a_dev,
                           int32_t shift, int32_t pool, void *workspace_dev, void *stream) {
  if (!plan || shift < 0 || shift > 31) return RNSWINO_E_INVALID;
  const Dims &d = plan->dims;
  // pooling inside the kernel pairs rows and columns of one output tile: tiles of 4 or 8, whole pooling windows per row
  if (pool && ((d.m != 4 && d.m != 8) || (d.Wo & 3) || (d.Ho & 1))) return RNSWINO_E_UNSUPPORTED;
  return conv2d_impl(plan, x_dev, U_dev, nullptr, workspace_dev, stream, nullptr, pool ? 2 : 1, shift, a_dev);
}

int rnswino_conv2d_events(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int32_t *y_dev,
                          void *workspace_dev, void *stream, void *const events[6]) {
  if (!events) return RNSWINO_E_INVALID;
  return conv2d_impl(plan, x_dev, U_dev, y_dev, workspace_dev, stream, events);
}

int rnswino_debug_empty_launch(uint32_t grid_x, uint32_t grid_y, void *stream, void *start_event, void *stop_event) {
  if (grid_x == 0 || grid_y == 0 || grid_y > 65535u) return RNSWINO_E_INVALID;
  Timing tm;
  tm.start = (hipEvent_t)start_event;
  tm.stop = (hipEvent_t)stop_event;
  launch(k_empty, dim3(grid_x, grid_y), 0, (hipStream_t)stream, tm, 0);
  return launch_status();
}

int64_t rnswino_kernel_variants(char *host_out, size_t capacity) {
  const std::string all = all_kernel_variants();
  if (host_out && capacity > all.size()) std::memcpy(host_out, all.c_str(), all.size() + 1);
  return (int64_t)all.size() + 1;
}

int rnswino_conv2d_static(const rnswino_plan_t *plan, const int8_t *x_dev, const void *U_dev, int32_t *y_dev, void *stream) {
  if (!plan) return RNSWINO_E_INVALID;
  if (plan->device < 0) return RNSWINO_E_NO_DEVICE;
  if (rnswino_workspace_bytes(plan) > (size_t)RNSWINO_STATIC_WORKSPACE_BYTES) return RNSWINO_E_WORKSPACE;
  void *ws = plan->device < MAX_DEVICES ? scratch_ptr[plan->device] : nullptr;   // set when the plan was made
  if (!ws) return RNSWINO_E_HIP;
  return conv2d_impl(plan, x_dev, U_dev, y_dev, ws, stream, nullptr);
}

int64_t rnswino_plan_describe(const rnswino_plan_t *plan, int32_t output_mode, char *host_out, size_t capacity) {
  if (!plan || output_mode < 0 || output_mode > 2) return RNSWINO_E_INVALID;
  const Dims &d = plan->dims;
  const KParams &P = *(const KParams *)plan->kparams;
  const K1Choice c1 = choose_k1(d);
  const K2Choice c2 = choose_k2(d, plan->desc.flags);
  const K3Choice c3 = choose_k3(d, P, plan->n_cus, output_mode);
  auto tf = [](bool b) { return b ? "true" : "false"; };
  char buf[1024];
  int len = std::snprintf(buf, sizeof(buf), "k1_input_transform<%d, %s, %s> grid=%ux%u\n", c1.KS1, tf(c1.wide), tf(c1.pack), c1.gx, c1.gy);
  if (c2.lds)
    len += std::snprintf(buf + len, sizeof(buf) - len, "k2_residue_gemm_lds<%d, %d, %d, %d, %d> grid=%u xgroup=%d\n", c2.WM, c2.WN, c2.RM,
                         c2.NTB, c2.S, c2.blocks, c2.xgroup);
  else
    len += std::snprintf(buf + len, sizeof(buf) - len, "k2_residue_gemm<%d, %d, %d, %s> grid=%u xgroup=%d\n", c2.KS, c2.NTB, c2.RM,
                         tf(c2.wide), c2.blocks, c2.xgroup);
  if (c3.stream)
    len += std::snprintf(buf + len, sizeof(buf) - len, "k3_inverse_crt_stream<%d, %d, %s, %s> grid=%ux%u lds=%zu\n", c3.NRES, c3.KS3,
                         tf(c3.fast), tf(c3.m8), c3.gx, c3.gy, c3.lds);
  else
    len += std::snprintf(buf + len, sizeof(buf) - len, "k3_inverse_crt<%d, %d, %s, %s> grid=%ux%u\n", c3.NRES, c3.KS3, tf(c3.wide),
                         tf(c3.fast), c3.gx, c3.gy);
  const char *conv = P.fastcrt == 1 ? "unreduced-binary32"
                     : P.fastcrt == 2 ? "unreduced-binary64"
                     : !P.crt24 ? "reduced-binary64-mul32"
                     : P.quot32 ? "reduced-binary32" : "reduced-binary64";
  len += std::snprintf(buf + len, sizeof(buf) - len, "conversion=%s\n", conv);
  if (host_out && capacity > (size_t)len) std::memcpy(host_out, buf, (size_t)len + 1);
  return (int64_t)len + 1;
}

// ---- direct convolution (the comparison baseline of section 8) ----
static int direct_params(int32_t N, int32_t C, int32_t K, int32_t H, int32_t W, int32_t r, int32_t pad, DirectParams &P) {
  if (N <= 0 || C <= 0 || K <= 0 || H <= 0 || W <= 0 || r <= 0 || pad < 0) return RNSWINO_E_INVALID;
  const long long Ho = (long long)H + 2LL * pad - r + 1, Wo = (long long)W + 2LL * pad - r + 1;
  if (Ho <= 0 || Wo <= 0) return RNSWINO_E_INVALID;
  if (r > 16) return RNSWINO_E_UNSUPPORTED;
  if ((unsigned __int128)16384u * (unsigned)r * (unsigned)r * (unsigned)C > 2147483647u) return RNSWINO_E_UNSUPPORTED;   // int32 sums
  P.N = N; P.C = C; P.K = K; P.H = H; P.W = W; P.r = r; P.pad = pad;
  P.Ho = (int)Ho; P.Wo = (int)Wo; P.Hp = H + 2 * pad; P.Wp = W + 2 * pad;
  P.Cp = (C + 63) / 64 * 64; P.Kp = (K + 15) / 16 * 16;
  const long long npix = (long long)N * Ho * Wo, xt = (long long)N * P.Hp * P.Wp * P.Cp;
  if (npix >= (1LL << 28) || xt >= (1LL << 31) || (long long)r * r * P.Kp * P.Cp >= (1LL << 31)) return RNSWINO_E_UNSUPPORTED;   // 32-bit offsets
  P.npix = (int)npix;
  return RNSWINO_OK;
}

size_t rnswino_direct_filter_bytes(int32_t C, int32_t K, int32_t r) {
  DirectParams P;
  if (direct_params(1, C, K, r, r, r, 0, P) != RNSWINO_OK) return 0;
  return align256((size_t)r * r * P.Kp * P.Cp);
}

size_t rnswino_direct_workspace_bytes(int32_t N, int32_t C, int32_t H, int32_t W, int32_t pad) {
  DirectParams P;
  if (direct_params(N, C, 1, H, W, 1, pad, P) != RNSWINO_OK) return 0;
  return align256((size_t)N * P.Hp * P.Wp * P.Cp);
}

int rnswino_direct_filter_pack(const int8_t *w_dev, void *wt_dev, int32_t C, int32_t K, int32_t r, void *stream) {
  if (!w_dev || !wt_dev) return RNSWINO_E_INVALID;
  if ((uintptr_t)wt_dev & 15) return RNSWINO_E_INVALID;
  DirectParams P;
  const int rc = direct_params(1, C, K, r, r, r, 0, P);
  if (rc != RNSWINO_OK) return rc;
  const long long total = (long long)r * r * P.Kp * (P.Cp / 16);
  hipLaunchKernelGGL(k_direct_pack_filter, dim3(blocks_for(total, 256)), dim3(256), 0, (hipStream_t)stream, P, w_dev, (int8_t *)wt_dev);
  return launch_status();
}

int rnswino_direct_conv2d(const int8_t *x_dev, const void *wt_dev, int32_t *y_dev, int32_t N, int32_t C, int32_t K, int32_t H,
                          int32_t W, int32_t r, int32_t pad, void *workspace_dev, void *stream) {
  if (!x_dev || !wt_dev || !y_dev || !workspace_dev) return RNSWINO_E_INVALID;
  if (((uintptr_t)wt_dev | (uintptr_t)workspace_dev) & 15) return RNSWINO_E_INVALID;
  DirectParams P;
  const int rc = direct_params(N, C, K, H, W, r, pad, P);
  if (rc != RNSWINO_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  int8_t *xt = (int8_t *)workspace_dev;
  const long long tblocks = (long long)N * P.Hp * (P.Cp / 64) * ((P.Wp + 63) / 64);
  hipLaunchKernelGGL(k_direct_to_nhwc, dim3((unsigned)tblocks), dim3(256), 0, st, P, x_dev, xt);
  // block shape: 128 x 128 when that still gives the chip two workgroups per compute unit, else 128 x 64, else 64 x 64;
  // layers with at most 64 filters take 64 x 256
  const long long nkb = P.Kp / 16, ntb = (P.npix + 15) / 16;
  auto blocks = [&](int brf, int btf) { return ((nkb + brf - 1) / brf) * (((ntb + btf - 1) / btf + 7) / 8 * 8); };
  if (P.Kp <= 64 && blocks(4, 16) >= 512)
    hipLaunchKernelGGL((k_direct_conv<1, 4, 4, 4, 3>), dim3((unsigned)blocks(4, 16)), dim3(256), 0, st, P, xt, (const int8_t *)wt_dev, y_dev);
  else if (P.Kp > 64 && blocks(8, 8) >= 512)
    hipLaunchKernelGGL((k_direct_conv<2, 2, 4, 4, 3>), dim3((unsigned)blocks(8, 8)), dim3(256), 0, st, P, xt, (const int8_t *)wt_dev, y_dev);
  else if (P.Kp > 64 && blocks(8, 4) >= 512)
    hipLaunchKernelGGL((k_direct_conv<4, 1, 2, 4, 4>), dim3((unsigned)blocks(8, 4)), dim3(256), 0, st, P, xt, (const int8_t *)wt_dev, y_dev);
  else
    hipLaunchKernelGGL((k_direct_conv<4, 1, 1, 4, 4>), dim3((unsigned)blocks(4, 4)), dim3(256), 0, st, P, xt, (const int8_t *)wt_dev, y_dev);
  return launch_status();
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

int64_t rnswino_plan_get_table(const rnswino_plan_t *plan, int which, int modulus_idx, int8_t *host_out, size_t capacity) {
  if (!plan || modulus_idx < 0 || modulus_idx >= plan->dims.n) return RNSWINO_E_INVALID;
  const Dims &d = plan->dims;
  const size_t planes = d.wide ? 2 : 1;
  size_t per, off;
  if (which == RNSWINO_TABLE_INPUT) { per = (size_t)d.CB1 * d.KS1 * planes * 1024; off = plan->off_KB; }
  else if (which == RNSWINO_TABLE_INVERSE) { per = (size_t)d.RB3 * d.KS3 * planes * 1024; off = plan->off_KA; }
  else return RNSWINO_E_INVALID;
  off += per * (size_t)modulus_idx;
  if (off + per > plan->h_tables.size()) return RNSWINO_E_INVALID;
  if (host_out && capacity >= per) std::memcpy(host_out, plan->h_tables.data() + off, per);
  return (int64_t)per;
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
  size_t bytes, skip = 0;
  if (stage == RNSWINO_STAGE_U) bytes = u_bytes(d);
  else if (stage == RNSWINO_STAGE_V) bytes = v_bytes(d);
  else if (stage == RNSWINO_STAGE_O) { bytes = o_bytes(d); skip = align256(v_bytes(d)); }
  else return RNSWINO_E_INVALID;
  std::vector<int8_t> raw(bytes);
  if (hipDeviceSynchronize() != hipSuccess ||
      hipMemcpy(raw.data(), (const char *)src_dev + skip, bytes, hipMemcpyDeviceToHost) != hipSuccess) {
    (void)hipGetLastError();
    return RNSWINO_E_HIP;
  }
  for (int i = 0; i < d.n; ++i) {
    const int64_t p = plan->desc.moduli[i];
    for (int pt = 0; pt < d.P2; ++pt) {
      const int slab = i * d.P2 + pt;
      auto value = [&](size_t narrow, size_t hi, size_t lo) -> int32_t {
        return d.wide ? sym_residue(256 * (int64_t)raw[hi] + (int64_t)raw[lo], p) : sym_residue((int64_t)raw[narrow], p);
      };
      if (stage == RNSWINO_STAGE_U) {
        // packed layers: the filter sits in every diagonal block (k * TL + tl, tl * Cq + c); block tl = 0 is read
        for (int k = 0; k < d.K; ++k)
          for (int c = 0; c < d.C; ++c) {
            const int kg = k * d.TL;
            host_out[((size_t)slab * d.K + k) * d.C + c] =
                d.wide ? value(0, u_offset_wide(slab, kg, c, d.Kp, d.Cp, 0), u_offset_wide(slab, kg, c, d.Kp, d.Cp, 1))
                       : value(u_offset(slab, kg, c, d.Kp, d.Cp), 0, 0);
          }
      } else if (stage == RNSWINO_STAGE_V) {
        for (int tau = 0; tau < d.T; ++tau)
          for (int c = 0; c < d.C; ++c) {
            const int tg = tau % d.Tg, cg = (tau / d.Tg) * d.Cq + c;       // GEMM column and channel (cg = c when TL = 1)
            host_out[((size_t)slab * d.T + tau) * d.C + c] =
                d.wide ? value(0, v_offset_wide(slab, d.n * d.P2, tg, cg, d.Cp, 0), v_offset_wide(slab, d.n * d.P2, tg, cg, d.Cp, 1))
                       : value(v_offset(slab, d.n * d.P2, tg, cg, d.Cp), 0, 0);
          }
      } else {
        for (int k = 0; k < d.K; ++k)
          for (int tau = 0; tau < d.T; ++tau) {
            const int kg = k * d.TL + tau / d.Tg, tg = tau % d.Tg;          // GEMM row and column
            host_out[((size_t)slab * d.K + k) * d.T + tau] =
                d.wide ? value(0, o_offset_wide(i, pt, kg, tg, d.n, d.Q, d.Kp, d.Tp, 0), o_offset_wide(i, pt, kg, tg, d.n, d.Q, d.Kp, d.Tp, 1))
                       : value(o_offset(i, pt, kg, tg, d.n, d.Q, d.Kp, d.Tp), 0, 0);
          }
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
    case RNSWINO_E_RANGE: return "dynamic range of the moduli set is below the output bound (worst case 2^14 r^2 C unless the caller gave a tighter one)";
    case RNSWINO_E_HIP: return "HIP runtime error";
    case RNSWINO_E_NO_DEVICE: return "plan is host-only or no GPU is available";
    case RNSWINO_E_WORKSPACE: return "the layer needs more workspace than the library's static buffer holds";
    default: return "unknown error";
  }
}

}  // extern "C"
