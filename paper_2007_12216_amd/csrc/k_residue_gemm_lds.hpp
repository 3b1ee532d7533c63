// K2, LDS-tiled form for 8-bit moduli: the residue-domain GEMM of paper section 6, eq. "gemm",
//   O[i][xi,nu][k][tau] = (sum_c U[i][xi,nu][k][c] V[i][xi,nu][tau][c]) mod p_i,
// with the operand fragments of a (rows x tiles) block shared by the four waves of a workgroup through LDS.
//
// A workgroup owns, for one residue i and one group q of four transform points, a block of 16*WM*RM rows (k) by
// 16*WN*NT tiles; wave (wm, wn) computes the 16*RM x 16*NT part of it.  The four points of the group are taken one
// after the other: per point the contraction over C runs in steps of 64 channels, each step needing WM*RM fragments
// of U and WN*NT fragments of V (1 KiB each, layout.hpp).  These travel from global memory straight into LDS
// (global_load_lds_dwordx4: no registers are held while a load is in flight), S steps deep, each wave issuing its
// share; a fragment lands in LDS in lane order, so one ds_read_b128 per lane hands a wave its operand.  Every fragment
// fetched from L2 feeds RM*WN (U) or NT*WM (V) products instead of RM or NT: the traffic between L2 and the compute
// unit per product drops by the sharing factor, which is what bounds the register-direct kernel on large layers.
// When a point's sum is complete it is reduced modulo p_i and its low byte is inserted into the lane's output words
// (byte e of a word of O is point 4q + e), so after the fourth point the wave holds finished words of O and stores
// them; no exchange between waves is needed.
//
// One barrier per step: a wave waits for its own loads of the step (they were issued S - 1 steps earlier), the
// barrier then says that everybody's have landed and that everybody is done reading the slot that is refilled next.
// The loads are issued from inline assembly and counted by hand (s_waitcnt vmcnt): left to the compiler, every read
// of LDS that might see such a load's data waits for all of them, which would leave a single step in flight.  The
// kernel has no other vector-memory loads, so the hand count is the whole count.
// Grid: one-dimensional, as for k2_residue_gemm (x = residue and point group, y = row block, z = tile block).
#pragma once
#include "kernels_common.hpp"

namespace rnswino {

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x0F70 | ((N >> 4) << 14));
}

// One 16-byte-per-lane load from global memory straight into LDS: lane l's 16 bytes from base + lane_off land at
// lds_addr + 16 l (lds_addr: wave-uniform byte address within LDS, passed in M0).  The s_nop is the wait state the
// instruction set asks for between a scalar write of M0 and an LDS-direct load that reads it (the compiler inserts it for
// its own code, not inside inline assembly).
__device__ __forceinline__ void load_to_lds16(const void *base, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}

template <int WM, int WN, int RM, int NT, int S>
__global__ __launch_bounds__(256) void k2_residue_gemm_lds(KParams P, const int8_t *__restrict__ U,
                                                            const int8_t *__restrict__ V, uint32_t *__restrict__ O, int xgroup) {
  static_assert(WM * WN == 4, "four waves per workgroup");
  constexpr int BRF = WM * RM, BTF = WN * NT;     // U and V fragments per step
  constexpr int NF = BRF + BTF;
  constexpr int LPW = (NF + 3) / 4;               // loads per wave and step (slots past NF are fillers, never read)
  constexpr int SLOTS = 4 * LPW;
  __shared__ __attribute__((aligned(16))) uint8_t stage[S * SLOTS * 1024];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int wm = wave / WN, wn = wave % WN;
  const int nkb = P.Kp >> 4, ntb = P.Tp >> 4, ncb = P.Cp >> 6;
  // work item from the linear id: same order as k2_residue_gemm (x on one XCD, groups of x, then rows, then tiles)
  const int gy = (nkb + BRF - 1) / BRF, gz = (ntb + BTF - 1) / BTF;
  int rest = blockIdx.x >> 3;
  const int xi = rest % xgroup;
  rest /= xgroup;
  const int by = rest % gy;
  rest /= gy;
  const int bz = rest % gz;
  const int bx = ((rest / gz) * xgroup + xi) * 8 + (blockIdx.x & 7);
  if (bx >= P.n * P.Q) return;                    // x is padded to a multiple of 8 (block-uniform: no barrier is skipped by part of a block)
  const int i = bx / P.Q, q = bx % P.Q;
  const int kb0 = by * BRF, tb0 = bz * BTF;
  const int p = P.p[i];
  const float inv = P.inv_p[i];
  const int npts = min(4, P.P2 - 4 * q);          // points of this group that exist (t*t need not be a multiple of 4)
  const int total = npts * ncb;                   // steps of the whole block
  const int slab0 = i * P.P2 + 4 * q;

  // This wave's loads of a step: fragment f = wave + 4 j, at base[j] + slab * slab_stride[j] + cb KiB (wave-uniform)
  // plus the lane's offset inside the fragment; row and tile blocks past the end are clamped to the last one (what
  // they produce is never stored).
  const int8_t *base[LPW];
  uint32_t slab_stride[LPW], lane_off[LPW];
#pragma unroll
  for (int j = 0; j < LPW; ++j) {
    const int f = min(wave + 4 * j, NF - 1);      // filler slots repeat the last fragment
    if (f < BRF) {
      base[j] = U + (size_t)min(kb0 + f, nkb - 1) * ncb * 1024;
      slab_stride[j] = (uint32_t)(nkb * ncb) * 1024u;
      lane_off[j] = (uint32_t)lane * 16u;
    } else {
      base[j] = V + (size_t)min(tb0 + f - BRF, ntb - 1) * (P.n * P.P2) * ncb * 1024;
      slab_stride[j] = (uint32_t)ncb * 1024u;
      lane_off[j] = (uint32_t)((lane & 15) * 64 + (lane >> 4) * 16);
    }
  }
  const uint32_t stage_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t *)stage;
  auto issue = [&](int step_e, int step_cb, int slot) {
#pragma unroll
    for (int j = 0; j < LPW; ++j)
      load_to_lds16(base[j] + (size_t)(slab0 + step_e) * slab_stride[j] + (size_t)step_cb * 1024, lane_off[j],
                    stage_lds + (uint32_t)((slot * SLOTS + wave + 4 * j) * 1024));
  };

  // prologue: the first S - 1 steps
  int pe = 0, pcb = 0;                            // the step the next issue() fetches
  auto advance = [&]() {
    if (++pcb == ncb) { pcb = 0; ++pe; }
  };
#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (pe < npts) { issue(pe, pcb, s); advance(); }

  v4i acc[RM][NT];
  uint32_t packed[RM][NT][4];
#pragma unroll
  for (int rm = 0; rm < RM; ++rm)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int j = 0; j < 4; ++j) packed[rm][nt][j] = 0;
#pragma unroll
  for (int rm = 0; rm < RM; ++rm)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[rm][nt] = (v4i){0, 0, 0, 0};

  const uint8_t *lds_a = stage + (wm * RM) * 1024 + lane * 16;
  const uint8_t *lds_b = stage + (BRF + wn * NT) * 1024 + lane * 16;
  int slot = 0, fill = S - 1;                     // slot read by this step, slot refilled by it
  int e = 0, cb = 0;
  for (int it = 0; it < total; ++it) {
    // this wave's loads of step `it` have landed once at most those of the later steps already issued (S - 2 of them,
    // fewer at the very end) are outstanding
    const int rem = total - 1 - it;
    if (rem >= S - 2) wait_vmcnt<LPW * (S - 2)>();
    else if (S >= 4 && rem == 1) wait_vmcnt<LPW>();
    else wait_vmcnt<0>();
    __syncthreads();
    if (pe < npts) { issue(pe, pcb, fill); advance(); }
    v4i a[RM];
#pragma unroll
    for (int rm = 0; rm < RM; ++rm) a[rm] = *(const v4i *)(lds_a + (slot * SLOTS + rm) * 1024);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const v4i b = *(const v4i *)(lds_b + (slot * SLOTS + nt) * 1024);
#pragma unroll
      for (int rm = 0; rm < RM; ++rm)
        acc[rm][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[rm], b, acc[rm][nt], 0, 0, 0);
    }
    if (++slot == S) slot = 0;
    if (++fill == S) fill = 0;
    ++cb;
    // 8-bit residues, |U|, |V| <= 127: 512 channels add at most 8.3e6, so reducing every 8 steps keeps |acc| < 2^24
    if ((cb & 7) == 0 && cb < ncb) {
#pragma unroll
      for (int rm = 0; rm < RM; ++rm)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[rm][nt][j] = mod_near(acc[rm][nt][j], inv, p);
    }
    if (cb == ncb) {
      // the point's sums are complete: low byte of the residue into byte e of the output words
      const uint32_t sel = e == 0 ? 0x03020104u : e == 1 ? 0x03020400u : e == 2 ? 0x03040100u : 0x04020100u;
#pragma unroll
      for (int rm = 0; rm < RM; ++rm)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            packed[rm][nt][j] = __builtin_amdgcn_perm(mod_lowbyte(acc[rm][nt][j], inv, -p), packed[rm][nt][j], sel);
#pragma unroll
      for (int rm = 0; rm < RM; ++rm)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[rm][nt] = (v4i){0, 0, 0, 0};
      cb = 0;
      ++e;
    }
  }
  // O is [Kp][n][Q][Tp] words and smaller than 4 GiB.  A lane holds rows 16 (kb) + 4 (lane / 16) + j and tile
  // 16 (tb) + lane % 16: sixteen lanes write 64 consecutive bytes of a row.
  const uint32_t krow = (uint32_t)(P.n * P.Q * P.Tp);
#pragma unroll
  for (int rm = 0; rm < RM; ++rm) {
    const int kb = kb0 + wm * RM + rm;
    if (kb >= nkb) break;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int tb = tb0 + wn * NT + nt;
      if (tb >= ntb) break;
      const uint32_t off = (uint32_t)(kb * 16 + 4 * (lane >> 4)) * krow + (uint32_t)((i * P.Q + q) * P.Tp + tb * 16 + (lane & 15));
#pragma unroll
      for (int j = 0; j < 4; ++j) O[off + j * krow] = packed[rm][nt][j];
    }
  }
}

}  // namespace rnswino
