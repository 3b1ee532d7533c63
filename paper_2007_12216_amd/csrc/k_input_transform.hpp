// K1: input transform on the matrix cores.
//
// V[i][xi,nu][tau][c] = (B^T_p d B_p)[xi,nu] mod p_i for every tile tau and channel c (paper section 6: shared
// by all K filters).  B^T d B = (B^T kron B^T) vec(d): per residue one dense (t*t) x (t*t) matrix applied to the
// t*t pixels of a tile, i.e. a GEMM whose columns are the (tile, channel) pairs.  MFMA roles
// (v_mfma_i32_16x16x64_i8): A operand = pixels (rows = 16 channels of one tile), B operand = the Kronecker
// table (columns = 16 transform points), contraction index = pixel.  A tile row takes RP1 = 4 ceil(t/4)
// contraction slots (its t pixels, then zero weights), the tile t * RP1 slots in KS1 = ceil(t * RP1 / 64) steps of
// 64 (t = 10: 120 slots, two steps; rows of 16 slots would need three).  A row segment is one unaligned 16-byte
// load of an image row, masked where the tile hangs over the image border (zero padding and ragged last tiles),
// of which the first RP1 bytes go to LDS; a lane's 16 operand bytes are then 16 consecutive slots.
//
// Block = (tile, block of 64 channels, one residue or all of them): its 64 x t x RP1 pixel patch is gathered once into
// LDS (the gather of 16-byte row segments is what costs; sharing it between the four waves pays), then each wave
// walks over its steps (residue, every fourth group of K1_CPW column blocks), the table fragments of the next
// step in flight while the current one is multiplied.  Accumulator rows are channels 4g+j, so the four channel
// groups u give one lane exactly the 16 bytes of V it has to store (channel order of layout.hpp).
// 16-bit moduli: the table has a high and a low byte plane, V = (256 * sum_h + sum_l) mod p, stored as two planes.
// Grid: x = T * Cp/64 rounded up to a multiple of 8 (see xcd_chunked), y = n (one residue per block) or 1 (the block
// walks over all residues with the same gathered patch); 256 threads; 64 * (4*KS1 + 1) * 16 bytes of LDS.
#pragma once
#include "kernels_common.hpp"

namespace rnswino {

constexpr int K1_CPW = 2;

// PACK: the layer packs TL tiles into one 64-channel block (plan.hpp): block channel c' holds channel c' % Cq of tile
// (c' / Cq) * Tg + tau, so every gathered row segment has its own tile origin; everything after the gather is the same.
template <int KS1, bool WIDE, bool PACK>
__global__ __launch_bounds__(256) void k1_input_transform(KParams P, const int8_t *__restrict__ x,
                                                           int8_t *__restrict__ V) {
  constexpr int ROWS = KS1 == 1 ? 8 : KS1 == 2 ? 10 : KS1 == 3 ? 12 : 16;   // largest t with this many steps
  constexpr int PL = WIDE ? 2 : 1;
  constexpr int CROW = (4 * KS1 + 1) * 16;   // bytes per channel in LDS: one 16-byte pad, so that the 16 channels a
                                             // fragment read touches fall into different banks
  __shared__ __attribute__((aligned(16))) uint8_t xs[64 * CROW];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: table addresses stay scalar
  const int lane = threadIdx.x & 63, g = lane >> 4;
  const int ncb = P.Cp >> 6;
  const int i0 = gridDim.y == 1 ? 0 : blockIdx.y, i1 = gridDim.y == 1 ? P.n : i0 + 1;   // residues of this block
  const int unit = xcd_chunked(blockIdx.x, gridDim.x, P.Tg * ncb);  // neighbouring tiles (shared image lines) on one XCD
  if (unit < 0) return;
  const int cb = unit % ncb, tau = unit / ncb;     // tau: GEMM column (a group of TL tiles when PACK)
  {
    const long long total = (long long)P.N * P.C * P.H * P.W;
    // origin, tile and channel of the row segment that goes to block channel cblk
    struct Seg { long long base; int y0, x0; bool ok; };
    auto tile_origin = [&](int tile, int ch) -> Seg {
      const int trow = tile / P.tw;
      const int tx = tile - trow * P.tw, img = trow / P.th, ty = trow - img * P.th;
      Seg sg;
      sg.y0 = ty * P.m - P.pad;
      sg.x0 = tx * P.m - P.pad;
      sg.ok = tile < P.T;
      sg.base = (((long long)img * P.C + ch) * P.H + sg.y0) * P.W + sg.x0;   // byte index of (ch, row y0, column x0)
      return sg;
    };
    const Seg block_seg = tile_origin(PACK ? 0 : tau, PACK ? 0 : cb * 64);   // not packed: one tile, block-uniform
    auto segment = [&](int cblk) -> Seg {
      if (PACK) {
        Seg sg = tile_origin((cblk / P.Cq) * P.Tg + tau, cblk % P.Cq);
        sg.ok = sg.ok && (cblk % P.Cq) < P.C;
        return sg;
      }
      Seg sg = block_seg;
      sg.ok = cb * 64 + cblk < P.C;
      sg.base += (cblk * P.H) * P.W;               // 64 * H * W stays far below 2^31
      return sg;
    };
    // columns b of the 16-pixel row segment that lie inside the image and inside the tile: [lo, hi)
    auto column_mask = [&](int x0, uint32_t (&cmask)[4]) {
      const int lo = x0 < 0 ? -x0 : 0;
      const int hi = min(P.t, P.W - x0);
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        uint32_t mk = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) mk |= ((4 * d + e) >= lo && (4 * d + e) < hi) ? (0xFFu << (8 * e)) : 0u;
        cmask[d] = mk;
      }
    };
    // A thread's NT row segments are requested together and only then masked and written to LDS (one after the
    // other, each load would be waited for in turn: three memory latencies instead of one).
    constexpr int NT = (64 * ROWS + 255) / 256;
    v4i val[NT];
    long long b0[NT];
    int sx0[NT];
    int state[NT];                                     // 0: nothing to load, 1: plain 16-byte load, 2: tensor edge
#pragma unroll
    for (int k = 0; k < NT; ++k) {
      const int task = threadIdx.x + 256 * k;
      const int c = task / ROWS, a = task - c * ROWS;
      const Seg sg = segment(c);
      const int gy = sg.y0 + a;
      val[k] = (v4i){0, 0, 0, 0};
      b0[k] = sg.base + (long long)a * P.W;
      sx0[k] = sg.x0;
      state[k] = 0;
      if (task < 64 * ROWS && sg.ok && a < P.t && gy >= 0 && gy < P.H)
        state[k] = (b0[k] >= 0 && b0[k] + 16 <= total) ? 1 : 2;
      if (state[k] == 1) __builtin_memcpy(&val[k], x + b0[k], 16);      // one unaligned 16-byte load
    }
#pragma unroll
    for (int k = 0; k < NT; ++k) {
      if (state[k] == 2) {                             // first / last bytes of the tensor
        uint32_t wv[4] = {0, 0, 0, 0};
        for (int b = 0; b < 16; ++b) {
          const long long o = b0[k] + b;
          if (o >= 0 && o < total) wv[b >> 2] |= (uint32_t)(uint8_t)x[o] << (8 * (b & 3));
        }
        val[k] = (v4i){(int)wv[0], (int)wv[1], (int)wv[2], (int)wv[3]};
      }
    }
#pragma unroll
    for (int k = 0; k < NT; ++k) {
      const int task = threadIdx.x + 256 * k;
      const int c = task / ROWS, a = task - c * ROWS;
      uint32_t cmask[4];
      column_mask(sx0[k], cmask);
      val[k][0] &= cmask[0]; val[k][1] &= cmask[1]; val[k][2] &= cmask[2]; val[k][3] &= cmask[3];
      // the first RP1 bytes of the segment are the row's slots (the slots past t * RP1 are never written: their
      // table entries are zero, and any byte times zero is zero)
      if (task < 64 * ROWS && a < P.t) {
        uint32_t *row = (uint32_t *)(xs + c * CROW + a * P.RP1);
        row[0] = (uint32_t)val[k][0];
        if (P.RP1 > 4) row[1] = (uint32_t)val[k][1];
        if (P.RP1 > 8) row[2] = (uint32_t)val[k][2];
        if (P.RP1 > 12) row[3] = (uint32_t)val[k][3];
      }
    }
  }
  // This wave's work: steps (residue i, column-block group cg) with cg = wave, wave + 4, ...  The table fragments
  // of step k+1 are requested before step k is multiplied; those of step 0 before the barrier, so that their
  // latency overlaps the gather.  A step's position is kept as wave-uniform scalars and advanced incrementally
  // (no divisions, and only a few scalar operations per column block: every instruction counts here).
  const int ncg = (P.CB1 + K1_CPW - 1) / K1_CPW;
  const int per_i = (ncg - wave + 3) >> 2;            // groups of this wave per residue
  const int nsteps = (i1 - i0) * per_i;
  struct Pos { int i, cg; };                          // residue and column-block group
  auto advance = [&](Pos &q) {
    q.cg += 4;
    if (q.cg >= ncg) { q.cg = wave; ++q.i; }
  };
  constexpr uint32_t FRAG = KS1 * PL * 1024;          // table bytes per column block (all steps and planes)
  const int8_t *KBl = P.KB + lane * 16;
  auto load_table = [&](const Pos &q, v4i (&b)[K1_CPW][KS1][PL]) {
#pragma unroll
    for (int cc = 0; cc < K1_CPW; ++cc) {
      const int cbk = min(q.cg * K1_CPW + cc, P.CB1 - 1);
      const int8_t *frag = KBl + (uint32_t)(q.i * P.CB1 + cbk) * FRAG;   // the whole table is far below 4 GiB
#pragma unroll
      for (int s = 0; s < KS1; ++s)
#pragma unroll
        for (int pl = 0; pl < PL; ++pl) b[cc][s][pl] = *(const v4i *)(frag + (s * PL + pl) * 1024);
    }
  };
  // Where a column block's 16 transform points go in V: wave-uniform 64-bit part (tile block, residue, column block,
  // channel block, tile) + the lane's 32-bit part (its point within the column block, its four channels), so the
  // address costs the vector unit next to nothing.  stride_pt = bytes between consecutive transform points.
  const uint32_t stride_pt = (uint32_t)(ncb * PL * 1024);
  const uint32_t lane_store = (uint32_t)(lane & 15) * stride_pt + g * 16;   // 16 points * ncb KiB: far below 2^32
  int8_t *const Vtile = V + ((size_t)(tau >> 4) * (size_t)(P.n * P.P2) * ncb + cb) * (PL * 1024) + (tau & 15) * 64;
  v4i bf[K1_CPW][KS1][PL], bn[K1_CPW][KS1][PL];
  Pos cur = {i0, wave};
  if (nsteps > 0) load_table(cur, bf);
  __syncthreads();
  if (nsteps <= 0) return;
  // All loads issued so far are awaited here, explicitly: otherwise the compiler, merging this entry state with the
  // loop's own, makes every step wait for the fragments it has just requested for the next one.
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), other counters untouched

  v4i af[4][KS1];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int s = 0; s < KS1; ++s) af[u][s] = *(const v4i *)(xs + (16 * u + (lane & 15)) * CROW + (4 * s + g) * 16);   // slots 64 s + 16 g ..

  // One step with the fragments in `b`, while those of the following step travel into `bnext`.  The loop below
  // alternates the two register sets instead of copying one into the other: a copy would have to wait for every
  // memory operation issued before it, the step's own stores included.
  auto do_step = [&](int step, v4i (&b)[K1_CPW][KS1][PL], v4i (&bnext)[K1_CPW][KS1][PL]) {
    const int i = cur.i, cg = cur.cg;
    advance(cur);
    if (step + 1 < nsteps) load_table(cur, bnext);
    const int p = P.p[i];
    const float inv = P.inv_p[i];
    const double invd = P.inv_pd[i];
#pragma unroll
    for (int cc = 0; cc < K1_CPW; ++cc) {
      const int cbk = cg * K1_CPW + cc;
      if (cbk >= P.CB1) break;
      v4i acc[PL][4];
#pragma unroll
      for (int pl = 0; pl < PL; ++pl)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[pl][u] = (v4i){0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KS1; ++s)
#pragma unroll
        for (int pl = 0; pl < PL; ++pl)
#pragma unroll
          for (int u = 0; u < 4; ++u)
            acc[pl][u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[u][s], b[cc][s][pl], acc[pl][u], 0, 0, 0);
      const int pt = 16 * cbk + (lane & 15);
      int8_t *dst = Vtile + (size_t)(uint32_t)(i * P.P2 + 16 * cbk) * stride_pt + lane_store;
      if (WIDE) {
        // per plane |acc| <= t*t * 128 * 128 = 2^22, so 256 * acc_h + acc_l fits 32 bits
        v4i out_h, out_l;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          uint32_t wh = 0, wl = 0;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int tot = acc[0][u][j] * 256 + acc[PL - 1][u][j];
            const int v = storable16(mod_near64((long long)tot, invd, p), p);
            const int lo = (int)(int8_t)(v & 0xFF), hi = (v - lo) >> 8;
            wh |= ((uint32_t)hi & 0xFFu) << (8 * j);
            wl |= ((uint32_t)lo & 0xFFu) << (8 * j);
          }
          out_h[u] = (int)wh;
          out_l[u] = (int)wl;
        }
        if (pt < P.P2) {
          *(v4i *)dst = out_h;
          *(v4i *)(dst + 1024) = out_l;
        }
      } else {
        // |acc| <= t*t * 126 * 128 < 2^24
        v4i out;
#pragma unroll
        for (int u = 0; u < 4; ++u)
          out[u] = (int)pack_low_bytes(mod_lowbyte(acc[0][u][0], inv, -p), mod_lowbyte(acc[0][u][1], inv, -p),
                                       mod_lowbyte(acc[0][u][2], inv, -p), mod_lowbyte(acc[0][u][3], inv, -p));
        if (pt < P.P2) *(v4i *)dst = out;
      }
    }
  };
  for (int step = 0; step < nsteps; step += 2) {
    do_step(step, bf, bn);
    if (step + 1 < nsteps) do_step(step + 1, bn, bf);
  }
}

}  // namespace rnswino
