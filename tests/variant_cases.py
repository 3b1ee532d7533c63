"""Layer shapes that, between them, run every kernel instantiation the library can launch.

The library reports which instantiation of each stage a plan launches (`rnswino_plan_describe`, no GPU needed) and the full
list of instantiations (`rnswino_kernel_variants`).  `select_cases()` walks over a fixed grid of small layers, cheapest first,
and keeps a layer whenever it launches a kernel (or takes a form of the conversion out of the RNS) that no kept layer has
launched yet.  The GPU test runs the kept layers against the direct-convolution oracle; a CPU test checks that together they
reach every instantiation.  Nothing here computes anything of the method.
"""
from __future__ import annotations

import functools
import itertools

import paper_2007_12216_amd as rn

PRIMES8 = (251, 241, 239, 233, 229, 227, 223, 211)
PRIMES16 = (65521, 65519, 65497, 65479, 65449, 65447, 65437, 65423)
HOST = rn.FLAG_HOST_ONLY
UNCHECKED = rn.FLAG_ALLOW_UNCHECKED_RANGE


def _candidates():
    """(cost, case) pairs; case = (N, C, K, H, W, r, m, pad, moduli, flags, output_mode).  output_mode as in
    rnswino_plan_describe: 0 = int32 output, 1 = fused shift/clamp to int8, 2 = the same with 2x2 max-pool."""
    out = []

    def add(N, C, K, H, W, r, m, pad, moduli, flags=0, mode=0):
        Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
        if Ho <= 0 or Wo <= 0 or m + r - 1 > 16 or m + r - 1 < 2:
            return
        P = 1
        for p in moduli:
            P *= p
        if not (flags & UNCHECKED) and (1 << 14) * r * r * C > (P - 1) // 2:
            return
        out.append((N * C * K * Ho * Wo * r * r, (N, C, K, H, W, r, m, pad, tuple(moduli), flags, mode)))

    # transform-tile sizes t = m + r - 1 that give every step count of the two transforms (t <= 8, 9-11, 12-13, 14-16)
    tiles = ((3, 4), (3, 8), (3, 10), (5, 12), (3, 14))
    # (a) small layers: every moduli count of both widths, every transform size, few / many channels, 1 / 2 / many tile blocks
    for (r, m), n, wide in itertools.product(tiles, range(1, 9), (False, True)):
        moduli = (PRIMES16 if wide else PRIMES8)[:n]
        for C, K, hw in ((3, 5, 4 * m), (5, 4, 8 * m), (20, 8, m), (70, 8, 2 * m), (130, 8, m), (192, 20, m), (256, 8, m)):
            for N in (1, 2):
                add(N, C, K, hw, hw, r, m, r // 2, moduli, UNCHECKED)
    # (b) contraction lengths of 1..4 channel blocks against 1, 2 and 3+ tile blocks (steps in flight of the GEMM), both widths
    for C, hw, wide in itertools.product((60, 128, 192, 256), (8, 24, 40), (False, True)):
        add(1, C, 24, hw, hw, 3, 6, 1, (PRIMES16[:2] if wide else PRIMES8[:4]))
        add(1, C, 24, 30, 30, 3, 6, 1, (PRIMES16[:2] if wide else PRIMES8[:4]))      # 25 tiles: two tile blocks
    # (b2) the same with fewer than 128 rows (the register-direct GEMM keeps those) and with 128 and more (LDS-tiled GEMM
    #      from three tile blocks on), ragged row and tile blocks included
    for C, K, hw in itertools.product((60, 128, 256), (24, 130, 200), (40, 64)):
        add(1, C, K, hw, hw, 3, 6, 1, PRIMES8[:4])
    add(1, 40, 136, 36, 36, 3, 7, 1, PRIMES8[:3])            # t = 9: a last point group with one point, LDS-tiled
    add(1, 70, 40, 40, 40, 3, 8, 1, PRIMES8[:4], rn.FLAG_GEMM_BLOCK_64X16)       # the measurement form of the LDS-tiled GEMM
    # (c) 64-row GEMM blocks: K >= 256, two or more channel blocks (even and odd), enough work items
    for C in (128, 192):
        add(3, C, 256, 64, 64, 3, 8, 1, PRIMES8[:4])
    # (d) streaming inverse transform: many (k, tile) units; 1..4 moduli; one and two contraction steps; 8 x 8 tiles and
    #     others; the three conversions (range checked with room: unreduced binary32; at the edge / unchecked: unreduced
    #     binary64; four large moduli unchecked: reduced); int32, int8 and pooled output
    for n, (r, m), mode in itertools.product(range(1, 5), ((3, 8), (3, 4), (3, 6), (3, 7)), (0, 1, 2)):
        for C, flags in ((33, 0), (33, UNCHECKED), (45, 0), (64, UNCHECKED), (200, UNCHECKED)):
            moduli = PRIMES8[:n]
            for N, K, hw in ((8, 96, 8 * m), (8, 64, 56), (4, 48, 16 * m)):
                if mode == 2 and (m not in (4, 8) or hw % 4):
                    continue
                add(N, C, K, hw, hw, r, m, 1, moduli, flags, mode)
    # 1 x 1 filters with 8 x 8 tiles: one contraction step together with the 8 x 8 store path
    for n, mode in itertools.product(range(1, 5), (0, 1, 2)):
        add(8, 40, 96, 64, 64, 1, 8, 0, PRIMES8[:n], UNCHECKED, mode)
    # four moduli whose product leaves the binary64 quotient of the unreduced form no room, on layers whose worst case
    # 2^14 r^2 C is above 0.38 of that product (binary32 has no room either): the conversion over reduced residues
    big4 = (253, 251, 247, 241)
    add(1, 9800, 8, 4, 4, 3, 2, 1, big4, UNCHECKED)          # one contraction step of the inverse transform (t = 4)
    add(1, 9800, 8, 8, 8, 3, 8, 1, big4, UNCHECKED)          # two (t = 10)
    add(1, 11600, 8, 8, 8, 3, 8, 1, big4, UNCHECKED)         # the same above 0.45 of the product: binary64 quotient
    add(1, 3600, 8, 8, 8, 5, 8, 2, big4, UNCHECKED)          # three (t = 12)
    for mode in (0, 1):
        add(1, 1800, 48, 64, 64, 7, 2, 3, big4, UNCHECKED, mode)     # streaming, t = 8
    for mode in (0, 1, 2):
        add(4, 1800, 48, 64, 64, 7, 4, 3, big4, UNCHECKED, mode)     # streaming, t = 10
    for mode in (0, 1):
        add(8, 64, 128, 56, 56, 3, 8, 1, PRIMES8[:3], UNCHECKED, mode)              # binary64 quotient, streaming
    out.sort(key=lambda cc: (cc[0], cc[1]))
    return out


@functools.lru_cache(maxsize=None)
def select_cases():
    """[(case, kernels, conversion)]: the cheapest layers of the grid that reach something new."""
    seen, kept = set(), []
    for _, case in _candidates():
        N, C, K, H, W, r, m, pad, moduli, flags, mode = case
        try:
            plan = rn.rnswino_plan(N, C, K, H, W, r, m, pad, moduli, flags=flags | HOST)
        except rn.RnsWinoError:
            continue
        d = rn.rnswino_plan_describe(plan, mode)
        keys = set(d["kernels"])
        if d["kernels"][2].startswith("k3_inverse_crt_stream"):
            keys.add(("stream", d["conversion"], mode))     # every conversion and output mode of the streaming kernel
        else:
            keys.add(("block", d["conversion"]))
        if keys - seen:
            seen |= keys
            kept.append((case, tuple(d["kernels"]), d["conversion"]))
    return kept


def case_id(entry) -> str:
    (N, C, K, H, W, r, m, pad, moduli, flags, mode), kernels, conversion = entry
    return f"N{N}-C{C}-K{K}-{H}x{W}-r{r}-m{m}-n{len(moduli)}{'w' if moduli[0] > 255 else ''}-f{flags}-o{mode}"
