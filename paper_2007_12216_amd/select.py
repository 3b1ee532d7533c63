"""Per-layer choice of the output tile m of F(m x m, r x r).

The paper picks the tile size of each layer from the operation counts of its Table 2 combined with measured GEMM
throughput (section 6).  Here the candidates are simply timed on the device through the C ABI: on this hardware
the transforms and the traffic of the transform-domain tensors decide, not the multiplication count, so the count
alone would pick the wrong tile.  Plumbing only: every timed step is an `rnswino_conv2d` call.
"""
from __future__ import annotations

import torch

from . import binding as B
from .layer import ConvLayer


def multiplication_reduction(m: int, r: int, n_moduli: int) -> float:
    """Direct-convolution multiplications per RNS-Winograd multiplication, m^2 r^2 / (t^2 n) with t = m + r - 1
    (closed form behind the paper's Table 2; tile-exact maps, transforms not counted)."""
    t = m + r - 1
    return (m * m * r * r) / float(t * t * n_moduli)


def candidate_tiles(r: int, moduli) -> list[int]:
    """Output tiles the library accepts for this filter size and moduli set (t = m + r - 1 <= 16, interpolation
    points invertible modulo every modulus: section 5)."""
    out = []
    for m in range(2, 17 - r + 1):
        try:
            B.rnswino_plan(1, 1, 1, max(m, r), max(m, r), r, m, r // 2, moduli,
                           flags=B.FLAG_HOST_ONLY | B.FLAG_ALLOW_UNCHECKED_RANGE)
        except B.RnsWinoError:
            continue
        out.append(m)
    return out


def fused_glue_supported(m: int, Ho: int, Wo: int, pool: bool) -> bool:
    """Whether rnswino_conv2d_requant takes this layer (pooling inside the kernel needs tiles of 4 or 8, Wo % 4 == 0 and
    an even Ho; without pooling every tile does)."""
    return (not pool) or (m in (4, 8) and Ho % 2 == 0 and Wo % 4 == 0)


MARGIN = 0.03            # a candidate replaces the specified setting only if it is faster by more than this fraction
WIDE_PAIR = (65521, 65519)


def output_bound_from_weights(w) -> int:
    """An upper bound on |y| of a layer with these int8 weights [K][C][r][r] and any int8 input: |x| <= 128, so
    |y[k]| <= 128 * sum_{c,i,j} |w[k][c][i][j]|; the maximum over k.  For rnswino_desc_t::output_bound: with it the range test
    of a plan is a statement about the layer's actual weights instead of the worst case 2^14 r^2 C (all |w| = 128)."""
    import numpy as np
    w = np.asarray(w)
    return int(128 * np.abs(w.astype(np.int64)).reshape(w.shape[0], -1).sum(axis=1).max())


def moduli_for_bound(bound: int, candidates=((251, 241, 239), (251, 241, 239, 233))):
    """The first (smallest) candidate moduli set whose dynamic range (prod - 1) / 2 holds `bound` (sections 3 and 5)."""
    for cand in candidates:
        prod = 1
        for p in cand:
            prod *= p
        if bound <= (prod - 1) // 2:
            return tuple(cand)
    raise ValueError("no candidate moduli set holds this bound")


def _time_layer(N, C, K, H, W, r, m, pad, moduli, flags, glue, dev, x, w, iters, warmup, rotate_bytes=300 << 20):
    """Microseconds per call of one layer as a chain runs it, the transformed filter taken from a rotation of copies larger
    than the on-chip caches (in a network every layer's filter comes from HBM)."""
    layer = ConvLayer(N, C, K, H, W, r, m, pad, moduli, flags, device=dev)
    layer.set_weights(w)
    p = layer.plan
    copies = [layer.U] + [layer.U.clone() for _ in range(max(1, min(15, rotate_bytes // max(1, layer.U.numel()))))]
    st = torch.cuda.current_stream(dev).cuda_stream
    if glue is None:
        step = lambda k: B.rnswino_conv2d(p, x, copies[k % len(copies)], layer.y, layer.workspace, st)
    else:
        shift, pool = glue
        act = torch.empty((N, K, p.Ho // 2, p.Wo // 2) if pool else (N, K, p.Ho, p.Wo), dtype=torch.int8, device=dev)
        if fused_glue_supported(m, p.Ho, p.Wo, bool(pool)):
            step = lambda k: B.rnswino_conv2d_requant(p, x, copies[k % len(copies)], act, shift, pool, layer.workspace, st)
        else:
            def step(k):
                B.rnswino_conv2d(p, x, copies[k % len(copies)], layer.y, layer.workspace, st)
                B.rnswino_requant_pool(layer.y, act, N * K, p.Ho, p.Wo, shift, pool, st)
    for k in range(warmup):
        step(k)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize(dev)
    start.record()
    for k in range(iters):
        step(warmup + k)
    stop.record()
    torch.cuda.synchronize(dev)
    return start.elapsed_time(stop) * 1e3 / iters


def number_system_candidates(C: int, r: int, moduli, flags: int = 0):
    """The layer's own moduli set first, then the alternatives whose dynamic range holds its worst case 2^14 r^2 C
    (sections 3 and 8; a range the caller trusts for his own set says nothing about another one): the two 16-bit moduli,
    and three 8-bit moduli where four were specified but three suffice."""
    worst = (1 << 14) * r * r * C
    out = [tuple(moduli)]
    for cand in (WIDE_PAIR, (251, 241, 239)):
        prod = 1
        for p in cand:
            prod *= p
        if cand not in out and worst <= (prod - 1) // 2 and (len(cand) < len(moduli) or cand == WIDE_PAIR):
            out.append(cand)
    return out


def table2_reduction(m: int, r: int, moduli) -> float:
    """The paper's predictor for this choice (section 7, Table 2): multiplications of the direct convolution per
    multiplication of the RNS-Winograd GEMM, a 16-bit multiplication counted as one."""
    return multiplication_reduction(m, r, len(moduli))


def select_number_system(N, C, K, H, W, r, m, pad, moduli, iters: int = 10, warmup: int = 3, device="cuda:0", glue=None,
                         flags: int = 0):
    """Times the layer with every candidate moduli set (number_system_candidates) and returns (chosen, {set: microseconds}).
    The specified set stays unless a candidate beats it by more than MARGIN (run-to-run noise must not pick).  Whatever is
    chosen computes the same exact result."""
    if not torch.cuda.is_available():
        raise RuntimeError("rnswino needs a GPU: there is no CPU execution path")
    dev = torch.device(device)
    gen = torch.Generator(device="cpu").manual_seed(12216)
    x = torch.randint(-128, 128, (N, C, H, W), dtype=torch.int8, generator=gen).to(dev)
    w = torch.randint(-128, 128, (K, C, r, r), dtype=torch.int8, generator=gen)
    times = {}
    for cand in number_system_candidates(C, r, moduli, flags):
        try:
            times[cand] = _time_layer(N, C, K, H, W, r, m, pad, cand, flags, glue, dev, x, w, iters, warmup)
        except B.RnsWinoError:
            continue
    base = tuple(moduli)
    best = min(times, key=times.get)
    if best != base and base in times and times[best] > (1.0 - MARGIN) * times[base]:
        best = base
    return best, times


def select_output_tile(N, C, K, H, W, r, pad, moduli, candidates=None, iters: int = 20, warmup: int = 3,
                       device="cuda:0", glue=None, flags: int = 0, prefer=None):
    """Times the layer for every candidate m on synthetic int8 data of the layer's shape.

    Without `glue` a timed step is one rnswino_conv2d call (int32 output).  With glue = (shift, pool) it is the layer as
    a chain runs it: rnswino_conv2d_requant where the library supports it, else rnswino_conv2d + rnswino_requant_pool.
    The transformed filter rotates over copies larger than the caches, as in a network.  `prefer`: the specified tile; it is
    kept unless another one is faster by more than MARGIN.
    Returns (best_m, {m: microseconds per call}).  Candidates the plan refuses (range, size limits) are left out.
    """
    if not torch.cuda.is_available():
        raise RuntimeError("rnswino needs a GPU: there is no CPU execution path")
    dev = torch.device(device)
    if candidates is None:
        candidates = candidate_tiles(r, moduli)   # (the range is checked again, with the layer's C, by the plan below)
    gen = torch.Generator(device="cpu").manual_seed(12216)
    x = torch.randint(-128, 128, (N, C, H, W), dtype=torch.int8, generator=gen).to(dev)
    w = torch.randint(-128, 128, (K, C, r, r), dtype=torch.int8, generator=gen)
    times = {}
    for m in candidates:
        try:
            times[m] = _time_layer(N, C, K, H, W, r, m, pad, moduli, flags, glue, dev, x, w, iters, warmup)
        except B.RnsWinoError:
            continue
    if not times:
        raise ValueError("no output tile is accepted for this layer")
    best = min(times, key=times.get)
    if prefer is not None and prefer in times and best != prefer and times[best] > (1.0 - MARGIN) * times[prefer]:
        best = prefer           # within the margin of the specified tile: keep it
    return best, times
