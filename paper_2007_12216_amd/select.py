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


def select_output_tile(N, C, K, H, W, r, pad, moduli, candidates=None, iters: int = 20, warmup: int = 3,
                       device="cuda:0", glue=None, flags: int = 0):
    """Times the layer for every candidate m on synthetic int8 data of the layer's shape.

    Without `glue` a timed step is one rnswino_conv2d call (int32 output).  With glue = (shift, pool) it is the layer as
    a chain runs it: rnswino_conv2d_requant where the library supports it, else rnswino_conv2d + rnswino_requant_pool.
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
            layer = ConvLayer(N, C, K, H, W, r, m, pad, moduli, flags, device=dev)
        except B.RnsWinoError:
            continue
        layer.set_weights(w)
        step = lambda: layer.forward(x)
        if glue is not None:
            shift, pool = glue
            p = layer.plan
            act = torch.empty((N, K, p.Ho // 2, p.Wo // 2) if pool else (N, K, p.Ho, p.Wo), dtype=torch.int8, device=dev)
            st = torch.cuda.current_stream(dev).cuda_stream
            if fused_glue_supported(m, p.Ho, p.Wo, bool(pool)):
                step = lambda: B.rnswino_conv2d_requant(p, x, layer.U, act, shift, pool, layer.workspace, st)
            else:
                def step():
                    B.rnswino_conv2d(p, x, layer.U, layer.y, layer.workspace, st)
                    B.rnswino_requant_pool(layer.y, act, N * K, p.Ho, p.Wo, shift, pool, st)
        for _ in range(warmup):
            step()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize(dev)
        start.record()
        for _ in range(iters):
            step()
        stop.record()
        torch.cuda.synchronize(dev)
        times[m] = start.elapsed_time(stop) * 1e3 / iters
        del layer
    if not times:
        raise ValueError("no output tile is accepted for this layer")
    best = min(times, key=times.get)
    return best, times
