#!/usr/bin/env python3
"""Benchmark of the RNS-Winograd int8 convolution hot path on one MI355X.

Headline (the JSON line's `value`): one step = one call of rnswino_conv2d (input transform, residue GEMM, inverse
transform + conversion out of the RNS) on the VGG16-style middle layer, workload 2: N=1, C=K=256, 56x56, 3x3, pad 1,
F(8x8,3x3), four 8-bit moduli.  The filter transform is offline (section 6 of the paper) and is not timed.  Inputs are
synthetic (seeded uniform int8) and already resident in HBM.  The metric is effective INT8 TOPS: the direct-convolution
operation count 2*N*K*C*Ho*Wo*r^2 divided by the time per step.

Timing: every step uses its own weight/input/workspace set out of a rotation larger than the on-chip caches (L2 +
Infinity Cache), so every step streams its operands from HBM ("cold"), as a network running layer after layer would.
After the warm-up, ROUNDS rounds of exactly --steps steps are timed, each bracketed by a device synchronisation; the
reported time per step is the median round (`config.timing` says so and lists every round).  With --warm the same loop
on one buffer set is timed as well.

The default run also times the other four workloads (single layers 1, 3, 4 the same way; workload 5, the 13-layer VGG16
stack at batch 8, as whole passes) and the library's own direct int8 convolution on every shape, and reports them under
`config.workloads`: time per step, effective TOPS, the dominant kernel with its HBM fraction, and whether the output of
the timed calls equals the CPU oracle's.  `--workload W` runs one workload alone as the headline instead.

One JSON line is printed: the contract fields plus
  roofline     -- the slowest of the three kernels of the headline workload: algorithmic bytes per launch / its average
                  duration, measured with HIP events that take each kernel's own start and stop timestamps on the launch
                  stream (a pass of its own over the same rotation, same step count), against 8 TB/s HBM; `traffic` is
                  the HBM bytes per launch recorded from rocprofv3 counters in profiles/hbm_traffic.json for exactly the
                  kernel instantiation that ran (null when the file has no entry for it);
  cpu_baseline -- the direct-convolution oracle timed on this machine's host cores (context only).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
INT8_MFMA_PEAK_TOPS = 5000.0
ROTATION_BYTES = 640 << 20      # operands cycled through in the cold loop (> 256 MB Infinity Cache + 32 MB L2)
ROUNDS = 5
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
STAGES = ("input_transform", "residue_gemm", "inverse_transform_crt")


class HipEvents:
    """hipEvent_t handles through the HIP runtime (PyTorch's events do not expose their handle portably)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.made = []

    def create(self) -> int:
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        self.made.append(ev.value)
        return ev.value

    def elapsed_ms(self, a: int, b: int) -> float:
        out = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(out), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return out.value

    def destroy_all(self):
        for e in self.made:
            self.hip.hipEventDestroy(e)
        self.made = []


def stage_bytes(cfg, plan):
    """Algorithmic HBM bytes per launch of each kernel: the tensors it must read and write once.

    Per unit (one residue and transform point): input transform writes T*C residues, the GEMM reads K*C + T*C
    and writes K*T, the inverse transform reads K*T; times n*t^2 units; plus x once and y (int32) once."""
    n, t2 = len(cfg["moduli"]), plan.t * plan.t
    N, C, K, H, W = cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"]
    rb = 1 if max(cfg["moduli"]) < 256 else 2
    T = plan.T
    xb = N * C * H * W
    vb = n * t2 * T * C * rb
    ub = n * t2 * K * C * rb
    ob = n * t2 * K * T * rb
    yb = N * K * plan.Ho * plan.Wo * 4
    return {"input_transform": xb + vb, "residue_gemm": ub + vb + ob, "inverse_transform_crt": ob + yb}


def stage_mfma_ops(cfg, plan):
    """int8 operations the matrix cores execute per launch of each kernel (2 per multiply-add, padding included):
    the GEMM over channels padded to 64, rows and tiles padded to 16; the two transforms as Kronecker products with the
    contraction padded to whole 64-element steps and the outputs to whole 16-row blocks.  16-bit moduli: four byte-plane
    products per multiply-add in the GEMM and in the inverse transform, two table planes in the input transform."""
    n, t, m = len(cfg["moduli"]), plan.t, cfg["m"]
    wide = max(cfg["moduli"]) >= 256
    up = lambda v, q: -(-v // q) * q
    Cp, Kp, Tp = up(cfg["C"], 64), up(cfg["K"], 16), up(plan.T, 16)
    slots1 = up(t * up(t, 4), 64)
    return {"input_transform": 2.0 * n * up(t * t, 16) * slots1 * plan.T * Cp * (2 if wide else 1),
            "residue_gemm": 2.0 * n * t * t * Kp * Cp * Tp * (4 if wide else 1),
            "inverse_transform_crt": 2.0 * n * up(m * m, 16) * up(t * t, 64) * cfg["K"] * plan.T * (4 if wide else 1)}


def recorded_traffic(kernel_name: str):
    """HBM bytes per launch of one kernel instantiation as recorded from rocprofv3 counters (profiles/hbm_traffic.json:
    FETCH_SIZE and WRITE_SIZE scaled by a copy of known size), or None when that instantiation was never measured."""
    try:
        with open(TRAFFIC_FILE) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None
    for entry in table.get("kernels", []):
        if entry.get("kernel") == kernel_name:
            return entry
    return None


def timed_rounds(step_fn, steps, warmup, sync):
    """Median seconds per step over ROUNDS rounds of exactly `steps` steps (each round between two synchronisations)."""
    k = 0
    for _ in range(warmup):
        step_fn(k)
        k += 1
    per_round = []
    for _ in range(ROUNDS):
        sync()
        t0 = time.perf_counter()
        for _ in range(steps):
            step_fn(k)
            k += 1
        sync()
        per_round.append((time.perf_counter() - t0) / steps)
    return statistics.median(per_round), per_round


def bench_layer(idx, steps, warmup, dev, with_cpu, warm=False, events=True):
    """One single-layer workload: cold time per call, per-kernel durations, roofline of the dominant kernel, the library's
    own direct convolution on the same shape, and the oracle comparison."""
    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2007_12216_amd as rn
    from paper_2007_12216_amd.layer import ConvLayer

    cfg = si.layer_config(idx)
    x_np, w_np = si.layer_tensors(cfg)
    layer = ConvLayer(cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], cfg["r"], cfg["m"], cfg["pad"], cfg["moduli"])
    plan = layer.plan
    layer.set_weights(w_np)
    x0 = torch.from_numpy(x_np).to(dev)
    ops = 2.0 * cfg["N"] * cfg["K"] * cfg["C"] * plan.Ho * plan.Wo * cfg["r"] ** 2
    sync = torch.cuda.synchronize

    # buffer rotation for the cold loop: every set holds its own U, x, workspace and y
    set_bytes = layer.U.numel() + layer.workspace.numel() + x0.numel() + layer.y.numel() * 4
    n_sets = max(2, min(64, -(-ROTATION_BYTES // set_bytes)))
    sets = [dict(U=layer.U.clone(), x=x0.clone(), ws=torch.empty_like(layer.workspace), y=torch.empty_like(layer.y))
            for _ in range(n_sets)]
    stream = torch.cuda.current_stream(dev).cuda_stream

    def step_cold(k):
        b = sets[k % n_sets]
        rn.rnswino_conv2d(plan, b["x"], b["U"], b["y"], b["ws"], stream)

    def step_warm(k):
        b = sets[0]
        rn.rnswino_conv2d(plan, b["x"], b["U"], b["y"], b["ws"], stream)

    sec_cold, rounds = timed_rounds(step_cold, steps, warmup, sync)
    last_set = (warmup + ROUNDS * steps - 1) % n_sets
    sec_warm = timed_rounds(step_warm, steps, warmup, sync)[0] if warm else None

    # per-kernel durations: HIP events around each kernel, same cold rotation, same step count
    names = STAGES
    stage_ms = None
    if events:
        evs = HipEvents()
        ev = [[evs.create() for _ in range(6)] for _ in range(steps)]
        for k in range(warmup):
            step_cold(k)
        sync()
        for k in range(steps):
            b = sets[(warmup + k) % n_sets]
            rn.rnswino_conv2d_events(plan, b["x"], b["U"], b["y"], b["ws"], stream, ev[k])
        sync()
        stage_ms = {nm: 0.0 for nm in names}
        for k in range(steps):
            for j, nm in enumerate(names):
                stage_ms[nm] += evs.elapsed_ms(ev[k][2 * j], ev[k][2 * j + 1])
        for nm in names:
            stage_ms[nm] /= steps
        last_set = (warmup + steps - 1) % n_sets
        # the floor of each stage: a chain of kernels that do nothing on that stage's grid, replayed from a HIP graph (so that
        # the host's launch rate does not enter), time per launch
        grids = {}
        for nm, g in zip(names, rn.rnswino_plan_describe(plan, 0)["grids"]):
            gx, _, gy = g.split()[0].split("=")[1].partition("x")
            grids[nm] = (int(gx), int(gy or 1))
        floor_ms = {}
        for nm in names:
            try:
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream(dev))
                with torch.cuda.stream(side):
                    rn.rnswino_debug_empty_launch(grids[nm][0], grids[nm][1], side.cuda_stream)
                torch.cuda.current_stream(dev).wait_stream(side)
                sync()
                graph, chain = torch.cuda.CUDAGraph(), 200
                with torch.cuda.graph(graph):
                    cs = torch.cuda.current_stream(dev).cuda_stream
                    for _ in range(chain):
                        rn.rnswino_debug_empty_launch(grids[nm][0], grids[nm][1], cs)
                for _ in range(2):
                    graph.replay()
                sync()
                t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                t0.record()
                graph.replay()
                t1.record()
                sync()
                floor_ms[nm] = t0.elapsed_time(t1) / chain
                del graph
            except Exception:        # graph capture unavailable: the floor is simply not reported
                floor_ms[nm] = None
        evs.destroy_all()

    described = rn.rnswino_plan_describe(plan, 0)
    kernel_of = dict(zip(names, described["kernels"]))
    bytes_per = stage_bytes(cfg, plan)
    mfma_ops = stage_mfma_ops(cfg, plan)
    roofline = None
    if stage_ms:
        dominant = max(names, key=lambda nm: stage_ms[nm])
        achieved = bytes_per[dominant] / (stage_ms[dominant] * 1e-3) / 1e9
        rec = recorded_traffic(kernel_of[dominant])
        roofline = {"bound": "hbm", "kernel": dominant, "instantiation": kernel_of[dominant], "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": rec["hbm_bytes"] if rec else None,
                    "traffic_source": ({"file": "profiles/hbm_traffic.json", "measured_at_commit": rec.get("commit"),
                                        "workload": rec.get("workload")} if rec else None),
                    "algorithmic_bytes": bytes_per[dominant],
                    "stage_us": {nm: round(stage_ms[nm] * 1e3, 2) for nm in names},
                    "stage_GBps": {nm: round(bytes_per[nm] / (stage_ms[nm] * 1e-3) / 1e9, 1) for nm in names},
                    # matrix-core utilisation per stage: int8 MFMA operations issued / duration / 5 POP/s dense int8 peak
                    "stage_mfma_frac": {nm: round(mfma_ops[nm] / (stage_ms[nm] * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS, 4)
                                        for nm in names},
                    # time per launch of a dependent chain of kernels that do nothing on the same grid (dispatch, ramp-up, completion)
                    "stage_empty_grid_us": {nm: (round(floor_ms[nm] * 1e3, 2) if floor_ms[nm] is not None else None) for nm in names},
                    "kernels": kernel_of, "conversion": described["conversion"]}

    sync()
    got = sets[last_set]["y"].cpu().numpy()

    # the library's own direct convolution (implicit GEMM on the matrix cores: the paper's comparison baseline) on this shape
    N, C, K, H, W, r, pad = (cfg[k] for k in ("N", "C", "K", "H", "W", "r", "pad"))
    wt = torch.empty(rn.rnswino_direct_filter_bytes(C, K, r), dtype=torch.uint8, device=dev)
    rn.rnswino_direct_filter_pack(torch.from_numpy(w_np).to(dev), wt, C, K, r, stream)
    dws = torch.empty(rn.rnswino_direct_workspace_bytes(N, C, H, W, pad), dtype=torch.uint8, device=dev)
    dsets = [dict(x=b["x"], y=b["y"]) for b in sets]

    def step_direct(k):
        b = dsets[k % n_sets]
        rn.rnswino_direct_conv2d(b["x"], wt, b["y"], N, C, K, H, W, r, pad, dws, stream)

    sec_direct = timed_rounds(step_direct, steps, min(warmup, 5), sync)[0]
    sync()
    got_direct = dsets[(min(warmup, 5) + ROUNDS * steps - 1) % n_sets]["y"].cpu().numpy()

    cpu, bit_exact, direct_exact = None, None, None
    if with_cpu is not None:
        from oracle import direct_conv2d, num_threads
        best, ref = float("inf"), None
        reps = 3 if (with_cpu and ops < 2e10) else 1
        for _ in range(reps):
            t0 = time.perf_counter()
            ref = direct_conv2d(x_np, w_np, cfg["pad"])
            best = min(best, time.perf_counter() - t0)
        bit_exact = bool(np.array_equal(got, ref))
        direct_exact = bool(np.array_equal(got_direct, ref))
        if with_cpu:
            cpu = {"value": round(ops / best / 1e12, 6), "unit": "TOPS", "cores": num_threads(), "kind": "oracle",
                   "sample": f"whole layer ({ops / 1e9:.3f} GOP), best of {reps} runs, {best * 1e3:.1f} ms"}
    del sets, dsets
    torch.cuda.empty_cache()
    return {"cfg": cfg, "ops": ops, "sec": sec_cold, "rounds": rounds, "sec_warm": sec_warm, "n_sets": n_sets,
            "set_bytes": set_bytes, "roofline": roofline, "bit_exact": bit_exact, "cpu": cpu,
            "direct_sec": sec_direct, "direct_bit_exact": direct_exact}


def layer_name(cfg):
    return (f"{cfg['name']}: N={cfg['N']} C={cfg['C']} K={cfg['K']} {cfg['H']}x{cfg['W']} r={cfg['r']} pad={cfg['pad']} "
            f"F({cfg['m']}x{cfg['m']},{cfg['r']}x{cfg['r']}) moduli={list(cfg['moduli'])}")


def bench_stack(steps, warmup, dev, with_cpu, trusted_range=False, measured_tiles=False, number_systems=False, per_layer=False,
                weight_bound=False, gemm_64x16=False):
    """Workload 5: one step = one pass of the 13-layer VGG16 conv stack at batch 8 (conv, shift/clamp, pool chain)."""
    import numpy as np
    import torch
    import synth_inputs as si
    import paper_2007_12216_amd as rn
    from paper_2007_12216_amd.stack import ConvStack

    steps, warmup = max(1, min(steps, 50)), min(warmup, 5)
    layers = si.vgg16_stack(batch=8, hw=224)
    if trusted_range:
        # the paper's own setting (its section 8): three 8-bit moduli on every layer, trusting that the outputs stay
        # inside their dynamic range instead of bounding them; the result is compared with the oracle below
        for l in layers:
            l["moduli"], l["flags"] = (251, 241, 239), rn.FLAG_ALLOW_UNCHECKED_RANGE
    weights = [si.int8_tensor(l["seed_w"], (l["K"], l["C"], l["r"], l["r"])) for l in layers]
    if weight_bound:
        # moduli count per layer from the bound its own weights give, 128 * max_k sum |w[k]|, instead of the worst case
        # 2^14 r^2 C: still a guarantee for every int8 input, but a statement about these weights
        from paper_2007_12216_amd import select
        for l, w in zip(layers, weights):
            l["output_bound"] = select.output_bound_from_weights(w)
            l["moduli"] = select.moduli_for_bound(l["output_bound"])
    if gemm_64x16:
        for l in layers:
            l["flags"] = l.get("flags", 0) | rn.FLAG_GEMM_BLOCK_64X16
    x_np = si.int8_tensor(si.VGG16_SEED_X, (8, 3, 224, 224))
    stack = ConvStack(layers, measured_tiles=measured_tiles, number_systems=number_systems)
    stack.set_weights(weights)
    x = torch.from_numpy(x_np).to(dev)
    sync = torch.cuda.synchronize
    sec, rounds = timed_rounds(lambda k: stack.forward(x), steps, warmup, sync)
    ops = stack.direct_ops()
    # algorithmic HBM bytes of one pass: per layer x + 2 V + U + 2 O + the int8 activations it stores (after pooling)
    pass_bytes = 0
    for l, p, a in zip(stack.cfg, stack.plans, stack.act):
        n, t2 = len(l["moduli"]), p.t * p.t
        rb = 1 if max(l["moduli"]) < 256 else 2
        pass_bytes += (l["N"] * l["C"] * l["H"] * l["W"] + rb * (2 * n * t2 * p.T * l["C"] + n * t2 * l["K"] * l["C"]
                       + 2 * n * t2 * l["K"] * p.T) + a.numel())
    roofline = {"bound": "hbm", "kernel": "whole pass (13 layers x 3 launches)", "achieved": round(pass_bytes / sec / 1e9, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(pass_bytes / sec / 1e9 / HBM_PEAK_GBS, 4),
                "traffic": None, "algorithmic_bytes": pass_bytes}
    sync()
    got = stack.act[-1].cpu().numpy()

    # the same chain through the library's own direct convolution (+ stand-alone glue), for comparison
    st = torch.cuda.current_stream(dev).cuda_stream
    dw, dws_bytes = [], 0
    for l, w in zip(layers, weights):
        wt = torch.empty(rn.rnswino_direct_filter_bytes(l["C"], l["K"], l["r"]), dtype=torch.uint8, device=dev)
        rn.rnswino_direct_filter_pack(torch.from_numpy(w).to(dev), wt, l["C"], l["K"], l["r"], st)
        dw.append(wt)
        dws_bytes = max(dws_bytes, rn.rnswino_direct_workspace_bytes(l["N"], l["C"], l["H"], l["W"], l["pad"]))
    dws = torch.empty(dws_bytes, dtype=torch.uint8, device=dev)
    dact = [torch.empty_like(a) for a in stack.act]

    def direct_pass(k):
        a = x
        for l, p, wt, out in zip(layers, stack.plans, dw, dact):
            rn.rnswino_direct_conv2d(a, wt, stack.y, l["N"], l["C"], l["K"], l["H"], l["W"], l["r"], l["pad"], dws, st)
            rn.rnswino_requant_pool(stack.y, out, l["N"] * l["K"], p.Ho, p.Wo, l["shift"], l["pool"], st)
            a = out

    sec_direct = timed_rounds(direct_pass, steps, min(warmup, 2), sync)[0]
    sync()
    got_direct = dact[-1].cpu().numpy()

    table = None
    if per_layer:
        # every layer on its own clock (events between the layers of the running chain), both paths
        iters = 10
        tot, totd = [0.0] * len(layers), [0.0] * len(layers)
        for _ in range(iters):
            marks = [torch.cuda.Event(enable_timing=True) for _ in range(len(layers) + 1)]
            a = x
            marks[0].record()
            for li in range(len(layers)):
                a = stack.forward_layer(li, a)
                marks[li + 1].record()
            sync()
            for li in range(len(layers)):
                tot[li] += marks[li].elapsed_time(marks[li + 1]) * 1e3 / iters
            marks = [torch.cuda.Event(enable_timing=True) for _ in range(len(layers) + 1)]
            a = x
            marks[0].record()
            for li, (l, p, wt, out) in enumerate(zip(layers, stack.plans, dw, dact)):
                rn.rnswino_direct_conv2d(a, wt, stack.y, l["N"], l["C"], l["K"], l["H"], l["W"], l["r"], l["pad"], dws, st)
                rn.rnswino_requant_pool(stack.y, out, l["N"] * l["K"], p.Ho, p.Wo, l["shift"], l["pool"], st)
                a = out
                marks[li + 1].record()
            sync()
            for li in range(len(layers)):
                totd[li] += marks[li].elapsed_time(marks[li + 1]) * 1e3 / iters
        table = [{"layer": l["name"], "C": l["C"], "K": l["K"], "map": l["H"], "m": l["m"], "moduli": list(l["moduli"]),
                  "kernels": rn.rnswino_plan_describe(p, 2 if l["pool"] else 1)["kernels"],
                  "rns_winograd_us": round(tot[li], 1), "own_direct_conv_us": round(totd[li], 1)}
                 for li, (l, p) in enumerate(zip(stack.cfg, stack.plans))]
    cpu, bit_exact, direct_exact = None, None, None
    if with_cpu is not None:
        from oracle import direct_conv2d, requant_shift_clamp, maxpool2x2, num_threads
        t0 = time.perf_counter()
        a = x_np
        for l, w in zip(layers, weights):
            a = requant_shift_clamp(direct_conv2d(a, w, l["pad"]), l["shift"])
            if l["pool"]:
                a = maxpool2x2(a)
        dt = time.perf_counter() - t0
        bit_exact = bool(np.array_equal(got, a))
        direct_exact = bool(np.array_equal(got_direct, a))
        if with_cpu:
            cpu = {"value": round(ops / dt / 1e12, 6), "unit": "TOPS", "cores": num_threads(), "kind": "oracle",
                   "sample": f"whole 13-layer chain once ({ops / 1e9:.1f} GOP), {dt:.1f} s"}
    name = ("config5: VGG16 conv stack, N=8, 224x224, 13 layers, " +
            ("output tile measured per layer" if measured_tiles else "F(8x8,3x3)") +
            (", number system measured per layer" if number_systems else "") +
            (", RNS(251,241,239) with a trusted range on every layer" if trusted_range else "") +
            (", moduli count per layer from the bound of its own weights" if weight_bound else "") +
            (", residue GEMM forced to 64 x 16 blocks (what a fused GEMM + inverse transform could hold on chip)" if gemm_64x16 else "") +
            ", shift/clamp + 2x2 max-pool fused into the inverse transform")
    return {"name": name, "ops": ops, "sec": sec, "rounds": rounds, "steps": steps, "warmup": warmup, "roofline": roofline,
            "bit_exact": bit_exact, "cpu": cpu, "tiles": [l["m"] for l in stack.cfg],
            "moduli": [list(l["moduli"]) for l in stack.cfg], "direct_sec": sec_direct, "direct_bit_exact": direct_exact,
            "per_layer": table}


def summary(res, name):
    """Compact entry of one workload for config.workloads."""
    out = {"workload": name, "ms_per_step": round(res["sec"] * 1e3, 5), "TOPS": round(res["ops"] / res["sec"] / 1e12, 3),
           "bit_exact_vs_oracle": res["bit_exact"],
           "direct_conv_ms": round(res["direct_sec"] * 1e3, 5), "direct_conv_TOPS": round(res["ops"] / res["direct_sec"] / 1e12, 3),
           "direct_conv_bit_exact_vs_oracle": res["direct_bit_exact"]}
    rf = res["roofline"]
    if rf:
        out.update({"dominant_kernel": rf.get("instantiation", rf["kernel"]), "frac": rf["frac"], "achieved_GBps": rf["achieved"]})
        if "stage_us" in rf:
            out["stage_us"] = rf["stage_us"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=0, choices=(0, 1, 2, 3, 4, 5),
                    help="0 (default): workload 2 as the headline plus the other four under config.workloads; "
                         "1-4: that single layer alone; 5: the 13-layer stack alone")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle (no cpu_baseline, no bit-exactness check)")
    ap.add_argument("--warm", action="store_true", help="also time the loop on one operand set (cache-warm)")
    ap.add_argument("--trusted-range", action="store_true",
                    help="workload 5 only: the paper's setting, three 8-bit moduli per layer with the range trusted, not bounded "
                         "(default: four moduli from the worst-case bound, as specified)")
    ap.add_argument("--measured-tiles", action="store_true",
                    help="workload 5 only: pick every layer's output tile by timing the candidates (default: F(8x8,3x3) as specified)")
    ap.add_argument("--number-systems", action="store_true",
                    help="workload 5 only: pick every layer's number system (8-bit moduli from the range bound, or two 16-bit moduli) "
                         "by timing both")
    ap.add_argument("--weight-bound", action="store_true",
                    help="workload 5 only: moduli count per layer from the output bound its own weights give (128 max_k sum |w|) "
                         "instead of the worst case 2^14 r^2 C")
    ap.add_argument("--gemm-64x16", action="store_true",
                    help="workload 5 only, measurement: residue GEMM on 64-row x 16-tile workgroup blocks, the largest block whose "
                         "output a workgroup could keep in LDS for a fused inverse transform (prices that fusion)")
    ap.add_argument("--per-layer", action="store_true", help="workload 5 only: add a per-layer, per-kernel table of durations")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K_steps, W_steps = max(1, args.steps), max(0, args.warmup)
    with_cpu = None if args.no_cpu_baseline else True

    common = {"metric": "effective INT8 TOPS per conv layer (direct-conv ops/s)", "unit": "TOPS", "n_gpus": 1,
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic"}
    timing = lambda r, steps: {"what": f"median of {ROUNDS} rounds of {steps} steps, each round between two device synchronisations",
                               "rounds_ms_per_step": [round(v * 1e3, 5) for v in r["rounds"]]}

    if args.workload == 5:
        r = bench_stack(K_steps, W_steps, dev, with_cpu, args.trusted_range, args.measured_tiles, args.number_systems, args.per_layer,
                        args.weight_bound, args.gemm_64x16)
        out = dict(common, value=round(r["ops"] / r["sec"] / 1e12, 3), steps=r["steps"], warmup=r["warmup"],
                   ms_per_step=round(r["sec"] * 1e3, 5),
                   config={"workload": r["name"], "output_tiles": r["tiles"], "moduli": r["moduli"],
                           "direct_conv_GOP": round(r["ops"] / 1e9, 2), "bit_exact_vs_oracle": r["bit_exact"],
                           "timing": timing(r, r["steps"]),
                           "own_direct_convolution": {"ms_per_pass": round(r["direct_sec"] * 1e3, 5),
                                                      "TOPS": round(r["ops"] / r["direct_sec"] / 1e12, 3),
                                                      "bit_exact_vs_oracle": r["direct_bit_exact"]},
                           "per_layer_us": r["per_layer"]},
                   roofline=r["roofline"], cpu_baseline=r["cpu"])
        print(json.dumps(out))
        return

    head_idx = args.workload or 2
    head = bench_layer(head_idx, K_steps, W_steps, dev, with_cpu, warm=args.warm)
    workloads = None
    if args.workload == 0:
        workloads = {}
        side_cpu = None if args.no_cpu_baseline else False      # compare with the oracle, do not time it
        for idx in (1, 3, 4):
            r = bench_layer(idx, K_steps, W_steps, dev, side_cpu)
            workloads[f"config{idx}"] = summary(r, layer_name(r["cfg"]))
        r5 = bench_stack(min(K_steps, 20), W_steps, dev, side_cpu)
        workloads["config5"] = summary(r5, r5["name"])
    cfg = head["cfg"]
    config = {"workload": layer_name(cfg), "direct_conv_GOP": round(head["ops"] / 1e9, 4),
              "cache": f"cold (rotation of {head['n_sets']} operand sets, {head['n_sets'] * head['set_bytes'] >> 20} MiB)",
              "timing": timing(head, K_steps),
              "warm_value_TOPS": round(head["ops"] / head["sec_warm"] / 1e12, 3) if head["sec_warm"] else None,
              "warm_ms_per_step": round(head["sec_warm"] * 1e3, 5) if head["sec_warm"] else None,
              "bit_exact_vs_oracle": head["bit_exact"],
              "own_direct_convolution": {"ms_per_step": round(head["direct_sec"] * 1e3, 5),
                                         "TOPS": round(head["ops"] / head["direct_sec"] / 1e12, 3),
                                         "bit_exact_vs_oracle": head["direct_bit_exact"],
                                         "what": "rnswino_direct_conv2d: implicit GEMM on the int8 matrix cores, layout copy included, "
                                                 "filter packing offline (the paper's comparison baseline on this chip)"}}
    if workloads is not None:
        config["workloads"] = workloads
    out = dict(common, value=round(head["ops"] / head["sec"] / 1e12, 3), steps=K_steps, warmup=W_steps,
               ms_per_step=round(head["sec"] * 1e3, 5), config=config, roofline=head["roofline"], cpu_baseline=head["cpu"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
