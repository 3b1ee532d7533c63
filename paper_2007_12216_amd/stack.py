"""A chain of stride-1 int8 convolution layers with shift/clamp re-quantisation and optional 2x2 max-pool
between them (the 13-layer VGG16-style workload).  Plumbing only: every step is a C-ABI call."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .select import fused_glue_supported


class ConvStack:
    def __init__(self, layers, device="cuda:0", measured_tiles: bool = False, number_systems: bool = False):
        """layers: list of dicts with N, C, K, H, W, r, m, pad, moduli, shift, pool and optionally flags (plan flags) and
        output_bound (the caller's bound on |y| for the layer's weights, see select.output_bound_from_weights)
        (see synth_inputs.vgg16_stack).

        measured_tiles: replace every layer's output tile m by the fastest one for its shape, timed on the device with the
        layer's own glue (the paper picks the tile per layer from operation counts and measured GEMM throughput, its
        section 6; here the whole layer is timed).  The result does not depend on m: it is the exact convolution.

        number_systems: likewise choose, per layer, between its 8-bit moduli set and the two 16-bit moduli (65521, 65519)
        by timing both (the paper's choice between the 8-bit 3-residue and the 16-bit 2-residue system, end of its
        section 7); the 16-bit system is taken only where it is faster by more than the margin of select.py."""
        if not torch.cuda.is_available():
            raise RuntimeError("rnswino needs a GPU: there is no CPU execution path")
        self.device = torch.device(device)
        self.cfg = [dict(l) for l in layers]
        if measured_tiles:
            from .select import select_output_tile
            chosen = {}
            for l in self.cfg:
                key = (l["N"], l["C"], l["K"], l["H"], l["W"], l["r"], l["pad"], tuple(l["moduli"]), l["shift"], bool(l["pool"]))
                if key not in chosen:
                    chosen[key], _ = select_output_tile(l["N"], l["C"], l["K"], l["H"], l["W"], l["r"], l["pad"], l["moduli"],
                                                        iters=10, device=self.device, glue=(l["shift"], l["pool"]),
                                                        flags=l.get("flags", 0), prefer=l["m"])
                l["m"] = chosen[key]
        if number_systems:
            from .select import select_number_system
            chosen = {}
            for l in self.cfg:
                key = (l["N"], l["C"], l["K"], l["H"], l["W"], l["r"], l["m"], l["pad"], tuple(l["moduli"]), l["shift"], bool(l["pool"]))
                if key not in chosen:
                    chosen[key], _ = select_number_system(l["N"], l["C"], l["K"], l["H"], l["W"], l["r"], l["m"], l["pad"],
                                                          l["moduli"], device=self.device, glue=(l["shift"], l["pool"]),
                                                          flags=l.get("flags", 0))
                l["moduli"] = chosen[key]
        self.plans, self.U, self.act = [], [], []
        ws_bytes, y_elems = 0, 0
        with torch.cuda.device(self.device):
            for l in self.cfg:
                p = B.rnswino_plan(l["N"], l["C"], l["K"], l["H"], l["W"], l["r"], l["m"], l["pad"], l["moduli"],
                                   l.get("flags", 0), output_bound=l.get("output_bound", 0))
                self.plans.append(p)
                self.U.append(torch.empty(B.rnswino_filter_bytes(p), dtype=torch.uint8, device=self.device))
                ws_bytes = max(ws_bytes, B.rnswino_workspace_bytes(p))
                y_elems = max(y_elems, l["N"] * l["K"] * p.Ho * p.Wo)
                Hq, Wq = (p.Ho // 2, p.Wo // 2) if l["pool"] else (p.Ho, p.Wo)
                self.act.append(torch.empty((l["N"], l["K"], Hq, Wq), dtype=torch.int8, device=self.device))
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=self.device)
        self.y = torch.empty(y_elems, dtype=torch.int32, device=self.device)

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def set_weights(self, weights) -> None:
        """weights: one int8 [K][C][r][r] array per layer; runs the offline filter transforms."""
        self.w = []
        for p, U, w in zip(self.plans, self.U, weights):
            wd = torch.from_numpy(np.ascontiguousarray(w)).to(self.device)
            self.w.append(wd)
            B.rnswino_filter_transform(p, wd, U, self._stream())

    def forward(self, x: torch.Tensor, keep_last_y: bool = False, fuse: bool = True):
        """x: int8 [N][C][H][W] of the first layer.  Returns the int8 activations of the last layer
        (and its raw int32 output if asked).  With fuse=True the re-quantisation (and pooling) runs inside the
        inverse-transform kernel wherever the library supports it."""
        a = x
        last = len(self.cfg) - 1
        for li in range(len(self.cfg)):
            a = self.forward_layer(li, a, fuse=fuse and not (keep_last_y and li == last))
        if keep_last_y:
            p = self.plans[-1]
            n = self.cfg[-1]["N"] * self.cfg[-1]["K"] * p.Ho * p.Wo
            return a, self.y[:n].view(self.cfg[-1]["N"], self.cfg[-1]["K"], p.Ho, p.Wo)
        return a

    def forward_layer(self, li: int, a: torch.Tensor, fuse: bool = True) -> torch.Tensor:
        """Layer li alone on input a (int8, on the device); returns its int8 activations."""
        st = self._stream()
        l, p, U, out = self.cfg[li], self.plans[li], self.U[li], self.act[li]
        if fuse and fused_glue_supported(p.m, p.Ho, p.Wo, bool(l["pool"])):
            B.rnswino_conv2d_requant(p, a, U, out, l["shift"], l["pool"], self.workspace, st)
        else:
            B.rnswino_conv2d(p, a, U, self.y, self.workspace, st)
            B.rnswino_requant_pool(self.y, out, l["N"] * l["K"], p.Ho, p.Wo, l["shift"], l["pool"], st)
        return out

    def direct_ops(self) -> float:
        return float(sum(2.0 * l["N"] * l["K"] * l["C"] * p.Ho * p.Wo * l["r"] ** 2 for l, p in zip(self.cfg, self.plans)))
