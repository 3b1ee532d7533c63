"""Device-buffer plumbing around the C-ABI calls (PyTorch supplies memory and streams only)."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


class ConvLayer:
    """One stride-1 int8 convolution layer bound to device buffers.

    Holds a plan, the transformed filter U, the workspace and the int32 output.  `forward` enqueues
    rnswino_conv2d on the current torch stream; nothing is computed in Python.
    """

    def __init__(self, N, C, K, H, W, r, m, pad, moduli, flags: int = 0, device="cuda:0", output_bound: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("rnswino needs a GPU: there is no CPU execution path")
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            self.plan = B.rnswino_plan(N, C, K, H, W, r, m, pad, moduli, flags, output_bound=output_bound)
        p = self.plan
        self.U = torch.empty(B.rnswino_filter_bytes(p), dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(B.rnswino_workspace_bytes(p), dtype=torch.uint8, device=self.device)
        self.y = torch.empty((N, K, p.Ho, p.Wo), dtype=torch.int32, device=self.device)

    def _stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def set_weights(self, w) -> None:
        """w: int8 [K][C][r][r] (numpy or torch); runs the offline filter transform."""
        if isinstance(w, np.ndarray):
            w = torch.from_numpy(np.ascontiguousarray(w))
        self.w = w.to(self.device).contiguous()
        assert self.w.dtype == torch.int8 and tuple(self.w.shape) == (self.plan.K, self.plan.C, self.plan.r, self.plan.r)
        B.rnswino_filter_transform(self.plan, self.w, self.U, self._stream())

    def forward(self, x: torch.Tensor, y: torch.Tensor | None = None) -> torch.Tensor:
        """x: int8 [N][C][H][W] on the device, contiguous.  Returns the int32 output tensor (owned by the layer
        unless `y` is given)."""
        p = self.plan
        assert x.dtype == torch.int8 and x.is_contiguous() and tuple(x.shape) == (p.N, p.C, p.H, p.W)
        out = self.y if y is None else y
        B.rnswino_conv2d(p, x, self.U, out, self.workspace, self._stream())
        return out

    def stage(self, which: int) -> np.ndarray:
        """Canonical residues of U / V / O as int32 numpy (synchronises)."""
        src = self.U if which == B.STAGE_U else self.workspace
        return B.rnswino_debug_stage(self.plan, which, src)
