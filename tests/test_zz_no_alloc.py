"""rnswino_conv2d_static (the entry point that allocates nothing: its workspace is a buffer inside the library's code
object) against rnswino_conv2d with a caller-provided workspace, through the C ABI, on two calls in a row, the second on a
smaller layer, so that the buffer still holds the first call's transform-domain tensors when the second one starts."""
import numpy as np
import pytest
import torch

import synth_inputs as si
import paper_2007_12216_amd as rn
from oracle import direct_conv2d

pytestmark = pytest.mark.gpu


def _layer(N, C, K, H, W, r, m, pad, moduli, seed):
    from paper_2007_12216_amd.layer import ConvLayer
    x = si.int8_tensor(seed, (N, C, H, W))
    w = si.int8_tensor(seed + 1, (K, C, r, r))
    layer = ConvLayer(N, C, K, H, W, r, m, pad, moduli)
    layer.set_weights(w)
    return layer, x, w, torch.from_numpy(x).to("cuda:0")


def test_static_workspace_entry_point_matches_the_workspace_one():
    print("static workspace: two calls in a row, the second smaller", flush=True)
    st = torch.cuda.current_stream().cuda_stream
    big = _layer(1, 256, 256, 56, 56, 3, 8, 1, (251, 241, 239, 233), 9101)      # workload 2's shape: 10.2 MB of workspace
    small = _layer(2, 20, 24, 13, 17, 3, 8, 1, (251, 241, 239), 9103)           # ragged tiles, three moduli
    assert rn.rnswino_workspace_bytes(big[0].plan) <= rn.STATIC_WORKSPACE_BYTES
    outs = []
    for layer, x, w, xd in (big, small):
        y_static = torch.zeros_like(layer.y)
        rn.rnswino_conv2d_static(layer.plan, xd, layer.U, y_static, st)          # no synchronisation in between
        outs.append(y_static)
    torch.cuda.synchronize()
    for (layer, x, w, xd), y_static in zip((big, small), outs):
        y_ws = layer.forward(xd)
        torch.cuda.synchronize()
        assert torch.equal(y_static, y_ws)
        assert np.array_equal(y_static.cpu().numpy(), direct_conv2d(x, w, layer.plan.pad))
    # and once more in the other order, 16-bit moduli in between (their workspace layout differs)
    wide = _layer(1, 32, 48, 28, 28, 3, 14, 1, (65521, 65519), 9105)
    for layer, x, w, xd in (small, wide, big):
        y_static = torch.zeros_like(layer.y)
        rn.rnswino_conv2d_static(layer.plan, xd, layer.U, y_static, st)
        torch.cuda.synchronize()
        assert np.array_equal(y_static.cpu().numpy(), direct_conv2d(x, w, layer.plan.pad))


def test_static_workspace_entry_point_refuses_layers_beyond_its_buffer():
    from paper_2007_12216_amd.layer import ConvLayer
    print("static workspace: size limit", flush=True)
    layer = ConvLayer(8, 64, 64, 112, 112, 3, 8, 1, (251, 241, 239, 233))       # 80 MB of V and O
    assert rn.rnswino_workspace_bytes(layer.plan) > rn.STATIC_WORKSPACE_BYTES
    x = torch.zeros((8, 64, 112, 112), dtype=torch.int8, device="cuda:0")
    sentinel = torch.full_like(layer.y, 77)
    with pytest.raises(rn.RnsWinoError) as e:
        rn.rnswino_conv2d_static(layer.plan, x, layer.U, sentinel, torch.cuda.current_stream().cuda_stream)
    assert e.value.code == -8 and "workspace" in str(e.value)
    torch.cuda.synchronize()
    assert bool((sentinel == 77).all())                                          # nothing was launched
