"""GPU parity of the library's own direct int8 convolution (implicit GEMM on the matrix cores: the comparison baseline of
the paper's section 8) against the CPU oracle, bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

import synth_inputs as si
import paper_2007_12216_amd as rn
from oracle import direct_conv2d

pytestmark = pytest.mark.gpu


def run_direct(x, w, pad):
    N, C, H, W = x.shape
    K, _, r, _ = w.shape
    dev = "cuda:0"
    st = torch.cuda.current_stream().cuda_stream
    wt = torch.empty(rn.rnswino_direct_filter_bytes(C, K, r), dtype=torch.uint8, device=dev)
    ws = torch.empty(rn.rnswino_direct_workspace_bytes(N, C, H, W, pad), dtype=torch.uint8, device=dev)
    y = torch.empty((N, K, H + 2 * pad - r + 1, W + 2 * pad - r + 1), dtype=torch.int32, device=dev)
    rn.rnswino_direct_filter_pack(torch.from_numpy(w).to(dev), wt, C, K, r, st)
    rn.rnswino_direct_conv2d(torch.from_numpy(x).to(dev), wt, y, N, C, K, H, W, r, pad, ws, st)
    torch.cuda.synchronize()
    return y.cpu().numpy()


CASES = [
    # N, C, K, H, W, r, pad
    (1, 16, 16, 16, 16, 3, 1),        # workload 1
    (1, 256, 256, 56, 56, 3, 1),      # workload 2
    (1, 128, 128, 28, 28, 5, 2),      # workload 3
    (1, 512, 512, 28, 28, 3, 1),      # workload 4
    (2, 3, 64, 40, 44, 3, 1),         # first-layer shape: 3 channels, 64 filters (64 x 256 blocks when large enough)
    (8, 64, 64, 56, 56, 3, 1),        # 64 filters, many pixels
    (2, 5, 7, 13, 17, 3, 1),          # ragged everything
    (1, 70, 130, 20, 21, 3, 0),       # no padding, ragged channel and filter blocks
    (3, 64, 200, 33, 35, 1, 0),       # 1 x 1 filter
    (1, 20, 24, 19, 19, 7, 3),        # 7 x 7 filter
    (2, 130, 136, 64, 64, 3, 1),      # 128 x 128 blocks with ragged rows
    (1, 8, 8, 6, 6, 5, 0),            # 2 x 2 outputs
]


@pytest.mark.parametrize("case", CASES)
def test_direct_convolution_is_bit_exact(case):
    N, C, K, H, W, r, pad = case
    print("direct case", case, flush=True)
    x = si.int8_tensor(801, (N, C, H, W))
    w = si.int8_tensor(802, (K, C, r, r))
    assert np.array_equal(run_direct(x, w, pad), direct_conv2d(x, w, pad))


@pytest.mark.parametrize("xv,wv", [(-128, -128), (-128, 127)])
def test_direct_convolution_with_extreme_values(xv, wv):
    print("direct extreme", xv, wv, flush=True)
    N, C, K, H, W, r, pad = 1, 2100, 32, 12, 12, 3, 1
    x = np.full((N, C, H, W), xv, dtype=np.int8)
    w = np.full((K, C, r, r), wv, dtype=np.int8)
    y = run_direct(x, w, pad)
    assert np.array_equal(y, direct_conv2d(x, w, pad))
    assert int(y[0, 0, 5, 5]) == xv * wv * 9 * C


def test_direct_and_rns_winograd_paths_agree_on_the_stack_layers():
    """Both paths of the library on the 13 layer shapes of the VGG16 stack (reduced plane), each equal to the oracle."""
    from paper_2007_12216_amd.layer import ConvLayer
    print("direct vs winograd", flush=True)
    for l in si.vgg16_stack(batch=2, hw=32):
        x = si.int8_tensor(811, (l["N"], l["C"], l["H"], l["W"]))
        w = si.int8_tensor(l["seed_w"], (l["K"], l["C"], 3, 3))
        layer = ConvLayer(l["N"], l["C"], l["K"], l["H"], l["W"], 3, l["m"], 1, l["moduli"])
        layer.set_weights(w)
        yw = layer.forward(torch.from_numpy(x).to("cuda:0"))
        torch.cuda.synchronize()
        yd = run_direct(x, w, 1)
        assert np.array_equal(yd, yw.cpu().numpy()), l["name"]
        assert np.array_equal(yd, direct_conv2d(x, w, 1)), l["name"]


def test_direct_entry_points_refuse_bad_arguments():
    assert rn.rnswino_direct_filter_bytes(0, 4, 3) == 0 and rn.rnswino_direct_workspace_bytes(1, 4, 0, 4, 1) == 0
    assert rn.rnswino_direct_filter_bytes(64, 64, 3) == 9 * 64 * 64
    assert rn.rnswino_direct_workspace_bytes(2, 3, 10, 12, 1) == 2 * 12 * 14 * 64
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(rn.RnsWinoError) as e:
        rn.rnswino_direct_conv2d(buf, buf, buf, 1, 4, 4, 2, 2, 5, 0, buf, 0)          # empty output
    assert e.value.code == -1
    with pytest.raises(rn.RnsWinoError) as e:
        rn.rnswino_direct_conv2d(buf, buf, buf, 1, 1 << 20, 4, 8, 8, 3, 1, buf, 0)    # sums beyond int32
    assert e.value.code == -2
