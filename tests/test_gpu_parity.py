"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element (bit-exact)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
import paper_2007_12216_amd as rn
from oracle import direct_conv2d
from oracle import rnswino as rw

import variant_cases as vc

pytestmark = pytest.mark.gpu


def run_layer(N, C, K, H, W, r, m, pad, moduli, x, w, flags=0):
    from paper_2007_12216_amd.layer import ConvLayer
    layer = ConvLayer(N, C, K, H, W, r, m, pad, moduli, flags)
    layer.set_weights(w)
    y = layer.forward(torch.from_numpy(x).to("cuda:0"))
    torch.cuda.synchronize()
    return layer, y.cpu().numpy()


def reorder_stage(arr, t):
    """oracle [n, xi, nu, a, b] -> [n, xi*t+nu, a, b]"""
    n = arr.shape[0]
    return arr.reshape(n, t * t, arr.shape[3], arr.shape[4])


STAGE_CASES = [
    # N, C, K, H, W, r, m, pad, moduli
    (1, 16, 16, 16, 16, 3, 8, 1, (251, 241, 239)),           # workload 1
    (2, 5, 7, 13, 17, 3, 8, 1, (251, 241, 239)),             # ragged tiles, odd channel counts, batch
    (1, 70, 40, 20, 20, 3, 8, 1, (251, 241, 239, 233)),      # C spans two 64-blocks, K spans 32-row blocks raggedly
    (1, 6, 5, 24, 24, 5, 12, 2, (251, 241, 239, 233)),       # 16x16 transform tile, 5x5 filter
    (1, 7, 3, 28, 14, 3, 14, 1, (65521, 65519)),             # 16-bit moduli
    (1, 4, 4, 12, 12, 3, 10, 1, (253, 251, 247)),            # the paper's running example (composite moduli)
    (1, 4, 4, 10, 10, 3, 8, 0, (251, 241, 239)),             # no padding
    (4, 3, 5, 61, 64, 3, 8, 1, (251, 241, 239)),             # 3 channels: 16 tiles share a 64-channel block (ragged last group)
    (2, 7, 6, 40, 44, 3, 8, 1, (251, 241, 239)),             # 7 channels: 8 tiles per block
    (1, 12, 9, 60, 52, 3, 6, 1, (251, 241, 239)),            # 12 channels: 4 tiles per block
    (1, 20, 18, 40, 24, 3, 4, 1, (65521, 65519)),            # 20 channels: 2 tiles per block, 16-bit moduli
]


@pytest.mark.parametrize("case", STAGE_CASES)
def test_every_stage_matches_the_reference(case):
    N, C, K, H, W, r, m, pad, moduli = case
    print("case", case, flush=True)
    x = si.int8_tensor(101, (N, C, H, W))
    w = si.int8_tensor(102, (K, C, r, r))
    layer, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w)
    ref_y, st = rw.conv2d(x, w, m, pad, moduli, return_stages=True)
    t = m + r - 1
    assert np.array_equal(layer.stage(rn.STAGE_U), reorder_stage(st["U"], t)), "U"
    assert np.array_equal(layer.stage(rn.STAGE_V), reorder_stage(st["V"], t)), "V"
    assert np.array_equal(layer.stage(rn.STAGE_O), reorder_stage(st["O"], t)), "O"
    assert np.array_equal(y, direct_conv2d(x, w, pad)), "y"
    assert np.array_equal(y.astype(np.int64), ref_y)


SHAPE_CASES = [
    (1, 3, 64, 32, 32, 3, 8, 1, (251, 241, 239)),            # first VGG layer shape (C=3) on a small plane
    (3, 64, 64, 24, 40, 3, 8, 1, (251, 241, 239, 233)),      # batch 3, non-square
    (1, 130, 34, 9, 9, 3, 8, 1, (251, 241, 239, 233)),       # a single ragged tile row/column
    (1, 1100, 16, 8, 8, 3, 8, 1, (251, 241, 239, 233)),      # C-sum longer than one accumulation span
    (1, 48, 64, 35, 35, 5, 12, 2, (251, 241, 239, 233)),     # Inception-v3 style 5x5 x 48 x 64
    (1, 32, 48, 28, 28, 3, 14, 1, (65521, 65519)),
    (2, 20, 20, 11, 11, 3, 6, 1, (251, 241, 239)),           # F(6x6,3x3), odd t*t? t = 8
    (1, 8, 8, 9, 9, 3, 7, 1, (251, 241, 239)),               # t = 9: 81 transform points, ragged group of four
    # LDS-tiled GEMM (128 and more rows, three and more tile blocks): contractions longer than its pipeline, ragged blocks
    (1, 1100, 130, 40, 40, 3, 6, 1, (251, 241, 239, 233)),   # 18 steps with a reduction in between, 49 tiles, ragged rows
    (1, 256, 200, 64, 64, 3, 6, 1, (251, 241, 239, 233)),    # 128 x 128 blocks: 121 tiles, 200 rows
    (2, 70, 136, 44, 44, 3, 7, 1, (251, 241, 239, 233)),     # 81 points: last point group holds one; 98 tiles
    (1, 192, 128, 96, 96, 3, 8, 1, (251, 241, 239, 233)),    # 144 tiles = two 128-tile blocks, the second mostly padding
]


@pytest.mark.parametrize("case", SHAPE_CASES)
def test_output_is_bit_exact(case):
    N, C, K, H, W, r, m, pad, moduli = case
    print("case", case, flush=True)
    x = si.int8_tensor(201, (N, C, H, W))
    w = si.int8_tensor(202, (K, C, r, r))
    _, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w)
    assert np.array_equal(y, direct_conv2d(x, w, pad))


@pytest.mark.parametrize("xv,wv", [(-128, -128), (-128, 127), (127, 127)])
def test_extreme_values(xv, wv):
    print("extreme", xv, wv, flush=True)
    N, C, K, H, W, r, m, pad, moduli = 1, 96, 32, 16, 16, 3, 8, 1, (251, 241, 239, 233)
    x = np.full((N, C, H, W), xv, dtype=np.int8)
    w = np.full((K, C, r, r), wv, dtype=np.int8)
    _, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w)
    ref = direct_conv2d(x, w, pad)
    assert np.array_equal(y, ref)
    assert abs(int(ref[0, 0, 5, 5])) == abs(xv * wv) * 9 * C


@pytest.mark.parametrize("C,K,moduli,xv,wv,hw", [(2100, 16, (251, 241, 239, 233), -128, -128, 8),
                                                 (2100, 16, (251, 241, 239, 233), -128, 127, 8),
                                                 (2100, 16, (65521, 65519), -128, -128, 8),
                                                 (70, 1030, (251, 241, 239, 233), 127, -128, 8),
                                                 (2100, 128, (251, 241, 239, 233), -128, -128, 36),
                                                 (2100, 128, (251, 241, 239, 233), -128, 127, 36)])
def test_long_sums_with_extreme_values(C, K, moduli, xv, wv, hw):
    """Accumulator headroom of the GEMM (reduced every 512 channels for 8-bit moduli, three byte-plane accumulators for
    16-bit ones) with every product at its largest magnitude, and a K that leaves a ragged last row block."""
    print("long sums", C, K, moduli, xv, wv, flush=True)
    N, H, W, r, m, pad = 1, hw, hw, 3, 6, 1                     # hw = 36: 36 tiles, the LDS-tiled GEMM
    x = np.full((N, C, H, W), xv, dtype=np.int8)
    w = np.full((K, C, r, r), wv, dtype=np.int8)
    _, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w)
    ref = direct_conv2d(x, w, pad)
    assert np.array_equal(y, ref)
    assert int(ref[0, 0, 4, 4]) == xv * wv * 9 * C


@pytest.mark.parametrize("C,moduli,sign", [(49, (251, 241, 239), 1), (49, (251, 241, 239), -1),
                                           (16, (251, 241, 239), 1), (512, (65521, 65519), -1),
                                           (42, (251, 241, 239), 1), (42, (251, 241, 239), -1),
                                           (43, (251, 241, 239), 1), (43, (251, 241, 239), -1),
                                           (11422, (251, 241, 239, 233), 1), (11422, (251, 241, 239, 233), -1)])
def test_results_at_the_edge_of_the_dynamic_range(C, moduli, sign):
    """All-extreme tensors drive |y| to 2^14 * 9 * C: with C = 49 and RNS(251,241,239) that is 7 225 344 of the
    7 228 674 the set can hold (section 3), so the CRT quotient is decided within 2.3e-4 of a half; C = 16 is the
    comfortable case (both precisions of the quotient estimate are exercised).  C = 42 is the largest channel count
    for which this moduli set still takes the conversion with unreduced accumulators (|y|/P = 0.428 plus twice its
    binary32 error bound stays below 0.49), C = 43 the first that takes the quotient in binary64.  C = 11422 is the
    largest channel count four 8-bit moduli can hold (|y| = 1 684 242 432 of 1 684 281 158): there two quotients are
    1.5e-10 apart, the tightest case of the binary64 form."""
    print("range edge", C, moduli, sign, flush=True)
    N, K, H, W, r, m, pad = 1, 16, 16, 16, 3, 8, 1
    x = np.full((N, C, H, W), -128, dtype=np.int8)
    w = np.full((K, C, r, r), -128 if sign > 0 else 127, dtype=np.int8)
    _, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w)
    ref = direct_conv2d(x, w, pad)
    assert np.array_equal(y, ref)
    assert abs(int(ref[0, 0, 5, 5])) == 128 * (128 if sign > 0 else 127) * 9 * C


def test_unchecked_range_returns_the_symmetric_residue():
    print("unchecked range", flush=True)
    N, C, K, H, W, r, m, pad, moduli = 1, 50, 16, 8, 8, 3, 8, 1, (251, 241, 239)
    x = np.full((N, C, H, W), -128, dtype=np.int8)
    w = np.full((K, C, r, r), -128, dtype=np.int8)
    _, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w, flags=rn.FLAG_ALLOW_UNCHECKED_RANGE)
    ref = rw.sym(direct_conv2d(x, w, pad).astype(np.int64), 251 * 241 * 239)
    assert np.array_equal(y.astype(np.int64), ref)
    assert y[0, 0, 3, 3] == -7084549


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_workloads_full_size(idx):
    cfg = si.layer_config(idx)
    print("workload", idx, cfg, flush=True)
    x, w = si.layer_tensors(cfg)
    _, y = run_layer(cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], cfg["r"], cfg["m"], cfg["pad"], cfg["moduli"], x, w)
    assert np.array_equal(y, direct_conv2d(x, w, cfg["pad"]))


def test_determinism_and_workspace_reuse():
    print("determinism", flush=True)
    cfg = si.layer_config(1)
    x, w = si.layer_tensors(cfg)
    layer, y1 = run_layer(cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], cfg["r"], cfg["m"], cfg["pad"], cfg["moduli"], x, w)
    xd = torch.from_numpy(x).to("cuda:0")
    for _ in range(3):
        y2 = layer.forward(xd)
    torch.cuda.synchronize()
    assert np.array_equal(y1, y2.cpu().numpy())


def test_requant_pool_matches_the_oracle_glue():
    from oracle import requant_shift_clamp, maxpool2x2
    print("requant", flush=True)
    y = (si.int8_tensor(301, (2, 5, 12, 16)).astype(np.int32)) * 3001 - 777
    yd = torch.from_numpy(y).to("cuda:0")
    for shift, pool in ((9, False), (11, True), (0, True)):
        shape = (2, 5, 6, 8) if pool else (2, 5, 12, 16)
        a = torch.empty(shape, dtype=torch.int8, device="cuda:0")
        rn.rnswino_requant_pool(yd, a, 10, 12, 16, shift, pool, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        ref = requant_shift_clamp(y, shift)
        if pool:
            ref = maxpool2x2(ref)
        assert np.array_equal(a.cpu().numpy(), ref)


def oracle_stack(layers, x, weights):
    """The 13-layer chain on the CPU: direct convolution, shift/clamp, optional 2x2 max-pool; all activations."""
    from oracle import requant_shift_clamp, maxpool2x2
    acts, a, y = [], x, None
    for l, w in zip(layers, weights):
        y = direct_conv2d(a, w, l["pad"])
        a = requant_shift_clamp(y, l["shift"])
        if l["pool"]:
            a = maxpool2x2(a)
        acts.append(a)
    return acts, y


@pytest.mark.parametrize("batch,hw,fuse", [(2, 32, True), (1, 48, True), (2, 32, False)])
def test_vgg16_stack_reduced_plane(batch, hw, fuse):
    from paper_2007_12216_amd.stack import ConvStack
    print("stack", batch, hw, flush=True)
    layers = si.vgg16_stack(batch=batch, hw=hw)
    weights = [si.int8_tensor(l["seed_w"], (l["K"], l["C"], l["r"], l["r"])) for l in layers]
    x = si.int8_tensor(si.VGG16_SEED_X, (batch, 3, hw, hw))
    stack = ConvStack(layers)
    stack.set_weights(weights)
    a, y = stack.forward(torch.from_numpy(x).to("cuda:0"), keep_last_y=True, fuse=fuse)
    torch.cuda.synchronize()
    ref_acts, ref_y = oracle_stack(layers, x, weights)
    for li, (got, ref) in enumerate(zip(stack.act, ref_acts)):
        assert np.array_equal(got.cpu().numpy(), ref), layers[li]["name"]
    assert np.array_equal(y.cpu().numpy(), ref_y)
    if fuse:   # and with the last layer fused as well
        a2 = stack.forward(torch.from_numpy(x).to("cuda:0"))
        torch.cuda.synchronize()
        assert np.array_equal(a2.cpu().numpy(), ref_acts[-1])
    # the re-quantisation keeps the activations alive: neither all zero nor all saturated
    last = ref_acts[-1].astype(np.int32)
    assert (last != 0).mean() > 0.5 and (np.abs(last) >= 127).mean() < 0.5


def test_vgg16_stack_with_measured_tiles():
    """Every layer's output tile picked by timing the candidates on the device: whatever tiles win, every layer's
    activations are those of the CPU chain (the result does not depend on the tile)."""
    from paper_2007_12216_amd.stack import ConvStack
    print("stack measured tiles", flush=True)
    batch, hw = 2, 64
    layers = si.vgg16_stack(batch=batch, hw=hw)
    weights = [si.int8_tensor(l["seed_w"], (l["K"], l["C"], l["r"], l["r"])) for l in layers]
    x = si.int8_tensor(si.VGG16_SEED_X, (batch, 3, hw, hw))
    stack = ConvStack(layers, measured_tiles=True)
    print("tiles", [l["m"] for l in stack.cfg], flush=True)
    assert all(2 <= l["m"] <= 14 for l in stack.cfg)
    stack.set_weights(weights)
    stack.forward(torch.from_numpy(x).to("cuda:0"))
    torch.cuda.synchronize()
    ref_acts, _ = oracle_stack(layers, x, weights)
    for li, (got, ref) in enumerate(zip(stack.act, ref_acts)):
        assert np.array_equal(got.cpu().numpy(), ref), layers[li]["name"]


def test_vgg16_stack_with_mixed_number_systems():
    """Layers of one chain in different number systems: every second layer over the two 16-bit moduli (with the fused
    re-quantisation and pooling of that path), the others over their 8-bit sets; every layer's activations are the CPU chain's."""
    from paper_2007_12216_amd.stack import ConvStack
    print("stack mixed number systems", flush=True)
    batch, hw = 2, 32
    layers = si.vgg16_stack(batch=batch, hw=hw)
    for li, l in enumerate(layers):
        if li % 2 == 1:
            l["moduli"] = (65521, 65519)
    weights = [si.int8_tensor(l["seed_w"], (l["K"], l["C"], l["r"], l["r"])) for l in layers]
    x = si.int8_tensor(si.VGG16_SEED_X, (batch, 3, hw, hw))
    stack = ConvStack(layers)
    stack.set_weights(weights)
    stack.forward(torch.from_numpy(x).to("cuda:0"))
    torch.cuda.synchronize()
    ref_acts, _ = oracle_stack(layers, x, weights)
    for li, (got, ref) in enumerate(zip(stack.act, ref_acts)):
        assert np.array_equal(got.cpu().numpy(), ref), layers[li]["name"]


def test_number_system_selection_times_the_candidates_and_the_stack_stays_exact():
    """Per-layer choice between the 8-bit moduli set of the range bound and the two 16-bit moduli (end of the paper's
    section 7), by timing both; the specified set stays unless the other is faster by more than the margin."""
    from paper_2007_12216_amd import select
    from paper_2007_12216_amd.stack import ConvStack
    print("number system selection", flush=True)
    four = (251, 241, 239, 233)
    assert select.number_system_candidates(256, 3, four) == [four, (65521, 65519)]
    assert select.number_system_candidates(3, 3, four) == [four, (65521, 65519), (251, 241, 239)]
    assert select.number_system_candidates(20000, 3, four, flags=rn.FLAG_ALLOW_UNCHECKED_RANGE) == [four]   # beyond both ranges
    best, times = select.select_number_system(1, 64, 64, 28, 28, 3, 8, 1, four, iters=5)
    assert set(times) == {four, (65521, 65519)} and best in times
    assert best == four or times[best] <= (1.0 - select.MARGIN) * times[four]
    batch, hw = 2, 32
    layers = si.vgg16_stack(batch=batch, hw=hw)
    weights = [si.int8_tensor(l["seed_w"], (l["K"], l["C"], l["r"], l["r"])) for l in layers]
    x = si.int8_tensor(si.VGG16_SEED_X, (batch, 3, hw, hw))
    stack = ConvStack(layers, number_systems=True)
    print("moduli", [l["moduli"] for l in stack.cfg], flush=True)
    stack.set_weights(weights)
    stack.forward(torch.from_numpy(x).to("cuda:0"))
    torch.cuda.synchronize()
    ref_acts, _ = oracle_stack(layers, x, weights)
    for li, (got, ref) in enumerate(zip(stack.act, ref_acts)):
        assert np.array_equal(got.cpu().numpy(), ref), layers[li]["name"]


def test_weight_derived_output_bound_is_tight_and_sufficient():
    """Three moduli on a 64-channel layer, admitted by the bound 128 * max_k sum |w[k]| of its actual weights (the worst case
    2^14 r^2 C would need four): exact on seeded inputs, and exact on the input that drives one filter's output to that bound
    (x = -128 where the filter is positive, 127 where it is negative), which sits beyond 0.3 of the moduli product."""
    from paper_2007_12216_amd import select
    print("weight bound", flush=True)
    N, C, K, H, W, r, m, pad, moduli = 1, 64, 32, 16, 16, 3, 8, 1, (251, 241, 239)
    w = si.int8_tensor(9201, (K, C, r, r))
    bound = select.output_bound_from_weights(w)
    with pytest.raises(rn.RnsWinoError):
        rn.rnswino_plan(N, C, K, H, W, r, m, pad, moduli, flags=rn.FLAG_HOST_ONLY)
    from paper_2007_12216_amd.layer import ConvLayer
    layer = ConvLayer(N, C, K, H, W, r, m, pad, moduli, output_bound=bound)
    layer.set_weights(w)
    k0 = int(np.abs(w.astype(np.int64)).reshape(K, -1).sum(axis=1).argmax())
    x_rand = si.int8_tensor(9202, (N, C, H, W))
    x_adv = np.zeros((N, C, H, W), dtype=np.int8)
    # the 3 x 3 patch around output (8, 8) of filter k0, chosen against the filter's signs: y[k0, 8, 8] = -128 * sum |w| + (#negative)
    x_adv[0, :, 7:10, 7:10] = np.where(w[k0] > 0, -128, 127).astype(np.int8)
    for x in (x_rand, x_adv):
        y = layer.forward(torch.from_numpy(x).to("cuda:0")).cpu().numpy()
        torch.cuda.synchronize()
        assert np.array_equal(y, direct_conv2d(x, w, pad))
    ref = direct_conv2d(x_adv, w, pad)
    assert bound - 128 * 576 <= abs(int(ref[0, k0, 8, 8])) <= bound and abs(int(ref[0, k0, 8, 8])) > 0.3 * 251 * 241 * 239


def test_vgg16_stack_with_weight_derived_bounds():
    """The stack with every layer's moduli count taken from the bound of its own weights (three moduli where 128 * max_k sum |w|
    fits their range: the two 64-channel layers besides the first one): every layer's activations are the CPU chain's."""
    from paper_2007_12216_amd import select
    from paper_2007_12216_amd.stack import ConvStack
    print("stack weight bounds", flush=True)
    batch, hw = 2, 32
    layers = si.vgg16_stack(batch=batch, hw=hw)
    weights = [si.int8_tensor(l["seed_w"], (l["K"], l["C"], l["r"], l["r"])) for l in layers]
    for l, w in zip(layers, weights):
        l["output_bound"] = select.output_bound_from_weights(w)
        l["moduli"] = select.moduli_for_bound(l["output_bound"])
    assert [len(l["moduli"]) for l in layers] == [3, 3, 3] + [4] * 10
    x = si.int8_tensor(si.VGG16_SEED_X, (batch, 3, hw, hw))
    stack = ConvStack(layers)
    stack.set_weights(weights)
    stack.forward(torch.from_numpy(x).to("cuda:0"))
    torch.cuda.synchronize()
    ref_acts, _ = oracle_stack(layers, x, weights)
    for li, (got, ref) in enumerate(zip(stack.act, ref_acts)):
        assert np.array_equal(got.cpu().numpy(), ref), layers[li]["name"]


def test_vgg16_stack_in_the_papers_setting():
    """Three 8-bit moduli on every layer with the range trusted (section 8 of the paper) instead of four from the worst-case
    bound: the outputs of the seeded data stay inside the dynamic range, so the chain is still the oracle's."""
    from paper_2007_12216_amd.stack import ConvStack
    print("stack trusted range", flush=True)
    batch, hw = 2, 32
    layers = si.vgg16_stack(batch=batch, hw=hw)
    for l in layers:
        l["moduli"], l["flags"] = (251, 241, 239), rn.FLAG_ALLOW_UNCHECKED_RANGE
    weights = [si.int8_tensor(l["seed_w"], (l["K"], l["C"], l["r"], l["r"])) for l in layers]
    x = si.int8_tensor(si.VGG16_SEED_X, (batch, 3, hw, hw))
    stack = ConvStack(layers)
    stack.set_weights(weights)
    stack.forward(torch.from_numpy(x).to("cuda:0"))
    torch.cuda.synchronize()
    ref_acts, _ = oracle_stack(layers, x, weights)
    for li, (got, ref) in enumerate(zip(stack.act, ref_acts)):
        assert np.array_equal(got.cpu().numpy(), ref), layers[li]["name"]


def test_vgg16_stack_full_size():
    """Workload 5: batch 8, 224x224, all 13 layers; every layer's activations bit-exact against the CPU chain."""
    from paper_2007_12216_amd.stack import ConvStack
    print("stack full size", flush=True)
    layers = si.vgg16_stack(batch=8, hw=224)
    weights = [si.int8_tensor(l["seed_w"], (l["K"], l["C"], l["r"], l["r"])) for l in layers]
    x = si.int8_tensor(si.VGG16_SEED_X, (8, 3, 224, 224))
    stack = ConvStack(layers)
    stack.set_weights(weights)
    a, y = stack.forward(torch.from_numpy(x).to("cuda:0"), keep_last_y=True)
    torch.cuda.synchronize()
    print("gpu done; oracle chain ...", flush=True)
    ref_acts, ref_y = oracle_stack(layers, x, weights)
    for li, (got, ref) in enumerate(zip(stack.act, ref_acts)):
        assert np.array_equal(got.cpu().numpy(), ref), layers[li]["name"]
    assert np.array_equal(y.cpu().numpy(), ref_y)


@pytest.mark.parametrize("m,pool,W", [(8, False, 28), (8, True, 28), (4, False, 28), (4, True, 28),
                                      (8, False, 14), (4, False, 30), (8, False, 22),    # rows not a multiple of 4 bytes
                                      (7, False, 28), (6, False, 27), (10, False, 21), (8, False, 21), (14, False, 28),
                                      (2, False, 9)])                                    # byte stores: any tile, odd rows
def test_fused_requant_matches_the_oracle_glue(m, pool, W):
    from oracle import requant_shift_clamp, maxpool2x2
    print("fused requant", m, pool, W, flush=True)
    N, C, K, H, r, pad, moduli, shift = 2, 20, 24, 20, 3, 1, (251, 241, 239), 10
    x = si.int8_tensor(401, (N, C, H, W))
    w = si.int8_tensor(402, (K, C, r, r))
    from paper_2007_12216_amd.layer import ConvLayer
    layer = ConvLayer(N, C, K, H, W, r, m, pad, moduli)
    layer.set_weights(w)
    shape = (N, K, H // 2, W // 2) if pool else (N, K, H, W)
    a = torch.empty(shape, dtype=torch.int8, device="cuda:0")
    rn.rnswino_conv2d_requant(layer.plan, torch.from_numpy(x).to("cuda:0"), layer.U, a, shift, pool, layer.workspace,
                              torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ref = requant_shift_clamp(direct_conv2d(x, w, pad), shift)
    if pool:
        ref = maxpool2x2(ref)
    assert np.array_equal(a.cpu().numpy(), ref)


def test_fused_pooling_refuses_unsupported_tiles():
    """Pooling inside the kernel needs output tiles of 4 or 8; without pooling every tile size is taken."""
    from paper_2007_12216_amd.layer import ConvLayer
    layer = ConvLayer(1, 4, 4, 12, 12, 3, 10, 1, (253, 251, 247))
    x = torch.zeros((1, 4, 12, 12), dtype=torch.int8, device="cuda:0")
    a = torch.empty((1, 4, 6, 6), dtype=torch.int8, device="cuda:0")
    with pytest.raises(rn.RnsWinoError) as e:
        rn.rnswino_conv2d_requant(layer.plan, x, layer.U, a, 9, True, layer.workspace, 0)
    assert e.value.code == -2


NETWORK_CASES = [
    # synthetic stand-ins with the shapes of other networks' stride-1 layers (the paper's Tables 4 and 5 name ResNet50's
    # 3x3 layers and Inception-v3's 5x5 layer); seeded uniform int8 values, batch 2
    # name, N, C, K, H, W, r, m, pad, moduli
    ("first layer 3x3 3->64 224x224", 1, 3, 64, 224, 224, 3, 8, 1, (251, 241, 239)),
    ("first layer 3x3 3->32 96x96, F(4,3)", 2, 3, 32, 96, 96, 3, 4, 1, (251, 241, 239)),
    ("5x5 16->32 48x48, F(12,5)", 2, 16, 32, 48, 48, 5, 12, 2, (251, 241, 239, 233)),
    ("resnet 3x3 64->64 56x56", 2, 64, 64, 56, 56, 3, 8, 1, (251, 241, 239, 233)),
    ("resnet 3x3 128->128 28x28", 2, 128, 128, 28, 28, 3, 8, 1, (251, 241, 239, 233)),
    ("resnet 3x3 256->256 14x14", 2, 256, 256, 14, 14, 3, 8, 1, (251, 241, 239, 233)),
    ("resnet 3x3 512->512 7x7", 2, 512, 512, 7, 7, 3, 6, 1, (251, 241, 239, 233)),
    ("resnet 3x3 256->256 14x14, 16-bit moduli", 1, 256, 256, 14, 14, 3, 14, 1, (65521, 65519)),
    ("inception 5x5 48->64 35x35, F(12,5)", 2, 48, 64, 35, 35, 5, 12, 2, (251, 241, 239, 233)),
    ("inception 5x5 48->64 35x35, F(4,5)", 2, 48, 64, 35, 35, 5, 4, 2, (251, 241, 239, 233)),
]


@pytest.mark.parametrize("case", NETWORK_CASES, ids=[c[0] for c in NETWORK_CASES])
def test_other_networks_layer_shapes(case):
    name, N, C, K, H, W, r, m, pad, moduli = case
    print("network shape", name, flush=True)
    x = si.int8_tensor(7100 + N * C + H, (N, C, H, W))
    w = si.int8_tensor(7200 + K + r, (K, C, r, r))
    _, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w)
    assert np.array_equal(y, direct_conv2d(x, w, pad))


def test_tile_selection_times_every_candidate_and_keeps_the_fastest():
    """Per-layer choice of the output tile (section 6), measured instead of counted; the chosen tile computes the
    same exact result as any other."""
    from paper_2007_12216_amd import select
    print("tile selection", flush=True)
    N, C, K, H, W, r, pad, moduli = 1, 64, 64, 28, 28, 3, 1, (251, 241, 239, 233)
    best, times = select.select_output_tile(N, C, K, H, W, r, pad, moduli, candidates=(4, 6, 8, 14), iters=5)
    assert set(times) == {4, 6, 8, 14} and best in times and times[best] == min(times.values())
    assert all(0.0 < t < 1e5 for t in times.values())
    x = si.int8_tensor(7301, (N, C, H, W))
    w = si.int8_tensor(7302, (K, C, r, r))
    _, y = run_layer(N, C, K, H, W, r, best, pad, moduli, x, w)
    assert np.array_equal(y, direct_conv2d(x, w, pad))


def _random_cases(count, seed):
    """Seeded random layer shapes covering odd sizes, every filter size up to 7, 1..8 moduli of both widths."""
    rng = np.random.default_rng(seed)
    primes8 = [251, 241, 239, 233, 229, 227, 223, 211, 199, 197, 193, 191]
    primes16 = [65521, 65519, 65497, 65479, 4001, 40009]
    cases = []
    while len(cases) < count:
        r = int(rng.choice([1, 2, 3, 3, 3, 5, 5, 7]))
        m = int(rng.integers(1, 17 - r + 1))
        if m + r - 1 < 2:
            continue
        wide = bool(rng.integers(0, 4) == 0)
        n = int(rng.integers(2, 4)) if wide else int(rng.integers(3, 9))
        moduli = tuple((primes16 if wide else primes8)[:n])
        N = int(rng.integers(1, 3))
        C = int(rng.choice([1, 3, 17, 64, 65, 130]))
        K = int(rng.choice([1, 5, 16, 33, 70]))
        H, W = int(rng.integers(max(1, r - 2), 30)), int(rng.integers(max(1, r - 2), 30))
        pad = int(rng.integers(0, r))
        if H + 2 * pad - r + 1 <= 0 or W + 2 * pad - r + 1 <= 0:
            continue
        P = 1
        for p in moduli:
            P *= p
        if (1 << 14) * r * r * C > (P - 1) // 2:
            continue
        cases.append((N, C, K, H, W, r, m, pad, moduli))
    return cases


@pytest.mark.parametrize("case", _random_cases(40, 2024))
def test_random_shapes_are_bit_exact(case):
    N, C, K, H, W, r, m, pad, moduli = case
    print("random case", case, flush=True)
    x = si.int8_tensor(501, (N, C, H, W))
    w = si.int8_tensor(502, (K, C, r, r))
    _, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w)
    assert np.array_equal(y, direct_conv2d(x, w, pad))


def _random_cases_many_rows(count, seed):
    """Seeded random layers with 128 and more filters and more than 32 tiles: the shapes the LDS-tiled GEMM takes (ragged row
    and tile blocks, one to five 64-channel steps, point groups with one to four points)."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        r = int(rng.choice([1, 3, 3, 5]))
        m = int(rng.integers(3, 9))
        N = int(rng.integers(1, 4))
        C = int(rng.choice([7, 40, 64, 100, 130, 260, 300]))
        K = int(rng.choice([128, 136, 200, 260]))
        H, W = int(rng.integers(28, 72)), int(rng.integers(28, 72))
        pad = int(rng.integers(0, r))
        moduli = (251, 241, 239, 233) if (1 << 14) * r * r * C > 7228674 else (251, 241, 239)
        if (1 << 14) * r * r * C > (251 * 241 * 239 * 233 - 1) // 2:
            continue
        cases.append((N, C, K, H, W, r, m, pad, moduli))
    return cases


@pytest.mark.parametrize("case", _random_cases_many_rows(14, 77))
def test_random_shapes_with_many_rows_are_bit_exact(case):
    N, C, K, H, W, r, m, pad, moduli = case
    print("random case (many rows)", case, flush=True)
    x = si.int8_tensor(503, (N, C, H, W))
    w = si.int8_tensor(504, (K, C, r, r))
    layer, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w)
    print(rn.rnswino_plan_describe(layer.plan)["kernels"], flush=True)
    assert np.array_equal(y, direct_conv2d(x, w, pad))


def test_two_streams_with_their_own_workspaces():
    """One plan and one transformed filter, two calls in flight on two streams, each with its own workspace and output:
    the entry point keeps no state between calls, so both results are the oracle's."""
    print("two streams", flush=True)
    from paper_2007_12216_amd.layer import ConvLayer
    N, C, K, H, W, r, m, pad, moduli = 2, 70, 40, 28, 28, 3, 8, 1, (251, 241, 239, 233)
    w = si.int8_tensor(77, (K, C, r, r))
    xs = [si.int8_tensor(78 + j, (N, C, H, W)) for j in range(2)]
    layer = ConvLayer(N, C, K, H, W, r, m, pad, moduli)
    layer.set_weights(w)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]          # default priority
    xd = [torch.from_numpy(x).to("cuda:0") for x in xs]
    ws = [torch.empty_like(layer.workspace) for _ in range(2)]
    ys = [torch.empty_like(layer.y) for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(3):
        for j in range(2):
            rn.rnswino_conv2d(layer.plan, xd[j], layer.U, ys[j], ws[j], streams[j].cuda_stream)
    torch.cuda.synchronize()
    for j in range(2):
        assert np.array_equal(ys[j].cpu().numpy(), direct_conv2d(xs[j], w, pad))


@pytest.mark.parametrize("K,hw", [(32, 24), (128, 48)])
def test_captured_graph_replays_match_the_eager_result(K, hw):
    """rnswino_conv2d neither allocates nor synchronises, so its three launches can be captured into a HIP graph; every
    replay (with eager work and synchronisations of the program's own in between) must give the eager result.  The second
    shape runs the LDS-tiled GEMM (its loads are issued from inline assembly: nothing a capture could trip over)."""
    print("graph capture", K, hw, flush=True)
    from paper_2007_12216_amd.layer import ConvLayer
    N, C, H, W, r, m, pad, moduli = 1, 64, hw, hw, 3, 8, 1, (251, 241, 239, 233)
    w = si.int8_tensor(91, (K, C, r, r))
    layer = ConvLayer(N, C, K, H, W, r, m, pad, moduli)
    layer.set_weights(w)
    x_static = torch.zeros((N, C, H, W), dtype=torch.int8, device="cuda:0")
    y_static = torch.empty_like(layer.y)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                  # warm-up on the capture stream, as graph capture asks
        rn.rnswino_conv2d(layer.plan, x_static, layer.U, y_static, layer.workspace, side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rn.rnswino_conv2d(layer.plan, x_static, layer.U, y_static, layer.workspace,
                          torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        x = si.int8_tensor(100 + rep, (N, C, H, W))
        x_static.copy_(torch.from_numpy(x).to("cuda:0"))
        eager = layer.forward(x_static).clone()                    # eager call between the replays (shares the workspace: ordered by the stream)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref = direct_conv2d(x, w, pad)
        assert np.array_equal(eager.cpu().numpy(), ref)
        assert np.array_equal(y_static.cpu().numpy(), ref), f"replay {rep}"


def test_the_papers_vgg16_setting_with_a_trusted_range():
    """Section 8 runs VGG16 with F(14x14,3x3) over RNS(251,241,239) on layers of up to 512 channels, trusting a measured
    output range instead of the worst case (which three 8-bit moduli cover only up to 49 channels).  Same setting here
    on a 256-channel 28x28 layer: the plan needs the unchecked-range flag, the outputs of the seeded data stay inside
    the dynamic range, and the result is the exact convolution."""
    print("paper setting", flush=True)
    N, C, K, H, W, r, m, pad, moduli = 1, 256, 64, 28, 28, 3, 14, 1, (251, 241, 239)
    with pytest.raises(rn.RnsWinoError):
        rn.rnswino_plan(N, C, K, H, W, r, m, pad, moduli, flags=rn.FLAG_HOST_ONLY)
    x = si.int8_tensor(8801, (N, C, H, W))
    w = si.int8_tensor(8802, (K, C, r, r))
    ref = direct_conv2d(x, w, pad)
    assert np.abs(ref.astype(np.int64)).max() <= (251 * 241 * 239 - 1) // 2
    _, y = run_layer(N, C, K, H, W, r, m, pad, moduli, x, w, flags=rn.FLAG_ALLOW_UNCHECKED_RANGE)
    assert np.array_equal(y, ref)


@pytest.mark.parametrize("entry", vc.select_cases(), ids=[vc.case_id(e) for e in vc.select_cases()])
def test_every_kernel_variant(entry):
    """Layers chosen (tests/variant_cases.py) so that every instantiation of the three kernels the library can launch, every
    form of the conversion out of the RNS and every output mode of the streaming inverse transform runs at least once:
    each against the direct-convolution oracle (reduced to the symmetric range of the moduli set where the range was left
    unchecked and is exceeded), for the int8 output modes followed by the oracle's shift/clamp and max-pool."""
    from oracle import requant_shift_clamp, maxpool2x2
    from paper_2007_12216_amd.layer import ConvLayer
    (N, C, K, H, W, r, m, pad, moduli, flags, mode), kernels, conversion = entry
    print("variant case", vc.case_id(entry), kernels, conversion, flush=True)
    x = si.int8_tensor(601, (N, C, H, W))
    w = si.int8_tensor(602, (K, C, r, r))
    layer = ConvLayer(N, C, K, H, W, r, m, pad, moduli, flags)
    d = rn.rnswino_plan_describe(layer.plan, mode)
    assert tuple(d["kernels"]) == kernels and d["conversion"] == conversion
    layer.set_weights(w)
    P = 1
    for p in moduli:
        P *= int(p)
    ref = direct_conv2d(x, w, pad)
    if (flags & rn.FLAG_ALLOW_UNCHECKED_RANGE) and P < (1 << 33):      # a larger product holds every int32 anyway
        ref = rw.sym(ref.astype(np.int64), P).astype(np.int32)
    xd = torch.from_numpy(x).to("cuda:0")
    if mode == 0:
        y = layer.forward(xd)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), ref)
        return
    shift = max(0, int(round(np.log2(74.0 * np.sqrt(float(r * r * C))))) - (0 if P > 1 << 24 else 8))
    Ho, Wo = layer.plan.Ho, layer.plan.Wo
    a = torch.empty((N, K, Ho // 2, Wo // 2) if mode == 2 else (N, K, Ho, Wo), dtype=torch.int8, device="cuda:0")
    rn.rnswino_conv2d_requant(layer.plan, xd, layer.U, a, shift, mode == 2, layer.workspace, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = requant_shift_clamp(ref, shift)
    if mode == 2:
        want = maxpool2x2(want)
    assert np.array_equal(a.cpu().numpy(), want)


def test_the_event_taking_entry_point_computes_the_same_output():
    """rnswino_conv2d_events is rnswino_conv2d with timestamps: same output, and six usable events."""
    import ctypes
    from paper_2007_12216_amd.layer import ConvLayer
    print("events entry", flush=True)
    cfg = si.layer_config(3)
    x, w = si.layer_tensors(cfg)
    layer = ConvLayer(cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], cfg["r"], cfg["m"], cfg["pad"], cfg["moduli"])
    layer.set_weights(w)
    xd = torch.from_numpy(x).to("cuda:0")
    y_plain = layer.forward(xd).clone()
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    events = []
    for _ in range(6):
        e = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
        events.append(e.value)
    y_ev = torch.zeros_like(layer.y)
    rn.rnswino_conv2d_events(layer.plan, xd, layer.U, y_ev, layer.workspace, torch.cuda.current_stream().cuda_stream, events)
    torch.cuda.synchronize()
    assert torch.equal(y_ev, y_plain)
    assert np.array_equal(y_ev.cpu().numpy(), direct_conv2d(x, w, cfg["pad"]))
    for j in range(3):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), events[2 * j], events[2 * j + 1]) == 0
        assert 0.0 < ms.value < 100.0
    for e in events:
        hip.hipEventDestroy(e)


def test_requant_pool_at_the_ends_of_the_shift_range():
    """Shift 0 (clamp only, negative values included) and shift 31 (only the sign survives) of the stand-alone glue kernel."""
    from oracle import requant_shift_clamp
    print("requant shift range", flush=True)
    y = np.array([[-2 ** 31, -2 ** 31 + 1, -129, -128, -1, 0, 1, 127, 128, 2 ** 31 - 1, 12345, -54321]], dtype=np.int32).reshape(1, 1, 2, 6)
    yd = torch.from_numpy(y).to("cuda:0")
    for shift in (0, 1, 30, 31):
        a = torch.empty(y.shape, dtype=torch.int8, device="cuda:0")
        rn.rnswino_requant_pool(yd, a, 1, 2, 6, shift, False, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert np.array_equal(a.cpu().numpy(), requant_shift_clamp(y, shift)), shift


def test_empty_launch_for_floor_measurements():
    """rnswino_debug_empty_launch: any grid, with and without events; bad grids are refused without a launch."""
    print("empty launch", flush=True)
    st = torch.cuda.current_stream().cuda_stream
    for grid in ((1, 1), (200, 4), (20000, 1)):
        rn.rnswino_debug_empty_launch(grid[0], grid[1], st)
    torch.cuda.synchronize()
    for grid in ((0, 1), (1, 0), (1, 70000)):
        with pytest.raises(rn.RnsWinoError) as e:
            rn.rnswino_debug_empty_launch(grid[0], grid[1], st)
        assert e.value.code == -1
