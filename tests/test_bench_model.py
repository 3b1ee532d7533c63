"""The byte and operation counts bench.py prices the kernels with, against the layer sizes worked out by hand."""
import types

import bench
import synth_inputs as si


def _plan_like(cfg):
    t = cfg["m"] + cfg["r"] - 1
    Ho = cfg["H"] + 2 * cfg["pad"] - cfg["r"] + 1
    th = -(-Ho // cfg["m"])
    return types.SimpleNamespace(t=t, T=cfg["N"] * th * th, Ho=Ho, Wo=Ho)


def test_algorithmic_bytes_of_workload_2():
    # x 256*56*56, V = O = 4*100*49*256, U = 4*100*256*256, y = 256*56*56*4 bytes
    cfg = si.layer_config(2)
    b = bench.stage_bytes(cfg, _plan_like(cfg))
    x, v, u, y = 802816, 5017600, 26214400, 3211264
    assert b == {"input_transform": x + v, "residue_gemm": u + 2 * v, "inverse_transform_crt": v + y}


def test_algorithmic_bytes_of_the_16_bit_workload():
    # two bytes per residue: V = O = 2*256*4*512*2, U = 2*256*512*512*2
    cfg = si.layer_config(4)
    b = bench.stage_bytes(cfg, _plan_like(cfg))
    assert b["residue_gemm"] == 268435456 + 2 * 2097152


def test_matrix_core_operation_counts_of_workload_2():
    # GEMM: 400 products of 256 x 256 x 64 (49 tiles padded to 64); input transform: 112 x 128 table (100 points padded to
    # 112, 10 rows of 12 slots padded to 128) per tile and channel; inverse: 64 x 128 table per (k, tile)
    cfg = si.layer_config(2)
    ops = bench.stage_mfma_ops(cfg, _plan_like(cfg))
    assert ops["residue_gemm"] == 2.0 * 400 * 256 * 256 * 64
    assert ops["input_transform"] == 2.0 * 4 * 112 * 128 * 49 * 256
    assert ops["inverse_transform_crt"] == 2.0 * 4 * 64 * 128 * 256 * 49
