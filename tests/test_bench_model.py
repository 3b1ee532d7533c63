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


def test_recorded_traffic_belongs_to_the_kernels_workload_2_launches():
    """profiles/hbm_traffic.json holds counter-derived HBM bytes per kernel instantiation; bench.py reports them as
    roofline.traffic only for an instantiation of that name.  A change of the dispatch must not leave stale figures behind:
    the recorded workload-2 kernels are exactly the ones the plan launches now, and their algorithmic bytes are bench.py's."""
    import json
    import os
    import paper_2007_12216_amd as rn
    table = json.load(open(os.path.join(os.path.dirname(os.path.abspath(bench.__file__)), "profiles", "hbm_traffic.json")))
    recorded = {e["kernel"]: e for e in table["kernels"] if e["workload"] == "config2"}
    cfg = si.layer_config(2)
    plan = rn.rnswino_plan(cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], cfg["r"], cfg["m"], cfg["pad"], cfg["moduli"],
                           flags=rn.FLAG_HOST_ONLY)
    launched = rn.rnswino_plan_describe(plan, 0)["kernels"]
    assert sorted(recorded) == sorted(launched)
    want = bench.stage_bytes(cfg, _plan_like(cfg))
    for stage, kernel in zip(bench.STAGES, launched):
        e = recorded[kernel]
        assert e["algorithmic_bytes"] == want[stage]
        assert e["hbm_bytes"] == e["hbm_read_bytes"] + e["hbm_write_bytes"] and 0.9 * want[stage] < e["hbm_bytes"] < 2.0 * want[stage]
        assert bench.recorded_traffic(kernel)["hbm_bytes"] == e["hbm_bytes"] and e["commit"]
    assert bench.recorded_traffic("k2_residue_gemm<9, 9, 9, false>") is None
