"""Host-side checks of the kernel selection (no GPU): the layers of tests/variant_cases.py reach every instantiation the
library can launch, the conversion out of the RNS takes the expected form at the edges the GPU parity cases sit on, and no
admissible moduli set is left without an instantiation."""
import itertools

import pytest

import paper_2007_12216_amd as rn
import variant_cases as vc

HOST = rn.FLAG_HOST_ONLY
UNCHECKED = rn.FLAG_ALLOW_UNCHECKED_RANGE


def test_the_variant_cases_reach_every_instantiation():
    kept = vc.select_cases()
    reached = {k for _, kernels, _ in kept for k in kernels}
    every = set(rn.rnswino_kernel_variants())
    assert len(every) > 100
    assert every - reached == set(), sorted(every - reached)
    assert reached - every == set()
    assert {c for _, _, c in kept} == {"unreduced-binary32", "unreduced-binary64", "reduced-binary32", "reduced-binary64",
                                       "reduced-binary64-mul32"}
    # the streaming inverse transform in all its output modes, with each conversion it can take
    stream = {(c, case[10]) for case, kernels, c in kept if kernels[2].startswith("k3_inverse_crt_stream")}
    assert stream >= {(c, mode) for c in ("unreduced-binary32", "unreduced-binary64", "reduced-binary32") for mode in (0, 1, 2)}
    # and the whole list stays affordable for the CPU oracle: direct-convolution operations of all cases together
    gop = sum(2.0 * c[0] * c[1] * c[2] * c[3] * c[4] * c[5] ** 2 for c, _, _ in kept) / 1e9
    assert gop < 600.0


def _conversion(C, moduli, r=3, m=8, flags=HOST, K=16, hw=16):
    plan = rn.rnswino_plan(1, C, K, hw, hw, r, m, r // 2, moduli, flags=flags)
    return rn.rnswino_plan_describe(plan)["conversion"]


def test_conversion_form_at_the_edges_the_gpu_cases_sit_on():
    """Which form of the conversion out of the RNS (section 3) a layer takes is decided on the host from its worst case
    2^14 r^2 C against the product of the moduli; the GPU parity cases at the edge of the dynamic range rely on these."""
    three, four = (251, 241, 239), (251, 241, 239, 233)
    assert _conversion(16, three) == "unreduced-binary32"
    assert _conversion(42, three) == "unreduced-binary32"       # largest C with room for the binary32 error bound
    assert _conversion(43, three) == "unreduced-binary64"
    assert _conversion(49, three) == "unreduced-binary64"       # the edge of the range of three moduli
    assert _conversion(50, three, flags=HOST | UNCHECKED) == "unreduced-binary64"
    assert _conversion(256, four) == "unreduced-binary32"       # the VGG16-style layer
    assert _conversion(11422, four) == "unreduced-binary64"     # the edge of the range of four moduli
    assert _conversion(512, three, flags=HOST | UNCHECKED) == "unreduced-binary64"     # the paper's setting, range trusted
    # four moduli near 253: two quotients are closer than the binary64 sum of unreduced accumulators resolves
    assert _conversion(9800, (253, 251, 247, 241), flags=HOST | UNCHECKED) == "reduced-binary32"      # |y| <= 0.45 P
    assert _conversion(11600, (253, 251, 247, 241), flags=HOST | UNCHECKED) == "reduced-binary64"
    assert _conversion(64, (253, 251, 247, 241)) == "unreduced-binary32"
    # five and more moduli: a partial product P/p_i no longer fits 24 bits
    assert _conversion(64, (251, 241, 239, 233, 229)) == "reduced-binary64-mul32"
    # 16-bit moduli always reduce (their accumulators are three byte-plane sums)
    assert _conversion(512, (65521, 65519), m=14) == "reduced-binary32"
    assert _conversion(14000, (65521, 65519), m=14) == "reduced-binary64"
    assert _conversion(16, (65521, 65519, 65497), m=14) == "reduced-binary64-mul32"


def test_workload_kernels():
    """The instantiations the five benchmark workloads launch (the names a kernel trace of bench.py shows)."""
    import synth_inputs as si
    want = {1: ("k1_input_transform<2, false, false>", "k2_residue_gemm<1, 1, 2, false>", "k3_inverse_crt<3, 2, false, true>"),
            2: ("k1_input_transform<2, false, false>", "k2_residue_gemm_lds<4, 1, 2, 4, 4>", "k3_inverse_crt<4, 2, false, true>"),
            3: ("k1_input_transform<4, false, false>", "k2_residue_gemm<2, 1, 2, false>", "k3_inverse_crt<4, 4, false, true>"),
            4: ("k1_input_transform<4, true, false>", "k2_residue_gemm<4, 1, 2, true>", "k3_inverse_crt<2, 4, true, false>")}
    for idx, kernels in want.items():
        c = si.layer_config(idx)
        plan = rn.rnswino_plan(c["N"], c["C"], c["K"], c["H"], c["W"], c["r"], c["m"], c["pad"], c["moduli"], flags=HOST)
        assert tuple(rn.rnswino_plan_describe(plan)["kernels"]) == kernels, idx


@pytest.mark.parametrize("t", [13, 14, 15, 16])
def test_every_admissible_set_of_four_moduli_has_an_instantiation(t):
    """With 13 and more interpolation points the reduced conversion has no instantiation for exactly four 8-bit moduli
    (no admissible set's product is large enough to need it): every such set must still give a plan, whatever the
    channel count."""
    r, m = 3, t - 2
    ok = [p for p in range(129, 254, 2) if rn_accepts(p, r, m)]
    top = sorted(ok)[-7:]
    tried = 0
    for moduli in itertools.combinations(top, 4):
        try:
            plan = rn.rnswino_plan(1, 12000, 8, m, m, r, m, 1, moduli, flags=HOST | UNCHECKED)
        except rn.RnsWinoError as e:
            assert e.code == -3, (moduli, e.code)       # not pairwise coprime: refused for that reason only
            continue
        assert rn.rnswino_plan_describe(plan)["conversion"].startswith("unreduced")
        tried += 1
    assert tried >= 10


def rn_accepts(p, r, m):
    try:
        rn.rnswino_plan(1, 1, 1, m, m, r, m, 1, (p,), flags=HOST | UNCHECKED)
    except rn.RnsWinoError:
        return False
    return True


def test_16_bit_moduli_refuse_contractions_of_1024_steps():
    """Three unreduced 32-bit byte-plane sums: the middle one gains up to 2^21 per 64-channel step."""
    def code(C):
        try:
            rn.rnswino_plan(1, C, 4, 4, 4, 1, 4, 0, (65521, 65519), flags=HOST | UNCHECKED)
        except rn.RnsWinoError as e:
            return e.code
        return 0
    assert code(65472) == 0 and code(65473) == -2
    assert code(131071) == -2


def test_measurement_flag_selects_the_64_by_16_gemm_blocks():
    plain = rn.rnswino_plan(8, 64, 64, 56, 56, 3, 8, 1, (251, 241, 239, 233), flags=HOST)
    forced = rn.rnswino_plan(8, 64, 64, 56, 56, 3, 8, 1, (251, 241, 239, 233), flags=HOST | rn.FLAG_GEMM_BLOCK_64X16)
    assert rn.rnswino_plan_describe(plan=plain)["kernels"][1] == "k2_residue_gemm<1, 4, 2, false>"
    assert rn.rnswino_plan_describe(plan=forced)["kernels"][1] == "k2_residue_gemm_lds<4, 1, 1, 1, 4>"
    wide = rn.rnswino_plan(1, 64, 64, 28, 28, 3, 14, 1, (65521, 65519), flags=HOST | rn.FLAG_GEMM_BLOCK_64X16)
    assert rn.rnswino_plan_describe(plan=wide)["kernels"][1].startswith("k2_residue_gemm<")      # 8-bit moduli only
