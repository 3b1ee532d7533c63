"""The seeded input generator: known-answer vector and distribution sanity."""
import numpy as np

import synth_inputs as si


def _scalar_splitmix64(seed, count):
    mask = (1 << 64) - 1
    out, state = [], seed
    for _ in range(count):
        state = (state + 0x9E3779B97F4A7C15) & mask
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        out.append(z ^ (z >> 31))
    return out


def test_splitmix64_known_answer():
    # first outputs of the public-domain splitmix64 reference for seed 1234567
    expect = [6457827717110365317, 3203168211198807973, 9817491932198370423,
              4593380528125082431, 16408922859458223821]
    assert [int(v) for v in si.splitmix64(1234567, 5)] == expect


def test_vectorised_matches_scalar():
    for seed in (0, 1001, 2**63 + 5):
        assert [int(v) for v in si.splitmix64(seed, 64)] == _scalar_splitmix64(seed, 64)


def test_int8_tensor_is_top_byte_in_memory_order():
    t = si.int8_tensor(2002, (3, 5, 7))
    ref = [(z >> 56) - 256 if (z >> 56) >= 128 else (z >> 56) for z in _scalar_splitmix64(2002, 105)]
    assert t.dtype == np.int8 and t.reshape(-1).tolist() == ref


def test_int8_tensor_chunking_is_seamless():
    big = si.int8_tensor(7, ((1 << 22) + 1000,))
    tail = _scalar_splitmix64(7 + ((1 << 22) - 2) * 0x9E3779B97F4A7C15, 4)
    # element k uses state seed + (k+1)*gamma: restart the scalar stream just before the chunk edge
    ref = [np.uint8(z >> 56).astype(np.int8) for z in tail]
    assert big[(1 << 22) - 2:(1 << 22) + 2].tolist() == [int(v) for v in ref]


def test_uniform_over_full_int8_range():
    t = si.int8_tensor(99, (1 << 16,))
    assert t.min() == -128 and t.max() == 127
    assert abs(float(t.astype(np.float64).mean())) < 1.5


def test_configs_shapes():
    c2 = si.layer_config(2)
    assert (c2["C"], c2["K"], c2["H"], c2["m"], c2["moduli"]) == (256, 256, 56, 8, (251, 241, 239, 233))
    stack = si.vgg16_stack()
    assert len(stack) == 13 and stack[0]["moduli"] == (251, 241, 239)
    assert [l["shift"] for l in stack] == [9, 11, 11, 11, 11, 12, 12, 12, 12, 12, 12, 12, 12]
