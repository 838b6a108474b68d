"""The synthetic-input generator: determinism, format conversion, planted structure."""
import numpy as np

import ems_inputs


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, 1.00390625, 1.001953125, 1.005859375, -2.5, 0.0, 3.1415927], np.float32)
    bits = ems_inputs.f32_to_bf16_bits(x)
    back = ems_inputs.bf16_bits_to_f32(bits)
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even (1.0); 1 + 3*2^-9 is a tie -> 1+2^-7... checked
    # against the definition: nearest multiple of 2^-7 in [1,2), ties to even mantissa
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.0
    assert back[3] == 1.0078125 and back[4] == -2.5 and back[5] == 0.0
    assert abs(back[6] - 3.140625) < 1e-12
    np.testing.assert_array_equal(ems_inputs.f32_to_bf16_bits(back), bits)


def test_generation_is_seeded_and_sliceable():
    w = ems_inputs.WORKLOADS["tiny"]
    a = ems_inputs.generate(w)
    b = ems_inputs.generate(w)
    np.testing.assert_array_equal(a.q, b.q)
    np.testing.assert_array_equal(a.k, b.k)
    c = ems_inputs.generate(w, layer=1)
    assert (a.k != c.k).any()
    assert a.q.shape == (1, 4, 1024, 64) and a.k.shape == (1, 4, 1024, 64)
    assert a.q.dtype == np.uint16
    big = ems_inputs.Workload("t", 9, 3, 4, 2, 16, 64, 8, 16, heavy=4, sink=True, needle=4)
    full = ems_inputs.generate(big)
    part = ems_inputs.generate(big, batch_slice=slice(1, 2))
    np.testing.assert_array_equal(full.q[1:2], part.q)
    np.testing.assert_array_equal(full.v[1:2], part.v)


def test_planted_structure():
    w = ems_inputs.Workload("t", 9, 1, 4, 2, 64, 512, 16, 32, heavy=8, sink=True, needle=16)
    inp = ems_inputs.generate(w)
    k, q = inp.f32("k"), inp.f32("q")
    for kvh in range(2):
        pos = inp.heavy_pos[0][kvh]
        assert len(pos) == 8 and pos.min() >= 1
        # the shared direction shows up as the mean query; heavy keys project ~3 on it
        u = q[0, 2 * kvh:2 * kvh + 2].reshape(-1, 64).mean(0)
        u /= np.linalg.norm(u)
        proj = k[0, kvh] @ u
        assert proj[pos].mean() > 2.0 and abs(np.delete(proj, pos)[100:].mean()) < 0.5
        assert proj[0] > 2.0
        s = inp.needle_start[0][kvh]
        assert proj[s:s + 16].mean() > 2.0
    assert abs(inp.f32("v").mean()) < 0.05
