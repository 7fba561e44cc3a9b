"""The seeded input generator: published SplitMix64 values, determinism, moments, bf16 rounding."""
import numpy as np

from paper_2504_03871_amd import synth as S


def test_splitmix64_known_values():
    # first outputs of SplitMix64 seeded with 0 and with 1234567 (values published with the
    # reference implementation of the generator)
    z = S.splitmix64(0, np.arange(3, dtype=np.uint64))
    assert [int(v) for v in z] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    z = S.splitmix64(1234567, np.arange(2, dtype=np.uint64))
    assert [int(v) for v in z] == [6457827717110365317, 3203168211198807973]


def test_blocks_are_order_independent():
    a = S.normal_block(42, 0, 1000)
    b = np.concatenate([S.normal_block(42, 0, 333), S.normal_block(42, 333, 667)])
    assert (a == b).all()
    c = S.normal_f32(42, (10, 100), threads=4, chunk=128)
    assert (c.reshape(-1) == a.astype(np.float32)).all()


def test_moments():
    a = S.normal_block(7, 0, 400000, std=0.02)
    assert abs(a.mean()) < 2e-4 and abs(a.std() / 0.02 - 1) < 5e-3
    assert abs(((a / 0.02) ** 4).mean() - 3.0) < 0.05


def test_bf16_rounding():
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -3.5, 0.0], np.float32)
    bits = S.f32_to_bf16_bits(f)
    back = S.bf16_bits_to_f32(bits)
    # ties go to the even mantissa; anything above the tie rounds up
    assert back.tolist() == [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7, -3.5, 0.0]


def test_workloads():
    w = S.WORKLOADS
    assert w["cfg4"].capacity == 2560 and w["cfg1"].capacity == 0
    assert w["cfg0"].dtype == S.DT_F32 and w["cfg3"].act == S.ACT_SWIGLU
    assert w["cfg1"].scaled(capacity_factor=1.0).capacity == 2048
    b = S.router_bias(w["cfg2"])
    assert b[0] == 0 and abs(b[15] + 1.2 * np.log(16)) < 1e-6
    lo, hi = S.partial_slices(w["cfg4"].scaled(E=4), np.array([10, 11, 12, 13]))
    assert lo.tolist() == [0, 0, 12 - 4, 13 - 5] and hi.tolist() == [10, 11, 12, 13]
    inp = S.make_inputs(w["cfg0"])
    assert inp["x"].shape == (512, 128) and inp["W1"].shape == (8, 128, 256) and "x_bits" not in inp
    small = w["cfg1"].scaled(T=64, d=64, f=128)
    inp = S.make_inputs(small)
    assert inp["x_bits"].dtype == np.uint16
    assert (S.bf16_bits_to_f32(inp["x_bits"]) == inp["x"]).all()
    assert abs(inp["Wr"].std() * 8 - 1) < 0.1


def test_f16_rounding_is_nearest_even_and_round_trips():
    a = np.array([1.0, 1.0 + 2 ** -11, 1.0 + 3 * 2 ** -11, 65504.0, 6e-8, -0.1], dtype=np.float32)
    bits = S.f32_to_f16_bits(a)
    back = S.f16_bits_to_f32(bits)
    # ties go to the even significand: 1 + 2^-11 -> 1, 1 + 3 * 2^-11 -> 1 + 2^-9
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.0 + 2 ** -9 and back[3] == 65504.0
    assert (S.f32_to_f16_bits(back) == bits).all()
    w = S.WORKLOADS["cfg1"].scaled(T=64, d=64, f=64, dtype=S.DT_F16)
    inp = S.make_inputs(w)
    assert (S.f16_bits_to_f32(inp["x_bits"]) == inp["x"]).all() and inp["Wr"].dtype == np.float32
