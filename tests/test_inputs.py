"""The seeded generators: determinism, counter-based addressing, ranges and rough moments."""
import numpy as np

from paper_2411_17887_amd import inputs


def test_splitmix64_reference_values():
    """First outputs of SplitMix64 from state 0, as listed with the generator's published definition
    (x += golden; mix) -- pins the constants and shift amounts."""
    z = inputs.splitmix64(0, 0, 3)
    assert [int(v) for v in z] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_counter_addressing_is_chunk_independent():
    a = inputs.f32_normal((1 << 22) + 1000, 5)
    b = inputs.f32_normal(1000, 5)
    assert np.array_equal(a[:1000], b)
    z = inputs.splitmix64(9, 12345, 10)
    assert np.array_equal(inputs.splitmix64(9, 0, 12355)[12345:], z)


def test_ranges_and_moments():
    n = 1 << 18
    x = inputs.int32_small(n, 1)
    assert x.dtype == np.int32 and x.min() == -128 and x.max() == 127 and abs(x.mean() + 0.5) < 1.0
    h = inputs.f16_uniform01(n, 2)
    assert h.dtype == np.float16 and h.min() >= 0 and h.max() < 1 and abs(float(h.astype(np.float64).mean()) - 0.5) < 5e-3
    m = inputs.mask_i8(n, 3)
    assert m.dtype == np.int8 and set(np.unique(m)) == {0, 1}
    g = inputs.f32_normal(n, 4).astype(np.float64)
    assert abs(g.mean()) < 1e-2 and abs(g.std() - 1) < 1e-2 and abs((g ** 3).mean()) < 5e-2
    b = (inputs.bf16_uniform_pm1(n, 5).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert b.min() >= -1 and b.max() <= 1 and abs(b.mean()) < 1e-2 and abs(b.var() - 1 / 3) < 1e-2
    t = inputs.tri_f32(n, 6)
    assert set(np.unique(t)) == {-1.0, 0.0, 1.0}


def test_bf16_rounding_is_nearest_even():
    v = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2 ** -9, -0.3], dtype=np.float32)
    bits = inputs.f32_to_bf16_bits(v)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties to 1 + 2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == 1.0
    assert abs(back[4] + 0.3) <= 2 ** -9


def test_configs_table():
    assert inputs.CONFIGS["C4"]["cols"] == 100_000_007 and inputs.CONFIGS["C5"]["rows"] * inputs.CONFIGS["C5"]["cols"] == 1 << 28
    x = inputs.make_config("C1")
    assert x.shape == (4096,) and x.dtype == np.int32
