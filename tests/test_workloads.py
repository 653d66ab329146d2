"""The seeded generators: determinism and the structure each configuration promises (CPU only)."""
import numpy as np

from workloads import bits_to_f64, lognormal_degree, make_config, rmat, round_to_bits, stream, uniform_fixed_degree


def test_streams_are_reproducible_and_independent():
    a = stream(0, 2, 1).random(4)
    b = stream(0, 2, 1).random(4)
    c = stream(0, 2, 2).random(4)
    assert np.array_equal(a, b) and not np.array_equal(a, c)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
    assert round_to_bits(x, "bf16").tolist() == [0x3F80, 0x3F80, 0x3F81, 0x3F82]
    assert bits_to_f64(np.array([0x3F80, 0xC000], dtype=np.uint16), "bf16").tolist() == [1.0, -2.0]


def test_fixed_degree_is_exact_and_distinct():
    deg = np.array([0, 1, 50, 64, 7])
    r, c = uniform_fixed_degree(5, 64, deg, stream(1, 0, 0))
    assert np.array_equal(np.bincount(r, minlength=5), deg)
    assert len(set(zip(r.tolist(), c.tolist()))) == deg.sum()


def test_rmat_quadrant_probabilities():
    r, c = rmat(1, 1 << 16, 0.57, 0.19, 0.19, 0.05, stream(2, 0, 0))
    n = r.shape[0]
    frac = [np.mean((r == i) & (c == j)) for i in (0, 1) for j in (0, 1)]  # a, b, c, d
    assert n == 1 << 17
    assert np.allclose(frac, [0.57, 0.19, 0.19, 0.05], atol=0.01)


def test_lognormal_degree_is_clipped():
    d = lognormal_degree(20000, 2.5, 1.0, 1, 4096, stream(3, 0, 0))
    assert d.min() >= 1 and d.max() <= 4096
    assert 10 < np.median(d) < 15  # exp(2.5) = 12.2


def test_shrunk_configs_have_the_promised_shape():
    c2 = make_config("cfg2_rmat16", shrink=16)
    A = c2["A"]
    assert A.M == 4096 and c2["spmm"][0].shape == (4096, 128) and c2["sddmm"][0].shape == (4096, 32)
    assert A.nnz < 16 * 4096 and np.diff(A.rowptr).max() > 200  # duplicates removed; heavy tail
    v = bits_to_f64(A.vals, "f16")
    assert v.min() >= 0 and v.max() <= 1
    c3 = make_config("cfg3_stencil", shrink=32)
    assert c3["A"].M == 32 * 32 and [b.shape[1] for b in c3["spmm"]] == [64, 256]
    c5 = make_config("cfg5_lognormal", shrink=64)
    assert c5["A"].M == 4096 and c5["sddmm"][0].shape == (4096, 64) and c5["chain"].shape == (4096, 256)
    s = bits_to_f64(c5["sddmm"][0].bits, "f16").std()
    assert abs(s - np.sqrt(1 / 8)) < 0.01
    c4 = make_config("cfg4_rmat20", shrink=256)
    assert c4["A"].dtype == "bf16" and c4["spmm"][0].dtype == "bf16" and c4["A"].M == 4096
