"""The seeded input generator: reproducible, prefix-stable, correctly rounded.  CPU only."""
import numpy as np

import mcf_inputs as mi


def test_reproducible_and_prefix_stable():
    w = mi.WORKLOADS["cfg3"]
    full = mi.make_inputs(mi.make_problem(3, 64, 64, 32, 64, "f16", True, "normal", w.seed), values=False)
    part = mi.make_inputs(mi.make_problem(3, 64, 64, 32, 64, "f16", True, "normal", w.seed), batch=2, values=False)
    for k in ("a_bits", "b_bits", "d_bits"):
        assert np.array_equal(full[k][:2], part[k])
    again = mi.draw(5, 1, (1000,), "uniform")
    assert np.array_equal(again, mi.draw(5, 1, (1000,), "uniform"))
    assert not np.array_equal(again, mi.draw(5, 2, (1000,), "uniform"))
    assert not np.array_equal(again, mi.draw(6, 1, (1000,), "uniform"))


def test_distributions():
    u = mi.draw(1, 1, (400000,), "uniform")
    assert u.min() >= -1 and u.max() < 1 and abs(u.mean()) < 5e-3 and abs(u.var() - 1 / 3) < 5e-3
    n = mi.draw(1, 1, (400000,), "normal")
    assert abs(n.mean()) < 5e-3 and abs(n.var() - 1) < 1e-2 and abs((n ** 3).mean()) < 3e-2
    assert np.isfinite(n).all()


def test_rounding_is_nearest_even_and_roundtrips():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -0.3, 1e-3, 0.0])
    bf = mi.from_bits(mi.to_bits(x, "bf16"), "bf16")
    assert bf[0] == 1.0 and bf[1] == 1.0 and bf[2] == 1.0 + 2 ** -6   # ties go to even mantissa
    assert np.all(np.abs(bf - x) <= np.abs(x) * 2 ** -8)
    h = mi.from_bits(mi.to_bits(x, "f16"), "f16")
    assert np.array_equal(h, x.astype(np.float16).astype(np.float64))
    for dt in ("f16", "bf16"):
        bits = np.arange(0, 0x7C00 if dt == "f16" else 0x7F80, 7, dtype=np.uint16)
        assert np.array_equal(mi.to_bits(mi.from_bits(bits, dt), dt), bits)


def test_workload_table_matches_accounting():
    w = mi.WORKLOADS
    assert [w[f"cfg{i}"].compulsory_bytes for i in range(1, 6)] == [294912, 16777216, 25165824, 10485760, 268435456]
    assert [w[f"cfg{i}"].flops for i in range(1, 6)] == [33554432, 4294967296, 6442450944, 8589934592, 549755813888]
    x = mi.make_inputs(mi.make_problem(2, 8, 16, 24, 32, "bf16", True, "normal", 1))
    assert x["b_bits"].shape == (2, 24, 16) and x["B"].shape == (2, 16, 24) and x["b_layout"] == "nk"
    assert np.array_equal(x["B"], mi.from_bits(x["b_bits"], "bf16").transpose(0, 2, 1))
