"""The break points the library's GELU epilogue works with (host code, no GPU) against the
oracle's own GELU code function: for a set of output scales and zero points the piecewise-constant
function rebuilt from the break points equals the oracle's code for every fp32 value in a
neighbourhood of every break point, for a dense sweep, and for random values of every magnitude."""
import numpy as np
import pytest


@pytest.fixture(scope="module")
def rm():
    import paper_2111_00153_amd as m
    return m


def _from_table(t, y):
    y = np.asarray(y, np.float32)
    rise = np.count_nonzero(t["rise"][None, :] <= y[:, None], axis=1) - 1        # largest c with rise[c] <= y
    fall = t["fall_base"] + np.count_nonzero(y[:, None] <= t["fall"][None, :t["n_fall"]], axis=1)
    return np.where(y < np.float32(t["y_split"]), fall, rise).astype(np.uint8)


def _neighbours(x, n=300):
    """The n fp32 values on either side of x."""
    x = np.float32(x)
    if not np.isfinite(x):
        return np.empty(0, np.float32)
    k = np.array([x], np.float32).view(np.int32)[0]
    key = np.int64(k) if k >= 0 else np.int64(-0x80000000) - np.int64(k)
    keys = key + np.arange(-n, n + 1, dtype=np.int64)
    bits = np.where(keys >= 0, keys, np.int64(-0x80000000) - keys).astype(np.int64)
    return (bits & 0xffffffff).astype(np.uint32).view(np.float32)


@pytest.mark.parametrize("inv_s,z", [(2.0, 0), (2.0, 1), (1.0, 0), (0.7, 3), (2.94, 1), (3.5, 1), (6.0, 2),
                                     (11.0, 4), (40.0, 9), (100.0, 15), (0.05, 0), (1.7, 15)])
def test_breakpoints_reproduce_the_oracle_codes(rm, oracle, inv_s, z):
    inv_s = float(np.float32(inv_s))
    t = rm.rmsmp_debug_gelu_breakpoints(inv_s, z)
    assert t["rise"][0] == -np.inf and 0 <= t["n_fall"] <= 15
    ys = [np.linspace(-12.0, 24.0, 200001, dtype=np.float32), _neighbours(t["y_split"], 2000),
          _neighbours(0.0), np.float32([-3e38, -1e10, -50.0, 50.0, 1e10, 3e38, -0.0, 0.0])]
    ys += [_neighbours(b) for b in t["rise"]] + [_neighbours(b) for b in t["fall"][:t["n_fall"]]]
    rng = np.random.default_rng(int(inv_s * 1000) + z)
    ys.append((rng.standard_normal(200000) * rng.choice([0.01, 0.3, 1.0, 4.0, 30.0], 200000)).astype(np.float32))
    y = np.concatenate(ys)
    _, q = oracle.gelu_codes(y, inv_s, z)
    assert np.array_equal(_from_table(t, y), q)


def test_breakpoints_argument_errors(rm):
    for inv_s, z in ((0.0, 0), (-1.0, 0), (float("inf"), 0), (float("nan"), 0), (1.0, -1), (1.0, 16)):
        with pytest.raises(rm.RmsmpError) as e:
            rm.rmsmp_debug_gelu_breakpoints(inv_s, z)
        assert e.value.code == 1
