"""Pins of the fractional quantiser (Sec. 4.3.2): a case worked out by hand from
the paper's interval formula, closed forms (edges are a geometric sequence from
v_max down to v_min; the means reproduce equal values exactly), invariants (every
magnitude lies in the interval its code names; the reproduction error is bounded by
the interval's width), and the bit budget of Table 1's "-Q" rows (q = 4)."""
import numpy as np
import pytest


def test_hand_worked_example(oracle):
    # q = 2: L = 2 intervals, alpha = sqrt(v_max / v_min) = sqrt(16 / 1) = 4,
    # I_1 = [16, 4], I_2 = [4, 1] (Sec. 4.3.2); a value on the shared edge 4 goes down.
    v = np.array([16.0, -8.0, 4.0, 2.0, -1.0, 5.0], np.float32)
    edges = oracle.quant_edges(v, 2)
    assert edges.tolist() == [16.0, 4.0]
    codes, means = oracle.quant_encode(v, 2)
    #           16   -8        4    2   -1        5
    assert codes.tolist() == [0, 0 | 2, 1, 1, 1 | 2, 0]
    assert means.tolist() == [np.float32(29.0 / 3.0), np.float32(7.0 / 3.0)]      # (16+8+5)/3, (4+2+1)/3
    out = oracle.quant_decode(codes, 2, means)
    assert np.allclose(out, [29 / 3, -29 / 3, 7 / 3, 7 / 3, -7 / 3, 29 / 3], rtol=1e-7)
    # stream layout: value k in bits [2k, 2k+2), low bit first: codes 0,2,1,1,3,0
    words = oracle.quant_pack(codes, 2)
    assert int(words[0]) == (0 | 2 << 2 | 1 << 4 | 1 << 6 | 3 << 8 | 0 << 10)


@pytest.mark.parametrize("q", [2, 3, 4, 6, 8])
def test_edges_are_the_geometric_sequence(oracle, q):
    rng = np.random.default_rng(q)
    v = (rng.standard_normal(5000) * 10.0 ** rng.uniform(-3, 1, 5000)).astype(np.float32)
    L = 1 << (q - 1)
    edges = oracle.quant_edges(v, q)
    vmax, vmin = np.abs(v).max().astype(np.float64), np.abs(v[v != 0]).min().astype(np.float64)
    assert edges[0] == vmax
    alpha = (vmax / vmin) ** (1.0 / L)
    assert np.allclose(edges, vmax / alpha ** np.arange(L), rtol=1e-12)
    assert np.isclose(edges[-1] / alpha, vmin, rtol=1e-12)        # the last interval ends at v_min


@pytest.mark.parametrize("q", [2, 4, 5])
def test_codes_name_the_interval_and_error_is_bounded(oracle, q):
    rng = np.random.default_rng(10 + q)
    v = (rng.standard_normal(20000) * np.exp(rng.standard_normal(20000))).astype(np.float32)
    v[::97] = 0.0
    L = 1 << (q - 1)
    codes, means = oracle.quant_encode(v, q)
    edges = oracle.quant_edges(v, q)
    lo = np.append(edges[1:], 0.0)                                # lower end of every interval (zeros included)
    l = (codes & (L - 1)).astype(np.int64)
    sign = codes >> (q - 1)
    m = np.abs(v).astype(np.float64)
    assert np.all(m <= edges[l]) and np.all(m >= lo[l] * (1 - 1e-15))
    assert np.all(m[l < L - 1] > edges[l[l < L - 1] + 1])        # strictly above the next edge
    assert np.array_equal(sign.astype(bool), np.signbit(v))
    for j in range(L):
        sel = l == j
        if sel.any():
            assert means[j] == np.float32(m[sel].sum() / sel.sum()) or \
                abs(float(means[j]) - m[sel].mean()) <= 1e-6 * m[sel].mean()
            assert lo[j] <= means[j] <= edges[j] * (1 + 1e-7)
        else:
            assert means[j] == 0
    out = oracle.quant_decode(codes, q, means)
    assert np.array_equal(np.signbit(out), np.signbit(v))
    # the reproduction stays inside the value's interval
    assert np.all(np.abs(out) <= edges[l] * (1 + 1e-7)) and np.all(np.abs(out) >= lo[l] * (1 - 1e-7))


def test_degenerate_inputs(oracle):
    codes, means = oracle.quant_encode(np.zeros(10, np.float32), 4)
    assert (codes & 7).tolist() == [7] * 10 and not means.any()        # zeros: last interval, mean 0
    assert not oracle.quant_decode(codes, 4, means).any()
    v = np.array([-2.5, 2.5, 2.5], np.float32)                    # one magnitude: alpha = 1, all on every edge
    codes, means = oracle.quant_encode(v, 4)
    assert (codes & 7).tolist() == [7, 7, 7] and means[7] == 2.5
    assert oracle.quant_decode(codes, 4, means).tolist() == [-2.5, 2.5, 2.5]
    v = np.array([3.0, 0.0, -0.0, 1e-3], np.float32)              # zeros go to the last interval
    codes, means = oracle.quant_encode(v, 3)
    assert (codes & 3).tolist() == [0, 3, 3, 3] and (codes >> 2).tolist() == [0, 0, 1, 0]
    with pytest.raises(ValueError):
        oracle.quant_encode(v, 1)


def test_bit_budget_of_the_quantised_rows_of_table_1(oracle):
    # Table 1, SSGD-MV-L8-Q: 4 bits per value, phi = 1e-2, H = 8 -> q-bar_val = 5e-3
    d, phi, q, H = 11173962, 1e-2, 4, 8
    n = round(phi * d)
    codes = np.zeros(n, np.uint8)
    words = oracle.quant_pack(codes, q)
    assert abs(words.size * 32 / (d * H) - 5e-3) < 1e-5
