"""Pins for the from-scratch aggregation (paper Section 3.2, Eq. 1): dense adjacency matmul written
from the definition, and textbook special cases."""
import itertools

import numpy as np
import pytest

import oracle


def _dense_ahat(n, src, dst, mode, self_loop):
    """Normalised dense adjacency from the definition: A[v,u] = 1 per edge u->v, plus I."""
    a = np.zeros((n, n))
    for u, v in zip(src, dst):
        if u != v:
            a[v, u] = 1.0
    if self_loop:
        a = a + np.eye(n)
    deg = a.sum(axis=1)
    with np.errstate(divide="ignore"):
        if mode == "sum":
            return a
        if mode == "mean":
            inv = np.where(deg > 0, 1.0 / deg, 0.0)
            return inv[:, None] * a
        inv = np.where(deg > 0, deg ** -0.5, 0.0)
        return inv[:, None] * a * inv[None, :]


def _matmul_loops(a, x):
    n, d = x.shape
    out = np.zeros((n, d))
    for i in range(n):
        for k in range(n):
            if a[i, k] != 0.0:
                for j in range(d):
                    out[i, j] += a[i, k] * x[k, j]
    return out


@pytest.mark.parametrize("mode,self_loop", list(itertools.product(["sum", "mean", "sym"], [False, True])))
def test_against_dense_matmul(mode, self_loop):
    rng = np.random.default_rng(7)
    n, d = 37, 5
    src = rng.integers(0, n, 160)
    dst = rng.integers(0, n, 160)
    dst[:10] = 3  # one hub
    dst[dst == 11] = 12  # node 11 has no in-edge
    x = rng.standard_normal((n, d))
    keys = oracle.canonicalise(src, dst, n)
    rp, col = oracle.csr_from_keys(keys, n)
    _, agg = oracle.aggregate(rp, col, x, mode, self_loop)
    ref = _matmul_loops(_dense_ahat(n, src, dst, mode, self_loop), x)
    assert np.allclose(agg, ref, rtol=1e-12, atol=1e-12)
    if not self_loop:
        assert np.all(agg[11] == 0.0)


def test_handmade_sum():
    # edges 0->2, 1->2, 2->0 ; x = [[1],[10],[100]]
    rp, col = oracle.csr_from_keys(oracle.canonicalise([0, 1, 2], [2, 2, 0], 3), 3)
    x = np.array([[1.0], [10.0], [100.0]])
    s, agg = oracle.aggregate(rp, col, x, "sum", False)
    assert agg.ravel().tolist() == [100.0, 0.0, 11.0]
    s, agg = oracle.aggregate(rp, col, x, "sum", True)
    assert agg.ravel().tolist() == [101.0, 10.0, 111.0]
    _, agg = oracle.aggregate(rp, col, x, "mean", True)
    assert np.allclose(agg.ravel(), [101.0 / 2, 10.0, 111.0 / 3])
    # sym: deg = [2,1,3]; row 2 = (x0/sqrt2 + x1/1 + x2/sqrt3)/sqrt3
    _, agg = oracle.aggregate(rp, col, x, "sym", True)
    assert np.isclose(agg[2, 0], (1 / np.sqrt(2) + 10 + 100 / np.sqrt(3)) / np.sqrt(3))
    assert np.isclose(agg[0, 0], (1 / np.sqrt(2) + 100 / np.sqrt(3)) / np.sqrt(2))


def test_direction_is_source_to_target():
    # a transposed operand would put the value in row 0 instead of row 1
    rp, col = oracle.csr_from_keys(oracle.canonicalise([0], [1], 2), 2)
    _, agg = oracle.aggregate(rp, col, np.array([[5.0], [7.0]]), "sum", False)
    assert agg.ravel().tolist() == [0.0, 5.0]


def test_empty_graph():
    n = 6
    x = np.arange(12.0).reshape(n, 2)
    rp, col = oracle.csr_from_keys(np.empty(0, dtype=np.uint64), n)
    for mode in ("sum", "mean", "sym"):
        _, agg = oracle.aggregate(rp, col, x, mode, True)
        assert np.allclose(agg, x)  # deg = 1 everywhere
        _, agg = oracle.aggregate(rp, col, x, mode, False)
        assert np.all(agg == 0.0)


def test_complete_graph_sum():
    n = 9
    x = np.random.default_rng(0).standard_normal((n, 4))
    src, dst = np.array([(u, v) for u in range(n) for v in range(n) if u != v]).T
    rp, col = oracle.csr_from_keys(oracle.canonicalise(src, dst, n), n)
    _, agg = oracle.aggregate(rp, col, x, "sum", True)
    assert np.allclose(agg, np.tile(x.sum(axis=0), (n, 1)))


def test_regular_graph_mean_and_sym():
    n, k = 12, 4  # ring lattice, undirected: each node linked to +-1, +-2
    src, dst = [], []
    for v in range(n):
        for o in (1, 2):
            src += [v, (v + o) % n]
            dst += [(v + o) % n, v]
    rp, col = oracle.csr_from_keys(oracle.canonicalise(src, dst, n), n)
    const = np.full((n, 3), 2.5)
    _, agg = oracle.aggregate(rp, col, const, "mean", True)
    assert np.allclose(agg, 2.5)
    x = np.random.default_rng(1).standard_normal((n, 3))
    s_sum, _ = oracle.aggregate(rp, col, x, "sum", True)
    _, agg = oracle.aggregate(rp, col, x, "sym", True)
    assert np.allclose(agg, s_sum / (k + 1))


def test_duplicates_and_self_loops_are_dropped():
    keys = oracle.canonicalise([0, 0, 1, 2, 2], [1, 1, 1, 0, 0], 3)
    assert keys.tolist() == [(0 << 32) | 2, (1 << 32) | 0]
    with pytest.raises(ValueError):
        oracle.canonicalise([0, 3], [1, 1], 3)


def test_adjoint_is_transpose():
    rng = np.random.default_rng(3)
    n, d = 25, 3
    keys = oracle.canonicalise(rng.integers(0, n, 90), rng.integers(0, n, 90), n)
    rp, col = oracle.csr_from_keys(keys, n)
    src, dst = (keys & np.uint64(0xFFFFFFFF)).astype(int), (keys >> np.uint64(32)).astype(int)
    for mode, sl in itertools.product(["sum", "mean", "sym"], [False, True]):
        a = _dense_ahat(n, src, dst, mode, sl)
        g = rng.standard_normal((n, d))
        assert np.allclose(oracle.aggregate_adjoint(rp, col, g, mode, sl), a.T @ g, atol=1e-12)
        x = rng.standard_normal((n, d))  # <A x, g> == <x, A^T g>
        _, ax = oracle.aggregate(rp, col, x, mode, sl)
        assert np.isclose((ax * g).sum(), (x * oracle.aggregate_adjoint(rp, col, g, mode, sl)).sum())


def test_row_sampled_form_equals_full():
    rng = np.random.default_rng(11)
    n, d = 60, 4
    keys = oracle.canonicalise(rng.integers(0, n, 300), rng.integers(0, n, 300), n)
    rp, col = oracle.csr_from_keys(keys, n)
    x = rng.standard_normal((n, d))
    rows = np.array([0, 7, 33, 59])
    for mode, sl in itertools.product(["sum", "mean", "sym"], [False, True]):
        s_full, agg_full = oracle.aggregate(rp, col, x, mode, sl)
        s, agg = oracle.aggregate_rows(rp, col, x, rows, mode, sl)
        assert np.allclose(s, s_full[rows], atol=1e-13) and np.allclose(agg, agg_full[rows], atol=1e-13)
