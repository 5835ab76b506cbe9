"""Pins for the CPU oracle: it is checked against things other than itself -- dense
brute force, closed forms worked out by hand, a library sparse product, algebraic
invariants and hand-written fixtures -- before anything is compared with it.

The paper prints no numeric example of this path, so every pin comes from the
definitions it states (section 1 "GNN" equation; section 7 GCN / GIN equations;
section 4.1 Steps 1-3; section 4.2) and from the mathematics.
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2209_06800_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = lambda s: np.random.default_rng(s)  # noqa: E731


# ----------------------------------------------------------------------------- helpers
def dense_adj(row_ptr, col, n):
    """Dense neighbour-count matrix (multiplicity kept, self-loops dropped)."""
    a = np.zeros((n, n), dtype=np.float64)
    for v in range(n):
        for e in range(row_ptr[v], row_ptr[v + 1]):
            if col[e] != v:
                a[v, col[e]] += 1.0
    return a


def dense_gcn_matrix(row_ptr, col, n):
    """D~^-1/2 (A + I) D~^-1/2 assembled densely with matrix products."""
    a = dense_adj(row_ptr, col, n)
    d = a.sum(axis=1) + 1.0
    s = np.diag(d ** -0.5)
    return s @ (a + np.eye(n)) @ s


def small_graph(n, avg_deg, seed):
    rng = RNG(seed)
    m = n * avg_deg // 2
    return inputs.canonical_csr(n, rng.integers(0, n, m), rng.integers(0, n, m))


def star(n):
    return inputs.csr_from_adjacency_lists([list(range(1, n))] + [[0]] * (n - 1))


def ring(n, k):
    """2k-regular ring lattice."""
    adj = [sorted({(v + s) % n for s in range(-k, k + 1) if s != 0}) for v in range(n)]
    return inputs.csr_from_adjacency_lists(adj)


# ----------------------------------------------------------------------------- GCN weights
def test_gcn_one_hot_features_give_normalised_adjacency():
    n = 48
    row_ptr, col = small_graph(n, 6, 11)
    out = oracle.aggregate(row_ptr, col, "gcn", np.eye(n, dtype=np.float64))
    deg = np.diff(row_ptr)
    for v in range(n):
        nb = set(col[row_ptr[v]:row_ptr[v + 1]].tolist())
        for u in range(n):
            if u == v:
                want = 1.0 / (deg[v] + 1)
            elif u in nb:
                want = 1.0 / math.sqrt((deg[u] + 1) * (deg[v] + 1))
            else:
                want = 0.0
            assert out[v, u] == pytest.approx(want, rel=1e-14, abs=1e-15)


def test_gcn_regular_graph_maps_ones_to_ones():
    for n, k in ((12, 1), (40, 3), (17, 8)):       # last one is the complete graph K17
        row_ptr, col = ring(n, k)
        out = oracle.aggregate(row_ptr, col, "gcn", np.ones((n, 3)))
        np.testing.assert_allclose(out, 1.0, rtol=1e-13)


def test_gcn_star_closed_form_fixture():
    cases = json.load(open(os.path.join(GOLDEN, "star_gcn.json")))["cases"]
    for c in cases:
        n = c["n"]
        row_ptr, col = star(n)
        out = oracle.aggregate(row_ptr, col, "gcn", np.ones((n, 1), dtype=np.float32))
        assert out[0, 0] == pytest.approx(c["centre"], rel=1e-13)
        np.testing.assert_allclose(out[1:, 0], c["leaf"], rtol=1e-13)


def test_gcn_hand_worked_leaf_rows():
    fx = json.load(open(os.path.join(GOLDEN, "tiny_partition.json")))
    row_ptr, col = inputs.csr_from_adjacency_lists(fx["adjacency"])
    x = np.array([[1.0, -2.0], [0.5, 4.0], [3.0, 1.0], [-1.0, 2.0],
                  [2.0, 2.0], [7.0, -3.0], [0.25, 8.0], [5.0, 5.0]])
    out = oracle.aggregate(row_ptr, col, "gcn", x)
    # node 3: one neighbour (node 2, degree 3): x2/sqrt(4*2) + x3/2
    np.testing.assert_allclose(out[3], x[2] / math.sqrt(8.0) + x[3] / 2.0, rtol=1e-14)
    # node 6: one neighbour (node 5, degree 3)
    np.testing.assert_allclose(out[6], x[5] / math.sqrt(8.0) + x[6] / 2.0, rtol=1e-14)
    # node 1: neighbours 0 (deg 3) and 2 (deg 3), own degree 2
    np.testing.assert_allclose(out[1], (x[0] + x[2]) / math.sqrt(12.0) + x[1] / 3.0, rtol=1e-14)


# ----------------------------------------------------------------------------- sums
@pytest.mark.parametrize("seed,n,avg,dim", [(1, 64, 4, 5), (2, 200, 12, 33), (3, 256, 40, 8)])
def test_aggregate_matches_dense_brute_force(seed, n, avg, dim):
    row_ptr, col = small_graph(n, avg, seed)
    x = RNG(seed + 100).standard_normal((n, dim))
    want_gcn = dense_gcn_matrix(row_ptr, col, n) @ x
    np.testing.assert_allclose(oracle.aggregate(row_ptr, col, "gcn", x), want_gcn, rtol=1e-12, atol=1e-13)
    for eps in (0.0, 0.3, -0.5):
        want_gin = (dense_adj(row_ptr, col, n) + (1.0 + eps) * np.eye(n)) @ x
        got = oracle.aggregate(row_ptr, col, "gin", x, eps=eps)
        np.testing.assert_allclose(got, want_gin, rtol=1e-12, atol=1e-13)


def test_aggregate_matches_scipy_sparse_product():
    n, dim = 3000, 24
    row_ptr, col = small_graph(n, 20, 7)
    x = RNG(8).standard_normal((n, dim))
    a = sp.csr_matrix((np.ones(col.size), col, row_ptr), shape=(n, n))
    dinv = 1.0 / np.sqrt(np.diff(row_ptr) + 1.0)
    a_hat = sp.diags(dinv) @ (a + sp.identity(n)) @ sp.diags(dinv)
    np.testing.assert_allclose(oracle.aggregate(row_ptr, col, "gcn", x), a_hat @ x, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(oracle.aggregate(row_ptr, col, "gin", x, eps=0.25),
                               (a + 1.25 * sp.identity(n)) @ x, rtol=1e-11, atol=1e-12)


def test_all_ones_gives_weighted_degree():
    n = 500
    row_ptr, col = small_graph(n, 9, 21)
    deg = np.diff(row_ptr)
    ones = np.ones((n, 2), dtype=np.float32)
    gin = oracle.aggregate(row_ptr, col, "gin", ones, eps=0.125)
    np.testing.assert_allclose(gin[:, 0], deg + 1.125, rtol=1e-14)
    gcn = oracle.aggregate(row_ptr, col, "gcn", ones)
    dinv = 1.0 / np.sqrt(deg + 1.0)
    want = np.array([dinv[v] * (dinv[col[row_ptr[v]:row_ptr[v + 1]]].sum() + dinv[v]) for v in range(n)])
    np.testing.assert_allclose(gcn[:, 1], want, rtol=1e-12)


def test_isolated_nodes_keep_their_own_embedding():
    row_ptr, col = inputs.csr_from_adjacency_lists([[], [2], [1], []])
    x = np.array([[3.0], [1.0], [5.0], [-2.0]])
    assert oracle.aggregate(row_ptr, col, "gcn", x)[[0, 3], 0].tolist() == [3.0, -2.0]
    assert oracle.aggregate(row_ptr, col, "gin", x, eps=0.5)[[0, 3], 0].tolist() == [4.5, -3.0]


def test_neighbour_order_inside_a_row_does_not_matter():
    n = 300
    row_ptr, col = small_graph(n, 14, 31)
    x = RNG(32).standard_normal((n, 7))
    shuffled = col.copy()
    rng = RNG(33)
    for v in range(n):
        rng.shuffle(shuffled[row_ptr[v]:row_ptr[v + 1]])
    for mode in ("gcn", "gin"):
        np.testing.assert_allclose(oracle.aggregate(row_ptr, shuffled, mode, x),
                                   oracle.aggregate(row_ptr, col, mode, x), rtol=1e-12, atol=1e-13)


def test_linearity_and_adjoint_identity():
    n = 400
    row_ptr, col = small_graph(n, 10, 41)
    rng = RNG(42)
    x, y = rng.standard_normal((n, 6)), rng.standard_normal((n, 6))
    for mode in ("gcn", "gin"):
        ax, ay = oracle.aggregate(row_ptr, col, mode, x), oracle.aggregate(row_ptr, col, mode, y)
        np.testing.assert_allclose(oracle.aggregate(row_ptr, col, mode, 2.5 * x - 0.75 * y),
                                   2.5 * ax - 0.75 * ay, rtol=1e-11, atol=1e-12)
        # undirected graph: the operator is symmetric, <y, A x> = <A y, x>
        assert np.vdot(y, ax) == pytest.approx(np.vdot(ay, x), rel=1e-11)


def test_column_sum_checksum():
    n = 800
    row_ptr, col = small_graph(n, 16, 51)
    x = RNG(52).standard_normal((n, 4))
    deg = np.diff(row_ptr)
    dinv = 1.0 / np.sqrt(deg + 1.0)
    c = np.array([dinv[u] * (dinv[col[row_ptr[u]:row_ptr[u + 1]]].sum() + dinv[u]) for u in range(n)])
    np.testing.assert_allclose(oracle.aggregate(row_ptr, col, "gcn", x).sum(axis=0), c @ x, rtol=1e-10)
    np.testing.assert_allclose(oracle.aggregate(row_ptr, col, "gin", x).sum(axis=0), (deg + 1.0) @ x, rtol=1e-10)


def test_input_self_loops_are_ignored_and_duplicates_count():
    # row 0 lists itself and lists node 1 twice
    row_ptr, col = inputs.csr_from_adjacency_lists([[0, 1, 1, 2], [0], [0]])
    x = np.array([[1.0], [10.0], [100.0]])
    gin = oracle.aggregate(row_ptr, col, "gin", x)
    assert gin[:, 0].tolist() == [1.0 + 10.0 + 10.0 + 100.0, 11.0, 101.0]
    want = dense_gcn_matrix(row_ptr, col, 3) @ x
    np.testing.assert_allclose(oracle.aggregate(row_ptr, col, "gcn", x), want, rtol=1e-14)
    assert oracle.degrees(row_ptr, col).tolist() == [3, 1, 1]


def test_directed_rows_use_each_nodes_own_row_length():
    # 0 <- {1, 2}; 1 <- {2}; 2 <- {}
    row_ptr, col = inputs.csr_from_adjacency_lists([[1, 2], [2], []])
    x = np.array([[1.0], [2.0], [4.0]])
    out = oracle.aggregate(row_ptr, col, "gcn", x)
    assert out[0, 0] == pytest.approx(2.0 / math.sqrt(2 * 3) + 4.0 / math.sqrt(1 * 3) + 1.0 / 3)
    assert out[1, 0] == pytest.approx(4.0 / math.sqrt(1 * 2) + 2.0 / 2)
    assert out[2, 0] == 4.0


def test_bf16_inputs_are_read_exactly():
    n = 120
    row_ptr, col = small_graph(n, 8, 61)
    xf = RNG(62).standard_normal((n, 16)).astype(np.float32)
    bits = inputs.to_bf16_bits(xf)
    as_f32 = inputs.bf16_bits_to_f32(bits)
    assert np.array_equal(inputs.to_bf16_bits(as_f32), bits)               # lossless widening
    assert np.max(np.abs(as_f32 - xf) / np.abs(xf)) <= 2.0 ** -8           # one bf16 rounding
    np.testing.assert_array_equal(oracle.aggregate(row_ptr, col, "gin", bits),
                                  oracle.aggregate(row_ptr, col, "gin", as_f32.astype(np.float64)))
    # round-to-nearest-even on exact ties: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
    assert inputs.bf16_bits_to_f32(inputs.to_bf16_bits(ties)).tolist() == [1.0, 1.0 + 2.0 ** -6]


# ----------------------------------------------------------------------------- partitioned
@pytest.mark.parametrize("parts", [1, 2, 3, 4, 8])
def test_partition_consistency(parts):
    """Concatenating every share's output reproduces the single-partition result, so the
    weights use whole-graph degrees and the halo lookup returns the right rows."""
    n, dim = 1000, 9
    rng = RNG(71)
    row_ptr, col = inputs.rmat_graph(10, 6000, 0.57, 0.19, 0.19, 0.05, rng)
    n = row_ptr.size - 1
    x = rng.standard_normal((n, dim)).astype(np.float32)
    bounds = inputs.equal_node_bounds(n, parts)
    for mode in ("gcn", "gin"):
        whole = oracle.aggregate(row_ptr, col, mode, x, eps=0.1)
        pieces = []
        for p in range(parts):
            part = oracle.build_partition(row_ptr, col, parts, p, bounds)
            lb, ub = part["lb"], part["ub"]
            pieces.append(oracle.aggregate(row_ptr, col, mode, x[lb:ub], lb=lb, ub=ub,
                                           x_halo=x[part["halo_gid"]], halo_gid=part["halo_gid"],
                                           eps=0.1))
        np.testing.assert_allclose(np.concatenate(pieces), whole, rtol=1e-12, atol=1e-13)


def test_row_selection_returns_the_same_rows():
    row_ptr, col = small_graph(600, 12, 81)
    x = RNG(82).standard_normal((600, 5)).astype(np.float32)
    full = oracle.aggregate(row_ptr, col, "gcn", x[100:400], lb=100, ub=400,
                            x_halo=x, halo_gid=np.arange(600, dtype=np.int32))
    rows = np.array([0, 7, 299, 150, 7])
    sel = oracle.aggregate(row_ptr, col, "gcn", x[100:400], lb=100, ub=400,
                           x_halo=x, halo_gid=np.arange(600, dtype=np.int32), rows=rows)
    np.testing.assert_array_equal(sel, full[rows])


def test_missing_halo_row_is_an_error():
    row_ptr, col = inputs.csr_from_adjacency_lists([[1], [0]])
    with pytest.raises(ValueError):
        oracle.aggregate(row_ptr, col, "gin", np.ones((1, 1)), lb=0, ub=1)


# ----------------------------------------------------------------------------- partition build
def test_partition_fixture_written_by_hand():
    fx = json.load(open(os.path.join(GOLDEN, "tiny_partition.json")))
    row_ptr, col = inputs.csr_from_adjacency_lists(fx["adjacency"])
    bounds = np.array(fx["bounds"])
    for p, want in enumerate(fx["parts"]):
        got = oracle.build_partition(row_ptr, col, 2, p, bounds)
        for key in ("local_row_ptr", "local_col", "remote_row_ptr", "remote_col", "halo_gid",
                    "halo_peer_ptr", "deg_own", "deg_halo"):
            assert got[key].tolist() == want[key], (p, key)
        for kind in ("local", "remote"):
            row, start, end = oracle.neighbor_groups(got[f"{kind}_row_ptr"], 2)
            g = want[f"groups_ps2_{kind}"]
            assert (row.tolist(), start.tolist(), end.tolist()) == (g["row"], g["start"], g["end"])


@pytest.mark.parametrize("parts,seed", [(1, 1), (2, 2), (4, 3), (7, 4)])
def test_partition_round_trip_and_invariants(parts, seed):
    rng = RNG(seed)
    row_ptr, col = inputs.rmat_graph(11, 20000, 0.57, 0.19, 0.19, 0.05, rng)
    n = row_ptr.size - 1
    cuts = np.sort(rng.integers(0, n + 1, parts - 1))
    bounds = np.concatenate([[0], cuts, [n]]).astype(np.int64)     # uneven, may hold empty ranges
    total_local = total_remote = 0
    for p in range(parts):
        part = oracle.build_partition(row_ptr, col, parts, p, bounds)
        lb, ub, hg = part["lb"], part["ub"], part["halo_gid"]
        assert np.all(np.diff(hg) > 0)                              # strictly increasing
        assert not np.any((hg >= lb) & (hg < ub))                   # disjoint from the owned range
        nl, nr = part["local_col"].size, part["remote_col"].size
        assert nl + nr == row_ptr[ub] - row_ptr[lb]
        total_local += nl
        total_remote += nr
        if parts == 1:
            assert nr == 0 and hg.size == 0
        for v in range(ub - lb):
            loc = part["local_col"][part["local_row_ptr"][v]:part["local_row_ptr"][v + 1]] + lb
            rem = hg[part["remote_col"][part["remote_row_ptr"][v]:part["remote_row_ptr"][v + 1]]]
            merged = np.sort(np.concatenate([loc, rem]))
            assert np.array_equal(merged, col[row_ptr[lb + v]:row_ptr[lb + v + 1]])
            assert np.all(np.diff(loc) > 0) and np.all(np.diff(rem) > 0)   # order kept
        assert np.array_equal(part["deg_own"], np.diff(row_ptr)[lb:ub])
        assert np.array_equal(part["deg_halo"], np.diff(row_ptr)[hg])
        hp = part["halo_peer_ptr"]
        assert hp[0] == 0 and hp[-1] == hg.size and hp[p] == hp[p + 1]
        for q in range(parts):
            span = hg[hp[q]:hp[q + 1]]
            assert np.all((span >= bounds[q]) & (span < bounds[q + 1]))
    assert total_local + total_remote == row_ptr[-1]


# ----------------------------------------------------------------------------- neighbour groups
@pytest.mark.parametrize("ps", [1, 2, 3, 16, 32, 10 ** 6])
def test_neighbour_groups_tile_every_row(ps):
    row_ptr, _ = small_graph(700, 11, 91)
    row, start, end = oracle.neighbor_groups(row_ptr, ps)
    deg = np.diff(row_ptr)
    assert row.size == int(np.sum(-(-deg // ps)))
    assert start[0] == 0 and end[-1] == row_ptr[-1]
    assert np.array_equal(start[1:], end[:-1])                      # no gap, no overlap
    assert np.all(end - start <= ps) and np.all(end > start)
    assert np.all(start >= row_ptr[row]) and np.all(end <= row_ptr[row + 1])   # inside one row
    if ps >= deg.max():                                             # "without neighbour partitioning"
        assert np.array_equal(row, np.nonzero(deg)[0])


# ----------------------------------------------------------------------------- update
def test_update_hand_example():
    a = np.array([[1.0, 2.0], [-3.0, 0.5]])
    w = np.array([[2.0, -1.0, 0.0], [0.5, 4.0, -2.0]])
    b = np.array([0.25, 0.0, 1.0])
    out = oracle.update(a, w, b, "none")
    assert out.tolist() == [[3.25, 7.0, -3.0], [-5.5, 5.0, 0.0]]
    assert oracle.update(a, w, b, "relu").tolist() == [[3.25, 7.0, 0.0], [0.0, 5.0, 0.0]]


def test_update_matches_numpy_matmul_and_is_not_transposed():
    rng = RNG(101)
    a, w, b = rng.standard_normal((57, 13)), rng.standard_normal((13, 29)), rng.standard_normal(29)
    np.testing.assert_allclose(oracle.update(a, w, b), a @ w + b, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.update(a, w), a @ w, rtol=1e-12, atol=1e-13)
    relu = oracle.update(a, w, b, "relu")
    assert relu.min() >= 0.0
    np.testing.assert_allclose(relu, np.maximum(a @ w + b, 0.0), rtol=1e-12, atol=1e-13)
    np.testing.assert_array_equal(oracle.update(a, np.eye(13)), a)
    # bf16 weights are widened exactly
    wb = inputs.to_bf16_bits(w.astype(np.float32))
    np.testing.assert_allclose(oracle.update(a, wb), a @ inputs.bf16_bits_to_f32(wb).astype(np.float64),
                               rtol=1e-12, atol=1e-13)


def test_layer_forward_is_aggregate_then_update():
    n = 150
    row_ptr, col = small_graph(n, 6, 111)
    rng = RNG(112)
    x, w1, w2 = rng.standard_normal((n, 10)), rng.standard_normal((10, 12)), rng.standard_normal((12, 4))
    gcn = oracle.layer_forward(row_ptr, col, "gcn", x, [w1], ["relu"])
    np.testing.assert_allclose(gcn, np.maximum(dense_gcn_matrix(row_ptr, col, n) @ x @ w1, 0.0),
                               rtol=1e-11, atol=1e-12)
    gin = oracle.layer_forward(row_ptr, col, "gin", x, [w1, w2], ["relu", "none"], eps=0.2)
    agg = (dense_adj(row_ptr, col, n) + 1.2 * np.eye(n)) @ x
    np.testing.assert_allclose(gin, np.maximum(agg @ w1, 0.0) @ w2, rtol=1e-11, atol=1e-11)


# ----------------------------------------------------------------------------- Algorithm 1
@pytest.mark.parametrize("parts", [1, 2, 4, 8, 13])
def test_edge_balanced_split_contract(parts):
    """Pins the stated contract (chunks balanced by edge count).  The pseudo-code the
    paper prints does not terminate as written, so parity with it is unpinned."""
    rng = RNG(121)
    row_ptr, _ = inputs.rmat_graph(12, 60000, 0.57, 0.19, 0.19, 0.05, rng)
    n, e = row_ptr.size - 1, int(row_ptr[-1])
    bounds = oracle.split_edge_balanced(row_ptr, parts)
    assert bounds[0] == 0 and bounds[-1] == n and np.all(np.diff(bounds) >= 0)
    per = -(-e // parts)
    maxdeg = int(np.diff(row_ptr).max())
    # independent statement: smallest index at or after the previous cut reaching the target
    last = 0
    for s in range(1, parts):
        target = min(row_ptr[last] + per, e)
        want = last + int(np.searchsorted(row_ptr[last:], target, side="left"))
        assert bounds[s] == want
        last = want
    chunk = row_ptr[bounds[1:]] - row_ptr[bounds[:-1]]
    assert chunk.sum() == e
    for s in range(parts - 1):
        if row_ptr[bounds[s]] + per <= e:
            assert per <= chunk[s] < per + maxdeg


def test_oracle_reports_thread_count():
    assert oracle.num_threads() >= 1


def test_update_softmax_pins():
    """Row softmax of the Update (section 7: Z = softmax(A-hat ReLU(A-hat X W0) W1)): the plain
    definition exp(z_j) / sum_k exp(z_k) evaluated directly, the library routine, the two-class
    closed form, and the properties a dropped normalisation, a column-wise instead of row-wise sum or
    a missing bias would break."""
    import scipy.special
    rng = np.random.default_rng(21)
    a = rng.standard_normal((37, 9))
    w = rng.standard_normal((9, 5))
    b = rng.standard_normal(5)
    z = a @ w + b
    got = oracle.update(a, w, b, "softmax")
    plain = np.exp(z) / np.exp(z).sum(axis=1, keepdims=True)
    np.testing.assert_allclose(got, plain, rtol=1e-13, atol=0)
    np.testing.assert_allclose(got, scipy.special.softmax(z, axis=1), rtol=1e-13, atol=0)
    np.testing.assert_allclose(got.sum(axis=1), 1.0, rtol=1e-14)
    assert np.all(got > 0) and np.array_equal(np.argmax(got, axis=1), np.argmax(z, axis=1))
    # adding a constant to every logit of a row changes nothing; logits of 800 do not overflow
    np.testing.assert_allclose(oracle.update(a, w, b + 800.0, "softmax"), got, rtol=1e-10)
    # two classes: softmax(z)_0 = 1 / (1 + exp(z_1 - z_0))
    z2 = oracle.update(a, w[:, :2], b[:2], "none")
    np.testing.assert_allclose(oracle.update(a, w[:, :2], b[:2], "softmax")[:, 0], 1.0 / (1.0 + np.exp(z2[:, 1] - z2[:, 0])), rtol=1e-13)
    # hand value: softmax([0, ln 2, ln 5]) = [1, 2, 5] / 8
    np.testing.assert_allclose(oracle.update(np.array([[1.0]]), np.array([[0.0, np.log(2.0), np.log(5.0)]]), None, "softmax"),
                               [[0.125, 0.25, 0.625]], rtol=1e-15)


def test_bag_sum_pins():
    """Embedding-bag sum (section 8.3: embedding lookup followed by element-wise addition): the hand
    value, numpy's segmented reduction, the equivalence with a GIN aggregation without the self term,
    and the cases a wrong offset or a dropped duplicate would break."""
    table = np.arange(12, dtype=np.float32).reshape(4, 3)
    got = oracle.bag_sum([0, 2, 2, 5], [0, 3, 1, 1, 2], table)
    assert got.tolist() == [[9.0, 11.0, 13.0], [0.0, 0.0, 0.0], [12.0, 15.0, 18.0]]      # rows 0+3; empty; rows 1+1+2
    rng = np.random.default_rng(13)
    t = rng.standard_normal((500, 7))
    sizes = rng.integers(0, 9, size=200)
    ptr = np.concatenate([[0], np.cumsum(sizes)])
    idx = rng.integers(0, 500, size=ptr[-1]).astype(np.int32)
    got = oracle.bag_sum(ptr, idx, t.astype(np.float32))
    want = np.zeros((200, 7))
    np.add.at(want, np.repeat(np.arange(200), sizes), t.astype(np.float32).astype(np.float64)[idx])
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)
    # a bag is a graph row whose neighbours are its lookups: GIN with eps = -1 has no self term left
    n = 200 + 500
    rows = [idx[ptr[b]:ptr[b + 1]] + 200 for b in range(200)] + [[] for _ in range(500)]
    row_ptr, col = inputs.csr_from_adjacency_lists([sorted(r) for r in rows])
    x = np.concatenate([rng.standard_normal((200, 7)), t]).astype(np.float32)
    agg = oracle.aggregate(row_ptr, col, "gin", x, eps=-1.0)[:200]
    np.testing.assert_allclose(agg, got, rtol=1e-12, atol=1e-12)
    # bf16 tables are read exactly
    tb = inputs.to_bf16_bits(t.astype(np.float32))
    np.testing.assert_allclose(oracle.bag_sum(ptr, idx, tb), oracle.bag_sum(ptr, idx, inputs.bf16_bits_to_f32(tb)), rtol=0, atol=0)
