"""Pins for the CPU oracle (no GPU): every oracle function is checked against
something other than itself -- closed forms of the carry-save array
multiplier, dense linear algebra on tiny graphs, library routines on special
cases, hand-evaluated sets, and invariants of the definitions."""
import numpy as np
import pytest

import oracle
import workloads as wl
from conftest import golden_path


def _csr(n, batch=1, flags=oracle.DEFAULT_FLAGS):
    aig = wl.csa_multiplier_aig(n)
    return aig, oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, batch, flags)


def _dense_from_aig(aig, self_loops=True):
    """Binary symmetric adjacency written straight from the fanin records."""
    n1 = aig.num_nodes
    A = np.zeros((n1, n1))
    for v in range(n1):
        if self_loops:
            A[v, v] = 1.0
        for lit in (aig.fanin0[v], aig.fanin1[v]):
            if lit >= 0:
                A[v, lit >> 1] = 1.0
                A[lit >> 1, v] = 1.0
    return A


# ---------------------------------------------------------------- adjacency
@pytest.mark.parametrize("n", [6, 8, 17, 32, 64])
def test_degree_histogram_closed_form(n):
    """Without the self-loop: 2n POs of degree 1, 2n^2-n nodes of degree 3,
    6n^2-11n of degree 4, n of degree 5, 2n PIs of degree n."""
    aig, (rowptr, col, val, pol) = _csr(n)
    deg = np.diff(rowptr) - 1
    hist = np.bincount(deg)
    want = {1: 2 * n, 3: 2 * n * n - n, 4: 6 * n * n - 11 * n, 5: n}
    want[n] = want.get(n, 0) + 2 * n
    for d in range(len(hist)):
        assert hist[d] == want.get(d, 0), (n, d)
    assert (deg[:2 * n] == n).all() and (deg[-2 * n:] == 1).all()
    # unique undirected edges 2*AND + PO, stored entries 2U + N
    U = 16 * n * n - 20 * n
    assert rowptr[-1] == 2 * U + aig.num_nodes == 40 * n * n - 47 * n


@pytest.mark.parametrize("n", [2, 3, 5, 16])
def test_csr_structure(n):
    aig, (rowptr, col, val, pol) = _csr(n)
    n1 = aig.num_nodes
    A = _dense_from_aig(aig)
    rows = np.repeat(np.arange(n1), np.diff(rowptr))
    B = np.zeros_like(A)
    B[rows, col] = 1.0
    assert np.array_equal(A, B)                       # same pattern, hence symmetric with self-loops
    assert len(col) == int(A.sum())                   # no duplicate entries
    for i in range(n1):                               # strictly ascending columns
        c = col[rowptr[i]:rowptr[i + 1]]
        assert (np.diff(c) > 0).all()
    deg = np.diff(rowptr).astype(np.float32)
    assert np.array_equal(val, (np.float32(1.0) / deg)[rows])    # correctly rounded fp32 1/deg
    # polarity byte: bit2 self-loop; bit1 the column drives the row; bit0 inverted record
    assert np.array_equal((pol & 4) != 0, rows == col)
    assert np.array_equal((pol & 2) != 0, col < rows)            # drivers precede their node
    for v in range(n1):
        for lit in {int(aig.fanin0[v]), int(aig.fanin1[v])} - {-1}:
            u = lit >> 1
            p = rowptr[v] + np.searchsorted(col[rowptr[v]:rowptr[v + 1]], u)
            q = rowptr[u] + np.searchsorted(col[rowptr[u]:rowptr[u + 1]], v)
            assert pol[p] & 1 == lit & 1 and pol[q] & 1 == lit & 1
    inverted_entries = int(((pol & 1) != 0).sum())
    pairs = {(int(l) >> 1, v, int(l) & 1) for v in range(n1) for l in (aig.fanin0[v], aig.fanin1[v]) if l >= 0}
    assert inverted_entries == 2 * sum(1 for _, _, inv in pairs if inv)


def test_csr_flags_and_batch():
    aig, full = _csr(4)
    n1 = aig.num_nodes
    # directed, no self-loops, unit weights: row v holds exactly its distinct drivers
    rowptr, col, val, pol = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, 1, 0)
    for v in range(n1):
        want = sorted({int(l) >> 1 for l in (aig.fanin0[v], aig.fanin1[v]) if l >= 0})
        assert list(col[rowptr[v]:rowptr[v + 1]]) == want
    assert (val == 1.0).all()
    # batch = block diagonal copies
    rp3, c3, v3, p3 = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, 3, oracle.DEFAULT_FLAGS)
    rp1, c1, v1, p1 = full
    nnz1 = rp1[-1]
    for c in range(3):
        assert np.array_equal(rp3[c * n1:(c + 1) * n1 + 1] - c * nnz1, rp1)
        assert np.array_equal(c3[c * nnz1:(c + 1) * nnz1], c1 + c * n1)
        assert np.array_equal(v3[c * nnz1:(c + 1) * nnz1], v1)
        assert np.array_equal(p3[c * nnz1:(c + 1) * nnz1], p1)


# --------------------------------------------------------------------- SpMM
@pytest.mark.parametrize("n", [2, 3])
def test_spmm_equals_dense_product(n):
    """The only multipliers with <= 64 nodes (18 and 51): dense D^-1 (A+I) X."""
    aig, (rowptr, col, val, pol) = _csr(n)
    A = _dense_from_aig(aig)
    w = (np.float32(1.0) / A.sum(axis=1).astype(np.float32)).astype(np.float64)
    X = wl.uniform_features_numpy(11, 0, aig.num_nodes, 12)
    want = (w[:, None] * A) @ X.astype(np.float64)
    want_abs = (w[:, None] * A) @ np.abs(X.astype(np.float64))
    Y, S = oracle.spmm_f64(rowptr, col, val, X)
    assert np.allclose(Y, want, rtol=0, atol=1e-15)
    assert np.allclose(S, want_abs, rtol=0, atol=1e-15)
    # unit vectors pick out columns of A_hat
    E = np.eye(aig.num_nodes, dtype=np.float32)
    Ycols, _ = oracle.spmm_f64(rowptr, col, val, E)
    assert np.array_equal(Ycols, w[:, None] * A)
    assert np.array_equal(oracle.dense_adjacency(rowptr, col, val), w[:, None] * A)


@pytest.mark.parametrize("n,batch", [(8, 1), (32, 2)])
def test_spmm_ones_gives_row_sums(n, batch):
    aig, (rowptr, col, val, pol) = _csr(n, batch)
    N = aig.num_nodes * batch
    ones = np.ones((N, 4), dtype=np.float32)
    Y, S = oracle.spmm_f64(rowptr, col, val, ones)
    deg = np.diff(rowptr)
    want = deg * (np.float32(1.0) / deg.astype(np.float32)).astype(np.float64)
    assert np.allclose(Y, want[:, None], rtol=0, atol=1e-15) and np.array_equal(Y, S)
    assert np.abs(Y - 1.0).max() < 2.0 ** -23
    # without normalisation the row sum is the degree, exactly
    rowptr, col, val, pol = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, batch,
                                             oracle.SYMMETRIC | oracle.SELF_LOOPS)
    Y, _ = oracle.spmm_f64(rowptr, col, val, ones)
    assert np.array_equal(Y, np.repeat(deg.astype(np.float64)[:, None], 4, axis=1))


def test_spmm_matches_scipy_on_stress_graph():
    import scipy.sparse as sp

    g = wl.stress_graph(5, 1 << 14, window=256, dmin=64, dmax=2048)
    X = wl.uniform_features_numpy(5, 0, g.n, 8)
    Y, S = oracle.spmm_f64(g.rowptr, g.col, g.val, X)
    M = sp.csr_matrix((g.val.astype(np.float64), g.col, g.rowptr), shape=(g.n, g.n))
    assert np.allclose(Y, M @ X.astype(np.float64), rtol=0, atol=1e-12)
    assert np.allclose(S, M @ np.abs(X.astype(np.float64)), rtol=0, atol=1e-12)


# --------------------------------------------------------------------- plan
@pytest.mark.parametrize("n,batch,T", [(8, 1, 7), (8, 2, 9), (32, 1, 32), (32, 1, 33), (64, 1, 12)])
def test_plan_on_multipliers(n, batch, T):
    aig, (rowptr, col, val, pol) = _csr(n, batch)
    N = aig.num_nodes * batch
    pl = oracle.plan(rowptr, T)
    deg = np.diff(rowptr)
    # only the 2n primary inputs of each copy (row length n+1) are high-degree for 7 <= T <= n+1
    assert len(pl["hd_rows"]) == 2 * n * batch
    want_hd = np.concatenate([np.arange(2 * n) + c * aig.num_nodes for c in range(batch)])
    assert np.array_equal(pl["hd_rows"], want_hd)
    assert np.array_equal(pl["row_class"], (deg >= T).astype(np.uint8))
    assert np.array_equal(np.sort(np.concatenate([pl["hd_rows"], pl["ld_rows"]])), np.arange(N))
    assert (np.diff(pl["ld_rows"]) > 0).all()
    # stable ascending-degree order == numpy's stable argsort of the LD degrees
    ld = pl["ld_rows"]
    assert np.array_equal(pl["ld_rows_by_degree"], ld[np.argsort(deg[ld], kind="stable")])
    hist = np.bincount(deg[ld], minlength=T)[:T]
    assert np.array_equal(pl["ld_deg_offsets"], np.concatenate([[0], np.cumsum(hist)]))


def test_plan_thresholds_on_stress_graph():
    g = wl.stress_graph(6, 1 << 15, window=256, dmin=64, dmax=1024)
    deg = np.diff(g.rowptr)
    prev = None
    for T in (16, 32, 64, 128):
        pl = oracle.plan(g.rowptr, T)
        assert np.array_equal(pl["hd_rows"], np.nonzero(deg >= T)[0])
        assert np.array_equal(pl["ld_rows"], np.nonzero(deg < T)[0])
        if prev is not None:
            assert len(pl["hd_rows"]) <= prev
        prev = len(pl["hd_rows"])
    with pytest.raises(ValueError):
        oracle.plan(g.rowptr, 0)


# ---------------------------------------------------------------- partition
def _parse_hand_cases():
    cases, cur = [], None
    for line in open(golden_path("regrow_hand_cases.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "case":
            cur = dict(name=t[1], n=int(t[2]), parts=[])
            cases.append(cur)
        elif t[0] == "edges":
            cur["edges"] = [tuple(int(x) for x in e.split("-")) for e in t[1:]]
        elif t[0] == "partof":
            cur["partof"] = np.array([int(x) for x in t[1:]], dtype=np.int32)
        elif t[0] == "part":
            kv = dict(x.split("=") for x in t[2:])
            cur["parts"].append(dict(p=int(t[1]), S=[int(x) for x in kv["S"].split(",")],
                                     B=[int(x) for x in kv["B"].split(",")],
                                     crossing=int(kv["crossing"]), kept=int(kv["kept"])))
    return cases


def _csr_from_edges(n, edges, self_loops):
    rows = [set() for _ in range(n)]
    for u, v in edges:
        rows[u].add(v)
        rows[v].add(u)
    if self_loops:
        for v in range(n):
            rows[v].add(v)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    col = []
    for v in range(n):
        col += sorted(rows[v])
        rowptr[v + 1] = len(col)
    col = np.array(col, dtype=np.int32)
    val = (np.float32(1) / np.diff(rowptr).astype(np.float32))[np.repeat(np.arange(n), np.diff(rowptr))]
    return rowptr, col, val.astype(np.float32)


@pytest.mark.parametrize("self_loops", [False, True])
def test_regrow_hand_cases(self_loops):
    for case in _parse_hand_cases():
        rowptr, col, val = _csr_from_edges(case["n"], case["edges"], self_loops)
        for want in case["parts"]:
            got = oracle.regrow_part(rowptr, col, val, case["partof"], want["p"])
            no, nh = got["n_owned"], got["n_halo"]
            assert list(got["global_id"][:no]) == want["S"], case["name"]
            assert list(got["global_id"][no:]) == want["B"], case["name"]
            assert got["n_crossing"] == want["crossing"]
            loops = (no + nh) if self_loops else 0
            assert got["rowptr"][-1] == 2 * want["kept"] + loops
            # without re-growth only E[S_p] survives
            bare = oracle.regrow_part(rowptr, col, val, case["partof"], want["p"], flags=0)
            assert bare["n_halo"] == 0 and list(bare["global_id"]) == want["S"]
            assert bare["rowptr"][-1] == 2 * (want["kept"] - want["crossing"]) + (no if self_loops else 0)


def test_partition_rule_closed_form():
    """part(v) = min(P-1, floor((v mod n1) P / n1)): a hand-evaluated case and the slice sizes
    ceil((p+1) n1 / P) - ceil(p n1 / P) that follow from the floor."""
    assert list(oracle.part_of_default(10, 10, 3)) == [0, 0, 0, 0, 1, 1, 1, 2, 2, 2]
    assert list(oracle.part_of_default(8, 4, 2)) == [0, 0, 1, 1, 0, 0, 1, 1]
    for n1, P, copies in ((51, 4, 1), (1000, 7, 3), (18, 16, 2), (522496, 16, 1)):
        part = oracle.part_of_default(n1 * copies, n1, P)
        ceil = lambda a, b: -(-a // b)
        want = [ceil((p + 1) * n1, P) - ceil(p * n1, P) for p in range(P)]
        assert list(np.bincount(part, minlength=P)) == [w * copies for w in want]
        assert part[0] == 0 and part[n1 - 1] == P - 1 and (np.diff(part[:n1]) >= 0).all()


def _sets_bruteforce(rowptr, col, part_of, p):
    """Eq. (1)-(2) with Python sets."""
    n = len(rowptr) - 1
    nbr = lambda u: {int(c) for c in col[rowptr[u]:rowptr[u + 1]] if c != u}
    S = {v for v in range(n) if part_of[v] == p}
    N = set().union(*[nbr(u) for u in S]) if S else set()
    B = N - S
    E = {(i, int(j)) for i in range(n) for j in col[rowptr[i]:rowptr[i + 1]]}
    C = {(i, j) for (i, j) in E if (i in S and j in B) or (i in B and j in S)}
    ES = {(i, j) for (i, j) in E if i in S and j in S}
    halo_loops = {(u, u) for u in B if (u, u) in E}
    return S, B, C, ES | C | halo_loops


@pytest.mark.parametrize("n,P", [(2, 2), (3, 2), (3, 3), (4, 3), (8, 5)])
def test_regrow_on_multipliers(n, P):
    aig, (rowptr, col, val, pol) = _csr(n, batch=2)
    N = 2 * aig.num_nodes
    part_of = oracle.part_of_default(N, aig.num_nodes, P)
    # contiguous slices of each copy, every part non-empty, non-decreasing inside a copy
    assert set(part_of) == set(range(P))
    assert (np.diff(part_of[:aig.num_nodes]) >= 0).all()
    assert np.array_equal(part_of[:aig.num_nodes], part_of[aig.num_nodes:])
    X = wl.uniform_features_numpy(2, 0, N, 8)
    Yfull, _ = oracle.spmm_f64(rowptr, col, val, X)
    Yback = np.full_like(Yfull, np.nan)
    total_cross, seen = 0, np.zeros(N, dtype=int)
    for p in range(P):
        got = oracle.regrow_part(rowptr, col, val, part_of, p)
        S, B, C, Eplus = _sets_bruteforce(rowptr, col, part_of, p)
        no, gid = got["n_owned"], got["global_id"]
        assert list(gid[:no]) == sorted(S) and list(gid[no:]) == sorted(B)
        assert got["n_crossing"] == len(C) // 2
        sub_rows = np.repeat(np.arange(len(gid)), np.diff(got["rowptr"]))
        assert {(int(gid[i]), int(gid[j])) for i, j in zip(sub_rows, got["col"])} == Eplus
        assert len(got["col"]) == len(Eplus)
        for li in range(len(gid)):
            c = got["col"][got["rowptr"][li]:got["rowptr"][li + 1]]
            assert (np.diff(c) > 0).all()
        # owned rows keep their whole neighbourhood and hence their global weight
        for li in range(no):
            g = gid[li]
            assert sorted(gid[got["col"][got["rowptr"][li]:got["rowptr"][li + 1]]]) == \
                list(col[rowptr[g]:rowptr[g + 1]])
        deg_local = np.diff(got["rowptr"]).astype(np.float32)
        assert np.array_equal(got["val"], (np.float32(1) / deg_local)[sub_rows])
        seen[gid[:no]] += 1
        total_cross += got["n_crossing"]
        Yp, _ = oracle.spmm_f64(got["rowptr"], got["col"], got["val"], X[gid])
        Yback[gid[:no]] = Yp[:no]
    assert (seen == 1).all()
    cut = sum(1 for i in range(N) for j in col[rowptr[i]:rowptr[i + 1]] if i < j and part_of[i] != part_of[j])
    assert total_cross == 2 * cut
    assert np.allclose(Yback, Yfull, rtol=0, atol=1e-15)


def test_regrow_one_way_edges_and_weight_modes():
    """Directed pattern: 0->1, 1->2, 2->0, 3->0 (+ self-loops), parts {0,1} | {2,3}."""
    rowptr = np.array([0, 2, 4, 6, 8], dtype=np.int64)
    col = np.array([0, 1, 1, 2, 0, 2, 0, 3], dtype=np.int32)
    val = np.array([.5, .25, 1., 2., 3., 4., 5., 6.], dtype=np.float32)
    part_of = np.array([0, 0, 1, 1], dtype=np.int32)
    g0 = oracle.regrow_part(rowptr, col, val, part_of, 0, weight_mode=2)
    # N(S_0) = {1, 2}; B_0 = {2}; node 3 points into S_0 but is not a neighbour of S_0
    assert list(g0["global_id"]) == [0, 1, 2] and g0["n_crossing"] == 2     # {1,2} and {2,0}
    assert list(g0["rowptr"]) == [0, 2, 4, 6]
    assert list(g0["col"]) == [0, 1, 1, 2, 0, 2] and list(g0["val"]) == [.5, .25, 1., 2., 3., 4.]
    g1 = oracle.regrow_part(rowptr, col, val, part_of, 1, weight_mode=0)
    assert list(g1["global_id"]) == [2, 3, 0] and g1["n_crossing"] == 2     # {2,0} and {3,0}
    assert list(g1["col"]) == [0, 2, 1, 2, 2] and (g1["val"] == 1).all()


def test_sage_forward_reduces_to_spmm():
    aig, (rowptr, col, val, pol) = _csr(4)
    N, F = aig.num_nodes, 8
    X = np.abs(wl.uniform_features_numpy(9, 0, N, F))
    I, Z, z = np.eye(F, dtype=np.float32), np.zeros((F, F), dtype=np.float32), np.zeros(F, dtype=np.float32)
    H1, H2 = oracle.sage_forward_f64(rowptr, col, val, X, I, Z, z, I, Z, z)
    Y1, _ = oracle.spmm_f64(rowptr, col, val, X)
    Y2, _ = oracle.spmm_f64(rowptr, col, val, Y1.astype(np.float32))
    assert np.array_equal(H1, Y1.astype(np.float32)) and np.allclose(H2, Y2, atol=1e-15)
    H1s, H2s = oracle.sage_forward_f64(rowptr, col, val, X, Z, I, z, Z, I, z + 1)
    assert np.array_equal(H1s, X) and np.allclose(H2s, X.astype(np.float64) + 1)


def _layer_inputs(n, F, seed):
    aig, (rowptr, col, val, pol) = _csr(n)
    N = aig.num_nodes
    A = _dense_from_aig(aig)
    A_hat = (np.float32(1.0) / A.sum(axis=1).astype(np.float32)).astype(np.float64)[:, None] * A
    X = wl.uniform_features_numpy(seed, 0, N, F)
    Wn = wl.uniform_features_numpy(seed + 1, 0, F, F) * np.float32(0.125)
    Ws = wl.uniform_features_numpy(seed + 2, 0, F, F) * np.float32(0.125)
    b = wl.uniform_features_numpy(seed + 3, 0, 1, F)[0] * np.float32(0.125)
    return (rowptr, col, val), A_hat, X, Wn, Ws, b


@pytest.mark.parametrize("n", [2, 3])
def test_sage_layer_equals_dense_layer(n):
    """Section "GNN and Edge Re-growth After Partition": a GraphSAGE-mean layer aggregates, then transforms.
    On the 18- and 51-node multipliers the layer is checked against the dense adjacency written from the
    fanin records, with the products associated the other way round (A_hat (X Wn) instead of (A_hat X) Wn),
    element by element in explicit loops for the 18-node case."""
    csr, A_hat, X, Wn, Ws, b, = _layer_inputs(n, 8, 41)
    X64, Wn64, Ws64, b64 = (np.asarray(a, dtype=np.float64) for a in (X, Wn, Ws, b))
    pre = A_hat @ (X64 @ Wn64) + X64 @ Ws64 + b64
    assert (pre < -1e-3).any() and (pre > 1e-3).any()          # ReLU has something to clip and something to keep
    for relu in (False, True):
        H, A, S = oracle.sage_layer_f64(*csr, X, Wn, Ws, b, relu)
        want = np.maximum(pre, 0.0) if relu else pre
        assert np.allclose(H, want, rtol=0, atol=1e-14)
        assert np.allclose(A, A_hat @ X64, rtol=0, atol=1e-15)
        assert np.allclose(S, A_hat @ np.abs(X64), rtol=0, atol=1e-15)
    H0, _, _ = oracle.sage_layer_f64(*csr, X, Wn, Ws, None, False)            # bias off = bias of zeros
    assert np.allclose(H0, pre - b64, rtol=0, atol=1e-14)
    if n == 2:
        N, F = X.shape
        H, _, _ = oracle.sage_layer_f64(*csr, X, Wn, Ws, b, True)
        for i in range(N):
            for o in range(F):
                acc = float(b[o])
                for k in range(F):
                    acc += sum(A_hat[i, j] * float(X[j, k]) for j in range(N)) * float(Wn[k, o])
                    acc += float(X[i, k]) * float(Ws[k, o])
                assert abs(H[i, o] - max(acc, 0.0)) <= 1e-14


def test_sage_layer_special_cases():
    """Wn = I, Ws = 0: the layer is the aggregation; Wn = 0, Ws = I: the layer is the identity on X (the self
    term); X = 1 with Wn = -I, Ws = I/4 and a bias that alternates between 1 and 1/2: every row aggregates to
    1 (row weights sum to 1 within 2^-23), so the layer gives 1/4 and -1/4, and ReLU, which acts after the
    bias, turns the second into exactly 0."""
    csr, A_hat, X, _, _, b = _layer_inputs(3, 6, 51)
    F = X.shape[1]
    I, Z = np.eye(F, dtype=np.float32), np.zeros((F, F), dtype=np.float32)
    Y, S = oracle.spmm_f64(*csr, X)
    H, A, S2 = oracle.sage_layer_f64(*csr, X, I, Z, None, False)
    assert np.array_equal(H, Y) and np.array_equal(A, Y) and np.array_equal(S2, S)
    H, _, _ = oracle.sage_layer_f64(*csr, X, Z, I, None, False)
    assert np.array_equal(H, X.astype(np.float64))
    H, _, _ = oracle.sage_layer_f64(*csr, X, Z, I, b, False)
    assert np.array_equal(H, X.astype(np.float64) + b.astype(np.float64))
    ones = np.ones_like(X)
    alt = np.where(np.arange(F) % 2 == 0, 1.0, 0.5).astype(np.float32)
    H, _, _ = oracle.sage_layer_f64(*csr, ones, -I, np.float32(0.25) * I, alt, False)
    assert np.allclose(H, np.where(np.arange(F) % 2 == 0, 0.25, -0.25)[None, :], rtol=0, atol=2e-7)
    H, _, _ = oracle.sage_layer_f64(*csr, ones, -I, np.float32(0.25) * I, alt, True)
    assert np.allclose(H[:, 0::2], 0.25, rtol=0, atol=2e-7) and (H[:, 1::2] == 0.0).all()


@pytest.mark.parametrize("n", [2, 3])
def test_sage_layer_backward_data_equals_autograd_of_the_dense_layer(n):
    """The oracle's input gradient of the layer against automatic differentiation of the dense layer
    relu(A_hat X Wn + X Ws + b) (dense adjacency written from the fanin records; loss = <H, R> for a random R),
    against central differences of the oracle's own forward layer along random directions, and through the
    adjoint identity with the linear part of the forward layer."""
    import torch
    csr, A_hat, X, Wn, Ws, b = _layer_inputs(n, 8, 43)
    N, F = X.shape
    rng = np.random.default_rng(7 + n)
    R = rng.uniform(-1, 1, (N, F))
    A_t, Wn_t, Ws_t, b_t = (torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in (A_hat, Wn, Ws, b))
    X_t = torch.from_numpy(X.astype(np.float64)).requires_grad_(True)
    Z_t = A_t @ X_t @ Wn_t + X_t @ Ws_t + b_t
    (torch.relu(Z_t) * torch.from_numpy(R)).sum().backward()
    Z = Z_t.detach().numpy()
    assert (Z > 1e-3).any() and (Z < -1e-3).any()
    dZ = (R * (Z > 0)).astype(np.float32)                      # the oracle takes fp32 inputs, as the library does
    # gradient for exactly this dZ: the loss <relu(Z), R'> with R' = dZ where Z > 0 has it
    X_t.grad = None
    Z_t = A_t @ X_t @ Wn_t + X_t @ Ws_t + b_t
    (Z_t * torch.from_numpy(dZ.astype(np.float64))).sum().backward()
    want = X_t.grad.numpy()
    dX, T, S = oracle.sage_layer_backward_data_f64(*csr, dZ, Wn, Ws)
    assert np.allclose(dX, want, rtol=0, atol=1e-14)
    assert np.allclose(T, A_hat.T @ dZ.astype(np.float64), rtol=0, atol=1e-15)
    assert np.allclose(S, np.abs(A_hat.T) @ np.abs(dZ.astype(np.float64)), rtol=0, atol=1e-15)
    # central differences of the forward layer without activation (it is linear in X: exact up to rounding)
    for trial in range(3):
        V = rng.uniform(-1, 1, (N, F)).astype(np.float32)
        Hp, _, _ = oracle.sage_layer_f64(*csr, (X + V).astype(np.float32), Wn, Ws, b, False)
        Hm, _, _ = oracle.sage_layer_f64(*csr, (X - V).astype(np.float32), Wn, Ws, b, False)
        directional = 0.5 * float(((Hp - Hm) * dZ.astype(np.float64)).sum())
        assert abs(directional - float((dX * V.astype(np.float64)).sum())) <= 1e-5 * max(1.0, abs(directional))
    # adjoint identity with the forward layer's linear part J V = (A_hat V) Wn + V Ws
    V = rng.uniform(-1, 1, (N, F)).astype(np.float32)
    JV, _, _ = oracle.sage_layer_f64(*csr, V, Wn, Ws, None, False)
    assert abs(float((JV * dZ.astype(np.float64)).sum()) - float((dX * V.astype(np.float64)).sum())) <= 1e-12


@pytest.mark.parametrize("n", [2, 3])
def test_sage_layer_backward_weights_equals_autograd_of_the_dense_layer(n):
    """The oracle's weight gradients of the layer against automatic differentiation of the dense layer (dense
    adjacency written from the fanin records) for the same dZ, and through the identity that ties them to the
    forward layer's value for other weights."""
    import torch
    csr, A_hat, X, Wn, Ws, b = _layer_inputs(n, 8, 47)
    N, F = X.shape
    rng = np.random.default_rng(17 + n)
    dZ = (rng.uniform(-1, 1, (N, F)) * (rng.random((N, F)) < 0.6)).astype(np.float32)
    A_t, X_t, b_t = (torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in (A_hat, X, b))
    Wn_t = torch.from_numpy(Wn.astype(np.float64)).requires_grad_(True)
    Ws_t = torch.from_numpy(Ws.astype(np.float64)).requires_grad_(True)
    Z_t = A_t @ X_t @ Wn_t + X_t @ Ws_t + b_t
    (Z_t * torch.from_numpy(dZ.astype(np.float64))).sum().backward()
    dWn, dWs, Sn, Ss = oracle.sage_layer_backward_weights_f64(*csr, X, dZ)
    assert np.allclose(dWn, Wn_t.grad.numpy(), rtol=0, atol=1e-13)
    assert np.allclose(dWs, Ws_t.grad.numpy(), rtol=0, atol=1e-13)
    X64, dZ64 = X.astype(np.float64), dZ.astype(np.float64)
    assert np.allclose(Sn, (A_hat @ np.abs(X64)).T @ np.abs(dZ64), rtol=0, atol=1e-13)
    assert np.allclose(Ss, np.abs(X64).T @ np.abs(dZ64), rtol=0, atol=1e-13)
    V, U = (rng.uniform(-1, 1, (F, F)).astype(np.float32) for _ in range(2))
    H, _, _ = oracle.sage_layer_f64(*csr, X, V, U, None, False)
    lhs = float((dWn * V.astype(np.float64)).sum() + (dWs * U.astype(np.float64)).sum())
    assert abs(lhs - float((H * dZ64).sum())) <= 1e-12


def test_sage_forward_is_two_layers():
    """The two-layer forward is the layer applied twice: ReLU and rounding to fp32 between the layers, none after."""
    csr, _, X, W1n, W1s, b1 = _layer_inputs(4, 8, 61)
    _, _, _, W2n, W2s, b2 = _layer_inputs(4, 8, 71)
    H1, H2 = oracle.sage_forward_f64(*csr, X, W1n, W1s, b1, W2n, W2s, b2)
    L1, _, _ = oracle.sage_layer_f64(*csr, X, W1n, W1s, b1, True)
    assert H1.dtype == np.float32 and np.array_equal(H1, L1.astype(np.float32))
    L2, _, _ = oracle.sage_layer_f64(*csr, H1, W2n, W2s, b2, False)
    assert np.allclose(H2, L2, rtol=0, atol=1e-14) and (H2 < 0).any()


# ---------------------------------------------------------- transposed SpMM
@pytest.mark.parametrize("n,flags", [(2, 7), (3, 7), (3, 0), (3, 4)])
def test_transposed_spmm_equals_dense_transpose(n, flags):
    aig, (rowptr, col, val, pol) = _csr(n, 1, flags)
    A = oracle.dense_adjacency(rowptr, col, val)
    Gm = wl.uniform_features_numpy(21, 0, aig.num_nodes, 6)
    out, S = oracle.spmm_t_f64(rowptr, col, val, Gm)
    assert np.allclose(out, A.T @ Gm.astype(np.float64), rtol=0, atol=1e-15)
    assert np.allclose(S, np.abs(A.T) @ np.abs(Gm.astype(np.float64)), rtol=0, atol=1e-15)
    t_rowptr, t_col, t_val = oracle.csr_transpose(rowptr, col, val)
    assert np.array_equal(oracle.dense_adjacency(t_rowptr, t_col, t_val), A.T)
    for j in range(aig.num_nodes):
        assert (np.diff(t_col[t_rowptr[j]:t_rowptr[j + 1]]) > 0).all()
    # forward product with the transposed matrix adds the same terms in the same order
    fwd, fS = oracle.spmm_f64(t_rowptr, t_col, t_val, Gm)
    assert np.array_equal(fwd, out) and np.array_equal(fS, S)


def test_transposed_spmm_adjoint_identity():
    """<A x, y> = <x, A^T y> ties the transposed product to the (separately pinned) forward product."""
    for graph in ("aig", "stress"):
        if graph == "aig":
            aig, (rowptr, col, val, pol) = _csr(16, 2)
            n = 2 * aig.num_nodes
        else:
            g = wl.stress_graph(8, 1 << 13, window=128, dmin=64, dmax=1024)
            rowptr, col, val, n = g.rowptr, g.col, g.val, g.n
        x = wl.uniform_features_numpy(31, 0, n, 3)
        y = wl.uniform_features_numpy(32, 0, n, 3)
        Ax, _ = oracle.spmm_f64(rowptr, col, val, x)
        Aty, _ = oracle.spmm_t_f64(rowptr, col, val, y)
        lhs, rhs = float((Ax * y).sum()), float((x.astype(np.float64) * Aty).sum())
        assert abs(lhs - rhs) <= 1e-9 * max(1.0, abs(lhs))
        # transposing twice gives the matrix back
        t = oracle.csr_transpose(rowptr, col, val)
        tt = oracle.csr_transpose(*t)
        assert np.array_equal(tt[0], rowptr) and np.array_equal(tt[1], col) and np.array_equal(tt[2], val)
