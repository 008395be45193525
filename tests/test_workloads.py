"""Pins for the seeded input generators (no GPU).

The CSA generator is checked against what the paper prints (two-bit worked
example, node and edge counts of the 1024-bit batch-16 graph), against
integer multiplication through the oracle's bit-parallel AIG evaluation, and
against closed-form gate counts of a carry-save array multiplier.
"""
import random

import numpy as np
import pytest

import oracle
import workloads as wl
from conftest import golden_path


def _parse_example():
    labels, features, functions, product, nodes = {}, {}, {}, None, None
    for line in open(golden_path("two_bit_csa_example.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "nodes":
            nodes = int(t[1])
        elif t[0] == "label":
            labels[int(t[1])] = int(t[2])
        elif t[0] == "feature":
            features[int(t[1])] = t[2]
        elif t[0] == "function":
            functions[int(t[1])] = t[2]
        elif t[0] == "product":
            product = (t[1], t[2], t[3])
    return nodes, labels, features, functions, product


def _exhaustive_words(n_pi):
    """word k of PI i = bit i of the pattern index, for all 2^n_pi <= 64 patterns"""
    words = np.zeros(n_pi, dtype=np.uint64)
    for pat in range(1 << n_pi):
        for i in range(n_pi):
            if (pat >> i) & 1:
                words[i] |= np.uint64(1) << np.uint64(pat)
    return words


def test_two_bit_example_matches_paper():
    nodes, labels, features, functions, product = _parse_example()
    aig = wl.csa_multiplier_aig(2)
    assert aig.num_nodes == nodes
    # node classes: label 4 -> PI, 0 -> PO, 1/2/3 -> internal AND node; the generator's own
    # classes (XOR root, MAJ/carry root, plain AND) are the paper's ground-truth labels
    assert len(labels) == nodes
    for nid, lab in labels.items():
        want = wl.PI if lab == 4 else wl.PO if lab == 0 else wl.AND
        assert aig.type[nid - 1] == want, nid
        assert aig.label[nid - 1] == lab, nid
    # the generator-side encoding reproduces every printed feature vector (PI 1, AND 5 and 10, PO 15)
    enc = wl.paper_node_features(aig)
    for nid, bits in features.items():
        assert "".join(str(int(b)) for b in enc[nid - 1]) == bits, nid
    assert enc.shape == (nodes, 4) and set(np.unique(enc)) <= {0.0, 1.0}
    # feature bits: type bits 00 PI / 11 AND; polarity bits = (left inverted, right inverted)
    for nid, bits in features.items():
        v = nid - 1
        if aig.type[v] == wl.PI:
            assert bits == "0000"
        elif aig.type[v] == wl.PO:
            assert bits[0] == "0"
        else:
            assert bits[:2] == "11"
            assert bits[2:] == f"{aig.fanin0[v] & 1}{aig.fanin1[v] & 1}"
    # node functions over all 16 input patterns
    words = oracle.aig_simulate(aig.type, aig.fanin0, aig.fanin1, _exhaustive_words(4))
    a0, a1, b0, b1 = (int(w) for w in words[:4])
    env = dict(a0=a0, a1=a1, b0=b0, b1=b1)
    for nid, expr in functions.items():
        assert int(words[nid - 1]) & 0xFFFF == eval(expr, {}, env) & 0xFFFF, nid
    # the multiplication example of the text
    a, b, m = (int(s, 2) for s in product)
    pat = a | (b << 2)
    got = sum(((int(words[14 + k]) >> pat) & 1) << k for k in range(4))
    assert got == m == a * b


@pytest.mark.parametrize("n", [2, 3, 8, 32])
def test_label_counts_and_functions(n):
    """n half adders and n(n-2) full adders: one MAJ root per adder, one XOR root per half adder and two
    per full adder; every XOR root computes the xor of its grandparents' inputs, every MAJ root a carry."""
    aig = wl.csa_multiplier_aig(n)
    hist = np.bincount(aig.label, minlength=5)
    ha, fa = n, n * (n - 2)
    assert hist[4] == 2 * n and hist[0] == 2 * n
    assert hist[1] == ha + fa and hist[2] == ha + 2 * fa
    assert hist[3] == (8 * n * n - 11 * n) - hist[1] - hist[2]
    rng = np.random.default_rng(n)
    words = oracle.aig_simulate(aig.type, aig.fanin0, aig.fanin1, rng.integers(0, 2 ** 63, 2 * n, dtype=np.uint64))
    lit = lambda l: words[l >> 1] ^ (np.uint64(0xFFFFFFFFFFFFFFFF) if l & 1 else np.uint64(0))
    for v in np.nonzero(aig.label == 2)[0]:
        # xor root t = AND(!g, !h) with g = AND(x, y), h = AND(!x, !y)
        g = aig.fanin0[v] >> 1
        x, y = aig.fanin0[g], aig.fanin1[g]
        assert words[v] == lit(x) ^ lit(y)


def test_paper_node_and_edge_count():
    want = {}
    for line in open(golden_path("paper_graph_sizes.txt")):
        t = line.split()
        if t and not t[0].startswith("#"):
            want[t[0]] = int(t[1])
    aig = wl.csa_multiplier_aig(want["bits"])
    assert aig.num_nodes * want["batch"] == want["nodes"]
    records = int((aig.fanin0 >= 0).sum() + (aig.fanin1 >= 0).sum())
    assert records * want["batch"] == want["edges"]


@pytest.mark.parametrize("n", [2, 3, 4, 5, 7, 8, 16, 32, 64, 100])
def test_multiplier_function_equals_integer_product(n):
    aig = wl.csa_multiplier_aig(n)
    rng = random.Random(1000 + n)
    ops = [(rng.getrandbits(n), rng.getrandbits(n)) for _ in range(60)]
    ops += [(0, 0), ((1 << n) - 1, (1 << n) - 1), (1, (1 << n) - 1), (1 << (n - 1), 1 << (n - 1))]
    pi = np.zeros(2 * n, dtype=np.uint64)
    for pat, (a, b) in enumerate(ops):
        for i in range(n):
            if (a >> i) & 1:
                pi[i] |= np.uint64(1) << np.uint64(pat)
            if (b >> i) & 1:
                pi[n + i] |= np.uint64(1) << np.uint64(pat)
    words = oracle.aig_simulate(aig.type, aig.fanin0, aig.fanin1, pi)
    po = words[-2 * n:]
    for pat, (a, b) in enumerate(ops):
        got = sum(((int(po[k]) >> pat) & 1) << k for k in range(2 * n))
        assert got == a * b, (n, a, b)


@pytest.mark.parametrize("n", [2, 4, 6, 8, 16, 32, 64, 96])
def test_booth_multiplier_function_and_degree_profile(n):
    """The radix-4 Booth generator multiplies (every pattern through the oracle's bit-parallel AIG
    evaluation), is a well-formed AIG, and has the degree profile it is there for: the recoding
    signals of the n/2 + 1 digit rows are high-degree nodes next to the primary inputs."""
    aig = wl.booth_multiplier_aig(n)
    n1 = aig.num_nodes
    assert (aig.type[:2 * n] == 0).all() and (aig.type[-2 * n:] == 2).all() and (aig.type[2 * n:-2 * n] == 1).all()
    ids = np.arange(n1)
    inner = aig.type == 1
    assert ((aig.fanin0[inner] >> 1) < ids[inner]).all() and ((aig.fanin1[inner] >> 1) < ids[inner]).all()   # topological
    assert (aig.fanin0[inner] >= 0).all() and (aig.fanin1[inner] >= 0).all()                                 # no constants left
    assert (aig.fanin0[-2 * n:] == aig.fanin1[-2 * n:]).all() and (aig.fanin0[-2 * n:] == aig.po_driver).all()
    rng = random.Random(2000 + n)
    ops = [(rng.getrandbits(n), rng.getrandbits(n)) for _ in range(58)]
    ops += [(0, 0), ((1 << n) - 1, (1 << n) - 1), (1, (1 << n) - 1), ((1 << n) - 1, 1),
            (1 << (n - 1), 1 << (n - 1)), ((1 << n) - 1, (1 << n) - 2)]
    pi = np.zeros(2 * n, dtype=np.uint64)
    for pat, (a, b) in enumerate(ops):
        for i in range(n):
            if (a >> i) & 1:
                pi[i] |= np.uint64(1) << np.uint64(pat)
            if (b >> i) & 1:
                pi[n + i] |= np.uint64(1) << np.uint64(pat)
    words = oracle.aig_simulate(aig.type, aig.fanin0, aig.fanin1, pi)
    po = words[-2 * n:]
    for pat, (a, b) in enumerate(ops):
        got = sum(((int(po[k]) >> pat) & 1) << k for k in range(2 * n))
        assert got == a * b, (n, a, b)
    if n >= 32:
        rowptr, _, _, _ = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, 1)
        deg = np.diff(rowptr)
        hot = int((deg >= n).sum())
        assert 2 * n <= hot <= 4 * n            # about 3.5 n rows of n .. 4n+8 entries (CSA: exactly 2n rows of n+1)
        assert deg.max() >= 2 * n
        assert (deg <= 6).mean() > 0.98


def test_booth_generator_rejects_odd_widths():
    for n in (0, 1, 3, 7, 4096):
        with pytest.raises(ValueError):
            wl.booth_multiplier_aig(n)


@pytest.mark.parametrize("n", [2, 3, 6, 8, 32, 256])
def test_gate_counts_closed_form(n):
    """n^2 partial products + n half adders (3 ANDs) + n(n-2) full adders (7 ANDs)."""
    aig = wl.csa_multiplier_aig(n)
    n_and = int((aig.type == wl.AND).sum())
    assert n_and == n * n + 3 * n + 7 * n * (n - 2) == 8 * n * n - 11 * n
    assert int((aig.type == wl.PI).sum()) == 2 * n and int((aig.type == wl.PO).sum()) == 2 * n
    assert aig.num_nodes == 8 * n * n - 7 * n
    # PIs first, POs last, fanins precede their node
    assert (aig.type[:2 * n] == wl.PI).all() and (aig.type[-2 * n:] == wl.PO).all()
    ids = np.arange(aig.num_nodes)
    inner = aig.type != wl.PI
    assert ((aig.fanin0[inner] >> 1) < ids[inner]).all() and ((aig.fanin1[inner] >> 1) < ids[inner]).all()
    # PO records repeat the driver literal
    po = aig.type == wl.PO
    assert (aig.fanin0[po] == aig.fanin1[po]).all() and (aig.fanin0[po] == aig.po_driver).all()
    if n >= 3:
        # inverted records: each xor has 4, each full adder 2 more (its carry AND),
        # every full-adder carry consumer sees an inverted literal
        inv = int((aig.fanin0[inner] & 1).sum() + (aig.fanin1[inner] & 1).sum())
        assert inv == 10 * n * n - 16 * n + 2


def test_uniform_features_torch_equals_numpy():
    import torch

    a = wl.uniform_features(7, 123, 123 + 999, 32, block_rows=100).numpy()
    b = wl.uniform_features_numpy(7, 123, 123 + 999, 32)
    assert np.array_equal(a, b)
    assert a.min() >= -1.0 and a.max() < 1.0
    assert abs(a.mean()) < 0.02 and abs(a.var() - 1.0 / 3.0) < 0.02
    # pure function of (seed, global row, k): a shifted window agrees on the overlap
    c = wl.uniform_features_numpy(7, 500, 600, 32)
    assert np.array_equal(c, b[500 - 123:600 - 123])
    assert not np.array_equal(wl.uniform_features_numpy(8, 0, 10, 32), wl.uniform_features_numpy(7, 0, 10, 32))


def test_node_features_columns():
    aig = wl.csa_multiplier_aig(8)
    x = wl.aig_node_features(aig, 0, 32)
    assert x.dtype == np.float32 and x.shape == (aig.num_nodes, 32)
    assert (x[:, :3].sum(axis=1) == 1).all()
    assert (x[:, 3] + x[:, 4] == np.where(aig.type == wl.PI, 0, 2)).all()
    # every fanin record is somebody's fanout record
    assert x[:, 3].sum() == x[:, 5].sum() and x[:, 4].sum() == x[:, 6].sum()
    assert (x[:, 7] == 1).all()
    assert np.array_equal(x[:, 8:], wl.uniform_features_numpy(0, 0, aig.num_nodes, 32)[:, 8:])


def test_stress_graph_distribution():
    n, window, dmin, dmax = 1 << 16, 512, 64, 4096
    g = wl.stress_graph(4, n, window=window, dmin=dmin, dmax=dmax)
    deg = np.diff(g.rowptr)
    heavy = np.array([wl.stress_is_heavy(4, i) for i in range(n)])
    assert 0.007 < heavy.mean() < 0.013
    assert set(np.unique(deg[~heavy])) <= {3, 4, 5}                 # 2-4 neighbours + self
    assert deg[heavy].min() >= dmin // 2 and deg[heavy].max() <= dmax + 1
    assert (deg[heavy] > 5).all()
    rows = np.repeat(np.arange(n), deg)
    # ascending, unique columns; self-loop present; weights 1/len
    same_row = rows[1:] == rows[:-1]
    assert (np.diff(g.col.astype(np.int64))[same_row] > 0).all()
    assert np.array_equal(np.bincount(rows[g.col == rows], minlength=n), np.ones(n, dtype=np.int64))
    assert np.array_equal(g.val, (1.0 / deg.astype(np.float32)).astype(np.float32)[rows])
    # light rows stay inside the window (cyclically)
    light = ~heavy[rows]
    d = np.abs(g.col[light].astype(np.int64) - rows[light])
    assert (np.minimum(d, n - d) <= window).all()
    # regenerating gives the same graph
    g2 = wl.stress_graph(4, n, window=window, dmin=dmin, dmax=dmax)
    assert np.array_equal(g.col, g2.col) and np.array_equal(g.rowptr, g2.rowptr)


@pytest.mark.parametrize("n,batch", [(2, 1), (5, 3), (32, 2)])
def test_lut4_graph_shape(n, batch):
    """Symmetric, self-loops, sorted rows, mean weights bit-exact, block-diagonal copies, and the degree
    profile the generator documents (2n input rows of 2n+1 entries, interior LUT rows of 7)."""
    g = wl.lut4_csa_graph(n, batch)
    n1 = g.n // batch
    assert n1 == 2 * n + 2 * n * n + 2 * n + 2 * n
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    pairs = set(zip(rows.tolist(), g.col.tolist()))
    assert all((c, r) in pairs for r, c in pairs)                       # symmetric
    assert all((v, v) in pairs for v in range(g.n))                     # self-loops
    assert all(r // n1 == c // n1 for r, c in pairs)                    # copies do not touch
    for v in range(g.n):
        seg = g.col[g.rowptr[v]:g.rowptr[v + 1]]
        assert (np.diff(seg) > 0).all()
    deg = np.diff(g.rowptr)
    want = (np.float32(1.0) / deg.astype(np.float32)).astype(np.float32)
    assert np.array_equal(g.val.view(np.uint32), np.repeat(want, deg).view(np.uint32))
    assert (deg[:2 * n] == 2 * n + 1).all()                             # every input feeds 2n LUTs
    if n >= 5:
        assert np.bincount(deg).argmax() == 7
    assert np.array_equal(deg[:n1], deg[n1 * (batch - 1):])             # same profile in every copy


@pytest.mark.parametrize("n,batch", [(2, 1), (5, 3), (32, 2)])
def test_cellmap_graph_shape(n, batch):
    """Standard-cell-mapped shape: symmetric, self-loops, sorted rows, mean weights bit-exact, block-diagonal
    copies, and the documented degree profile (2n input rows of n+1 entries, AND2 rows of 4, adder rows of
    at most 6)."""
    g = wl.cellmap_csa_graph(n, batch)
    n1 = g.n // batch
    assert n1 == 2 * n + 2 * n * n + n + 2 * n
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    pairs = set(zip(rows.tolist(), g.col.tolist()))
    assert all((c, r) in pairs for r, c in pairs)
    assert all((v, v) in pairs for v in range(g.n))
    assert all(r // n1 == c // n1 for r, c in pairs)
    for v in range(g.n):
        seg = g.col[g.rowptr[v]:g.rowptr[v + 1]]
        assert (np.diff(seg) > 0).all()
    deg = np.diff(g.rowptr)
    want = (np.float32(1.0) / deg.astype(np.float32)).astype(np.float32)
    assert np.array_equal(g.val.view(np.uint32), np.repeat(want, deg).view(np.uint32))
    assert (deg[:2 * n] == n + 1).all()                                 # every input feeds n AND2 cells
    and2 = 2 * n + 2 * np.arange(n * n)
    assert (deg[and2] == 4).all()                                       # two inputs, its adder, itself
    assert deg[2 * n:n1].max() <= 6
    assert np.array_equal(deg[:n1], deg[n1 * (batch - 1):])
