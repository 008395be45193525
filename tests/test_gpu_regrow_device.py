"""GPU parity of the device-side partition with boundary edge re-growth (Eq. (1), Eq. (2), Algorithm 1
of the paper) and of the plan built from its device arrays, against the CPU oracle: ids, row pointers,
columns, counts and weight bits compared exactly; the aggregation on the device-built plan within the
floating point tolerance."""
import numpy as np
import pytest

import oracle
import workloads as wl
from util import assert_close_to_oracle, ensure_built, layer_tolerance

pytestmark = pytest.mark.gpu

ensure_built()
import paper_2511_18297_amd as G  # noqa: E402


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    assert torch.cuda.is_available(), "these tests need a GPU"
    torch.cuda.set_device(0)
    return torch


def _resident_plan(g, T=32, F=4):
    plan = G.groot_spmm_plan(g, T)
    G.groot_plan_upload(plan, F)
    return plan


def _check_part(torch, plan, rowptr, col, val, part_of, P, p, flags, weight_mode, use_rule, what):
    print(f"device regrow: {what} P={P} p={p} flags={flags}", flush=True)
    po_dev = None if use_rule else torch.from_numpy(part_of).cuda()
    part = G.groot_partition_regrow_device(plan, P, p, po_dev, flags)
    view = G.groot_dev_part_view(part)
    want = oracle.regrow_part(rowptr, col, val, part_of, p, flags, weight_mode)
    for k in ("n_owned", "n_halo", "n_crossing"):
        assert view[k] == want[k], (what, p, k, view[k], want[k])
    assert view["nnz"] == want["col"].shape[0], (what, p)
    got = G.groot_dev_part_download(part)
    assert np.array_equal(got["global_id"], want["global_id"]), (what, p, "global_id")
    assert np.array_equal(got["rowptr"], want["rowptr"]), (what, p, "rowptr")
    assert np.array_equal(got["col"], want["col"]), (what, p, "col")
    if weight_mode == 2:
        assert np.array_equal(got["val"].view(np.uint32), want["val"].view(np.uint32)), (what, p, "val")
    else:
        assert "val" not in got and view["val"] is None
    return part, want


@pytest.mark.parametrize("n,batch,P", [(2, 1, 2), (8, 1, 5), (16, 2, 16), (32, 3, 4), (64, 1, 3)])
@pytest.mark.parametrize("flags", [G.GROOT_REGROW, 0])
def test_multiplier_default_rule(torch_cuda, n, batch, P, flags):
    """The built-in rule (p-th contiguous slice of every copy) on carry-save multipliers; the 32-bit x 3 and
    64-bit cases span several blocks of 4096 rows with a ragged tail."""
    aig = wl.csa_multiplier_aig(n)
    g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, batch)
    rowptr, col, val, _ = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, batch)
    part_of = oracle.part_of_default(len(rowptr) - 1, aig.num_nodes, P)
    plan = _resident_plan(g)
    for p in range(P):
        _check_part(torch_cuda, plan, rowptr, col, val, part_of, P, p, flags, 1, True, f"csa{n}x{batch}")


def test_user_parts_weight_modes_and_directed_graph(torch_cuda):
    rng = np.random.default_rng(11)
    aig = wl.csa_multiplier_aig(24)
    part_of = rng.integers(0, 4, size=2 * aig.num_nodes).astype(np.int32)
    # random assignment on the mean-normalised graph (boundaries everywhere)
    g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, 2)
    rowptr, col, val, _ = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, 2)
    plan = _resident_plan(g)
    for p in range(4):
        _check_part(torch_cuda, plan, rowptr, col, val, part_of, 4, p, G.GROOT_REGROW, 1, False, "random parts, mean")
    # unit weights
    g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, 2, 3)
    rowptr, col, val, _ = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, 2, 3)
    plan = _resident_plan(g)
    _check_part(torch_cuda, plan, rowptr, col, val, part_of, 4, 1, G.GROOT_REGROW, 0, False, "random parts, ones")
    # directed graph with explicit weights and long rows: one-way crossing edges, weights copied
    s = wl.stress_graph(9, 3 * 4096 + 77, window=32, dmin=64, dmax=1024)
    w = rng.random(len(s.col)).astype(np.float32)
    g = G.groot_graph_from_csr(s.rowptr, s.col, w)
    plan = _resident_plan(g)
    part_of = rng.integers(0, 3, size=s.n).astype(np.int32)
    for flags in (G.GROOT_REGROW, 0):
        for p in range(3):
            _check_part(torch_cuda, plan, s.rowptr, s.col, w, part_of, 3, p, flags, 2, False, "stress, explicit")
    # contiguous thirds of the same graph through the built-in rule (one copy)
    part_of = oracle.part_of_default(s.n, s.n, 3)
    for p in range(3):
        _check_part(torch_cuda, plan, s.rowptr, s.col, w, part_of, 3, p, G.GROOT_REGROW, 2, True, "stress, rule")
    # an empty part is legal and has no rows
    part_of = np.zeros(s.n, dtype=np.int32)
    part, _ = _check_part(torch_cuda, plan, s.rowptr, s.col, w, part_of, 2, 1, G.GROOT_REGROW, 2, False, "empty part")
    with pytest.raises(G.GrootError) as e:
        G.groot_dev_part_plan(part, 32, 64)
    assert e.value.status == G.GROOT_EINVAL
    # the only part is the whole graph
    part, want = _check_part(torch_cuda, plan, s.rowptr, s.col, w, part_of, 1, 0, G.GROOT_REGROW, 2, False, "one part")
    assert want["n_halo"] == 0 and np.array_equal(want["rowptr"], s.rowptr)


@pytest.mark.parametrize("n,batch,P,T,F", [(32, 2, 4, 32, 64), (48, 1, 5, 8, 32), (24, 3, 2, 200, 20)])
def test_device_built_plans_fill_the_full_result(torch_cuda, n, batch, P, T, F):
    """Partitioned mode with nothing built on the host: every part re-grown on the device, its plan made from
    the device arrays, its owned rows computed into place.  Every element against the oracle on the full
    graph; the plan's lists against the oracle's plan of the oracle's sub-graph."""
    torch = torch_cuda
    aig = wl.csa_multiplier_aig(n)
    g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, batch)
    rowptr, col, val, _ = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, batch)
    N = batch * aig.num_nodes
    part_of = oracle.part_of_default(N, aig.num_nodes, P)
    X_np = wl.uniform_features_numpy(21, 0, N, F)
    X = torch.from_numpy(X_np).cuda()
    guard = 2
    buf = torch.full((N + 2 * guard, F), float("nan"), device="cuda")
    buf[:guard] = 555.0
    buf[N + guard:] = 555.0
    Y = buf[guard:N + guard]
    full = _resident_plan(g, T, F)
    for p in range(P):
        part, want = _check_part(torch, full, rowptr, col, val, part_of, P, p, G.GROOT_REGROW, 1, True, f"csa{n}x{batch}")
        view = G.groot_dev_part_view(part)
        n_loc = view["n_owned"] + view["n_halo"]
        plan = G.groot_dev_part_plan(part, T, F)
        after = G.groot_dev_part_view(part)
        assert after["rowptr"] is None and after["col"] is None and after["global_id"] is not None
        with pytest.raises(G.GrootError):
            G.groot_dev_part_plan(part, T, F)                       # the sub-graph has moved
        with pytest.raises(G.GrootError):
            G.groot_plan_view(plan)                                 # no host lists
        G.groot_plan_upload(plan, F)                                # no-op
        with pytest.raises(G.GrootError):
            G.groot_plan_upload(plan, F + 4)
        # lists of the device-built plan
        wp = oracle.plan(want["rowptr"], T)
        dev = dict(device="cuda")
        row_class = torch.empty(n_loc, dtype=torch.uint8, **dev)
        hd, ld, by = (torch.empty(n_loc, dtype=torch.int32, **dev) for _ in range(3))
        off = torch.empty(T + 1, dtype=torch.int64, **dev)
        counts = torch.empty(2, dtype=torch.int64, **dev)
        G.groot_plan_lists_device(plan, row_class, hd, ld, by, off, counts)
        n_hd, n_ld = (int(v) for v in counts.cpu())
        assert n_hd == wp["hd_rows"].shape[0] and n_ld == wp["ld_rows"].shape[0]
        assert np.array_equal(hd.cpu().numpy()[:n_hd], wp["hd_rows"])
        assert np.array_equal(by.cpu().numpy()[:n_ld], wp["ld_rows_by_degree"])
        # gather, aggregate the owned rows into place
        ids = after["global_id"]
        Xp = torch.empty((n_loc, F), device="cuda")
        G.groot_rows_gather(ids, X, Xp, F)
        G.groot_spmm_execute_rows(plan, Xp, Y, F, view["n_owned"], ids)
        torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert (out[:guard] == 555.0).all() and (out[N + guard:] == 555.0).all(), "wrote outside Y"
    Y64, S = oracle.spmm_f64(rowptr, col, val, X_np)
    assert_close_to_oracle(out[guard:N + guard], Y64, S, f"device-built parts, P={P} T={T} F={F}")


@pytest.mark.parametrize("n,batch,P,T,F", [(32, 2, 4, 32, 64), (48, 1, 5, 8, 32), (24, 3, 2, 200, 20)])
@pytest.mark.parametrize("built_on", ["device", "host"])
def test_parts_read_the_whole_feature_matrix_in_place(torch_cuda, built_on, n, batch, P, T, F):
    """Partitioned mode without any row copies: the columns of every part's plan are renamed to global rows once
    (groot_plan_use_global_columns), then one groot_spmm_execute_rows per part reads the whole graph's X in
    place and writes the owned rows of Y in place.  Every element against the oracle on the full graph."""
    torch = torch_cuda
    aig = wl.csa_multiplier_aig(n)
    g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, batch)
    rowptr, col, val, _ = oracle.csr_build(aig.type, aig.fanin0, aig.fanin1, batch)
    N = batch * aig.num_nodes
    X_np = wl.uniform_features_numpy(23, 0, N, F)
    X = torch.from_numpy(X_np).cuda()
    guard = 2
    buf = torch.full((N + 2 * guard, F), float("nan"), device="cuda")
    buf[:guard] = 555.0
    buf[N + guard:] = 555.0
    Y = buf[guard:N + guard]
    full = _resident_plan(g, T, F)
    host_parts = G.groot_partition_regrow(g, P) if built_on == "host" else None
    for p in range(P):
        if built_on == "device":
            part = G.groot_partition_regrow_device(full, P, p)
            view = G.groot_dev_part_view(part)
            n_owned, ids = view["n_owned"], view["global_id"]
            plan = G.groot_dev_part_plan(part, T, F)
        else:
            pv = G.groot_parts_view(host_parts, p)
            n_owned, ids = pv["n_owned"], torch.from_numpy(pv["global_id"].copy()).cuda()
            plan = G.groot_spmm_plan(pv["sub"], T)
            G.groot_plan_upload(plan, F)
        print(f"global columns: {built_on} part {p}/{P} csa{n}x{batch} T={T} F={F}", flush=True)
        G.groot_plan_use_global_columns(plan, ids, N)
        with pytest.raises(G.GrootError):
            G.groot_plan_use_global_columns(plan, ids, N)           # only once
        with pytest.raises(ValueError):
            G.groot_spmm_execute_rows(plan, X[:N - 1], Y, F, n_owned, ids)   # X is the whole matrix now
        G.groot_spmm_execute_rows(plan, X, Y, F, n_owned, ids)
        torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert (out[:guard] == 555.0).all() and (out[N + guard:] == 555.0).all(), "wrote outside Y"
    Y64, S = oracle.spmm_f64(rowptr, col, val, X_np)
    assert_close_to_oracle(out[guard:N + guard], Y64, S, f"global columns, {built_on}-built parts, P={P} T={T} F={F}")


def test_device_built_plan_with_split_high_degree_rows_and_nested_partition(torch_cuda):
    """Explicit weights, rows far above the piece size (several pieces per row), all kernels of the
    device-built plan against the oracle on the oracle's sub-graph; then the sub-graph is partitioned again
    from the device-built plan."""
    torch = torch_cuda
    rng = np.random.default_rng(3)
    s = wl.stress_graph(4, 1 << 14, window=64, dmin=64, dmax=4096)
    w = rng.random(len(s.col)).astype(np.float32)
    g = G.groot_graph_from_csr(s.rowptr, s.col, w)
    full = _resident_plan(g, 32, 64)
    part_of = oracle.part_of_default(s.n, s.n, 2)
    part, want = _check_part(torch, full, s.rowptr, s.col, w, part_of, 2, 1, G.GROOT_REGROW, 2, True, "stress halves")
    n_loc = want["n_owned"] + want["n_halo"]
    for T, F in ((32, 64), (16, 32)):
        if T != 32:
            part = G.groot_partition_regrow_device(full, 2, 1)
        plan = G.groot_dev_part_plan(part, T, F)
        deg = np.diff(want["rowptr"])
        pieces = int(np.ceil(deg[deg >= T] / 512).sum())
        assert pieces > int((deg >= T).sum()), "the case must contain rows of several pieces"
        assert G.groot_plan_query(plan, "hd_pieces") == pieces
        X_np = wl.uniform_features_numpy(8, 0, n_loc, F)
        X = torch.from_numpy(X_np).cuda()
        Y = torch.full((n_loc, F), float("nan"), device="cuda")
        G.groot_spmm_execute(plan, X, Y, F)
        torch.cuda.synchronize()
        Y64, S = oracle.spmm_f64(want["rowptr"], want["col"], want["val"], X_np)
        assert_close_to_oracle(Y.cpu().numpy(), Y64, S, f"device-built plan T={T} F={F}")
    # nested: three parts of the sub-graph, from the device-built plan (one copy of n_loc nodes)
    sub_part_of = oracle.part_of_default(n_loc, n_loc, 3)
    for p in range(3):
        _check_part(torch, plan, want["rowptr"], want["col"], want["val"], sub_part_of, 3, p, G.GROOT_REGROW, 2,
                    True, "nested")


@pytest.mark.parametrize("T,hd_chunk", [(32, 512), (16, 64), (200, 300)])
def test_device_built_schedule_of_high_degree_rows_is_the_host_plans(torch_cuda, T, hd_chunk):
    """The launch list of the HD kernel that groot_dev_part_plan cuts and orders on the device, against the list
    a host plan makes from the oracle's copy of the same sub-graph: piece by piece, bit for bit (rows of one and
    of many pieces, piece sizes 64, 300 and 512).  The fused layer on the device-built plan (its high-degree sums
    go through the schedule that names rows by rank) against the fp64 layer."""
    torch = torch_cuda
    rng = np.random.default_rng(5)
    s = wl.stress_graph(6, 1 << 14, window=64, dmin=64, dmax=4096)
    w = rng.random(len(s.col)).astype(np.float32)
    g = G.groot_graph_from_csr(s.rowptr, s.col, w)
    full = _resident_plan(g, 32, 64)
    part_of = oracle.part_of_default(s.n, s.n, 2)
    want = oracle.regrow_part(s.rowptr, s.col, w, part_of, 0, G.GROOT_REGROW, 2)
    n_loc = want["n_owned"] + want["n_halo"]
    G.groot_set_tuning("hd_chunk", hd_chunk)
    try:
        print(f"device HD schedule: T={T} hd_chunk={hd_chunk} rows={n_loc}", flush=True)
        part = G.groot_partition_regrow_device(full, 2, 0)
        dev_plan = G.groot_dev_part_plan(part, T, 64)
        sub = G.groot_graph_from_csr(want["rowptr"], want["col"], want["val"])
        host_plan = G.groot_spmm_plan(sub, T)
        G.groot_plan_upload(host_plan, 64)
    finally:
        G.groot_set_tuning("hd_chunk", 512)
    got, ref = G.groot_plan_hd_pieces(dev_plan), G.groot_plan_hd_pieces(host_plan)
    deg = np.diff(want["rowptr"])
    hd = deg[deg >= T]
    pieces = np.maximum(1, -(-hd // hd_chunk))
    assert len(ref["row"]) == int(pieces.sum()) and (pieces > 1).any() and (pieces == 1).any()
    for k in ("begin", "len", "row", "slot"):
        assert np.array_equal(got[k], ref[k]), (k, T, hd_chunk)
    for k in ("hd_pieces", "hd_partials", "nnz_hd"):
        assert G.groot_plan_query(dev_plan, k) == G.groot_plan_query(host_plan, k), k
    assert G.groot_plan_query(dev_plan, "nnz_hd") == int(hd.sum())
    # every entry of every high-degree row is in exactly one piece
    covered = np.zeros(len(want["col"]), np.int32)
    for b, ln in zip(got["begin"], got["len"]):
        covered[b:b + ln] += 1
    is_hd = np.repeat(deg >= T, deg)
    assert np.array_equal(covered, is_hd.astype(np.int32))
    # fused layer on the device-built plan
    F = 64
    X = wl.uniform_features_numpy(9, 0, n_loc, F)
    Wn, Ws = (rng.uniform(-0.125, 0.125, (F, F)).astype(np.float32) for _ in range(2))
    b = rng.uniform(-0.125, 0.125, F).astype(np.float32)
    dev = lambda a: torch.from_numpy(a).cuda()
    H = torch.full((n_loc, F), float("nan"), device="cuda")
    G.groot_sage_layer_forward(dev_plan, dev(X), dev(Wn), dev(Ws), dev(b), True, H, F)
    torch.cuda.synchronize()
    ref_H, A, S = oracle.sage_layer_f64(want["rowptr"], want["col"], want["val"], X, Wn, Ws, b, True)
    a64 = lambda a: np.abs(a.astype(np.float64))
    scale = np.abs(A) @ a64(Wn) + a64(X) @ a64(Ws) + a64(b)
    err = np.abs(H.cpu().numpy().astype(np.float64) - ref_H)
    tol = layer_tolerance(S, scale, a64(Wn))
    assert np.isfinite(err).all() and (err <= tol).all(), float(np.max(err / tol))


def test_error_paths(torch_cuda):
    torch = torch_cuda
    aig = wl.csa_multiplier_aig(8)
    g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, 1)
    plan = G.groot_spmm_plan(g, 32)
    with pytest.raises(G.GrootError) as e:
        G.groot_partition_regrow_device(plan, 2, 0)                 # not resident
    assert e.value.status == G.GROOT_EINVAL
    G.groot_plan_upload(plan, 4)
    bad = torch.full((aig.num_nodes,), 2, dtype=torch.int32, device="cuda")
    for kw in (dict(num_parts=0, p=0), dict(num_parts=aig.num_nodes + 1, p=0), dict(num_parts=2, p=2),
               dict(num_parts=2, p=-1), dict(num_parts=2, p=0, flags=2), dict(num_parts=2, p=0, part_of=bad)):
        with pytest.raises(G.GrootError) as e:
            G.groot_partition_regrow_device(plan, **kw)
        assert e.value.status == G.GROOT_EINVAL, kw
    part = G.groot_partition_regrow_device(plan, 2, 0)
    for T, F in ((0, 64), (2000, 64), (32, 3), (32, 516)):
        with pytest.raises(G.GrootError):
            G.groot_dev_part_plan(part, T, F)
    pl = G.groot_dev_part_plan(part, 32, 64)
    assert G.groot_plan_query(pl, "hd_pieces") >= 0
    # the sub-graph has moved into the plan: its arrays can no longer be downloaded, the ids still can
    import paper_2511_18297_amd.binding as B
    view = G.groot_dev_part_view(part)
    host = np.empty(view["n_owned"] + view["n_halo"] + 1, dtype=np.int64)
    assert B._lib.groot_dev_part_download(part.handle, None, host.ctypes.data, None, None, None) == G.GROOT_EINVAL
    assert B._lib.groot_dev_part_download(part.handle, host.ctypes.data, None, None, None, None) == G.GROOT_OK
    assert "rowptr" not in G.groot_dev_part_download(part)
    # row-uniform weights: there is no weight array to download
    part = G.groot_partition_regrow_device(plan, 2, 1)
    wbuf = np.empty(G.groot_dev_part_view(part)["nnz"], dtype=np.float32)
    assert B._lib.groot_dev_part_download(part.handle, None, None, None, wbuf.ctypes.data, None) == G.GROOT_EINVAL
