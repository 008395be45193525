"""GPU parity of the device-side degree plan (degree classes and the stable
count sort of the low-degree rows) against the CPU oracle: integer outputs,
compared bit for bit; entries past the written counts must stay untouched."""
import numpy as np
import pytest

import oracle
import workloads as wl
from util import ensure_built

pytestmark = pytest.mark.gpu

ensure_built()
import paper_2511_18297_amd as G  # noqa: E402

CANARY = -7


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    assert torch.cuda.is_available(), "these tests need a GPU"
    torch.cuda.set_device(0)
    return torch


def _check(torch, g, rowptr, T, what):
    n = rowptr.shape[0] - 1
    plan = G.groot_spmm_plan(g, T)
    G.groot_plan_upload(plan, 4)
    dev = dict(device="cuda")
    row_class = torch.full((max(n, 1),), 9, dtype=torch.uint8, **dev)
    hd = torch.full((max(n, 1),), CANARY, dtype=torch.int32, **dev)
    ld = torch.full((max(n, 1),), CANARY, dtype=torch.int32, **dev)
    by = torch.full((max(n, 1),), CANARY, dtype=torch.int32, **dev)
    off = torch.full((T + 1,), CANARY, dtype=torch.int64, **dev)
    counts = torch.full((2,), CANARY, dtype=torch.int64, **dev)
    print(f"device plan: {what} n={n} T={T}", flush=True)
    G.groot_plan_lists_device(plan, row_class, hd, ld, by, off, counts)
    want = oracle.plan(rowptr, T)
    n_hd, n_ld = (int(v) for v in counts.cpu())
    assert n_hd == want["hd_rows"].shape[0] and n_ld == want["ld_rows"].shape[0], what
    assert np.array_equal(row_class.cpu().numpy()[:n], want["row_class"]), what
    assert np.array_equal(off.cpu().numpy(), want["ld_deg_offsets"]), what
    for got, key in ((hd, "hd_rows"), (ld, "ld_rows"), (by, "ld_rows_by_degree")):
        a = got.cpu().numpy()
        k = want[key].shape[0]
        assert np.array_equal(a[:k], want[key]), f"{what}: {key}"
        assert (a[k:] == CANARY).all(), f"{what}: {key} written past its count"
    # the host plan of the library agrees as well
    view = G.groot_plan_view(plan)
    assert np.array_equal(view["ld_rows_by_degree"], want["ld_rows_by_degree"])


@pytest.mark.parametrize("T", [4, 5, 33])
def test_multiplier_batch(torch_cuda, T):
    """32-bit multiplier x 3 copies: 23,904 rows = 5 full blocks of 4096 and a ragged one."""
    aig = wl.csa_multiplier_aig(32)
    g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, 3)
    rowptr = G.groot_graph_view(g)["rowptr"]
    _check(torch_cuda, g, rowptr, T, "csa32 x3")


@pytest.mark.parametrize("T", [1, 3, 64, 1024])
def test_polarized_degrees(torch_cuda, T):
    s = wl.stress_graph(5, 1 << 16, window=4096, dmin=64, dmax=16384)
    g = G.groot_graph_from_csr(s.rowptr, s.col, s.val)
    _check(torch_cuda, g, s.rowptr, T, "stress")


@pytest.mark.parametrize("n,T", [(1, 2), (5, 3), (63, 9), (64, 9), (4096, 17), (4097, 17), (20000, 40), (20000, 12)])
def test_mixed_degrees_in_every_chunk(torch_cuda, n, T):
    """Row lengths drawn uniformly from 0..min(n,40): every 64-row chunk holds many distinct degrees,
    empty rows included; with T = 12 a large share of the rows is high-degree."""
    rng = np.random.default_rng(100 + n + T)
    deg = rng.integers(0, min(n, 40) + 1, size=n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    start = rng.integers(0, n, size=n)
    col = np.concatenate([np.sort((start[i] + np.arange(deg[i])) % n) for i in range(n)] + [np.zeros(0, dtype=np.int64)])
    col = col.astype(np.int32)
    val = np.ones(col.shape[0], dtype=np.float32)
    g = G.groot_graph_from_csr(rowptr, col, val)
    _check(torch_cuda, g, rowptr, T, "mixed")


def test_threshold_above_the_device_limit(torch_cuda):
    torch = torch_cuda
    aig = wl.csa_multiplier_aig(4)
    g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, 1)
    n = G.groot_graph_view(g)["n"]
    plan = G.groot_spmm_plan(g, 1025)
    G.groot_plan_upload(plan, 4)
    bufs = [torch.zeros(n, dtype=torch.uint8, device="cuda")] + \
           [torch.zeros(n, dtype=torch.int32, device="cuda") for _ in range(3)] + \
           [torch.zeros(1026, dtype=torch.int64, device="cuda"), torch.zeros(2, dtype=torch.int64, device="cuda")]
    with pytest.raises(G.GrootError) as e:
        G.groot_plan_lists_device(plan, *bufs)
    assert e.value.status == G.GROOT_ERANGE
