"""The entry point for callers that cannot allocate: groot_plan_lists_device_static must give, bit for bit,
the lists of groot_plan_lists_device (integer outputs), on two calls in a row that share the library's
fixed scratch array, the second on a smaller graph; and it must refuse a graph whose block table does not
fit that array."""
import numpy as np
import pytest

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


def _buffers(torch, n, T):
    dev = dict(device="cuda")
    return [torch.full((max(n, 1),), 9, dtype=torch.uint8, **dev)] + \
           [torch.full((max(n, 1),), CANARY, dtype=torch.int32, **dev) for _ in range(3)] + \
           [torch.full((T + 1,), CANARY, dtype=torch.int64, **dev), torch.full((2,), CANARY, dtype=torch.int64, **dev)]


def _both(torch, g, T, what):
    n = G.groot_graph_view(g)["n"]
    plan = G.groot_spmm_plan(g, T)
    G.groot_plan_upload(plan, 4)
    ref, got = _buffers(torch, n, T), _buffers(torch, n, T)
    print(f"no-alloc plan lists: {what} n={n} T={T}", flush=True)
    G.groot_plan_lists_device(plan, *ref)
    G.groot_plan_lists_device_static(plan, *got)
    torch.cuda.synchronize()
    names = ("row_class", "hd_rows", "ld_rows", "ld_rows_by_degree", "ld_deg_offsets", "counts")
    for name, a, b in zip(names, ref, got):
        assert torch.equal(a, b), f"{what}: {name} differs (canaries past the counts included)"
    view = G.groot_plan_view(plan)
    n_hd, n_ld = (int(v) for v in got[5].cpu())
    assert n_hd == view["n_hd"] and n_ld == view["n_ld"]
    assert np.array_equal(got[3].cpu().numpy()[:n_ld], view["ld_rows_by_degree"])
    return plan


def test_two_calls_in_a_row_second_smaller(torch_cuda):
    """A 64-bit multiplier x 5 copies (162,560 rows = 40 blocks of 4096) and then, through the same scratch
    bytes, a 17-bit multiplier (2,193 rows, a single ragged block) with another threshold: stale table
    entries of the first call must not reach the second."""
    big = wl.csa_multiplier_aig(64)
    g_big = G.groot_graph_build(big.type, big.fanin0, big.fanin1, 5)
    small = wl.csa_multiplier_aig(17)
    g_small = G.groot_graph_build(small.type, small.fanin0, small.fanin1, 1)
    keep = [_both(torch_cuda, g_big, 32, "csa64 x5"), _both(torch_cuda, g_small, 5, "csa17"),
            _both(torch_cuda, g_big, 6, "csa64 x5 again")]
    del keep


def test_polarized_degrees_and_wide_threshold(torch_cuda):
    s = wl.stress_graph(5, 1 << 16, window=4096, dmin=64, dmax=16384)
    g = G.groot_graph_from_csr(s.rowptr, s.col, s.val)
    for T in (1024, 3):
        _both(torch_cuda, g, T, "stress")


def test_scratch_limit_is_an_error(torch_cuda):
    """2^21 empty rows at T = 1024: 512 blocks x 1026 columns x 4 bytes = 2.1 MB fits; 2^23 rows (8.4 MB) do not."""
    torch = torch_cuda
    T = 1024
    for n, fits in ((1 << 21, True), (1 << 23, False)):
        rowptr = np.zeros(n + 1, dtype=np.int64)
        g = G.groot_graph_from_csr(rowptr, np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float32))
        plan = G.groot_spmm_plan(g, T)
        G.groot_plan_upload(plan, 4)
        bufs = _buffers(torch, n, T)
        if fits:
            G.groot_plan_lists_device_static(plan, *bufs)
            torch.cuda.synchronize()
            assert [int(v) for v in bufs[5].cpu()] == [0, n]
            assert int(bufs[4][1]) == n and int(bufs[4][0]) == 0          # every row has degree 0
        else:
            with pytest.raises(G.GrootError) as e:
                G.groot_plan_lists_device_static(plan, *bufs)
            assert e.value.status == G.GROOT_ERANGE and "scratch" in str(e.value)
            assert int(bufs[5][0]) == CANARY                              # outputs untouched
