"""End to end on the GPU, with nothing but the generator's own data: the paper's node features (4-bit
vectors) and node labels (PI / AND / XOR / MAJ / PO) of a carry-save multiplier, a small GraphSAGE-mean
classifier trained on the 8-bit multiplier with the library's aggregation in the forward pass and the
transposed aggregation in the backward pass, then inference on a larger multiplier: on the whole graph, and
part by part with and without the re-grown boundary (Section "GNN and Edge Re-growth After Partition":
without the boundary edges the nodes at a cut lose neighbours and accuracy drops; re-growth gives every owned
node its full one-hop neighbourhood back).

This is a qualitative reproduction on synthetic stand-ins (no dataset, no trained weights of the paper), so
the assertions are about the direction of the effect, not about the paper's percentages."""
import numpy as np
import pytest

import workloads as wl
from util import ensure_built

pytestmark = pytest.mark.gpu

ensure_built()
import paper_2511_18297_amd as G  # noqa: E402

HIDDEN, CLASSES, T = 32, 5, 32


def _plans(g, F):
    plan = G.groot_spmm_plan(g, T)
    G.groot_plan_upload(plan, F)
    gt = G.groot_graph_transpose(g)
    plan_t = G.groot_spmm_plan(gt, T)
    G.groot_plan_upload(plan_t, F)
    return plan, plan_t, gt


def _model(torch):
    class Aggregate(torch.autograd.Function):
        """Y = A_hat X through the library; dX = A_hat^T dY through the plan of the transposed graph."""

        @staticmethod
        def forward(ctx, X, plan, plan_t):
            X = X.contiguous()
            Y = torch.empty_like(X)
            G.groot_spmm_execute(plan, X, Y, X.shape[1])
            ctx.plan_t = plan_t
            return Y

        @staticmethod
        def backward(ctx, dY):
            dY = dY.contiguous()
            dX = torch.empty_like(dY)
            G.groot_spmm_execute(ctx.plan_t, dY, dX, dY.shape[1])
            return dX, None, None

    class Sage(torch.nn.Module):
        def __init__(self):
            super().__init__()
            gen = torch.Generator().manual_seed(7)
            dims = [(4, HIDDEN), (HIDDEN, HIDDEN), (HIDDEN, HIDDEN)]
            mk = lambda a, b: torch.nn.Parameter((torch.rand((a, b), generator=gen) - 0.5) * (2.0 / np.sqrt(a)))
            self.wn = torch.nn.ParameterList([mk(a, b) for a, b in dims])
            self.ws = torch.nn.ParameterList([mk(a, b) for a, b in dims])
            self.b = torch.nn.ParameterList([torch.nn.Parameter(torch.zeros(b)) for _, b in dims])
            self.out = torch.nn.Linear(HIDDEN, CLASSES)

        def forward(self, X, plan, plan_t=None):
            h = X
            for wn, ws, b in zip(self.wn, self.ws, self.b):
                agg = Aggregate.apply(h, plan, plan_t)
                h = torch.relu(agg @ wn + h @ ws + b)
            return self.out(h)

    return Sage()


def test_training_through_the_library_and_the_regrowth_ablation():
    import torch

    assert torch.cuda.is_available(), "these tests need a GPU"
    torch.cuda.set_device(0)
    torch.manual_seed(0)

    # ---- train on the 8-bit multiplier (the paper trains on 8-bit designs)
    small = wl.csa_multiplier_aig(8)
    g_small = G.groot_graph_build(small.type, small.fanin0, small.fanin1, 1)
    plan, plan_t, _gt = _plans(g_small, HIDDEN)
    X = torch.from_numpy(wl.paper_node_features(small)).cuda()
    y = torch.from_numpy(small.label.astype(np.int64)).cuda()
    model = _model(torch).cuda()
    # class weights: XOR / MAJ roots are rarer than plain AND nodes
    counts = torch.bincount(y, minlength=CLASSES).float()
    weight = (counts.sum() / (CLASSES * counts.clamp(min=1))).cuda()
    opt = torch.optim.Adam(model.parameters(), lr=1e-2)
    first = None
    for epoch in range(400):
        opt.zero_grad()
        loss = torch.nn.functional.cross_entropy(model(X, plan, plan_t), y, weight=weight)
        if first is None:
            first = float(loss.detach())
        loss.backward()
        opt.step()
    last = float(loss.detach())
    print(f"training loss {first:.4f} -> {last:.4f}", flush=True)
    assert np.isfinite(last) and last < 0.5 * first, "the gradients through the transposed aggregation must train the model"
    model.eval()

    # ---- the gradient of the aggregation is the transposed aggregation: check against autograd on a dense matrix
    view = G.groot_graph_view(g_small)
    A = torch.zeros((view["n"], view["n"]), dtype=torch.float64)
    rows = np.repeat(np.arange(view["n"]), np.diff(view["rowptr"]))
    A[torch.from_numpy(rows), torch.from_numpy(view["col"].astype(np.int64))] = torch.from_numpy(view["val"].astype(np.float64))
    Z = torch.randn((view["n"], 8), generator=torch.Generator().manual_seed(1))
    Zg = Z.cuda().requires_grad_(True)
    Wt = torch.randn((view["n"], 8), generator=torch.Generator().manual_seed(2))
    p8, p8t, _g8t = _plans(g_small, 8)
    # d/dZ sum(Wt * (A Z)) = A^T Wt
    from_lib = torch.autograd.grad((_aggregate(torch, Zg, p8, p8t) * Wt.cuda()).sum(), Zg)[0].cpu().double()
    want = A.T @ Wt.double()
    assert torch.allclose(from_lib, want, rtol=1e-5, atol=1e-6)

    # ---- inference on the 64-bit multiplier: whole graph, then 8 parts with and without re-growth
    big = wl.csa_multiplier_aig(64)
    g_big = G.groot_graph_build(big.type, big.fanin0, big.fanin1, 1)
    n = big.num_nodes
    Xb = torch.from_numpy(wl.paper_node_features(big)).cuda()
    yb = torch.from_numpy(big.label.astype(np.int64)).cuda()
    plan_big = G.groot_spmm_plan(g_big, T)
    G.groot_plan_upload(plan_big, HIDDEN)
    with torch.no_grad():
        pred_full = model(Xb, plan_big).argmax(1)
    acc_full = float((pred_full == yb).float().mean())

    # the gradient of a trained 32 -> 32 layer with respect to its input: the fused call against autograd through
    # the library's aggregation and its transposed aggregation (the way the model above was trained)
    plan_big_t = G.groot_spmm_plan(G.groot_graph_transpose(g_big), T)
    G.groot_plan_upload(plan_big_t, HIDDEN)
    gen = torch.Generator(device="cuda").manual_seed(3)
    h_in = torch.rand((n, HIDDEN), generator=gen, device="cuda").requires_grad_(True)
    R = torch.rand((n, HIDDEN), generator=gen, device="cuda") - 0.5
    wn1, ws1, b1 = (p.detach().clone().requires_grad_(True) for p in (model.wn[1], model.ws[1], model.b[1]))
    Zl = _aggregate(torch, h_in, plan_big, plan_big_t) @ wn1 + h_in @ ws1 + b1
    want_dx, want_dwn, want_dws = torch.autograd.grad((torch.relu(Zl) * R).sum(), (h_in, wn1, ws1))
    wn1, ws1 = wn1.detach(), ws1.detach()
    dZ = (R * (Zl.detach() > 0)).contiguous()
    scaled = torch.empty_like(dZ)
    G.groot_rows_over_degree(plan_big, dZ, scaled)
    got_dx = torch.empty_like(dZ)
    G.groot_sage_layer_backward_data(plan_big, scaled, wn1.t().contiguous(), ws1.t().contiguous(), got_dx)
    torch.cuda.synchronize()
    assert float((got_dx - want_dx).abs().max()) <= 1e-5 * float(want_dx.abs().max())
    # ... and with respect to its weights: one fused pass against autograd's two products over all rows
    ws_buf = torch.empty((G.groot_sage_layer_backward_weights_workspace(plan_big, HIDDEN) // 4,), device="cuda")
    got_dw = torch.empty((2, HIDDEN, HIDDEN), device="cuda")
    G.groot_sage_layer_backward_weights(plan_big, h_in.detach(), dZ, got_dw[0], got_dw[1], ws_buf)
    torch.cuda.synchronize()
    assert float((got_dw[0] - want_dwn).abs().max()) <= 2e-5 * float(want_dwn.abs().max())
    assert float((got_dw[1] - want_dws).abs().max()) <= 2e-5 * float(want_dws.abs().max())

    # the two 32 -> 32 layers through the fused layer kernel give the same classification
    with torch.no_grad():
        h = Xb
        agg = torch.empty_like(h)
        G.groot_spmm_execute(plan_big, h, agg, 4)
        h = torch.relu(agg @ model.wn[0] + h @ model.ws[0] + model.b[0]).contiguous()
        for layer in (1, 2):
            nxt = torch.empty_like(h)
            G.groot_sage_layer_forward(plan_big, h, model.wn[layer].detach().contiguous(), model.ws[layer].detach().contiguous(),
                                       model.b[layer].detach().contiguous(), True, nxt, HIDDEN)
            h = nxt
        logits_fused = model.out(h)
        logits_full = model(Xb, plan_big)
    assert float((logits_fused - logits_full).abs().max()) <= 1e-3 * float(logits_full.abs().max())
    assert bool((logits_fused.argmax(1) == pred_full).all())

    # the whole model through the fused layer kernel and nothing else: the 4 feature columns padded with zero
    # columns (and zero weight rows) to the narrowest input width, 32; the 5-class head as a layer without
    # aggregation (Wn = 0) and without ReLU, its 5 output columns padded with zero weights to 16
    # The same with the layer's cheaper dense products (two bf16 pieces per operand instead of three): the
    # classification does not change.
    def whole_model_fused():
        with torch.no_grad():
            pad_rows = lambda w: torch.cat([w.detach(), torch.zeros((HIDDEN - w.shape[0], w.shape[1]), device=w.device)]).contiguous()
            h = torch.cat([Xb, torch.zeros((n, HIDDEN - Xb.shape[1]), device="cuda")], dim=1).contiguous()
            for layer in range(3):
                wn, ws = model.wn[layer], model.ws[layer]
                if layer == 0:
                    wn, ws = pad_rows(wn), pad_rows(ws)
                nxt = torch.empty((n, HIDDEN), device="cuda")
                G.groot_sage_layer_forward_io(plan_big, h, wn.detach().contiguous(), ws.detach().contiguous(),
                                              model.b[layer].detach().contiguous(), True, nxt, HIDDEN, HIDDEN)
                h = nxt
            head_w = torch.zeros((HIDDEN, 16), device="cuda")
            head_w[:, :CLASSES] = model.out.weight.detach().t()
            head_b = torch.zeros(16, device="cuda")
            head_b[:CLASSES] = model.out.bias.detach()
            out16 = torch.empty((n, 16), device="cuda")
            G.groot_sage_layer_forward_io(plan_big, h, torch.zeros_like(head_w), head_w, head_b, False, out16, HIDDEN, 16)
            torch.cuda.synchronize()
        return out16

    try:
        for pieces in (3, 2):
            G.groot_set_tuning("sage_pieces", pieces)
            out16 = whole_model_fused()
            assert float(out16[:, CLASSES:].abs().max()) == 0.0
            assert float((out16[:, :CLASSES] - logits_full).abs().max()) <= 1e-3 * float(logits_full.abs().max()), pieces
            assert bool((out16[:, :CLASSES].argmax(1) == pred_full).all()), pieces
    finally:
        G.groot_set_tuning("sage_pieces", 3)

    P = 8
    vb = G.groot_graph_view(g_big)
    part_of = np.minimum(P - 1, (np.arange(n) * P) // n)
    src = np.repeat(np.arange(n), np.diff(vb["rowptr"]))
    at_cut = np.zeros(n, dtype=bool)
    cross = part_of[src] != part_of[vb["col"]]
    at_cut[src[cross]] = True
    at_cut_t = torch.from_numpy(at_cut).cuda()

    def partitioned(flags):
        parts = G.groot_partition_regrow(g_big, P, None, flags)
        pred = torch.full((n,), -1, dtype=torch.int64, device="cuda")
        for p in range(P):
            pv = G.groot_parts_view(parts, p)
            ids = torch.from_numpy(pv["global_id"].copy()).cuda()
            sub_plan = G.groot_spmm_plan(pv["sub"], T)
            G.groot_plan_upload(sub_plan, HIDDEN)
            with torch.no_grad():
                logits = model(Xb[ids].contiguous(), sub_plan)
            pred[ids[:pv["n_owned"]]] = logits[:pv["n_owned"]].argmax(1)
        assert int((pred < 0).sum()) == 0, "every node is owned by exactly one part"
        return pred

    pred_re = partitioned(G.GROOT_REGROW)
    pred_no = partitioned(0)
    acc = lambda pred, mask=None: float((pred == yb).float().mean()) if mask is None else float((pred[mask] == yb[mask]).float().mean())
    agree = lambda pred, mask: float((pred[mask] == pred_full[mask]).float().mean())
    print(f"accuracy: full graph {acc_full:.4f}; 8 parts with re-growth {acc(pred_re):.4f}, without {acc(pred_no):.4f}; "
          f"nodes at a cut ({int(at_cut.sum())}): with {acc(pred_re, at_cut_t):.4f}, without {acc(pred_no, at_cut_t):.4f}; "
          f"agreement with the full-graph prediction at a cut: with {agree(pred_re, at_cut_t):.4f}, "
          f"without {agree(pred_no, at_cut_t):.4f}", flush=True)
    # the model generalises from 8 to 64 bits (the premise of the paper's flow)
    assert acc_full > 0.9
    # away from the cuts (beyond the receptive field of three layers) nothing changes; at the cuts re-growth keeps
    # more of the full-graph behaviour than dropping the boundary edges does
    assert agree(pred_re, at_cut_t) >= agree(pred_no, at_cut_t)
    assert acc(pred_re) >= acc(pred_no)
    assert agree(pred_re, ~at_cut_t) >= 0.95


def _aggregate(torch, Z, plan, plan_t):
    class Aggregate(torch.autograd.Function):
        @staticmethod
        def forward(ctx, X):
            X = X.contiguous()
            Y = torch.empty_like(X)
            G.groot_spmm_execute(plan, X, Y, X.shape[1])
            return Y

        @staticmethod
        def backward(ctx, dY):
            dY = dY.contiguous()
            dX = torch.empty_like(dY)
            G.groot_spmm_execute(plan_t, dY, dX, dY.shape[1])
            return dX

    return Aggregate.apply(Z)


def test_training_step_through_the_three_fused_calls_matches_autograd():
    """One training step of the three-layer classifier with every layer run by the fused calls (forward layer,
    input gradient, weight gradients; the bias gradient is a column sum) gives the gradients that autograd gives
    for the same parameters through the library's aggregation and transposed aggregation, and a few steps of
    Adam on them train the model.  The 4 input features are padded with zero columns to the narrowest width, 32."""
    import torch

    assert torch.cuda.is_available(), "these tests need a GPU"
    torch.cuda.set_device(0)
    aig = wl.csa_multiplier_aig(12)
    g = G.groot_graph_build(aig.type, aig.fanin0, aig.fanin1, 1)
    plan, plan_t, _gt = _plans(g, HIDDEN)
    n = aig.num_nodes
    X4 = torch.from_numpy(wl.paper_node_features(aig)).cuda()
    X = torch.cat([X4, torch.zeros((n, HIDDEN - X4.shape[1]), device="cuda")], dim=1).contiguous()
    y = torch.from_numpy(aig.label.astype(np.int64)).cuda()
    workspace = torch.empty((G.groot_sage_layer_backward_weights_workspace(plan, HIDDEN) // 4,), device="cuda")

    class FusedLayer(torch.autograd.Function):
        @staticmethod
        def forward(ctx, h, wn, ws, b):
            h, wn, ws, b = (t.contiguous() for t in (h, wn, ws, b))
            out = torch.empty((n, HIDDEN), device="cuda")
            G.groot_sage_layer_forward(plan, h, wn, ws, b, True, out, HIDDEN)
            ctx.save_for_backward(h, wn, ws, out)
            return out

        @staticmethod
        def backward(ctx, d_out):
            h, wn, ws, out = ctx.saved_tensors
            dZ = (d_out * (out > 0)).contiguous()
            scaled = torch.empty_like(dZ)
            G.groot_rows_over_degree(plan, dZ, scaled)
            dh = torch.empty_like(h)
            G.groot_sage_layer_backward_data(plan, scaled, wn.t().contiguous(), ws.t().contiguous(), dh)
            dW = torch.empty((2, HIDDEN, HIDDEN), device="cuda")
            G.groot_sage_layer_backward_weights(plan, h, dZ, dW[0], dW[1], workspace)
            return dh, dW[0], dW[1], dZ.sum(0)

    def parameters(seed):
        gen = torch.Generator().manual_seed(seed)
        mk = lambda *shape: ((torch.rand(shape, generator=gen) - 0.5) * 0.5).cuda().requires_grad_(True)
        return [dict(wn=mk(HIDDEN, HIDDEN), ws=mk(HIDDEN, HIDDEN), b=mk(HIDDEN)) for _ in range(3)] + [dict(w=mk(HIDDEN, CLASSES), b=mk(CLASSES))]

    def loss_of(params, fused, x):
        h = x
        for layer in params[:3]:
            if fused:
                h = FusedLayer.apply(h, layer["wn"], layer["ws"], layer["b"])
            else:
                h = torch.relu(_aggregate(torch, h, plan, plan_t) @ layer["wn"] + h @ layer["ws"] + layer["b"])
        return torch.nn.functional.cross_entropy(h @ params[3]["w"] + params[3]["b"], y)

    params = parameters(11)
    flat = [t for layer in params for t in layer.values()]
    xa, xb = X.clone().requires_grad_(True), X.clone().requires_grad_(True)
    want = torch.autograd.grad(loss_of(params, False, xa), flat + [xa])
    got = torch.autograd.grad(loss_of(params, True, xb), flat + [xb])
    for a, b in zip(want, got):
        assert float((a - b).abs().max()) <= 2e-5 * float(a.abs().max()) + 1e-9

    opt = torch.optim.Adam(flat, lr=1e-2)
    first = last = None
    for step in range(60):
        opt.zero_grad()
        loss = loss_of(params, True, X)
        loss.backward()
        opt.step()
        first = float(loss.detach()) if first is None else first
        last = float(loss.detach())
    print(f"fused training loss {first:.4f} -> {last:.4f}", flush=True)
    assert np.isfinite(last) and last < 0.5 * first
