"""Forward and backward passes composed: the two GCN layers of configuration 2's model (500 -> 16 -> 3, scaled down),
gradient of a linear loss with respect to both weight matrices and the input, against the oracle's chain; and the same
four calls recorded into a HIP graph."""
import numpy as np
import pytest
import torch

import oracle
import saga_inputs as si
from helpers import TOL_F32, assert_sum_close, new_context

pytestmark = pytest.mark.gpu


def _setup(ctx, scale=12):
    wl = si.workload(2, scale=scale)
    g = wl.graph
    graph = ctx.graph_create_csc(g.n, g.col_ptr.cuda(), g.row_idx.cuda())
    graph.set_edge_data(wl.edge_weight.cuda())
    return wl, graph


class _Step:
    """Buffers and the four calls of one training step's forward and backward pass."""

    def __init__(self, ctx, graph, wl, R):
        n = wl.graph.n
        d = "cuda"
        self.ctx, self.graph = ctx, graph
        self.X, self.W1, self.W2, self.R = wl.X.to(d).clone(), wl.W.to(d), wl.extra["W2"].to(d), R.to(d)
        self.A1, self.H = torch.empty(n, 500, device=d), torch.empty(n, 16, device=d)
        self.A2, self.Y = torch.empty(n, 16, device=d), torch.empty(n, 3, device=d)
        self.dH, self.dX = torch.empty(n, 16, device=d), torch.empty(n, 500, device=d)
        self.dW1, self.dW2 = torch.empty(500, 16, device=d), torch.empty(16, 3, device=d)

    def run(self):
        c, g = self.ctx, self.graph
        c.layer_forward(g, self.X, self.H, edge_op="mul_weight", W=self.W1, act="relu", accum_out=self.A1)
        c.layer_forward(g, self.H, self.Y, edge_op="mul_weight", W=self.W2, act="none", accum_out=self.A2)
        # loss = sum(R * Y): dY = R
        c.layer_backward(g, self.A2, self.R, self.W2, self.dW2, edge_op="mul_weight", act="none", dX=self.dH)
        c.layer_backward(g, self.A1, self.dH, self.W1, self.dW1, Y=self.H, edge_op="mul_weight", act="relu", dX=self.dX)


def test_two_layer_gcn_gradients_match_the_oracle_chain():
    with new_context() as ctx:
        wl, graph = _setup(ctx)
        g = wl.graph
        cp, ri, w = g.col_ptr.numpy(), g.row_idx.numpy(), wl.edge_weight.numpy()
        R = si.normal_features(g.n, 3, 11)
        step = _Step(ctx, graph, wl, R)
        step.run()
        torch.cuda.synchronize()
        W1, W2 = wl.W.numpy(), wl.extra["W2"].numpy()
        f1 = oracle.layer(cp, ri, wl.X.numpy(), "mul_weight", w, W=W1, act="relu")
        H = f1["Y"].astype(np.float32)
        f2 = oracle.layer(cp, ri, H, "mul_weight", w, W=W2, act="none")
        b2 = oracle.layer_backward(cp, ri, H, f2["A"], R.numpy(), W2, "mul_weight", w, act="none")
        dH = b2["dX"].astype(np.float32)
        b1 = oracle.layer_backward(cp, ri, wl.X.numpy(), f1["A"], dH, W1, "mul_weight", w, act="relu")
        assert_sum_close(step.Y.cpu().numpy(), f2["Y"], f2["Y_abs"], TOL_F32, "Y")
        assert_sum_close(step.dW2.cpu().numpy(), b2["dW"], b2["dW_abs"], TOL_F32, "dW2")
        assert_sum_close(step.dH.cpu().numpy(), b2["dX"], b2["dX_abs"], TOL_F32, "dH")
        # layer 1's gradients inherit layer 2's rounding through dH and the ReLU mask: the mask is the same unless a hidden
        # unit sits within rounding of zero, which these inputs avoid; the tolerance is doubled for the inherited error
        mask_gpu, mask_ref = (step.H.cpu().numpy() > 0), (f1["Y"] > 0)
        assert (mask_gpu == mask_ref).all()
        assert_sum_close(step.dW1.cpu().numpy(), b1["dW"], b1["dW_abs"], 2 * TOL_F32, "dW1")
        assert_sum_close(step.dX.cpu().numpy(), b1["dX"], b1["dX_abs"], 2 * TOL_F32, "dX")
        graph.destroy()


def test_training_step_records_into_a_hip_graph():
    with new_context() as ctx:
        wl, graph = _setup(ctx, scale=11)
        R = si.normal_features(wl.graph.n, 3, 12)
        step = _Step(ctx, graph, wl, R)
        inputs = [step.X.clone(), torch.roll(step.X, 5, 0) * 0.5, -step.X + 0.25]
        eager = []
        for inp in inputs:                      # the first call builds both edge orders and sizes every workspace
            step.X.copy_(inp)
            step.run()
            torch.cuda.synchronize()
            eager.append((step.dW1.clone(), step.dW2.clone(), step.dX.clone()))
        hg = torch.cuda.CUDAGraph()
        step.X.copy_(inputs[0])
        torch.cuda.synchronize()
        with torch.cuda.graph(hg):
            step.run()
        torch.cuda.synchronize()
        for k, inp in enumerate(inputs):
            step.X.copy_(inp)
            for t in (step.dW1, step.dW2, step.dX):
                t.fill_(float("nan"))
            hg.replay()
            torch.cuda.synchronize()
            for got, ref, name in zip((step.dW1, step.dW2, step.dX), eager[k], ("dW1", "dW2", "dX")):
                assert torch.equal(got, ref), f"replay {k}: {name} differs from the eager result"
            junk = torch.empty_like(step.H)      # eager work of the same library between replays
            ctx.layer_forward(graph, torch.randn_like(step.X), junk, edge_op="mul_weight", W=step.W1, act="relu")
            torch.cuda.synchronize()
        graph.destroy()
