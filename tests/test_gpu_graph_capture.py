"""A layer call can be recorded into a HIP graph once its buffers exist (no allocation, no
synchronisation and no memset in the steady state) and replayed with new inputs."""
import numpy as np
import pytest
import torch

import saga_inputs as si
from helpers import new_context

pytestmark = pytest.mark.gpu


def _two_layer(ctx, graph, X, H, Y, wl, W2):
    ctx.layer_forward(graph, X, H, edge_op="mul_weight", W=wl.W_dev, act="relu")
    ctx.layer_forward(graph, H, Y, edge_op="mul_weight", W=W2, act="none")


@pytest.mark.parametrize("kind", ["gcn2", "gated"])
def test_replays_equal_eager_results(kind):
    with new_context() as ctx:
        if kind == "gcn2":
            wl = si.workload(2, scale=12)
            n = wl.graph.n
            graph = ctx.graph_create_csc(n, wl.graph.col_ptr.cuda(), wl.graph.row_idx.cuda())
            graph.set_edge_data(wl.edge_weight.cuda())
            wl.W_dev, W2 = wl.W.cuda(), wl.extra["W2"].cuda()
            X = wl.X.cuda().clone()
            H = torch.empty(n, 16, device="cuda")
            Y = torch.empty(n, 3, device="cuda")
            run = lambda: _two_layer(ctx, graph, X, H, Y, wl, W2)
        else:
            wl = si.workload(4, scale=12, f_in=64, f_out=32)
            n = wl.graph.n
            graph = ctx.graph_create_csc(n, wl.graph.col_ptr.cuda(), wl.graph.row_idx.cuda())
            Wg, bg, Wm, W = wl.W_gate.cuda(), wl.b_gate.cuda(), wl.W_msg.cuda(), wl.W.cuda()
            X = wl.X.cuda().clone()
            Y = torch.empty(n, 32, device="cuda")
            run = lambda: ctx.layer_forward(graph, X, Y, edge_op="gated", W_gate=Wg, b_gate=bg, W_msg=Wm, W=W, act="relu")
        inputs = [X.clone(), torch.roll(X, 7, 0) * 0.5, -X + 1.0, X.clone()]
        eager = []
        for inp in inputs:                      # eager results; the first call also sizes every workspace
            X.copy_(inp)
            run()
            torch.cuda.synchronize()
            eager.append(Y.clone())
        g = torch.cuda.CUDAGraph()
        X.copy_(inputs[0])
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            run()
        torch.cuda.synchronize()
        for k, inp in enumerate(inputs):
            X.copy_(inp)
            Y.fill_(float("nan"))
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(Y, eager[k]), f"replay {k} differs from the eager result"
            # eager work of the same library between replays must not disturb the recorded buffers' contents
            junk = torch.empty_like(Y)
            X2 = torch.randn_like(X)
            if kind == "gcn2":
                H2 = torch.empty(n, 16, device="cuda")
                ctx.layer_forward(graph, X2, H2, edge_op="mul_weight", W=wl.W_dev, act="relu")
            else:
                ctx.layer_forward(graph, X2, junk, edge_op="gated", W_gate=Wg, b_gate=bg, W_msg=Wm, W=W, act="relu")
            torch.cuda.synchronize()
        graph.destroy()
