"""A step captured in a HIP graph (through torch.cuda.CUDAGraph on a side stream given to the
library with accordion_set_stream) replays to exactly what eager launches give: every replay is
checked, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2010_16248_amd import binding as B
from paper_2010_16248_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _contexts(method, layers, W, **kw):
    lt = H.layer_tuples(layers)
    q0 = None
    if method == B.ACC_POWERSGD:
        q0 = np.random.default_rng(1).standard_normal(sum(c for (_, r, c, m) in lt if m) * 2).astype(np.float32)
    args = {B.ACC_TOPK: (10, 1), B.ACC_POWERSGD: (2, 1), B.ACC_BATCH: (1, 1)}[method]
    mk = lambda: B.Accordion(method, lt, W, args[0], args[1], 100, 0.5, 1, q0, **kw)
    return mk(), mk()


@pytest.mark.parametrize("method,micro", [(B.ACC_TOPK, 1), (B.ACC_POWERSGD, 1), (B.ACC_BATCH, 2)])
@pytest.mark.parametrize("update", [False, True])
def test_captured_step_replays_like_eager(method, micro, update):
    import torch
    print(f"case graph method={method} update={update}", flush=True)
    layers = wl.make_layers([(64, 576, 1), (1, 8192 + 300, 0), (10, 512, 1), (1, 7, 0)])
    N = wl.total_params(layers)
    W = 2
    kw = dict(batch_multiplier=2, initial_level=0) if method == B.ACC_BATCH else {}
    lt = H.layer_tuples(layers)
    if method == B.ACC_BATCH:
        mk = lambda: B.Accordion(method, lt, W, 1, 1, 100, 0.5, 0, None, batch_multiplier=2)
        graphed, eager = mk(), mk()
    else:
        graphed, eager = _contexts(method, layers, W)
    rng = np.random.default_rng(3)
    dev = torch.device("cuda:0")
    # static buffers of the graph: `micro` sets of W gradients, output, weights, velocity
    static_g = [[torch.zeros(N, device=dev) for _ in range(W)] for _ in range(micro)]
    out_g, out_e = H.dev_out(N), H.dev_out(N)
    w0 = rng.standard_normal(N).astype(np.float32)
    wg, vg = H.to_dev(w0), H.to_dev(np.zeros(N, np.float32))
    we, ve = H.to_dev(w0), H.to_dev(np.zeros(N, np.float32))
    out_g.zero_(); out_e.zero_()

    def run(ctx, grads, out, wt, vel):
        for m in range(micro):
            if update:
                ctx.step_all_update(grads[m], wt, vel, 0.1, 0.9, 1e-4)
            else:
                ctx.step_all(grads[m], out)

    def fresh():
        return [[(rng.standard_normal(N) * 0.01).astype(np.float32) for _ in range(W)] for _ in range(micro)]

    # one eager step on both first: the captured step is a steady-state one
    g0 = fresh()
    run(graphed, [[H.to_dev(x) for x in ws] for ws in g0], out_g, wg, vg)
    run(eager, [[H.to_dev(x) for x in ws] for ws in g0], out_e, we, ve)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graphed.set_stream(side.cuda_stream)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(graphed, static_g, out_g, wg, vg)
    torch.cuda.synchronize()
    for rep in range(4):
        gs = fresh()
        for m in range(micro):
            for w in range(W):
                static_g[m][w].copy_(H.to_dev(gs[m][w]))
        torch.cuda.synchronize()
        graph.replay()
        run(eager, [[H.to_dev(x) for x in ws] for ws in gs], out_e, we, ve)
        torch.cuda.synchronize()
        # eager work of the program itself between the replays
        assert np.isfinite(float((out_e * 2.0).sum().item()))
        if update:
            H.assert_bits_equal(wg.cpu().numpy(), we.cpu().numpy(), f"replay {rep}: weights")
            H.assert_bits_equal(vg.cpu().numpy(), ve.cpu().numpy(), f"replay {rep}: velocity")
        else:
            H.assert_bits_equal(out_g.cpu().numpy(), out_e.cpu().numpy(), f"replay {rep}: output")
        assert np.array_equal(graphed.get_state(), eager.get_state()), f"replay {rep}: state"
        assert graphed.payload_words()[1] == eager.payload_words()[1]
    graphed.destroy()
    eager.destroy()
