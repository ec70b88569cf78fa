"""A whole lsgd_step recorded into a HIP graph and replayed: the library enqueues kernels and device-to-device
copies only (no allocation, no memset, no host synchronisation on the step path), so a launch-bound loop can be
replayed as one graph.  Every replay is checked against the same step made eagerly, and against the oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_1905_10395_amd as L
from gpu_util import DEV, Pair, dev

pytestmark = pytest.mark.gpu


def build(x0, off, P, stream, batch_of):
    """population on `stream` with device buffers the test refills between steps"""
    W, ld = x0.shape
    G = len(off) - 1
    with torch.cuda.stream(stream):
        x = dev(x0)
        g = torch.zeros_like(x)
        m = torch.zeros_like(x)
        Z = torch.zeros((G + 1, ld), device=DEV)
        losses = torch.zeros(W, device=DEV)
    stream.synchronize()
    pop = L.Population(x, g, G, m=m, z_snapshot=Z, P=P, group_offsets=list(off), momentum=0.9, stream=stream,
                       largest_batch=batch_of(losses))
    return pop, x, g, m, Z, losses


@pytest.mark.parametrize("W,G,P,ld", [(8, 2, 4099, 4160), (16, 4, 300_000, 300_032)])
def test_step_replayed_from_a_graph_equals_eager_steps(W, G, P, ld):
    off = wl.equal_group_offsets(W, G)
    x0, _, _ = wl.stress_state(W, P, ld, seed=W + 5)
    eta, lamL, lamG = 0.05, 0.1, 0.05
    ext = lambda lo: L.ExternalBatch(lo)
    s_e, s_g = torch.cuda.Stream(), torch.cuda.Stream()
    pe, xe, ge, me, Ze, le = build(x0, off, P, s_e, ext)          # eager
    pg, xg, gg, mg, Zg, lg = build(x0, off, P, s_g, ext)          # graph
    be, bg = ext(le), ext(lg)
    ora = Pair(x0, off, P=P, momentum=0.9)                        # its oracle twin; its GPU half is unused

    def feed(t, g_buf, l_buf, stream):
        with torch.cuda.stream(stream):
            g_buf.copy_(dev(wl.stress_grad(W, P, ld, t, seed=W)))
            l_buf.copy_(dev(wl.stress_losses(W, t, seed=W + G)))

    # step 0 eagerly on both (first use configures the kernels; nothing of that kind may happen under capture)
    for pop, gb, lb, b, st in ((pe, ge, le, be, s_e), (pg, gg, lg, bg, s_g)):
        feed(0, gb, lb, st)
        pop.step(b, eta, lamL, lamG)
    torch.cuda.synchronize()
    # record one step (leaders re-selected every step: the same launches every time)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s_g):
        pg.step(bg, eta, lamL, lamG)
    torch.cuda.synchronize()
    assert torch.equal(xg, xe) and torch.equal(mg, me)             # recording executed nothing
    for t in range(1, 6):
        feed(t, ge, le, s_e)
        pe.step(be, eta, lamL, lamG)
        feed(t, gg, lg, s_g)                                       # eager work between the replays
        with torch.cuda.stream(s_g):
            graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(xg, xe), f"replay {t}: x differs from the eager step"
        assert torch.equal(mg, me), f"replay {t}: m differs from the eager step"
        assert torch.equal(Zg, Ze), f"replay {t}: kept leader copies differ"
        assert pg.get_leaders() == pe.get_leaders()
    # and the eager twin is the oracle's result
    ora.ora.x[:] = x0
    for t in range(0, 6):
        ora.ora.g[:] = wl.stress_grad(W, P, ld, t, seed=W)
        ora.ora.losses[:] = wl.stress_losses(W, t, seed=W + G)
        ora.ora.select(); ora.ora.update(eta, lamL, lamG)
    lead, gl = pe.get_leaders()
    assert lead == ora.ora.lead.tolist() and gl == int(ora.ora.glead[0])
    d = np.abs(xe.cpu().numpy()[:, :P] - ora.ora.x[:, :P]).max()
    assert d <= 1e-5 * np.abs(ora.ora.x[:, :P]).max()


def test_fused_mlp_step_replayed_from_a_graph():
    """The step with the most launches: forward, selection, copy capture, backward kernels that apply the update."""
    dims, W, G, B = [192, 256, 128, 10], 4, 2, 128
    P = wl.mlp_param_count(dims)
    ld = wl.padded_ld(P)
    x0 = wl.mlp_init(W, dims, ld=ld, seed=11)
    means = wl.gmm_means(dims[0], dims[-1], seed=11)
    off = wl.equal_group_offsets(W, G)
    eta, lamL, lamG = 0.05, 0.1, 0.05

    def make(stream):
        with torch.cuda.stream(stream):
            x = dev(x0); g = torch.zeros_like(x); m = torch.zeros_like(x)
            Z = torch.zeros((G + 1, ld), device=DEV)
            xb = torch.zeros((W, ld), dtype=torch.bfloat16, device=DEV)
            X = torch.zeros((W, B, dims[0]), dtype=torch.bfloat16, device=DEV)
            y = torch.zeros((W, B), dtype=torch.int32, device=DEV)
        stream.synchronize()
        batch = L.MLPBatch(dims, X, y)
        pop = L.Population(x, g, G, m=m, z_snapshot=Z, x_bf16=xb, P=P, group_offsets=list(off), momentum=0.9,
                           flags=L.WRITE_BF16_SHADOW | L.FUSED_MLP_UPDATE, largest_batch=batch, stream=stream)
        return pop, batch, x, m, Z, xb, X, y

    s_e, s_g = torch.cuda.Stream(), torch.cuda.Stream()
    pe, be, xe, me, Ze, xbe, Xe, ye = make(s_e)
    pg, bg, xg, mg, Zg, xbg, Xg, yg = make(s_g)

    def feed(t, X, y, stream):
        Xb, yb = wl.gmm_batch(W, B, means, t, seed=11)
        with torch.cuda.stream(stream):
            X.copy_(dev(Xb.view(np.int16)).view(torch.bfloat16)); y.copy_(dev(yb))

    for pop, b, X, y, st in ((pe, be, Xe, ye, s_e), (pg, bg, Xg, yg, s_g)):
        feed(0, X, y, st)
        pop.step(b, eta, lamL, lamG)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s_g):
        pg.step(bg, eta, lamL, lamG)
    torch.cuda.synchronize()
    assert torch.equal(xg, xe)
    for t in range(1, 5):
        feed(t, Xe, ye, s_e)
        pe.step(be, eta, lamL, lamG)
        feed(t, Xg, yg, s_g)
        with torch.cuda.stream(s_g):
            graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(xg, xe) and torch.equal(mg, me), f"replay {t}"
        assert torch.equal(Zg, Ze) and torch.equal(xbg, xbe), f"replay {t}: kept copies / bf16 copy"
        assert pg.get_leaders() == pe.get_leaders() and pg.get_losses() == pe.get_losses()
