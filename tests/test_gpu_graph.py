"""The three batched calls recorded into a HIP graph and replayed: every replay must give the bits of the eager run.

The library allocates nothing and takes every table as a kernel argument, so a captured sequence holds all it
needs; the inverse of the two large factors forks to the library's own streams (look-ahead of the blocked sweep,
the small factors beside the large ones) and joins back inside the capture.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2206_15143_amd as kf
from workloads.shapes import LayerSpec

import gpu_util as gu


def test_three_calls_captured_in_a_graph_replay_like_eager():
    layers = [LayerSpec("conv", 16, 16, 3, 1, 1, 8),            # A factor from autocorrelations
              LayerSpec("conv", 3, 8, 3, 1, 1, 8),              # patch extraction + block-tile kernel
              LayerSpec("conv", 8, 8, 1, 1, 0, 4),
              LayerSpec("linear", 70, 20, rows=40),
              LayerSpec("linear", 1300, 12, rows=24),           # two factors of order 1301: the two-level inverse with
              LayerSpec("linear", 1300, 12, rows=24)]           # its look-ahead on the library's second stream
    batch = 4
    inputs = gu.draw_inputs(layers, batch, 8800, "relu_normal", 0.05)
    scales = gu.scales_for(layers, batch)
    n = len(layers)
    descs = [kf.LayerDesc.from_spec(l, kf.KFAC_F32) for l in layers]
    b, h, w = gu.batch_args(layers, batch)
    acts = [gu.to_dev(i[0]) for i in inputs]
    gouts = [gu.to_dev(i[1]) for i in inputs]
    grads = [gu.to_dev(i[2]) for i in inputs]
    dA = [kf.kfac_dim_A(d) for d in descs]
    dG = [kf.kfac_dim_G(d) for d in descs]
    A_run = [torch.eye(a, device=gu.DEV) for a in dA]
    G_run = [torch.eye(g, device=gu.DEV) for g in dG]
    A_inv = [torch.zeros((a, a), device=gu.DEV) for a in dA]
    G_inv = [torch.zeros((g, g), device=gu.DEV) for g in dG]
    outs = [torch.zeros((g, a), device=gu.DEV) for a, g in zip(dA, dG)]
    info = torch.zeros((2 * n,), dtype=torch.int32, device=gu.DEV)
    sA = [s[0] for s in scales]
    sG = [s[1] for s in scales]
    ws = gu.workspace(kf.kfac_workspace_bytes_batched(descs, b, h, w))

    def reset():
        for t in A_run + G_run:
            t.copy_(torch.eye(t.shape[0], device=gu.DEV))
        for t in A_inv + G_inv + outs:
            t.fill_(float("nan"))
        info.fill_(-1)

    def step():
        kf.kfac_update_factors_batched(descs, acts, gouts, b, h, w, sA, sG, 0.9, A_run, G_run, ws)
        kf.kfac_invert_batched(descs, A_run, G_run, 0.02, 0.02, A_inv, G_inv, info, ws)
        kf.kfac_precondition_batched(descs, A_inv, G_inv, grads, outs, ws)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in A_run + G_run + A_inv + G_inv + outs] + [info.clone()]

    # eager reference (also the warm-up: one-time attribute calls and the second stream are made here)
    reset()
    step()
    ref = snapshot()
    assert int(ref[-1].abs().sum().item()) == 0
    # the eager run itself against the CPU oracle (the replays are then compared with it bit for bit)
    for i, l in enumerate(layers):
        want = gu.run_layer_oracle(l, inputs[i], scales[i], 0.9, 0.02)
        got = dict(A=ref[i].cpu().numpy(), G=ref[n + i].cpu().numpy(), A_inv=ref[2 * n + i].cpu().numpy(),
                   G_inv=ref[3 * n + i].cpu().numpy(), P=ref[4 * n + i].cpu().numpy(), info=np.zeros(2, dtype=np.int32))
        gu.check_layer(got, want, tag=f"eager layer {i}")

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    reset()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for replay in range(3):
        reset()                                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for k, (g, r) in enumerate(zip(got, ref)):
            assert torch.equal(g, r), f"replay {replay}: tensor {k} differs from the eager run"
