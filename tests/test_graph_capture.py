"""The stage's microbatch loop under HIP graph capture.

The library only enqueues kernels (and one device-to-device copy) on the caller's stream, so a caller
may capture all forwards and all backward/accumulate pairs of a step into one graph and replay it
(worth it for launch-bound stages such as C1).  The replays are checked against the eager run bit by
bit, several times, with eager work between them; the optimizer step stays outside the graph because
its bias corrections are kernel arguments that change every step.
"""
import numpy as np
import pytest
import torch

import paper_2507_10392_amd as zs
from harness import dev, tdtype
from workloads import get_config, make_inputs
from workloads.configs import DTYPE_BF16

pytestmark = pytest.mark.gpu


def wide_cut_config():
    """A one-layer stage wide enough for its grouped weight gradients to leave partly filled rounds of 256x256 tiles
    (Wd: 33 x 8 = 264 tiles), so that the launches of the cut K range and the kernel that adds the partial tiles are
    captured as well."""
    cfg = get_config("C3t").with_(layers=1, hidden=2048, heads=16, ffn=8448, seq=256, num_microbatches=4, pair_wgrad=4)
    assert zs.wgrad_parts_scratch_bytes(cfg.ffn, cfg.hidden, cfg.tokens, cfg.tokens, 4, 1) > 0
    return cfg


@pytest.mark.parametrize("name", ["C1", "C3t", "wide-cut"])
def test_microbatch_loop_replays_from_a_graph(gpu_device, name):
    cfg = wide_cut_config() if name == "wide-cut" else get_config(name)
    print(f"[case] graph capture {name}", flush=True)
    inp = make_inputs(cfg, perturbed=True)
    M, T, H = cfg.num_microbatches, cfg.tokens, cfg.hidden
    td = tdtype(cfg)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        cc = zs.make_config(cfg)
        P, mem, _ = zs.query(cc)
        b, e = cc.shard_begin, cc.shard_end
        params = dev(inp.params, td)
        master = dev(inp.master[b:e]) if cfg.dtype == DTYPE_BF16 else None
        grad = torch.zeros(P, dtype=torch.float32, device="cuda")
        m = torch.zeros(max(e - b, 1), device="cuda")
        v = torch.zeros(max(e - b, 1), device="cuda")
        ws = torch.empty(mem["workspace"], dtype=torch.uint8, device="cuda")
        xs = [dev(inp.x[i], td) for i in range(M)]
        dys = [dev(inp.dy[i], td) for i in range(M)]
        ys = [torch.empty(T, H, dtype=td, device="cuda") for _ in range(M)]
        dxs = [torch.empty(T, H, dtype=td, device="cuda") for _ in range(M)]
        stage = zs.Stage(cc, params, master, grad, m, v, ws, stream=side)

        def loop():
            for i in range(M):
                stage.forward(i, xs[i], ys[i], None, None)
            for i in reversed(range(M)):
                stage.backward(i, dys[i], dxs[i], 1.0 / M)
                stage.accumulate(i)

        # eager run: the reference, and the warm-up that configures every kernel before the capture
        loop()
        side.synchronize()
        ref_grad = grad.clone()
        ref_y = [y.clone() for y in ys]
        ref_dx = [d.clone() for d in dxs]
        stage.optimizer_step(1)
        side.synchronize()
        ref_params = params.clone()
        # restore the state the reference started from
        params.copy_(dev(inp.params, td))
        if master is not None:
            master.copy_(dev(inp.master[b:e]))
        m.zero_()
        v.zero_()
        assert float(grad.abs().max()) == 0.0            # the optimizer step left the accumulator empty
        side.synchronize()

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            loop()
        for rep in range(3):
            for t in ys + dxs:                           # eager work between the replays
                t.fill_(float("nan"))
            grad.zero_()
            side.synchronize()
            graph.replay()
            side.synchronize()
            assert torch.equal(grad, ref_grad), f"replay {rep}: gradients differ from the eager run"
            for a, r in zip(ys + dxs, ref_y + ref_dx):
                assert torch.equal(a, r), f"replay {rep}: outputs differ from the eager run"
        stage.optimizer_step(1)                          # eager, on what the last replay accumulated
        side.synchronize()
        assert torch.equal(params, ref_params)
        # a further step made of a replay only: the library is told, then accepts the optimizer step
        with pytest.raises(zs.StageError):
            stage.optimizer_step(2)
        graph.replay()
        stage.graph_replayed(M)
        stage.optimizer_step(2)
        side.synchronize()
        assert bool(torch.isfinite(params.float()).all()) and not torch.equal(params, ref_params)
        stage.close()
    torch.cuda.synchronize()
