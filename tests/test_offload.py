"""Boundary-activation offload (Section 4.1.3, Section 5.4): with recompute on, the layer inputs of the forwarded
microbatches live in pinned host memory and the device keeps two microbatch slots.  The arithmetic is
untouched, so the step must match the oracle to the usual bar and the run without offload bit by bit, in
every call order."""
import numpy as np
import pytest
import torch

import paper_2507_10392_amd as zs
from harness import TOL, GpuStage, compare_optimizer, compare_step, dev, oracle_step, tdtype
from workloads import get_config, make_inputs

pytestmark = pytest.mark.gpu


def _same(a, b, cfg):
    assert np.array_equal(a["grad"], b["grad"])
    for key in ("loss",) if cfg.has_head else ("y",):
        for u, v in zip(a[key], b[key]):
            assert np.array_equal(np.asarray(u), np.asarray(v))
    if not cfg.has_embed:
        for u, v in zip(a["dx"], b["dx"]):
            assert np.array_equal(u, v)


@pytest.mark.parametrize("name,M", [("C4bt", None), ("C3t", 5), ("C5t", 4), ("C1", 4), ("C2t", 1)])
def test_offloaded_step_matches_oracle_and_the_resident_run(gpu_device, name, M):
    base = get_config(name).with_(recompute=1)
    M = base.num_microbatches if M is None else M
    print(f"[case] offload {name} M={M}", flush=True)
    inp = make_inputs(base, perturbed=True, num_microbatches=M)
    tol = TOL[base.dtype]
    outs = []
    TH = base.tokens * base.hidden * (2 if base.dtype else 4)
    per_mb = (base.layers + base.has_head) * TH          # one microbatch's boundary activations
    for off in (0, 1):
        cfg = base.with_(offload_acts=off)
        g = GpuStage(cfg, inp, max_microbatches=M)
        assert g.mem["host_stash"] == (M * per_mb if off else 0)
        out = g.run_microbatches(inp, M=M)
        if off and not cfg.has_embed:
            # what reached the host: each microbatch's first layer input is the stage input itself
            torch.cuda.synchronize()
            td = tdtype(cfg)
            for i in range(M):
                first = g.host[i * per_mb:i * per_mb + TH].view(td)
                assert torch.equal(first, dev(inp.x[i], td).cpu().reshape(-1))
        outs.append(out)
        if off:
            ora = oracle_step(cfg, inp, M=M)
            compare_step(cfg, out, ora, tol)
            res = g.step(1)
            compare_optimizer(cfg, inp, g.shard, out["grad"], res, ora["grad"], tol)
        g.stage.close()
    _same(outs[0], outs[1], base)


def _run_schedule(cfg, inp, M, schedule):
    """schedule: list of ('F', i) / ('B', i).  Returns y, dx per microbatch and the gradient."""
    g = GpuStage(cfg, inp, max_microbatches=M)
    td = tdtype(cfg)
    T, H = cfg.tokens, cfg.hidden
    xs = [dev(inp.x[i], td) for i in range(len(inp.x))]
    dys = [dev(inp.dy[i], td) for i in range(len(inp.dy))]
    ys, dxs = {}, {}
    n = 0
    for kind, slot, data in schedule:
        if kind == "F":
            ys[data] = torch.empty(T, H, dtype=td, device="cuda")
            g.stage.forward(slot, xs[data], ys[data], None, None)
        else:
            dxs[data] = torch.empty(T, H, dtype=td, device="cuda")
            g.stage.backward(slot, dys[data], dxs[data], 1.0)
            g.stage.accumulate(slot)
            n += 1
    torch.cuda.synchronize()
    out = {"grad": g.grad.cpu().numpy().copy(), "y": [ys[i].float().cpu().numpy() for i in sorted(ys)],
           "dx": [dxs[i].float().cpu().numpy() for i in sorted(dxs)]}
    g.stage.close()
    return out


SCHEDULES = {
    # all forwards, then backwards in the SAME order: the prefetch guess (mb - 1) is always wrong
    "ascending": [("F", i, i) for i in range(5)] + [("B", i, i) for i in range(5)],
    # one-forward-one-backward with slots reused for later data while older microbatches wait
    "interleaved": [("F", 0, 0), ("F", 1, 1), ("F", 2, 2), ("B", 0, 0), ("F", 0, 3), ("B", 2, 2), ("B", 1, 1),
                    ("F", 3, 4), ("F", 1, 5), ("B", 0, 3), ("B", 1, 5), ("B", 3, 4)],
    # backwards jump around
    "scattered": [("F", i, i) for i in range(6)] + [("B", i, i) for i in (3, 0, 5, 4, 1, 2)],
}


@pytest.mark.parametrize("sched", sorted(SCHEDULES))
def test_offload_in_any_call_order(gpu_device, sched):
    """Whatever the order, the device slots and the host copies must hand every backward its own microbatch."""
    print(f"[case] offload schedule {sched}", flush=True)
    base = get_config("C4bt").with_(recompute=1)
    schedule = SCHEDULES[sched]
    ndata = 1 + max(d for _, _, d in schedule)
    M = 1 + max(s for _, s, _ in schedule)
    inp = make_inputs(base, perturbed=True, num_microbatches=ndata)
    a = _run_schedule(base.with_(offload_acts=0), inp, M, schedule)
    b = _run_schedule(base.with_(offload_acts=1), inp, M, schedule)
    _same(a, b, base)
    assert np.abs(b["grad"]).max() > 0


def test_offload_over_two_steps(gpu_device):
    """The slots carry state from one step to the next; a second step must still be exact."""
    print("[case] offload two steps", flush=True)
    base = get_config("C3t").with_(recompute=1)
    inp = make_inputs(base, perturbed=True, num_microbatches=4)
    res = []
    for off in (0, 1):
        g = GpuStage(base.with_(offload_acts=off), inp, max_microbatches=4)
        g.run_microbatches(inp, M=4)
        g.step(1)
        out = g.run_microbatches(inp, M=4)
        r = g.step(2)
        res.append((out, r["params"].copy()))
        g.stage.close()
    _same(res[0][0], res[1][0], base)
    assert np.array_equal(res[0][1], res[1][1])


def test_offload_argument_and_state_errors(gpu_device):
    print("[case] offload errors", flush=True)
    cfg = get_config("C4bt")
    with pytest.raises(zs.StageError) as ei:
        zs.query(zs.make_config(cfg.with_(recompute=0, offload_acts=1)))
    assert ei.value.code == zs.STAGE_ERR_ARG
    inp = make_inputs(cfg.with_(recompute=1), num_microbatches=2)
    # not configured for offload: attaching is an argument error
    g = GpuStage(cfg.with_(recompute=1, offload_acts=0), inp, max_microbatches=2)
    host = torch.empty(1 << 20, dtype=torch.uint8, pin_memory=True)
    with pytest.raises(zs.StageError) as ei:
        g.stage.attach_host_stash(host)
    assert ei.value.code == zs.STAGE_ERR_ARG
    g.stage.close()
    # configured, nothing attached yet: forward refuses
    ocfg = cfg.with_(recompute=1, offload_acts=1)
    cc = zs.make_config(ocfg, max_microbatches=2)
    P, mem, _ = zs.query(cc)
    td = tdtype(ocfg)
    b, e = cc.shard_begin, cc.shard_end
    bufs = dict(params=dev(inp.params, td), master=dev(inp.master[b:e]), grad=torch.zeros(P, device="cuda"),
                m=torch.zeros(e - b, device="cuda"), v=torch.zeros(e - b, device="cuda"),
                ws=torch.empty(mem["workspace"], dtype=torch.uint8, device="cuda"))
    st = zs.Stage(cc, bufs["params"], bufs["master"], bufs["grad"], bufs["m"], bufs["v"], bufs["ws"])
    x = dev(inp.x[0], td)
    y = torch.empty_like(x)
    with pytest.raises(zs.StageError) as ei:
        st.forward(0, x, y)
    assert ei.value.code == zs.STAGE_ERR_STATE
    with pytest.raises(zs.StageError) as ei:     # too small
        st.attach_host_stash(torch.empty(mem["host_stash"] - 1, dtype=torch.uint8, pin_memory=True))
    assert ei.value.code == zs.STAGE_ERR_ARG
    with pytest.raises(zs.StageError) as ei:     # pageable memory
        st.attach_host_stash(torch.empty(mem["host_stash"], dtype=torch.uint8))
    assert ei.value.code == zs.STAGE_ERR_ARG
    with pytest.raises(zs.StageError) as ei:     # device memory
        st.attach_host_stash(torch.empty(mem["host_stash"], dtype=torch.uint8, device="cuda"))
    assert ei.value.code == zs.STAGE_ERR_ARG
    good = torch.empty(mem["host_stash"], dtype=torch.uint8, pin_memory=True)
    st.attach_host_stash(good)
    with pytest.raises(zs.StageError) as ei:
        st.attach_host_stash(good)
    assert ei.value.code == zs.STAGE_ERR_STATE
    with pytest.raises(zs.StageError) as ei:
        st.graph_replayed(1)
    assert ei.value.code == zs.STAGE_ERR_ARG
    st.forward(0, x, y)                           # and now it runs
    dx = torch.empty_like(x)
    st.backward(0, dev(inp.dy[0], td), dx, 1.0)
    st.accumulate(0)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dx.float()).all())
    st.close()
