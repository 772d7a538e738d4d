"""Several ministages time-multiplexed on one GPU (Sections 4.1.1, 4.1.2, 5.1, 5.4): K stages of one shape share
two parameter slots and two optimizer-state slots on the device, everything else waits in pinned host memory,
and each ministage's optimizer runs right after its backward.  Checked against the oracle of the whole
K x L-layer stack and, bit by bit over two steps, against K stages that stay resident."""
import types

import numpy as np
import pytest
import torch

import paper_2507_10392_amd as zs
from harness import TOL, GpuStage, dev, hp32, rel_err, tdtype
from oracle import stage_oracle as so
from workloads import get_config, make_inputs

pytestmark = pytest.mark.gpu


class Group:
    """Host block, arena and the Ministages object for K ministages cut from a K*L-layer input set."""

    def __init__(self, cfg, K, inp_full):
        self.cfg, self.K = cfg, K
        self.cc = zs.make_config(cfg)
        self.P, self.smem, _ = zs.query(self.cc)
        self.mem = zs.ministages_query(self.cc, K)
        self.td = tdtype(cfg)
        self.b, self.e = self.cc.shard_begin, self.cc.shard_end
        m = self.mem
        self.host = torch.zeros(m["host_bytes"], dtype=torch.uint8).pin_memory()
        for k in range(K):
            self.params(k).copy_(torch.from_numpy(inp_full.params[k * self.P:(k + 1) * self.P]).to(self.td))
            if m["off_master"] >= 0:
                self.state(k, "master").copy_(torch.from_numpy(inp_full.master[k * self.P + self.b:k * self.P + self.e]))
        self.arena = torch.empty(m["device_bytes"], dtype=torch.uint8, device="cuda")
        self.ms = zs.Ministages(self.cc, K, self.host, self.arena)
        g0 = min(K, 2) * m["param_slot"] + min(K, 3) * m["state_slot"]
        self.grad = self.arena[g0:g0 + 4 * self.P].view(torch.float32)     # the shared gradient buffer (test only)

    def params(self, k):
        o = k * self.mem["per_stage_host"] + self.mem["off_params"]
        return self.host[o:o + self.P * self.host.new_empty(0, dtype=self.td).element_size()].view(self.td)

    def state(self, k, which):
        o = k * self.mem["per_stage_host"] + self.mem["off_" + which]
        return self.host[o:o + 4 * (self.e - self.b)].view(torch.float32)


def gpipe_step(fwd, bwd, acc, opt, K, M, xs, dys, T, H, td, t, grads_of=None):
    """All forwards ministage by ministage, then the backwards in reverse with each ministage's optimizer
    right after its own backward.  Returns final outputs, first-ministage input gradients, per-ministage gradients."""
    cur = xs
    for k in range(K):
        nxt = [torch.empty(T, H, dtype=td, device="cuda") for _ in range(M)]
        for i in range(M):
            fwd(k, i, cur[i], nxt[i])
        cur = nxt
    ys = cur
    g = dys
    grads = [None] * K
    for k in reversed(range(K)):
        nxt = [torch.empty(T, H, dtype=td, device="cuda") for _ in range(M)]
        for i in reversed(range(M)):
            bwd(k, i, g[i], nxt[i], 1.0)
            acc(k, i)
        if grads_of is not None:
            torch.cuda.synchronize()
            grads[k] = grads_of(k).clone()
        opt(k, t)
        g = nxt
    torch.cuda.synchronize()
    return ys, g, grads


@pytest.mark.parametrize("name,K,L,M", [("C3t", 3, 2, 3), ("C1", 4, 1, 2), ("C2t", 2, 2, 2), ("C4at", 1, 2, 2)])
def test_ministages_match_the_oracle_of_the_whole_stack(gpu_device, name, K, L, M):
    cfg = get_config(name).with_(layers=L, num_microbatches=M, has_embed=0, has_head=0, vocab=0, recompute=0)
    full = cfg.with_(layers=K * L)
    print(f"[case] ministages {name} K={K} L={L} M={M}", flush=True)
    inp = make_inputs(full, perturbed=True)
    tol = TOL[cfg.dtype]
    G = Group(cfg, K, inp)
    td, T, H = G.td, cfg.tokens, cfg.hidden
    xs = [dev(inp.x[i], td) for i in range(M)]
    dys = [dev(inp.dy[i], td) for i in range(M)]
    ys, dxs, grads = gpipe_step(G.ms.forward, G.ms.backward, G.ms.accumulate, G.ms.optimizer_step, K, M, xs, dys, T, H, td, 1,
                                grads_of=lambda k: G.grad)
    ora = so.stage_step(hp32(full), inp.params, inp.x[:M], inp.dy[:M])
    for i in range(M):
        assert rel_err(ys[i].float().cpu().numpy(), ora["y"][i]) <= tol
        assert rel_err(dxs[i].float().cpu().numpy(), ora["dx"][i]) <= tol
    P = G.P
    for k in range(K):
        gk = grads[k].cpu().numpy().astype(np.float64)
        for nm, off, r, c in so.layout(cfg):
            o = ora["grad"][k * P + off:k * P + off + r * c]
            assert rel_err(gk[off:off + r * c], o) <= tol, (k, nm)
    # the optimizer of every ministage: oracle AdamW fed the GPU's own gradients must land on what came back to the host
    c32 = hp32(cfg)
    b, e = G.b, G.e
    for k in range(K):
        p0 = inp.master[k * P:(k + 1) * P].astype(np.float64)
        new, m_o, v_o = so.stage_optimizer_step(c32, p0, grads[k].cpu().numpy().astype(np.float64), np.zeros(e - b), np.zeros(e - b), 1, (b, e))
        assert rel_err(G.state(k, "m").numpy(), m_o) <= 1e-6 and rel_err(G.state(k, "v").numpy(), v_o) <= 1e-6
        got = (G.state(k, "master") if cfg.dtype else G.params(k)[b:e]).numpy().astype(np.float64)
        assert np.abs(got - new[b:e]).max() <= 1e-6 * cfg.lr + 1.2e-7 * np.abs(new[b:e]).max()
        if cfg.dtype:   # the working copy is the bf16 rounding of the master, the rest of the parameters is untouched
            assert torch.equal(G.params(k)[b:e], G.state(k, "master").to(torch.bfloat16))
            assert torch.equal(G.params(k)[e:], torch.from_numpy(inp.params[k * P + e:(k + 1) * P]).to(td))
    h2d, d2h = G.ms.traffic()
    E = 2 if cfg.dtype else 4
    per_state = (e - b) * 4 * (3 if cfg.dtype else 2)
    assert d2h == K * ((e - b) * E + per_state)
    assert h2d >= K * (P * E + per_state) and h2d <= (3 * K) * P * E + K * per_state
    assert float(G.grad.abs().max()) == 0.0          # freed by the last optimizer step
    G.ms.close()


def test_ministages_equal_resident_stages_over_two_steps(gpu_device):
    """The same K stages kept on the device, driven in the same order, give the same bits: outputs, input
    gradients and, after two steps, parameters, master copy and both moments (through the host block)."""
    K, L, M = 3, 2, 2
    cfg = get_config("C3t").with_(layers=L, num_microbatches=M)
    full = cfg.with_(layers=K * L)
    print("[case] ministages vs resident stages", flush=True)
    inp = make_inputs(full, perturbed=True)
    td, T, H = tdtype(cfg), cfg.tokens, cfg.hidden
    xs = [dev(inp.x[i], td) for i in range(M)]
    dys = [dev(inp.dy[i], td) for i in range(M)]
    G = Group(cfg, K, inp)
    P = G.P
    res = [GpuStage(cfg, types.SimpleNamespace(params=inp.params[k * P:(k + 1) * P], master=inp.master[k * P:(k + 1) * P]))
           for k in range(K)]
    for t in (1, 2):
        a = gpipe_step(G.ms.forward, G.ms.backward, G.ms.accumulate, G.ms.optimizer_step, K, M, xs, dys, T, H, td, t)
        r = gpipe_step(lambda k, i, x, y: res[k].stage.forward(i, x, y), lambda k, i, dy, dx, ls: res[k].stage.backward(i, dy, dx, ls),
                       lambda k, i: res[k].stage.accumulate(i), lambda k, tt: res[k].stage.optimizer_step(tt), K, M, xs, dys, T, H, td, t)
        for u, v in zip(a[0] + a[1], r[0] + r[1]):
            assert torch.equal(u, v), f"step {t}"
    b, e = G.b, G.e
    for k in range(K):
        assert torch.equal(G.params(k)[b:e], res[k].params[b:e].cpu())
        assert torch.equal(G.state(k, "master"), res[k].master.cpu())
        assert torch.equal(G.state(k, "m"), res[k].m.cpu()) and torch.equal(G.state(k, "v"), res[k].v.cpu())
        assert float(G.state(k, "v").abs().max()) > 0
        res[k].stage.close()
    G.ms.close()


@pytest.mark.parametrize("recompute,offload,group", [(1, 0, 0), (1, 1, 0), (0, 0, 4)])
def test_ministages_with_recompute_offload_and_grouped_gradients(gpu_device, recompute, offload, group):
    """The options of a stage pass through to the ministages: per-layer recompute, boundary activations in the host
    block (two microbatch slots per ministage on the device), weight gradients in groups.  All ministages share
    one scratch buffer.  Same bits as resident stages with the same options, over two steps."""
    K, L, M = 3, 2, 4
    cfg = get_config("C3t").with_(layers=L, num_microbatches=M, recompute=recompute, offload_acts=offload, pair_wgrad=group)
    full = cfg.with_(layers=K * L)
    print(f"[case] ministages recompute={recompute} offload={offload} group={group}", flush=True)
    inp = make_inputs(full, perturbed=True)
    td, T, H = tdtype(cfg), cfg.tokens, cfg.hidden
    xs = [dev(inp.x[i], td) for i in range(M)]
    dys = [dev(inp.dy[i], td) for i in range(M)]
    G = Group(cfg, K, inp)
    P = G.P
    assert (G.mem["off_stash"] >= 0) == bool(offload)
    res = [GpuStage(cfg, types.SimpleNamespace(params=inp.params[k * P:(k + 1) * P], master=inp.master[k * P:(k + 1) * P]))
           for k in range(K)]
    for t in (1, 2):
        a = gpipe_step(G.ms.forward, G.ms.backward, G.ms.accumulate, G.ms.optimizer_step, K, M, xs, dys, T, H, td, t)
        r = gpipe_step(lambda k, i, x, y: res[k].stage.forward(i, x, y), lambda k, i, dy, dx, ls: res[k].stage.backward(i, dy, dx, ls),
                       lambda k, i: res[k].stage.accumulate(i), lambda k, tt: res[k].stage.optimizer_step(tt), K, M, xs, dys, T, H, td, t)
        for u, v in zip(a[0] + a[1], r[0] + r[1]):
            assert torch.equal(u, v), f"step {t}"
    b, e = G.b, G.e
    for k in range(K):
        assert torch.equal(G.params(k)[b:e], res[k].params[b:e].cpu())
        assert torch.equal(G.state(k, "m"), res[k].m.cpu()) and torch.equal(G.state(k, "v"), res[k].v.cpu())
        res[k].stage.close()
    # against the oracle too: one more step from the same state is not needed, the first step's outputs are
    ora = so.stage_step(hp32(full), inp.params, inp.x[:M], inp.dy[:M])
    G2 = Group(cfg, K, inp)
    ys, dxs, _ = gpipe_step(G2.ms.forward, G2.ms.backward, G2.ms.accumulate, G2.ms.optimizer_step, K, M, xs, dys, T, H, td, 1)
    for i in range(M):
        assert rel_err(ys[i].float().cpu().numpy(), ora["y"][i]) <= TOL[cfg.dtype]
        assert rel_err(dxs[i].float().cpu().numpy(), ora["dx"][i]) <= TOL[cfg.dtype]
    G.ms.close()
    G2.ms.close()


def test_ministages_state_and_argument_errors(gpu_device):
    print("[case] ministages errors", flush=True)
    K, M = 2, 1
    cfg = get_config("C4at").with_(layers=1, num_microbatches=M)
    inp = make_inputs(cfg.with_(layers=K), perturbed=True)
    cc = zs.make_config(cfg)
    mem = zs.ministages_query(cc, K)
    arena = torch.empty(mem["device_bytes"], dtype=torch.uint8, device="cuda")
    with pytest.raises(zs.StageError) as ei:      # pageable host memory
        zs.Ministages(cc, K, torch.zeros(mem["host_bytes"], dtype=torch.uint8), arena)
    assert ei.value.code == zs.STAGE_ERR_ARG
    pinned = torch.zeros(mem["host_bytes"], dtype=torch.uint8).pin_memory()
    with pytest.raises(zs.StageError) as ei:      # host block too small
        zs.Ministages(cc, K, pinned[:-256], arena)
    assert ei.value.code == zs.STAGE_ERR_ARG
    with pytest.raises(zs.StageError) as ei:      # arena too small
        zs.Ministages(cc, K, pinned, arena[:-256])
    assert ei.value.code == zs.STAGE_ERR_WORKSPACE
    G = Group(cfg, K, inp)
    td, T, H = G.td, cfg.tokens, cfg.hidden
    x, dy = dev(inp.x[0], td), dev(inp.dy[0], td)
    y0, y1, d1, d0 = (torch.empty(T, H, dtype=td, device="cuda") for _ in range(4))
    with pytest.raises(zs.StageError) as ei:
        G.ms.forward(2, 0, x, y0)
    assert ei.value.code == zs.STAGE_ERR_ARG
    G.ms.forward(0, 0, x, y0)
    G.ms.forward(1, 0, y0, y1)
    with pytest.raises(zs.StageError) as ei:      # nothing accumulated yet
        G.ms.optimizer_step(1, 1)
    assert ei.value.code == zs.STAGE_ERR_STATE
    G.ms.backward(1, 0, dy, d1)
    G.ms.accumulate(1, 0)
    with pytest.raises(zs.StageError) as ei:      # ministage 1's gradients are still in the shared buffer
        G.ms.backward(0, 0, d1, d0)
    assert ei.value.code == zs.STAGE_ERR_STATE
    G.ms.optimizer_step(1, 1)
    G.ms.backward(0, 0, d1, d0)
    G.ms.accumulate(0, 0)
    G.ms.optimizer_step(0, 1)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(d0.float()).all())
    G.ms.close()


def test_ministages_at_full_shape_equal_resident_stages(gpu_device):
    """7B-class layer shape, one layer per ministage, two microbatches: here a ministage computes for less time
    than its parameters and optimizer state need to travel, so every wait between the two streams is exercised.
    Inputs are drawn on the device (same distributions as the benchmark); the property checked holds at any
    size: same bits as three stages that stay resident, after two steps."""
    K, M = 3, 2
    cfg = get_config("C3").with_(layers=1, num_microbatches=M, pair_wgrad=1)
    print(f"[case] ministages full shape K={K}: T={cfg.tokens} H={cfg.hidden} F={cfg.ffn}", flush=True)
    cc = zs.make_config(cfg)
    P, smem, _ = zs.query(cc)
    mem = zs.ministages_query(cc, K)
    b, e = cc.shard_begin, cc.shard_end
    T, H, td = cfg.tokens, cfg.hidden, torch.bfloat16
    gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
    host = torch.zeros(mem["host_bytes"], dtype=torch.uint8).pin_memory()
    res = []
    for k in range(K):
        p = torch.empty(P, dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=gen)
        for nm, off, r, c in zs.layout(cc):
            if r == 1:
                p[off:off + c] = 1.0
        pb = p.to(td)
        o = k * mem["per_stage_host"]
        host[o + mem["off_params"]:o + mem["off_params"] + 2 * P].view(td).copy_(pb)
        host[o + mem["off_master"]:o + mem["off_master"] + 4 * (e - b)].view(torch.float32).copy_(pb[b:e].float())
        r_ = types.SimpleNamespace(params=pb, master=pb[b:e].float().contiguous(), grad=torch.zeros(P, device="cuda"),
                                   m=torch.zeros(e - b, device="cuda"), v=torch.zeros(e - b, device="cuda"),
                                   ws=torch.empty(smem["workspace"], dtype=torch.uint8, device="cuda"))
        r_.stage = zs.Stage(cc, r_.params, r_.master, r_.grad, r_.m, r_.v, r_.ws)
        res.append(r_)
        del p
    arena = torch.empty(mem["device_bytes"], dtype=torch.uint8, device="cuda")
    ms = zs.Ministages(cc, K, host, arena)
    xs = [torch.randn(T, H, device="cuda", generator=gen).to(td) for _ in range(M)]
    dys = [(torch.randn(T, H, device="cuda", generator=gen) * 0.01).to(td) for _ in range(M)]
    for t in (1, 2):
        a = gpipe_step(ms.forward, ms.backward, ms.accumulate, ms.optimizer_step, K, M, xs, dys, T, H, td, t)
        r = gpipe_step(lambda k, i, x, y: res[k].stage.forward(i, x, y), lambda k, i, dy, dx, ls: res[k].stage.backward(i, dy, dx, ls),
                       lambda k, i: res[k].stage.accumulate(i), lambda k, tt: res[k].stage.optimizer_step(tt), K, M, xs, dys, T, H, td, t)
        for u, v in zip(a[0] + a[1], r[0] + r[1]):
            assert torch.equal(u, v), f"step {t}"
        assert bool(torch.isfinite(a[1][0].float()).all())
    for k in range(K):
        o = k * mem["per_stage_host"]
        assert torch.equal(host[o + mem["off_params"]:o + mem["off_params"] + 2 * P].view(td), res[k].params.cpu())
        for which, ref in (("master", res[k].master), ("m", res[k].m), ("v", res[k].v)):
            assert torch.equal(host[o + mem["off_" + which]:o + mem["off_" + which] + 4 * (e - b)].view(torch.float32), ref.cpu()), (k, which)
        res[k].stage.close()
    h2d, d2h = ms.traffic()
    print(f"[ministages] copied {h2d / 1e9:.2f} GB to the device, {d2h / 1e9:.2f} GB back, arena {mem['device_bytes'] / 1e9:.2f} GB "
          f"against {mem['resident_bytes'] / 1e9:.2f} GB resident", flush=True)
    ms.close()
