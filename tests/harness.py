"""Shared test plumbing: runs one optimizer step of a stage through the C-ABI library on the GPU
and through the oracle on the CPU, from the same seeded inputs, and compares tensor by tensor.

Error metric (written here so that every test states it the same way): for a tensor pair
(gpu a, oracle o)   err = max_i |a_i - o_i| / max_i |o_i|   (max-norm relative error).
Tolerances: 1e-4 for the fp32 configuration, 2e-2 for bf16 configurations (fp32 accumulate).
Beside it every comparison of a step reports the scaled element-wise error
                    serr = max_i |a_i - o_i| / (|o_i| + 1e-2 * max_i |o_i|),
which does not let a large element hide the error of a small one.  On the fp32 configurations it is held to 5e-4:
a sum of K fp32 products carries an absolute error of about 6e-8 * sqrt(K) times the size of its terms whatever the
size of the sum itself, so an element a hundred times below the largest one has up to a hundred times its relative
error (measured worst 1.0e-4 against max-norm errors of 1e-6).  On the 16-bit configurations, where one rounding of
a small element is already 4e-3 of it, the figure is reported only.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2507_10392_amd as zs
from oracle import stage_oracle as so
from workloads.configs import DTYPE_BF16, DTYPE_F16

TOL = {0: 1e-4, 1: 2e-2, 2: 3e-3}   # fp16 rounds 8 times finer than bf16
SCALED_TOL_F32 = 5e-4


def rel_err(a, o):
    a = np.asarray(a, dtype=np.float64)
    o = np.asarray(o, dtype=np.float64)
    if o.size == 0:                       # an empty optimizer shard: nothing to differ
        assert a.size == 0
        return 0.0
    den = np.abs(o).max()
    if den == 0.0:
        return float(np.abs(a).max())
    return float(np.abs(a - o).max() / den)


SCALED_FLOOR = 1e-2


def scaled_err(a, o, floor=SCALED_FLOOR):
    """max_i |a_i - o_i| / (|o_i| + floor * max|o|): an element-wise relative error whose denominator cannot vanish.
    Elements above `floor` of the largest one are held to (almost) their own size, smaller ones to the floor; the
    max-norm error above divides every element's error by the largest element."""
    a = np.asarray(a, dtype=np.float64)
    o = np.asarray(o, dtype=np.float64)
    if o.size == 0:
        return 0.0
    den = np.abs(o).max()
    if den == 0.0:
        return float(np.abs(a).max())
    return float((np.abs(a - o) / (np.abs(o) + floor * den)).max())


def update_err(a, o, p_new, nsteps=1):
    """Max-norm relative error of a parameter update read back from fp32 storage.

    The update is recovered as p_new - p_old from values stored in fp32, so each element carries up
    to half an fp32 ulp of p_new that no arithmetic can avoid (for a gain of 1.0 that is 6e-8 against
    an update of 1e-4), once per optimizer step taken.  That floor is subtracted before the relative
    error is formed.
    """
    if np.size(o) == 0:
        return 0.0
    floor = nsteps * 0.5 * np.spacing(np.abs(p_new).astype(np.float32)).astype(np.float64) * 1.01
    d = np.maximum(np.abs(a - o) - floor, 0.0)
    return float(d.max() / np.abs(o).max())


def hp32(cfg):
    """The config with its float hyper-parameters rounded to fp32: the values the C struct carries,
    so that the oracle is run with exactly the numbers the library was given."""
    f = lambda x: float(np.float32(x))
    return cfg.with_(lr=f(cfg.lr), beta1=f(cfg.beta1), beta2=f(cfg.beta2), adam_eps=f(cfg.adam_eps),
                     weight_decay=f(cfg.weight_decay), norm_eps=f(cfg.norm_eps), rope_base=f(cfg.rope_base))


def tdtype(cfg):
    return torch.bfloat16 if cfg.dtype == DTYPE_BF16 else torch.float16 if cfg.dtype == DTYPE_F16 else torch.float32


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


class GpuStage:
    """Allocates every buffer with torch and binds a Stage to them."""

    def __init__(self, cfg, inp, shard=None, max_microbatches=None):
        self.cfg = cfg
        self.cc = zs.make_config(cfg, shard, max_microbatches)
        P, mem, _ = zs.query(self.cc)
        b, e = self.cc.shard_begin, self.cc.shard_end
        self.shard = (b, e)
        self.params = dev(inp.params, tdtype(cfg))
        self.master = dev(inp.master[b:e]) if cfg.dtype != 0 else None
        self.grad = torch.zeros(P, dtype=torch.float32, device="cuda")
        self.m = torch.zeros(max(e - b, 1), dtype=torch.float32, device="cuda")
        self.v = torch.zeros(max(e - b, 1), dtype=torch.float32, device="cuda")
        self.ws = torch.empty(mem["workspace"], dtype=torch.uint8, device="cuda")
        self.mem = mem
        self.stage = zs.Stage(self.cc, self.params, self.master, self.grad, self.m, self.v, self.ws)
        self.host = None
        if getattr(cfg, "offload_acts", 0):
            self.host = torch.empty(mem["host_stash"], dtype=torch.uint8, pin_memory=True)
            self.stage.attach_host_stash(self.host)

    def run_microbatches(self, inp, M=None, loss_scale=None, order=None):
        cfg = self.cfg
        M = cfg.num_microbatches if M is None else M
        td = tdtype(cfg)
        T, H = cfg.tokens, cfg.hidden
        ys, dxs, losses = [None] * M, [None] * M, [None] * M
        keep = []
        for i in range(M):
            if cfg.has_embed:
                xin = dev(inp.ids[i].reshape(-1))
            else:
                xin = dev(inp.x[i], td)
            y = torch.empty(T, H, dtype=td, device="cuda")
            tg = dev(inp.targets[i].reshape(-1)) if cfg.has_head else None
            loss = torch.zeros(1, dtype=torch.float32, device="cuda") if cfg.has_head else None
            self.stage.forward(i, xin, y, tg, loss)
            keep.append((xin, tg))
            ys[i], losses[i] = y, loss
        ls = (1.0 / M) if loss_scale is None else loss_scale
        for i in (reversed(range(M)) if order is None else order):
            dy = None if cfg.has_head else dev(inp.dy[i], td)
            dx = None if cfg.has_embed else torch.empty(T, H, dtype=td, device="cuda")
            self.stage.backward(i, dy, dx, ls)
            self.stage.accumulate(i)
            dxs[i] = dx
        torch.cuda.synchronize()
        out = {"grad": self.grad.cpu().numpy().astype(np.float64)}
        if cfg.has_head:
            out["loss"] = [float(l.item()) for l in losses]
        else:
            out["y"] = [y.float().cpu().numpy() for y in ys]
        if not cfg.has_embed:
            out["dx"] = [d.float().cpu().numpy() for d in dxs]
        return out

    def step(self, t=1, grad_scale=1.0):
        self.stage.optimizer_step(t, grad_scale)
        torch.cuda.synchronize()
        b, e = self.shard
        res = {"m": self.m[:e - b].cpu().numpy(), "v": self.v[:e - b].cpu().numpy(),
               "params": self.params.float().cpu().numpy(), "params_raw": self.params,
               "grad_after": self.grad.cpu().numpy()}
        res["master"] = self.master.cpu().numpy() if self.master is not None else res["params"][b:e]
        return res


def oracle_step(cfg, inp, M=None, loss_scale=None):
    cfg = hp32(cfg)
    M = cfg.num_microbatches if M is None else M
    if cfg.has_head:
        ls = (1.0 / M) if loss_scale is None else loss_scale
        return so.stage_step(cfg, inp.params, inp.ids[:M], None, inp.targets[:M], ls)
    return so.stage_step(cfg, inp.params, inp.x[:M], inp.dy[:M])


def log_report(title, rows):
    """Appends error figures to the text file named by the environment variable STAGE_PARITY_REPORT, if it is set."""
    import os
    path = os.environ.get("STAGE_PARITY_REPORT")
    if path:
        with open(path, "a") as f:
            f.write(title + "\n")
            for name, e, *more in rows:
                f.write(f"    {name:28s} {e:.3e}" + "".join(f"  scaled {x:.3e}" for x in more) + "\n")


def compare_step(cfg, gpu, ora, tol, report=None, zero_scale=None):
    """Checks outputs, input gradients, loss and every gradient segment; returns the worst error.

    A segment whose oracle gradient is exactly zero must be exactly zero on the GPU, unless zero_scale is given:
    then the zero comes from a cancellation that only exact arithmetic makes complete (softmax over a single key:
    dS = P (dP - sum P dP) with P = 1), and the GPU's values must stay below tol * zero_scale."""
    worst = 0.0

    def chk(name, a, o):
        nonlocal worst
        e = rel_err(a, o)
        se = scaled_err(a, o)
        if report is not None:
            report.append((name, e, se))
        worst = max(worst, e)
        assert e <= tol, f"{cfg.name}: {name}: max-norm relative error {e:.3e} > {tol:g}"
        if cfg.dtype == 0:
            assert se <= SCALED_TOL_F32, f"{cfg.name}: {name}: scaled element-wise error {se:.3e} > {SCALED_TOL_F32:g}"

    if cfg.has_head:
        for i, (a, o) in enumerate(zip(gpu["loss"], ora["loss"])):
            chk(f"loss[{i}]", [a], [o])
    else:
        for i, (a, o) in enumerate(zip(gpu["y"], ora["y"])):
            chk(f"y[{i}]", a, o)
    if not cfg.has_embed:
        for i, (a, o) in enumerate(zip(gpu["dx"], ora["dx"])):
            chk(f"dx[{i}]", a, o)
    for name, off, r, c in so.layout(cfg):
        o = ora["grad"][off:off + r * c]
        a = gpu["grad"][off:off + r * c]
        if np.abs(o).max() == 0.0:
            if zero_scale is None:
                assert np.abs(a).max() == 0.0, f"{name}: oracle gradient is exactly zero, GPU's is not"
            else:
                assert np.abs(a).max() <= tol * zero_scale, f"{name}: {np.abs(a).max():.3e} where the oracle has zero"
            continue
        chk("grad " + name, a, o)
    return worst


def compare_optimizer(cfg, inp, shard, gpu_grad, res, ora_grad, tol, t=1):
    """Checks m, v, the parameter UPDATE (not the parameter), bf16 rounding and the untouched rest.

    The update of the first step is ~ lr*g/(|g|+eps), discontinuous in sign(g) at 0, so it is
    compared where |g_oracle| >= 10*tol*max|g| of the segment; elsewhere it must obey the
    closed-form bound |dp + lr*wd*p| <= lr.
    """
    b, e = shard
    cfg = hp32(cfg)
    p0 = inp.master.astype(np.float64)
    new, m_o, v_o = so.stage_optimizer_step(cfg, p0, ora_grad, np.zeros(e - b), np.zeros(e - b), t, (b, e))
    assert rel_err(res["m"], m_o) <= tol
    assert rel_err(res["v"], v_o) <= 2 * tol + tol * tol          # v is quadratic in g
    dp_gpu = res["master"].astype(np.float64) - p0[b:e]
    dp_ora = new[b:e] - p0[b:e]
    frac_masked = []
    for name, off, r, c in so.layout(cfg):
        lo, hi = max(off, b), min(off + r * c, e)
        if lo >= hi:
            continue
        g = ora_grad[lo:hi]
        if np.abs(g).max() == 0.0:
            big = np.zeros(hi - lo, dtype=bool)
        else:
            big = np.abs(g) >= 10 * tol * np.abs(ora_grad[off:off + r * c]).max()
        a, o = dp_gpu[lo - b:hi - b], dp_ora[lo - b:hi - b]
        if big.any():
            err = update_err(a[big], o[big], new[lo:hi][big])
            assert err <= tol, f"{cfg.name}: update of {name}: {err:.3e} > {tol:g}"
        small = ~big
        if small.any():
            bound = np.abs(a[small] + cfg.lr * cfg.weight_decay * p0[lo:hi][small])
            assert bound.max() <= cfg.lr * (1 + 1e-3), f"{name}: update exceeds the closed-form cap"
        frac_masked.append((name, float(small.mean())))
    # the same update recomputed by the oracle from the GPU's own gradient: isolates the optimizer arithmetic
    new2, m2, v2 = so.stage_optimizer_step(cfg, p0, gpu_grad, np.zeros(e - b), np.zeros(e - b), t, (b, e))
    dp2 = new2[b:e] - p0[b:e]
    assert update_err(dp_gpu, dp2, new2[b:e]) <= 2e-5
    assert rel_err(res["m"], m2) <= 1e-6 and rel_err(res["v"], v2) <= 1e-6
    # outside the shard nothing moves; grad_acc is zero everywhere afterwards
    par = res["params"].astype(np.float64)
    assert np.array_equal(par[:b], inp.params[:b].astype(np.float64)) and np.array_equal(par[e:], inp.params[e:].astype(np.float64))
    assert not res["grad_after"].any()
    if cfg.dtype != 0:
        want = torch.from_numpy(res["master"]).to(tdtype(cfg))          # round-to-nearest-even, bit exact
        got = res["params_raw"][b:e].cpu()
        assert torch.equal(want.view(torch.int16), got.view(torch.int16))
    return frac_masked
