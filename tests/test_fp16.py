"""fp16 mixed precision with loss scaling (the precision the paper trains in, Section 6.1): IEEE-half activations
and working parameters, fp32 master copy, gradients and moments.  The upstream gradient is multiplied by the
loss scale before it is rounded to half, the optimizer step divides it out again (grad_scale); a step whose
gradients are not finite is detected on the device and skipped."""
import numpy as np
import pytest
import torch

import paper_2507_10392_amd as zs
from harness import TOL, GpuStage, compare_optimizer, compare_step, hp32, oracle_step, rel_err
from oracle import stage_oracle as so
from workloads import get_config, make_inputs

pytestmark = pytest.mark.gpu
SCALE = 1024.0


@pytest.mark.parametrize("name", ["C3h", "C2h", "C5h"])
def test_fp16_stage_step_matches_oracle(gpu_device, name):
    cfg = get_config(name)
    print(f"[case] fp16 stage step {name}", flush=True)
    inp = make_inputs(cfg, perturbed=True, dy_scale=SCALE)
    tol = TOL[cfg.dtype]
    M = cfg.num_microbatches
    g = GpuStage(cfg, inp)
    gpu = g.run_microbatches(inp, loss_scale=SCALE / M)
    ora = oracle_step(cfg, inp, loss_scale=SCALE / M)           # the oracle sees the same scaled seeds
    rep = []
    compare_step(cfg, gpu, ora, tol, rep)
    worst = max(rep, key=lambda r: r[1])
    print(f"[parity] {name}: worst {worst[0]} = {worst[1]:.3e} (tol {tol:g})", flush=True)
    # the optimizer takes the scale out again: compare with the oracle's AdamW on gradients divided by the scale
    res = g.step(1, grad_scale=1.0 / SCALE)
    b, e = g.shard
    c32 = hp32(cfg)
    p0 = inp.master.astype(np.float64)
    new, m_o, v_o = so.stage_optimizer_step(c32, p0, gpu["grad"], np.zeros(e - b), np.zeros(e - b), 1, (b, e),
                                            grad_scale=float(np.float32(1.0 / SCALE)))
    assert rel_err(res["m"], m_o) <= 1e-6 and rel_err(res["v"], v_o) <= 1e-6
    assert np.abs(res["master"].astype(np.float64) - new[b:e]).max() <= 1e-6 * cfg.lr + 1.2e-7 * np.abs(new[b:e]).max()
    want = torch.from_numpy(res["master"]).to(torch.float16)                 # working copy = half(master), bit exact
    assert torch.equal(want.view(torch.int16), res["params_raw"][b:e].cpu().view(torch.int16))
    # and unscaled, the accumulated gradient is the oracle's gradient of the unscaled problem
    plain = make_inputs(cfg, perturbed=True)
    if not cfg.has_head:                                                      # same draws, only dy differs by the scale
        o1 = oracle_step(cfg, plain)
        assert rel_err(gpu["grad"] / SCALE, o1["grad"]) <= 2 * tol
    g.stage.close()


def test_overflowing_step_is_detected_and_skipped(gpu_device):
    """A loss scale that pushes the seed beyond the largest half (65504) makes every gradient non-finite: the
    flag comes up, parameters, master copy and moments stay bit for bit, the gradients are dropped; the usual
    rule then halves the scale until a step goes through, and that step matches the oracle."""
    cfg = get_config("C3h").with_(num_microbatches=2)
    print("[case] fp16 overflow", flush=True)
    base = make_inputs(cfg, perturbed=True)
    g = GpuStage(cfg, base)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    zs.lib().stage_set_overflow_flag(g.stage.h, flag.data_ptr())
    scale, good, t = 2.0 ** 24, 0, 0
    before = [x.clone() for x in (g.params, g.master, g.m, g.v)]
    skipped = 0
    for attempt in range(12):
        inp = make_inputs(cfg, perturbed=True, dy_scale=scale)
        expect_overflow = so.gradients_overflow_fp16(max(float(np.abs(d).max()) for d in inp.dy))
        out = g.run_microbatches(inp)
        flag.zero_()
        g.stage.optimizer_step(t + 1, 1.0 / scale)
        torch.cuda.synchronize()
        found = int(flag.item())
        assert float(g.grad.abs().max()) == 0.0                              # dropped either way
        o_scale, o_good = so.loss_scale_update(scale, good, found, growth_interval=3)
        sc, gd = zs.loss_scale_update(scale, good, found, 0.5, 2.0, 3)
        assert (sc, gd) == (o_scale, o_good)
        if found:
            assert expect_overflow or not np.isfinite(out["grad"]).all()
            for a, b0 in zip((g.params, g.master, g.m, g.v), before):
                assert torch.equal(a, b0)
            skipped += 1
        else:
            assert np.isfinite(out["grad"]).all() and not expect_overflow
            t += 1
            b, e = g.shard
            new, m_o, v_o = so.stage_optimizer_step(hp32(cfg), base.master.astype(np.float64), out["grad"], np.zeros(e - b),
                                                    np.zeros(e - b), 1, (b, e), grad_scale=float(np.float32(1.0 / scale)))
            assert rel_err(g.m.cpu().numpy(), m_o) <= 1e-6
            assert np.abs(g.master.cpu().numpy().astype(np.float64) - new[b:e]).max() <= 1e-6 * cfg.lr + 1.2e-7 * np.abs(new[b:e]).max()
            ora = oracle_step(cfg, inp)
            assert rel_err(out["grad"], ora["grad"]) <= 2 * TOL[cfg.dtype]
            break
        scale, good = sc, gd
    assert skipped >= 2 and t == 1, (skipped, t)
    zs.lib().stage_set_overflow_flag(g.stage.h, None)
    g.stage.close()
