"""GPU checks at the benchmark's full shapes, in the launch configuration bench.py times.

One decoder layer and one microbatch of the 7B-class (C3), 1.3B-class (C2) and 13B-class (C4a) stages, and of
the last stage with its embedding, LM head and loss (C5), are compared with the oracle element by element (the
oracle needs ten to thirty seconds per case on the host);
whole heads of the full-size attention are compared with the oracle's attention; and properties
that hold at any size (bit-identical repeats, recompute neutrality, two equal microbatches
accumulate to exactly twice one) are checked on a full-shape stage.
"""
import numpy as np
import pytest
import torch

import paper_2507_10392_amd as zs
from harness import TOL, GpuStage, compare_step, dev, log_report, oracle_step, rel_err
from oracle import stage_oracle as so
from workloads import get_config, make_inputs, round_bf16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,dtype", [("C3", 1), ("C2", 1), ("C3", 2), ("C4a", 1), ("C5", 1)])
def test_one_layer_one_microbatch_at_full_shape(gpu_device, name, dtype):
    cfg = get_config(name).with_(layers=1, num_microbatches=1, shard_num=1, shard_den=1, dtype=dtype)
    print(f"[case] full-shape single layer {name} dtype={dtype}: T={cfg.tokens} H={cfg.hidden} F={cfg.ffn}", flush=True)
    inp = make_inputs(cfg, perturbed=True, dy_scale=1024.0 if dtype == 2 else 1.0)   # fp16 runs with a loss scale
    g = GpuStage(cfg, inp)
    gpu = g.run_microbatches(inp)
    g.stage.close()
    ora = oracle_step(cfg, inp)
    rep = []
    compare_step(cfg, gpu, ora, TOL[cfg.dtype], rep)
    log_report(f"full-shape single layer {name} dtype={dtype}", sorted(rep, key=lambda r: -r[1])[:8])


def test_c4b_recompute_under_budget(gpu_device):
    """The 13B-class stage as the benchmark configures its 12-layer run: microbatches of 2 x 2048 tokens, per-layer
    checkpoints with recompute (Section 4.1.3) and a fixed activation budget of 96e9 bytes.
    - The stash is exactly M * L * T * H * D bytes and stash + scratch fit the budget, for the full 12-layer,
      8-microbatch configuration and for the cuts run here; a budget the stash cannot meet is refused on the host.
    - One of the 12 layers, two microbatches, recompute and budget as configured: outputs, input gradients and every
      gradient segment against the oracle (about a minute on the host).
    - Two layers, two microbatches: bit for bit the same stage without recompute, and bit for bit two chained
      one-layer stages (the property the oracle is pinned by), which carries the one-layer comparison to depth.
    The oracle comparison stays one layer deep on purpose: with N(0,1) inputs at this width the attention scores have
    a standard deviation of 2, so the bf16 rounding of q and k alone moves the softmax weights by half a per cent, and
    the measured max-norm error of a gain gradient is 1.1e-2 after one layer and 2.2e-2 after two against the 2e-2 bar;
    whole steps of full depth are compared with the oracle on the scaled twins (C4bt)."""
    full = get_config("C4b")
    assert full.recompute == 1 and full.act_budget_bytes == 96 * 10**9 and full.layers == 12
    _, mem_full, _ = zs.query(zs.make_config(full))
    assert mem_full["activations"] == full.num_microbatches * full.layers * full.tokens * full.hidden * 2
    assert mem_full["activations"] + mem_full["scratch"] <= full.act_budget_bytes
    with pytest.raises(zs.StageError) as ei:
        zs.query(zs.make_config(full.with_(act_budget_bytes=4 * 10**9)))       # below the 4.03 GB stash
    assert ei.value.code == zs.STAGE_ERR_BUDGET

    one = full.with_(layers=1, num_microbatches=2, shard_num=1, shard_den=1)
    print(f"[case] C4b cut: L=1 M=2 T={one.tokens} H={one.hidden} F={one.ffn} recompute=1 budget={one.act_budget_bytes}", flush=True)
    inp = make_inputs(one, perturbed=True)
    g = GpuStage(one, inp)
    assert g.mem["activations"] == one.num_microbatches * one.layers * one.tokens * one.hidden * 2
    gpu = g.run_microbatches(inp)
    g.stage.close()
    del g
    ora = oracle_step(one, inp)
    rep = []
    compare_step(one, gpu, ora, TOL[one.dtype], rep)
    log_report("C4b cut (1 layer, 2 microbatches, recompute, 96e9 B budget)", sorted(rep, key=lambda r: -r[1])[:8])
    del inp, ora, gpu

    two = full.with_(layers=2, num_microbatches=2, shard_num=1, shard_den=1)
    print("[case] C4b cut: L=2 M=2, recompute on/off and chained one-layer stages", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(4)
    P, T, H, ppl = two.n_params, two.tokens, two.hidden, two.params_per_layer
    params = (torch.randn(P, device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
    xs = [torch.randn(T, H, device="cuda", generator=gen).to(torch.bfloat16) for _ in range(2)]
    dys = [(torch.randn(T, H, device="cuda", generator=gen) * 0.01).to(torch.bfloat16) for _ in range(2)]

    def run(c, par, x_in, dy_in):
        cc = zs.make_config(c)
        n, mem, _ = zs.query(cc)
        if c.recompute:
            assert mem["activations"] == c.num_microbatches * c.layers * T * H * 2
        grad = torch.zeros(n, device="cuda")
        m, v = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
        ws = torch.empty(mem["workspace"], dtype=torch.uint8, device="cuda")
        stage = zs.Stage(cc, par.clone(), par.float(), grad, m, v, ws)
        ys = [torch.empty(T, H, dtype=torch.bfloat16, device="cuda") for _ in x_in]
        dxs = [torch.empty(T, H, dtype=torch.bfloat16, device="cuda") for _ in x_in]
        for i, x in enumerate(x_in):
            stage.forward(i, x, ys[i])
        for i in reversed(range(len(x_in))):
            stage.backward(i, dy_in[i], dxs[i])
            stage.accumulate(i)
        torch.cuda.synchronize()
        stage.close()
        return ys, dxs, grad

    y_r, dx_r, g_r = run(two, params, xs, dys)
    y_p, dx_p, g_p = run(two.with_(recompute=0, act_budget_bytes=0), params, xs, dys)
    assert torch.equal(g_r, g_p) and all(torch.equal(a, b) for a, b in zip(y_r + dx_r, y_p + dx_p))
    lay = two.with_(layers=1)
    y0, _, _ = run(lay, params[:ppl], xs, dys)                       # layer 0 forward gives layer 1's input
    y1, dx1, g1 = run(lay, params[ppl:], y0, dys)
    _, dx0, g0 = run(lay, params[:ppl], xs, dx1)
    assert all(torch.equal(a, b) for a, b in zip(y1 + dx0, y_r + dx_r))
    assert torch.equal(torch.cat([g0, g1]), g_r)
    assert bool(torch.isfinite(g_r).all()) and float(g_r.abs().max()) > 0


@pytest.mark.parametrize("S,nh", [(4096, 32), (4100, 16)], ids=["C3", "ragged"])
def test_attention_full_size_heads_match_oracle(gpu_device, S, nh):
    """32 heads of 128 at S = 4096, and a sequence length that is no multiple of any block (both take the kernels with
    256-row blocks): every row of the first and the last head, forward and backward."""
    mb, d = 1, 128
    H = nh * d
    print(f"[case] full-size attention S={S} nh={nh}", flush=True)
    rng = np.random.default_rng(21)
    qkv = round_bf16(rng.standard_normal((S, 3 * H)).astype(np.float32))
    do = round_bf16(rng.standard_normal((S, H)).astype(np.float32))
    dq_in = dev(qkv, torch.bfloat16)
    o = torch.empty(S, H, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(nh * S, device="cuda")
    delta = torch.empty(nh * S, device="cuda")
    dqkv = torch.empty(S, 3 * H, dtype=torch.bfloat16, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    qp, kp, vp = (torch.as_strided(dq_in, (S, H), (3 * H, 1), i * H) for i in range(3))
    dqp, dkp, dvp = (torch.as_strided(dqkv, (S, H), (3 * H, 1), i * H) for i in range(3))
    zs.ops.attention_fwd(st, 1, mb, S, nh, d, qp, kp, vp, 3 * H, o, H, lse, 2)
    zs.ops.attention_bwd(st, 1, mb, S, nh, d, qp, kp, vp, 3 * H, o, dev(do, torch.bfloat16), H, lse, delta, dqp, dkp,
                         dvp, 3 * H, 2)
    torch.cuda.synchronize()
    og, dg = o.float().cpu().numpy(), dqkv.float().cpu().numpy()
    rows = []
    for h in (0, nh - 1):
        sl = slice(h * d, (h + 1) * d)
        q, k, v = (qkv[:, i * H + h * d:i * H + (h + 1) * d].astype(np.float64).reshape(1, S, 1, d) for i in range(3))
        o_o = so.attention_fwd(q, k, v)[0, :, 0]
        dq_o, dk_o, dv_o = so.attention_bwd(do[:, sl].astype(np.float64).reshape(1, S, 1, d), q, k, v)
        rows += [(f"o h{h}", rel_err(og[:, sl], o_o)), (f"dq h{h}", rel_err(dg[:, sl], dq_o[0, :, 0])),
                 (f"dk h{h}", rel_err(dg[:, H + h * d:H + (h + 1) * d], dk_o[0, :, 0])),
                 (f"dv h{h}", rel_err(dg[:, 2 * H + h * d:2 * H + (h + 1) * d], dv_o[0, :, 0]))]
    log_report("full-size attention", rows)
    for n, e in rows:
        assert e <= 2e-2, (n, e)


def test_full_shape_stage_properties(gpu_device):
    """C3's shape with 2 layers: a repeat is bit-identical (fixed reduction orders; every element of the gradient
    accumulator has one owner workgroup per launch and launches are stream-ordered), recompute changes nothing, and
    accumulating the same microbatch twice gives exactly twice the gradient of one (fp32 x + x is exact)."""
    cfg = get_config("C3").with_(layers=2, num_microbatches=2, shard_num=1, shard_den=1)
    print("[case] full-shape stage properties", flush=True)
    g = torch.Generator(device="cuda").manual_seed(3)
    P = cfg.n_params
    T, H = cfg.tokens, cfg.hidden
    params = (torch.randn(P, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    x = torch.randn(T, H, device="cuda", generator=g).to(torch.bfloat16)
    dy = (torch.randn(T, H, device="cuda", generator=g) * 0.01).to(torch.bfloat16)

    def run(recompute, n_mb):
        c = cfg.with_(recompute=recompute)
        cc = zs.make_config(c)
        _, mem, _ = zs.query(cc)
        grad = torch.zeros(P, device="cuda")
        m, v = torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
        master = params.float()
        ws = torch.empty(mem["workspace"], dtype=torch.uint8, device="cuda")
        stage = zs.Stage(cc, params.clone(), master, grad, m, v, ws)
        ys, dxs = [], []
        for i in range(n_mb):
            y = torch.empty(T, H, dtype=torch.bfloat16, device="cuda")
            stage.forward(i, x, y)
            ys.append(y)
        for i in reversed(range(n_mb)):
            dx = torch.empty(T, H, dtype=torch.bfloat16, device="cuda")
            stage.backward(i, dy, dx)
            stage.accumulate(i)
            dxs.append(dx)
        torch.cuda.synchronize()
        stage.close()
        return ys, dxs, grad

    y1, dx1, g1 = run(0, 1)
    y1b, dx1b, g1b = run(0, 1)
    assert torch.equal(y1[0], y1b[0]) and torch.equal(dx1[0], dx1b[0]) and torch.equal(g1, g1b)
    yr, dxr, gr = run(1, 1)
    assert torch.equal(y1[0], yr[0]) and torch.equal(dx1[0], dxr[0]) and torch.equal(g1, gr)
    y2, dx2, g2 = run(0, 2)
    assert torch.equal(y2[0], y1[0]) and torch.equal(y2[1], y1[0]) and torch.equal(dx2[0], dx1[0])
    assert torch.equal(g2, 2.0 * g1)
    assert bool(torch.isfinite(g1).all()) and float(g1.abs().max()) > 0


def test_grouped_weight_gradients_with_cut_rounds_at_full_shape(gpu_device):
    """C3's shape, one layer, 8 microbatches with inputs of their own: with pair_wgrad = 8 the products for Wd (688 tiles)
    and Wg (1376) have the tiles beyond whole rounds of 256 workgroups cut over the microbatches (partial tiles in scratch,
    added in a fixed order).  The accumulated gradient equals the one of eight separate accumulations up to rounding order,
    a repeat gives the same bits, and the stage asks for the scratch that the cut needs."""
    base = get_config("C3").with_(layers=1, num_microbatches=8, shard_num=1, shard_den=1)
    print("[case] full-shape grouped weight gradients with cut rounds", flush=True)
    assert zs.wgrad_parts_scratch_bytes(base.ffn, base.hidden, base.tokens, base.tokens, 8, 1) > 0      # Wd
    assert zs.wgrad_parts_scratch_bytes(base.hidden, base.ffn, base.tokens, base.tokens, 8, 2) > 0      # Wg: gate and up
    g = torch.Generator(device="cuda").manual_seed(5)
    P, T, H = base.n_params, base.tokens, base.hidden
    params = (torch.randn(P, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    xs = [torch.randn(T, H, device="cuda", generator=g).to(torch.bfloat16) for _ in range(8)]
    dys = [(torch.randn(T, H, device="cuda", generator=g) * 0.01).to(torch.bfloat16) for _ in range(8)]

    def run(group):
        cc = zs.make_config(base.with_(pair_wgrad=group))
        _, mem, _ = zs.query(cc)
        grad = torch.zeros(P, device="cuda")
        m, v = torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
        ws = torch.empty(mem["workspace"], dtype=torch.uint8, device="cuda")
        stage = zs.Stage(cc, params.clone(), params.float(), grad, m, v, ws)
        y = torch.empty(T, H, dtype=torch.bfloat16, device="cuda")
        dx = torch.empty(T, H, dtype=torch.bfloat16, device="cuda")
        for i in range(8):
            stage.forward(i, xs[i], y)
        for i in reversed(range(8)):
            stage.backward(i, dys[i], dx)
            stage.accumulate(i)
        torch.cuda.synchronize()
        stage.close()
        return grad, mem

    g0, mem0 = run(0)
    g8, mem8 = run(8)
    g8b, _ = run(8)
    assert torch.equal(g8, g8b), "a repeat must give the same bits"
    assert mem8["scratch"] - mem0["scratch"] >= 7 * 5 * T * H * 2 + (160 << 20)          # kept operands + partial tiles
    worst = 0.0
    for name, off, rows, cols in zs.layout(zs.make_config(base)):
        n = rows * cols
        a, b = g8[off:off + n], g0[off:off + n]
        scale = float(b.abs().max())
        if scale > 0:
            worst = max(worst, float((a - b).abs().max()) / scale)
    print(f"[info] worst segment difference grouped vs separate: {worst:.3e}", flush=True)
    assert worst <= 2e-5 and bool(torch.isfinite(g8).all())
