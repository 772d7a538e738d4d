"""GPU parity of the whole stage step (C ABI -> HIP kernels) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2507_10392_amd as zs

from harness import TOL, GpuStage, compare_optimizer, compare_step, log_report, oracle_step
from workloads import get_config, make_inputs

pytestmark = pytest.mark.gpu

STEP_CASES = [("C1", False), ("C1", True), ("L1", True), ("C2t", False), ("C2t", True), ("C3t", False),
              ("C3t", True), ("C4at", True), ("C4bt", False), ("C5t", False), ("C5t", True)]


@pytest.mark.parametrize("name,perturbed", STEP_CASES)
def test_stage_step_matches_oracle(gpu_device, name, perturbed):
    cfg = get_config(name)
    print(f"[case] stage step {name} perturbed={perturbed}", flush=True)
    inp = make_inputs(cfg, perturbed=perturbed)
    tol = TOL[cfg.dtype]
    g = GpuStage(cfg, inp)
    gpu = g.run_microbatches(inp)
    ora = oracle_step(cfg, inp)
    rep = []
    compare_step(cfg, gpu, ora, tol, rep)
    worst = max(rep, key=lambda r: r[1])
    log_report(f"stage step {name} perturbed={perturbed} tol={tol:g}", sorted(rep, key=lambda r: -r[1])[:6])
    print(f"[parity] {name}: worst {worst[0]} = {worst[1]:.3e} (tol {tol:g})", flush=True)
    res = g.step(1)
    masked = compare_optimizer(cfg, inp, g.shard, gpu["grad"], res, ora["grad"], tol)
    print(f"[parity] {name}: largest masked fraction {max(m for _, m in masked):.3f}", flush=True)
    g.stage.close()


@pytest.mark.parametrize("name,seq,mb", [("C3t", 200, 2), ("C5t", 72, 3), ("C2t", 136, 1)])
def test_stage_step_with_ragged_sequence_lengths(gpu_device, name, seq, mb):
    """Sequence lengths that are no multiple of the attention tiles (64 keys, 128 queries) and token counts
    that are no multiple of the GEMM tiles, several sequences per microbatch: positions, causal masks and
    the fused rotation must follow the sequence boundaries."""
    cfg = get_config(name).with_(seq=seq, microbatch=mb, num_microbatches=3)
    print(f"[case] ragged stage step {name} S={seq} mb={mb}", flush=True)
    inp = make_inputs(cfg, perturbed=True)
    g = GpuStage(cfg, inp)
    gpu = g.run_microbatches(inp)
    g.stage.close()
    ora = oracle_step(cfg, inp)
    rep = []
    compare_step(cfg, gpu, ora, TOL[cfg.dtype], rep)
    log_report(f"ragged stage step {name} S={seq} mb={mb}", sorted(rep, key=lambda r: -r[1])[:6])


@pytest.mark.parametrize("name,M,group", [("C3t", 16, 1), ("C3t", 3, 1), ("C2t", 8, 1), ("C5t", 5, 1), ("C4at", 2, 1),
                                          ("C3t", 16, 16), ("C3t", 16, 4), ("C3t", 7, 3), ("C3t", 5, 64), ("C2t", 8, 8),
                                          ("C5t", 5, 4), ("C3h", 4, 4)])
def test_paired_weight_gradients_match_oracle(gpu_device, name, M, group):
    """pair_wgrad = 1: every other backward leaves its weight-gradient products to the next one, which runs them
    over both microbatches' tokens; pair_wgrad = g >= 2: groups of g microbatches (at most 16) share one K loop,
    and a last group may be smaller.  Same sums, so the accumulated gradient and everything else must match the
    oracle as before."""
    cfg = get_config(name).with_(num_microbatches=M, pair_wgrad=group)
    print(f"[case] paired wgrad {name} M={M} group={group}", flush=True)
    inp = make_inputs(cfg, perturbed=True)
    g = GpuStage(cfg, inp)
    gpu = g.run_microbatches(inp)
    ora = oracle_step(cfg, inp)
    rep = []
    compare_step(cfg, gpu, ora, TOL[cfg.dtype], rep)
    log_report(f"paired wgrad {name} M={M} group={group}", sorted(rep, key=lambda r: -r[1])[:6])
    res = g.step(1)
    compare_optimizer(cfg, inp, g.shard, gpu["grad"], res, ora["grad"], TOL[cfg.dtype])
    g.stage.close()


@pytest.mark.parametrize("dtype", [1, 2])
def test_grouped_weight_gradients_with_cut_rounds_match_oracle(gpu_device, dtype):
    """A one-layer stage wide enough (hidden 2048, FFN 8448: 264 and 528 tiles of 256x256) for the grouped weight gradients of
    Wd and Wg to leave partly filled rounds: those tiles' K range is cut over the 4 microbatches, partial tiles go through
    scratch and are added in a fixed order.  Everything against the oracle, as for the uncut products."""
    cfg = get_config("C3t").with_(layers=1, hidden=2048, heads=16, ffn=8448, seq=256, num_microbatches=4, pair_wgrad=4, dtype=dtype)
    print(f"[case] grouped wgrad with cut rounds, dtype={dtype}", flush=True)
    assert zs.wgrad_parts_scratch_bytes(cfg.ffn, cfg.hidden, cfg.tokens, cfg.tokens, 4, 1) > 0
    assert zs.wgrad_parts_scratch_bytes(cfg.hidden, cfg.ffn, cfg.tokens, cfg.tokens, 4, 2) > 0
    inp = make_inputs(cfg, perturbed=True)
    g = GpuStage(cfg, inp)
    gpu = g.run_microbatches(inp)
    ora = oracle_step(cfg, inp)
    rep = []
    compare_step(cfg, gpu, ora, TOL[cfg.dtype], rep)
    log_report(f"grouped wgrad with cut rounds dtype={dtype}", sorted(rep, key=lambda r: -r[1])[:6])
    g.stage.close()


@pytest.mark.parametrize("group", [1, 3, 4])
def test_paired_weight_gradients_with_interleaved_calls(gpu_device, group):
    """Orders other than all-forwards-then-all-backwards: a deferred microbatch whose slot is reused is flushed
    first, a backward with nothing else outstanding is not deferred, and the sum is the same."""
    cfg = get_config("C3t").with_(num_microbatches=4, pair_wgrad=group)
    print(f"[case] paired wgrad, interleaved order, group={group}", flush=True)
    inp = make_inputs(cfg, perturbed=True)
    td = torch.bfloat16
    T, H = cfg.tokens, cfg.hidden
    g = GpuStage(cfg, inp)
    x = [torch.from_numpy(np.ascontiguousarray(inp.x[i])).cuda().to(td) for i in range(4)]
    dy = [torch.from_numpy(np.ascontiguousarray(inp.dy[i])).cuda().to(td) for i in range(4)]
    y = [torch.empty(T, H, dtype=td, device="cuda") for _ in range(4)]
    dx = [torch.empty(T, H, dtype=td, device="cuda") for _ in range(4)]
    st = g.stage
    fwd = lambda slot, i: st.forward(slot, x[i], y[i], None, None)
    def bwd(slot, i):
        st.backward(slot, dy[i], dx[i], 1.0)
        st.accumulate(slot)
    fwd(0, 0); fwd(1, 1)
    bwd(1, 1)            # deferred (microbatch 0 is still outstanding)
    fwd(1, 2)            # reuses the deferred slot: its products run now
    bwd(1, 2)            # deferred again
    fwd(2, 3)
    bwd(2, 3)            # runs for microbatches 2 and 3
    bwd(0, 0)            # nothing else outstanding: not deferred
    torch.cuda.synchronize()
    ora = oracle_step(cfg, inp)
    err = float(np.abs(g.grad.cpu().numpy().astype(np.float64) - ora["grad"]).max() / np.abs(ora["grad"]).max())
    log_report("paired wgrad, interleaved order", [("grad", err)])
    assert err <= TOL[cfg.dtype]
    for i in range(4):
        assert float(np.abs(dx[i].float().cpu().numpy() - ora["dx"][i]).max() / np.abs(ora["dx"][i]).max()) <= TOL[cfg.dtype]
    st.close()


@pytest.mark.parametrize("name", ["C3t", "C5t", "C2t"])
def test_recompute_is_result_neutral(gpu_device, name):
    """Per-layer checkpointing recomputes what it dropped (Section 4.1.3): same kernels, same inputs,
    so outputs and gradients are bit-identical with it on and off."""
    cfg = get_config(name)
    print(f"[case] recompute neutrality {name}", flush=True)
    inp = make_inputs(cfg, perturbed=True, num_microbatches=3)
    outs = []
    for rc in (0, 1):
        g = GpuStage(cfg.with_(recompute=rc), inp, max_microbatches=3)
        outs.append(g.run_microbatches(inp, M=3))
        g.stage.close()
    assert np.array_equal(outs[0]["grad"], outs[1]["grad"])
    key = "loss" if cfg.has_head else "y"
    for a, b in zip(outs[0][key], outs[1][key]):
        assert np.array_equal(np.asarray(a), np.asarray(b))


def test_second_step_and_determinism(gpu_device):
    """Two optimizer steps in a row (t = 1, 2) match the oracle run the same way, and a repeat of
    the whole sequence is bit-identical (no atomics, fixed reduction orders)."""
    from harness import hp32
    from oracle import stage_oracle as so
    cfg = get_config("C1")
    print("[case] two steps C1", flush=True)
    inp = make_inputs(cfg, perturbed=True)
    runs = []
    for rep in range(2):
        g = GpuStage(cfg, inp)
        g1 = g.run_microbatches(inp)
        r1 = g.step(1)
        g2 = g.run_microbatches(inp)
        r2 = g.step(2)
        runs.append((g1["grad"], r1["params"].copy(), g2["grad"], r2["params"].copy(), r2["m"].copy(), r2["v"].copy()))
        g.stage.close()
    for a, b in zip(runs[0], runs[1]):
        assert np.array_equal(a, b)
    # Step-2 gradient against the oracle run the same way (oracle parameters after its own first step).
    b, e = cfg.shard_range
    cfg = hp32(cfg)
    p0 = inp.master.astype(np.float64)
    o1 = oracle_step(cfg, inp)
    p1, m1, v1 = so.stage_optimizer_step(cfg, p0, o1["grad"], np.zeros(e - b), np.zeros(e - b), 1, (b, e))
    inp2 = make_inputs(cfg, perturbed=True)
    inp2.params = p1
    o2 = oracle_step(cfg, inp2)
    from harness import rel_err, update_err
    assert rel_err(runs[0][2], o2["grad"]) <= 1e-4
    # AdamW at t = 2 with non-zero moments: the oracle fed the GPU's own two gradients must land on the
    # GPU's parameters and moments to fp32 rounding (the update itself is discontinuous in sign(g), so it
    # is not compared across slightly different gradients).
    q1, n1, w1 = so.stage_optimizer_step(cfg, p0, runs[0][0], np.zeros(e - b), np.zeros(e - b), 1, (b, e))
    q2, n2, w2 = so.stage_optimizer_step(cfg, q1, runs[0][2], n1, w1, 2, (b, e))
    assert rel_err(runs[0][4], n2) <= 1e-6 and rel_err(runs[0][5], w2) <= 1e-6
    assert update_err(runs[0][3].astype(np.float64) - p0, q2 - p0, q2, nsteps=2) <= 2e-5


@pytest.mark.parametrize("name", ["C3t", "C1", "C5t"])
@pytest.mark.parametrize("shard", ["empty", "whole", "odd"])
def test_optimizer_shard_edges(gpu_device, name, shard):
    """Degenerate optimizer ranges: an empty shard (the rank owns nothing of this stage: the step only drops the
    gradients), the whole parameter vector, and a range whose ends are not multiples of the kernels' vector width."""
    cfg = get_config(name).with_(num_microbatches=2)
    from oracle import stage_oracle as so
    P = so.n_params(cfg)
    b, e = {"empty": (1000, 1000), "whole": (0, P), "odd": (5, P - 3)}[shard]
    print(f"[case] shard edge {name} [{b}, {e})", flush=True)
    inp = make_inputs(cfg, perturbed=True)
    g = GpuStage(cfg, inp, shard=(b, e))
    gpu = g.run_microbatches(inp)
    res = g.step(1)
    g.stage.close()
    ora = oracle_step(cfg, inp)
    compare_step(cfg, gpu, ora, TOL[cfg.dtype])
    compare_optimizer(cfg, inp, (b, e), gpu["grad"], res, ora["grad"], TOL[cfg.dtype])


@pytest.mark.parametrize("name,seq,mb,M", [("C3t", 1, 1, 1), ("C1", 1, 1, 2), ("C5t", 1, 8, 1), ("L1", 3, 1, 1), ("C2t", 8, 1, 1)])
def test_stage_step_with_the_shortest_sequences(gpu_device, name, seq, mb, M):
    """One token per sequence (the attention of a token with itself only), one token per microbatch (products with a
    single row, norms and column sums over one row), and a single microbatch."""
    cfg = get_config(name).with_(seq=seq, microbatch=mb, num_microbatches=M)
    print(f"[case] shortest sequences {name} S={seq} mb={mb} M={M}", flush=True)
    inp = make_inputs(cfg, perturbed=True)
    g = GpuStage(cfg, inp)
    gpu = g.run_microbatches(inp)
    res = g.step(1)
    g.stage.close()
    ora = oracle_step(cfg, inp)
    # S = 1: the gradients of the Q and K projections vanish by an exact cancellation in the oracle
    compare_step(cfg, gpu, ora, TOL[cfg.dtype], zero_scale=np.abs(ora["grad"]).max() if seq == 1 else None)
    compare_optimizer(cfg, inp, g.shard, gpu["grad"], res, ora["grad"], TOL[cfg.dtype])
