"""Runtime profile for a planner (Section 4.3, "Profiling"): the stage is timed at small microbatch sizes, a line
is fitted by the library, and the line predicts a size that was not measured.  The timing call must hand the
stage back untouched."""
import numpy as np
import pytest
import torch

import paper_2507_10392_amd as zs
from harness import GpuStage, dev, tdtype
from oracle import stage_oracle as so
from workloads import get_config, make_inputs

pytestmark = pytest.mark.gpu


def _time(cfg, mb, reps=3):
    c = cfg.with_(microbatch=mb, num_microbatches=1)
    inp = make_inputs(c)
    g = GpuStage(c, inp)
    td = tdtype(c)
    x, dy = dev(inp.x[0], td), dev(inp.dy[0], td)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    f, b = g.stage.time_layers(x, y, dy, dx, reps=reps)
    g.stage.close()
    return f, b


def test_timing_call_leaves_the_stage_as_it_found_it(gpu_device):
    print("[case] stage_time_layers state", flush=True)
    cfg = get_config("C3t")
    inp = make_inputs(cfg, perturbed=True)
    ref = GpuStage(cfg, inp)
    want = ref.run_microbatches(inp)
    ref.stage.close()
    g = GpuStage(cfg, inp)
    td = tdtype(cfg)
    x, dy = dev(inp.x[0], td), dev(inp.dy[0], td)
    y, dx = torch.empty_like(x), torch.empty_like(x)
    f, b = g.stage.time_layers(x, y, dy, dx, reps=2)
    assert f > 0 and b > 0 and float(g.grad.abs().max()) == 0.0
    with pytest.raises(zs.StageError) as ei:          # nothing was accumulated as far as the schedule knows
        g.stage.optimizer_step(1)
    assert ei.value.code == zs.STAGE_ERR_STATE
    got = g.run_microbatches(inp)
    assert np.array_equal(got["grad"], want["grad"])
    for a, o in zip(got["y"] + got["dx"], want["y"] + want["dx"]):
        assert np.array_equal(a, o)
    g.stage.forward(0, x, y)
    with pytest.raises(zs.StageError) as ei:          # not with a microbatch outstanding
        g.stage.time_layers(x, y, dy, dx)
    assert ei.value.code == zs.STAGE_ERR_STATE
    g.stage.close()


def test_line_fitted_at_small_sizes_predicts_a_larger_one(gpu_device):
    """7B-class layer at sequence 1024: fit on microbatch sizes 2, 3, 4 and 6, predict 8 (work per layer is linear
    in the number of sequences at fixed sequence length)."""
    print("[case] runtime line fit", flush=True)
    cfg = get_config("C3").with_(layers=1, seq=1024, shard_num=1, shard_den=8)
    sizes = [2, 3, 4, 6]
    t = {mb: _time(cfg, mb) for mb in sizes + [8]}
    for which, name in ((0, "forward"), (1, "backward")):
        a, b, r2 = zs.fit_linear([float(m) for m in sizes], [t[m][which] for m in sizes])
        pred = a + b * 8
        print(f"[planner] {name}: {a:.3f} + {b:.3f} * mb ms, r2 {r2:.4f}; mb=8 predicted {pred:.3f} measured {t[8][which]:.3f}", flush=True)
        # Structure only: more sequences take longer, and the library's line is the oracle's least-squares line through
        # the same points.  How well the line predicts is a measured figure (printed above, reported under profiles/),
        # not a pass criterion: the clock of a fresh box is not something a test can fix.
        assert b > 0 and t[8][which] > t[2][which] > 0
        oa, ob, or2 = so.linear_fit([float(m) for m in sizes], [t[m][which] for m in sizes])
        assert abs(a - oa) <= 1e-9 * max(1.0, abs(oa)) and abs(b - ob) <= 1e-9 * abs(ob) and abs(r2 - or2) <= 1e-9
        assert 0.25 * t[8][which] <= pred <= 4.0 * t[8][which]
