"""Writes tests/golden/oracle_c1_summary.json from the oracle alone (calls only oracle/ and the
seeded input generator).  The stored values are a drift alarm for the oracle's arithmetic:
they are produced by the oracle, not by the paper (which prints no worked example of this
path) and never by the HIP path.  Run: python tests/golden/make_oracle_golden.py"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import stage_oracle as so  # noqa: E402
from workloads import get_config, make_inputs  # noqa: E402


def summary(name):
    cfg = get_config(name)
    inp = make_inputs(cfg)
    if cfg.has_head:
        r = so.stage_step(cfg, inp.params, inp.ids, None, inp.targets, 1.0 / cfg.num_microbatches)
    else:
        r = so.stage_step(cfg, inp.params, inp.x, inp.dy)
    b, e = cfg.shard_range
    master, m, v = so.stage_optimizer_step(cfg, inp.master, r["grad"], np.zeros(e - b), np.zeros(e - b), 1, (b, e))
    idx = [0, 1, 12345, cfg.n_params // 2, cfg.n_params - 1]
    out = {"config": name, "grad_l2": float(np.linalg.norm(r["grad"])),
           "grad_at": {str(i): float(r["grad"][i]) for i in idx},
           "delta_p_l2": float(np.linalg.norm(master - inp.master.astype(np.float64)))}
    if cfg.has_head:
        out["loss"] = [float(x) for x in r["loss"]]
    else:
        out["y0_l2"] = float(np.linalg.norm(r["y"][0]))
        out["dx0_l2"] = float(np.linalg.norm(r["dx"][0]))
        out["y0_at_17_5"] = float(r["y"][0][17, 5])
    return out


if __name__ == "__main__":
    res = [summary("C1"), summary("L1")]
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_c1_summary.json"), "w") as f:
        json.dump(res, f, indent=1)
    print(json.dumps(res, indent=1))
