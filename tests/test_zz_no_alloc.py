"""stage_op_attention_bwd_noalloc: the attention backward whose delta scratch lives in a fixed device array of the
library, for callers that cannot allocate.  Called through the C ABI and compared bit for bit with
stage_op_attention_bwd (same kernels, caller-provided delta) on two calls in a row, the second on a smaller input,
so that whatever the first call left in the shared array is in the way of the second."""
import numpy as np
import pytest
import torch

import paper_2507_10392_amd as zs
from workloads import round_bf16

pytestmark = pytest.mark.gpu


def _case(dtype, impl, mb, S, nh, d, seed):
    print(f"[case] attention_bwd_noalloc dtype={dtype} impl={impl} mb={mb} S={S} nh={nh} d={d}", flush=True)
    td = {0: torch.float32, 1: torch.bfloat16}[dtype]
    H, T = nh * d, mb * S
    rng = np.random.default_rng(seed)
    rnd = round_bf16 if dtype == 1 else (lambda a: a)
    qkv = torch.from_numpy(rnd(rng.standard_normal((T, 3 * H)).astype(np.float32))).cuda().to(td)
    do = torch.from_numpy(rnd(rng.standard_normal((T, H)).astype(np.float32))).cuda().to(td)
    q, k, v = (torch.as_strided(qkv, (T, H), (3 * H, 1), i * H) for i in range(3))
    o = torch.empty(T, H, dtype=td, device="cuda")
    lse = torch.empty(mb * nh * S, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    zs.ops.attention_fwd(st, dtype, mb, S, nh, d, q, k, v, 3 * H, o, H, lse, impl)
    outs = []
    for which in ("workspace argument", "static array"):
        dqkv = torch.full((T, 3 * H), float("nan"), dtype=td, device="cuda")
        dq, dk, dv = (torch.as_strided(dqkv, (T, H), (3 * H, 1), i * H) for i in range(3))
        if which == "static array":
            zs.ops.attention_bwd_noalloc(st, dtype, mb, S, nh, d, q, k, v, 3 * H, o, do, H, lse, dq, dk, dv, 3 * H, impl)
        else:
            delta = torch.empty(mb * nh * S, device="cuda")
            zs.ops.attention_bwd(st, dtype, mb, S, nh, d, q, k, v, 3 * H, o, do, H, lse, delta, dq, dk, dv, 3 * H, impl)
        torch.cuda.synchronize()
        outs.append(dqkv)
    assert bool(torch.isfinite(outs[0].float()).all())
    assert torch.equal(outs[0], outs[1]), "static-array variant differs from the workspace variant"


@pytest.mark.parametrize("dtype,impl,d", [(1, 2, 128), (0, 1, 64)], ids=["bf16_mfma", "fp32_plain"])
def test_two_calls_in_a_row_second_one_smaller(gpu_device, dtype, impl, d):
    _case(dtype, impl, 2, 448, 4, d, 31)      # 3584 rows of delta, ragged against the 128-row blocks
    _case(dtype, impl, 1, 200, 2, d, 32)      # 400 rows: the array still holds the first call's sums behind them


def test_sizes_beyond_the_array_are_refused_before_anything_runs(gpu_device):
    fake = torch.zeros(8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    L = zs.lib()
    rows_max = 1 << 20
    p = fake.data_ptr()
    code = L.stage_op_attention_bwd_noalloc(st, 1, 1, rows_max + 1, 1, 128, p, p, p, 384, p, p, 128, p, p, p, p, 384, 0)
    assert code == zs.STAGE_ERR_WORKSPACE
    code = L.stage_op_attention_bwd_noalloc(st, 1, 4, 1 << 17, 4, 128, p, p, p, 384, p, p, 128, p, p, p, p, 384, 0)
    assert code == zs.STAGE_ERR_WORKSPACE
    assert L.stage_op_attention_bwd_noalloc(st, 1, 0, 16, 1, 128, p, p, p, 384, p, p, 128, p, p, p, p, 384, 0) == zs.STAGE_ERR_ARG
