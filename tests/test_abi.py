"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and the host-side
validation, layout and memory accounting behave as the header states.  No kernel is launched."""
import ctypes as C
import os
import re

import pytest

import paper_2507_10392_amd as zs
from oracle import stage_oracle as so
from workloads import CONFIGS, get_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = []
    for h in ("stage.h", "stage_ops.h", "ministages.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b((?:stage|ministages)_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    L = zs.lib()
    syms = declared_symbols()
    assert {"stage_query", "stage_layout", "stage_init", "stage_forward", "stage_backward", "stage_accumulate",
            "stage_optimizer_step", "stage_last_error", "stage_destroy", "stage_op_gemm", "stage_op_adamw"} <= set(syms)
    for s in syms:
        assert hasattr(L, s), s


@pytest.mark.parametrize("name", list(CONFIGS))
def test_layout_and_param_count_match_oracle(name):
    cfg = get_config(name)
    cc = zs.make_config(cfg)
    P, mem, ns = zs.query(cc) if cfg.name != "C4b" else zs.query(cc)
    assert P == cfg.n_params == so.n_params(cfg)
    assert zs.layout(cc) == so.layout(cfg)
    E = 2 if cfg.dtype else 4
    sh = cfg.shard_range[1] - cfg.shard_range[0]
    assert mem["params"] == P * E and mem["grads"] == 4 * P
    assert mem["optim"] == sh * (12 if cfg.dtype else 8)
    assert mem["workspace"] >= mem["activations"] + mem["scratch"] and mem["workspace"] % 256 == 0


def test_recompute_stash_is_exactly_the_papers_formula():
    """Section 4.1.3: B x L boundary activations of S x H x D bytes each."""
    for name in ("C4b", "C4bt"):
        cfg = get_config(name)
        _, mem, _ = zs.query(zs.make_config(cfg))
        assert mem["activations"] == cfg.num_microbatches * cfg.layers * cfg.tokens * cfg.hidden * 2
    c3 = get_config("C3")
    _, full, _ = zs.query(zs.make_config(c3))
    _, rc, _ = zs.query(zs.make_config(c3.with_(recompute=1)))
    assert rc["activations"] == 16 * 8 * 4096 * 4096 * 2 and full["activations"] > 10 * rc["activations"]


def test_offload_keeps_two_microbatches_on_the_device():
    """Section 4.1.3: with the boundary activations offloaded, only the microbatch in use and the one being
    prefetched stay on the GPU; all B x L tensors of S x H x D bytes live on the host."""
    for name in ("C4b", "C4bt", "C5"):
        cfg = get_config(name).with_(recompute=1)
        one = cfg.tokens * cfg.hidden * 2
        per_mb = (cfg.layers + cfg.has_head) * one      # a head stage also keeps the final norm's input
        _, res, _ = zs.query(zs.make_config(cfg))
        _, off, _ = zs.query(zs.make_config(cfg.with_(offload_acts=1)))
        small = 4 * cfg.tokens * (cfg.has_embed + cfg.has_head) * cfg.num_microbatches   # ids / targets stay on the device
        assert res["host_stash"] == 0 and off["host_stash"] == cfg.num_microbatches * per_mb
        assert abs(res["activations"] - (cfg.num_microbatches * per_mb + small)) <= 512 * cfg.num_microbatches
        assert abs(off["activations"] - (2 * per_mb + small)) <= 512 * cfg.num_microbatches
        assert off["scratch"] == res["scratch"]
    # an activation budget that the resident stash breaks is met with offloading
    c4b = get_config("C4b")
    with pytest.raises(zs.StageError) as ei:
        zs.query(zs.make_config(c4b.with_(act_budget_bytes=3 * 10**9)))
    assert ei.value.code == zs.STAGE_ERR_BUDGET
    zs.query(zs.make_config(c4b.with_(act_budget_bytes=3 * 10**9, offload_acts=1)))
    with pytest.raises(zs.StageError) as ei:             # only boundary activations are offloaded
        zs.query(zs.make_config(c4b.with_(recompute=0, offload_acts=1)))
    assert ei.value.code == zs.STAGE_ERR_ARG


def test_ministages_memory_report():
    """Section 4.1.1: two ministages' parameters on the GPU instead of all K; Section 4.1.2: one gradient buffer,
    freed by each ministage's optimizer step."""
    cfg = get_config("C3").with_(layers=2)
    cc = zs.make_config(cfg)
    P, mem, _ = zs.query(cc)
    sh = cc.shard_end - cc.shard_begin
    for K in (1, 2, 4, 9):
        m = zs.ministages_query(cc, K)
        up = lambda n: (n + 255) // 256 * 256
        assert m["off_params"] == 0 and m["off_master"] == up(2 * P) and m["off_m"] == m["off_master"] + up(4 * sh)
        assert m["per_stage_host"] == up(2 * P) + 3 * up(4 * sh) and m["host_bytes"] == K * m["per_stage_host"]
        act, scratch = up(mem["activations"]), mem["workspace"] - up(mem["activations"])
        assert m["workspace_each"] == act and m["scratch"] == scratch and m["off_stash"] == -1
        assert m["device_bytes"] == min(K, 2) * up(2 * P) + min(K, 3) * 3 * up(4 * sh) + up(4 * P) + scratch + K * act
        assert m["resident_bytes"] == K * (mem["params"] + mem["grads"] + mem["optim"] + mem["workspace"])
    assert "ministages_forward" in declared_symbols() and "ministages_destroy" in declared_symbols()
    with pytest.raises(zs.StageError) as ei:
        zs.ministages_query(cc, 0)
    assert ei.value.code == zs.STAGE_ERR_ARG
    # with the boundary activations offloaded each ministage keeps two microbatch slots, its stash joins the host block
    oc = zs.make_config(cfg.with_(recompute=1, offload_acts=1))
    _, omem, _ = zs.query(oc)
    m = zs.ministages_query(oc, 4)
    assert m["off_stash"] == m["off_v"] + up(4 * sh) and m["per_stage_host"] == m["off_stash"] + up(omem["host_stash"])
    assert m["workspace_each"] == up(omem["activations"]) and omem["host_stash"] == 16 * 2 * 4096 * 4096 * 2


def test_library_line_fit_matches_oracle():
    """stage_fit_linear is host-only arithmetic, so its parity with the oracle runs without a GPU."""
    import numpy as np
    rng = np.random.default_rng(11)
    for n in (2, 3, 5, 40):
        x = np.sort(rng.uniform(1.0, 64.0, n))
        y = 0.3 + 1.7 * x + rng.standard_normal(n) * 0.5
        a, b, r2 = zs.fit_linear(list(x), list(y))
        oa, ob, or2 = so.linear_fit(x, y)
        assert abs(a - oa) <= 1e-9 * max(1.0, abs(oa)) and abs(b - ob) <= 1e-9 * abs(ob) and abs(r2 - or2) <= 1e-9
    assert zs.fit_linear([1.0, 2.0], [5.0, 5.0]) == (5.0, 0.0, 1.0)
    for bad in (([1.0], [2.0]), ([3.0, 3.0, 3.0], [1.0, 2.0, 3.0])):
        with pytest.raises(zs.StageError) as ei:
            zs.fit_linear(*bad)
        assert ei.value.code == zs.STAGE_ERR_ARG


def test_loss_scale_rule_matches_oracle():
    """stage_loss_scale_update is host-only: compared with the oracle over a scripted sequence of good and
    overflowing steps (halving, doubling after an unbroken run, the count restarting after an overflow)."""
    scale, good, o = 65536.0, 0, (65536.0, 0)
    for found in (0, 0, 1, 0, 0, 0, 0, 1, 1, 0, 0, 0, 0, 0, 0):
        scale, good = zs.loss_scale_update(scale, good, found, 0.5, 2.0, 3)
        o = so.loss_scale_update(o[0], o[1], found, 0.5, 2.0, 3)
        assert (scale, good) == o
    assert o == (65536.0, 0)          # /2, x2, /2, /2, x2, x2 with the counts in between
    for bad in ((0.0, 0, 0, 0.5, 2.0, 3), (1.0, 0, 0, 1.5, 2.0, 3), (1.0, 0, 0, 0.5, 1.0, 3), (1.0, 0, 0, 0.5, 2.0, 0)):
        with pytest.raises(zs.StageError):
            zs.loss_scale_update(*bad)


def test_bad_configs_are_rejected_on_the_host():
    cfg = get_config("C1")
    for kw in (dict(heads=3), dict(hidden=250, heads=5), dict(layers=0), dict(arch=2), dict(dtype=3),
               dict(recompute=2), dict(has_head=1, vocab=0), dict(norm_eps=0.0), dict(beta1=1.0)):
        with pytest.raises(zs.StageError) as ei:
            zs.query(zs.make_config(cfg.with_(**kw)))
        assert ei.value.code == zs.STAGE_ERR_ARG, kw
    for shard in ((-1, 10), (10, 5), (0, cfg.n_params + 1)):
        with pytest.raises(zs.StageError) as ei:
            zs.query(zs.make_config(cfg, shard=shard))
        assert ei.value.code == zs.STAGE_ERR_ARG


def test_activation_budget_is_enforced():
    cfg = get_config("C4b")
    zs.query(zs.make_config(cfg))                                     # 96e9 bytes: fits
    with pytest.raises(zs.StageError) as ei:
        zs.query(zs.make_config(cfg.with_(act_budget_bytes=10**9)))
    assert ei.value.code == zs.STAGE_ERR_BUDGET
    with pytest.raises(zs.StageError) as ei:                          # without recompute the 12-layer stage does not fit 40 GB
        zs.query(zs.make_config(cfg.with_(recompute=0, act_budget_bytes=40 * 10**9)))
    assert ei.value.code == zs.STAGE_ERR_BUDGET


def test_init_rejects_bad_buffers_before_touching_the_device():
    cfg = get_config("C1")
    cc = zs.make_config(cfg)
    L = zs.lib()
    h = C.c_void_p()
    fake = C.c_void_p(0x10000)          # never dereferenced: every check below fails first
    _, mem, _ = zs.query(cc)
    code = L.stage_init(C.byref(cc), None, None, None, fake, fake, fake, fake, mem["workspace"], C.byref(h))
    assert code == zs.STAGE_ERR_ARG and not h.value
    code = L.stage_init(C.byref(cc), None, fake, fake, fake, fake, fake, fake, mem["workspace"], C.byref(h))
    assert code == zs.STAGE_ERR_ARG and b"master must be NULL" in L.stage_last_error(None)
    code = L.stage_init(C.byref(cc), None, fake, None, fake, fake, fake, fake, mem["workspace"] - 1, C.byref(h))
    assert code == zs.STAGE_ERR_WORKSPACE
    code = L.stage_init(C.byref(cc), None, fake, None, fake, fake, fake, C.c_void_p(0x10010), mem["workspace"], C.byref(h))
    assert code == zs.STAGE_ERR_WORKSPACE
    code = L.stage_init(C.byref(cc), None, C.c_void_p(0x10004), None, fake, fake, fake, fake, mem["workspace"], C.byref(h))
    assert code == zs.STAGE_ERR_ARG


def test_ops_reject_bad_arguments_on_the_host():
    L = zs.lib()
    fake = C.c_void_p(0x10000)
    assert L.stage_op_gemm(None, 5, 0, 0, 8, 8, 8, fake, 8, fake, 8, fake, 8, 0, None, None, 0, 1, 0, 0, 0, 0, 0, 0, 0) == zs.STAGE_ERR_ARG
    assert L.stage_op_gemm(None, 0, 0, 0, 8, 8, 8, None, 8, fake, 8, fake, 8, 0, None, None, 0, 1, 0, 0, 0, 0, 0, 0, 0) == zs.STAGE_ERR_ARG
    assert L.stage_op_gemm(None, 0, 0, 0, 8, 8, 8, fake, 8, fake, 8, fake, 8, 0, None, None, 0, 1, 0, 0, 0, 0, 3, 0, 0) == zs.STAGE_ERR_ARG
    assert L.stage_op_adamw(None, 1, 8, 0, fake, None, fake, fake, fake, 1e-4, 0.9, 0.999, 1e-8, 0.01, 1, 1.0) == zs.STAGE_ERR_ARG
    assert L.stage_op_mfma_rate(None, 8, 10, fake, fake) == zs.STAGE_ERR_ARG      # only the shapes 16 and 32 exist
    assert L.stage_op_mfma_rate(None, 16, 0, fake, fake) == zs.STAGE_ERR_ARG
    assert L.stage_op_mfma_rate(None, 16, 10, None, fake) == zs.STAGE_ERR_ARG
    good, far, odd = (C.c_int32 * 64)(*[16 * l for l in range(64)]), (C.c_int32 * 64)(*[20992] * 64), (C.c_int32 * 64)(*[8] * 64)
    assert L.stage_op_lds_probe(None, 2, good, fake, 10, fake) == zs.STAGE_ERR_ARG     # kinds 0 and 1 only
    assert L.stage_op_lds_probe(None, 0, far, fake, 10, fake) == zs.STAGE_ERR_ARG      # offset beyond the probe's LDS
    assert L.stage_op_lds_probe(None, 0, odd, fake, 10, fake) == zs.STAGE_ERR_ARG      # 16-byte reads at 16-byte offsets
    assert L.stage_op_lds_probe(None, 1, good, None, 10, fake) == zs.STAGE_ERR_ARG
    assert L.stage_op_adamw(None, 0, 8, 0, fake, None, fake, fake, fake, 1e-4, 0.9, 0.999, 1e-8, 0.01, 0, 1.0) == zs.STAGE_ERR_ARG
    # weight gradients with the last round cut along K: sizes, a shape that is cut but gets no scratch, a float dtype
    assert L.stage_op_wgrad_parts_scratch_bytes(0, 8, 128, 128, 2, 1) == -zs.STAGE_ERR_ARG
    assert L.stage_op_wgrad_parts_scratch_bytes(4096, 4096, 4096, 4096, 8, 1) == 0            # 256 tiles: whole rounds
    assert L.stage_op_wgrad_parts_scratch_bytes(4096, 4096, 4096, 4096, 1, 1) == 0            # one part: nothing to cut
    need = L.stage_op_wgrad_parts_scratch_bytes(11008, 4096, 4096, 4096, 8, 1)                # 688 tiles: 176 beyond two rounds
    assert need > 0 and need % (256 * 256 * 4) == 0 and need <= 256 << 20
    parts = (C.c_void_p * 8)(*[0x10000] * 8)
    cut = L.stage_op_wgrad_parts_cut
    assert cut(None, 1, 11008, 4096, 4096, 4096, 8, parts, 11008, parts, 4096, fake, 4096, 1, 0, 0, 0, None, 0) == zs.STAGE_ERR_WORKSPACE
    assert cut(None, 1, 11008, 4096, 4096, 4096, 8, parts, 11008, parts, 4096, fake, 4096, 1, 0, 0, 0, fake, need - 1) == zs.STAGE_ERR_WORKSPACE
    assert cut(None, 0, 11008, 4096, 4096, 4096, 8, parts, 11008, parts, 4096, fake, 4096, 1, 0, 0, 0, fake, need) == zs.STAGE_ERR_ARG
    assert cut(None, 1, 11008, 4096, 4096, 4096, 8, None, 11008, parts, 4096, fake, 4096, 1, 0, 0, 0, fake, need) == zs.STAGE_ERR_ARG
    assert L.stage_op_norm_fwd(None, 1, 1, 4, 12, fake, fake, None, 1e-5, fake, fake, None) == zs.STAGE_ERR_ARG
    assert L.stage_op_attention_fwd(None, 1, 1, 16, 1, 12, fake, fake, fake, 12, fake, 12, fake, 0) == zs.STAGE_ERR_ARG
    # fused gated unit: unknown mode, missing buffer, and a forced MFMA kernel with float or unaligned arguments
    glu = L.stage_op_gemm_glu
    assert glu(None, 1, 3, 8, 8, 8, fake, 8, fake, 8, 64, fake, fake, 0) == zs.STAGE_ERR_ARG
    assert glu(None, 1, 1, 8, 8, 8, fake, 8, fake, 8, 64, fake, None, 0) == zs.STAGE_ERR_ARG
    assert glu(None, 0, 1, 8, 8, 8, fake, 8, fake, 8, 64, fake, fake, 2) == zs.STAGE_ERR_ARG
    assert glu(None, 1, 1, 8, 12, 8, fake, 8, fake, 12, 96, fake, fake, 2) == zs.STAGE_ERR_ARG
    assert glu(None, 1, 2, 8, 8, 8, fake, 8, fake, 8, 0, fake, fake, 5) == zs.STAGE_ERR_ARG
