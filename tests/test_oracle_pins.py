"""Pins for the fp64 oracle: everything here runs on the CPU and uses nothing from the HIP path.

Each pin checks the oracle against something other than itself: central finite
differences, an independently written torch float64 autograd model built from
library routines, torch.optim.AdamW, closed forms and invariants that the
mathematics fixes.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import stage_oracle as so
from workloads import StageConfig, get_config, make_inputs
from workloads.configs import ARCH_GPT, ARCH_LLAMA, DTYPE_F32, segments


def tiny(arch, head=False, **kw):
    base = dict(name="tiny", arch=arch, dtype=DTYPE_F32, layers=2, hidden=16, heads=2, ffn=24 if arch else 32,
                seq=8, microbatch=2, num_microbatches=3, seed=7 + arch + 10 * head)
    if head:
        base.update(vocab=37, has_embed=1, has_head=1)
    base.update(kw)
    return StageConfig(**base)


TINY = [tiny(ARCH_GPT), tiny(ARCH_LLAMA), tiny(ARCH_LLAMA, head=True)]


def draw(cfg, scale_w=10.0):
    """Perturbed inputs in fp64; weights scaled up so that attention and the nonlinearities are far from linear."""
    inp = make_inputs(cfg, perturbed=True)
    p = inp.params.astype(np.float64)
    for name, off, r, c, kind in segments(cfg):
        if kind == "matrix":
            p[off:off + r * c] *= scale_w
    return inp, p


def scalar_fn(cfg, p, inp, i, xi=None):
    """phi = <dY, y> for interior stages, the loss for a head stage."""
    if cfg.has_head:
        loss, _ = so.stage_forward(cfg, p, inp.ids[i], inp.targets[i])
        return loss
    y, _ = so.stage_forward(cfg, p, inp.x[i] if xi is None else xi)
    return float((y * inp.dy[i].astype(np.float64)).sum())


# ---------------------------------------------------------------- finite differences


@pytest.mark.parametrize("cfg", TINY, ids=lambda c: f"arch{c.arch}_head{c.has_head}")
def test_param_grads_match_central_differences(cfg):
    inp, p = draw(cfg)
    rng = np.random.default_rng(1)
    if cfg.has_head:
        _, cache = so.stage_forward(cfg, p, inp.ids[0], inp.targets[0])
        _, g = so.stage_backward(cfg, cache, None, 1.0)
    else:
        _, cache = so.stage_forward(cfg, p, inp.x[0])
        _, g = so.stage_backward(cfg, cache, inp.dy[0].astype(np.float64))
    # sampled single coordinates in every segment
    for name, off, r, c in so.layout(cfg):
        for j in rng.choice(r * c, size=min(3, r * c), replace=False):
            k = off + int(j)
            h = 1e-5 * max(1.0, abs(p[k]))
            pp, pm = p.copy(), p.copy()
            pp[k] += h
            pm[k] -= h
            fd = (scalar_fn(cfg, pp, inp, 0) - scalar_fn(cfg, pm, inp, 0)) / (2 * h)
            if name == "embed.E" and fd == 0.0:
                assert g[k] == 0.0       # a row no token selects
                continue
            assert abs(fd - g[k]) <= 1e-7 * max(abs(fd), abs(g).max()), (name, k, fd, g[k])
    # one random direction over all parameters
    vdir = rng.standard_normal(p.size)
    h = 1e-6
    fd = (scalar_fn(cfg, p + h * vdir, inp, 0) - scalar_fn(cfg, p - h * vdir, inp, 0)) / (2 * h)
    assert abs(fd - g @ vdir) <= 1e-7 * abs(fd)


@pytest.mark.parametrize("cfg", TINY[:2], ids=["gpt", "llama"])
def test_input_grad_matches_central_differences(cfg):
    inp, p = draw(cfg)
    x = inp.x[0].astype(np.float64)
    _, cache = so.stage_forward(cfg, p, x)
    dx, _ = so.stage_backward(cfg, cache, inp.dy[0].astype(np.float64))
    rng = np.random.default_rng(2)
    vdir = rng.standard_normal(x.shape)
    h = 1e-6
    fd = (scalar_fn(cfg, p, inp, 0, x + h * vdir) - scalar_fn(cfg, p, inp, 0, x - h * vdir)) / (2 * h)
    assert abs(fd - (dx * vdir).sum()) <= 1e-7 * abs(fd)
    for _ in range(6):
        t, j = rng.integers(x.shape[0]), rng.integers(x.shape[1])
        xp, xm = x.copy(), x.copy()
        hh = 1e-5 * max(1.0, abs(x[t, j]))
        xp[t, j] += hh
        xm[t, j] -= hh
        fd = (scalar_fn(cfg, p, inp, 0, xp) - scalar_fn(cfg, p, inp, 0, xm)) / (2 * hh)
        assert abs(fd - dx[t, j]) <= 1e-7 * max(abs(fd), np.abs(dx).max())


# ---------------------------------------------------------------- independent torch float64 model


def torch_stage(cfg, P, x_or_ids, targets, mb):
    """The same stage written with torch library routines (layer_norm, rms_norm,
    scaled_dot_product_attention, gelu, silu, cross_entropy, embedding; RoPE as a
    complex multiplication).  Shares nothing with the oracle's code."""
    H, nh, S = cfg.hidden, cfg.heads, cfg.seq
    d = H // nh

    def heads(a):
        return a.reshape(mb, S, nh, d).transpose(1, 2)           # [mb, nh, S, d]

    def rope_c(a):                                               # a: [mb, nh, S, d]
        ac = torch.view_as_complex(a.reshape(mb, nh, S, d // 2, 2).contiguous())
        inv = 1.0 / (cfg.rope_base ** (torch.arange(0, d, 2, dtype=torch.float64) / d))
        ang = torch.outer(torch.arange(S, dtype=torch.float64), inv)
        rot = torch.polar(torch.ones_like(ang), ang)
        return torch.view_as_real(ac * rot).reshape(mb, nh, S, d)

    x = F.embedding(torch.as_tensor(np.asarray(x_or_ids).reshape(-1), dtype=torch.long), P["embed.E"]) \
        if cfg.has_embed else x_or_ids
    for l in range(cfg.layers):
        g = lambda n: P[f"L{l}.{n}"]
        if cfg.arch == ARCH_GPT:
            n1 = F.layer_norm(x, (H,), g("ln1.g"), g("ln1.b"), cfg.norm_eps)
            qkv = F.linear(n1, g("Wqkv").T, g("bqkv"))
            q, k, v = (heads(t) for t in qkv.split(H, dim=1))
            o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(-1, H)
            x = x + F.linear(o, g("Wo").T, g("bo"))
            n2 = F.layer_norm(x, (H,), g("ln2.g"), g("ln2.b"), cfg.norm_eps)
            x = x + F.linear(F.gelu(F.linear(n2, g("W1").T, g("b1"))), g("W2").T, g("b2"))
        else:
            n1 = F.rms_norm(x, (H,), g("rms1.g"), cfg.norm_eps)
            q, k, v = rope_c(heads(n1 @ g("Wq"))), rope_c(heads(n1 @ g("Wk"))), heads(n1 @ g("Wv"))
            o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(-1, H)
            x = x + o @ g("Wo")
            n2 = F.rms_norm(x, (H,), g("rms2.g"), cfg.norm_eps)
            x = x + (F.silu(n2 @ g("Wg")) * (n2 @ g("Wu"))) @ g("Wd")
    if cfg.has_head:
        z = F.rms_norm(x, (H,), P["final_norm.g"], cfg.norm_eps) @ P["head.Wh"]
        return F.cross_entropy(z, torch.as_tensor(np.asarray(targets).reshape(-1), dtype=torch.long))
    return x


@pytest.mark.parametrize("cfg", TINY + [tiny(ARCH_GPT, hidden=32, heads=4, seq=16, layers=3)],
                         ids=lambda c: f"arch{c.arch}_head{c.has_head}_H{c.hidden}")
def test_against_torch_float64_autograd(cfg):
    inp, p = draw(cfg, scale_w=8.0)
    P = {n: torch.tensor(a, dtype=torch.float64, requires_grad=True) for n, a in so.unpack(cfg, p).items()}
    if cfg.has_head:
        loss_o, cache = so.stage_forward(cfg, p, inp.ids[1], inp.targets[1])
        _, g = so.stage_backward(cfg, cache, None, 0.25)
        loss_t = torch_stage(cfg, P, inp.ids[1], inp.targets[1], cfg.microbatch)
        (0.25 * loss_t).backward()
        assert abs(loss_o - loss_t.item()) <= 1e-12 * abs(loss_t.item())
    else:
        x = torch.tensor(inp.x[1], dtype=torch.float64, requires_grad=True)
        dy = inp.dy[1].astype(np.float64)
        y_o, cache = so.stage_forward(cfg, p, inp.x[1])
        dx_o, g = so.stage_backward(cfg, cache, dy)
        y_t = torch_stage(cfg, P, x, None, cfg.microbatch)
        y_t.backward(torch.tensor(dy))
        np.testing.assert_allclose(y_o, y_t.detach().numpy(), rtol=0, atol=1e-11 * np.abs(y_o).max())
        np.testing.assert_allclose(dx_o, x.grad.numpy(), rtol=0, atol=1e-11 * np.abs(dx_o).max())
    G = so.unpack(cfg, g)
    for n in P:
        ref = P[n].grad.numpy()
        np.testing.assert_allclose(G[n], ref, rtol=0, atol=1e-11 * max(np.abs(ref).max(), 1e-30), err_msg=n)


# ---------------------------------------------------------------- accumulation, composition


@pytest.mark.parametrize("cfg", TINY, ids=lambda c: f"arch{c.arch}_head{c.has_head}")
def test_accumulated_microbatches_equal_concatenated_batch(cfg):
    inp, p = draw(cfg)
    M = cfg.num_microbatches
    if cfg.has_head:
        step = so.stage_step(cfg, p, inp.ids, None, inp.targets, loss_scale=1.0 / M)
        ids, tg = np.concatenate(inp.ids, 0), np.concatenate(inp.targets, 0)
        loss, cache = so.stage_forward(cfg, p, ids, tg, mb=M * cfg.microbatch)
        _, g = so.stage_backward(cfg, cache, None, 1.0)
        assert abs(np.mean(step["loss"]) - loss) <= 1e-13 * abs(loss)
    else:
        step = so.stage_step(cfg, p, inp.x, inp.dy)
        xs = np.concatenate(inp.x, 0).astype(np.float64)
        y, cache = so.stage_forward(cfg, p, xs, mb=M * cfg.microbatch)
        dx, g = so.stage_backward(cfg, cache, np.concatenate(inp.dy, 0).astype(np.float64))
        np.testing.assert_allclose(np.concatenate(step["y"], 0), y, rtol=0, atol=1e-13 * np.abs(y).max())
        np.testing.assert_allclose(np.concatenate(step["dx"], 0), dx, rtol=0, atol=1e-13 * np.abs(dx).max())
    np.testing.assert_allclose(step["grad"], g, rtol=0, atol=1e-12 * np.abs(g).max())


@pytest.mark.parametrize("arch", [ARCH_GPT, ARCH_LLAMA])
def test_stage_equals_chained_single_layer_stages(arch):
    cfg = tiny(arch, layers=3)
    inp, p = draw(cfg)
    x, dy = inp.x[0].astype(np.float64), inp.dy[0].astype(np.float64)
    y, cache = so.stage_forward(cfg, p, x)
    dx, g = so.stage_backward(cfg, cache, dy)
    one = cfg.with_(layers=1)
    ppl = cfg.params_per_layer
    caches, cur = [], x
    for l in range(3):
        cur, c = so.stage_forward(one, p[l * ppl:(l + 1) * ppl], cur)
        caches.append(c)
    np.testing.assert_allclose(cur, y, rtol=0, atol=1e-13 * np.abs(y).max())
    d = dy
    for l in reversed(range(3)):
        d, gl = so.stage_backward(one, caches[l], d)
        np.testing.assert_allclose(gl, g[l * ppl:(l + 1) * ppl], rtol=0, atol=1e-13 * np.abs(g).max())
    np.testing.assert_allclose(d, dx, rtol=0, atol=1e-13 * np.abs(dx).max())


# ---------------------------------------------------------------- AdamW


def test_adamw_first_step_closed_form():
    rng = np.random.default_rng(3)
    p0, g = rng.standard_normal(1000), rng.standard_normal(1000) * 1e-3
    lr, b1, b2, eps, wd = 1e-4, 0.9, 0.999, 1e-8, 0.01
    p1, m1, v1 = so.adamw(p0, g, np.zeros(1000), np.zeros(1000), 1, lr, b1, b2, eps, wd)
    np.testing.assert_allclose(m1, (1 - b1) * g, rtol=1e-14)
    np.testing.assert_allclose(v1, (1 - b2) * g * g, rtol=1e-14)
    np.testing.assert_allclose(p1, p0 - lr * wd * p0 - lr * g / (np.abs(g) + eps), rtol=0, atol=1e-15)


def test_adamw_constant_gradient_and_zero_gradient():
    rng = np.random.default_rng(4)
    p, g = rng.standard_normal(64), rng.standard_normal(64)
    lr, b1, b2, eps, wd = 1e-3, 0.9, 0.999, 1e-8, 0.0
    m, v = np.zeros(64), np.zeros(64)
    for t in range(1, 8):
        pn, m, v = so.adamw(p, g, m, v, t, lr, b1, b2, eps, wd)
        # bias-corrected moments equal g and g^2 exactly, so every step moves by lr*sign-like amount
        np.testing.assert_allclose(pn - p, -lr * g / (np.abs(g) + eps), rtol=1e-10)
        p = pn
    p0 = rng.standard_normal(64)
    p1, m1, v1 = so.adamw(p0, np.zeros(64), np.zeros(64), np.zeros(64), 1, 1e-4, 0.9, 0.999, 1e-8, 0.01)
    np.testing.assert_allclose(p1, p0 * (1 - 1e-4 * 0.01), rtol=1e-15)
    assert not m1.any() and not v1.any()


def test_adamw_matches_torch_optim_over_steps_and_grad_scale():
    rng = np.random.default_rng(5)
    n = 513
    p0 = rng.standard_normal(n)
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=3e-3, betas=(0.8, 0.95), eps=1e-6, weight_decay=0.1)
    p, m, v = p0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 11):
        g = rng.standard_normal(n) * 10.0 ** rng.integers(-4, 2)
        tp.grad = torch.tensor(0.5 * g)
        opt.step()
        p, m, v = so.adamw(p, g, m, v, t, 3e-3, 0.8, 0.95, 1e-6, 0.1, grad_scale=0.5)
        # torch scales p by (1 - lr*wd) before the Adam move: differs from the
        # single-expression form by lr^2*wd*|move| ~ 1e-9 relative here.
        np.testing.assert_allclose(p, tp.detach().numpy(), rtol=0, atol=2e-8)


def test_optimizer_step_touches_only_the_shard():
    cfg = tiny(ARCH_LLAMA)
    rng = np.random.default_rng(6)
    P = cfg.n_params
    master, g = rng.standard_normal(P), rng.standard_normal(P)
    b, e = 100, 1234
    new, m, v = so.stage_optimizer_step(cfg, master, g, np.zeros(e - b), np.zeros(e - b), 1, (b, e))
    assert np.array_equal(new[:b], master[:b]) and np.array_equal(new[e:], master[e:])
    assert np.all(new[b:e] != master[b:e]) and m.shape == (e - b,)
    np.testing.assert_allclose(m, 0.1 * g[b:e], rtol=1e-14)


# ---------------------------------------------------------------- norms, activations


def test_norm_statistics_and_scale_invariance():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((5, 64)) * 3 + 1
    eps = 1e-5
    n, _ = so.layernorm_fwd(x, np.ones(64), np.zeros(64), eps)
    var = x.var(axis=1)
    np.testing.assert_allclose(n.mean(axis=1), 0, atol=1e-14)
    np.testing.assert_allclose(n.var(axis=1), var / (var + eps), rtol=1e-12)
    r, _ = so.rmsnorm_fwd(x, np.ones(64), eps)
    ms = (x * x).mean(axis=1)
    np.testing.assert_allclose((r * r).mean(axis=1), ms / (ms + eps), rtol=1e-12)
    n2, _ = so.layernorm_fwd(1e3 * x, np.ones(64), np.zeros(64), 0.0)
    n0, _ = so.layernorm_fwd(x, np.ones(64), np.zeros(64), 0.0)
    np.testing.assert_allclose(n2, n0, rtol=1e-10, atol=1e-12)
    g, b = rng.standard_normal(64), rng.standard_normal(64)
    ng, _ = so.layernorm_fwd(x, g, b, eps)
    np.testing.assert_allclose(ng, n * g + b, rtol=1e-14)


def test_gelu_and_silu_identities():
    z = np.linspace(-6, 6, 101)
    assert so.gelu(np.array([0.0]))[0] == 0.0
    assert so.gelu_grad(np.array([0.0]))[0] == 0.5
    np.testing.assert_allclose(so.gelu(z) - so.gelu(-z), z, atol=1e-15)
    ref = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in z])
    np.testing.assert_allclose(so.gelu(z), ref, rtol=1e-15, atol=1e-300)
    silu = z * so.sigmoid(z)
    np.testing.assert_allclose(silu - (-z) * so.sigmoid(-z), z, atol=1e-15)
    np.testing.assert_allclose(so.gelu(z), F.gelu(torch.tensor(z)).numpy(), rtol=1e-13, atol=1e-16)
    h = 1e-6
    np.testing.assert_allclose(so.gelu_grad(z), (so.gelu(z + h) - so.gelu(z - h)) / (2 * h), atol=1e-9)


# ---------------------------------------------------------------- attention, RoPE


def test_attention_causality_rowsum_and_special_cases():
    rng = np.random.default_rng(9)
    q, k, v = (rng.standard_normal((2, 12, 3, 8)) for _ in range(3))
    o = so.attention_fwd(q, k, v)
    k2, v2, q2 = k.copy(), v.copy(), q.copy()
    k2[:, 7:], v2[:, 7:], q2[:, 7:] = 5.0, -3.0, 2.0
    o2 = so.attention_fwd(q2, k2, v2)
    assert np.array_equal(o[:, :7], o2[:, :7])
    p = so._probs(q[0, :, 0], k[0, :, 0])
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-14)
    assert np.all(np.triu(p, 1) == 0)
    np.testing.assert_allclose(o[:, 0], v[:, 0], rtol=1e-14)               # first position sees only itself
    ke = np.broadcast_to(k[:, :1], k.shape)
    om = so.attention_fwd(q, ke, v)                                          # equal keys -> running mean of v
    run = np.cumsum(v, axis=1) / np.arange(1, 13)[None, :, None, None]
    np.testing.assert_allclose(om, run, rtol=1e-12, atol=1e-14)
    # explicit brute force on one head
    b, h, i = 1, 2, 9
    s = np.array([q[b, i, h] @ k[b, j, h] / math.sqrt(8) for j in range(i + 1)])
    w = np.exp(s - s.max())
    w /= w.sum()
    np.testing.assert_allclose(o[b, i, h], sum(w[j] * v[b, j, h] for j in range(i + 1)), rtol=1e-13)


def test_rope_properties():
    rng = np.random.default_rng(10)
    u = rng.standard_normal((2, 10, 3, 8))
    r = so.rope(u, 10000.0)
    np.testing.assert_allclose(r[:, 0], u[:, 0], rtol=0, atol=0)                                  # position 0: identity
    np.testing.assert_allclose(r[..., 0::2] ** 2 + r[..., 1::2] ** 2, u[..., 0::2] ** 2 + u[..., 1::2] ** 2, rtol=1e-13)
    np.testing.assert_allclose(so.rope(r, 10000.0, sign=-1.0), u, rtol=1e-13, atol=1e-15)         # inverse / backward map
    # explicit value: pair i at position t rotates by t * base^(-2i/d)
    t, i = 7, 2
    th = t * 10000.0 ** (-2 * i / 8)
    a, b = u[1, t, 0, 2 * i], u[1, t, 0, 2 * i + 1]
    np.testing.assert_allclose(r[1, t, 0, 2 * i], a * math.cos(th) - b * math.sin(th), rtol=1e-14)
    np.testing.assert_allclose(r[1, t, 0, 2 * i + 1], a * math.sin(th) + b * math.cos(th), rtol=1e-14)
    # relative-position property: shifting every position by a constant leaves attention unchanged
    q, k, v = (rng.standard_normal((1, 10, 2, 8)) for _ in range(3))
    o0 = so.attention_fwd(so.rope(q, 100.0), so.rope(k, 100.0), v)
    o5 = so.attention_fwd(so.rope(q, 100.0, pos0=5), so.rope(k, 100.0, pos0=5), v)
    np.testing.assert_allclose(o0, o5, rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- cross entropy, embedding


def test_cross_entropy_uniform_and_dominant_logits():
    cfg = tiny(ARCH_LLAMA, head=True)
    inp, p = draw(cfg)
    P = so.unpack(cfg, p)
    P["head.Wh"] = np.zeros_like(P["head.Wh"])
    p0 = so.pack(cfg, P)
    loss, cache = so.stage_forward(cfg, p0, inp.ids[0], inp.targets[0])
    assert abs(loss - math.log(cfg.vocab)) < 1e-14
    _, g = so.stage_backward(cfg, cache, None, 1.0)
    T = cfg.tokens
    # dWh = nf^T dz with dz = (1/V - onehot)/T
    dz = np.full((T, cfg.vocab), 1.0 / cfg.vocab)
    dz[np.arange(T), inp.targets[0].reshape(-1)] -= 1.0
    np.testing.assert_allclose(so.unpack(cfg, g)["head.Wh"], cache["nf"].T @ (dz / T), rtol=1e-12, atol=1e-16)
    # ln 32000 for the benchmark vocabulary
    assert abs(math.log(32000) - 10.373491181781864) < 1e-12


def test_embedding_rows_and_repeated_ids():
    cfg = tiny(ARCH_LLAMA, head=True, layers=1)
    inp, p = draw(cfg)
    ids = inp.ids[0].copy()
    ids[0, :4] = 5                                   # a repeated id
    _, cache = so.stage_forward(cfg, p, ids, inp.targets[0])
    E = so.unpack(cfg, p)["embed.E"]
    _, g = so.stage_backward(cfg, cache, None, 1.0)
    dE = so.unpack(cfg, g)["embed.E"]
    used = np.unique(ids)
    assert not dE[np.setdiff1d(np.arange(cfg.vocab), used)].any()
    assert dE[5].any()
    # brute force scatter with a python loop, using the layer-0 input gradient recomputed by finite differences
    # of the rows: d loss / d E[5] must equal the sum over the 4+ positions that read row 5
    h = 1e-6
    for col in (0, 7):
        Ep, Em = E.copy(), E.copy()
        Ep[5, col] += h
        Em[5, col] -= h
        Pp, Pm = so.unpack(cfg, p), so.unpack(cfg, p)
        Pp["embed.E"], Pm["embed.E"] = Ep, Em
        fp, _ = so.stage_forward(cfg, so.pack(cfg, Pp), ids, inp.targets[0])
        fm, _ = so.stage_forward(cfg, so.pack(cfg, Pm), ids, inp.targets[0])
        assert abs((fp - fm) / (2 * h) - dE[5, col]) <= 1e-7 * np.abs(dE).max()


# ---------------------------------------------------------------- layout


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4a", "C4b", "C5", "C3t", "C5t"])
def test_layout_matches_workload_segments_and_counts(name):
    cfg = get_config(name)
    a = so.layout(cfg)
    b = [(n, o, r, c) for n, o, r, c, _ in segments(cfg)]
    assert a == b
    assert so.n_params(cfg) == cfg.n_params
    expect = {"C1": 1579520, "C2": 302149632, "C3": 1619066880, "C4a": 951613440, "C4b": 3806453760,
              "C5": 1071681536}
    if name in expect:
        assert cfg.n_params == expect[name]


def test_oracle_has_not_drifted_from_stored_summary():
    """tests/golden/oracle_c1_summary.json is written by tests/golden/make_oracle_golden.py from the oracle alone."""
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_oracle_golden", os.path.join(here, "make_oracle_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(here, "oracle_c1_summary.json")) as f:
        stored = json.load(f)
    for rec in stored:
        now = mod.summary(rec["config"])
        for k, v in rec.items():
            if isinstance(v, float):
                assert abs(now[k] - v) <= 1e-9 * abs(v), (rec["config"], k)
            elif isinstance(v, dict):
                for kk, vv in v.items():
                    assert abs(now[k][kk] - vv) <= 1e-9 * max(abs(vv), 1e-12), (rec["config"], k, kk)


# ---------------------------------------------------------------- runtime model


def test_linear_fit_recovers_lines_and_matches_library_least_squares():
    """Pins of the oracle's least-squares line: exact recovery of a line, numpy's polynomial fit and its
    correlation coefficient on noisy data, invariance of r2 under shifts and scalings, the two-point case."""
    rng = np.random.default_rng(5)
    x = np.array([1.0, 2.0, 3.0, 4.0, 6.0, 8.0])
    a, b, r2 = so.linear_fit(x, 0.75 + 2.5 * x)
    assert abs(a - 0.75) < 1e-12 and abs(b - 2.5) < 1e-12 and abs(r2 - 1.0) < 1e-12
    y = 3.0 - 0.4 * x + rng.standard_normal(x.size) * 0.3
    a, b, r2 = so.linear_fit(x, y)
    pb, pa = np.polyfit(x, y, 1)
    assert abs(a - pa) < 1e-10 and abs(b - pb) < 1e-10
    assert abs(r2 - np.corrcoef(x, y)[0, 1] ** 2) < 1e-10
    a2, b2, r22 = so.linear_fit(10.0 * x - 3.0, 2.0 * y + 7.0)
    assert abs(r22 - r2) < 1e-10 and abs(b2 - 2.0 * b / 10.0) < 1e-10
    a, b, r2 = so.linear_fit([2.0, 5.0], [1.0, 7.0])              # two points: the line through them
    assert abs(b - 2.0) < 1e-12 and abs(a + 3.0) < 1e-12 and abs(r2 - 1.0) < 1e-12
    assert so.linear_fit([1.0, 2.0, 3.0], [4.0, 4.0, 4.0]) == (4.0, 0.0, 1.0)


def test_half_overflow_criterion_is_round_to_nearest_even():
    """The overflow criterion of fp16 training (the paper's precision, Section 6.1) against the library's own
    conversion to IEEE half: a magnitude overflows exactly when numpy's round-to-nearest-even float16 of it is
    not finite.  65504 is the largest finite half; values up to just below 65520 still round down to it; the
    tie 65520 goes to the even side, which is 2**16 = inf."""
    with np.errstate(over="ignore", invalid="ignore"):
        for x in (0.0, 1.0, 65503.9, 65504.0, 65504.1, 65519.9, np.nextafter(65520.0, 0.0), 65520.0,
                  np.nextafter(65520.0, 1e9), 65536.0, 1e30, float("inf"), float("nan"), -65519.9, -65520.0):
            finite_as_half = bool(np.isfinite(np.float64(x).astype(np.float16)))
            assert so.gradients_overflow_fp16(x) == (not finite_as_half), x
    # the hand-derived boundary, independent of the library: largest finite + half a spacing of 32
    assert not so.gradients_overflow_fp16(65504.0 + 15.999) and so.gradients_overflow_fp16(65504.0 + 16.0)


def test_loss_scale_rule_hand_traced():
    """Dynamic loss scaling (fp16 mixed precision, Section 6.1; the rule is the reading stated in the oracle) over a
    scripted run with growth interval 3, every (scale, good-step count) written out by hand: an overflow halves the
    scale and restarts the count; the third good step in a row doubles the scale and restarts the count."""
    script = [  # found_inf, scale after, count after
        (0, 65536.0, 1), (0, 65536.0, 2), (1, 32768.0, 0), (0, 32768.0, 1), (0, 32768.0, 2),
        (0, 65536.0, 0), (0, 65536.0, 1), (1, 32768.0, 0), (1, 16384.0, 0), (0, 16384.0, 1),
        (0, 16384.0, 2), (0, 32768.0, 0), (0, 32768.0, 1), (0, 32768.0, 2), (0, 65536.0, 0)]
    scale, good = 65536.0, 0
    for found, want_scale, want_good in script:
        scale, good = so.loss_scale_update(scale, good, found, 0.5, 2.0, 3)
        assert (scale, good) == (want_scale, want_good), (found, scale, good)
    # the defaults: halving, doubling, 2000 good steps between doublings
    assert so.loss_scale_update(8.0, 5, 1) == (4.0, 0)
    assert so.loss_scale_update(8.0, 1998, 0) == (8.0, 1999)
    assert so.loss_scale_update(8.0, 1999, 0) == (16.0, 0)
    # other factors are honoured as given
    assert so.loss_scale_update(8.0, 0, 1, backoff=0.25) == (2.0, 0)
    assert so.loss_scale_update(8.0, 0, 0, growth=4.0, growth_interval=1) == (32.0, 0)
