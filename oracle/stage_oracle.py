"""CPU fp64 oracle for the per-stage training step.  TEST INFRASTRUCTURE ONLY.

This module is the plain, slow, written-out definition of what one pipeline
(mini)stage computes in the paper's schedule: forward over the stage's decoder
layers for every microbatch, backward for every microbatch with gradients summed
across microbatches (Section 4.1.1: all forwards of a ministage, then all its
backwards), then one optimizer update restricted to the rank's data-parallel
shard, after which the gradients are dropped (Section 4.1.2).  The paper fixes
that structure but not the layer math or the optimizer; those are the standard
definitions of the components the benchmark configs name (GPT: pre-LayerNorm,
GELU, biases; Llama: pre-RMSNorm, SwiGLU, RoPE; AdamW with decoupled decay),
written here in numpy float64 with no blocking, fusion or reordering.
np.matmul, np.exp and scipy.special.erf are the only library primitives.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this file.  It shares no code with the HIP path and does not import it.

Parity pins (tests/test_oracle_pins.py): central finite differences on every
parameter segment and on the stage input; an independent torch float64 autograd
model; torch.optim.AdamW and the first-step / constant-gradient closed forms;
k accumulated microbatches == one concatenated batch; causality; RoPE relative
position property; cross-entropy = ln V at zero head weights; L-layer stage ==
L chained one-layer stages; the least-squares line against numpy.polyfit; the
half-precision overflow criterion against numpy's float16 conversion at the
boundary values; the loss-scale rule against a hand-written trace.  No function
here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

ARCH_GPT = 0
ARCH_LLAMA = 1

# --------------------------------------------------------------------------
# flat parameter layout
# --------------------------------------------------------------------------


def layout(cfg):
    """[(name, offset, rows, cols)] in flat order: [embed] layer_0..layer_{L-1} [final_norm, head].

    Matrices are row-major [in, out], applied as y = x @ W.  GPT's Wqkv has its
    columns ordered [Q | K | V], each block `hidden` wide, head h occupying
    columns h*d..(h+1)*d-1 of its block.
    """
    H, F, V = cfg.hidden, cfg.ffn, cfg.vocab
    segs = []
    off = 0

    def add(name, rows, cols):
        nonlocal off
        segs.append((name, off, rows, cols))
        off += rows * cols

    if cfg.has_embed:
        add("embed.E", V, H)
    for l in range(cfg.layers):
        p = "L%d." % l
        if cfg.arch == ARCH_GPT:
            for name, r, c in (("ln1.g", 1, H), ("ln1.b", 1, H), ("Wqkv", H, 3 * H), ("bqkv", 1, 3 * H),
                               ("Wo", H, H), ("bo", 1, H), ("ln2.g", 1, H), ("ln2.b", 1, H),
                               ("W1", H, F), ("b1", 1, F), ("W2", F, H), ("b2", 1, H)):
                add(p + name, r, c)
        else:
            for name, r, c in (("rms1.g", 1, H), ("Wq", H, H), ("Wk", H, H), ("Wv", H, H), ("Wo", H, H),
                               ("rms2.g", 1, H), ("Wg", H, F), ("Wu", H, F), ("Wd", F, H)):
                add(p + name, r, c)
    if cfg.has_head:
        add("final_norm.g", 1, H)
        add("head.Wh", H, V)
    return segs


def n_params(cfg):
    name, off, r, c = layout(cfg)[-1]
    return off + r * c


def unpack(cfg, flat):
    """name -> float64 view-shaped copy of the segment ([cols] for vectors, [rows, cols] for matrices)."""
    flat = np.asarray(flat, dtype=np.float64)
    out = {}
    for name, off, r, c in layout(cfg):
        seg = flat[off:off + r * c]
        out[name] = seg.reshape(c) if r == 1 else seg.reshape(r, c)
    return out


def pack(cfg, named):
    flat = np.zeros(n_params(cfg), dtype=np.float64)
    for name, off, r, c in layout(cfg):
        flat[off:off + r * c] = np.asarray(named[name], dtype=np.float64).reshape(-1)
    return flat


# --------------------------------------------------------------------------
# elementary operations and their derivatives
# --------------------------------------------------------------------------


def layernorm_fwd(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)   # biased variance
    r = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * r
    return xhat * g + b, (xhat, r)


def layernorm_bwd(dn, g, cache):
    xhat, r = cache
    u = dn * g
    dx = r * (u - u.mean(axis=-1, keepdims=True) - xhat * (u * xhat).mean(axis=-1, keepdims=True))
    return dx, (dn * xhat).sum(axis=0), dn.sum(axis=0)


def rmsnorm_fwd(x, g, eps):
    r = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    xhat = x * r
    return xhat * g, (xhat, r)


def rmsnorm_bwd(dn, g, cache):
    xhat, r = cache
    u = dn * g
    dx = r * (u - xhat * (u * xhat).mean(axis=-1, keepdims=True))
    return dx, (dn * xhat).sum(axis=0)


def gelu(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))        # z * Phi(z)


def gelu_grad(z):
    Phi = 0.5 * (1.0 + erf(z / np.sqrt(2.0)))
    phi = np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)
    return Phi + z * phi


def sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def rope(u, base, sign=1.0, pos0=0):
    """Rotate adjacent pairs (2i, 2i+1) of each head by theta = t * base**(-2i/d).

    u: [mb, S, nh, d]; positions t = pos0 .. pos0+S-1.  sign=-1 applies the
    inverse rotation, which is also the backward map for the gradients.
    """
    mb, S, nh, d = u.shape
    i = np.arange(d // 2, dtype=np.float64)
    t = np.arange(S, dtype=np.float64) + pos0
    theta = t[:, None] * base ** (-2.0 * i / d)[None, :]           # [S, d/2]
    c = np.cos(theta)[None, :, None, :]
    s = sign * np.sin(theta)[None, :, None, :]
    a, b = u[..., 0::2], u[..., 1::2]
    out = np.empty_like(u)
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


def _probs(q, k):
    """Causal softmax probabilities of one (sequence, head): q, k are [S, d]."""
    S, d = q.shape
    s = (q @ k.T) / np.sqrt(d)
    s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def attention_fwd(q, k, v):
    """o_i = sum_{j<=i} softmax_j(q_i.k_j / sqrt(d)) v_j per (sequence, head); q,k,v: [mb, S, nh, d]."""
    mb, S, nh, d = q.shape
    o = np.empty_like(q)
    for b in range(mb):
        for h in range(nh):
            o[b, :, h, :] = _probs(q[b, :, h, :], k[b, :, h, :]) @ v[b, :, h, :]
    return o


def attention_bwd(do, q, k, v):
    mb, S, nh, d = q.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    for b in range(mb):
        for h in range(nh):
            qh, kh, vh, doh = q[b, :, h, :], k[b, :, h, :], v[b, :, h, :], do[b, :, h, :]
            p = _probs(qh, kh)
            dv[b, :, h, :] = p.T @ doh
            dp = doh @ vh.T
            ds = p * (dp - (p * dp).sum(axis=-1, keepdims=True))
            dq[b, :, h, :] = (ds @ kh) / np.sqrt(d)
            dk[b, :, h, :] = (ds.T @ qh) / np.sqrt(d)
    return dq, dk, dv


# --------------------------------------------------------------------------
# decoder layers
# --------------------------------------------------------------------------


def _heads(cfg, a):
    return a.reshape(cfg.microbatch_now, cfg.seq, cfg.heads, cfg.hidden // cfg.heads)


class _Shape:
    """Shape facts a layer needs; microbatch_now lets a caller run a different batch size."""

    def __init__(self, cfg, mb=None):
        self.arch, self.hidden, self.heads, self.ffn, self.seq = cfg.arch, cfg.hidden, cfg.heads, cfg.ffn, cfg.seq
        self.microbatch_now = cfg.microbatch if mb is None else mb
        self.norm_eps, self.rope_base = cfg.norm_eps, cfg.rope_base


def gpt_layer_fwd(sh, P, pre, x):
    H = sh.hidden
    n1, c1 = layernorm_fwd(x, P[pre + "ln1.g"], P[pre + "ln1.b"], sh.norm_eps)
    qkv = n1 @ P[pre + "Wqkv"] + P[pre + "bqkv"]
    q, k, v = _heads(sh, qkv[:, :H]), _heads(sh, qkv[:, H:2 * H]), _heads(sh, qkv[:, 2 * H:])
    o = attention_fwd(q, k, v).reshape(-1, H)
    x2 = x + o @ P[pre + "Wo"] + P[pre + "bo"]
    n2, c2 = layernorm_fwd(x2, P[pre + "ln2.g"], P[pre + "ln2.b"], sh.norm_eps)
    z = n2 @ P[pre + "W1"] + P[pre + "b1"]
    a = gelu(z)
    y = x2 + a @ P[pre + "W2"] + P[pre + "b2"]
    return y, dict(n1=n1, c1=c1, q=q, k=k, v=v, o=o, n2=n2, c2=c2, z=z, a=a)


def gpt_layer_bwd(sh, P, pre, C, dy, G):
    H = sh.hidden
    da = dy @ P[pre + "W2"].T
    G[pre + "W2"] = C["a"].T @ dy
    G[pre + "b2"] = dy.sum(axis=0)
    dz = da * gelu_grad(C["z"])
    dn2 = dz @ P[pre + "W1"].T
    G[pre + "W1"] = C["n2"].T @ dz
    G[pre + "b1"] = dz.sum(axis=0)
    dxn, G[pre + "ln2.g"], G[pre + "ln2.b"] = layernorm_bwd(dn2, P[pre + "ln2.g"], C["c2"])
    dx2 = dy + dxn
    do = dx2 @ P[pre + "Wo"].T
    G[pre + "Wo"] = C["o"].T @ dx2
    G[pre + "bo"] = dx2.sum(axis=0)
    dq, dk, dv = attention_bwd(_heads(sh, do), C["q"], C["k"], C["v"])
    dqkv = np.concatenate([dq.reshape(-1, H), dk.reshape(-1, H), dv.reshape(-1, H)], axis=1)
    dn1 = dqkv @ P[pre + "Wqkv"].T
    G[pre + "Wqkv"] = C["n1"].T @ dqkv
    G[pre + "bqkv"] = dqkv.sum(axis=0)
    dxn, G[pre + "ln1.g"], G[pre + "ln1.b"] = layernorm_bwd(dn1, P[pre + "ln1.g"], C["c1"])
    return dx2 + dxn


def llama_layer_fwd(sh, P, pre, x):
    H = sh.hidden
    n1, c1 = rmsnorm_fwd(x, P[pre + "rms1.g"], sh.norm_eps)
    q = rope(_heads(sh, n1 @ P[pre + "Wq"]), sh.rope_base)
    k = rope(_heads(sh, n1 @ P[pre + "Wk"]), sh.rope_base)
    v = _heads(sh, n1 @ P[pre + "Wv"])
    o = attention_fwd(q, k, v).reshape(-1, H)
    x2 = x + o @ P[pre + "Wo"]
    n2, c2 = rmsnorm_fwd(x2, P[pre + "rms2.g"], sh.norm_eps)
    gt = n2 @ P[pre + "Wg"]
    up = n2 @ P[pre + "Wu"]
    a = gt * sigmoid(gt) * up                                   # silu(gate) * up
    y = x2 + a @ P[pre + "Wd"]
    return y, dict(n1=n1, c1=c1, q=q, k=k, v=v, o=o, n2=n2, c2=c2, gt=gt, up=up, a=a)


def llama_layer_bwd(sh, P, pre, C, dy, G):
    H = sh.hidden
    da = dy @ P[pre + "Wd"].T
    G[pre + "Wd"] = C["a"].T @ dy
    sg = sigmoid(C["gt"])
    dup = da * C["gt"] * sg
    dgt = da * C["up"] * sg * (1.0 + C["gt"] * (1.0 - sg))
    dn2 = dgt @ P[pre + "Wg"].T + dup @ P[pre + "Wu"].T
    G[pre + "Wg"] = C["n2"].T @ dgt
    G[pre + "Wu"] = C["n2"].T @ dup
    dxn, G[pre + "rms2.g"] = rmsnorm_bwd(dn2, P[pre + "rms2.g"], C["c2"])
    dx2 = dy + dxn
    do = dx2 @ P[pre + "Wo"].T
    G[pre + "Wo"] = C["o"].T @ dx2
    dq, dk, dv = attention_bwd(_heads(sh, do), C["q"], C["k"], C["v"])
    dq = rope(dq, sh.rope_base, sign=-1.0).reshape(-1, H)
    dk = rope(dk, sh.rope_base, sign=-1.0).reshape(-1, H)
    dv = dv.reshape(-1, H)
    dn1 = dq @ P[pre + "Wq"].T + dk @ P[pre + "Wk"].T + dv @ P[pre + "Wv"].T
    G[pre + "Wq"] = C["n1"].T @ dq
    G[pre + "Wk"] = C["n1"].T @ dk
    G[pre + "Wv"] = C["n1"].T @ dv
    dxn, G[pre + "rms1.g"] = rmsnorm_bwd(dn1, P[pre + "rms1.g"], C["c1"])
    return dx2 + dxn


# --------------------------------------------------------------------------
# one microbatch through the stage
# --------------------------------------------------------------------------


def stage_forward(cfg, flat_params, x_or_ids, targets=None, mb=None):
    """Forward of one microbatch.

    Interior stage: x_or_ids is [T, H]; returns (y [T,H], cache).
    has_embed: x_or_ids is int ids [mb, S], x = E[ids].
    has_head: additionally z = RMSNorm(y; g_f) @ Wh and the microbatch loss
    -(1/T) sum_t log softmax(z_t)[target_t]; returns (loss, cache) instead of y.
    """
    sh = _Shape(cfg, mb)
    P = unpack(cfg, flat_params)
    cache = {"P": P, "sh": sh, "layers": []}
    if cfg.has_embed:
        ids = np.asarray(x_or_ids).reshape(-1)
        cache["ids"] = ids
        x = P["embed.E"][ids, :]
    else:
        x = np.asarray(x_or_ids, dtype=np.float64)
    fwd = gpt_layer_fwd if cfg.arch == ARCH_GPT else llama_layer_fwd
    for l in range(cfg.layers):
        x, C = fwd(sh, P, "L%d." % l, x)
        cache["layers"].append(C)
    cache["y"] = x
    if not cfg.has_head:
        return x, cache
    nf, cf = rmsnorm_fwd(x, P["final_norm.g"], sh.norm_eps)
    z = nf @ P["head.Wh"]
    tg = np.asarray(targets).reshape(-1)
    zs = z - z.max(axis=-1, keepdims=True)
    logp = zs - np.log(np.exp(zs).sum(axis=-1, keepdims=True))
    T = z.shape[0]
    loss = -logp[np.arange(T), tg].sum() / T
    cache.update(nf=nf, cf=cf, logp=logp, tg=tg)
    return loss, cache


def stage_backward(cfg, cache, dy=None, loss_scale=1.0):
    """Backward of one microbatch: returns (dx [T,H] or None for has_embed, flat gradient fp64[P]).

    Interior stage: dy is the upstream gradient of y.  has_head: the seed is
    dz = loss_scale * (softmax(z) - onehot(target)) / T.
    """
    P, sh = cache["P"], cache["sh"]
    G = {}
    if cfg.has_head:
        T = cache["logp"].shape[0]
        dz = np.exp(cache["logp"])
        dz[np.arange(T), cache["tg"]] -= 1.0
        dz *= loss_scale / T
        G["head.Wh"] = cache["nf"].T @ dz
        dnf = dz @ P["head.Wh"].T
        dcur, G["final_norm.g"] = rmsnorm_bwd(dnf, P["final_norm.g"], cache["cf"])
    else:
        dcur = np.asarray(dy, dtype=np.float64)
    bwd = gpt_layer_bwd if cfg.arch == ARCH_GPT else llama_layer_bwd
    for l in reversed(range(cfg.layers)):
        dcur = bwd(sh, P, "L%d." % l, cache["layers"][l], dcur, G)
    if cfg.has_embed:
        dE = np.zeros_like(P["embed.E"])
        np.add.at(dE, cache["ids"], dcur)                 # repeated ids sum their rows
        G["embed.E"] = dE
        dcur = None
    return dcur, pack(cfg, G)


# --------------------------------------------------------------------------
# optimizer and the whole step
# --------------------------------------------------------------------------


def adamw(p, g, m, v, t, lr, beta1, beta2, eps, wd, grad_scale=1.0):
    """One AdamW update (decoupled weight decay) of step t >= 1 on equally shaped fp64 arrays.

    Decay uses the pre-update p; eps is added after the bias-corrected square root.
    Returns new (p, m, v).
    """
    g = grad_scale * g
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    p = p - lr * (mhat / (np.sqrt(vhat) + eps) + wd * p)
    return p, m, v


def stage_optimizer_step(cfg, master, grad_acc, m, v, t, shard, grad_scale=1.0):
    """AdamW on flat indices [shard[0], shard[1]) only; m, v are shard-sized.  Returns new (master, m, v)."""
    b, e = shard
    master = np.array(master, dtype=np.float64)
    pn, mn, vn = adamw(master[b:e], np.asarray(grad_acc, dtype=np.float64)[b:e], np.asarray(m, dtype=np.float64),
                       np.asarray(v, dtype=np.float64), t, cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps,
                       cfg.weight_decay, grad_scale)
    master[b:e] = pn
    return master, mn, vn


def stage_step(cfg, compute_params, xs, dys=None, targets=None, loss_scale=1.0):
    """All forwards, then all backwards with gradients summed over microbatches.

    compute_params are the values the layers use (bf16-rounded for bf16 configs).
    Returns dict(y=[...] or loss=[...], dx=[...], grad=fp64[P]).
    """
    M = len(xs)
    outs, caches = [], []
    for i in range(M):
        o, c = stage_forward(cfg, compute_params, xs[i], None if targets is None else targets[i])
        outs.append(o)
        caches.append(c)
    grad = np.zeros(n_params(cfg), dtype=np.float64)
    dxs = [None] * M
    for i in reversed(range(M)):
        dx, g = stage_backward(cfg, caches[i], None if dys is None else dys[i], loss_scale)
        dxs[i] = dx
        grad += g
        caches[i] = None
    key = "loss" if cfg.has_head else "y"
    return {key: outs, "dx": dxs, "grad": grad}


# --------------------------------------------------------------------------
# runtime model for the planner
# --------------------------------------------------------------------------


def linear_fit(x, y):
    """Ordinary least squares y = a + b*x (the paper's Section 4.3, "Profiling": a linear model fitted to
    runtimes measured at small batch sizes predicts the others).  The textbook definition: b = cov(x, y) /
    var(x), a = mean(y) - b*mean(x); r2 = 1 - SS_res / SS_tot (1 when all y are equal).
    Returns (a, b, r2)."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    xb, yb = x.mean(), y.mean()
    b = ((x - xb) * (y - yb)).sum() / ((x - xb) ** 2).sum()
    a = yb - b * xb
    ss_res = ((y - (a + b * x)) ** 2).sum()
    ss_tot = ((y - yb) ** 2).sum()
    return float(a), float(b), float(1.0 - ss_res / ss_tot) if ss_tot > 0 else 1.0



# --------------------------------------------------------------------------
# dynamic loss scaling (fp16 mixed precision)
# --------------------------------------------------------------------------


def loss_scale_update(scale, good_steps, found_inf, backoff=0.5, growth=2.0, growth_interval=2000):
    """The usual dynamic loss-scaling rule for fp16 mixed precision (the precision the paper trains in,
    Section 6.1; the paper does not spell the rule out): a step whose gradients overflowed is skipped and
    multiplies the scale by backoff; growth_interval consecutive good steps multiply it by growth.
    Returns the new (scale, good_steps)."""
    if found_inf:
        return scale * backoff, 0
    good_steps += 1
    if good_steps >= growth_interval:
        return scale * growth, 0
    return scale, good_steps


def gradients_overflow_fp16(dy_scaled_max):
    """Whether an upstream gradient of that magnitude turns into inf (or is nan) when it is rounded to IEEE half
    with round-to-nearest-even, the precision the paper trains in (Section 6.1): then the seed itself is not
    finite and every gradient downstream of it is not either.  The largest finite half is
    (2 - 2**-10) * 2**15 = 65504 and the spacing in its binade is 32, so everything below the midpoint
    65504 + 16 = 65520 still rounds to a finite half; the midpoint itself is a tie between 65504 (odd last
    mantissa bit) and 2**16 (even), goes to the even side and overflows."""
    x = abs(float(dy_scaled_max))
    largest_finite = (2.0 - 2.0 ** -10) * 2.0 ** 15
    half_spacing = 2.0 ** (15 - 10) / 2.0
    return not (x < largest_finite + half_spacing)      # also true for nan
