"""GPU parity of single kernels (stage_op_* entry points) against the oracle's functions."""
import numpy as np
import pytest
import torch

import paper_2507_10392_amd as zs
from harness import dev, log_report, rel_err
from oracle import stage_oracle as so
from workloads import round_bf16, round_f16

pytestmark = pytest.mark.gpu

TD = {0: torch.float32, 1: torch.bfloat16, 2: torch.float16}
TOL = {0: 2e-5, 1: 1e-2, 2: 1.5e-3}   # single kernels: one rounding step, so tighter than the whole-step bar


def draw(rng, shape, dtype, scale=1.0):
    a = (rng.standard_normal(shape) * scale).astype(np.float32)
    return round_bf16(a) if dtype == 1 else round_f16(a) if dtype == 2 else a


def st():
    return torch.cuda.current_stream().cuda_stream


def back(t):
    torch.cuda.synchronize()
    return t.float().cpu().numpy().astype(np.float64)


# ----------------------------------------------------------------------------- GEMM

GEMM_CASES = [
    # (M, N, K, transA, transB, batch, kseg, bias, resid, accum)
    (256, 256, 64, 0, 1, 1, 0, False, False, False),
    (256, 256, 128, 0, 0, 1, 0, False, False, False),
    (256, 256, 128, 1, 0, 1, 0, False, False, True),
    (256, 256, 128, 1, 1, 1, 0, False, False, False),
    (512, 768, 320, 0, 0, 1, 0, True, True, False),
    (300, 264, 200, 0, 1, 1, 0, True, False, False),      # ragged in every dimension
    (304, 264, 200, 1, 0, 2, 0, False, False, True),
    (72, 1376, 40, 0, 0, 3, 0, False, True, False),
    (130, 520, 3 * 136, 0, 1, 1, 136, False, False, False),   # segmented K, segment not a multiple of 64
    (257, 512, 1024, 0, 1, 1, 512, False, False, False),
    (8, 8, 8, 0, 0, 1, 0, False, False, False),
    (1000, 40, 2048, 1, 0, 1, 0, False, False, True),
    # K a multiple of 32, ragged in M and N
    (300, 264, 224, 0, 1, 1, 0, True, False, False),
    (304, 264, 224, 1, 0, 2, 0, False, False, True),
    (264, 1376, 96, 0, 0, 3, 0, False, True, False),
    (296, 520, 160, 1, 1, 1, 0, False, False, False),
    (130, 520, 3 * 160, 0, 1, 1, 160, False, False, False),
]


@pytest.mark.parametrize("impl", [1, 2, 3, 4])
@pytest.mark.parametrize("dtype", [0, 1, 2])
@pytest.mark.parametrize("case", GEMM_CASES, ids=lambda c: "x".join(str(int(v)) for v in c))
def test_gemm_matches_float64_matmul(gpu_device, case, dtype, impl):
    M, N, K, ta, tb, batch, kseg, use_bias, use_res, accum = case
    if impl >= 2 and dtype == 0:
        pytest.skip("the MFMA kernel is bf16 only")
    print(f"[case] gemm {case} dtype={dtype} impl={impl}", flush=True)
    rng = np.random.default_rng(hash(case) % 2**32)
    A = draw(rng, (batch, K, M) if ta else (batch, M, K), dtype)
    nseg = K // kseg if kseg else 1
    if kseg:
        B = draw(rng, (nseg, N, kseg), dtype, 0.05)             # transB=1 segments stored one after another
    else:
        B = draw(rng, (batch, N, K) if tb else (batch, K, N), dtype, 0.05)
    bias = draw(rng, (batch, N), dtype) if use_bias else None
    R = draw(rng, (batch, M, N), dtype) if use_res else None
    C0 = rng.standard_normal((batch, M, N)).astype(np.float32) if accum else None
    # oracle: plain float64 products
    want = np.empty((batch, M, N))
    for z in range(batch):
        a = A[z].astype(np.float64).T if ta else A[z].astype(np.float64)
        if kseg:
            b = np.concatenate([B[s].astype(np.float64).T for s in range(nseg)], axis=0)
        else:
            b = B[z].astype(np.float64).T if tb else B[z].astype(np.float64)
        want[z] = a @ b
        if use_bias:
            want[z] += bias[z][None, :]
        if use_res:
            want[z] += R[z]
        if accum:
            want[z] += C0[z]
    td = TD[dtype]
    dA, dB = dev(A, td), dev(B, td)
    dbias = dev(bias, td) if use_bias else None
    dR = dev(R, td) if use_res else None
    dC = dev(C0) if accum else torch.full((batch, M, N), float("nan"), dtype=td, device="cuda")
    lda = M if ta else K
    ldb = (kseg if kseg else K) if tb else N
    sB = 0 if kseg else (N * K)
    zs.ops.gemm(st(), dtype, ta, tb, M, N, K, dA, lda, dB, ldb, dC, N, int(accum), dbias, dR, N, batch,
                M * K, sB, M * N, N, kseg, N * kseg if kseg else 0, impl)
    got = back(dC)
    err = rel_err(got, want)
    tol = 2e-5 if (dtype == 0 or accum) else 1e-2
    log_report(f"gemm {case} dtype={dtype} impl={impl}", [("C", err)])
    assert err <= tol


@pytest.mark.parametrize("dtype", [1, 2])
def test_gemm_full_shape_sampled_outputs(gpu_device, dtype):
    """The three products of the 7B-class FFN down projection at full size (T=4096, H=4096, F=11008),
    checked on 256 sampled outputs each, every one recomputed as a float64 dot product."""
    rng = np.random.default_rng(11)
    T, H, F = 4096, 4096, 11008
    g = torch.Generator(device="cuda").manual_seed(5)
    a = torch.randn(T, F, device="cuda", generator=g).to(TD[dtype])
    W = (torch.randn(F, H, device="cuda", generator=g) * 0.02).to(TD[dtype])
    dy = (torch.randn(T, H, device="cuda", generator=g) * 0.01).to(TD[dtype])
    y = torch.empty(T, H, dtype=TD[dtype], device="cuda")
    da = torch.empty(T, F, dtype=TD[dtype], device="cuda")
    dW = torch.zeros(F, H, dtype=torch.float32, device="cuda")
    print("[case] gemm full shape NN", flush=True)
    zs.ops.gemm(st(), dtype, 0, 0, T, H, F, a, F, W, H, y, H, 0, None, None, 0, 1, 0, 0, 0, 0, 0, 0, 0)
    print("[case] gemm full shape NT", flush=True)
    zs.ops.gemm(st(), dtype, 0, 1, T, F, H, dy, H, W, H, da, F, 0, None, None, 0, 1, 0, 0, 0, 0, 0, 0, 0)
    print("[case] gemm full shape TN", flush=True)
    zs.ops.gemm(st(), dtype, 1, 0, F, H, T, a, F, dy, H, dW, H, 1, None, None, 0, 1, 0, 0, 0, 0, 0, 0, 0)
    torch.cuda.synchronize()
    a64, W64, dy64 = (t.float().cpu().numpy().astype(np.float64) for t in (a, W, dy))
    yh, dah, dWh = y.float().cpu().numpy(), da.float().cpu().numpy(), dW.cpu().numpy()
    ii = rng.integers(0, T, 256)
    jh, jf = rng.integers(0, H, 256), rng.integers(0, F, 256)
    want_y = np.einsum("sk,ks->s", a64[ii, :], W64[:, jh])
    want_da = np.einsum("sk,sk->s", dy64[ii, :], W64[jf, :])
    want_dW = np.einsum("ks,ks->s", a64[:, jf], dy64[:, jh])
    ey = np.abs(yh[ii, jh] - want_y).max() / np.abs(want_y).max()
    eda = np.abs(dah[ii, jf] - want_da).max() / np.abs(want_da).max()
    edw = np.abs(dWh[jf, jh] - want_dW).max() / np.abs(want_dW).max()
    log_report("gemm full shape sampled", [("y", ey), ("da", eda), ("dW", edw)])
    assert ey <= 1e-2 and eda <= 1e-2 and edw <= 1e-4


@pytest.mark.parametrize("dtype", [1, 2])
def test_gemm_whose_last_round_runs_on_small_tiles(gpu_device, dtype):
    """4096 x 11008 outputs in a batch of two are 1376 tiles of 256 x 256: five rounds on 256 CUs and 96 tiles.  The
    dispatcher runs the leading 40 tile columns on big tiles and the last 768 columns on 128 x 128 tiles.  Sampled
    outputs on both sides of the cut against float64 dot products, for the forward form (bias and residual
    added), the segmented input-gradient form and the grouped weight gradient."""
    rng = np.random.default_rng(23)
    T, H, F, K = 4096, 4096, 11008, 256
    td = TD[dtype]
    g = torch.Generator(device="cuda").manual_seed(13)
    x = torch.randn(T, K, device="cuda", generator=g).to(td)
    W = (torch.randn(2, K, F, device="cuda", generator=g) * 0.05).to(td)
    bias = torch.randn(2, F, device="cuda", generator=g).to(td)
    res = torch.randn(2, T, F, device="cuda", generator=g).to(td)
    y = torch.empty(2, T, F, dtype=td, device="cuda")
    print("[case] gemm tail split NN batch 2", flush=True)
    zs.ops.gemm(st(), dtype, 0, 0, T, F, K, x, K, W, F, y, F, 0, bias, res, F, 2, 0, K * F, T * F, F, 0, 0, 0)
    torch.cuda.synchronize()
    ii = rng.integers(0, T, 400)
    jj = np.concatenate([rng.integers(0, F, 300), rng.integers(10240 - 4, 10240 + 4, 50), rng.integers(F - 300, F, 50)])
    zz = rng.integers(0, 2, 400)
    x64, W64 = x.float().cpu().numpy().astype(np.float64), W.float().cpu().numpy().astype(np.float64)
    want = np.einsum("sk,sk->s", x64[ii], W64[zz, :, jj]) + bias.float().cpu().numpy()[zz, jj] + res.float().cpu().numpy()[zz, ii, jj]
    got = y.float().cpu().numpy()[zz, ii, jj]
    assert np.abs(got - want).max() / np.abs(want).max() <= 1e-2

    print("[case] gemm tail split TN batch 2, three parts", flush=True)
    parts = 3
    xs = [torch.randn(256, H, device="cuda", generator=g).to(td) for _ in range(parts)]
    dys = [(torch.randn(256, 2 * F, device="cuda", generator=g) * 0.05).to(td) for _ in range(parts)]
    dW = torch.zeros(2, H, F, dtype=torch.float32, device="cuda")
    zs.wgrad_parts(st(), dtype, H, F, 256, 256, xs, H, dys, 2 * F, dW, F, 2, 0, F, H * F, 0)
    torch.cuda.synchronize()
    rr = rng.integers(0, H, 400)
    X = np.concatenate([t.float().cpu().numpy() for t in xs]).astype(np.float64)
    D = np.concatenate([t.float().cpu().numpy() for t in dys]).astype(np.float64)
    want = np.einsum("ks,ks->s", X[:, rr], D[:, zz * F + jj])
    got = dW.cpu().numpy()[zz, rr, jj]
    assert np.abs(got - want).max() / np.abs(want).max() <= 2e-5


def test_gemm_with_operands_beyond_the_kernels_offset_range(gpu_device):
    """Token-sized operands of more than 2^30 bytes (26 624 tokens x 22 016 columns of bf16): the dispatcher cuts
    the product into launches of the MFMA kernel over row ranges (forward and input-gradient products, also
    with the fused rotation) or over ranges of K (weight gradient).  256 sampled outputs each against float64
    dot products, and the samples include rows and K ranges on both sides of every cut."""
    rng = np.random.default_rng(17)
    T, F2, N, S, d = 26624, 22016, 512, 2048, 128
    g = torch.Generator(device="cuda").manual_seed(9)
    big = torch.randn(T, F2, device="cuda", generator=g).to(torch.bfloat16)
    assert big.numel() * 2 > 2 ** 30
    W = (torch.randn(N, F2, device="cuda", generator=g) * 0.02).to(torch.bfloat16)       # [N, K]: two K segments of F2/2
    Wn = (torch.randn(F2, N, device="cuda", generator=g) * 0.02).to(torch.bfloat16)      # [K, N]
    x = torch.randn(T, N, device="cuda", generator=g).to(torch.bfloat16)
    res = torch.randn(T, N, device="cuda", generator=g).to(torch.bfloat16)
    big64 = None
    ii = np.concatenate([rng.integers(0, T, 250), [0, T - 1, 24319, 24320, 22527, 22528]])
    jj = rng.integers(0, N, ii.size)

    print("[case] gemm big operand NT segmented", flush=True)
    c = torch.empty(T, N, dtype=torch.bfloat16, device="cuda")
    zs.ops.gemm(st(), 1, 0, 1, T, N, F2, big, F2, W, F2, c, N, 0, None, res, N, 1, 0, 0, 0, 0, F2 // 2, F2 // 2, 0)
    torch.cuda.synchronize()
    A = big[torch.from_numpy(ii).cuda()].float().cpu().numpy().astype(np.float64)
    want = np.einsum("sk,sk->s", A, W.float().cpu().numpy().astype(np.float64)[jj]) + res.float().cpu().numpy()[ii, jj]
    got = c.float().cpu().numpy()[ii, jj]
    assert np.abs(got - want).max() / np.abs(want).max() <= 1e-2

    print("[case] gemm big operand NN with fused rotation", flush=True)
    table = torch.empty(S * d, dtype=torch.float32, device="cuda")
    zs.ops.rope_table(st(), S, d, 10000.0, table)
    c2 = torch.empty(T, N, dtype=torch.bfloat16, device="cuda")
    zs.ops.gemm_rope(st(), 1, 0, 0, T, N, F2, big, F2, Wn, N, c2, N, 0, None, None, 0, 1, 0, 0, 0, 0, 0, 0, 0, table, S, d, 1)
    torch.cuda.synchronize()
    Wn64 = Wn.float().cpu().numpy().astype(np.float64)
    pair = jj // 2 * 2
    u0 = np.einsum("sk,ks->s", A, Wn64[:, pair])
    u1 = np.einsum("sk,ks->s", A, Wn64[:, pair + 1])
    ang = (ii % S) * 10000.0 ** (-2.0 * ((pair % d) // 2) / d)
    want = np.where(jj % 2 == 0, u0 * np.cos(ang) - u1 * np.sin(ang), u0 * np.sin(ang) + u1 * np.cos(ang))
    got = c2.float().cpu().numpy()[ii, jj]
    assert np.abs(got - want).max() / np.abs(want).max() <= 1e-2

    print("[case] gemm big operand TN", flush=True)
    dW = torch.zeros(2 * N * (F2 // 2), dtype=torch.float32, device="cuda")
    zs.ops.gemm(st(), 1, 1, 0, N, F2 // 2, T, x, N, big, F2, dW, F2 // 2, 1, None, None, 0, 2, 0, F2 // 2, N * (F2 // 2), 0, 0, 0, 0)
    torch.cuda.synchronize()
    rows, cols = rng.integers(0, N, 64), rng.integers(0, F2, 64)
    x64 = x.float().cpu().numpy().astype(np.float64)
    B = big[:, torch.from_numpy(cols).cuda()].float().cpu().numpy().astype(np.float64)
    want = np.einsum("ks,ks->s", x64[:, rows], B)
    dWh = dW.cpu().numpy().reshape(2, N, F2 // 2)
    got = dWh[cols // (F2 // 2), rows, cols % (F2 // 2)]
    assert np.abs(got - want).max() / np.abs(want).max() <= 1e-4


# ----------------------------------------------------------------------------- norms


@pytest.mark.parametrize("dtype", [0, 1, 2])
@pytest.mark.parametrize("kind", [0, 1])
# (T, H, blocks of the vector-gradient partials; 0 = rows/8); H = 64 lanes x vector x {1,2,4,8,10} selects the
# register-resident kernels
@pytest.mark.parametrize("T,H,nblk", [(37, 256, 7), (130, 640, 7), (5, 8, 5), (37, 512, 0), (130, 2048, 0), (61, 1024, 0),
                                      (21, 5120, 0), (9, 4096, 0), (40, 2560, 0)])
def test_norm_fwd_bwd(gpu_device, dtype, kind, T, H, nblk):
    print(f"[case] norm kind={kind} dtype={dtype} T={T} H={H} nblk={nblk}", flush=True)
    rng = np.random.default_rng(3)
    x = draw(rng, (T, H), dtype, 2.0)
    g = draw(rng, (H,), dtype) + 1
    g = round_bf16(g) if dtype == 1 else round_f16(g) if dtype == 2 else g
    b = draw(rng, (H,), dtype)
    dn = draw(rng, (T, H), dtype)
    dres = draw(rng, (T, H), dtype)
    eps = float(np.float32(1e-5))
    if kind == 0:
        n_o, cache = so.layernorm_fwd(x.astype(np.float64), g, b, eps)
        dx_o, dg_o, db_o = so.layernorm_bwd(dn.astype(np.float64), g.astype(np.float64), cache)
    else:
        n_o, cache = so.rmsnorm_fwd(x.astype(np.float64), g, eps)
        dx_o, dg_o = so.rmsnorm_bwd(dn.astype(np.float64), g.astype(np.float64), cache)
    td = TD[dtype]
    dxd, dg_, db_, dnd, dresd = dev(x, td), dev(g, td), dev(b, td), dev(dn, td), dev(dres, td)
    n = torch.empty(T, H, dtype=td, device="cuda")
    rstd = torch.empty(T, device="cuda")
    mean = torch.empty(T, device="cuda")
    zs.ops.norm_fwd(st(), dtype, kind, T, H, dxd, dg_, db_ if kind == 0 else None, eps, n, rstd, mean if kind == 0 else None)
    assert rel_err(back(n), n_o) <= TOL[dtype]
    assert rel_err(back(rstd), cache[1][:, 0]) <= 2e-6
    nblk = nblk or (T + 7) // 8
    dx = torch.empty(T, H, dtype=td, device="cuda")
    pg = torch.empty(nblk, H, device="cuda")
    pb = torch.empty(nblk, H, device="cuda")
    zs.ops.norm_bwd(st(), dtype, kind, T, H, dnd, dxd, dg_, rstd, mean if kind == 0 else None, dresd, dx, pg,
                    pb if kind == 0 else None, nblk)
    assert rel_err(back(dx), dx_o + dres) <= TOL[dtype]
    assert rel_err(back(pg).sum(axis=0), dg_o) <= 2e-5
    if kind == 0:
        assert rel_err(back(pb).sum(axis=0), db_o) <= 2e-5
    # every row block on its own: block k holds the rows [k*rpb, (k+1)*rpb) and nothing else
    rpb = -(-T // nblk)
    prod = dn.astype(np.float64) * cache[0]
    scale = max(np.abs(dg_o).max(), 1e-30)
    for k in range(nblk):
        rows = slice(k * rpb, min(T, (k + 1) * rpb))
        assert np.abs(back(pg)[k] - prod[rows].sum(axis=0)).max() <= 2e-5 * scale
        if kind == 0:
            assert np.abs(back(pb)[k] - dn[rows].astype(np.float64).sum(axis=0)).max() <= 2e-5 * max(np.abs(db_o).max(), 1e-30)


# ----------------------------------------------------------------------------- RoPE, activations


@pytest.mark.parametrize("dtype", [0, 1, 2])
def test_rope_and_inverse(gpu_device, dtype):
    print(f"[case] rope dtype={dtype}", flush=True)
    rng = np.random.default_rng(4)
    mb, S, nh, d = 2, 300, 3, 128
    u = draw(rng, (mb * S, 3 * nh * d), dtype)
    want = u.astype(np.float64).copy()
    qk = so.rope(want[:, :2 * nh * d].reshape(mb, S, 2 * nh, d), 10000.0)
    want[:, :2 * nh * d] = qk.reshape(mb * S, -1)
    a = dev(u, TD[dtype])
    table = torch.empty(S * d, device="cuda")
    zs.ops.rope(st(), dtype, mb * S, S, 2 * nh * d, d, a, 3 * nh * d, 10000.0, 1.0, table)
    assert rel_err(back(a), want) <= (4e-3 if dtype else 2e-6)
    assert np.array_equal(back(a)[:, 2 * nh * d:], u[:, 2 * nh * d:].astype(np.float64))       # V untouched
    if dtype == 0:
        zs.ops.rope(st(), dtype, mb * S, S, 2 * nh * d, d, a, 3 * nh * d, 10000.0, -1.0, table)
        assert rel_err(back(a), u) <= 2e-6


@pytest.mark.parametrize("dtype", [0, 1, 2])
def test_gelu_and_swiglu(gpu_device, dtype):
    print(f"[case] activations dtype={dtype}", flush=True)
    rng = np.random.default_rng(5)
    T, F = 33, 1376
    td = TD[dtype]
    z = draw(rng, (T, F), dtype, 2.0)
    da = draw(rng, (T, F), dtype)
    out = torch.empty(T, F, dtype=td, device="cuda")
    zs.ops.gelu(st(), dtype, T * F, dev(z, td), None, out, 0)
    assert rel_err(back(out), so.gelu(z.astype(np.float64))) <= TOL[dtype]
    zs.ops.gelu(st(), dtype, T * F, dev(z, td), dev(da, td), out, 1)
    assert rel_err(back(out), da * so.gelu_grad(z.astype(np.float64))) <= TOL[dtype]
    gu = draw(rng, (T, 2 * F), dtype, 2.0)
    g64, u64 = gu[:, :F].astype(np.float64), gu[:, F:].astype(np.float64)
    zs.ops.swiglu(st(), dtype, T, F, dev(gu, td), None, out, 0)
    assert rel_err(back(out), g64 * so.sigmoid(g64) * u64) <= TOL[dtype]
    dgu = torch.empty(T, 2 * F, dtype=td, device="cuda")
    zs.ops.swiglu(st(), dtype, T, F, dev(gu, td), dev(da, td), dgu, 1)
    sg = so.sigmoid(g64)
    want = np.concatenate([da * u64 * sg * (1 + g64 * (1 - sg)), da * g64 * sg], axis=1)
    assert rel_err(back(dgu), want) <= TOL[dtype]


GLU_CASES = [(264, 136, 72), (512, 384, 128), (300, 1376, 200), (64, 8, 8), (2048, 8704, 64)]   # (M, N, K); the last: whole rounds of big tiles + a tail of small ones


@pytest.mark.parametrize("impl", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("dtype", [0, 1, 2])
@pytest.mark.parametrize("case", GLU_CASES, ids=lambda c: "x".join(str(v) for v in c))
def test_gemm_with_fused_gated_unit(gpu_device, dtype, impl, case):
    """Gate and up projections with the gated unit in the store, and the down projection's input gradient turned into
    (dgate, dup) in the store, against the fp64 formulas of the Llama-style FFN; the forward must also leave exactly
    the bits of the batched product followed by the activation kernel."""
    M, N, K = case
    print(f"[case] gemm_glu dtype={dtype} impl={impl} M={M} N={N} K={K}", flush=True)
    if dtype == 0 and impl >= 2:
        pytest.skip("the MFMA kernel is 16-bit")
    rng = np.random.default_rng(97)
    td = TD[dtype]
    x = draw(rng, (M, K), dtype)
    W = draw(rng, (2, K, N), dtype, K ** -0.5 * 2.0)          # pre-activations of order 2: the sigmoid is far from linear
    x_d, W_d = dev(x, td), dev(W, td)
    a = torch.full((M, N), 7.0, dtype=td, device="cuda")
    gu = torch.full((M, 2 * N), 7.0, dtype=td, device="cuda")
    zs.ops.gemm_glu(st(), dtype, 1, M, N, K, x_d, K, W_d, N, K * N, a, gu, impl)
    g64, u64 = x.astype(np.float64) @ W[0].astype(np.float64), x.astype(np.float64) @ W[1].astype(np.float64)
    assert rel_err(back(gu)[:, :N], g64) <= TOL[dtype] and rel_err(back(gu)[:, N:], u64) <= TOL[dtype]
    assert rel_err(back(a), g64 * so.sigmoid(g64) * u64) <= 2 * TOL[dtype]
    # the unfused route: batched product into [gate | up], then the activation kernel
    gu2 = torch.empty_like(gu)
    a2 = torch.empty_like(a)
    zs.ops.gemm(st(), dtype, 0, 0, M, N, K, x_d, K, W_d, N, gu2, 2 * N, 0, None, None, 0, 2, 0, K * N, N, 0, 0, 0, min(impl, 2))
    zs.ops.swiglu(st(), dtype, M, N, gu2, None, a2, 0)
    torch.cuda.synchronize()
    if dtype != 0:
        assert torch.equal(gu.view(torch.int16), gu2.view(torch.int16)) and torch.equal(a.view(torch.int16), a2.view(torch.int16))
    else:
        assert torch.equal(gu, gu2) and torch.equal(a, a2)

    # backward: dy [M, K2] through Wd stored [N, K2]
    K2 = K
    dy = draw(rng, (M, K2), dtype)
    Wd = draw(rng, (N, K2), dtype, K2 ** -0.5)
    gu0 = back(gu)                                              # the saved (rounded) pre-activations
    scratch = torch.empty(M, N, dtype=td, device="cuda")
    zs.ops.gemm_glu(st(), dtype, 2, M, N, K2, dev(dy, td), K2, dev(Wd, td), K2, 0, scratch, gu, impl)
    da = dy.astype(np.float64) @ Wd.astype(np.float64).T
    gt, up = gu0[:, :N], gu0[:, N:]
    sg = so.sigmoid(gt)
    want = np.concatenate([da * up * sg * (1.0 + gt * (1.0 - sg)), da * gt * sg], axis=1)
    assert rel_err(back(gu), want) <= 2 * TOL[dtype]


# ----------------------------------------------------------------------------- attention

ATTN_CASES = [(2, 128, 4, 64), (1, 256, 4, 128), (2, 200, 3, 128), (1, 1, 2, 128), (1, 65, 1, 128), (1, 576, 2, 128)]


@pytest.mark.parametrize("impl", [1, 2])
@pytest.mark.parametrize("dtype", [0, 1, 2])
@pytest.mark.parametrize("mb,S,nh,d", ATTN_CASES)
def test_attention_fwd_bwd(gpu_device, mb, S, nh, d, dtype, impl):
    if impl == 2 and (dtype == 0 or d != 128):
        pytest.skip("the MFMA attention kernel is bf16, head dim 128")
    print(f"[case] attention mb={mb} S={S} nh={nh} d={d} dtype={dtype} impl={impl}", flush=True)
    rng = np.random.default_rng(6)
    H = nh * d
    qkv = draw(rng, (mb * S, 3 * H), dtype)
    do = draw(rng, (mb * S, H), dtype)
    q, k, v = (qkv[:, i * H:(i + 1) * H].astype(np.float64).reshape(mb, S, nh, d) for i in range(3))
    o_o = so.attention_fwd(q, k, v)
    td = TD[dtype]
    dqkv_in = dev(qkv, td)
    o = torch.empty(mb * S, H, dtype=td, device="cuda")
    lse = torch.empty(mb * nh * S, device="cuda")
    E = dqkv_in.element_size()
    qp, kp, vp = (torch.as_strided(dqkv_in, (mb * S, H), (3 * H, 1), i * H) for i in range(3))
    zs.ops.attention_fwd(st(), dtype, mb, S, nh, d, qp, kp, vp, 3 * H, o, H, lse, impl)
    tol = 1e-2 if dtype else 2e-5
    assert rel_err(back(o), o_o.reshape(mb * S, H)) <= tol
    # lse against the definition
    b, h = mb - 1, nh - 1
    s = (q[b, :, h] @ k[b, :, h].T) / np.sqrt(d)
    s = np.where(np.tril(np.ones((S, S), bool)), s, -np.inf)
    mx = s.max(axis=1)
    lse_o = mx + np.log(np.exp(s - mx[:, None]).sum(axis=1))
    assert np.abs(back(lse).reshape(mb, nh, S)[b, h] - lse_o).max() <= (2e-2 if dtype else 1e-5)
    # backward, fed with the oracle's o rounded like the forward output would be
    dq_o, dk_o, dv_o = so.attention_bwd(do.astype(np.float64).reshape(mb, S, nh, d), q, k, v)
    delta = torch.empty(mb * nh * S, device="cuda")
    dqkv = torch.full((mb * S, 3 * H), float("nan"), dtype=td, device="cuda")
    dq_, dk_, dv_ = (torch.as_strided(dqkv, (mb * S, H), (3 * H, 1), i * H) for i in range(3))
    zs.ops.attention_bwd(st(), dtype, mb, S, nh, d, qp, kp, vp, 3 * H, o, dev(do, td), H, lse, delta, dq_, dk_, dv_,
                         3 * H, impl)
    got = back(dqkv)
    errs = [("dq", rel_err(got[:, :H], dq_o.reshape(mb * S, H))), ("dk", rel_err(got[:, H:2 * H], dk_o.reshape(mb * S, H))),
            ("dv", rel_err(got[:, 2 * H:], dv_o.reshape(mb * S, H)))]
    log_report(f"attention mb={mb} S={S} nh={nh} d={d} dtype={dtype} impl={impl}", errs)
    for n, e in errs:
        assert e <= (2e-2 if dtype else 5e-5), n


@pytest.mark.parametrize("impl", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("dtype", [0, 1, 2])
@pytest.mark.parametrize("shape", [(296, 520, 128, 72, 2), (256, 256, 64, 64, 1), (1000, 40, 1024, 200, 1), (304, 264, 100, 64, 1)])
def test_weight_gradient_of_two_microbatches(gpu_device, dtype, impl, shape):
    """C += A1^T B1 + A2^T B2 in one product over both parts' rows, against float64."""
    M, N, K1, K2, batch = shape
    if impl >= 2 and (dtype == 0 or K1 % 128):
        pytest.skip("the MFMA kernel is 16-bit only and needs the first part to be a multiple of 128 rows")
    print(f"[case] wgrad pair {shape} dtype={dtype} impl={impl}", flush=True)
    rng = np.random.default_rng(41)
    td = TD[dtype]
    A1, A2 = draw(rng, (K1, M), dtype), draw(rng, (K2, M), dtype)
    B1, B2 = draw(rng, (K1, N * batch), dtype, 0.05), draw(rng, (K2, N * batch), dtype, 0.05)
    C0 = rng.standard_normal((batch, M, N)).astype(np.float32)
    want = np.stack([C0[z] + A1.astype(np.float64).T @ B1[:, z * N:(z + 1) * N].astype(np.float64)
                     + A2.astype(np.float64).T @ B2[:, z * N:(z + 1) * N].astype(np.float64) for z in range(batch)])
    C = dev(C0)
    zs.ops.wgrad_pair(st(), dtype, M, N, K1, K2, dev(A1, td), dev(A2, td), M, dev(B1, td), dev(B2, td), N * batch, C, N, batch,
                      0, N, M * N, impl)
    err = rel_err(back(C), want)
    log_report(f"wgrad pair {shape} dtype={dtype} impl={impl}", [("C", err)])
    assert err <= 2e-5


@pytest.mark.parametrize("impl", [0, 1, 3, 4])
@pytest.mark.parametrize("dtype", [1, 2])
@pytest.mark.parametrize("shape", [(200, 136, 128, 128, 3, 1), (384, 520, 128, 40, 5, 2), (72, 264, 256, 256, 16, 1),
                                   (256, 256, 128, 200, 2, 1), (136, 64, 320, 320, 1, 1), (264, 136, 384, 520, 4, 1),
                                   (128, 128, 64, 64, 3, 1)])
def test_weight_gradient_of_several_microbatches(gpu_device, dtype, impl, shape):
    """C += sum_p A_p^T B_p over up to 16 parts in one K loop (the last part may have its own length, also one
    that is longer than the others or no multiple of the slab), against float64."""
    M, N, K_each, K_last, nparts, batch = shape
    if impl >= 3 and nparts > 1 and K_each % 128:
        pytest.skip("the MFMA kernel needs parts of a multiple of 128 rows")
    print(f"[case] wgrad parts {shape} dtype={dtype} impl={impl}", flush=True)
    rng = np.random.default_rng(43)
    td = TD[dtype]
    rows = [K_each] * (nparts - 1) + [K_last]
    A = [draw(rng, (k, M), dtype) for k in rows]
    B = [draw(rng, (k, N * batch), dtype, 0.05) for k in rows]
    C0 = rng.standard_normal((batch, M, N)).astype(np.float32)
    want = np.stack([C0[z] + sum(a.astype(np.float64).T @ b[:, z * N:(z + 1) * N].astype(np.float64) for a, b in zip(A, B))
                     for z in range(batch)])
    C = dev(C0)
    zs.wgrad_parts(st(), dtype, M, N, K_each, K_last, [dev(a, td) for a in A], M, [dev(b, td) for b in B], N * batch, C, N,
                   batch, 0, N, M * N, impl)
    err = rel_err(back(C), want)
    log_report(f"wgrad parts {shape} dtype={dtype} impl={impl}", [("C", err)])
    assert err <= 2e-5


# (M, N, K_each, K_last, parts, batch): grids of 256x256 tiles that fill one round of 256 workgroups and leave 16 tiles (one
# tile row: first two cases, ragged in the second), 96 (three tile columns of two batches: third case) or 14 (no whole row
# or column, ragged both ways; in the last case the 14 tiles lie in the second batch).
@pytest.mark.parametrize("dtype", [1, 2])
@pytest.mark.parametrize("shape", [(4352, 4096, 128, 128, 4, 1), (4344, 4088, 256, 72, 5, 1), (4096, 2808, 1536, 1000, 8, 2),
                                   (4600, 3832, 128, 128, 4, 1), (2304, 3832, 256, 200, 5, 2)])
def test_weight_gradient_with_the_last_round_cut_along_k(gpu_device, dtype, shape):
    """stage_op_wgrad_parts_cut: the tiles beyond whole rounds of workgroups have their K range cut into chunks whose partial
    tiles a second kernel adds to C.  Against float64 on whole rows and columns that cross both regions; two calls give the
    same bits; and the scratch buffer is checked."""
    M, N, K_each, K_last, nparts, batch = shape
    print(f"[case] wgrad parts cut {shape} dtype={dtype}", flush=True)
    need = zs.wgrad_parts_scratch_bytes(M, N, K_each, K_last, nparts, batch)
    assert need > 0 and need % (256 * 256 * 4) == 0, "these shapes are meant to be cut"
    rng = np.random.default_rng(47)
    td = TD[dtype]
    rows = [K_each] * (nparts - 1) + [K_last]
    A = [draw(rng, (k, M), dtype) for k in rows]
    B = [draw(rng, (k, N * batch), dtype, 0.05) for k in rows]
    C0 = rng.standard_normal((batch, M, N)).astype(np.float32)
    Ad, Bd = [dev(a, td) for a in A], [dev(b, td) for b in B]
    scratch = torch.full((need // 4,), float("nan"), device="cuda")           # stale content must not matter
    outs = []
    for rep in range(2):
        C = dev(C0)
        zs.wgrad_parts_cut(st(), dtype, M, N, K_each, K_last, Ad, M, Bd, N * batch, C, N, batch, 0, N, M * N, scratch, need)
        torch.cuda.synchronize()
        outs.append(back(C))
    assert np.array_equal(outs[0], outs[1]), "a repeat must give the same bits"
    A64 = np.concatenate([a.astype(np.float64) for a in A])                    # [K, M]
    B64 = np.concatenate([b.astype(np.float64) for b in B])                    # [K, N * batch]
    pick_m = np.unique(np.concatenate([rng.integers(0, M, 24), [0, 255, 256, M - 257, M - 256, M - 1]]))
    pick_n = np.unique(np.concatenate([rng.integers(0, N, 24), [0, 255, 256, N - 257, N - 256, N - 1]]))
    worst = 0.0
    for z in range(batch):
        Bz = B64[:, z * N:(z + 1) * N]
        want_rows = C0[z][pick_m] + A64[:, pick_m].T @ Bz                      # whole rows
        want_cols = C0[z][:, pick_n] + A64.T @ Bz[:, pick_n]                   # whole columns
        scale = max(np.abs(want_rows).max(), np.abs(want_cols).max())
        worst = max(worst, np.abs(outs[0][z][pick_m] - want_rows).max() / scale, np.abs(outs[0][z][:, pick_n] - want_cols).max() / scale)
    log_report(f"wgrad parts cut {shape} dtype={dtype}", [("C", worst)])
    assert worst <= 2e-5
    # the uncut product on the same kernel: same sums up to rounding order
    C = dev(C0)
    zs.wgrad_parts(st(), dtype, M, N, K_each, K_last, Ad, M, Bd, N * batch, C, N, batch, 0, N, M * N, 3)
    assert rel_err(back(C), outs[0]) <= 2e-6
    with pytest.raises(zs.StageError) as ei:
        zs.wgrad_parts_cut(st(), dtype, M, N, K_each, K_last, Ad, M, Bd, N * batch, C, N, batch, 0, N, M * N, scratch, need - 1)
    assert ei.value.code == zs.STAGE_ERR_WORKSPACE


@pytest.mark.parametrize("impl", [1, 2, 3, 4])
@pytest.mark.parametrize("dtype", [0, 1, 2])
def test_gemm_with_fused_rotation(gpu_device, dtype, impl):
    """Q|K|V projection as a batch of three products whose first two results are rotated in the store:
    against float64 matmul followed by the oracle's rotation; V must be the plain product."""
    if impl >= 2 and dtype == 0:
        pytest.skip("the MFMA kernel is bf16 only")
    print(f"[case] gemm+rope dtype={dtype} impl={impl}", flush=True)
    rng = np.random.default_rng(31)
    mb, S, nh, d, K = 2, 150, 3, 128, 96          # 300 rows (ragged tile), 384 columns
    T, H = mb * S, nh * d
    td = TD[dtype]
    A = draw(rng, (T, K), dtype)
    B = draw(rng, (3, K, H), dtype, 0.1)
    R = draw(rng, (3, T, H), dtype)
    want = np.stack([A.astype(np.float64) @ B[z].astype(np.float64) + R[z] for z in range(3)])
    for z in range(2):
        want[z] = so.rope(want[z].reshape(mb, S, nh, d), 10000.0).reshape(T, H)
    table = torch.empty(S * d, device="cuda")
    zs.ops.rope_table(st(), S, d, 10000.0, table)
    C = torch.full((3, T, H), float("nan"), dtype=td, device="cuda")
    zs.ops.gemm_rope(st(), dtype, 0, 0, T, H, K, dev(A, td), K, dev(B, td), H, C, H, 0, None, dev(R, td), H, 3, 0, K * H,
                     T * H, 0, 0, 0, impl, table, S, d, 2)
    got = back(C)
    errs = [(f"z{z}", rel_err(got[z], want[z])) for z in range(3)]
    log_report(f"gemm+rope dtype={dtype} impl={impl}", errs)
    for n, e in errs:
        assert e <= (1e-2 if dtype else 2e-5), n


@pytest.mark.parametrize("impl", [1, 2])
@pytest.mark.parametrize("dtype", [0, 1, 2])
def test_attention_bwd_with_fused_inverse_rotation(gpu_device, dtype, impl):
    """dq and dk leave the backward kernels rotated back: against the oracle's gradients, rotated by
    the oracle with sign -1; dv is unchanged."""
    if impl == 2 and dtype == 0:
        pytest.skip("the MFMA attention kernel is bf16")
    print(f"[case] attention bwd + inverse rope dtype={dtype} impl={impl}", flush=True)
    rng = np.random.default_rng(32)
    mb, S, nh, d = 2, 200, 2, 128
    H = nh * d
    td = TD[dtype]
    qkv = draw(rng, (mb * S, 3 * H), dtype)
    do = draw(rng, (mb * S, H), dtype)
    q, k, v = (qkv[:, i * H:(i + 1) * H].astype(np.float64).reshape(mb, S, nh, d) for i in range(3))
    dq_o, dk_o, dv_o = so.attention_bwd(do.astype(np.float64).reshape(mb, S, nh, d), q, k, v)
    dq_o, dk_o = so.rope(dq_o, 10000.0, sign=-1.0), so.rope(dk_o, 10000.0, sign=-1.0)
    dqkv_in = dev(qkv, td)
    qp, kp, vp = (torch.as_strided(dqkv_in, (mb * S, H), (3 * H, 1), i * H) for i in range(3))
    o = torch.empty(mb * S, H, dtype=td, device="cuda")
    lse = torch.empty(mb * nh * S, device="cuda")
    zs.ops.attention_fwd(st(), dtype, mb, S, nh, d, qp, kp, vp, 3 * H, o, H, lse, impl)
    table = torch.empty(S * d, device="cuda")
    zs.ops.rope_table(st(), S, d, 10000.0, table)
    delta = torch.empty(mb * nh * S, device="cuda")
    dqkv = torch.full((mb * S, 3 * H), float("nan"), dtype=td, device="cuda")
    dq_, dk_, dv_ = (torch.as_strided(dqkv, (mb * S, H), (3 * H, 1), i * H) for i in range(3))
    zs.ops.attention_bwd_rope(st(), dtype, mb, S, nh, d, qp, kp, vp, 3 * H, o, dev(do, td), H, lse, delta, dq_, dk_, dv_,
                              3 * H, impl, table)
    got = back(dqkv)
    errs = [("dq", rel_err(got[:, :H], dq_o.reshape(mb * S, H))), ("dk", rel_err(got[:, H:2 * H], dk_o.reshape(mb * S, H))),
            ("dv", rel_err(got[:, 2 * H:], dv_o.reshape(mb * S, H)))]
    log_report(f"attention bwd + inverse rope dtype={dtype} impl={impl}", errs)
    for n, e in errs:
        assert e <= (2e-2 if dtype else 5e-5), n


# ----------------------------------------------------------------------------- embedding, cross entropy, AdamW


@pytest.mark.parametrize("dtype", [0, 1, 2])
def test_embedding_is_bit_exact_and_scatter_matches(gpu_device, dtype):
    print(f"[case] embedding dtype={dtype}", flush=True)
    rng = np.random.default_rng(7)
    T, H, V = 700, 64, 50                       # many repeated ids
    td = TD[dtype]
    E = draw(rng, (V, H), dtype)
    ids = rng.integers(0, V, T).astype(np.int32)
    dx = draw(rng, (T, H), dtype)
    x = torch.empty(T, H, dtype=td, device="cuda")
    dE = dev(rng.standard_normal((V, H)).astype(np.float32))
    dE0 = back(dE).copy()
    zs.ops.embed(st(), dtype, T, H, V, dev(ids), dev(E, td), x, None, None, 0)
    assert np.array_equal(back(x), E[ids].astype(np.float64))           # integer indexing: bit exact
    zs.ops.embed(st(), dtype, T, H, V, dev(ids), None, None, dev(dx, td), dE, 1)
    want = dE0.copy()
    np.add.at(want, ids, dx.astype(np.float64))
    assert rel_err(back(dE), want) <= 2e-6


@pytest.mark.parametrize("dtype", [0, 1, 2])
@pytest.mark.parametrize("V", [2000, 1001])     # whole 16-byte vectors per row, and a width that needs the element-wise kernels
def test_cross_entropy(gpu_device, dtype, V):
    print(f"[case] cross entropy dtype={dtype} V={V}", flush=True)
    rng = np.random.default_rng(8)
    T = 97
    td = TD[dtype]
    z = draw(rng, (T, V), dtype, 3.0)
    tg = rng.integers(0, V, T).astype(np.int32)
    z64 = z.astype(np.float64)
    mx = z64.max(axis=1, keepdims=True)
    lse_o = (mx + np.log(np.exp(z64 - mx).sum(axis=1, keepdims=True)))[:, 0]
    loss_o = (lse_o - z64[np.arange(T), tg]).mean()
    zd = dev(z, td)
    lse, rowloss, loss = torch.empty(T, device="cuda"), torch.empty(T, device="cuda"), torch.empty(1, device="cuda")
    zs.ops.cross_entropy(st(), dtype, T, V, zd, V, dev(tg), lse, rowloss, loss, 0.0, 0)
    assert np.abs(back(lse) - lse_o).max() <= 1e-5 * np.abs(lse_o).max()
    assert abs(back(loss)[0] - loss_o) <= 1e-5 * abs(loss_o)
    scale = 0.25 / T
    zs.ops.cross_entropy(st(), dtype, T, V, zd, V, dev(tg), lse, None, None, scale, 1)
    want = np.exp(z64 - lse_o[:, None])
    want[np.arange(T), tg] -= 1
    assert rel_err(back(zd), want * scale) <= (4e-3 if dtype else 1e-5)


def test_cross_entropy_rows_without_a_valid_target(gpu_device):
    """The boundary's rule for indices it cannot check on the host: a target outside [0, V) makes its row an ignored
    one, 0 in the loss sum (the mean still divides by T) and an exactly zero gradient row, so that loss and gradient
    agree; the other rows are those of the definition."""
    print("[case] cross entropy with out-of-range targets", flush=True)
    rng = np.random.default_rng(18)
    T, V = 33, 700
    z = draw(rng, (T, V), 0, 3.0)
    tg = rng.integers(0, V, T).astype(np.int32)
    bad = np.array([0, 7, 32])
    tg[bad] = [-1, V, 2**31 - 1]
    ok = np.setdiff1d(np.arange(T), bad)
    z64 = z.astype(np.float64)
    mx = z64.max(axis=1, keepdims=True)
    lse_o = (mx + np.log(np.exp(z64 - mx).sum(axis=1, keepdims=True)))[:, 0]
    loss_o = (lse_o[ok] - z64[ok, tg[ok]]).sum() / T
    zd = dev(z)
    lse, rowloss, loss = torch.empty(T, device="cuda"), torch.empty(T, device="cuda"), torch.empty(1, device="cuda")
    zs.ops.cross_entropy(st(), 0, T, V, zd, V, dev(tg), lse, rowloss, loss, 0.0, 0)
    assert np.all(back(rowloss)[bad] == 0.0)
    assert abs(back(loss)[0] - loss_o) <= 1e-5 * abs(loss_o)
    zs.ops.cross_entropy(st(), 0, T, V, zd, V, dev(tg), lse, None, None, 1.0 / T, 1)
    got = back(zd)
    assert np.all(got[bad] == 0.0)
    want = np.exp(z64 - lse_o[:, None])
    want[ok, tg[ok]] -= 1
    assert rel_err(got[ok], want[ok] / T) <= 1e-5


@pytest.mark.parametrize("dtype", [0, 1, 2])
@pytest.mark.parametrize("n,begin", [(1 << 16, 0), (100003, 8), (1001, 5), (3, 0), (0, 0)])
def test_adamw_kernel_matches_oracle_for_t_1_2_10(gpu_device, dtype, n, begin):
    print(f"[case] adamw dtype={dtype} n={n} begin={begin}", flush=True)
    rng = np.random.default_rng(9)
    f32 = lambda x: float(np.float32(x))
    lr, b1, b2, eps, wd, gs = f32(1e-4), f32(0.9), f32(0.999), f32(1e-8), f32(0.01), f32(0.5)
    P = begin + n + 13
    p0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    master = dev(p0[begin:begin + n]) if dtype else None
    rnd = round_bf16 if dtype == 1 else round_f16
    params = dev(rnd(p0), TD[dtype]) if dtype else dev(p0)
    m = torch.zeros(max(n, 1), device="cuda")
    v = torch.zeros(max(n, 1), device="cuda")
    po, mo, vo = p0[begin:begin + n].astype(np.float64), np.zeros(n), np.zeros(n)
    for t in (1, 2, 10):
        g = (rng.standard_normal(P) * 10.0 ** rng.integers(-6, 0, P)).astype(np.float32)
        grad = dev(g)
        zs.ops.adamw(st(), dtype, n, begin, params, master, grad, m, v, lr, b1, b2, eps, wd, t, gs)
        prev = po
        po, mo, vo = so.adamw(po, g[begin:begin + n].astype(np.float64), mo, vo, t, lr, b1, b2, eps, wd, gs)
        if n == 0:
            continue
        got_p = back(master) if dtype else back(params)[begin:begin + n]
        assert rel_err(back(m)[:n], mo) <= 1e-6 and rel_err(back(v)[:n], vo) <= 1e-6
        floor = 0.5 * np.spacing(np.abs(po).astype(np.float32)).astype(np.float64) * 1.01
        d = np.maximum(np.abs((got_p - prev) - (po - prev)) - floor, 0)
        assert d.max() <= 2e-6 * np.abs(po - prev).max()
        gz = back(grad)
        assert not gz[begin:begin + n].any() and np.array_equal(gz[:begin], g[:begin].astype(np.float64))
        assert np.array_equal(gz[begin + n:], g[begin + n:].astype(np.float64))
        if dtype:
            want = master.to(TD[dtype]).cpu()
            assert torch.equal(want.view(torch.int16), params[begin:begin + n].cpu().view(torch.int16))
            assert np.array_equal(back(params)[:begin], rnd(p0)[:begin].astype(np.float64))
        po = got_p.copy()      # continue from the GPU's fp32 state so that only one step's rounding is compared
        mo, vo = back(m)[:n].copy(), back(v)[:n].copy()


def test_cross_entropy_backward_beyond_65535_tokens(gpu_device):
    """More tokens than a grid's y and z dimensions can count (65535): the rows ride on grid.x.  Sampled rows against the
    definition, first and last row included."""
    print("[case] cross entropy backward T=70001", flush=True)
    rng = np.random.default_rng(28)
    T, V = 70001, 24
    z = draw(rng, (T, V), 0, 2.0)
    tg = rng.integers(0, V, T).astype(np.int32)
    zd = dev(z)
    lse, rowloss, loss = torch.empty(T, device="cuda"), torch.empty(T, device="cuda"), torch.empty(1, device="cuda")
    zs.ops.cross_entropy(st(), 0, T, V, zd, V, dev(tg), lse, rowloss, loss, 0.0, 0)
    zs.ops.cross_entropy(st(), 0, T, V, zd, V, dev(tg), lse, None, None, 1.0, 1)
    got = back(zd)
    rows = np.concatenate([[0, 65534, 65535, 65536, T - 1], rng.integers(0, T, 200)])
    z64 = z[rows].astype(np.float64)
    p = np.exp(z64 - z64.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    p[np.arange(len(rows)), tg[rows]] -= 1
    assert rel_err(got[rows], p) <= 1e-5
    z_all = z.astype(np.float64)
    lse_o = np.log(np.exp(z_all).sum(axis=1))
    assert abs(back(loss)[0] - (lse_o - z_all[np.arange(T), tg]).mean()) <= 1e-5


@pytest.mark.gpu
def test_mfma_rate_loop_matches_the_product_it_repeats(gpu_device):
    """stage_op_mfma_rate is a measurement aid, but its loop is a real product: every thread's sum over its accumulators
    must equal iters times what one pass of the wave tile gives on the operand fragments the kernel reads (fp32
    accumulation of exact bf16 products, so a float64 reference applies)."""
    import torch
    st = torch.cuda.current_stream().cuda_stream
    torch.manual_seed(5)
    operands = (torch.randint(-4, 5, (32768,), device=gpu_device).float() / 4).to(torch.bfloat16)   # exact in fp32 sums
    sink = torch.empty(256 * 512, device=gpu_device, dtype=torch.float32)
    frags = operands.double().view(4096, 8).cpu()
    lane = torch.arange(64)
    for shape, iters in ((16, 3), (32, 3)):
        zs.ops.mfma_rate(st, shape, iters, operands, sink)
        torch.cuda.synchronize()
        got = sink.view(256, 8, 64).double().cpu()
        assert torch.equal(got[0], got[255])                      # every workgroup does the same work
        for wave in (0, 5):
            t = wave * 64 + lane
            idx = lambda o: (t * 16 + o) % 4096                   # fragment index of thread t at offset o
            if shape == 16:
                # acc[i][j] = b_j (16 x 32, rows = lanes%16) times a_i^T per 16x16x32 instruction: D[r][c] = sum_k B[r][k] A[c][k]
                A = [frags[idx(i)] for i in range(8)]             # [64 lanes, 8] each: lane l holds row l%16, k = 8*(l/16)..+7
                B = [frags[idx(8 + j)] for j in range(4)]
                def full(fr):                                      # [16 rows, 32 k]
                    m = torch.zeros(16, 32, dtype=torch.float64)
                    for l in range(64):
                        m[l % 16, 8 * (l // 16):8 * (l // 16) + 8] = fr[l]
                    return m
                total = torch.zeros(64, dtype=torch.float64)
                for i in range(8):
                    for j in range(4):
                        D = full(B[j]) @ full(A[i]).T             # lane l holds D[4*(l/16) + r][l%16], r = 0..3
                        for l in range(64):
                            total[l] += D[4 * (l // 16):4 * (l // 16) + 4, l % 16].sum()
            else:
                A = [[frags[idx(s * 4 + i)] for i in range(4)] for s in range(2)]
                B = [[frags[idx(8 + s * 2 + j)] for j in range(2)] for s in range(2)]
                def full(fr):                                      # [32 rows, 16 k]: lane l holds row l%32, k = 8*(l/32)..+7
                    m = torch.zeros(32, 16, dtype=torch.float64)
                    for l in range(64):
                        m[l % 32, 8 * (l // 32):8 * (l // 32) + 8] = fr[l]
                    return m
                total = torch.zeros(64, dtype=torch.float64)
                for s in range(2):
                    for i in range(4):
                        for j in range(2):
                            D = full(B[s][j]) @ full(A[s][i]).T    # lane l holds rows 8*(r/4) + 4*(l/32) + r%4 of column l%32
                            for l in range(64):
                                rows = [8 * (r // 4) + 4 * (l // 32) + r % 4 for r in range(16)]
                                total[l] += D[rows, l % 32].sum()
            assert torch.allclose(got[0, wave], iters * total, rtol=0, atol=1e-3), (shape, wave)


@pytest.mark.gpu
def test_lds_probe_tells_a_conflict_from_none(gpu_device):
    """stage_op_lds_probe: 64 lanes on 64 different 16-byte pieces of one 1 KB line cost the pattern-free minimum; 16 rows
    that all start in the same bank (256 bytes apart) cost several times as much."""
    import ctypes
    import torch
    st = torch.cuda.current_stream().cuda_stream
    cyc = torch.zeros(2, dtype=torch.int64, device=gpu_device)
    def cost(f, kind=0):
        host = (ctypes.c_int32 * 64)(*[f(l) for l in range(64)])
        devoff = torch.tensor(list(host), dtype=torch.int32, device=gpu_device)
        for _ in range(2):
            zs.ops.lds_probe(st, kind, host, devoff, 2000, cyc)
        torch.cuda.synchronize()
        return int(cyc[0].item()) / (2000 * 8 * 8)
    free = cost(lambda l: 16 * l)
    clash = cost(lambda l: (l % 16) * 256 + (l // 16) * 16)
    assert 3.5 < free < 6.0, free
    assert clash > 3 * free, (free, clash)
    assert 2.5 < cost(lambda l: 8 * l, kind=1) < 5.0
