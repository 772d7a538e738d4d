#!/usr/bin/env python3
"""Throughput of the per-stage training step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: M microbatch
forwards, M backwards each followed by its gradient accumulation, then the AdamW update of the
data-parallel shard (which also zeroes the gradient accumulators).  Inputs, parameters and
optimizer state are resident in HBM before the timed region starts.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3]

prints ONE JSON line: tokens/s of the stage step, the roofline figures of the dominant kernel
(from HIP events recorded around every launch on the stage's stream during the timed steps), the
model-FLOP utilisation, and the fp64 CPU oracle timed on a bounded sample of the same workload.
Everything runs on one GPU; --gpus above 1 is refused.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak (256 CUs x 4 SIMDs x 1024 flop/clk x 2.4 GHz)
PEAK_HBM_GBS = 8000.0

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "stage_step_C3_hbm_traffic.txt")


def kernel_sources_digest():
    """sha256 over the HIP sources the library is built from (file names and contents, sorted): the counter summary
    under profiles/ names the digest it was measured at, and a figure measured at other sources is not reported."""
    import hashlib
    d = os.path.join(ROOT, "paper_2507_10392_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel, cfg):
    """HBM-side bytes per launch of a kernel class from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under
    profiles/ (lines `traffic <workload> <kernel class> <wgrad group> <bytes per launch>` after a line
    `sources <digest>`).  This run measures no counters itself, so the figure is given only when the summary was
    made from the kernel sources this run uses; otherwise null."""
    group = 0 if not cfg.pair_wgrad else min(max(cfg.pair_wgrad, 2), 16, cfg.num_microbatches)
    try:
        with open(TRAFFIC_FILE) as f:
            lines = [ln.split() for ln in f]
    except OSError:
        return None
    digest = next((ln[1] for ln in lines if len(ln) >= 2 and ln[0] == "sources"), None)
    if digest != kernel_sources_digest():
        return None
    for ln in lines:
        if len(ln) >= 5 and ln[0] == "traffic" and ln[1] == workload and ln[2] == kernel and ln[3] in (str(group), "any"):
            return float(ln[4])
    return None


def model_flops_per_step(cfg):
    """Algorithmic FLOPs: 3 x forward; forward per token per layer = 2*P_mat + 4*H*(S+1)/2 (causal half)."""
    H, F, S = cfg.hidden, cfg.ffn, cfg.seq
    p_mat = 4 * H * H + (3 if cfg.arch == 1 else 2) * H * F
    per_tok = cfg.layers * (2 * p_mat + 4 * H * (S + 1) / 2)
    if cfg.has_head:
        per_tok += 2 * H * cfg.vocab
    return 3.0 * per_tok * cfg.tokens * cfg.num_microbatches


def fill_params(cfg, params, torch):
    from workloads.configs import segments
    for name, off, r, c, kind in segments(cfg):
        seg = params[off:off + r * c]
        if kind == "matrix":
            seg.normal_(0.0, 0.02)
        elif kind == "gain":
            seg.fill_(1.0)
        else:
            seg.zero_()


def cpu_baseline(cfg, shard_elems):
    """The oracle as it stands, on the host cores, on a bounded sample: ONE decoder layer x ONE microbatch
    at the workload's full shape, forward + backward in fp64 (numpy, BLAS threads as found), and its AdamW
    update on 2^24 elements.  The stage-step figure extrapolates both: tokens of a step / (layer time x
    layers x microbatches + AdamW time x shard / sample).  For head stages the embedding / LM head are
    left out of the sample, which makes the figure an upper bound."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import stage_oracle as so
    from workloads import make_inputs
    sample = cfg.with_(layers=1, num_microbatches=1, has_embed=0, has_head=0, vocab=0)
    inp = make_inputs(sample)
    t0 = time.time()
    y, cache = so.stage_forward(sample, inp.params, inp.x[0])
    so.stage_backward(sample, cache, inp.dy[0].astype(np.float64))
    dt = time.time() - t0
    n = 1 << 24
    rng = np.random.default_rng(cfg.seed)
    p, g, m, v = (rng.standard_normal(n) for _ in range(4))
    t0 = time.time()
    so.adamw(p, g, m, v * v, 1, cfg.lr, cfg.beta1, cfg.beta2, cfg.adam_eps, cfg.weight_decay, 1.0 / cfg.num_microbatches)
    dt_opt = time.time() - t0
    threads = max([q.get("num_threads", 1) for q in threadpool_info()] + [1])
    step_s = dt * cfg.layers * cfg.num_microbatches + dt_opt * shard_elems / n
    tokps = cfg.tokens * cfg.num_microbatches / step_s
    return {"value": tokps, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"1 of {cfg.layers} layers x 1 of {cfg.num_microbatches} microbatches ({sample.tokens} tokens) at full "
                      f"shape, fwd+bwd in fp64 numpy: {dt:.1f} s; AdamW on 2^24 of {shard_elems} shard elements: {dt_opt:.2f} s; "
                      f"value = step tokens / (layer time x layers x microbatches + AdamW time x shard / sample) "
                      f"= an extrapolated step of {step_s:.0f} s"}


class MinistageRunner:
    """The workload's layers cut into K ministages of equal depth that share two parameter slots on the GPU
    (include/ministages.h); a step runs them in the paper's order: all forwards ministage by ministage, then the
    backwards in reverse with each ministage's optimizer step right after its own backward."""

    def __init__(self, torch, zs, cfg, K, xs, dys):
        self.torch, self.K, self.M = torch, K, cfg.num_microbatches
        sub = cfg.with_(layers=cfg.layers // K)
        self.cc = zs.make_config(sub)
        self.P, _, _ = zs.query(self.cc)
        self.mem = mem = zs.ministages_query(self.cc, K)
        b, e = self.cc.shard_begin, self.cc.shard_end
        self.shard_elems = K * (e - b)
        td = torch.bfloat16 if cfg.dtype == 1 else torch.float32
        E = 2 if cfg.dtype == 1 else 4
        self.host = torch.empty(mem["host_bytes"], dtype=torch.uint8, pin_memory=True)
        self.host.zero_()
        tmp = torch.empty(self.P, dtype=td, device="cuda")
        for k in range(K):
            fill_params(sub, tmp, torch)
            o = k * mem["per_stage_host"]
            self.host[o + mem["off_params"]:o + mem["off_params"] + E * self.P].view(td).copy_(tmp)
            if mem["off_master"] >= 0:
                self.host[o + mem["off_master"]:o + mem["off_master"] + 4 * (e - b)].view(torch.float32).copy_(tmp[b:e].float())
        self.probe = self.host[mem["off_params"]:mem["off_params"] + E * (e - b)].view(td)   # ministage 0's shard
        del tmp
        self.arena = torch.empty(mem["device_bytes"], dtype=torch.uint8, device="cuda")
        self.ms = zs.Ministages(self.cc, K, self.host, self.arena)
        self.xs, self.dys = xs, dys
        T, H = cfg.tokens, cfg.hidden
        self.bufs = [[torch.empty(T, H, dtype=td, device="cuda") for _ in range(self.M)] for _ in range(2)]

    def step(self, t):
        ms, M = self.ms, self.M
        cur = self.xs
        for k in range(self.K):
            nxt = self.bufs[k % 2]
            for i in range(M):
                ms.forward(k, i, cur[i], nxt[i])
            cur = nxt
        g = self.dys
        for k in reversed(range(self.K)):
            nxt = self.bufs[k % 2]
            for i in reversed(range(M)):
                ms.backward(k, i, g[i], nxt[i], 1.0 / M)
                ms.accumulate(k, i)
            ms.optimizer_step(k, t)
            g = nxt

    def profile(self, on):
        for k in range(self.K):
            self.ms.stage_profile(k, on)

    def profile_read(self):
        tot = {}
        for k in range(self.K):
            for name, st in self.ms.stage_profile_read(k).items():
                d = tot.setdefault(name, dict(launches=0, ms=0.0, flops=0.0, bytes=0.0))
                for key in d:
                    d[key] += st[key]
        return tot

    def close(self):
        self.ms.close()


def mfma_ceiling():
    """What the matrix cores sustain with nothing else going on (stage_op_mfma_rate): the inner loop of the GEMM's wave tile
    on random operands held in registers, no LDS and no memory traffic, for both bf16 MFMA shapes.  The MI355X runs such a
    loop at its power limit, so this is the rate a bf16 GEMM can approach on it; 2.5 PFLOP/s stays the roofline's peak."""
    import torch
    import paper_2507_10392_amd as zs
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    torch.manual_seed(0)
    operands = torch.randn(32768, device=dev).to(torch.bfloat16)           # 64 KB
    sink = torch.empty(256 * 512, device=dev, dtype=torch.float32)
    flops_per_iter = 2.0 * 128 * 64 * 32 * 8 * 256                          # a 128 x 64 wave tile advances 32 columns of k per iteration
    out = {}
    for name, shape in (("32x32x16", 32), ("16x16x32", 16)):
        zs.ops.mfma_rate(st, shape, 20000, operands, sink)                 # warm-up, and brings the clock down to its sustained value
        runs = []
        for _ in range(3):
            iters = 60000
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            zs.ops.mfma_rate(st, shape, iters, operands, sink)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b)
            runs.append({"ms": ms, "tflops": flops_per_iter * iters / ms / 1e9})
        out[name] = {"tflops": sorted(r["tflops"] for r in runs)[1], "runs": runs, "frac_of_2500": sorted(r["tflops"] for r in runs)[1] / 2500.0}
    print(json.dumps({"mfma_sustained": out, "unit": "TFLOP/s", "dtype": "bf16", "finite": bool(torch.isfinite(sink).all().item()),
                      "note": "register-resident operands (random bf16), 128 accumulator registers per wave, 2 waves per SIMD, "
                              "256 workgroups; median of 3 launches of about 35 ms each"}))


def lds_patterns():
    """LDS time per wave read (stage_op_lds_probe) for the access patterns between which the GEMM's slab layouts were chosen:
    fragment reads and slab stores of k-contiguous slabs with padded rows and with permuted unpadded rows, transposing
    reads of row-contiguous slabs with and without the chunk swap, and the 32x32x16 fragment shapes for comparison."""
    import ctypes
    import torch
    import paper_2507_10392_amd as zs
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    LDR = 288   # elements per k-line of a 256-row [k][row] slab
    pats = [
        ("16-byte reads, lane l at 16 l (no pattern)", 0, lambda l: 16 * l),
        ("k-contiguous slab, 32x32x16 fragment (row l%32, piece l/32), rows padded to 144 bytes", 0, lambda l: (l % 32) * 144 + (l // 32) * 16),
        ("k-contiguous slab, 16x16x32 fragment (row l%16, piece l/16), rows padded to 144 bytes", 0, lambda l: (l % 16) * 144 + (l // 16) * 16),
        ("k-contiguous slab, 16x16x32 fragment, 128-byte rows, piece p of row r at p ^ r%8 (in use)", 0, lambda l: (l % 16) * 128 + (((l // 16) ^ (l % 8)) * 16)),
        ("k-contiguous slab, store of 8 rows x 8 pieces, rows padded to 144 bytes", 0, lambda l: (l // 8) * 144 + (l % 8) * 16),
        ("k-contiguous slab, store of 8 rows x 8 pieces, 128-byte rows, permuted pieces (in use)", 0, lambda l: (l // 8) * 128 + (((l % 8) ^ ((l // 8) % 8)) * 16)),
        ("row-contiguous slab, store of 2 k-lines x 32 pieces, chunks swapped (in use)", 0, lambda l: (l // 32) * LDR * 2 + (l % 32) * 16),
        ("transposing reads, lane l at 8 l (no pattern)", 1, lambda l: 8 * l),
        ("row-contiguous slab, 32x32x16 fragment (k-lines 8 (g/2) + r/4, rows 16 (g%2) + 4 (r%4))", 1,
         lambda l: ((8 * ((l >> 4) >> 1) + ((l & 15) >> 2)) * LDR + 16 * ((l >> 4) & 1) + 4 * (l & 3)) * 2),
        ("row-contiguous slab, 16x16x32 fragment (k-lines 8 g + r/4, rows 4 (r%4)), no swap", 1,
         lambda l: ((8 * (l >> 4) + ((l & 15) >> 2)) * LDR + 4 * (l & 3)) * 2),
        ("row-contiguous slab, 16x16x32 fragment, 16-row chunks swapped on odd eights of k (in use)", 1,
         lambda l: ((8 * (l >> 4) + ((l & 15) >> 2)) * LDR + ((4 * (l & 3)) ^ (((l >> 4) & 1) << 4))) * 2),
    ]
    iters = 4000
    cyc = torch.zeros(2, dtype=torch.int64, device=dev)
    rows = []
    for name, kind, f in pats:
        host = (ctypes.c_int32 * 64)(*[f(l) for l in range(64)])
        devoff = torch.tensor(list(host), dtype=torch.int32, device=dev)
        for _ in range(2):
            zs.ops.lds_probe(st, kind, host, devoff, iters, cyc)
        torch.cuda.synchronize()
        rows.append({"pattern": name, "kind": "ds_read_b64_tr_b16" if kind else "ds_read_b128",
                     "cycles_per_wave_read": round(int(cyc[0].item()) / (iters * 8 * 8), 2)})
    print(json.dumps({"lds_patterns": rows, "note": "one workgroup of 8 waves, 8 independent reads in flight per wave; "
                      "4.6 (16-byte) and 3.6 (transposing) cycles per wave read are the conflict-free figures"}))


def gemm_scan():
    """Three measurements of the bf16 GEMM that the tile and stream decisions rest on.  (1) Time against K at one round of
    256 tiles (M = N = 4096): the slope is the K loop's rate, the intercept what a launch costs beyond it (launch, first
    loads, the store pass).  (2) Time against the number of 256x256 tiles at K = 4096: a grid pays for whole rounds of 256
    workgroups.  (3) The dX products of one layer and a grouped weight-gradient product, enqueued on one stream and on two."""
    import numpy as np
    import torch
    import paper_2507_10392_amd as zs
    dev = torch.device("cuda:0")
    main = torch.cuda.current_stream()

    def product(M, N, K, ta, tb, accum, impl=2):
        A = torch.randn(M * K, device=dev).to(torch.bfloat16)
        B = (torch.randn(K * N, device=dev) * 0.02).to(torch.bfloat16)
        C = torch.zeros(M * N, device=dev, dtype=torch.float32 if accum else torch.bfloat16)
        lda, ldb = (M if ta else K), (K if tb else N)
        return lambda st: zs.ops.gemm(st.cuda_stream, 1, ta, tb, M, N, K, A, lda, B, ldb, C, N, int(accum), None, None, 0, 1,
                                      M * K, K * N, M * N, 0, 0, 0, impl)

    def us(f, n=30, w=5):
        for _ in range(w):
            f(main)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            f(main)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n * 1e3

    forms = (("nt", 0, 1, 0), ("nn", 0, 0, 0), ("tn_accumulate", 1, 0, 1))
    k_scan = []
    for name, ta, tb, acc in forms:
        ks = [2048, 4096, 8192, 16384]
        ts = [us(product(4096, 4096, K, ta, tb, acc)) for K in ks]
        slope, fixed = np.polyfit(np.array(ks, float), np.array(ts), 1)
        k_scan.append({"form": name, "us_at_K": dict(zip(map(str, ks), [round(t, 1) for t in ts])), "fixed_us": round(float(fixed), 1),
                       "k_loop_tflops": round(2.0 * 4096 * 4096 / slope / 1e6, 0)})
    rounds = []
    for N in (4096, 8192, 11008, 12288):
        tiles = 16 * ((N + 255) // 256)
        t = us(product(4096, N, 4096, 0, 1, 0, impl=3))
        rounds.append({"N": N, "tiles_256x256": tiles, "rounds": round(tiles / 256.0, 3), "us": round(t, 1),
                       "tflops": round(2.0 * 4096 * N * 4096 / t / 1e6, 0)})
    T, H, F = 4096, 4096, 11008
    chain = [product(T, F, H, 0, 1, 0), product(T, H, F, 0, 1, 0), product(T, H, H, 0, 1, 0), product(T, H, H, 0, 1, 0)]
    wgrad = product(F, H, 8 * T, 1, 0, 1)
    second = torch.cuda.Stream()                                         # default priority

    def both(two_streams, layers=40, groups=10):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(layers):
            if i < groups:
                wgrad(second if two_streams else main)
            for f in chain:
                f(main)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    both(False), both(True)
    one = sorted(both(False) for _ in range(3))[1]
    two = sorted(both(True) for _ in range(3))[1]
    del chain, wgrad
    torch.cuda.empty_cache()

    # (4) the weight gradients of a group of microbatches whose tiles do not fill whole rounds: as one K loop per tile
    # (the last round on 128x128 tiles where the dispatcher chooses so), and with the last round's K range cut into chunks
    def grouped(M, N, batch, parts):
        A = [torch.randn(T, M, device=dev).to(torch.bfloat16) for _ in range(parts)]
        B = [(torch.randn(T, N * batch, device=dev) * 0.02).to(torch.bfloat16) for _ in range(parts)]
        C = torch.zeros(batch * M * N, device=dev)
        need = zs.wgrad_parts_scratch_bytes(M, N, T, T, parts, batch)
        ws = torch.empty(max(need, 256) // 4, device=dev)
        uncut = lambda st: zs.wgrad_parts(st.cuda_stream, 1, M, N, T, T, A, M, B, N * batch, C, N, batch, 0, N, M * N, 2)
        cut = lambda st: zs.wgrad_parts_cut(st.cuda_stream, 1, M, N, T, T, A, M, B, N * batch, C, N, batch, 0, N, M * N, ws, need)
        tu, tc = us(uncut, 10, 3), us(cut, 10, 3)
        flops = 2.0 * M * N * batch * T * parts
        return {"M": M, "N": N, "batch": batch, "parts": parts, "tiles": batch * ((M + 255) // 256) * ((N + 255) // 256),
                "scratch_MiB": need >> 20, "uncut_us": round(tu, 0), "cut_us": round(tc, 0),
                "uncut_tflops": round(flops / tu / 1e6, 0), "cut_tflops": round(flops / tc / 1e6, 0)}

    cuts = [grouped(F, H, 1, 8), grouped(H, F, 2, 8), grouped(F, H, 1, 4), grouped(H, H, 3, 8)]
    print(json.dumps({"gemm_scan": {"time_against_K": k_scan, "time_against_tiles": rounds,
                                    "streams": {"one_stream_ms": round(one, 2), "two_streams_ms": round(two, 2),
                                                "work": "40 x (4 dX products of a C3 layer) + 10 x (dWd over 8 microbatches)"},
                                    "last_round_cut_along_K": cuts},
                      "dtype": "bf16", "note": "M = N = 4096 for the K scan (256 tiles of 256x256: one round); least-squares line over "
                      "the four K; the tile scan forces the 256x256 tile"}))


def planner_profile(cfg):
    """What the paper's planner takes from a GPU (Section 4.3, "Profiling" and "Memory Model"): the stage timed at
    small microbatch sizes with stage_time_layers, the library's least-squares line per pass, the line's
    prediction against a measurement at larger sizes, and the four memory terms of stage_query."""
    import torch
    import paper_2507_10392_amd as zs
    dev = torch.device("cuda:0")
    td = torch.bfloat16 if cfg.dtype == 1 else torch.float32
    base = cfg.with_(layers=min(cfg.layers, 2), num_microbatches=1, has_embed=0, has_head=0, vocab=0, recompute=0, offload_acts=0)
    fit_sizes, held_out = [1, 2, 3, 4], [6, 8]
    points = {}
    for mb in fit_sizes + held_out:
        c = base.with_(microbatch=mb * cfg.microbatch)
        cc = zs.make_config(c)
        P, mem, _ = zs.query(cc)
        b, e = cc.shard_begin, cc.shard_end
        params = torch.empty(P, dtype=td, device=dev)
        fill_params(c, params, torch)
        master = params[b:e].float() if cfg.dtype == 1 else None
        grad = torch.zeros(P, dtype=torch.float32, device=dev)
        m, v = torch.zeros(max(e - b, 1), device=dev), torch.zeros(max(e - b, 1), device=dev)
        ws = torch.empty(mem["workspace"], dtype=torch.uint8, device=dev)
        x = torch.randn(c.tokens, c.hidden, device=dev).to(td)
        dy = (torch.randn(c.tokens, c.hidden, device=dev) * 0.01).to(td)
        y, dx = torch.empty_like(x), torch.empty_like(x)
        st = zs.Stage(cc, params, master, grad, m, v, ws)
        f, bw = st.time_layers(x, y, dy, dx, reps=3)
        st.close()
        points[mb] = (f / base.layers, bw / base.layers)
        del params, master, grad, m, v, ws, x, dy, y, dx
    out = {"workload": f"{cfg.name}: one layer, microbatch sizes in units of {cfg.microbatch} x {cfg.seq} tokens",
           "ms_per_layer": {str(k): {"fwd": round(p[0], 4), "bwd": round(p[1], 4)} for k, p in points.items()}}
    for i, name in enumerate(("fwd", "bwd")):
        a, sl, r2 = zs.fit_linear([float(k) for k in fit_sizes], [points[k][i] for k in fit_sizes])
        out[name] = {"intercept_ms": a, "slope_ms_per_unit": sl, "r2": r2, "fitted_on": fit_sizes,
                     "held_out": {str(k): {"predicted": a + sl * k, "measured": points[k][i],
                                            "error": (a + sl * k) / points[k][i] - 1.0} for k in held_out}}
    _, mem, _ = zs.query(zs.make_config(cfg))
    out["memory_model_bytes"] = {k: mem[k] for k in ("params", "grads", "optim", "activations")}
    out["memory_model_bytes"]["total"] = sum(out["memory_model_bytes"].values())
    print(json.dumps({"planner_profile": out}))


def describe(cfg, M, shard_elems, P, ministages=0):
    return (f"{cfg.name}: {cfg.layers} layers, hidden {cfg.hidden}, heads {cfg.heads}, ffn {cfg.ffn}, "
            f"seq {cfg.seq}, microbatch {cfg.microbatch} x {M} microbatches, "
            f"{'Llama' if cfg.arch else 'GPT'}-style"
            + (f", embedding + LM head over {cfg.vocab} tokens" if cfg.has_head else "")
            + f", AdamW shard {shard_elems} of {P} params, "
            f"recompute {cfg.recompute}, pair_wgrad {cfg.pair_wgrad}, offload_acts {cfg.offload_acts}"
            + (f", activation budget {cfg.act_budget_bytes} B" if cfg.act_budget_bytes else "")
            + (f", {ministages} ministages of {cfg.layers // ministages} layers time-multiplexed" if ministages else ""))


def run_workload(torch, zs, cfg, steps, warmup, *, kernel_events=True, graph_mode=False, ministages=0, loss_scale=1.0,
                 fp16_flag=False, workload_key=None):
    """Allocates one workload's buffers, runs `warmup` untimed and `steps` timed stage steps and returns the
    figures of the run; everything it allocated is released when it returns."""
    dev = torch.device("cuda:0")
    torch.manual_seed(cfg.seed)
    cc = zs.make_config(cfg)
    P, mem, _ = zs.query(cc)
    b, e = cc.shard_begin, cc.shard_end
    bf = cfg.dtype != 0
    td = torch.bfloat16 if cfg.dtype == 1 else torch.float16 if cfg.dtype == 2 else torch.float32
    M, T, H = cfg.num_microbatches, cfg.tokens, cfg.hidden

    if not ministages:
        params = torch.empty(P, dtype=td, device=dev)
        fill_params(cfg, params, torch)
        master = params[b:e].float() if bf else None
        grad = torch.zeros(P, dtype=torch.float32, device=dev)
        m = torch.zeros(max(e - b, 1), dtype=torch.float32, device=dev)
        v = torch.zeros(max(e - b, 1), dtype=torch.float32, device=dev)
        ws = torch.empty(mem["workspace"], dtype=torch.uint8, device=dev)
    if cfg.has_embed:
        xs = [torch.randint(0, cfg.vocab, (T,), dtype=torch.int32, device=dev) for _ in range(M)]
    else:
        xs = [torch.randn(T, H, device=dev).to(td) for _ in range(M)]
    tgs = [torch.randint(0, cfg.vocab, (T,), dtype=torch.int32, device=dev) for _ in range(M)] if cfg.has_head else [None] * M
    losses = [torch.zeros(1, device=dev) for _ in range(M)] if cfg.has_head else [None] * M
    dys = [None] * M if cfg.has_head else [(torch.randn(T, H, device=dev) * (0.01 * loss_scale)).to(td) for _ in range(M)]
    ys = [torch.empty(T, H, dtype=td, device=dev) for _ in range(M)]
    dxs = [None] * M if cfg.has_embed else [torch.empty(T, H, dtype=td, device=dev) for _ in range(M)]
    if ministages:
        stage = MinistageRunner(torch, zs, cfg, ministages, xs, dys)
        params, mem, shard_elems = stage.probe, stage.mem, stage.shard_elems
    else:
        stage = zs.Stage(cc, params, master, grad, m, v, ws)
        shard_elems = e - b
    if cfg.offload_acts and not ministages:
        stage.attach_host_stash(torch.empty(mem["host_stash"], dtype=torch.uint8, pin_memory=True))

    def microbatches():
        for i in range(M):
            stage.forward(i, xs[i], ys[i], tgs[i], losses[i])
        for i in reversed(range(M)):
            stage.backward(i, dys[i], dxs[i], loss_scale / M)
            stage.accumulate(i)

    graph = None
    overflow = None
    if fp16_flag:
        overflow = torch.zeros(1, dtype=torch.int32, device=dev)
        zs.lib().stage_set_overflow_flag(stage.h, overflow.data_ptr())

    def step(t):
        if ministages:
            return stage.step(t)
        if graph is not None:
            graph.replay()
            stage.graph_replayed(M)
        else:
            microbatches()
        stage.optimizer_step(t, 1.0 / loss_scale)

    t = 0
    main_stream = torch.cuda.current_stream()
    if graph_mode:
        # one eager step configures every kernel; then the loop is captured on a side stream the stage is bound to
        kernel_events = False
        stage.close()
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            stage = zs.Stage(cc, params, master, grad, m, v, ws, stream=side)
            t += 1
            step(t)
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                microbatches()
            graph = g
        torch.cuda.set_stream(side)
    for _ in range(warmup):
        t += 1
        step(t)
    torch.cuda.synchronize()
    # Per-kernel HIP events bracket every launch of the LAST timed step only: two event records per
    # launch leave small gaps in the queue (2-3 % of a C3 step), which one step in K keeps out of `value`
    # almost entirely while the kernel figures still come from inside the timed region.
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]   # on the stage's stream
    t0 = time.perf_counter()
    marks[0].record()
    enqueue_ms = []          # host time to enqueue each step (no synchronisation inside): must stay below the step time
    for i in range(steps):
        t += 1
        if i == steps - 1 and kernel_events:
            stage.profile(True)
        h0 = time.perf_counter()
        step(t)
        enqueue_ms.append((time.perf_counter() - h0) * 1e3)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    in_order_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    per_step_ms = sorted(in_order_ms)
    stats = stage.profile_read() if kernel_events else {}
    stage.profile(False)
    finite = bool(torch.isfinite(params.float().sum()).item())

    ms_per_step = dt * 1e3 / steps
    tokens = T * M
    value = tokens / (dt / steps)
    mflops = model_flops_per_step(cfg)
    mfu = mflops / (dt / steps) / (PEAK_BF16_TFLOPS * 1e12)

    kernels = {}
    for name, st in stats.items():
        if st["launches"] == 0:
            continue
        avg_ms = st["ms"] / st["launches"]
        k = {"launches_per_step": st["launches"], "avg_ms": avg_ms, "ms_per_step": st["ms"]}
        if st["flops"] > 0:
            k["tflops"] = st["flops"] / st["ms"] / 1e9
        if st["bytes"] > 0:
            k["gbs"] = st["bytes"] / st["ms"] / 1e6
        kernels[name] = k
    roofline = None
    if kernels:
        dom = max(kernels, key=lambda n: kernels[n]["ms_per_step"])
        k = kernels[dom]
        if "tflops" in k:
            roofline = {"kernel": dom, "bound": "mfma", "achieved": k["tflops"], "peak": PEAK_BF16_TFLOPS,
                        "unit": "TFLOP/s", "frac": k["tflops"] / PEAK_BF16_TFLOPS}
        else:
            roofline = {"kernel": dom, "bound": "hbm", "achieved": k.get("gbs", 0.0), "peak": PEAK_HBM_GBS,
                        "unit": "GB/s", "frac": k.get("gbs", 0.0) / PEAK_HBM_GBS}
        roofline["avg_launch_ms"] = k["avg_ms"]
        roofline["traffic"] = measured_traffic(workload_key or cfg.name, dom, cfg)

    out = {
        "value": value, "ms_per_step": ms_per_step,
        "dtype": {0: "f32", 1: "bf16", 2: "f16"}[cfg.dtype],
        "config": {"workload": describe(cfg, M, shard_elems, P, ministages), "tokens_per_step": tokens,
                   "shard_elems": shard_elems},
        "ms_each_step": [round(x, 2) for x in in_order_ms], "enqueue_ms_each_step": [round(x, 2) for x in enqueue_ms],
        "ms_per_step_min": per_step_ms[0], "ms_per_step_median": per_step_ms[len(per_step_ms) // 2],
        "mfu_model_flops": mfu, "hfu_executed_flops": mfu * (4.0 / 3.0 if cfg.recompute else 1.0),
        "model_tflop_per_step": mflops / 1e12, "finite": finite,
        "roofline": roofline, "kernels": kernels, "hip_graph": bool(graph_mode),
        "memory_bytes": mem,
    }
    if overflow is not None:
        out["fp16"] = {"loss_scale": loss_scale, "overflow_flag": int(overflow.item())}
    if "adamw" in kernels and "gbs" in kernels["adamw"]:
        # The update kernel reads p, g, m, v and writes p, m, v and the 16-bit copy: 30 B per shard element (28 B in
        # fp32), exactly its algorithmic bytes.  Dropping the gradients (Section 4.1.2) is a fill over the whole
        # accumulator right after it (class zero_grads, 4 B per stage parameter); optimizer_phase is both together.
        out["adamw_hbm_frac"] = kernels["adamw"]["gbs"] / PEAK_HBM_GBS
        ph = [kernels[k] for k in ("adamw", "zero_grads", "overflow_check") if k in kernels]
        ms = sum(k["ms_per_step"] for k in ph)
        nbytes = sum(k.get("gbs", 0.0) * 1e6 * k["ms_per_step"] for k in ph)
        out["optimizer_phase"] = {"ms": ms, "bytes": nbytes, "gbs": nbytes / ms / 1e6, "hbm_frac": nbytes / ms / 1e6 / PEAK_HBM_GBS}
    if ministages:
        h2d, d2h = stage.ms.traffic()
        nsteps = steps + warmup
        out["ministages"] = {"K": ministages, "device_arena_bytes": mem["device_bytes"], "resident_bytes": mem["resident_bytes"],
                             "host_bytes": mem["host_bytes"], "h2d_bytes_per_step": h2d / nsteps, "d2h_bytes_per_step": d2h / nsteps}
    stage.close()
    if graph_mode:
        torch.cuda.set_stream(main_stream)
    out["_shard_elems"] = shard_elems
    return out


OTHER_WORKLOADS = ("C1", "C2", "C4a", "C4b", "C5")


def brief(r):
    """What the line carries for each of the other workloads."""
    d = {"workload": r["config"]["workload"], "tokens_per_s": r["value"], "ms_per_step": r["ms_per_step"],
         "ms_per_step_min": r["ms_per_step_min"], "steps": len(r["ms_each_step"]), "dtype": r["dtype"],
         "mfu_model_flops": r["mfu_model_flops"], "hfu_executed_flops": r["hfu_executed_flops"],
         "model_tflop_per_step": r["model_tflop_per_step"], "finite": r["finite"]}
    if r["roofline"]:
        rf = r["roofline"]
        d["dominant_kernel"] = {"kernel": rf["kernel"], "bound": rf["bound"], "achieved": rf["achieved"], "unit": rf["unit"],
                                "frac": rf["frac"], "avg_launch_ms": rf["avg_launch_ms"]}
    if "adamw_hbm_frac" in r:
        d["adamw_hbm_frac"] = r["adamw_hbm_frac"]
    d["activation_bytes"] = r["memory_bytes"].get("activations")
    return d


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=None,
                    help="C1 | C2 | C3 | C4a | C4b | C5: time that workload alone.  Without it the headline workload C3 is "
                         "timed with --steps / --warmup and then each of the others for 3 steps after 1 warm-up step "
                         "(block other_workloads of the same line)")
    ap.add_argument("--no-other-workloads", action="store_true", help="headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not bracket launches with HIP events")
    ap.add_argument("--no-pair-wgrad", action="store_true",
                    help="every backward runs its own weight-gradient products (stage_config.pair_wgrad = 0)")
    ap.add_argument("--wgrad-group", type=int, default=16, metavar="G",
                    help="microbatches whose weight-gradient products share one K loop (stage_config.pair_wgrad = G, "
                         "at most 16 and at most the number of microbatches)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the microbatch loop of a step in a HIP graph and replay it (for launch-bound stages); "
                         "per-kernel events are off in this mode")
    ap.add_argument("--recompute", action="store_true", help="run the workload with per-layer recompute (stage_config.recompute = 1)")
    ap.add_argument("--offload", action="store_true",
                    help="keep the boundary activations in pinned host memory (stage_config.offload_acts = 1; implies --recompute)")
    ap.add_argument("--fp16", action="store_true",
                    help="run the workload in fp16 mixed precision (stage_config.dtype = 2) with a loss scale of 1024 on the "
                         "upstream gradient, taken out again by the optimizer step, and the overflow test switched on")
    ap.add_argument("--ministages", type=int, default=0, metavar="K",
                    help="cut the workload's layers into K ministages that share two parameter slots on the GPU, the rest "
                         "waiting in pinned host memory (include/ministages.h); interior stages only")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="time a register-resident loop of bf16 MFMAs of both shapes: the matrix-core rate that the chip sustains")
    ap.add_argument("--lds-patterns", action="store_true",
                    help="time the LDS access patterns between which the GEMM's slab layouts were chosen")
    ap.add_argument("--gemm-scan", action="store_true",
                    help="time the bf16 GEMM against K, against the number of tiles, and on one stream against two")
    ap.add_argument("--planner-profile", action="store_true",
                    help="time one layer at small microbatch sizes, fit the runtime lines and print them with the memory terms")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the stage step on ONE GPU only (no collectives, no sharding across GPUs); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2507_10392_amd as zs
    from workloads import get_config

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    headline = args.workload or "C3"
    variant = bool(args.workload or args.recompute or args.offload or args.fp16 or args.ministages or args.graph
                   or args.no_pair_wgrad or args.planner_profile)

    def configured(name):
        return get_config(name).with_(pair_wgrad=0 if args.no_pair_wgrad else max(args.wgrad_group, 1))

    cfg = configured(headline)
    if args.recompute or args.offload:
        cfg = cfg.with_(recompute=1, offload_acts=1 if args.offload else 0)
    loss_scale = 1.0
    if args.fp16:
        if cfg.dtype != 1 or args.ministages:
            print("bench.py: --fp16 applies to the bf16 workloads and not to --ministages", file=sys.stderr)
            sys.exit(2)
        cfg, loss_scale = cfg.with_(dtype=2), 1024.0
    if args.offload and args.graph:
        print("bench.py: --offload cannot be combined with --graph", file=sys.stderr)
        sys.exit(2)
    if args.ministages and (args.graph or cfg.has_embed or cfg.has_head or cfg.layers % args.ministages):
        print("bench.py: --ministages K needs an interior stage whose layer count K divides, and no --graph",
              file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(torch.device("cuda:0"))
    if args.mfma_ceiling:
        mfma_ceiling()
        return
    if args.lds_patterns:
        lds_patterns()
        return
    if args.gemm_scan:
        gemm_scan()
        return
    if args.planner_profile:
        planner_profile(cfg)
        return

    r = run_workload(torch, zs, cfg, args.steps, args.warmup, kernel_events=not args.no_kernel_events, graph_mode=args.graph,
                     ministages=args.ministages, loss_scale=loss_scale, fp16_flag=args.fp16, workload_key=headline)
    shard_elems = r.pop("_shard_elems")
    out = {"metric": "stage train tokens/s on 1 MI355X (fwd+bwd+AdamW); MFMA util % of bf16 peak",
           "value": r.pop("value"), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": r.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": r.pop("dtype"), "data": "synthetic"}
    out.update(r)
    if not variant and not args.no_other_workloads:
        # The other benchmark stages, each as configured (C4b: 12 layers, full recompute, inside its activation budget),
        # one after the other with their buffers released in between; 1 warm-up step and 3 timed steps each.
        others = {}
        for name in OTHER_WORKLOADS:
            torch.cuda.empty_cache()
            try:
                o = run_workload(torch, zs, configured(name), 3, 1, kernel_events=True, workload_key=name)
                others[name] = brief(o)
                if o["ms_per_step"] < 100.0:
                    # a stage whose step is made of hundreds of short launches: the same step with its microbatch loop
                    # captured once in a HIP graph and replayed (the library only enqueues, so a caller may do this)
                    torch.cuda.empty_cache()
                    g = run_workload(torch, zs, configured(name), 3, 1, graph_mode=True, workload_key=name)
                    others[name]["hip_graph_replay"] = {"tokens_per_s": g["value"], "ms_per_step": g["ms_per_step"],
                                                        "mfu_model_flops": g["mfu_model_flops"], "finite": g["finite"]}
            except Exception as ex:      # reported, never hidden: a workload that does not run says so in the line
                others[name] = {"error": f"{type(ex).__name__}: {ex}"}
        out["other_workloads"] = others
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, shard_elems)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
