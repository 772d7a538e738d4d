"""Stage shape records for the synthetic workloads.

A "stage" is one ministage of the paper's interleaved pipeline (Section 4.1.1):
a contiguous block of decoder layers that runs all of its microbatches' forward
passes, then all backward passes, then its own optimizer step on the
data-parallel shard (Section 4.1.2).  The records below are stage-sized slices
of Llama/GPT-shaped models like the ones the paper trains (Section 6.1), plus
scaled "twins" of the large ones that a plain fp64 CPU implementation can
finish in seconds.  Only shapes and hyper-parameters live here.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

ARCH_GPT = 0    # pre-LayerNorm, GELU FFN, biases, no RoPE
ARCH_LLAMA = 1  # pre-RMSNorm, SwiGLU FFN, RoPE, no biases
DTYPE_F32 = 0   # fp32 everywhere
DTYPE_BF16 = 1  # bf16 params/activations, fp32 master weights, grads, moments
DTYPE_F16 = 2   # the same with IEEE half; used with loss scaling (the mixed precision the paper trains in)


@dataclass(frozen=True)
class StageConfig:
    name: str
    arch: int
    dtype: int
    layers: int
    hidden: int
    heads: int
    ffn: int
    seq: int
    microbatch: int
    num_microbatches: int
    vocab: int = 0
    has_embed: int = 0
    has_head: int = 0
    recompute: int = 0
    pair_wgrad: int = 0            # library option: fold every other backward's weight gradients into the next one's
    offload_acts: int = 0          # library option (with recompute): boundary activations kept in pinned host memory
    act_budget_bytes: int = 0
    shard_num: int = 1      # the shard is the first shard_num/shard_den of the flat parameters
    shard_den: int = 1
    norm_eps: float = 1e-5
    rope_base: float = 10000.0
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    weight_decay: float = 0.01
    seed: int = 20250710

    @property
    def tokens(self) -> int:
        """Tokens in one microbatch."""
        return self.seq * self.microbatch

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    @property
    def params_per_layer(self) -> int:
        H, F = self.hidden, self.ffn
        if self.arch == ARCH_GPT:
            return 4 * H * H + 2 * H * F + 9 * H + F
        return 4 * H * H + 3 * H * F + 2 * H

    @property
    def n_params(self) -> int:
        n = self.layers * self.params_per_layer
        if self.has_embed:
            n += self.vocab * self.hidden
        if self.has_head:
            n += self.hidden + self.hidden * self.vocab
        return n

    @property
    def shard_range(self) -> tuple[int, int]:
        return 0, (self.n_params * self.shard_num) // self.shard_den

    def with_(self, **kw) -> "StageConfig":
        return replace(self, **kw)


def _mk() -> dict[str, StageConfig]:
    c = {}
    # The five benchmark stages (index = position in the benchmark list, seed = base + index).
    c["C1"] = StageConfig("C1", ARCH_GPT, DTYPE_F32, 2, 256, 4, 1024, 128, 2, 4, seed=20250710)
    c["C2"] = StageConfig("C2", ARCH_GPT, DTYPE_BF16, 6, 2048, 16, 8192, 2048, 1, 8,
                          shard_num=1, shard_den=4, seed=20250711)
    c["C3"] = StageConfig("C3", ARCH_LLAMA, DTYPE_BF16, 8, 4096, 32, 11008, 4096, 1, 16,
                          shard_num=1, shard_den=2, seed=20250712)
    c["C4a"] = StageConfig("C4a", ARCH_LLAMA, DTYPE_BF16, 3, 5120, 40, 13824, 2048, 2, 8,
                           shard_num=1, shard_den=3, seed=20250713)
    c["C4b"] = StageConfig("C4b", ARCH_LLAMA, DTYPE_BF16, 12, 5120, 40, 13824, 2048, 2, 8,
                           recompute=1, act_budget_bytes=96 * 10**9,
                           shard_num=1, shard_den=3, seed=20250713)
    c["C5"] = StageConfig("C5", ARCH_LLAMA, DTYPE_BF16, 4, 4096, 32, 11008, 4096, 1, 8,
                          vocab=32000, has_embed=1, has_head=1, seed=20250714)
    # Scaled twins: same architecture, head dim 128, number of microbatches,
    # shard fraction and recompute mode; smaller hidden/ffn/seq/layers/vocab.
    # ffn 1376 and vocab 2000 are deliberately not multiples of the GEMM tiles.
    c["C2t"] = StageConfig("C2t", ARCH_GPT, DTYPE_BF16, 2, 512, 4, 2048, 256, 1, 8,
                           shard_num=1, shard_den=4, seed=20250721)
    c["C3t"] = StageConfig("C3t", ARCH_LLAMA, DTYPE_BF16, 2, 512, 4, 1376, 256, 1, 16,
                           shard_num=1, shard_den=2, seed=20250722)
    c["C4at"] = StageConfig("C4at", ARCH_LLAMA, DTYPE_BF16, 2, 640, 5, 1728, 128, 2, 8,
                            shard_num=1, shard_den=3, seed=20250723)
    c["C4bt"] = StageConfig("C4bt", ARCH_LLAMA, DTYPE_BF16, 3, 640, 5, 1728, 128, 2, 8,
                            recompute=1, act_budget_bytes=96 * 10**9,
                            shard_num=1, shard_den=3, seed=20250723)
    c["C5t"] = StageConfig("C5t", ARCH_LLAMA, DTYPE_BF16, 2, 512, 4, 1376, 256, 1, 8,
                           vocab=2000, has_embed=1, has_head=1, seed=20250724)
    # fp16 twins (the paper's mixed precision): same shapes as C3t / C2t / C5t, fewer microbatches
    c["C3h"] = StageConfig("C3h", ARCH_LLAMA, DTYPE_F16, 2, 512, 4, 1376, 256, 1, 4,
                           shard_num=1, shard_den=2, seed=20250742)
    c["C2h"] = StageConfig("C2h", ARCH_GPT, DTYPE_F16, 2, 512, 4, 2048, 256, 1, 3,
                           shard_num=1, shard_den=4, seed=20250741)
    c["C5h"] = StageConfig("C5h", ARCH_LLAMA, DTYPE_F16, 2, 512, 4, 1376, 256, 1, 3,
                           vocab=2000, has_embed=1, has_head=1, seed=20250744)
    # fp32 Llama-style and GPT-with-head minis used to exercise every code path in fp32.
    c["L1"] = StageConfig("L1", ARCH_LLAMA, DTYPE_F32, 2, 256, 4, 688, 128, 2, 4,
                          vocab=1000, has_embed=1, has_head=1, seed=20250731)
    return c


CONFIGS = _mk()


def get_config(name: str) -> StageConfig:
    return CONFIGS[name]


def segments(cfg: StageConfig) -> list[tuple[str, int, int, int, str]]:
    """Flat parameter order of a stage as (name, offset, rows, cols, kind).

    kind is "matrix" (drawn N(0, std 0.02)), "gain" (1), "bias" (0) — used only
    to pick the distribution each segment is drawn from.  Matrices are row-major
    [in, out] and applied as y = x @ W.
    """
    H, F, V = cfg.hidden, cfg.ffn, cfg.vocab
    out: list[tuple[str, int, int, int, str]] = []
    off = 0

    def add(name, rows, cols, kind):
        nonlocal off
        out.append((name, off, rows, cols, kind))
        off += rows * cols

    if cfg.has_embed:
        add("embed.E", V, H, "matrix")
    for l in range(cfg.layers):
        p = f"L{l}."
        if cfg.arch == ARCH_GPT:
            add(p + "ln1.g", 1, H, "gain"); add(p + "ln1.b", 1, H, "bias")
            add(p + "Wqkv", H, 3 * H, "matrix"); add(p + "bqkv", 1, 3 * H, "bias")
            add(p + "Wo", H, H, "matrix"); add(p + "bo", 1, H, "bias")
            add(p + "ln2.g", 1, H, "gain"); add(p + "ln2.b", 1, H, "bias")
            add(p + "W1", H, F, "matrix"); add(p + "b1", 1, F, "bias")
            add(p + "W2", F, H, "matrix"); add(p + "b2", 1, H, "bias")
        else:
            add(p + "rms1.g", 1, H, "gain")
            add(p + "Wq", H, H, "matrix"); add(p + "Wk", H, H, "matrix")
            add(p + "Wv", H, H, "matrix"); add(p + "Wo", H, H, "matrix")
            add(p + "rms2.g", 1, H, "gain")
            add(p + "Wg", H, F, "matrix"); add(p + "Wu", H, F, "matrix")
            add(p + "Wd", F, H, "matrix")
    if cfg.has_head:
        add("final_norm.g", 1, H, "gain")
        add("head.Wh", H, V, "matrix")
    assert off == cfg.n_params
    return out
