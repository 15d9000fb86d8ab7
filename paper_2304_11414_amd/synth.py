"""Seeded synthetic inputs for the MoE-layer forward: shapes and value distributions only.

This module holds none of the method's arithmetic (no gating, no permutation, no FFN): it draws
tokens, router weights, router bias and expert weights with NumPy's PCG64 generator, and rounds them
to bf16-representable float32 values where a configuration is bf16.  Both the HIP path and the CPU
oracle are fed from here, so they see identical numbers.

The paper trains on a private corpus with GPT-3-style backbones (Section 4.1: sequence length 2048,
hidden 1024 / 4096, 64 experts, top-1); these synthetic tensors stand in for one MoE layer's input at
those shapes.

Weight layout: arrays are drawn directly in the library's [out, in] layout
(Wg_t[E, d], W1_t[N, F, d], W2_t[N, d, F]); the paper's math shapes (h x E, A: h x 4h, B: 4h x h)
are transposed *views* of the same memory, see ``math_views``.
"""

from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int                      # tokens = batch x sequence
    d: int                      # hidden size h
    F: int                      # FFN inner size (4h in every configuration here)
    E: int                      # experts in the tensor-parallel group
    top_k: int
    local_begin: int = 0        # this device holds experts [local_begin, local_begin + local_count)
    local_count: int = -1       # -1: all E
    capacity_factor: float = 0.0
    renorm_topk: bool = False
    in_dtype: str = "bf16"      # "bf16" | "f16" | "f32": tokens, router and expert weights, H, y_sliced
    out_dtype: str = "bf16"     # "bf16" | "f16" | "f32": the partial output
    seed: int = 0
    bias_kind: str = "none"     # "none" | "zipf": bias[e] = -bias_scale * bias_s * ln(e + 1)
    bias_s: float = 0.0
    bias_scale: float = 1.0

    @property
    def n_local(self) -> int:
        return self.E if self.local_count < 0 else self.local_count

    def scaled(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


# The five workloads, plus a sixth that is not a MoE layer: with a single expert the layer is the
# dense tensor-parallel FFN shard Y_i = GeLU(X A_i) B_i of Section 3.1.3 (one of 8 column/row slices
# of a d -> 4d -> d FFN, float32 partial sum), run on the same kernels.
# CONFIGS[1] is the headline (d=2048, E=8, top-1, bf16).
# bias_scale of "zipf5" was found offline by bisection so that the heaviest expert receives about
# 45 % of the 2*T assignments under top-2 (a token picks an expert at most once, so 50 % is the
# ceiling); a CPU test checks the realised share.
CONFIGS = [
    LayerConfig("tiny_f32", T=256, d=256, F=1024, E=4, top_k=1, in_dtype="f32", out_dtype="f32",
                seed=0),
    LayerConfig("gpt_top1", T=8192, d=2048, F=8192, E=8, top_k=1, seed=2),
    LayerConfig("capacity_top2", T=16384, d=2048, F=8192, E=16, top_k=2, capacity_factor=1.25,
                renorm_topk=True, seed=3, bias_kind="zipf", bias_s=1.1),
    LayerConfig("tp_slice_8of64", T=16384, d=4096, F=16384, E=64, top_k=1, local_begin=0,
                local_count=8, out_dtype="f32", seed=4),
    LayerConfig("wide_skewed_top2", T=32768, d=5120, F=20480, E=8, top_k=2, renorm_topk=True,
                seed=5, bias_kind="zipf", bias_s=1.5, bias_scale=1.55),
    LayerConfig("dense_tp_ffn_shard", T=8192, d=2048, F=1024, E=1, top_k=1, out_dtype="f32", seed=6),
]


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even), returned as float32 (in place)."""
    assert a.dtype == np.float32 and a.flags.c_contiguous
    u = a.view(np.uint32)
    u += np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    u &= np.uint32(0xFFFF0000)
    return a


def round_to_f16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest IEEE half (ties to even), returned as float32 (in place)."""
    assert a.dtype == np.float32
    a[...] = a.astype(np.float16).astype(np.float32)
    return a


def _normal(seed_seq, shape, std, bf16, threads=8):
    """N(0, std) float32 array, drawn in independent row-chunks (one child seed per chunk).
    bf16: False (keep float32), True or "bf16" (round to bf16), "f16" (round to IEEE half)."""
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(-1)
    n = flat.size
    chunk = 1 << 24
    n_chunks = max(1, (n + chunk - 1) // chunk)
    children = seed_seq.spawn(n_chunks)

    def fill(i):
        lo, hi = i * chunk, min(n, (i + 1) * chunk)
        g = np.random.Generator(np.random.PCG64(children[i]))
        g.standard_normal(hi - lo, dtype=np.float32, out=flat[lo:hi])
        if std != 1.0:
            flat[lo:hi] *= np.float32(std)
        if bf16 == "f16":
            round_to_f16(flat[lo:hi])
        elif bf16:
            round_to_bf16(flat[lo:hi])

    if n_chunks == 1:
        fill(0)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out


def router_bias(cfg: LayerConfig):
    if cfg.bias_kind == "none":
        return None
    if cfg.bias_kind == "zipf":
        e = np.arange(cfg.E, dtype=np.float64)
        return (-cfg.bias_scale * cfg.bias_s * np.log(e + 1.0)).astype(np.float32)
    raise ValueError(cfg.bias_kind)


def make_inputs(cfg: LayerConfig, parts=("x", "Wg_t", "bias", "W1_t", "W2_t")):
    """Draw the layer's inputs.  Each tensor has its own child seed, so any subset can be drawn and
    is identical to the same tensor in a full draw."""
    bf16 = {"bf16": True, "f16": "f16", "f32": False}[cfg.in_dtype]
    root = np.random.SeedSequence([0x2304_1141, cfg.seed])
    s_x, s_wg, s_w1, s_w2 = root.spawn(4)
    N = cfg.n_local
    out = {}
    if "x" in parts:
        out["x"] = _normal(s_x, (cfg.T, cfg.d), 1.0, bf16)
    if "Wg_t" in parts:
        out["Wg_t"] = _normal(s_wg, (cfg.E, cfg.d), 0.02, bf16)
    if "bias" in parts:
        out["bias"] = router_bias(cfg)
    if "W1_t" in parts:
        out["W1_t"] = _normal(s_w1, (N, cfg.F, cfg.d), 0.02, bf16)
    if "W2_t" in parts:
        out["W2_t"] = _normal(s_w2, (N, cfg.d, cfg.F), 0.02, bf16)
    return out


def math_views(inp):
    """The paper's math shapes as transposed views: Wg [d, E], W1[i] = A_i [d, F], W2[i] = B_i [F, d]."""
    v = {}
    if "Wg_t" in inp:
        v["Wg"] = inp["Wg_t"].T
    if "W1_t" in inp:
        v["W1"] = inp["W1_t"].transpose(0, 2, 1)
    if "W2_t" in inp:
        v["W2"] = inp["W2_t"].transpose(0, 2, 1)
    return v


def random_logits(T, E, seed, tie_fraction=0.0):
    """float32 router logits ~ N(0, 0.9^2) (the spread d=2048, std-0.02 weights give), optionally
    with a fraction of tokens carrying exactly duplicated values to exercise tie-breaking."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([0x10617, seed])))
    logits = (0.9 * g.standard_normal((T, E))).astype(np.float32)
    if tie_fraction > 0 and E > 1:
        n_tie = int(T * tie_fraction)
        rows = g.choice(T, size=n_tie, replace=False)
        src = g.integers(0, E, size=n_tie)
        dst = (src + 1 + g.integers(0, E - 1, size=n_tie)) % E
        logits[rows, dst] = logits[rows, src]
        rows_all = rows[: n_tie // 4]
        logits[rows_all, :] = logits[rows_all, :1]
    return logits
