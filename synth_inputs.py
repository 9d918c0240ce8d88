"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module only *draws* inputs (sample sizes, segment lengths, tensors).  It holds none of the
method's arithmetic: no grouping, no normalisation, no attention, no GEMM.  Both sides receive
exactly the arrays produced here, so they see identical (bf16-representable) values.

The shapes follow the paper's workload (Sec. 5.2 "Implementation Details": roughly 1K ViT tokens
per image tile; App. D: up to 12 tiles per sample) and the block shapes of the five benchmark
configurations.  The paper's datasets are not available; these draws stand in for their size
distributions only.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

# ----------------------------------------------------------------------------------------------
# Block shapes of the five benchmark configurations.
# ----------------------------------------------------------------------------------------------

NORM_LAYERNORM, NORM_RMSNORM = 0, 1
MLP_GELU, MLP_SWIGLU = 0, 1
MASK_BIDIR, MASK_CAUSAL = 0, 1


@dataclass(frozen=True)
class BlockShape:
    name: str
    n_blocks: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp_dim: int
    norm: int
    mlp: int
    mask: int
    use_rotary: bool
    has_bias: bool
    kind: str                      # "tiny" | "vit" | "llm"
    budget: int                    # tiles per mini-batch (vit) or tokens per mini-batch (llm)
    rotary_base: float = 10000.0
    norm_eps: float = field(default=1e-5)

    @property
    def d_qkv(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def up_rows(self) -> int:
        return self.mlp_dim * (2 if self.mlp == MLP_SWIGLU else 1)


VIT_TILE_TOKENS = 1025          # 32x32 patches + cls token per 448-px tile
LLM_TOKENS_PER_TILE = 256       # visual tokens per tile after the connector's sub-sampling
TEXT_MEDIAN, TEXT_SIGMA, TEXT_CAP = 300.0, 1.0, 4096
MAX_TILES = 12
# pmf over 1..12 tiles per sample, skewed toward 1-4 (72 % of the mass), mean 3.705
TILE_PMF = (0.22, 0.20, 0.16, 0.14, 0.07, 0.06, 0.04, 0.03, 0.03, 0.02, 0.015, 0.015)

CONFIGS = {
    1: BlockShape("tiny", 1, 256, 4, 4, 64, 1024, NORM_LAYERNORM, MLP_GELU, MASK_CAUSAL,
                  False, True, "tiny", 1024, norm_eps=1e-5),
    2: BlockShape("vit-300m", 24, 1024, 16, 16, 64, 4096, NORM_LAYERNORM, MLP_GELU, MASK_BIDIR,
                  False, True, "vit", 12, norm_eps=1e-5),
    3: BlockShape("llm-7b-stage", 8, 4096, 32, 8, 128, 14336, NORM_RMSNORM, MLP_SWIGLU,
                  MASK_CAUSAL, True, False, "llm", 16384, norm_eps=1e-6),
    4: BlockShape("vit-6b-stage", 12, 3200, 25, 25, 128, 12800, NORM_RMSNORM, MLP_GELU,
                  MASK_BIDIR, False, False, "vit", 16, norm_eps=1e-6),
    5: BlockShape("llm-20b-stage", 12, 6144, 48, 8, 128, 16384, NORM_RMSNORM, MLP_SWIGLU,
                  MASK_CAUSAL, True, False, "llm", 32768, norm_eps=1e-6),
}


def small_shape(**kw) -> BlockShape:
    """A free-form small shape for unit tests."""
    base = dict(name="unit", n_blocks=1, hidden=64, n_q_heads=1, n_kv_heads=1, head_dim=64,
                mlp_dim=128, norm=NORM_LAYERNORM, mlp=MLP_GELU, mask=MASK_CAUSAL,
                use_rotary=False, has_bias=True, kind="tiny", budget=0)
    base.update(kw)
    return BlockShape(**base)


# ----------------------------------------------------------------------------------------------
# bf16 rounding (round-to-nearest-even) so that both sides start from identical values.
# ----------------------------------------------------------------------------------------------

def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Return float32 values that are exactly representable in bf16 (RNE)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of already-bf16-representable float32 values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


# ----------------------------------------------------------------------------------------------
# Synthetic dataset: per-sample tile count and LLM-side token count.
# ----------------------------------------------------------------------------------------------

def synthetic_dataset(n_samples: int = 20000, seed: int = 0):
    """Per-sample (tiles, llm_tokens) int32 arrays.

    tiles ~ TILE_PMF by inverse CDF; text ~ round(lognormal(median 300, sigma 1)) clipped to
    [1, 4096]; llm_tokens = 256 * tiles + text.
    """
    rng = np.random.default_rng([seed, 0x0B1])
    cdf = np.cumsum(np.asarray(TILE_PMF, dtype=np.float64))
    cdf[-1] = 1.0
    u = rng.random(n_samples)
    tiles = (np.searchsorted(cdf, u, side="right") + 1).astype(np.int32)
    tiles = np.minimum(tiles, MAX_TILES).astype(np.int32)
    z = rng.standard_normal(n_samples)
    text = np.rint(np.exp(np.log(TEXT_MEDIAN) + TEXT_SIGMA * z))
    text = np.clip(text, 1, TEXT_CAP).astype(np.int32)
    llm_tokens = (LLM_TOKENS_PER_TILE * tiles + text).astype(np.int32)
    return tiles, llm_tokens


def tiny_segment_lengths(seed: int = 0, n_seg: int = 4, lo: int = 64, hi: int = 384,
                         cap: int = 1024) -> np.ndarray:
    """Config-1 segment lengths: n_seg integer-uniform draws in [lo, hi]; all redrawn while
    their sum exceeds cap."""
    rng = np.random.default_rng([seed, 0x5E6])
    while True:
        lens = rng.integers(lo, hi + 1, size=n_seg)
        if int(lens.sum()) <= cap:
            return lens.astype(np.int32)


def lengths_to_cu(lens) -> np.ndarray:
    """Segment lengths -> int32 prefix offsets (a plain cumulative count, used by tests that
    need an arbitrary layout; the product's builders live in the library and in the oracle)."""
    lens = np.asarray(lens, dtype=np.int64)
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    return cu


# ----------------------------------------------------------------------------------------------
# Tensors.
# ----------------------------------------------------------------------------------------------

WEIGHT_NAMES = ("n1_g", "n1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                "n2_g", "n2_b", "w_up", "b_up", "w_down", "b_down")


def weight_shapes(shape: BlockShape) -> dict:
    H, F = shape.hidden, shape.mlp_dim
    out = {
        "n1_g": (H,), "w_qkv": (shape.d_qkv, H), "w_o": (H, shape.n_q_heads * shape.head_dim),
        "n2_g": (H,), "w_up": (shape.up_rows, H), "w_down": (H, F),
    }
    if shape.has_bias:
        out.update({"b_qkv": (shape.d_qkv,), "b_o": (H,), "b_up": (shape.up_rows,),
                    "b_down": (H,)})
        if shape.norm == NORM_LAYERNORM:
            out.update({"n1_b": (H,), "n2_b": (H,)})
    return out


def block_weights(shape: BlockShape, seed: int = 0, block: int = 0, std: float = 0.02) -> dict:
    """bf16-representable float32 weights: linear weights, biases and beta ~ N(0, std^2);
    gamma = 1 + N(0, std^2).  Absent tensors are omitted from the dict."""
    rng = np.random.default_rng([seed, 0xB10C, block])
    w = {}
    for name, shp in weight_shapes(shape).items():
        a = rng.standard_normal(shp, dtype=np.float32) * np.float32(std)
        if name in ("n1_g", "n2_g"):
            a = a + np.float32(1.0)
        w[name] = round_to_bf16(a)
    return w


def activations(total_tokens: int, hidden: int, seed: int = 0, std: float = 0.02):
    """x ~ N(0, std^2) and upstream gradient dy ~ N(0, 1), both bf16-representable float32."""
    rng = np.random.default_rng([seed, 0xAC7])
    x = round_to_bf16(rng.standard_normal((total_tokens, hidden), dtype=np.float32)
                      * np.float32(std))
    dy = round_to_bf16(rng.standard_normal((total_tokens, hidden), dtype=np.float32))
    return x, dy


def qkv_tensors(total_tokens: int, nq: int, nkv: int, d: int, seed: int = 0, std: float = 1.0):
    """q, k, v and upstream d_o for stand-alone attention tests (bf16-representable)."""
    rng = np.random.default_rng([seed, 0xA77])
    mk = lambda n: round_to_bf16(rng.standard_normal((total_tokens, n, d), dtype=np.float32)
                                 * np.float32(std))
    return mk(nq), mk(nkv), mk(nkv), mk(nq)


# ----------------------------------------------------------------------------------------------
# ViT -> LLM hand-over (sub-sampling + connector): weights and the visual rows of a packed batch
# ----------------------------------------------------------------------------------------------

CONNECTOR_NAMES = ("n_g", "n_b", "w1", "b1", "w2", "b2")


def connector_weights(vit_hidden: int, llm_hidden: int, seed: int = 0, std: float = 0.02) -> dict:
    """bf16-representable float32 weights: LayerNorm gain 1 + N(0, std^2) and beta over 4 Hv
    channels, W1 [Ht, 4 Hv], W2 [Ht, Ht], biases."""
    rng = np.random.default_rng([seed, 0xC0EC])
    W = 4 * vit_hidden
    shapes = {"n_g": (W,), "n_b": (W,), "w1": (llm_hidden, W), "b1": (llm_hidden,),
              "w2": (llm_hidden, llm_hidden), "b2": (llm_hidden,)}
    w = {}
    for name, shp in shapes.items():
        a = rng.standard_normal(shp, dtype=np.float32) * np.float32(std)
        if name == "n_g":
            a = a + np.float32(1.0)
        w[name] = round_to_bf16(a)
    return w


def visual_rows(tiles_per_sample, text_per_sample, tokens_per_tile: int = LLM_TOKENS_PER_TILE):
    """Rows of the packed LLM batch that hold visual tokens: each sample is laid out as its
    tiles' visual tokens followed by its text tokens.  Returns (dst_rows int32 [sum tiles *
    tokens_per_tile], cu int32 [n_samples + 1])."""
    rows, cu, pos = [], [0], 0
    for nt, tx in zip(tiles_per_sample, text_per_sample):
        nv = int(nt) * tokens_per_tile
        rows.append(np.arange(pos, pos + nv, dtype=np.int32))
        pos += nv + int(tx)
        cu.append(pos)
    return np.concatenate(rows) if rows else np.zeros(0, np.int32), np.asarray(cu, dtype=np.int32)
