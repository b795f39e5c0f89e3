"""Seeded synthetic inputs for the freeze-aware stage backward and the masked
optimizer pass.  numpy only; holds no arithmetic of the method itself: shapes,
random draws, the bf16 storage format, and mask/permutation draws.  The same
bytes produced here are handed to the fp64 CPU oracle (exactly up-cast) and to
the HIP library.

The inputs take the SHAPES of the paper's LLaMA fine-tuning workloads
(Table exp_setup: LLaMA-3.2-1B / LLaMA-3-8B split over 4 pipeline stages) and
stand in for its datasets and pretrained weights, which are not available.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

SEED_BASE = 260205754

# random streams
S_W, S_X, S_DY, S_MASK, S_GRAD, S_RATIO, S_BITS, S_STATE = range(8)


def rng(cfg_id: int, stream: int, layer: int = 0, microbatch: int = 0) -> np.random.Generator:
    """Independent PCG64 stream per (config, stream, layer, microbatch)."""
    ss = np.random.SeedSequence([SEED_BASE, int(cfg_id), int(stream), int(layer), int(microbatch)])
    return np.random.Generator(np.random.PCG64(ss))


@dataclass(frozen=True)
class StageConfig:
    cfg_id: int
    name: str
    blocks: int
    d: int
    kv: int          # total K/V projection width (n_kv_heads * head_dim)
    ffn: int
    T: int           # tokens per backward call (microbatch * seq)
    dtype: str       # "f32" or "bf16": storage type of W, X, dY, dX
    dw_dtype: str    # storage type of dW
    w_std: float = 0.02
    x_std: float = 1.0
    dy_std: float = 1e-3
    g_std: float = 1e-3
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1
    ema_decay: float = 0.99
    microbatches: int = 1

    @property
    def block_shapes(self) -> List[Tuple[int, int]]:
        d, kv, f = self.d, self.kv, self.ffn
        # (in_features K, out_features N) for q, k, v, o, gate, up, down
        return [(d, d), (d, kv), (d, kv), (d, d), (d, f), (d, f), (f, d)]

    @property
    def shapes(self) -> List[Tuple[int, int]]:
        return self.block_shapes * self.blocks

    @property
    def n_layers(self) -> int:
        return 7 * self.blocks

    @property
    def n_params(self) -> int:
        return sum(k * n for k, n in self.shapes)


LAYER_NAMES = ["q", "k", "v", "o", "gate", "up", "down"]

CONFIGS = {
    # tiny LLaMA-style stage, fp32, CPU oracle in seconds
    1: StageConfig(1, "tiny-f32", blocks=2, d=256, kv=256, ffn=688, T=2 * 128,
                   dtype="f32", dw_dtype="f32"),
    # LLaMA-1B-shaped stage, bf16 with fp32 master weights / Adam states
    2: StageConfig(2, "llama1b-stage-bf16", blocks=4, d=2048, kv=512, ffn=8192, T=4 * 2048,
                   dtype="bf16", dw_dtype="bf16"),
    # LLaMA-8B-shaped single stage (one of 4 stages of a 32-layer model)
    3: StageConfig(3, "llama8b-stage-bf16", blocks=8, d=4096, kv=1024, ffn=14336, T=1 * 4096,
                   dtype="bf16", dw_dtype="bf16", dy_std=1e-4),
    # same tensors, elementwise pass only
    4: StageConfig(4, "llama8b-elementwise", blocks=8, d=4096, kv=1024, ffn=14336, T=0,
                   dtype="bf16", dw_dtype="bf16"),
    # 8 microbatches of 1x1024, fp32 dW accumulators
    5: StageConfig(5, "llama8b-1f1b-8mb", blocks=8, d=4096, kv=1024, ffn=14336, T=1024,
                   dtype="bf16", dw_dtype="f32", dy_std=1e-4, microbatches=8),
}

R_SWEEP = {1: [0.5], 2: [0.0, 0.25, 0.5, 0.75, 0.9], 3: [0.0, 0.5, 0.9], 4: [0.3, 0.7],
           5: [0.2, 0.4, 0.6, 0.8]}


def scaled(cfg: StageConfig, **kw) -> StageConfig:
    """A copy of cfg with some fields replaced (reduced-size parity cases)."""
    from dataclasses import replace
    return replace(cfg, **kw)


# ----------------------------------------------------------------------------
# bf16 storage format (1-8-7, the upper half of an IEEE binary32)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even binary32 -> bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) >> 16).astype(np.uint16)
    r[nan] = ((u[nan] >> 16) | 0x0040).astype(np.uint16)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


def _normal(g: np.random.Generator, shape, std: float, dtype: str) -> np.ndarray:
    a = g.standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    if dtype == "bf16":
        a = round_to_bf16(a)
    return a


# ----------------------------------------------------------------------------
# stage-backward inputs
# ----------------------------------------------------------------------------
def gen_weight(cfg: StageConfig, l: int) -> np.ndarray:
    """Master weight of layer l, float32 [K, N], N(0, w_std^2)."""
    K, N = cfg.shapes[l]
    return _normal(rng(cfg.cfg_id, S_W, l), (K, N), cfg.w_std, "f32")


def gen_layer(cfg: StageConfig, l: int, T: Optional[int] = None, microbatch: int = 0):
    """(W, X, dY) of layer l as float32 arrays holding values representable in
    cfg.dtype.  W is the stored (low-precision) copy of gen_weight."""
    K, N = cfg.shapes[l]
    T = cfg.T if T is None else T
    W = gen_weight(cfg, l)
    if cfg.dtype == "bf16":
        W = round_to_bf16(W)
    X = _normal(rng(cfg.cfg_id, S_X, l, microbatch), (T, K), cfg.x_std, cfg.dtype)
    dY = _normal(rng(cfg.cfg_id, S_DY, l, microbatch), (T, N), cfg.dy_std, cfg.dtype)
    return W, X, dY


def gen_grad(cfg: StageConfig, l: int, step: int, dtype: str = "bf16") -> np.ndarray:
    """Synthetic gradient of layer l for optimizer step `step`, N(0, g_std^2)."""
    K, N = cfg.shapes[l]
    return _normal(rng(cfg.cfg_id, S_GRAD, l, step), (K * N,), cfg.g_std, dtype)


def gen_state(cfg: StageConfig, l: int):
    """Non-zero optimizer / stability state (m, v, E, A) for timing a step that
    is not the first: plausible magnitudes, v and A non-negative."""
    K, N = cfg.shapes[l]
    g = rng(cfg.cfg_id, S_STATE, l)
    n = K * N
    m = _normal(g, (n,), cfg.g_std * 0.3, "f32")
    v = np.square(_normal(g, (n,), cfg.g_std, "f32"))
    E = _normal(g, (n,), cfg.lr * 0.1, "f32")
    A = np.abs(_normal(g, (n,), cfg.lr, "f32")) + np.abs(E)
    return m, v, E, A


# ----------------------------------------------------------------------------
# masks
# ----------------------------------------------------------------------------
def n_frozen_tensors(r: float, L: int) -> int:
    """Tensor count frozen at ratio r: ceil(r*L) (guarded against float fuzz)."""
    return max(0, min(L, int(math.ceil(r * L - 1e-9))))


def permutation_mask(cfg: StageConfig, r: float, microbatch: int = 0, L: Optional[int] = None) -> np.ndarray:
    """Tensor-granular freeze mask (uint8, 1 = frozen): the first ceil(r L)
    entries of a seeded permutation of the L tensors."""
    L = cfg.n_layers if L is None else L
    perm = rng(cfg.cfg_id, S_MASK, 0, microbatch).permutation(L)
    mask = np.zeros(L, dtype=np.uint8)
    mask[perm[: n_frozen_tensors(r, L)]] = 1
    return mask


def microbatch_ratios(cfg: StageConfig, choices=(0.2, 0.4, 0.6, 0.8)) -> List[float]:
    g = rng(cfg.cfg_id, S_RATIO)
    return [float(x) for x in g.choice(np.asarray(choices), size=cfg.microbatches)]


def bernoulli_elem_mask(cfg: StageConfig, l: int, numel: int, r: float) -> np.ndarray:
    """Element-granular freeze mask: uint8 per element, 1 = frozen w.p. r."""
    g = rng(cfg.cfg_id, S_BITS, l)
    return (g.random(numel, dtype=np.float32) < np.float32(r)).astype(np.uint8)


def pack_mask_bits(mask_u8: np.ndarray) -> np.ndarray:
    """uint8-per-element mask -> uint32 words, element j at bit (j & 31) of
    word (j >> 5); the tail of the last word is zero (= not frozen)."""
    n = mask_u8.size
    nw = (n + 31) // 32
    padded = np.zeros(nw * 32, dtype=np.uint8)
    padded[:n] = mask_u8
    b = np.packbits(padded.reshape(nw, 4, 8), axis=-1, bitorder="little").reshape(nw, 4)
    return (b[:, 0].astype(np.uint32) | (b[:, 1].astype(np.uint32) << 8)
            | (b[:, 2].astype(np.uint32) << 16) | (b[:, 3].astype(np.uint32) << 24))


def frozen_param_fraction(cfg: StageConfig, mask: np.ndarray) -> float:
    """phi = sum over frozen tensors of K*N / P (fraction of dW FLOPs skipped)."""
    sh = cfg.shapes
    return sum(sh[l][0] * sh[l][1] for l in range(len(mask)) if mask[l]) / float(
        sum(k * n for k, n in sh[: len(mask)]))
