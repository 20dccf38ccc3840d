"""Seeded synthetic workloads for the segmented multi-LoRA path.

This module only *draws inputs*: token/adapter structure and bf16 tensors of the
shapes the paper's setting implies (Llama-3-8B projections with grouped-query
attention, LoRA on all seven projections, a few adapters, batches ordered
fine-tune | prefill+evaluation | decode as in Algorithm 1).  It contains none of
the method's arithmetic and is shared by the tests, the benchmark, the CPU
oracle's callers and the GPU path's callers, so that both sides see identical bits.

All floating point inputs are drawn in fp32 from numpy's PCG64 generator and
rounded once to bfloat16 (round to nearest even); the rounded bit patterns
(uint16) are what every consumer receives.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

KIND_FINETUNE = 0
KIND_PREFILL = 1  # evaluation requests share this kind (Section 3.3)
KIND_DECODE = 2


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit pattern (uint16), round to nearest even.  Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit pattern (uint16) -> fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def normal_bf16(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(std))


@dataclass
class Batch:
    """Token structure of one mixed batch (no tensors)."""
    token_adapter: np.ndarray  # int32[T], -1 = no adapter (row left untouched)
    token_kind: np.ndarray     # uint8[T]
    name: str = ""

    @property
    def n_tokens(self) -> int:
        return int(self.token_adapter.shape[0])


@dataclass
class Problem:
    """One call of the path: one linear layer's LoRA update over one batch."""
    name: str
    d_in: int
    d_out: int
    ranks: np.ndarray            # int32[n_adapters]
    scales: np.ndarray           # float32[n_adapters]
    A: List[np.ndarray]          # per adapter uint16[r, d_in]   (bf16 bits)
    B: List[np.ndarray]          # per adapter uint16[r, d_out]  (bf16 bits)
    x: np.ndarray                # uint16[T, d_in]
    y0: np.ndarray               # uint16[T, d_out]
    batch: Batch
    dy: Optional[np.ndarray] = None  # uint16[T, d_out], only for the backward workload
    meta: dict = field(default_factory=dict)

    @property
    def n_tokens(self) -> int:
        return self.batch.n_tokens

    @property
    def n_adapters(self) -> int:
        return int(self.ranks.shape[0])


# ----------------------------------------------------------------------------------------------
# batch structures
# ----------------------------------------------------------------------------------------------

def _concat_batch(parts, name) -> Batch:
    ad = np.concatenate([np.asarray(p[0], dtype=np.int32) for p in parts]) if parts else np.zeros(0, np.int32)
    kd = np.concatenate([np.asarray(p[1], dtype=np.uint8) for p in parts]) if parts else np.zeros(0, np.uint8)
    return Batch(ad.astype(np.int32), kd.astype(np.uint8), name)


def _run(adapter: int, kind: int, n: int):
    return (np.full(n, adapter, np.int32), np.full(n, kind, np.uint8))


def batch_tiny(rng) -> Batch:
    """Config 1: 64 fine-tune tokens on adapter 0, 32 prefill tokens on adapter 1, 6 decode tokens over {0..3}."""
    dec = rng.integers(0, 4, size=6)
    parts = [_run(0, KIND_FINETUNE, 64), _run(1, KIND_PREFILL, 32),
             (dec.astype(np.int32), np.full(6, KIND_DECODE, np.uint8))]
    return _concat_batch(parts, "tiny")


def batch_decode_heavy(rng, n_tokens=256, n_adapters=64) -> Batch:
    """Config 2: decode tokens only, adapter id uniform over the pool."""
    ad = rng.integers(0, n_adapters, size=n_tokens)
    return Batch(ad.astype(np.int32), np.full(n_tokens, KIND_DECODE, np.uint8), "decode_heavy")


def batch_unified(rng) -> Batch:
    """Config 3: 2 fine-tune sequences of 2048 (adapters 0, 1), 8 prefills of 64 (adapters 2..9),
    256 decode tokens uniform over a pool of 32 adapters."""
    parts = [_run(0, KIND_FINETUNE, 2048), _run(1, KIND_FINETUNE, 2048)]
    parts += [_run(2 + i, KIND_PREFILL, 64) for i in range(8)]
    dec = rng.integers(0, 32, size=256)
    parts.append((dec.astype(np.int32), np.full(256, KIND_DECODE, np.uint8)))
    return _concat_batch(parts, "unified")


def zipf_lengths(rng, total: int, s: float = 1.2, cap: int = 1024) -> np.ndarray:
    """Segment lengths from the truncated Zipf pmf P(L=k) ~ k^-s, k = 1..cap, drawn by inverse CDF
    until they cover `total` tokens; the last one is trimmed."""
    k = np.arange(1, cap + 1, dtype=np.float64)
    cdf = np.cumsum(k ** (-s))
    cdf /= cdf[-1]
    out, acc = [], 0
    while acc < total:
        L = int(np.searchsorted(cdf, rng.random(), side="left")) + 1
        L = min(L, total - acc)
        out.append(L)
        acc += L
    return np.asarray(out, dtype=np.int64)


def batch_zipf(rng, total=8192, n_adapters=32, finetune_frac=0.10) -> Batch:
    """Config 4: Zipf(1.2) segment lengths capped at 1024, adapter uniform per segment; segments are
    marked fine-tune (in a shuffled order) until >= 10 % of the tokens are covered, the rest are
    decode (length 1) or prefill.  Emitted in the order fine-tune | prefill | decode."""
    lens = zipf_lengths(rng, total)
    n = len(lens)
    adapters = rng.integers(0, n_adapters, size=n)
    order = rng.permutation(n)
    kinds = np.where(lens == 1, KIND_DECODE, KIND_PREFILL).astype(np.uint8)
    covered = 0
    for i in order:
        if covered >= finetune_frac * total:
            break
        kinds[i] = KIND_FINETUNE
        covered += int(lens[i])
    parts = []
    for kind in (KIND_FINETUNE, KIND_PREFILL, KIND_DECODE):
        for i in range(n):
            if kinds[i] == kind:
                parts.append(_run(int(adapters[i]), kind, int(lens[i])))
    return _concat_batch(parts, "zipf")


def batch_layer_stack(rng) -> Batch:
    """Config 5: 4096 fine-tune tokens (2 x 2048 on adapters 0, 1), 1024 prefill tokens (16 x 64 on
    adapters 0..15), 512 decode tokens uniform over 16 adapters."""
    parts = [_run(0, KIND_FINETUNE, 2048), _run(1, KIND_FINETUNE, 2048)]
    parts += [_run(i, KIND_PREFILL, 64) for i in range(16)]
    dec = rng.integers(0, 16, size=512)
    parts.append((dec.astype(np.int32), np.full(512, KIND_DECODE, np.uint8)))
    return _concat_batch(parts, "layer_stack")


# ----------------------------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------------------------

def make_problem(name: str, batch: Batch, d_in: int, d_out: int, ranks, scales, seed: int,
                 with_dy: bool = False, y0_zero: bool = False, w_std: float = 0.02) -> Problem:
    rng = np.random.default_rng(seed)
    ranks = np.asarray(ranks, dtype=np.int32)
    scales = np.asarray(scales, dtype=np.float32)
    A = [normal_bf16(rng, (int(r), d_in), w_std) for r in ranks]
    B = [normal_bf16(rng, (int(r), d_out), w_std) for r in ranks]
    T = batch.n_tokens
    x = normal_bf16(rng, (T, d_in), 1.0)
    y0 = np.zeros((T, d_out), np.uint16) if y0_zero else normal_bf16(rng, (T, d_out), 1.0)
    dy = normal_bf16(rng, (T, d_out), 1.0) if with_dy else None
    return Problem(name, d_in, d_out, ranks, scales, A, B, x, y0, batch, dy)


LAYER_PROJECTIONS = (  # Llama-3-8B decoder layer with grouped-query attention: name, d_in, d_out
    ("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
    ("gate", 4096, 14336), ("up", 4096, 14336), ("down", 14336, 4096),
)
N_LAYERS = 32


def config_seed(config: int, layer: int = 0, projection: int = 0) -> int:
    return 1000 * config + 10 * layer + projection


def config1(y0_zero=False) -> Problem:
    rng = np.random.default_rng(config_seed(1) + 500)
    return make_problem("cfg1_tiny", batch_tiny(rng), 256, 256, [8] * 4, [2.0] * 4, config_seed(1), y0_zero=y0_zero)


def config2(y0_zero=False, seed_offset=0) -> Problem:
    rng = np.random.default_rng(config_seed(2) + 500 + seed_offset)
    return make_problem("cfg2_decode_heavy", batch_decode_heavy(rng), 4096, 4096, [16] * 64, [32.0 / 16] * 64,
                        config_seed(2) + seed_offset, y0_zero=y0_zero)


def config3(y0_zero=False) -> Problem:
    rng = np.random.default_rng(config_seed(3) + 500)
    return make_problem("cfg3_unified", batch_unified(rng), 4096, 4096, [16] * 32, [2.0] * 32, config_seed(3),
                        y0_zero=y0_zero)


def config4(which: str = "up", y0_zero=False) -> Problem:
    rng = np.random.default_rng(config_seed(4) + 500)
    batch = batch_zipf(rng)
    ranks = [(8, 16, 32, 64)[i % 4] for i in range(32)]
    scales = [32.0 / r for r in ranks]
    d_in, d_out = (4096, 11008) if which == "up" else (11008, 4096)
    return make_problem("cfg4_mlp_" + which, batch, d_in, d_out, ranks, scales,
                        config_seed(4, 0, 0 if which == "up" else 1), y0_zero=y0_zero)


def config5_batch() -> Batch:
    return batch_layer_stack(np.random.default_rng(config_seed(5) + 500))


def config5(layer: int, projection: int, with_dy=True, y0_zero=False, batch: Optional[Batch] = None) -> Problem:
    """One (layer, projection) call of the 32-layer stack; the batch structure is shared by all 224 calls."""
    name, d_in, d_out = LAYER_PROJECTIONS[projection]
    batch = batch if batch is not None else config5_batch()
    return make_problem(f"cfg5_L{layer}_{name}", batch, d_in, d_out, [32] * 16, [2.0] * 16,
                        config_seed(5, layer, projection), with_dy=with_dy, y0_zero=y0_zero)


def small_mixed(seed: int, T: int, d_in: int, d_out: int, ranks, n_kinds: int = 3, drop_frac: float = 0.0,
                scales=None, y0_zero=False, with_dy=False, w_std: float = 0.02) -> Problem:
    """Free-form small problem for unit tests: per-token adapter and kind uniform at random
    (so segments are ragged and appear in arbitrary order), optionally some tokens with no adapter."""
    rng = np.random.default_rng(seed)
    ranks = np.asarray(ranks, dtype=np.int32)
    n_ad = len(ranks)
    ad = rng.integers(0, n_ad, size=T).astype(np.int32)
    if drop_frac > 0:
        ad[rng.random(T) < drop_frac] = -1
    kd = rng.integers(0, n_kinds, size=T).astype(np.uint8)
    if scales is None:
        scales = rng.uniform(0.25, 4.0, size=n_ad)
    return make_problem(f"small_{seed}", Batch(ad, kd, "small"), d_in, d_out, ranks, scales, seed + 77,
                        y0_zero=y0_zero, with_dy=with_dy, w_std=w_std)
