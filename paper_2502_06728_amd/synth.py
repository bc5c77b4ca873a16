"""Seeded synthetic inputs for the optimizer hot path.

This module only *makes data*: shard sizes taken from model shapes, Gaussian tensors,
index/value payloads of valid structure.  It contains none of the optimizer's
arithmetic, so both the CPU oracle's tests and the GPU library's tests can feed the
same bytes to both sides.

The paper trains T5 on Opus Books, ViT-B/16 on CIFAR-100 and OLMo2-1B on Dolma
(sections "T5: Translation Task", "ViT: Image Classification", "OLMo2: Causal Language
Modeling").  The hot path never sees a dataset, only one rank's flat slice of the
parameters, its gradient and its momentum; the tensors below have those models'
shapes and sizes and stand in for them.

Every tensor is generated in independent blocks of ``BLOCK`` elements keyed by
(seed, tensor tag, block number), so any sub-range can be regenerated on the host
without materialising the whole array.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

BLOCK = 1 << 22  # elements per independently seeded block

TAG_GRAD, TAG_MOMENTUM, TAG_PARAMS, TAG_OUTLIER, TAG_PAY_IDX, TAG_PAY_VAL = 1, 2, 3, 4, 5, 6


# ----------------------------------------------------------------- shard sizes

def t5_base_params() -> int:
    d, ff, vocab = 768, 3072, 32128
    attn = 4 * d * d
    ffn = 2 * d * ff
    enc = attn + ffn + 2 * d
    dec = 2 * attn + ffn + 3 * d
    return vocab * d + 12 * enc + 12 * dec + 2 * d


def vit_b16_params() -> int:
    d, ff, classes, tokens = 768, 3072, 1000, 197
    patch = 3 * 16 * 16 * d + d
    block = 2 * d + (d * 3 * d + 3 * d) + (d * d + d) + 2 * d + (d * ff + ff) + (ff * d + d)
    return patch + d + tokens * d + 12 * block + 2 * d + (d * classes + classes)


def olmo_1b_params() -> int:
    d, ff, layers, vocab = 2048, 8192, 16, 50304
    return vocab * d + layers * (4 * d * d + 3 * d * ff)


def olmo_7b_params() -> int:
    d, ff, layers, vocab = 4096, 11008, 32, 50304
    return 2 * vocab * d + layers * (4 * d * d + 3 * d * ff)


def shard_len(total: int, world: int = 8, rank: int = 0) -> int:
    """Length of rank's contiguous slice when `total` elements are cut into `world`
    near-equal contiguous slices (earlier ranks take the remainder)."""
    base, rem = divmod(total, world)
    return base + (1 if rank < rem else 0)


@dataclass(frozen=True)
class Workload:
    """One of the benchmark configurations: shapes, dtypes and hyper-parameters."""
    name: str
    n: int
    chunk: int = 64
    topk: int = 32
    replicas: int = 1
    grad_bf16: bool = False
    params_bf16: bool = False
    grad_std: float = 1e-3
    momentum_std: float = 1e-3
    params_std: float = 0.02
    outlier_frac: float = 0.0
    outlier_scale: float = 100.0
    decay: float = 0.999
    lr: float = 1e-3
    weight_decay: float = 0.0
    sign: bool = True
    seed: int = 0
    extra: dict = field(default_factory=dict)


def workloads() -> dict[str, Workload]:
    return {
        "flat-1m": Workload("flat-1m", 1 << 20, chunk=64, topk=8, replicas=1),
        "t5-base-1of8": Workload("t5-base-1of8", shard_len(t5_base_params()), 64, 32, 2),
        "vit-b16-1of8": Workload("vit-b16-1of8", shard_len(vit_b16_params()), 64, 16, 2),
        "olmo-1b-1of8": Workload("olmo-1b-1of8", shard_len(olmo_1b_params()), 64, 32, 4,
                                 grad_bf16=True, params_bf16=True, outlier_frac=0.01),
        "olmo-7b-1of8": Workload("olmo-7b-1of8", shard_len(olmo_7b_params()), 64, 32, 4,
                                 grad_bf16=True, params_bf16=True),
    }


# --------------------------------------------------------------- block streams

def _rng(seed: int, tag: int, block: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) ^ tag, block]))


def _blocks(start: int, stop: int):
    b = start // BLOCK
    while b * BLOCK < stop:
        lo, hi = max(start, b * BLOCK), min(stop, (b + 1) * BLOCK)
        yield b, lo - b * BLOCK, hi - b * BLOCK
        b += 1


def normal(seed: int, tag: int, n: int, std: float, start: int = 0, stop: int | None = None,
           outlier_frac: float = 0.0, outlier_scale: float = 1.0) -> np.ndarray:
    """Elements [start, stop) of an n-element N(0, std^2) fp32 tensor; a seeded fraction
    of the entries is multiplied by `outlier_scale` (heavy tail)."""
    stop = n if stop is None else min(stop, n)
    out = np.empty(max(stop - start, 0), dtype=np.float32)
    pos = 0
    for b, lo, hi in _blocks(start, stop):
        x = _rng(seed, tag, b).standard_normal(BLOCK, dtype=np.float32)
        x *= np.float32(std)
        if outlier_frac > 0.0:
            u = _rng(seed, TAG_OUTLIER ^ (tag << 4), b).random(BLOCK, dtype=np.float32)
            x[u < outlier_frac] *= np.float32(outlier_scale)
        out[pos:pos + hi - lo] = x[lo:hi]
        pos += hi - lo
    return out


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16) with the library conversion of PyTorch."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> fp32 (exact widening)."""
    return (b.astype(np.uint32) << 16).view(np.float32)


def shard(w: Workload, seed_offset: int = 0, start: int = 0, stop: int | None = None):
    """(grad, momentum, params) for elements [start, stop) of workload `w`.
    bf16 tensors come back as uint16 bit patterns."""
    seed = w.seed + seed_offset
    g = normal(seed, TAG_GRAD, w.n, w.grad_std, start, stop, w.outlier_frac, w.outlier_scale)
    m = normal(seed, TAG_MOMENTUM, w.n, w.momentum_std, start, stop)
    p = normal(seed, TAG_PARAMS, w.n, w.params_std, start, stop)
    if w.grad_bf16:
        g = to_bf16_bits(g)
    if w.params_bf16:
        p = to_bf16_bits(p)
    return g, m, p


def structured_payload(seed: int, n_chunks: int, chunk: int, topk: int, std: float,
                       c0: int = 0, c1: int | None = None):
    """A structurally valid payload for chunks [c0, c1): per chunk, k ascending distinct
    chunk-local indices (one drawn uniformly from each of k consecutive groups of
    floor(s/k) positions) and N(0, std^2) values.  Used where a full-size payload is
    needed without running either implementation's compress.  Chunk-block keyed, so
    sub-ranges regenerate independently."""
    c1 = n_chunks if c1 is None else min(c1, n_chunks)
    cb = max(BLOCK // chunk, 1)  # chunks per block
    group = chunk // topk
    idx_parts, val_parts = [], []
    b = c0 // cb
    while b * cb < c1:
        lo, hi = max(c0, b * cb) - b * cb, min(c1, (b + 1) * cb) - b * cb
        r = _rng(seed, TAG_PAY_IDX, b)
        idx = r.integers(0, group, size=(cb, topk), dtype=np.int32)
        idx += (np.arange(topk, dtype=np.int32) * group)[None, :]
        val = _rng(seed, TAG_PAY_VAL, b).standard_normal((cb, topk), dtype=np.float32)
        val *= np.float32(std)
        idx_parts.append(idx[lo:hi])
        val_parts.append(val[lo:hi])
        b += 1
    if not idx_parts:
        return np.empty(0, np.int32), np.empty(0, np.float32)
    return (np.concatenate(idx_parts).reshape(-1), np.concatenate(val_parts).reshape(-1))
