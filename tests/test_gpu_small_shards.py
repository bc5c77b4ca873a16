"""The compress half at chunk size 64 and 128 picks its kernels by shard size (include/detonation.h,
DETO_SMALL_SHARD_TILES): a small shard spreads every 64-chunk tile over more wavefronts (chunk 64:
two coefficient classes instead of a lane per chunk; chunk 128: four classes instead of two).
Both choices against the oracle on the same inputs: every k family, bf16 and fp32 storage,
partial tiles with a ragged last chunk, ties."""
import numpy as np
import pytest

from oracle import Config
from tests.test_gpu_parity import H, full_step, tie_case  # noqa: F401  (H: the fixture)

pytestmark = pytest.mark.gpu

CHOICES = {"large-shard kernels": "0", "small-shard kernels": "1000000000"}


@pytest.fixture(params=list(CHOICES))
def choice(request, monkeypatch):
    monkeypatch.setenv("DETO_SMALL_SHARD_TILES", CHOICES[request.param])
    return request.param


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("s,k", [(64, 1), (64, 4), (64, 16), (64, 32), (64, 5), (64, 7), (64, 20),
                                 (128, 1), (128, 4), (128, 16), (128, 64), (128, 6), (128, 30)])
def test_both_kernel_choices(H, choice, s, k, bf16):
    # 9 full tiles, then a partial tile of 37 chunks and a ragged one
    n = s * (64 * 9 + 37) + s // 3
    cfg = Config(chunk=s, topk=k, sign=True)
    full_step(H, cfg, n, R=2, seed=s + k, grad_bf16=bf16, params_bf16=bf16,
              outliers=0.01 if bf16 else 0.0)


@pytest.mark.parametrize("s,k", [(64, 16), (64, 32), (128, 16), (128, 64)])
@pytest.mark.parametrize("tail", ["63 chunks and a ragged one", "a ragged one only", "one chunk",
                                  "63 chunks", "none"])
def test_partial_tiles(H, choice, s, k, tail):
    extra = {"63 chunks and a ragged one": 63 * s + s // 2 + 1, "a ragged one only": s - 3,
             "one chunk": s, "63 chunks": 63 * s, "none": 0}[tail]
    n = s * 64 * 2 + extra
    cfg = Config(chunk=s, topk=k, sign=True)
    full_step(H, cfg, n, R=3, seed=s + k)


@pytest.mark.parametrize("s,k", [(64, 1), (64, 8), (64, 16), (64, 32), (64, 13), (128, 16), (128, 64)])
def test_ties(H, choice, s, k):
    tie_case(H, s, k)


def test_default_limit_is_between_the_benchmark_shards(H, monkeypatch):
    """With the variable unset the ViT-B/16 and T5-base shards (2,641 and 6,802 tiles at chunk
    64) count as small and the OLMo shards (35,912 and up) as large; either way the results are
    the oracle's.  (Which kernel ran does not show in the results: the kernel traces under
    profiles/ name them.)"""
    monkeypatch.delenv("DETO_SMALL_SHARD_TILES", raising=False)
    cfg = Config(chunk=64, topk=16, sign=True)
    full_step(H, cfg, 64 * (64 * 30 + 5) + 7, R=2, seed=5)


def _random_shapes():
    """Seeded shapes over the chunk sizes of the wavefront-per-class kernels: any k up to the chunk
    size, shard lengths with every kind of tail (none, whole chunks, a ragged chunk, fewer
    chunks than one tile), R, storage type."""
    rng = np.random.default_rng(20250206728)
    shapes = []
    for i in range(48):
        s = int(rng.choice([64, 96, 128, 192, 256]))
        k = int(rng.integers(1, s + 1)) if i % 4 == 0 else int(rng.integers(1, s // 2 + 1))
        tiles = int(rng.integers(0, 4))
        tail_chunks = int(rng.integers(0, 64))
        ragged = int(rng.integers(0, s)) if i % 3 else 0
        n = s * (64 * tiles + tail_chunks) + ragged
        if n == 0:
            n = s + 1
        shapes.append((s, k, n, int(rng.integers(1, 6)), bool(i % 2)))
    return shapes


@pytest.mark.parametrize("s,k,n,R,bf16", _random_shapes())
def test_random_shapes(H, choice, s, k, n, R, bf16):
    cfg = Config(chunk=s, topk=k, sign=bool(k % 2))
    full_step(H, cfg, n, R=R, seed=n % 1000, grad_bf16=bf16, params_bf16=bf16,
              outliers=0.01 if bf16 else 0.0)
