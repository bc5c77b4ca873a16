"""The seeded input generator: shard sizes of the benchmark configurations, block-keyed
reproducibility (any sub-range regenerates on its own), value statistics of the recipe."""
import numpy as np

from paper_2502_06728_amd import synth


def test_shard_sizes_of_the_benchmark_configurations():
    w = synth.workloads()
    assert synth.t5_base_params() == 222_902_784 and w["t5-base-1of8"].n == 27_862_848
    assert synth.vit_b16_params() == 86_567_656 and w["vit-b16-1of8"].n == 10_820_957
    assert synth.olmo_1b_params() == 1_176_764_416 and w["olmo-1b-1of8"].n == 147_095_552
    assert synth.olmo_7b_params() == 6_888_095_744 and w["olmo-7b-1of8"].n == 861_011_968
    assert w["flat-1m"].n == 1 << 20
    # the eight ranks' slices tile the flat parameter list
    total = synth.vit_b16_params()
    assert sum(synth.shard_len(total, 8, r) for r in range(8)) == total


def test_sub_ranges_regenerate_independently():
    n = 3 * synth.BLOCK + 12345
    full = synth.normal(7, synth.TAG_GRAD, n, 1e-3, outlier_frac=0.01, outlier_scale=100.0)
    for a, b in [(0, 100), (synth.BLOCK - 5, synth.BLOCK + 5), (2 * synth.BLOCK + 1, n), (n - 1, n)]:
        part = synth.normal(7, synth.TAG_GRAD, n, 1e-3, a, b, outlier_frac=0.01, outlier_scale=100.0)
        assert np.array_equal(part, full[a:b])
    other = synth.normal(8, synth.TAG_GRAD, n, 1e-3)
    assert not np.array_equal(other[:1000], full[:1000])
    assert not np.array_equal(synth.normal(7, synth.TAG_MOMENTUM, 1000, 1e-3), full[:1000])


def test_recipe_statistics():
    w = synth.Workload("t", 1 << 21, grad_bf16=True, params_bf16=True, outlier_frac=0.01)
    g, m, p = synth.shard(w)
    assert g.dtype == np.uint16 and p.dtype == np.uint16 and m.dtype == np.float32
    gf = synth.from_bf16_bits(g).astype(np.float64)
    assert abs(m.std() - 1e-3) < 2e-5 and abs(synth.from_bf16_bits(p).std() - 0.02) < 4e-4
    big = np.abs(gf) > 8e-3                       # beyond 8 sigma of the bulk: the x100 outliers
    assert 0.006 < big.mean() < 0.011
    assert abs(np.median(np.abs(gf)) / 1e-3 - 0.6745) < 0.02


def test_structured_payload_is_valid_and_block_keyed():
    C, s, k = 100_000, 64, 32
    idx, val = synth.structured_payload(3, C, s, k, 1e-3)
    idx = idx.reshape(C, k)
    assert idx.min() >= 0 and idx.max() < s and (np.diff(idx, axis=1) > 0).all()
    i2, v2 = synth.structured_payload(3, C, s, k, 1e-3, 70_000, 70_010)
    assert np.array_equal(i2, idx[70_000:70_010].ravel())
    assert np.array_equal(v2, val.reshape(C, k)[70_000:70_010].ravel())
    assert abs(val.std() - 1e-3) < 2e-5
