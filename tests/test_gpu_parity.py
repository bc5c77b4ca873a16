"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the
same seeded inputs (staged protocol of tests/parity.py)."""
import numpy as np
import pytest

import oracle
from oracle import Config, SCHEME_RANDOM, SCHEME_STRIDE, SCHEME_TOPK
from paper_2502_06728_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H(gpu):
    from tests import gpu_harness
    from paper_2502_06728_amd import binding
    binding.load()
    return gpu_harness


def make_inputs(n, seed=0, grad_bf16=False, params_bf16=False, outliers=0.0):
    w = synth.Workload("t", n, grad_bf16=grad_bf16, params_bf16=params_bf16,
                       outlier_frac=outliers, seed=seed)
    return synth.shard(w)


def full_step(H, cfg, n, R=1, seed=0, grad_bf16=False, params_bf16=False, outliers=0.0):
    """One whole step on both sides.  Replica 0's payload is the shard's own; replicas
    1..R-1 come from the oracle's compress on independently seeded shards."""
    g, m, th = make_inputs(n, seed, grad_bf16, params_bf16, outliers)
    send_idx = cfg.scheme == SCHEME_TOPK
    m_gpu, idx_gpu, val_gpu, coeff_gpu = H.gpu_compress(cfg, g, m, want_idx=send_idx)
    st_c = parity.check_compress(cfg, g, m, m_gpu, idx_gpu, val_gpu, coeff_gpu)
    # payloads for the decompress half: all produced by the oracle
    pays = []
    for r in range(R):
        gr, mr, _ = make_inputs(n, seed + 1000 * r, grad_bf16, params_bf16, outliers)
        _, i_r, v_r = oracle.compress(cfg, gr, mr)
        pays.append((i_r, v_r))
    idx = np.stack([p[0] for p in pays]) if send_idx else None
    val = np.stack([p[1] for p in pays])
    th_gpu, y_gpu = H.gpu_decompress(cfg, idx, val, th)
    st_d = parity.check_decompress(cfg, idx, val, th, th_gpu, y_gpu)
    return st_c, st_d


def test_config0_flat_1m(H):
    cfg = Config(chunk=64, topk=8, decay=0.999, lr=1e-3, sign=True)
    st_c, st_d = full_step(H, cfg, 1 << 20, R=1, seed=0)
    assert st_c["chunks"] == 16384
    print(st_c, st_d)


@pytest.mark.parametrize("sign", [True, False])
@pytest.mark.parametrize("s,k", [(32, 1), (32, 4), (32, 16), (64, 1), (64, 4), (64, 16), (64, 32),
                                 (128, 1), (128, 4), (128, 16), (128, 64)])
def test_vit_like_sweep_ragged(H, s, k, sign):
    # the ViT-B/16 shard length is not a multiple of 32 (tail of 29): same raggedness, smaller n
    n = 32 * 9000 + 29
    cfg = Config(chunk=s, topk=k, sign=sign)
    full_step(H, cfg, n, R=2, seed=s + k)


@pytest.mark.parametrize("s,k", [(16, 2), (96, 6), (96, 96), (192, 12), (256, 16), (256, 256),
                                 (1, 1), (2, 1), (3, 2), (65, 7), (200, 100), (128, 30), (192, 10),
                                 (192, 96), (192, 97), (256, 6), (256, 128), (256, 129), (96, 49),
                                 (192, 16), (192, 17), (192, 32), (192, 33)])
def test_other_chunk_sizes(H, s, k):
    cfg = Config(chunk=s, topk=k, sign=True)
    full_step(H, cfg, s * 700 + (s // 3), R=3, seed=3)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("s,k", [(96, 12), (128, 16), (128, 6), (192, 24), (256, 32), (256, 5)])
@pytest.mark.parametrize("tail", ["63 chunks and a ragged one", "a ragged one only", "one chunk",
                                  "63 chunks"])
def test_partial_tiles_above_chunk_64(H, s, k, tail, bf16):
    # the chunks past the last full 64-chunk tile form one partial tile; its last chunk may be
    # ragged, and with 63 complete chunks before it the partial tile has all 64 rows in use
    extra = {"63 chunks and a ragged one": 63 * s + s // 2 + 1, "a ragged one only": s - 3,
             "one chunk": s, "63 chunks": 63 * s}[tail]
    n = s * 64 * 2 + extra
    cfg = Config(chunk=s, topk=k, sign=True)
    full_step(H, cfg, n, R=3, seed=s + k, grad_bf16=bf16, params_bf16=bf16,
              outliers=0.01 if bf16 else 0.0)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("k", [1, 2, 3, 4, 8, 16])
def test_chunk_size_16(H, k, bf16):
    # the smallest chunk of the Appendix B sweep: lane-per-chunk kernels for k in {1,2,4,8}
    cfg = Config(chunk=16, topk=k, sign=True)
    full_step(H, cfg, 16 * (64 * 40 + 17) + 5, R=3, seed=k, grad_bf16=bf16, params_bf16=bf16,
              outliers=0.01 if bf16 else 0.0)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("k", [6, 12, 24, 48, 5, 96])
def test_chunk_size_96(H, k, bf16):
    # 96 = 3 * 32: lane-per-chunk kernels whose fast DCT ends in 3-point transforms
    # (k in {6, 12, 24, 48}); other k on the matrix-core kernels
    cfg = Config(chunk=96, topk=k, sign=True)
    full_step(H, cfg, 96 * (64 * 20 + 31) + 50, R=3, seed=k, grad_bf16=bf16, params_bf16=bf16,
              outliers=0.01 if bf16 else 0.0)


@pytest.mark.parametrize("s,k", [(96, 12), (128, 16), (128, 64), (128, 6), (192, 24), (192, 10),
                                 (256, 32), (256, 128), (256, 20)])
def test_ties_above_chunk_64(H, s, k):
    tie_case(H, s, k)


def tie_case(H, s, k):
    # zero chunks tie everywhere; single spikes give coefficients of pairwise equal magnitude;
    # chunks of +-1 patterns tie in groups.  Mixed with ordinary chunks in the same tiles, so
    # that the whole-wavefront tie pass and the staged path meet in one workgroup; a ragged tail.
    n = s * (64 * 3 + 17) + s // 2
    C = -(-n // s)
    cfg = Config(chunk=s, topk=k, decay=0.0)
    rng = np.random.default_rng(s + k)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    for c in range(0, C - 1, 3):
        g[c * s:(c + 1) * s] = 0.0
        if c % 2:
            g[c * s + (7 * c) % s] = 1.0 + c
    for c in range(1, C - 1, 11):
        g[c * s:(c + 1) * s] = np.where(np.arange(s) % 3 == 0, 1.0, -1.0)
    m = np.zeros(n, np.float32)
    m_gpu, idx_gpu, val_gpu, coeff_gpu = H.gpu_compress(cfg, g, m)
    parity.check_compress(cfg, g, m, m_gpu, idx_gpu, val_gpu, coeff_gpu)
    assert np.array_equal(idx_gpu.reshape(-1, k)[0], np.arange(k))      # an all-zero chunk


@pytest.mark.parametrize("grad_bf16,params_bf16", [(True, True), (True, False), (False, True)])
def test_bf16_storage_with_outliers(H, grad_bf16, params_bf16):
    cfg = Config(chunk=64, topk=32, sign=True)
    full_step(H, cfg, 64 * 20000 + 5, R=4, seed=7, grad_bf16=grad_bf16, params_bf16=params_bf16,
              outliers=0.01)


@pytest.mark.parametrize("scheme", [SCHEME_STRIDE, SCHEME_RANDOM])
@pytest.mark.parametrize("dct", [False, True])
@pytest.mark.parametrize("step", [0, 1, 2, 3])
def test_striding_and_random(H, scheme, dct, step):
    cfg = Config(chunk=64, topk=32, scheme=scheme, dct=dct, seed=42, step=step, sign=True)
    full_step(H, cfg, 64 * 6000 + 11, R=4, seed=step, grad_bf16=True, params_bf16=True)


@pytest.mark.parametrize("scheme", [SCHEME_STRIDE, SCHEME_RANDOM])
@pytest.mark.parametrize("s,k", [(32, 5), (128, 16), (96, 12), (256, 3)])
def test_striding_and_random_other_shapes(H, scheme, s, k):
    cfg = Config(chunk=s, topk=k, scheme=scheme, dct=(s == 128), seed=2**63 + 9, step=2**33 + 1,
                 sign=False)
    full_step(H, cfg, s * 900 + 1, R=2, seed=5)


@pytest.mark.parametrize("scheme", [SCHEME_STRIDE, SCHEME_RANDOM])
@pytest.mark.parametrize("dct", [False, True])
@pytest.mark.parametrize("s,k", [(64, 16), (64, 8), (32, 16), (32, 8), (32, 4), (32, 2), (32, 1),
                                 (64, 4), (64, 2), (64, 1), (16, 2), (16, 1)])
def test_striding_and_random_low_rates(H, scheme, dct, s, k):
    # the rates of the paper's experiments (chunk 32, k from 16 down to 1): lane-per-chunk kernels
    cfg = Config(chunk=s, topk=k, scheme=scheme, dct=dct, seed=77, step=s + k, sign=True)
    full_step(H, cfg, s * (64 * 30 + 9) + 3, R=3, seed=k, grad_bf16=(k % 2 == 0),
              params_bf16=(k % 2 == 0))


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("step", [0, 5, 2**40 + 3])
@pytest.mark.parametrize("s,k", [(128, 16), (256, 32), (256, 1), (96, 12), (48, 6), (100, 7), (64, 3),
                                 (200, 100), (7, 2), (1, 1), (192, 191)])
def test_striding_raw_domain_any_shape(H, s, k, step, bf16):
    """Striding keeps every n-th position whatever the values are: at shapes without a
    lane-per-chunk kernel a plain streaming kernel serves it.  Several workgroup spans, chunk
    boundaries inside a lane's span, k that does not divide s, a ragged last chunk."""
    cfg = Config(chunk=s, topk=k, scheme=SCHEME_STRIDE, seed=1, step=step, sign=(step != 5), lr=1e-3,
                 weight_decay=0.01 if step == 5 else 0.0)
    n = 2048 * 3 + 517 + s // 2
    full_step(H, cfg, n, R=3, seed=s + k, grad_bf16=bf16, params_bf16=bf16,
              outliers=0.01 if bf16 else 0.0)
    # the indices, when the caller asks for them
    g, m, _ = make_inputs(n, s + k, bf16, bf16, 0.01 if bf16 else 0.0)
    _, idx_gpu, _, _ = H.gpu_compress(cfg, g, m, want_idx=True)
    assert np.array_equal(idx_gpu, oracle.select(cfg, None, -(-n // s)))


@pytest.mark.parametrize("n", [1, 5, 63, 64, 65, 64 * 64, 64 * 64 + 1, 64 * 129 - 1])
def test_small_and_ragged_lengths(H, n):
    cfg = Config(chunk=64, topk=8)
    full_step(H, cfg, n, R=2, seed=n)


def test_zero_inputs_select_lowest_indices(H):
    # all magnitudes tie at zero: the rule keeps the k lowest indices; sign(0) = 0 moves nothing
    n, s, k = 64 * 300 + 7, 64, 8
    cfg = Config(chunk=s, topk=k)
    g = np.zeros(n, np.float32)
    m = np.zeros(n, np.float32)
    th = synth.normal(1, synth.TAG_PARAMS, n, 0.02)
    m_gpu, idx_gpu, val_gpu, coeff_gpu = H.gpu_compress(cfg, g, m)
    assert np.array_equal(idx_gpu.reshape(-1, k), np.tile(np.arange(k, dtype=np.int32), (301, 1)))
    assert not m_gpu.any() and not val_gpu.any()
    th_gpu, y = H.gpu_decompress(cfg, idx_gpu[None], val_gpu[None], th)
    assert np.array_equal(th_gpu, th)


def test_hand_built_ties(H):
    s, k = 64, 4
    # a chunk that is one DCT basis vector has a single large coefficient and the rest near 0;
    # an all-zero chunk ties everywhere and keeps the k lowest indices
    cfg = Config(chunk=s, topk=k, decay=0.0)
    D = oracle.dct_matrix(s)
    g = np.concatenate([D[5], -D[9], D[0], np.zeros(s)]).astype(np.float32)
    m = np.zeros_like(g)
    m_gpu, idx_gpu, val_gpu, coeff_gpu = H.gpu_compress(cfg, g, m)
    parity.check_compress(cfg, g, m, m_gpu, idx_gpu, val_gpu, coeff_gpu)
    assert 5 in idx_gpu[:k] and 9 in idx_gpu[k:2 * k] and 0 in idx_gpu[2 * k:3 * k]
    assert list(idx_gpu[3 * k:]) == [0, 1, 2, 3]


def test_k_equals_s_is_lossless_and_reduces_to_sgd_momentum(H):
    # nothing dropped, one replica, no sign: theta' = theta - eta*(beta*m + g)
    s, n = 64, 64 * 500
    cfg = Config(chunk=s, topk=s, sign=False, decay=0.9, lr=0.05)
    g, m, th = make_inputs(n, 11)
    m_gpu, idx_gpu, val_gpu, coeff_gpu = H.gpu_compress(cfg, g, m)
    m1 = 0.9 * m.astype(np.float64) + g
    assert np.abs(m_gpu).max() < 2e-6 * np.abs(m1).max()
    th_gpu, _ = H.gpu_decompress(cfg, idx_gpu[None], val_gpu[None], th)
    want = th.astype(np.float64) - np.float64(np.float32(0.05)) * (
        np.float64(np.float32(0.9)) * m.astype(np.float64) + g.astype(np.float64))
    assert np.abs(th_gpu - want).max() < 2e-6 * np.abs(want).max()


@pytest.mark.parametrize("R", [1, 2, 4, 7])
def test_replica_counts_weight_decay_and_strides(H, R):
    import torch
    from paper_2502_06728_amd import binding
    s, k, n = 64, 16, 64 * 3000 + 3
    cfg = Config(chunk=s, topk=k, sign=(R % 2 == 0), lr=1e-2, weight_decay=0.1)
    full_step(H, cfg, n, R=R, seed=R)
    # replica strides larger than the payload (an all_gather buffer with padding)
    entries = -(-n // s) * k
    stride = entries + 24
    pays = [oracle.compress(cfg, *make_inputs(n, 50 + r)[:2])[1:] for r in range(R)]
    idx = np.full((R, stride), 999, np.int32)
    val = np.full((R, stride), np.nan, np.float32)
    for r, (i_r, v_r) in enumerate(pays):
        idx[r, :entries], val[r, :entries] = i_r, v_r
    th = make_inputs(n, 77)[2]
    p = H.to_dev(th)
    y = torch.empty(n, dtype=torch.float32, device=H.DEV)
    binding.detonation_decompress_step(H.bcfg(cfg), R, H.to_dev(idx), H.to_dev(val), p, y,
                                       idx_replica_stride=stride, val_replica_stride=stride)
    torch.cuda.synchronize()
    parity.check_decompress(cfg, np.stack([q[0] for q in pays]), np.stack([q[1] for q in pays]),
                            th, H.to_host(p), H.to_host(y))


def test_duplicate_and_out_of_range_payload_indices(H):
    s, k, n = 64, 4, 64 * 50
    cfg = Config(chunk=s, topk=k, sign=False)
    rng = np.random.default_rng(0)
    idx = rng.integers(-3, s + 3, size=(2, 50 * k)).astype(np.int32)     # dups + out of range
    idx[0, :8] = [5, 5, 5, 5, 64, -1, 7, 7]
    val = rng.standard_normal((2, 50 * k)).astype(np.float32)
    th = make_inputs(n, 3)[2]
    th_gpu, y_gpu = H.gpu_decompress(cfg, idx, val, th)
    parity.check_decompress(cfg, idx, val, th, th_gpu, y_gpu)


def test_deterministic_and_debug_outputs_do_not_change_results(H):
    cfg = Config(chunk=64, topk=32)
    g, m, th = make_inputs(64 * 10000 + 17, 21, grad_bf16=True, params_bf16=True)
    a = H.gpu_compress(cfg, g, m, want_coeff=True)
    b = H.gpu_compress(cfg, g, m, want_coeff=False)
    c = H.gpu_compress(cfg, g, m, want_coeff=False)
    for x, y, z in zip(a[:3], b[:3], c[:3]):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
        assert np.array_equal(y.view(np.uint32), z.view(np.uint32))
    idx, val = np.stack([a[1]] * 3), np.stack([a[2]] * 3)
    p1, _ = H.gpu_decompress(cfg, idx, val, th, want_presign=True)
    p2, _ = H.gpu_decompress(cfg, idx, val, th, want_presign=False)
    assert np.array_equal(p1, p2)


@pytest.mark.size_dispatch
def test_t5_base_shard_full_size(H):
    # the T5-base-shaped 1/8 shard (27.9M parameters), chunk 64, top-k 32, R = 2
    w = synth.workloads()["t5-base-1of8"]
    assert w.n == 27_862_848
    cfg = Config(chunk=w.chunk, topk=w.topk, decay=w.decay, lr=w.lr, sign=True)
    st_c, st_d = full_step(H, cfg, w.n, R=2, seed=0)
    print(st_c, st_d)
    assert st_c["chunks"] == 435_357


@pytest.mark.size_dispatch
@pytest.mark.parametrize("sign", [True, False])
@pytest.mark.parametrize("s,k", [(s, k) for s in (32, 64, 128) for k in (1, 4, 16, s // 2)])
def test_vit_b16_shard_full_size(H, s, k, sign):
    # every point of the ViT-B/16 sweep (chunk x top-k x sign, R = 2) on the whole 10.8 M-parameter
    # shard, whose length is not a multiple of any of the chunk sizes
    w = synth.workloads()["vit-b16-1of8"]
    assert w.n == 10_820_957 and w.n % 32 == 29
    st_c, st_d = full_step(H, Config(chunk=s, topk=k, sign=sign, decay=w.decay, lr=w.lr), w.n,
                           R=2, seed=1)
    assert st_c["chunks"] == -(-w.n // s)


def _sample_runs(C, run=256, count=24, seed=5):
    """Chunk ranges to check at full size: the first and last tiles, the ragged end, and
    seeded random runs of `run` consecutive chunks."""
    rng = np.random.default_rng(seed)
    starts = [0, max(C - run, 0)] + [int(x) for x in rng.integers(0, max(C - run, 1), count)]
    return sorted({(s0, min(s0 + run, C)) for s0 in starts})


def _slabs(C, slab=65536):
    """Every chunk of the shard, in consecutive slabs that bound the oracle's host memory."""
    return [(c0, min(c0 + slab, C)) for c0 in range(0, C, slab)]


def _payload_indices(cfg, idx, R, c0, c1):
    """The index arrays the oracle is given for chunks [c0, c1): the transmitted ones, or, for
    Striding / Random, the oracle's own selection keyed by the chunks' global numbers (the same
    for every replica, since all replicas regenerate them from the shared seed and step)."""
    k = cfg.topk
    if idx is not None:
        return idx[:, c0 * k:c1 * k]
    own = oracle.select(cfg, None, c1 - c0, chunk0=c0)
    return np.tile(own, (R, 1))


def _full_size_check(H, w, cfg, ranges=None):
    """Parity at a benchmark configuration's full size, in the launch configuration bench.py
    times (debug outputs off).  `ranges` = chunk ranges handed to the oracle; by default every
    chunk of the shard, slab by slab, element by element."""
    s, k, R, n = cfg.chunk, cfg.topk, w.replicas, w.n
    C = -(-n // s)
    ranges = _slabs(C) if ranges is None else ranges
    g, m, th = synth.shard(w)
    send_idx = cfg.scheme == SCHEME_TOPK
    # the timed configuration: no debug outputs
    m_a, idx_a, val_a, _ = H.gpu_compress(cfg, g, m, want_idx=send_idx, want_coeff=False)
    # same call with the coefficient export, which must not change any result
    m_b, idx_b, val_b, coeff = H.gpu_compress(cfg, g, m, want_idx=send_idx, want_coeff=True)
    assert np.array_equal(m_a.view(np.uint32), m_b.view(np.uint32))
    assert np.array_equal(val_a.view(np.uint32), val_b.view(np.uint32))
    if send_idx:
        assert np.array_equal(idx_a, idx_b)
        assert idx_a.min() >= 0 and idx_a.max() < s
        assert (np.diff(idx_a.reshape(C, k), axis=1) > 0).all()        # holds at any size
    del m_b, val_b, idx_b
    worst = {"coeff": 0.0, "momentum": 0.0, "flips": 0, "chunks": 0}
    for c0, c1 in ranges:
        e0, e1 = c0 * s, min(c1 * s, n)
        st = parity.check_compress(cfg, g[e0:e1], m[e0:e1], m_a[e0:e1],
                                   idx_a[c0 * k:c1 * k] if send_idx else None,
                                   val_a[c0 * k:c1 * k], coeff[c0 * s:c1 * s], chunk0=c0)
        worst["coeff"] = max(worst["coeff"], st["coeff"])
        worst["momentum"] = max(worst["momentum"], st["momentum"])
        worst["flips"] += st["flips"]
        worst["chunks"] += st["chunks"]
    del m_a, coeff, g, m
    # decompress: R structurally valid payloads from the generator (not from either compress)
    idx = np.empty((R, C * k), np.int32) if send_idx else None
    val = np.empty((R, C * k), np.float32)
    for r in range(R):
        i_r, val[r] = synth.structured_payload(w.seed + 10 + r, C, s, k, w.momentum_std)
        if send_idx:
            idx[r] = i_r
    th_a, _ = H.gpu_decompress(cfg, idx, val, th, want_presign=False)
    th_b, y = H.gpu_decompress(cfg, idx, val, th, want_presign=True)
    assert np.array_equal(th_a, th_b)
    del th_b
    worst["presign"] = 0.0
    worst["sign_flips"] = 0
    for c0, c1 in ranges:
        e0, e1 = c0 * s, min(c1 * s, n)
        st = parity.check_decompress(cfg, _payload_indices(cfg, idx, R, c0, c1),
                                     val[:, c0 * k:c1 * k], th[e0:e1], th_a[e0:e1], y[e0:e1])
        worst["presign"] = max(worst["presign"], st["presign"])
        worst["sign_flips"] += st["sign_flips_vs_oracle"]
    return worst


@pytest.mark.size_dispatch
def test_olmo_1b_shard_full_size_bench_configuration(H):
    # the benchmark's workload: 147,095,552 parameters, bf16 grads/params with outliers,
    # chunk 64, top-k 32, R = 4
    w = synth.workloads()["olmo-1b-1of8"]
    assert w.n == 147_095_552
    cfg = Config(chunk=w.chunk, topk=w.topk, decay=w.decay, lr=w.lr, sign=w.sign)
    worst = _full_size_check(H, w, cfg)
    print("olmo-1b full size:", worst)
    assert worst["chunks"] == 2_298_368      # every chunk of the shard went through the oracle


@pytest.mark.size_dispatch
@pytest.mark.parametrize("scheme,dct", [(SCHEME_STRIDE, False), (SCHEME_RANDOM, False),
                                        (SCHEME_STRIDE, True)])
def test_olmo_1b_shard_full_size_striding_random(H, scheme, dct):
    # the same shard under the index-free schemes, every chunk: Random's positions are keyed by
    # the chunk's global number, so only a full-size run shows the kernel's chunk numbering
    w = synth.workloads()["olmo-1b-1of8"]
    cfg = Config(chunk=w.chunk, topk=w.topk, scheme=scheme, dct=dct, seed=99, step=5,
                 decay=w.decay, lr=w.lr, sign=w.sign)
    worst = _full_size_check(H, w, cfg)
    print("olmo-1b full size, scheme", scheme, "dct", dct, worst)
    assert worst["chunks"] == 2_298_368


@pytest.mark.size_dispatch
@pytest.mark.timeout(900)
@pytest.mark.parametrize("scheme,dct", [(SCHEME_TOPK, False), (SCHEME_STRIDE, False),
                                        (SCHEME_RANDOM, False), (SCHEME_RANDOM, True)])
def test_olmo_7b_shard_full_size(H, scheme, dct):
    """The OLMo-7B-shaped 1/8 shard (861,011,968 parameters; chunk 64, k = 32, R = 4), top-k
    against Striding and Random.  At this size the inputs are drawn on the device with
    torch's seeded generator (same recipe: N(0,1e-3) grads and momentum, N(0,0.02) parameters,
    bf16 storage); the sampled chunk runs are copied to the host for the oracle."""
    import torch
    from paper_2502_06728_amd import binding
    w = synth.workloads()["olmo-7b-1of8"]
    assert w.n == 861_011_968
    n, s, k, R = w.n, w.chunk, w.topk, w.replicas
    C = n // s
    cfg = Config(chunk=s, topk=k, scheme=scheme, dct=dct, seed=2024, step=3, decay=w.decay,
                 lr=w.lr, sign=True)
    dev = H.DEV
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    g = (torch.randn(n, generator=gen, device=dev) * w.grad_std).to(torch.bfloat16)
    m = torch.randn(n, generator=gen, device=dev) * w.momentum_std
    th = (torch.randn(n, generator=gen, device=dev) * w.params_std).to(torch.bfloat16)
    m0 = m.clone()
    th0 = th.clone()
    send_idx = scheme == SCHEME_TOPK
    idx = torch.empty(C * k, dtype=torch.int32, device=dev) if send_idx else None
    val = torch.empty(C * k, dtype=torch.float32, device=dev)
    coeff = torch.empty(C * s, dtype=torch.float32, device=dev)
    binding.detonation_compress(H.bcfg(cfg), g, m, idx, val, coeff)
    torch.cuda.synchronize()
    for c0, c1 in _sample_runs(C, count=10):
        e0, e1 = c0 * s, c1 * s
        parity.check_compress(cfg, H.to_host(g[e0:e1]), H.to_host(m0[e0:e1]), H.to_host(m[e0:e1]),
                              H.to_host(idx[c0 * k:c1 * k]) if send_idx else None,
                              H.to_host(val[c0 * k:c1 * k]), H.to_host(coeff[e0:e1]), chunk0=c0)
    del coeff, m0
    # R payloads of valid structure: one position drawn from each of k groups of s/k, ascending
    pv = torch.randn((R, C * k), generator=gen, device=dev) * w.momentum_std
    pi = None
    if send_idx:
        grp = s // k
        pi = torch.randint(0, grp, (R, C * k), generator=gen, device=dev, dtype=torch.int32)
        pi += (torch.arange(C * k, device=dev, dtype=torch.int32) % k) * grp
    y = torch.empty(n, dtype=torch.float32, device=dev)
    binding.detonation_decompress_step(H.bcfg(cfg), R, pi, pv, th, y)
    torch.cuda.synchronize()
    # Striding / Random transmit no indices: the oracle is handed its own selection for the
    # sampled chunks' global numbers, the same for every replica
    for c0, c1 in _sample_runs(C, count=10, seed=8):
        e0, e1 = c0 * s, c1 * s
        i_run = (H.to_host(pi[:, c0 * k:c1 * k].contiguous()) if send_idx
                 else _payload_indices(cfg, None, R, c0, c1))
        parity.check_decompress(cfg, i_run, H.to_host(pv[:, c0 * k:c1 * k].contiguous()),
                                H.to_host(th0[e0:e1]), H.to_host(th[e0:e1]),
                                H.to_host(y[e0:e1]))


@pytest.mark.parametrize("scheme", [SCHEME_TOPK, SCHEME_STRIDE, SCHEME_RANDOM])
def test_multi_step_trajectory(H, scheme):
    """Algorithm 1 is iterative: T steps of compress -> (exchange) -> decompress with evolving
    momentum and parameters, the Striding offset and the Random stream advancing with the
    step.  Every step is checked from the GPU's own state (staged protocol), the energy of
    the momentum is book-kept, and a free-running oracle trajectory measures the drift."""
    n, s, k, T, R = 64 * 1500 + 21, 64, 16, 6, 2
    rng = np.random.default_rng(11)
    m_gpu = synth.normal(3, synth.TAG_MOMENTUM, n, 1e-3)
    th_gpu = synth.normal(3, synth.TAG_PARAMS, n, 0.02)
    m_free, th_free = m_gpu.copy(), th_gpu.copy()         # oracle running on its own
    m_other = synth.normal(4, synth.TAG_MOMENTUM, n, 1e-3)  # the other replica's momentum
    send_idx = scheme == SCHEME_TOPK
    seen = np.zeros(s, dtype=int)
    for step in range(T):
        cfg = Config(chunk=s, topk=k, scheme=scheme, seed=5, step=step, decay=0.9, lr=1e-3,
                     sign=True)
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        g_other = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        # the other replica lives in the oracle
        m_other, idx_o, val_o = oracle.compress(cfg, g_other, m_other)
        # this replica on the GPU, judged from its own state
        m_new, idx_g, val_g, coeff_g = H.gpu_compress(cfg, g, m_gpu, want_idx=send_idx)
        parity.check_compress(cfg, g, m_gpu, m_new, idx_g, val_g, coeff_g)
        # energy over the complete chunks (the ragged last chunk sheds what falls on its pad)
        nf, cf = (n // s) * s, n // s
        m1 = oracle.fold(cfg, g, m_gpu).astype(np.float64)[:nf]
        e_in = (m1 ** 2).sum()
        e_out = ((m_new[:nf].astype(np.float64) ** 2).sum() +
                 (val_g[:cf * k].astype(np.float64) ** 2).sum())
        assert abs(e_in - e_out) < 1e-5 * e_in                  # nothing lost, nothing made up
        if scheme == SCHEME_STRIDE:
            own_idx = oracle.select(cfg, None, 1)
            seen[own_idx] += 1
        # exchange: [own payload, other replica's payload]
        val = np.stack([val_g, val_o])
        idx = np.stack([idx_g, idx_o]) if send_idx else None
        th_new, y = H.gpu_decompress(cfg, idx, val, th_gpu)
        parity.check_decompress(cfg, idx, val, th_gpu, th_new, y)
        # free-running oracle with the same gradients and the same other replica
        m_free, idx_f, val_f = oracle.compress(cfg, g, m_free)
        th_free = oracle.decompress_step(cfg, np.stack([idx_f, idx_o]) if send_idx else None,
                                         np.stack([val_f, val_o]), th_free)
        m_gpu, th_gpu = m_new, th_new
    if scheme == SCHEME_STRIDE:
        assert seen.sum() == T * k and seen.max() - seen.min() <= 1   # offset rotates evenly
    # drift of the free-running oracle from the GPU trajectory: a flipped near-tie or sign
    # moves single elements by a coefficient or 2*eta, so compare in the mean
    assert np.abs(th_free - th_gpu).mean() < 1e-3 * 1e-3
    assert np.abs(m_free - m_gpu).mean() < 1e-3 * np.abs(m_free).mean()


@pytest.mark.parametrize("val_dtype", [oracle.BF16, oracle.F16])
@pytest.mark.parametrize("idx_u8", [True, False])
@pytest.mark.parametrize("s,k,n", [(64, 32, 64 * 3000 + 13), (64, 8, 64 * 2000), (32, 4, 32 * 777 + 5),
                                   (96, 12, 96 * 300 + 1),
                                   # chunk 32 at the rates 1/2 ... 1/32; 336 chunks, so every
                                   # replica's arrays start 16-byte aligned (lane-per-chunk kernels)
                                   (32, 16, 32 * 335 + 5), (32, 8, 32 * 335 + 5), (32, 4, 32 * 335 + 5),
                                   (32, 2, 32 * 335 + 5), (32, 1, 32 * 335 + 5)])
def test_packed_payload_formats(H, val_dtype, idx_u8, s, k, n):
    """16-bit transfer values (Appendix B, communication dtype) and byte indices: the payload is
    the fp32 payload rounded to the transfer dtype, and the momentum keeps the rounding error."""
    cfg = Config(chunk=s, topk=k, sign=True, decay=0.999, lr=1e-3)
    g, m, th = make_inputs(n, seed=s + k, grad_bf16=True, params_bf16=True, outliers=0.01)
    m_gpu, idx_gpu, vbits_gpu, coeff_gpu = H.gpu_compress_packed(cfg, g, m, val_dtype, idx_u8)
    parity.check_compress_packed(cfg, g, m, m_gpu, idx_gpu, vbits_gpu, coeff_gpu, val_dtype)
    R = 3
    pays = [oracle.compress_q(cfg, *make_inputs(n, seed=900 + r, grad_bf16=True, outliers=0.01)[:2],
                              val_dtype)[1:] for r in range(R)]
    idx = np.stack([p[0] for p in pays])
    vbits = np.stack([p[1] for p in pays])
    th_gpu, y_gpu = H.gpu_decompress_packed(cfg, idx, vbits, th, val_dtype, idx_u8)
    parity.check_decompress_packed(cfg, idx, vbits, val_dtype, th, th_gpu, y_gpu)


def test_packed_striding_random_values_only(H):
    # Striding / Random ship values only; with a 16-bit transfer dtype they run on the general kernels
    import torch
    from paper_2502_06728_amd import binding
    n, s, k = 64 * 500 + 3, 64, 16
    for scheme in (SCHEME_STRIDE, SCHEME_RANDOM):
        cfg = Config(chunk=s, topk=k, scheme=scheme, seed=9, step=2, sign=False)
        g, m, th = make_inputs(n, seed=31)
        m1 = oracle.fold(cfg, g, m)
        coeff = oracle.transform(cfg, m1)
        idx_o = oracle.select(cfg, None, -(-n // s))
        vb_o, m_o = oracle.extract_q(cfg, m1, coeff, idx_o, oracle.F16)
        gm, gg = H.to_dev(m), H.to_dev(g)
        val = torch.zeros(idx_o.size, dtype=torch.float16, device=H.DEV)
        binding.detonation_compress_packed(H.bcfg(cfg), gg, gm, None, val)
        torch.cuda.synchronize()
        assert np.array_equal(val.view(torch.int16).cpu().numpy().view(np.uint16), vb_o)
        assert np.array_equal(H.to_host(gm), m_o)            # raw domain: exact arithmetic
        p = H.to_dev(th)
        y = torch.empty(n, dtype=torch.float32, device=H.DEV)
        binding.detonation_decompress_step_packed(H.bcfg(cfg), 2, None, torch.stack([val, val]), p, y)
        torch.cuda.synchronize()
        y_o = oracle.presign_q(cfg, n, np.stack([idx_o, idx_o]), np.stack([vb_o, vb_o]), oracle.F16)
        assert np.array_equal(H.to_host(y), y_o)


@pytest.mark.parametrize("amsgrad", [False, True])
@pytest.mark.parametrize("s,k,n,params_bf16", [(64, 32, 64 * 2500 + 7, True), (64, 16, 64 * 1000, False),
                                               (32, 8, 32 * 900 + 3, False), (32, 16, 32 * 4000 + 9, True),
                                               (32, 2, 32 * 3000, False), (32, 1, 32 * 3000 + 1, True),
                                               # the wavefront-per-class decompress (any k, AdamW)
                                               (64, 20, 64 * 700 + 9, True), (64, 5, 64 * 500 + 3, False),
                                               (96, 10, 96 * 300 + 5, True), (96, 12, 96 * 200, False),
                                               (128, 30, 128 * 300 + 1, False), (128, 16, 128 * 200, True)])
def test_decoupled_adamw_steps(H, amsgrad, s, k, n, params_bf16):
    """Decoupled AdamW as the underlying optimizer (section "Decoupled AdamW"): T steps with
    local moments; every step is judged from the GPU's own state, sign decided on the GPU's
    pre-sign values."""
    import torch
    from paper_2502_06728_amd import binding
    T, R = 4, 2
    cfg = Config(chunk=s, topk=k, sign=True, lr=1e-3, weight_decay=0.01)
    th = make_inputs(n, 5, params_bf16=params_bf16)[2]
    p = H.to_dev(th)
    m = torch.zeros(n, device=H.DEV)
    v = torch.zeros(n, device=H.DEV)
    vm = torch.zeros(n, device=H.DEV) if amsgrad else None
    for t in range(1, T + 1):
        pays = [oracle.compress(cfg, *make_inputs(n, 100 * t + r)[:2])[1:] for r in range(R)]
        idx = np.stack([q[0] for q in pays])
        val = np.stack([q[1] for q in pays])
        th_in, m_in, v_in = H.to_host(p), m.cpu().numpy(), v.cpu().numpy()
        vm_in = vm.cpu().numpy() if amsgrad else None
        y = torch.empty(n, dtype=torch.float32, device=H.DEV)
        opt = oracle.AdamW(0.9, 0.95, 1e-8, amsgrad, t)
        binding.detonation_decompress_adamw_step(
            H.bcfg(cfg), binding.AdamW(0.9, 0.95, 1e-8, amsgrad, t), R, H.to_dev(idx), H.to_dev(val),
            p, m, v, vm, y)
        torch.cuda.synchronize()
        y_gpu = H.to_host(y)
        y_o = oracle.presign(cfg, n, idx, val)
        assert parity.rel_chunk_err(y_gpu, y_o, s) <= parity.TOL_F32
        th_o, m_o, v_o, vm_o = oracle.adamw_update(cfg, opt, y_gpu, th_in, m_in, v_in, vm_in)
        assert np.abs(m.cpu().numpy() - m_o).max() <= 1e-5 * np.abs(m_o).max()
        assert np.abs(v.cpu().numpy() - v_o).max() <= 1e-5 * np.abs(v_o).max()
        if amsgrad:
            assert np.abs(vm.cpu().numpy() - vm_o).max() <= 1e-5 * np.abs(vm_o).max()
        got = H.to_host(p)
        if params_bf16:
            got = synth.from_bf16_bits(got).astype(np.float64)
            want = synth.from_bf16_bits(th_o).astype(np.float64)
            tol = parity.TOL_BF16
        else:
            got, want, tol = got.astype(np.float64), th_o.astype(np.float64), parity.TOL_F32
        assert (np.abs(got - want) <= tol * np.abs(want) + tol * cfg.lr).all()


def test_maximum_replicas_and_chunk(H):
    # R = 64 (the most the library accepts) and s = k = 256 (the largest chunk, nothing dropped)
    cfg = Config(chunk=64, topk=4, sign=False)
    full_step(H, cfg, 64 * 200 + 9, R=64, seed=2)
    cfg = Config(chunk=256, topk=256, sign=True)
    full_step(H, cfg, 256 * 40 + 100, R=2, seed=3)


def test_step_inside_a_hip_graph(H):
    """Both calls only enqueue kernels on the caller's stream and allocate nothing, so a whole
    step can be captured into a HIP graph.  The graph is replayed several times with eager work
    and synchronisations in between; every replay must equal the eager result bit for bit."""
    import torch
    from paper_2502_06728_amd import binding
    n, s, k, R = 64 * 4096 + 64 * 7 + 3, 64, 32, 3
    cfg = Config(chunk=s, topk=k, sign=True)
    g, m0, th0 = make_inputs(n, 17, grad_bf16=True, params_bf16=True)
    entries = -(-n // s) * k
    pays = [oracle.compress(cfg, *make_inputs(n, 40 + r, grad_bf16=True)[:2])[1:] for r in range(R)]
    idx_np = np.stack([q[0] for q in pays])
    val_np = np.stack([q[1] for q in pays])
    gd = H.to_dev(g)
    bc = H.bcfg(cfg)

    def fresh():
        return (H.to_dev(m0), H.to_dev(th0), H.to_dev(idx_np.copy()), H.to_dev(val_np.copy()))

    # eager reference: compress writes replica 0's slot, decompress consumes all R
    m_e, th_e, idx_e, val_e = fresh()
    binding.detonation_compress(bc, gd, m_e, idx_e[0], val_e[0])
    binding.detonation_decompress_step(bc, R, idx_e, val_e, th_e)
    torch.cuda.synchronize()
    want = [H.to_host(t) for t in (m_e, th_e, idx_e, val_e)]

    m_g, th_g, idx_g, val_g = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):     # warm-up on the capture stream
        binding.detonation_compress(bc, gd, m_g, idx_g[0], val_g[0])
        binding.detonation_decompress_step(bc, R, idx_g, val_g, th_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        binding.detonation_compress(bc, gd, m_g, idx_g[0], val_g[0])
        binding.detonation_decompress_step(bc, R, idx_g, val_g, th_g)
    for replay in range(3):
        # reset the in-place state with eager copies, do unrelated eager work, then replay
        m_g.copy_(H.to_dev(m0))
        th_g.copy_(H.to_dev(th0))
        idx_g.copy_(H.to_dev(idx_np))
        val_g.copy_(H.to_dev(val_np))
        junk = torch.randn(1 << 20, device=H.DEV).sum().item()
        assert np.isfinite(junk)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [H.to_host(t) for t in (m_g, th_g, idx_g, val_g)]
        for a, b in zip(got, want):
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), f"replay {replay}"


def test_sign_of_subnormal_and_huge_updates(H):
    # sign() must be exact for every non-zero finite value, including fp32 subnormals and
    # values near overflow; zero (of either sign) leaves the parameter alone
    s, k, n = 64, 32, 64 * 130
    cfg = Config(chunk=s, topk=k, scheme=SCHEME_STRIDE, sign=True, lr=1e-3)   # raw domain: y = val
    C = n // s
    special = np.array([1e-45, -1e-45, 1e-40, -3e-39, 1.1754942e-38, 3e38, -3e38, 0.0, -0.0, 1e-30],
                       dtype=np.float32)
    val = np.tile(special, C * k // special.size + 1)[:C * k].copy()
    th = make_inputs(n, 9)[2]
    th_gpu, y_gpu = H.gpu_decompress(cfg, None, val[None, :], th)
    parity.check_decompress(cfg, None, val[None, :], th, th_gpu, y_gpu)
    idx = oracle.select(cfg, None, C).reshape(C, k)
    flat = (np.arange(C)[:, None] * s + idx).ravel()
    moved = (th_gpu - th)[flat]
    want = -np.float32(1e-3) * np.sign(val)
    assert np.abs(moved - want).max() < 1e-8


def test_byte_indices_with_fp32_values(H):
    # index width and value dtype are independent: fp32 values + byte indices go through the
    # same staged check as the plain format (these run on the general kernels)
    import torch
    from paper_2502_06728_amd import binding
    n, s, k, R = 64 * 700 + 11, 64, 16, 2
    cfg = Config(chunk=s, topk=k, sign=True)
    g, m, th = make_inputs(n, 23)
    entries = -(-n // s) * k
    gm = H.to_dev(m)
    idx8 = torch.zeros(entries, dtype=torch.uint8, device=H.DEV)
    val = torch.zeros(entries, dtype=torch.float32, device=H.DEV)
    coeff = torch.zeros(-(-n // s) * s, dtype=torch.float32, device=H.DEV)
    binding.detonation_compress_packed(H.bcfg(cfg), H.to_dev(g), gm, idx8, val, coeff)
    torch.cuda.synchronize()
    parity.check_compress(cfg, g, m, H.to_host(gm), idx8.cpu().numpy().astype(np.int32),
                          H.to_host(val), H.to_host(coeff))
    pays = [oracle.compress(cfg, *make_inputs(n, 60 + r)[:2])[1:] for r in range(R)]
    idx = np.stack([q[0] for q in pays])
    vals = np.stack([q[1] for q in pays])
    p = H.to_dev(th)
    y = torch.empty(n, dtype=torch.float32, device=H.DEV)
    binding.detonation_decompress_step_packed(
        H.bcfg(cfg), R, torch.from_numpy(idx.astype(np.uint8)).to(H.DEV), H.to_dev(vals), p, y)
    torch.cuda.synchronize()
    parity.check_decompress(cfg, idx, vals, th, H.to_host(p), H.to_host(y))


@pytest.mark.parametrize("idx_u8", [False, True])
@pytest.mark.parametrize("s,k,n", [(64, 32, 64 * 3000 + 13), (64, 16, 64 * 1000), (32, 4, 32 * 777 + 5),
                                   (96, 20, 96 * 300 + 1), (128, 48, 128 * 100), (16, 2, 16 * 500 + 3),
                                   # the paper's own setting: chunk 32, signs only, rates 1/2 ... 1/32
                                   (32, 16, 32 * 335 + 5), (32, 8, 32 * 335 + 5), (32, 4, 32 * 335 + 5),
                                   (32, 2, 32 * 335 + 5), (32, 1, 32 * 335 + 5)])
def test_ternary_payload(H, idx_u8, s, k, n):
    """The sign taken before the exchange (Discussion): only sign(c) of the kept coefficients travels,
    two bits per entry; the momentum loses the extracted components themselves."""
    cfg = Config(chunk=s, topk=k, sign=True, decay=0.999, lr=1e-3)
    g, m, th = make_inputs(n, seed=s + k, grad_bf16=True, params_bf16=True, outliers=0.01)
    m_gpu, idx_gpu, words_gpu, coeff_gpu = H.gpu_compress_ternary(cfg, g, m, idx_u8)
    C = -(-n // s)
    kept = coeff_gpu.reshape(C, s)[np.arange(C)[:, None], idx_gpu.reshape(C, k)].reshape(-1)
    # coefficients, selection and momentum: the fp32 protocol with the kept values as payload
    parity.check_compress(cfg, g, m, m_gpu, idx_gpu, kept, coeff_gpu)
    assert np.array_equal(words_gpu, oracle.encode_ternary(cfg, n, kept))
    R = 3
    pays = [oracle.compress_t(cfg, *make_inputs(n, seed=900 + r, grad_bf16=True, outliers=0.01)[:2])[1:]
            for r in range(R)]
    idx = np.stack([p[0] for p in pays])
    words = np.stack([p[1] for p in pays])
    th_gpu, y_gpu = H.gpu_decompress_ternary(cfg, idx, words, th, idx_u8)
    signs = np.stack([oracle.decode_ternary(cfg, n, w) for w in words])
    parity.check_decompress(cfg, idx, signs, th, th_gpu, y_gpu)


@pytest.mark.parametrize("dct", [False, True])
@pytest.mark.parametrize("scheme", [SCHEME_STRIDE, SCHEME_RANDOM])
@pytest.mark.parametrize("val_dtype", [oracle.BF16, oracle.F16, oracle.TERNARY])
@pytest.mark.parametrize("s,k", [(32, 16), (32, 4), (32, 2), (32, 1), (64, 32), (64, 4)])
def test_narrow_payload_striding_random(H, s, k, val_dtype, scheme, dct):
    """Striding / Random with 16-bit values or signs only, no indices on the wire (the paper's
    experiments synchronise only signs at chunk size 32): 336 chunks, so every replica's array
    starts 16-byte aligned and the lane-per-chunk kernels take five tiles plus a ragged tail."""
    n, R = s * 335 + 5, 3
    C = -(-n // s)
    cfg = Config(chunk=s, topk=k, scheme=scheme, dct=dct, seed=5, step=3, sign=True, decay=0.999, lr=1e-3)
    g, m, th = make_inputs(n, seed=s + k, grad_bf16=True, params_bf16=True, outliers=0.01)
    others = [make_inputs(n, seed=900 + r, grad_bf16=True, outliers=0.01)[:2] for r in range(R)]
    if val_dtype == oracle.TERNARY:
        m_gpu, idx_gpu, words_gpu, coeff_gpu = H.gpu_compress_ternary(cfg, g, m, True)
        kept = coeff_gpu.reshape(C, s)[np.arange(C)[:, None], idx_gpu.reshape(C, k)].reshape(-1)
        parity.check_compress(cfg, g, m, m_gpu, idx_gpu, kept, coeff_gpu)
        assert np.array_equal(words_gpu, oracle.encode_ternary(cfg, n, kept))
        pays = [oracle.compress_t(cfg, *o)[1:] for o in others]
        idx = np.stack([p[0] for p in pays])
        words = np.stack([p[1] for p in pays])
        th_gpu, y_gpu = H.gpu_decompress_ternary(cfg, None, words, th, False)
        signs = np.stack([oracle.decode_ternary(cfg, n, w) for w in words])
        parity.check_decompress(cfg, idx, signs, th, th_gpu, y_gpu)
    else:
        m_gpu, idx_gpu, vbits_gpu, coeff_gpu = H.gpu_compress_packed(cfg, g, m, val_dtype, True)
        parity.check_compress_packed(cfg, g, m, m_gpu, idx_gpu, vbits_gpu, coeff_gpu, val_dtype)
        pays = [oracle.compress_q(cfg, *o, val_dtype)[1:] for o in others]
        idx = np.stack([p[0] for p in pays])
        vbits = np.stack([p[1] for p in pays])
        th_gpu, y_gpu = H.gpu_decompress_packed(cfg, None, vbits, th, val_dtype, False)
        parity.check_decompress_packed(cfg, idx, vbits, val_dtype, th, th_gpu, y_gpu)


@pytest.mark.parametrize("scheme", [SCHEME_STRIDE, SCHEME_RANDOM])
def test_ternary_payload_striding_random(H, scheme):
    # values only; identity domain: the pre-sign update is an exact average of signs
    n, s, k = 64 * 400 + 9, 64, 16
    cfg = Config(chunk=s, topk=k, scheme=scheme, seed=4, step=3, sign=False)
    g, m, th = make_inputs(n, seed=12)
    m_gpu, _, words_gpu, _ = H.gpu_compress_ternary(cfg, g, m, False, want_idx=False)
    m_o, idx_o, words_o = oracle.compress_t(cfg, g, m)
    assert np.array_equal(words_gpu, words_o) and np.array_equal(m_gpu, m_o)
    words = np.stack([words_o, oracle.compress_t(cfg, *make_inputs(n, seed=13)[:2])[2]])
    th_gpu, y_gpu = H.gpu_decompress_ternary(cfg, None, words, th, False)
    assert np.array_equal(y_gpu, oracle.presign_t(cfg, n, None, words))
    th_o = oracle.update(cfg, y_gpu, th)
    assert np.abs(th_gpu - th_o).max() <= 1e-6 * np.abs(th_o).max()


@pytest.mark.parametrize("bf16", [False, True])
def test_diloco_cycle_accumulate_then_full_synchronisation(H, bf16):
    """DiLoCo as a replicator (synchronises only on every n-th optimizer step): the steps in
    between only accumulate (detonation_accumulate), the n-th extracts the whole momentum
    (Striding with k = s) and averages it over the replicas.  Raw domain: momentum, payload
    and averaged update equal the oracle's bit for bit."""
    import torch
    from paper_2502_06728_amd import binding
    s, every, T, R = 64, 3, 7, 2
    for n in (64 * 700 + 13, 37):
        g0, m0, th0 = make_inputs(n, seed=n, grad_bf16=bf16, params_bf16=bf16)
        m_dev, th_dev = H.to_dev(m0), H.to_dev(th0)
        m_o = m0.copy()
        m_other = make_inputs(n, seed=n + 1)[1]
        for step in range(T):
            cfg = Config(chunk=s, topk=s, scheme=SCHEME_STRIDE, decay=0.9, lr=1e-2, sign=False,
                         step=step)
            g = make_inputs(n, seed=100 + step, grad_bf16=bf16)[0]
            g_other = make_inputs(n, seed=200 + step)[0]
            if (step + 1) % every:
                binding.detonation_accumulate(H.bcfg(cfg), H.to_dev(g), m_dev)
                torch.cuda.synchronize()
                m_o = oracle.fold(cfg, g, m_o)
                m_other = oracle.fold(cfg, g_other, m_other)
                assert np.array_equal(H.to_host(m_dev), m_o)
                continue
            m_other, _, val_other = oracle.compress(cfg, g_other, m_other)
            m_new, _, val_g, _ = H.gpu_compress(cfg, g, H.to_host(m_dev), want_idx=False,
                                                want_coeff=False)
            m_o, _, val_o = oracle.compress(cfg, g, m_o)
            assert np.array_equal(val_g, val_o) and not m_new.any() and not m_o.any()
            m_dev = H.to_dev(m_new)
            val = np.stack([val_g, val_other])
            th_in = H.to_host(th_dev)
            th_new, y = H.gpu_decompress(cfg, None, val, th_in)
            assert np.array_equal(y, oracle.presign(cfg, n, None, val))
            parity.check_decompress(cfg, None, val, th_in, th_new, y)   # one rounding of theta
            th_dev = H.to_dev(th_new)


@pytest.mark.parametrize("scheme", [SCHEME_STRIDE, SCHEME_RANDOM])
@pytest.mark.parametrize("s,n", [(64, 64 * 900 + 7), (32, 32 * 100), (6, 6 * 50 + 1), (256, 256 * 9 + 100)])
def test_every_position_kept_in_the_raw_domain(H, scheme, s, n):
    # k = s without the transform: the payload is the folded momentum, the momentum restarts
    # from zero, the receivers average dense arrays (streaming kernels)
    cfg = Config(chunk=s, topk=s, scheme=scheme, seed=2, step=5, sign=True, lr=1e-3,
                 weight_decay=0.05)
    st_c, st_d = full_step(H, cfg, n, R=3, seed=s, grad_bf16=True, params_bf16=True)
    g, m, th = make_inputs(n, seed=1)
    m_gpu, idx_gpu, val_gpu, coeff_gpu = H.gpu_compress(cfg, g, m, want_idx=True)
    C = -(-n // s)
    assert np.array_equal(idx_gpu.reshape(C, s), np.tile(np.arange(s, dtype=np.int32), (C, 1)))
    assert not m_gpu.any()
    assert np.array_equal(val_gpu[:n], oracle.fold(cfg, g, m)) and not val_gpu[n:].any()
    assert np.array_equal(coeff_gpu, val_gpu)


@pytest.mark.parametrize("s,k", [(96, 12), (96, 24), (96, 48), (128, 64), (64, 32), (16, 8),
                                 (192, 24), (192, 10), (256, 32), (256, 128), (256, 6)])
def test_unordered_payloads_on_every_vector_scatter(H, s, k):
    # duplicates, disorder and out-of-range indices at the k values whose chunks straddle the
    # 64-lane vectors of the scatter (k not dividing 256) and at those that do not
    n = s * 64 * 6
    C = n // s
    cfg = Config(chunk=s, topk=k, sign=False)
    rng = np.random.default_rng(s + k)
    idx = np.stack([np.sort(rng.integers(0, s, size=(C, k)), axis=1).reshape(-1),      # repeats
                    rng.integers(-2, s + 2, size=C * k),                                # anything
                    np.tile(np.arange(k), C)]).astype(np.int32)                         # clean
    # a clean chunk sequence broken exactly at vector boundaries (entry 256*j - 1 and 256*j)
    for j in range(1, (C * k) // 256):
        idx[2, 256 * j] = idx[2, 256 * j - 1]
    val = rng.standard_normal((3, C * k)).astype(np.float32)
    th = make_inputs(n, 3)[2]
    th_gpu, y_gpu = H.gpu_decompress(cfg, idx, val, th)
    parity.check_decompress(cfg, idx, val, th, th_gpu, y_gpu)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("s,k,scheme", [(64, 32, SCHEME_TOPK), (128, 64, SCHEME_TOPK), (256, 32, SCHEME_TOPK),
                                        (64, 16, SCHEME_RANDOM), (64, 64, SCHEME_STRIDE)])
def test_buffers_aligned_to_their_element_size_only(H, bf16, s, k, scheme):
    """The ABI asks for element-size alignment only: every buffer here starts one element past a
    16-byte boundary (slices of larger tensors), which sends the calls to the general kernels."""
    import torch
    from paper_2502_06728_amd import binding
    n, R = s * 300 + 11, 2
    C = -(-n // s)
    cfg = Config(chunk=s, topk=k, scheme=scheme, seed=3, step=1, sign=True, lr=1e-3)
    g, m, th = make_inputs(n, seed=s + k, grad_bf16=bf16, params_bf16=bf16)
    send_idx = scheme == SCHEME_TOPK

    def off(a_np=None, size=None, dtype=None, fill=None):
        """a device tensor whose data pointer is one element past a 16-byte boundary"""
        if a_np is not None:
            src = H.to_dev(a_np)
            big = torch.empty(src.numel() + 1, dtype=src.dtype, device=H.DEV)
            big[1:].copy_(src)
            return big[1:]
        big = torch.full((size + 1,), fill, dtype=dtype, device=H.DEV)
        return big[1:]

    gd, md = off(g), off(m)
    idx = off(size=C * k, dtype=torch.int32, fill=-7) if send_idx else None
    val = off(size=C * k, dtype=torch.float32, fill=float("nan"))
    coeff = off(size=C * s, dtype=torch.float32, fill=float("nan"))
    assert gd.data_ptr() % 16 != 0 and md.data_ptr() % 16 != 0 and val.data_ptr() % 16 != 0
    binding.detonation_compress(H.bcfg(cfg), gd, md, idx, val, coeff)
    torch.cuda.synchronize()
    parity.check_compress(cfg, g, m, H.to_host(md), None if idx is None else H.to_host(idx),
                          H.to_host(val), H.to_host(coeff))
    pays = [oracle.compress(cfg, *make_inputs(n, seed=40 + r)[:2])[1:] for r in range(R)]
    idx_np = np.stack([p[0] for p in pays]) if send_idx else None
    val_np = np.stack([p[1] for p in pays])
    stride = C * k + 3                                  # replica 1 is misaligned differently
    vbuf = off(size=R * stride, dtype=torch.float32, fill=float("nan"))
    ibuf = off(size=R * stride, dtype=torch.int32, fill=999) if send_idx else None
    for r in range(R):
        vbuf[r * stride:r * stride + C * k].copy_(H.to_dev(val_np[r]))
        if send_idx:
            ibuf[r * stride:r * stride + C * k].copy_(H.to_dev(idx_np[r]))
    pd, yd = off(th), off(size=n, dtype=torch.float32, fill=float("nan"))
    binding.detonation_decompress_step(H.bcfg(cfg), R, ibuf, vbuf, pd, yd,
                                       idx_replica_stride=stride, val_replica_stride=stride)
    torch.cuda.synchronize()
    parity.check_decompress(cfg, idx_np, val_np, th, H.to_host(pd), H.to_host(yd))
    # accumulate on misaligned buffers
    m2 = off(m)
    binding.detonation_accumulate(H.bcfg(cfg), gd, m2)
    torch.cuda.synchronize()
    assert np.array_equal(H.to_host(m2), oracle.fold(cfg, g, m))


@pytest.mark.parametrize("scheme", [SCHEME_STRIDE, SCHEME_RANDOM])
@pytest.mark.parametrize("s,k,params_bf16", [(32, 8, False), (64, 32, True), (32, 2, False), (96, 12, False)])
def test_decoupled_adamw_without_transmitted_indices(H, scheme, s, k, params_bf16):
    """Decoupled AdamW under the Striding / Random replicators (values only; the indices are
    regenerated): three steps, the moments local to the rank."""
    import torch
    from paper_2502_06728_amd import binding
    n, R, amsgrad = s * (64 * 12 + 5) + 3, 3, True
    th = make_inputs(n, 5, params_bf16=params_bf16)[2]
    p = H.to_dev(th)
    m = torch.zeros(n, device=H.DEV)
    v = torch.zeros(n, device=H.DEV)
    vm = torch.zeros(n, device=H.DEV)
    for t in (1, 2, 3):
        cfg = Config(chunk=s, topk=k, scheme=scheme, seed=8, step=t, sign=True, lr=1e-3,
                     weight_decay=0.01)
        val = np.stack([oracle.compress(cfg, *make_inputs(n, 100 * t + r)[:2])[2] for r in range(R)])
        th_in, m_in, v_in, vm_in = H.to_host(p), m.cpu().numpy(), v.cpu().numpy(), vm.cpu().numpy()
        y = torch.empty(n, dtype=torch.float32, device=H.DEV)
        binding.detonation_decompress_adamw_step(
            H.bcfg(cfg), binding.AdamW(0.9, 0.95, 1e-8, amsgrad, t), R, None, H.to_dev(val),
            p, m, v, vm, y)
        torch.cuda.synchronize()
        y_gpu = H.to_host(y)
        assert parity.rel_chunk_err(y_gpu, oracle.presign(cfg, n, None, val), s) <= parity.TOL_F32
        th_o, m_o, v_o, vm_o = oracle.adamw_update(cfg, oracle.AdamW(0.9, 0.95, 1e-8, amsgrad, t),
                                                   y_gpu, th_in, m_in, v_in, vm_in)
        assert np.abs(m.cpu().numpy() - m_o).max() <= 1e-5 * np.abs(m_o).max()
        assert np.abs(v.cpu().numpy() - v_o).max() <= 1e-5 * np.abs(v_o).max()
        assert np.abs(vm.cpu().numpy() - vm_o).max() <= 1e-5 * np.abs(vm_o).max()
        got = H.to_host(p)
        if params_bf16:
            got = synth.from_bf16_bits(got).astype(np.float64)
            want = synth.from_bf16_bits(th_o).astype(np.float64)
            tol = parity.TOL_BF16
        else:
            got, want, tol = got.astype(np.float64), th_o.astype(np.float64), parity.TOL_F32
        assert (np.abs(got - want) <= tol * np.abs(want) + tol * cfg.lr).all()


@pytest.mark.parametrize("scheme", [SCHEME_TOPK, SCHEME_RANDOM])
@pytest.mark.parametrize("val_dtype", [oracle.BF16, oracle.F16, oracle.TERNARY])
@pytest.mark.parametrize("s,k,params_bf16", [(32, 16, True), (32, 4, False), (32, 1, True), (64, 32, True),
                                             (96, 12, False)])
def test_decoupled_adamw_narrow_payloads(H, s, k, params_bf16, val_dtype, scheme):
    """Decoupled AdamW on what the paper's experiments put on the wire (signs only at chunk
    size 32, "Overall Setup") and on 16-bit values: byte indices under top-k, no indices under
    Random; two steps with local moments.  336 chunks, so the replicas' arrays start 16-byte
    aligned (lane-per-chunk kernels; chunk 96 runs on the general ones)."""
    import torch
    from paper_2502_06728_amd import binding
    n, R, amsgrad = s * 335 + 5, 3, True
    th = make_inputs(n, 5, params_bf16=params_bf16)[2]
    p = H.to_dev(th)
    m = torch.zeros(n, device=H.DEV)
    v = torch.zeros(n, device=H.DEV)
    vm = torch.zeros(n, device=H.DEV)
    for t in (1, 2):
        cfg = Config(chunk=s, topk=k, scheme=scheme, seed=8, step=t, sign=True, lr=1e-3,
                     weight_decay=0.01)
        ins = [make_inputs(n, 100 * t + r)[:2] for r in range(R)]
        if val_dtype == oracle.TERNARY:
            pays = [oracle.compress_t(cfg, *i)[1:] for i in ins]
            val = np.stack([q[1] for q in pays])
            val_dev = torch.from_numpy(np.ascontiguousarray(val).view(np.int32)).to(H.DEV)
        else:
            pays = [oracle.compress_q(cfg, *i, val_dtype)[1:] for i in ins]
            val = np.stack([q[1] for q in pays])
            val_dev = H.bits16_to_dev(np.ascontiguousarray(val), val_dtype)
        idx = np.stack([q[0] for q in pays])
        idx_dev = (torch.from_numpy(np.ascontiguousarray(idx.reshape(R, -1).astype(np.uint8))).to(H.DEV)
                   if scheme == SCHEME_TOPK else None)
        th_in, m_in, v_in, vm_in = H.to_host(p), m.cpu().numpy(), v.cpu().numpy(), vm.cpu().numpy()
        y = torch.empty(n, dtype=torch.float32, device=H.DEV)
        binding.detonation_decompress_adamw_step_packed(
            H.bcfg(cfg), binding.AdamW(0.9, 0.95, 1e-8, amsgrad, t), R, idx_dev, val_dev,
            p, m, v, vm, y)
        torch.cuda.synchronize()
        y_gpu = H.to_host(y)
        y_o = (oracle.presign_t(cfg, n, idx, val) if val_dtype == oracle.TERNARY
               else oracle.presign_q(cfg, n, idx, val, val_dtype))
        # replicas can cancel: the scale is the chunk's largest transmitted magnitude (1 for signs)
        C = -(-n // s)
        if val_dtype == oracle.TERNARY:
            vmax = np.ones(C)
        else:
            dec = ((val.astype(np.uint32) << 16).view(np.float32) if val_dtype == oracle.BF16
                   else val.view(np.float16).astype(np.float32))
            vmax = np.abs(dec.astype(np.float64).reshape(R, C, k)).max(axis=(0, 2))
        scale = np.maximum(np.repeat(vmax, s)[:n], parity.parity_chunk_max(y_o, s))
        assert parity.rel_chunk_err(y_gpu, y_o, s, scale=scale) <= parity.TOL_F32
        th_o, m_o, v_o, vm_o = oracle.adamw_update(cfg, oracle.AdamW(0.9, 0.95, 1e-8, amsgrad, t),
                                                   y_gpu, th_in, m_in, v_in, vm_in)
        assert np.abs(m.cpu().numpy() - m_o).max() <= 1e-5 * np.abs(m_o).max()
        assert np.abs(v.cpu().numpy() - v_o).max() <= 1e-5 * np.abs(v_o).max()
        assert np.abs(vm.cpu().numpy() - vm_o).max() <= 1e-5 * np.abs(vm_o).max()
        got = H.to_host(p)
        if params_bf16:
            got = synth.from_bf16_bits(got).astype(np.float64)
            want = synth.from_bf16_bits(th_o).astype(np.float64)
            tol = parity.TOL_BF16
        else:
            got, want, tol = got.astype(np.float64), th_o.astype(np.float64), parity.TOL_F32
        assert (np.abs(got - want) <= tol * np.abs(want) + tol * cfg.lr).all()


@pytest.mark.parametrize("R", [9, 64])
@pytest.mark.parametrize("mode", ["topk-f32", "random-f32", "topk-signs", "random-signs", "random-f16"])
@pytest.mark.parametrize("s,k", [(32, 1), (32, 4), (64, 8)])
def test_large_replication_groups(H, s, k, mode, R):
    """The replication group of the paper's scaling runs has 64 members ("OLMo2: Scaling Up").
    Decompress keeps several replicas' payloads in flight and requests the others in batches:
    replica counts that are and are not a multiple of the batch, on every payload path (144
    chunks, so each replica's arrays start 16-byte aligned and the lane-per-chunk kernels run)."""
    n = s * 143 + 5
    scheme = SCHEME_TOPK if mode.startswith("topk") else SCHEME_RANDOM
    cfg = Config(chunk=s, topk=k, scheme=scheme, seed=3, step=R, sign=(R != 9), lr=1e-3)
    th = make_inputs(n, seed=R, params_bf16=(R == 64))[2]
    # the other replicas' shards: any values will do, drawn directly (the seeded generator of
    # the benchmark shards works in 4 Mi-element blocks, far more than these few thousand)
    rng = np.random.default_rng(1000 + R)
    ins = [(rng.standard_normal(n).astype(np.float32) * 1e-3,
            rng.standard_normal(n).astype(np.float32) * 1e-3) for _ in range(R)]
    if mode.endswith("f32"):
        pays = [oracle.compress(cfg, *i)[1:] for i in ins]
        idx, val = np.stack([q[0] for q in pays]), np.stack([q[1] for q in pays])
        th_gpu, y_gpu = H.gpu_decompress(cfg, idx if scheme == SCHEME_TOPK else None, val, th)
        parity.check_decompress(cfg, idx, val, th, th_gpu, y_gpu)
    elif mode.endswith("signs"):
        pays = [oracle.compress_t(cfg, *i)[1:] for i in ins]
        idx, words = np.stack([q[0] for q in pays]), np.stack([q[1] for q in pays])
        th_gpu, y_gpu = H.gpu_decompress_ternary(cfg, idx if scheme == SCHEME_TOPK else None,
                                                 words, th, True)
        signs = np.stack([oracle.decode_ternary(cfg, n, w) for w in words])
        parity.check_decompress(cfg, idx, signs, th, th_gpu, y_gpu)
    else:
        pays = [oracle.compress_q(cfg, *i, oracle.F16)[1:] for i in ins]
        idx, vbits = np.stack([q[0] for q in pays]), np.stack([q[1] for q in pays])
        th_gpu, y_gpu = H.gpu_decompress_packed(cfg, None, vbits, th, oracle.F16, False)
        parity.check_decompress_packed(cfg, idx, vbits, oracle.F16, th, th_gpu, y_gpu)
