"""GPU parity for the chunk sizes and k values beyond the headline kernels: the matrix-core
kernels (chunk size a multiple of 32 without a lane-per-chunk kernel), the two-lanes-per-chunk
kernels (chunk 192 and 256) and the lane-per-chunk kernels of chunk 96 and 128, against the CPU
oracle with the staged protocol of tests/parity.py.  Every shard here has full tiles, tail
chunks that fall to the general kernels, and a ragged last chunk."""
import numpy as np
import pytest

import oracle
from oracle import Config
from paper_2502_06728_amd import synth
from tests import parity
from tests.test_gpu_parity import H, full_step, make_inputs  # noqa: F401  (fixture + helpers)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("s,k", [(32, 20), (64, 48), (96, 12), (96, 48), (128, 8), (128, 64),
                                 (160, 20), (192, 24), (224, 28), (256, 32), (256, 128)])
def test_every_chunk_size_of_the_matrix_core_path(H, s, k, bf16):
    n = s * (32 * 5 + 11) + s // 2 + 1          # 5 tiles, 11 tail chunks, a ragged chunk
    cfg = Config(chunk=s, topk=k, sign=True, decay=0.999, lr=1e-3)
    st_c, st_d = full_step(H, cfg, n, R=4, seed=s + k, grad_bf16=bf16, params_bf16=bf16,
                           outliers=0.01 if bf16 else 0.0)
    assert st_c["chunks"] == 32 * 5 + 12


@pytest.mark.parametrize("s,k", [(128, 1), (128, 127), (128, 128), (256, 1), (256, 256), (96, 96)])
def test_extreme_k(H, s, k):
    cfg = Config(chunk=s, topk=k, sign=False)
    full_step(H, cfg, s * 100 + 3, R=2, seed=k)


def test_many_tiles_per_workgroup(H):
    # more tiles than the persistent grid has workgroups at s = 256: every workgroup loops
    s, k = 256, 32
    tiles = 256 * 4 * 2 + 37
    n = s * 32 * tiles + 5
    cfg = Config(chunk=s, topk=k)
    g, m, th = make_inputs(n, 4)
    m_gpu, idx_gpu, val_gpu, coeff_gpu = H.gpu_compress(cfg, g, m)
    parity.check_compress(cfg, g, m, m_gpu, idx_gpu, val_gpu, coeff_gpu)
    th_gpu, y_gpu = H.gpu_decompress(cfg, idx_gpu[None], val_gpu[None], th)
    parity.check_decompress(cfg, idx_gpu[None], val_gpu[None], th, th_gpu, y_gpu)


def test_zero_and_single_spike_chunks_tie_on_magnitude(H):
    # zero chunks tie everywhere (the k lowest indices win); a chunk with one non-zero element
    # has coefficients of pairwise equal magnitude (|cos| is symmetric in the row index)
    s, k = 128, 16
    n = s * 96
    cfg = Config(chunk=s, topk=k, decay=0.0)
    g = np.zeros(n, np.float32)
    for c in range(0, 96, 3):
        g[c * s + (7 * c) % s] = 1.0 + c
    m = np.zeros(n, np.float32)
    m_gpu, idx_gpu, val_gpu, coeff_gpu = H.gpu_compress(cfg, g, m)
    parity.check_compress(cfg, g, m, m_gpu, idx_gpu, val_gpu, coeff_gpu)
    idx = idx_gpu.reshape(-1, k)
    assert np.array_equal(idx[1], np.arange(k))          # a zero chunk
    assert not m_gpu.reshape(-1, s)[1].any()


def test_duplicate_unordered_and_out_of_range_indices(H):
    s, k, n = 128, 12, 128 * 64
    cfg = Config(chunk=s, topk=k, sign=False)
    rng = np.random.default_rng(1)
    idx = rng.integers(-3, s + 3, size=(3, 64 * k)).astype(np.int32)
    idx[0, :k] = [5, 5, 5, 5, 128, -1, 7, 7, 127, 0, 0, 200]
    idx[1] = np.sort(idx[1].reshape(-1, k), axis=1).reshape(-1)      # ascending with repeats
    val = rng.standard_normal((3, 64 * k)).astype(np.float32)
    th = make_inputs(n, 3)[2]
    th_gpu, y_gpu = H.gpu_decompress(cfg, idx, val, th)
    parity.check_decompress(cfg, idx, val, th, th_gpu, y_gpu)


@pytest.mark.parametrize("val_dtype", [oracle.BF16, oracle.F16])
@pytest.mark.parametrize("idx_u8", [True, False])
@pytest.mark.parametrize("s,k", [(128, 16), (256, 32), (192, 12)])
def test_packed_payload_formats(H, val_dtype, idx_u8, s, k):
    n = s * 200 + 9
    cfg = Config(chunk=s, topk=k, sign=True, decay=0.999, lr=1e-3)
    g, m, th = make_inputs(n, seed=8, grad_bf16=True, params_bf16=True, outliers=0.01)
    m_gpu, idx_gpu, vbits_gpu, coeff_gpu = H.gpu_compress_packed(cfg, g, m, val_dtype, idx_u8)
    parity.check_compress_packed(cfg, g, m, m_gpu, idx_gpu, vbits_gpu, coeff_gpu, val_dtype)
    pays = [oracle.compress_q(cfg, *make_inputs(n, seed=700 + r, grad_bf16=True)[:2], val_dtype)[1:]
            for r in range(3)]
    idx = np.stack([p[0] for p in pays])
    vbits = np.stack([p[1] for p in pays])
    th_gpu, y_gpu = H.gpu_decompress_packed(cfg, idx, vbits, th, val_dtype, idx_u8)
    parity.check_decompress_packed(cfg, idx, vbits, val_dtype, th, th_gpu, y_gpu)


@pytest.mark.parametrize("amsgrad", [False, True])
@pytest.mark.parametrize("s,k", [(128, 64), (256, 32), (192, 24), (160, 20)])
def test_decoupled_adamw(H, amsgrad, s, k):
    import torch
    from paper_2502_06728_amd import binding
    n, R = s * 150 + 5, 2
    cfg = Config(chunk=s, topk=k, sign=True, lr=1e-3, weight_decay=0.01)
    th = make_inputs(n, 5)[2]
    p = H.to_dev(th)
    m = torch.zeros(n, device=H.DEV)
    v = torch.zeros(n, device=H.DEV)
    vm = torch.zeros(n, device=H.DEV) if amsgrad else None
    for t in (1, 2, 3):
        pays = [oracle.compress(cfg, *make_inputs(n, 100 * t + r)[:2])[1:] for r in range(R)]
        idx = np.stack([q[0] for q in pays])
        val = np.stack([q[1] for q in pays])
        th_in, m_in, v_in = H.to_host(p), m.cpu().numpy(), v.cpu().numpy()
        vm_in = vm.cpu().numpy() if amsgrad else None
        y = torch.empty(n, dtype=torch.float32, device=H.DEV)
        binding.detonation_decompress_adamw_step(
            H.bcfg(cfg), binding.AdamW(0.9, 0.95, 1e-8, amsgrad, t), R, H.to_dev(idx), H.to_dev(val),
            p, m, v, vm, y)
        torch.cuda.synchronize()
        y_gpu = H.to_host(y)
        assert parity.rel_chunk_err(y_gpu, oracle.presign(cfg, n, idx, val), s) <= parity.TOL_F32
        th_o, m_o, v_o, vm_o = oracle.adamw_update(cfg, oracle.AdamW(0.9, 0.95, 1e-8, amsgrad, t),
                                                   y_gpu, th_in, m_in, v_in, vm_in)
        assert np.abs(m.cpu().numpy() - m_o).max() <= 1e-5 * np.abs(m_o).max()
        assert np.abs(v.cpu().numpy() - v_o).max() <= 1e-5 * np.abs(v_o).max()
        if amsgrad:
            assert np.abs(vm.cpu().numpy() - vm_o).max() <= 1e-5 * np.abs(vm_o).max()
        got, want = H.to_host(p).astype(np.float64), th_o.astype(np.float64)
        assert (np.abs(got - want) <= parity.TOL_F32 * np.abs(want) + parity.TOL_F32 * cfg.lr).all()


@pytest.mark.size_dispatch
@pytest.mark.timeout(600)
@pytest.mark.parametrize("s,k", [(128, 64), (256, 32), (96, 12), (192, 24), (128, 16), (64, 20)])
def test_olmo_1b_shard_full_size_chunk_sweep(H, s, k):
    # the OLMo-1B shard (147,095,552 parameters) at the larger chunk sizes of the Appendix B
    # sweep, in the launch configuration bench.py --chunk/--topk times; sampled chunk runs
    # ((64, 20): a k the lane-per-chunk kernels are not instantiated for, so the two-class
    # kernels at full size)
    import dataclasses
    from tests.test_gpu_parity import _full_size_check, _sample_runs
    w = dataclasses.replace(synth.workloads()["olmo-1b-1of8"], chunk=s, topk=k)
    cfg = Config(chunk=s, topk=k, decay=w.decay, lr=w.lr, sign=w.sign)
    worst = _full_size_check(H, w, cfg, ranges=_sample_runs(-(-w.n // s), count=10))
    print(f"olmo-1b full size, chunk {s}, k {k}:", worst)
