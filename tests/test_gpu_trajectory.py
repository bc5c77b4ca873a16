"""Long trajectories: Algorithm 1 is iterative, so single-step parity does not show how errors
accumulate.  T = 50 optimizer steps of compress -> (exchange) -> decompress with evolving state
on the GPU, every step judged from the GPU's own state by the staged protocol, the momentum's
energy book-kept, and a free-running oracle trajectory beside it to bound the drift.

Two settings: DeMo-SGD with fp32 payloads on bf16 gradients and parameters (the benchmark's
storage types), and the setting of the paper's own experiments ("Overall Setup", "Decoupled
AdamW"): chunk size 32, only the signs of the kept components on the wire, Decoupled AdamW as
the underlying optimizer, top-k and Random."""
import numpy as np
import pytest

import oracle
from oracle import Config, SCHEME_RANDOM, SCHEME_STRIDE, SCHEME_TOPK
from paper_2502_06728_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

T_STEPS = 50


@pytest.fixture(scope="module")
def H(gpu):
    from tests import gpu_harness
    from paper_2502_06728_amd import binding
    binding.load()
    return gpu_harness


def _bf16(a):
    return synth.to_bf16_bits(a)


def _f32(bits):
    return synth.from_bf16_bits(bits)


def _energy_check(cfg, g, m_in, m_out, kept, n):
    """Nothing lost, nothing made up: over the complete chunks the folded momentum's energy is
    the residual's plus the extracted components' (orthonormal transform, or plain selection)."""
    s, k = cfg.chunk, cfg.topk
    nf, cf = (n // s) * s, n // s
    m1 = oracle.fold(cfg, g, m_in).astype(np.float64)[:nf]
    e_in = (m1 ** 2).sum()
    e_out = (m_out[:nf].astype(np.float64) ** 2).sum() + (kept[:cf * k].astype(np.float64) ** 2).sum()
    assert abs(e_in - e_out) < 1e-5 * e_in, (e_in, e_out)


@pytest.mark.parametrize("scheme", [SCHEME_TOPK, SCHEME_STRIDE, SCHEME_RANDOM])
def test_fifty_steps_demo_sgd_bf16_storage(H, scheme):
    """DeMo-SGD, chunk 64, k 16, fp32 payload, bf16 gradients and parameters, two replicas: the
    other replica lives in the oracle.  Per step: staged parity of both halves from the GPU's
    state, energy bookkeeping; at the end: drift of a free-running oracle."""
    n, s, k = 64 * 1100 + 21, 64, 16
    rng = np.random.default_rng(17)
    m_gpu = synth.normal(3, synth.TAG_MOMENTUM, n, 1e-3)
    th_gpu = _bf16(synth.normal(3, synth.TAG_PARAMS, n, 0.02))
    m_free, th_free = m_gpu.copy(), th_gpu.copy()
    m_other = synth.normal(4, synth.TAG_MOMENTUM, n, 1e-3)
    send_idx = scheme == SCHEME_TOPK
    worst = {"coeff": 0.0, "momentum": 0.0, "presign": 0.0, "flips": 0, "sign_flips": 0}
    for step in range(T_STEPS):
        cfg = Config(chunk=s, topk=k, scheme=scheme, seed=5, step=step, decay=0.9, lr=1e-3,
                     sign=True)
        g = _bf16((rng.standard_normal(n) * 1e-3).astype(np.float32))
        g_other = _bf16((rng.standard_normal(n) * 1e-3).astype(np.float32))
        m_other, idx_o, val_o = oracle.compress(cfg, g_other, m_other)
        m_new, idx_g, val_g, coeff_g = H.gpu_compress(cfg, g, m_gpu, want_idx=send_idx)
        st = parity.check_compress(cfg, g, m_gpu, m_new, idx_g, val_g, coeff_g)
        _energy_check(cfg, g, m_gpu, m_new, val_g, n)
        val = np.stack([val_g, val_o])
        idx = np.stack([idx_g, idx_o]) if send_idx else None
        th_new, y = H.gpu_decompress(cfg, idx, val, th_gpu)
        sd = parity.check_decompress(cfg, idx, val, th_gpu, th_new, y)
        for key in ("coeff", "momentum"):
            worst[key] = max(worst[key], st[key])
        worst["presign"] = max(worst["presign"], sd["presign"])
        worst["flips"] += st["flips"]
        worst["sign_flips"] += sd["sign_flips_vs_oracle"]
        # the oracle running on its own, same gradients, same other replica
        m_free, idx_f, val_f = oracle.compress(cfg, g, m_free)
        th_free = oracle.decompress_step(cfg, np.stack([idx_f, idx_o]) if send_idx else None,
                                         np.stack([val_f, val_o]), th_free)
        m_gpu, th_gpu = m_new, th_new
    print("50 steps, scheme", scheme, worst)
    # the per-step errors do not grow along the trajectory (every step starts from the GPU's state)
    assert worst["coeff"] <= parity.TOL_F32 and worst["momentum"] <= parity.TOL_F32
    # drift: a flipped near-tie or sign moves single elements by a coefficient or 2*eta, and a
    # bf16 parameter by one rounding step; in the mean both trajectories stay together
    d_th = np.abs(_f32(th_free).astype(np.float64) - _f32(th_gpu).astype(np.float64))
    assert d_th.mean() < 1e-3 * 1e-3 * T_STEPS / 6
    assert (d_th > 0).mean() < 0.01                 # all but a few parameters are bit-identical
    assert np.abs(m_free - m_gpu).mean() < 1e-3 * np.abs(m_free).mean()


@pytest.mark.parametrize("params_bf16", [False, True])
@pytest.mark.parametrize("scheme,k", [(SCHEME_TOPK, 4), (SCHEME_RANDOM, 4), (SCHEME_TOPK, 1)])
def test_fifty_steps_in_the_papers_setting(H, scheme, k, params_bf16):
    """Chunk size 32, signs only on the wire (two bits per entry; byte indices under top-k, none
    under Random), Decoupled AdamW with local moments, three replicas of which two live in the
    oracle.  Per step: the compress half by the staged protocol (coefficients, selection,
    momentum, bit-exact sign words), the averaged signs before the update, the moments and the
    parameters from the GPU's own state."""
    import torch
    from paper_2502_06728_amd import binding
    n, s, R = 32 * 2100 + 13, 32, 3
    C = -(-n // s)
    rng = np.random.default_rng(23)
    send_idx = scheme == SCHEME_TOPK
    m_gpu = synth.normal(7, synth.TAG_MOMENTUM, n, 1e-3)
    th0 = synth.normal(7, synth.TAG_PARAMS, n, 0.02)
    th0 = _bf16(th0) if params_bf16 else th0
    p = H.to_dev(th0)
    ea = torch.zeros(n, device=H.DEV)
    es = torch.zeros(n, device=H.DEV)
    m_others = [synth.normal(8 + r, synth.TAG_MOMENTUM, n, 1e-3) for r in range(R - 1)]
    # the free-running oracle: its own momentum, parameters and moments
    m_free, th_free = m_gpu.copy(), th0.copy()
    ea_free, es_free = np.zeros(n, np.float32), np.zeros(n, np.float32)
    worst = {"coeff": 0.0, "momentum": 0.0, "presign": 0.0}
    for step in range(T_STEPS):
        t = step + 1
        cfg = Config(chunk=s, topk=k, scheme=scheme, seed=11, step=step, decay=0.999, lr=1e-3,
                     weight_decay=0.01, sign=True)
        opt_o = oracle.AdamW(0.9, 0.95, 1e-8, False, t)
        g = _bf16((rng.standard_normal(n) * 1e-3).astype(np.float32))
        others = []
        for r in range(R - 1):
            g_r = _bf16((rng.standard_normal(n) * 1e-3).astype(np.float32))
            m_others[r], idx_r, words_r = oracle.compress_t(cfg, g_r, m_others[r])
            others.append((idx_r, words_r))
        # compress on the GPU
        m_new, idx_g, words_g, coeff_g = H.gpu_compress_ternary(cfg, g, m_gpu, True)
        kept = coeff_g.reshape(C, s)[np.arange(C)[:, None], idx_g.reshape(C, k)].reshape(-1)
        st = parity.check_compress(cfg, g, m_gpu, m_new, idx_g, kept, coeff_g)
        assert np.array_equal(words_g, oracle.encode_ternary(cfg, n, kept))
        _energy_check(cfg, g, m_gpu, m_new, kept, n)
        # exchange and Decoupled AdamW on the GPU
        idx = np.stack([idx_g] + [o[0] for o in others])
        words = np.stack([words_g] + [o[1] for o in others])
        idx_dev = (torch.from_numpy(np.ascontiguousarray(idx.astype(np.uint8))).to(H.DEV)
                   if send_idx else None)
        words_dev = torch.from_numpy(np.ascontiguousarray(words).view(np.int32)).to(H.DEV)
        th_in, ea_in, es_in = H.to_host(p), ea.cpu().numpy(), es.cpu().numpy()
        y = torch.empty(n, dtype=torch.float32, device=H.DEV)
        binding.detonation_decompress_adamw_step_packed(
            H.bcfg(cfg), binding.AdamW(0.9, 0.95, 1e-8, False, t), R, idx_dev, words_dev, p, ea, es,
            None, y)
        torch.cuda.synchronize()
        y_gpu = H.to_host(y)
        y_o = oracle.presign_t(cfg, n, idx, words)
        scale = np.maximum(1.0, parity.parity_chunk_max(y_o, s))     # signs: magnitude 1
        e_y = parity.rel_chunk_err(y_gpu, y_o, s, scale=scale)
        assert e_y <= parity.TOL_F32
        th_o, ea_o, es_o, _ = oracle.adamw_update(cfg, opt_o, y_gpu, th_in, ea_in, es_in, None)
        assert np.abs(ea.cpu().numpy() - ea_o).max() <= 1e-5 * max(np.abs(ea_o).max(), 1e-30)
        assert np.abs(es.cpu().numpy() - es_o).max() <= 1e-5 * max(np.abs(es_o).max(), 1e-30)
        got = H.to_host(p)
        if params_bf16:
            gotf, wantf, tol = _f32(got).astype(np.float64), _f32(th_o).astype(np.float64), parity.TOL_BF16
        else:
            gotf, wantf, tol = got.astype(np.float64), th_o.astype(np.float64), parity.TOL_F32
        assert (np.abs(gotf - wantf) <= tol * np.abs(wantf) + tol * cfg.lr).all()
        for key in ("coeff", "momentum"):
            worst[key] = max(worst[key], st[key])
        worst["presign"] = max(worst["presign"], e_y)
        # free-running oracle
        m_free, idx_f, words_f = oracle.compress_t(cfg, g, m_free)
        y_f = oracle.presign_t(cfg, n, np.stack([idx_f] + [o[0] for o in others]),
                               np.stack([words_f] + [o[1] for o in others]))
        th_free, ea_free, es_free, _ = oracle.adamw_update(cfg, opt_o, y_f, th_free, ea_free, es_free,
                                                           None)
        m_gpu = m_new
    print("50 steps, paper setting, scheme", scheme, "k", k, "bf16" if params_bf16 else "fp32", worst)
    assert worst["coeff"] <= parity.TOL_F32 and worst["momentum"] <= parity.TOL_F32
    th_end = H.to_host(p)
    a = (_f32(th_end) if params_bf16 else th_end).astype(np.float64)
    b = (_f32(th_free) if params_bf16 else th_free).astype(np.float64)
    # an AdamW step with sign input moves a parameter by about eta; T of them by at most T*eta.
    # The two trajectories differ where a near-tie or a sign flipped: small in the mean
    assert np.abs(a - b).mean() < 0.02 * T_STEPS * 1e-3
    assert np.abs(m_free - m_gpu).mean() < 1e-3 * np.abs(m_free).mean()
    assert np.abs(ea.cpu().numpy() - ea_free).mean() < 1e-2 * np.abs(ea_free).mean()
