"""Staged comparison of the GPU library's results with the CPU oracle's.

Floating point decides two discrete things on this path: which coefficients are kept
(top-k) and the sign of the averaged update.  A last-bit difference between the fp32
kernels and the double-precision oracle can flip either for a near-tie, after which
everything downstream differs by a whole coefficient or by 2*eta.  So each discrete
decision is judged by running the ORACLE's rule on the GPU's own floating-point values
(exported through the library's debug outputs), and the floating-point values
themselves are compared stage by stage:

  compress   (i)   coeff_gpu           vs oracle coefficients          (tolerance)
             (ii)  idx_gpu             == oracle selection on coeff_gpu (bit-exact)
             (iii) val_gpu             == coeff_gpu[idx_gpu]            (bit-exact)
                   momentum_gpu        vs oracle residual driven by coeff_gpu, idx_gpu
  decompress (iv)  presign_gpu         vs oracle y on the same payload bytes
             (v)   params_gpu          vs oracle update applied to presign_gpu

Tolerances (fp32 path): 1e-5 relative to the largest magnitude of the quantity in its
chunk; where the quantity is obtained by cancellation the scale is that of what cancels:
the chunk's folded momentum m1 for the residual momentum, and the chunk's largest payload
value for the averaged update (replicas can cancel each other).  Parameters: 1e-5 (fp32) or 1e-2 (bf16) relative, plus
the same fraction of eta.
"""
from __future__ import annotations

import numpy as np

import oracle

TOL_F32 = 1e-5
TOL_BF16 = 1e-2


def _chunk_max(a: np.ndarray, s: int) -> np.ndarray:
    """Per-element: the largest |a| within the element's chunk (a zero-padded to chunks)."""
    n = a.size
    C = -(-n // s)
    pad = np.zeros(C * s, dtype=np.float64)
    pad[:n] = np.abs(a)
    mx = pad.reshape(C, s).max(axis=1)
    return np.repeat(mx, s)[:n]


def parity_chunk_max(a: np.ndarray, s: int) -> np.ndarray:
    return _chunk_max(a.astype(np.float64), s)


def rel_chunk_err(got: np.ndarray, want: np.ndarray, s: int, scale: np.ndarray | None = None) -> float:
    """max over elements of |got-want| / (largest |scale| in the element's chunk)."""
    if got.size == 0:
        return 0.0
    ref = want if scale is None else scale
    den = np.maximum(_chunk_max(ref.astype(np.float64), s), 1e-30)
    return float((np.abs(got.astype(np.float64) - want.astype(np.float64)) / den).max())


def check_compress(cfg: oracle.Config, grad: np.ndarray, mom_in: np.ndarray, mom_gpu: np.ndarray,
                   idx_gpu, val_gpu: np.ndarray, coeff_gpu: np.ndarray, chunk0: int = 0,
                   tol: float = TOL_F32) -> dict:
    """grad/mom_in: the inputs (grad may be bf16 bits); *_gpu: what the library produced.
    chunk0: global number of the first chunk (keys the Random scheme).  Returns error stats;
    raises AssertionError on a parity failure."""
    s, k = cfg.chunk, cfg.topk
    n = mom_in.size
    m1 = oracle.fold(cfg, grad, mom_in)
    coeff_o = oracle.transform(cfg, m1)
    # (i) coefficients
    e_coeff = rel_chunk_err(coeff_gpu, coeff_o, s)
    assert e_coeff <= tol, f"coefficients differ: {e_coeff:.3e}"
    # (ii) the oracle's selection on the GPU's coefficients
    idx_stage = oracle.select(cfg, coeff_gpu, chunk0=chunk0)
    if idx_gpu is not None:
        assert np.array_equal(idx_gpu, idx_stage), "selected indices differ from the oracle's rule"
    # (iii) values are the kept coefficients; residual momentum
    val_stage, m_stage = oracle.extract(cfg, m1, coeff_gpu, idx_stage)
    assert np.array_equal(val_gpu.view(np.uint32), val_stage.view(np.uint32)), "payload values"
    e_mom = rel_chunk_err(mom_gpu, m_stage, s, scale=m1)
    assert e_mom <= tol, f"residual momentum differs: {e_mom:.3e}"
    # un-staged: how often does the oracle's own selection differ, and only on near-ties?
    idx_own = oracle.select(cfg, coeff_o, chunk0=chunk0)
    diff = (idx_own.reshape(-1, k) != idx_stage.reshape(-1, k)).any(axis=1)
    flips = int(diff.sum())
    if flips:
        co = np.abs(coeff_o.reshape(-1, s)[diff].astype(np.float64))
        srt = -np.sort(-co, axis=1)
        if k < s:
            # the kept/dropped boundary of a flipped chunk must be a near-tie
            a = np.take_along_axis(co, idx_own.reshape(-1, k)[diff], 1)
            b = np.take_along_axis(co, idx_stage.reshape(-1, k)[diff], 1)
            gap = np.abs(np.sort(a, 1) - np.sort(b, 1)).max(axis=1)
            assert (gap <= 4 * tol * srt[:, 0] + 1e-30).all(), "selection differs beyond a near-tie"
    # strict (un-staged) momentum error, reported only
    _, m_own = oracle.extract(cfg, m1, coeff_o, idx_own)
    e_mom_own = rel_chunk_err(mom_gpu[: n], m_own, s, scale=m1) if not flips else float("nan")
    return {"coeff": e_coeff, "momentum": e_mom, "momentum_unstaged": e_mom_own, "flips": flips,
            "chunks": coeff_o.size // s}


def check_decompress(cfg: oracle.Config, idx, val: np.ndarray, params_in: np.ndarray,
                     params_gpu: np.ndarray, presign_gpu: np.ndarray, tol: float = TOL_F32) -> dict:
    """idx/val: the payload bytes both sides were given ([R, C*k]); params as fp32 or bf16 bits."""
    s = cfg.chunk
    n = params_in.size
    y_o = oracle.presign(cfg, n, idx, val)
    # (iv) averaged update before sign; scale: the larger of the chunk's result and the
    # chunk's largest payload value (the sum over replicas can cancel)
    k = cfg.topk
    C = -(-n // s)
    vmax = np.abs(np.asarray(val, dtype=np.float64).reshape(-1, C, k)).max(axis=(0, 2))
    scale = np.maximum(np.repeat(vmax, s)[:n], parity_chunk_max(y_o, s))
    e_y = rel_chunk_err(presign_gpu, y_o, s, scale=scale)
    assert e_y <= tol, f"pre-sign update differs: {e_y:.3e}"
    # (v) the oracle's sign + update on the GPU's pre-sign values
    p_stage = oracle.update(cfg, presign_gpu, params_in)
    if params_in.dtype == np.uint16:
        got = (params_gpu.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        want = (p_stage.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        ptol = TOL_BF16
    else:
        got, want, ptol = params_gpu.astype(np.float64), p_stage.astype(np.float64), tol
    err = np.abs(got - want)
    bound = ptol * np.abs(want) + ptol * abs(cfg.lr)
    assert (err <= bound).all(), f"parameters differ: max {err.max():.3e}"
    exact = float((params_gpu == p_stage).mean()) if n else 1.0
    sign_flips = int((np.sign(presign_gpu) != np.sign(y_o)).sum())
    return {"presign": e_y, "params_max_err": float(err.max()) if n else 0.0,
            "params_bit_exact_frac": exact, "sign_flips_vs_oracle": sign_flips}


def check_compress_packed(cfg: oracle.Config, grad, mom_in, mom_gpu, idx_gpu, val_bits_gpu,
                          coeff_gpu, val_dtype: int, tol: float = TOL_F32) -> dict:
    """Staged check of the compress half with 16-bit payload values: coefficients, the oracle's
    selection on the GPU's coefficients, bit-exact encoded values, and the residual that removes
    what the receivers decode."""
    s = cfg.chunk
    m1 = oracle.fold(cfg, grad, mom_in)
    coeff_o = oracle.transform(cfg, m1)
    e_coeff = rel_chunk_err(coeff_gpu, coeff_o, s)
    assert e_coeff <= tol, f"coefficients differ: {e_coeff:.3e}"
    idx_stage = oracle.select(cfg, coeff_gpu)
    assert np.array_equal(idx_gpu, idx_stage), "selected indices differ from the oracle's rule"
    val_stage, m_stage = oracle.extract_q(cfg, m1, coeff_gpu, idx_stage, val_dtype)
    assert np.array_equal(val_bits_gpu, val_stage), "encoded payload values"
    e_mom = rel_chunk_err(mom_gpu, m_stage, s, scale=m1)
    assert e_mom <= tol, f"residual momentum differs: {e_mom:.3e}"
    return {"coeff": e_coeff, "momentum": e_mom}


def check_decompress_packed(cfg: oracle.Config, idx, val_bits, val_dtype, params_in, params_gpu,
                            presign_gpu, tol: float = TOL_F32) -> dict:
    s, k = cfg.chunk, cfg.topk
    n = params_in.size
    C = -(-n // s)
    y_o = oracle.presign_q(cfg, n, idx, val_bits, val_dtype)
    dec = ((val_bits.astype(np.uint32) << 16).view(np.float32) if val_dtype == oracle.BF16
           else val_bits.view(np.float16).astype(np.float32))
    vmax = np.abs(dec.astype(np.float64).reshape(-1, C, k)).max(axis=(0, 2))
    scale = np.maximum(np.repeat(vmax, s)[:n], parity_chunk_max(y_o, s))
    e_y = rel_chunk_err(presign_gpu, y_o, s, scale=scale)
    assert e_y <= tol, f"pre-sign update differs: {e_y:.3e}"
    p_stage = oracle.update(cfg, presign_gpu, params_in)
    if params_in.dtype == np.uint16:
        got = (params_gpu.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        want = (p_stage.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        ptol = TOL_BF16
    else:
        got, want, ptol = params_gpu.astype(np.float64), p_stage.astype(np.float64), tol
    err = np.abs(got - want)
    assert (err <= ptol * np.abs(want) + ptol * abs(cfg.lr)).all(), f"parameters differ: {err.max():.3e}"
    return {"presign": e_y}
