"""CPU oracle for the FlexDeMo / DeMo-SGD optimizer step (arXiv 2502.06728, Algorithm 1).

TEST INFRASTRUCTURE ONLY.  This package wraps ``detonation_oracle.c`` (plain C,
double arithmetic) with numpy in/out.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the GPU library never does, and the two
share no code.  bf16 arrays are carried as ``numpy.uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "detonation_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

SCHEME_TOPK, SCHEME_STRIDE, SCHEME_RANDOM = 0, 1, 2
F32, BF16, F16, TERNARY = 0, 1, 2, 3
FLAG_SIGN, FLAG_DCT = 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (+OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Config(ctypes.Structure):
    _fields_ = [("chunk", ctypes.c_int32), ("topk", ctypes.c_int32), ("scheme", ctypes.c_int32),
                ("flags", ctypes.c_uint32), ("decay", ctypes.c_float), ("lr", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("seed", ctypes.c_uint64),
                ("step", ctypes.c_uint64)]


@dataclass
class Config:
    """Hyper-parameters of Algorithm 1 plus the replication scheme."""
    chunk: int = 64
    topk: int = 8
    scheme: int = SCHEME_TOPK
    sign: bool = True
    dct: bool = False          # coefficient-domain variant of Striding / Random
    decay: float = 0.999
    lr: float = 1e-3
    weight_decay: float = 0.0
    seed: int = 0
    step: int = 0

    def c(self) -> _Config:
        flags = (FLAG_SIGN if self.sign else 0) | (FLAG_DCT if self.dct else 0)
        return _Config(self.chunk, self.topk, self.scheme, flags, self.decay, self.lr,
                       self.weight_decay, self.seed, self.step)

    @property
    def uses_dct(self) -> bool:
        return self.scheme == SCHEME_TOPK or self.dct


class _AdamW(ctypes.Structure):
    _fields_ = [("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("amsgrad", ctypes.c_int32), ("step", ctypes.c_uint64)]


@dataclass
class AdamW:
    """Decoupled AdamW hyper-parameters (moments are local, never synchronised)."""
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    amsgrad: bool = False
    step: int = 1

    def c(self) -> _AdamW:
        return _AdamW(self.beta1, self.beta2, self.eps, int(self.amsgrad), self.step)


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_threads.restype = ctypes.c_int
        _lib.orc_double_to_bf16.restype = ctypes.c_uint16
        _lib.orc_double_to_bf16.argtypes = [ctypes.c_double]
        _lib.orc_float_to_f16.restype = ctypes.c_uint16
        _lib.orc_float_to_f16.argtypes = [ctypes.c_float]
        _lib.orc_f16_to_float.restype = ctypes.c_float
        _lib.orc_f16_to_float.argtypes = [ctypes.c_uint16]
        _lib.orc_ternary_words.restype = ctypes.c_int64
    return _lib


def threads() -> int:
    return int(lib().orc_threads())


def set_threads(t: int) -> None:
    lib().orc_set_threads(ctypes.c_int(t))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(rc: int) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle returned status {rc}")


def _dtype_of(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"expected float32 or uint16 (bf16 bits), got {a.dtype}")


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def n_chunks(cfg: Config, n: int) -> int:
    return (n + cfg.chunk - 1) // cfg.chunk


def double_to_bf16(v: float) -> int:
    return int(lib().orc_double_to_bf16(float(v)))


def float_to_f16(v: float) -> int:
    return int(lib().orc_float_to_f16(float(v)))


def f16_to_float(bits: int) -> float:
    return float(lib().orc_f16_to_float(int(bits)))


def dct_matrix(s: int) -> np.ndarray:
    D = np.empty((s, s), dtype=np.float64)
    _chk(lib().orc_dct_matrix(ctypes.c_int32(s), _p(D)))
    return D


def fold(cfg: Config, grad: np.ndarray, m: np.ndarray) -> np.ndarray:
    grad = np.ascontiguousarray(grad)
    m = _c(m, np.float32)
    m1 = np.empty_like(m)
    _chk(lib().orc_fold(ctypes.byref(cfg.c()), ctypes.c_int64(m.size), _p(grad),
                        ctypes.c_int(_dtype_of(grad)), _p(m), _p(m1)))
    return m1


def transform(cfg: Config, x: np.ndarray) -> np.ndarray:
    x = _c(x, np.float32)
    C = n_chunks(cfg, x.size)
    coeff = np.empty(C * cfg.chunk, dtype=np.float32)
    _chk(lib().orc_transform(ctypes.byref(cfg.c()), ctypes.c_int64(x.size), _p(x), _p(coeff)))
    return coeff


def select(cfg: Config, coeff, n_chunks_: int | None = None, chunk0: int = 0) -> np.ndarray:
    if coeff is not None:
        coeff = _c(coeff, np.float32)
        C = coeff.size // cfg.chunk
    else:
        C = int(n_chunks_)
    idx = np.empty(C * cfg.topk, dtype=np.int32)
    _chk(lib().orc_select(ctypes.byref(cfg.c()), ctypes.c_int64(C), ctypes.c_int64(chunk0),
                          _p(coeff), _p(idx)))
    return idx


def extract(cfg: Config, m1: np.ndarray, coeff: np.ndarray, idx: np.ndarray):
    m1 = _c(m1, np.float32)
    coeff = _c(coeff, np.float32)
    idx = _c(idx, np.int32)
    val = np.empty(idx.size, dtype=np.float32)
    m_new = np.empty_like(m1)
    _chk(lib().orc_extract(ctypes.byref(cfg.c()), ctypes.c_int64(m1.size), _p(m1), _p(coeff),
                           _p(idx), _p(val), _p(m_new)))
    return val, m_new


def extract_q(cfg: Config, m1: np.ndarray, coeff: np.ndarray, idx: np.ndarray, val_dtype: int):
    """Payload values in a 16-bit transfer dtype (uint16 bit patterns) and the residual momentum
    that removes exactly what the receivers decode."""
    m1 = _c(m1, np.float32)
    coeff = _c(coeff, np.float32)
    idx = _c(idx, np.int32)
    val = np.empty(idx.size, dtype=np.uint16)
    m_new = np.empty_like(m1)
    _chk(lib().orc_extract_q(ctypes.byref(cfg.c()), ctypes.c_int64(m1.size), _p(m1), _p(coeff),
                             _p(idx), ctypes.c_int(val_dtype), _p(val), _p(m_new)))
    return val, m_new


def compress_q(cfg: Config, grad: np.ndarray, momentum: np.ndarray, val_dtype: int):
    """Compress half with 16-bit payload values: the steps in order.  Returns (m_new, idx, val_bits)."""
    m1 = fold(cfg, grad, momentum)
    coeff = transform(cfg, m1)
    idx = select(cfg, coeff)
    val, m_new = extract_q(cfg, m1, coeff, idx, val_dtype)
    return m_new, idx, val


def presign_q(cfg: Config, n: int, idx, val_bits: np.ndarray, val_dtype: int) -> np.ndarray:
    val_bits = _c(val_bits, np.uint16)
    if val_bits.ndim == 1:
        val_bits = val_bits[None, :]
    R = val_bits.shape[0]
    if idx is not None:
        idx = _c(idx, np.int32).reshape(R, -1)
    y = np.empty(n, dtype=np.float32)
    _chk(lib().orc_presign_q(ctypes.byref(cfg.c()), ctypes.c_int64(n), ctypes.c_int32(R), _p(idx),
                             ctypes.c_int64(0 if idx is None else idx.shape[1]), _p(val_bits),
                             ctypes.c_int(val_dtype), ctypes.c_int64(val_bits.shape[1]), _p(y)))
    return y


def ternary_words(cfg: Config, n: int) -> int:
    """32-bit words of one replica's ternary payload: chunks * ceil(k/16)."""
    return int(lib().orc_ternary_words(ctypes.byref(cfg.c()), ctypes.c_int64(n)))


def encode_ternary(cfg: Config, n: int, val: np.ndarray) -> np.ndarray:
    """sign(val) packed two bits per entry (0, 1 = +1, 3 = -1), each chunk on a word boundary."""
    val = _c(val, np.float32)
    words = np.empty(ternary_words(cfg, n), dtype=np.uint32)
    _chk(lib().orc_encode_ternary(ctypes.byref(cfg.c()), ctypes.c_int64(n), _p(val), _p(words)))
    return words


def decode_ternary(cfg: Config, n: int, words: np.ndarray) -> np.ndarray:
    words = _c(words, np.uint32)
    val = np.empty(n_chunks(cfg, n) * cfg.topk, dtype=np.float32)
    _chk(lib().orc_decode_ternary(ctypes.byref(cfg.c()), ctypes.c_int64(n), _p(words), _p(val)))
    return val


def compress_t(cfg: Config, grad: np.ndarray, momentum: np.ndarray):
    """Compress half with the ternary payload: the steps of compress(), then only the signs of
    the kept values travel.  Returns (m_new, idx, words); the momentum is that of compress()."""
    m_new, idx, val = compress(cfg, grad, momentum)
    return m_new, idx, encode_ternary(cfg, np.asarray(momentum).size, val)


def presign_t(cfg: Config, n: int, idx, words: np.ndarray) -> np.ndarray:
    words = _c(words, np.uint32)
    if words.ndim == 1:
        words = words[None, :]
    R = words.shape[0]
    if idx is not None:
        idx = _c(idx, np.int32).reshape(R, -1)
    y = np.empty(n, dtype=np.float32)
    _chk(lib().orc_presign_t(ctypes.byref(cfg.c()), ctypes.c_int64(n), ctypes.c_int32(R), _p(idx),
                             ctypes.c_int64(0 if idx is None else idx.shape[1]), _p(words),
                             ctypes.c_int64(words.shape[1]), _p(y)))
    return y


def compress(cfg: Config, grad: np.ndarray, momentum: np.ndarray, want_coeff: bool = False):
    """Returns (m_new, idx, val[, coeff]); inputs are not modified."""
    grad = np.ascontiguousarray(grad)
    m = _c(momentum, np.float32).copy()
    C = n_chunks(cfg, m.size)
    idx = np.empty(C * cfg.topk, dtype=np.int32)
    val = np.empty(C * cfg.topk, dtype=np.float32)
    coeff = np.empty(C * cfg.chunk, dtype=np.float32) if want_coeff else None
    _chk(lib().orc_compress(ctypes.byref(cfg.c()), ctypes.c_int64(m.size), _p(grad),
                            ctypes.c_int(_dtype_of(grad)), _p(m), _p(idx), _p(val), _p(coeff)))
    return (m, idx, val, coeff) if want_coeff else (m, idx, val)


def presign(cfg: Config, n: int, idx, val: np.ndarray) -> np.ndarray:
    """idx, val are [R, C*k] (idx may be None for Striding/Random)."""
    val = _c(val, np.float32)
    if val.ndim == 1:
        val = val[None, :]
    R = val.shape[0]
    if idx is not None:
        idx = _c(idx, np.int32).reshape(R, -1)
    y = np.empty(n, dtype=np.float32)
    _chk(lib().orc_presign(ctypes.byref(cfg.c()), ctypes.c_int64(n), ctypes.c_int32(R), _p(idx),
                           ctypes.c_int64(0 if idx is None else idx.shape[1]), _p(val),
                           ctypes.c_int64(val.shape[1]), _p(y)))
    return y


def update(cfg: Config, y: np.ndarray, params: np.ndarray) -> np.ndarray:
    y = _c(y, np.float32)
    p = np.ascontiguousarray(params).copy()
    _chk(lib().orc_update(ctypes.byref(cfg.c()), ctypes.c_int64(y.size), _p(y), _p(p),
                          ctypes.c_int(_dtype_of(p))))
    return p


def decompress_step(cfg: Config, idx, val: np.ndarray, params: np.ndarray,
                    want_presign: bool = False):
    """Returns new params (and the pre-sign update y); inputs are not modified."""
    val = _c(val, np.float32)
    if val.ndim == 1:
        val = val[None, :]
    R = val.shape[0]
    if idx is not None:
        idx = _c(idx, np.int32).reshape(R, -1)
    p = np.ascontiguousarray(params).copy()
    n = p.size
    y = np.empty(n, dtype=np.float32) if want_presign else None
    _chk(lib().orc_decompress_step(ctypes.byref(cfg.c()), ctypes.c_int64(n), ctypes.c_int32(R),
                                   _p(idx), ctypes.c_int64(0 if idx is None else idx.shape[1]),
                                   _p(val), ctypes.c_int64(val.shape[1]), _p(p),
                                   ctypes.c_int(_dtype_of(p)), _p(y)))
    return (p, y) if want_presign else p


def adamw_update(cfg: Config, opt: AdamW, y: np.ndarray, params: np.ndarray, exp_avg: np.ndarray,
                 exp_avg_sq: np.ndarray, max_exp_avg_sq=None):
    """One Decoupled-AdamW parameter step driven by the averaged update y.  Returns new
    (params, exp_avg, exp_avg_sq, max_exp_avg_sq); inputs are not modified."""
    y = _c(y, np.float32)
    p = np.ascontiguousarray(params).copy()
    m = _c(exp_avg, np.float32).copy()
    v = _c(exp_avg_sq, np.float32).copy()
    vm = None if max_exp_avg_sq is None else _c(max_exp_avg_sq, np.float32).copy()
    _chk(lib().orc_adamw_update(ctypes.byref(cfg.c()), ctypes.byref(opt.c()), ctypes.c_int64(y.size),
                                _p(y), _p(p), ctypes.c_int(_dtype_of(p)), _p(m), _p(v), _p(vm)))
    return p, m, v, vm
