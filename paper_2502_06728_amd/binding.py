"""ctypes binding of the C-ABI library (include/detonation.h).

Argument marshalling only: device tensors in, raw pointers out; every step of the path
runs in the HIP kernels.  There is no CPU fallback — if the library has not been built
the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
# DETONATION_LIB points the binding at another build of the same library
LIB_PATH = os.environ.get("DETONATION_LIB", os.path.join(_HERE, "libdetonation.so"))

SCHEME_TOPK, SCHEME_STRIDE, SCHEME_RANDOM = 0, 1, 2
F32, BF16, F16, TERNARY = 0, 1, 2, 3
IDX_I32, IDX_U8 = 0, 1
FLAG_SIGN, FLAG_DCT = 1, 2

EXPORTS = ("detonation_compress", "detonation_decompress_step", "detonation_compress_packed",
           "detonation_accumulate",
           "detonation_decompress_step_packed", "detonation_decompress_adamw_step",
           "detonation_decompress_adamw_step_packed",
           "detonation_payload_entries", "detonation_ternary_words",
           "detonation_status_string", "detonation_version")


class deto_config(ctypes.Structure):
    _fields_ = [("chunk", ctypes.c_int32), ("topk", ctypes.c_int32), ("scheme", ctypes.c_int32),
                ("flags", ctypes.c_uint32), ("decay", ctypes.c_float), ("lr", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("seed", ctypes.c_uint64),
                ("step", ctypes.c_uint64)]


class deto_adamw(ctypes.Structure):
    _fields_ = [("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("amsgrad", ctypes.c_int32), ("step", ctypes.c_uint64)]


@dataclass
class AdamW:
    """Host-side mirror of deto_adamw (Decoupled AdamW: local, never synchronised moments)."""
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    amsgrad: bool = False
    step: int = 1

    def c(self) -> deto_adamw:
        return deto_adamw(self.beta1, self.beta2, self.eps, int(self.amsgrad), self.step)


@dataclass
class Config:
    """Host-side mirror of deto_config (Algorithm 1's eta, beta, s, k plus scheme and flags)."""
    chunk: int = 64
    topk: int = 8
    scheme: int = SCHEME_TOPK
    sign: bool = True
    dct: bool = False
    decay: float = 0.999
    lr: float = 1e-3
    weight_decay: float = 0.0
    seed: int = 0
    step: int = 0

    def c(self) -> deto_config:
        flags = (FLAG_SIGN if self.sign else 0) | (FLAG_DCT if self.dct else 0)
        return deto_config(self.chunk, self.topk, self.scheme, flags, self.decay, self.lr,
                           self.weight_decay, self.seed, self.step)


class DetonationError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"detonation status {status}: {status_string(status)}")


_lib = None


def load() -> ctypes.CDLL:
    """Load libdetonation.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2502_06728_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        cfgp = ctypes.POINTER(deto_config)
        lib.detonation_compress.argtypes = [cfgp, i64, vp, ctypes.c_int, vp, vp, vp, vp, vp]
        lib.detonation_compress.restype = ctypes.c_int
        lib.detonation_decompress_step.argtypes = [cfgp, i64, i32, vp, i64, vp, i64, vp,
                                                   ctypes.c_int, vp, vp]
        lib.detonation_decompress_step.restype = ctypes.c_int
        lib.detonation_compress_packed.argtypes = [cfgp, i64, vp, ctypes.c_int, vp, vp, ctypes.c_int,
                                                   vp, ctypes.c_int, vp, vp]
        lib.detonation_compress_packed.restype = ctypes.c_int
        lib.detonation_decompress_step_packed.argtypes = [cfgp, i64, i32, vp, ctypes.c_int, i64, vp,
                                                          ctypes.c_int, i64, vp, ctypes.c_int, vp, vp]
        lib.detonation_decompress_step_packed.restype = ctypes.c_int
        lib.detonation_decompress_adamw_step.argtypes = [cfgp, ctypes.POINTER(deto_adamw), i64, i32,
                                                         vp, i64, vp, i64, vp, ctypes.c_int, vp,
                                                         vp, vp, vp, vp]
        lib.detonation_decompress_adamw_step.restype = ctypes.c_int
        lib.detonation_decompress_adamw_step_packed.argtypes = [
            cfgp, ctypes.POINTER(deto_adamw), i64, i32, vp, ctypes.c_int, i64, vp, ctypes.c_int,
            i64, vp, ctypes.c_int, vp, vp, vp, vp, vp]
        lib.detonation_decompress_adamw_step_packed.restype = ctypes.c_int
        lib.detonation_accumulate.argtypes = [cfgp, i64, vp, ctypes.c_int, vp, vp]
        lib.detonation_accumulate.restype = ctypes.c_int
        lib.detonation_payload_entries.argtypes = [cfgp, i64]
        lib.detonation_payload_entries.restype = i64
        lib.detonation_ternary_words.argtypes = [cfgp, i64]
        lib.detonation_ternary_words.restype = i64
        lib.detonation_status_string.argtypes = [ctypes.c_int]
        lib.detonation_status_string.restype = ctypes.c_char_p
        lib.detonation_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().detonation_status_string(int(status)).decode()


def version() -> int:
    return int(load().detonation_version())


def payload_entries(cfg: Config, n: int) -> int:
    return int(load().detonation_payload_entries(ctypes.byref(cfg.c()), n))


def ternary_words(cfg: Config, n: int) -> int:
    return int(load().detonation_ternary_words(ctypes.byref(cfg.c()), n))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dtype(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _val_dtype(t) -> int:
    """Payload value format from the tensor's dtype; an int32 tensor holds ternary words."""
    import torch
    return TERNARY if t.dtype == torch.int32 else _dtype(t)


def _idx_dtype(t) -> int:
    import torch
    if t is None or t.dtype == torch.int32:
        return IDX_I32
    if t.dtype == torch.uint8:
        return IDX_U8
    raise TypeError(f"unsupported index dtype {t.dtype}")


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    h = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    return ctypes.c_void_p(h)


def _check(*tensors):
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def _need(t, name: str, dtypes, numel: int, optional: bool = False) -> None:
    """A wrong element type or a short buffer would become an out-of-bounds access on the
    device: refuse it here, on the host."""
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} is required")
    if t.dtype not in dtypes:
        raise ValueError(f"{name}: dtype {t.dtype}, expected one of {[str(d) for d in dtypes]}")
    if t.numel() < numel:
        raise ValueError(f"{name}: {t.numel()} elements, at least {numel} needed")


def _n_chunks(cfg: Config, n: int) -> int:
    return (n + cfg.chunk - 1) // cfg.chunk


def _check_compress(cfg, n, grad, momentum, idx_out, val_out, coeff_dbg, packed: bool) -> None:
    import torch
    if n < 0:
        raise ValueError("n must not be negative")
    entries = _n_chunks(cfg, n) * cfg.topk
    _need(grad, "grad", (torch.float32, torch.bfloat16), n)
    _need(momentum, "momentum", (torch.float32,), n)
    _need(coeff_dbg, "coeff_dbg", (torch.float32,), _n_chunks(cfg, n) * cfg.chunk, optional=True)
    idx_types = (torch.int32, torch.uint8) if packed else (torch.int32,)
    _need(idx_out, "idx_out", idx_types, entries, optional=cfg.scheme != SCHEME_TOPK)
    if packed and val_out is not None and val_out.dtype == torch.int32:
        _need(val_out, "val_out", (torch.int32,), _n_chunks(cfg, n) * ((cfg.topk + 15) // 16))
    else:
        val_types = ((torch.float32, torch.bfloat16, torch.float16) if packed
                     else (torch.float32,))
        _need(val_out, "val_out", val_types, entries)


def _check_decompress(cfg, n, R, idx, istr, val, vs, params, presign_dbg, packed: bool,
                      moments=()) -> None:
    import torch
    if n < 0 or R < 1:
        raise ValueError("n must not be negative and R must be at least 1")
    C = _n_chunks(cfg, n)
    entries = C * cfg.topk
    ternary = packed and val is not None and val.dtype == torch.int32
    val_elems = C * ((cfg.topk + 15) // 16) if ternary else entries
    if R > 1 and (vs < val_elems or (idx is not None and istr < entries)):
        raise ValueError("a replica stride is shorter than one replica's payload")
    idx_types = (torch.int32, torch.uint8) if packed else (torch.int32,)
    _need(idx, "idx", idx_types, (R - 1) * istr + entries, optional=cfg.scheme != SCHEME_TOPK)
    val_types = ((torch.float32, torch.bfloat16, torch.float16, torch.int32) if packed
                 else (torch.float32,))
    _need(val, "val", val_types, (R - 1) * vs + val_elems)
    _need(params, "params", (torch.float32, torch.bfloat16), n)
    _need(presign_dbg, "presign_dbg", (torch.float32,), n, optional=True)
    for name, t, optional in moments:
        _need(t, name, (torch.float32,), n, optional=optional)


def detonation_compress(cfg: Config, grad, momentum, idx_out, val_out, coeff_dbg=None,
                        stream=None, n: int | None = None) -> None:
    """Enqueue the compress half on `stream`.  momentum, idx_out, val_out (and coeff_dbg)
    are written in place by the kernels."""
    _check(grad, momentum, idx_out, val_out, coeff_dbg)
    n = momentum.numel() if n is None else n
    _check_compress(cfg, n, grad, momentum, idx_out, val_out, coeff_dbg, packed=False)
    rc = load().detonation_compress(ctypes.byref(cfg.c()), n, _ptr(grad), _dtype(grad),
                                    _ptr(momentum), _ptr(idx_out), _ptr(val_out),
                                    _ptr(coeff_dbg), _stream(stream))
    if rc != 0:
        raise DetonationError(rc)


def detonation_decompress_step(cfg: Config, R: int, idx, val, params, presign_dbg=None,
                               stream=None, n: int | None = None,
                               idx_replica_stride: int | None = None,
                               val_replica_stride: int | None = None) -> None:
    """Enqueue the decompress-and-update half on `stream`.  idx/val hold R payloads
    (replica r at offset r*stride); params is updated in place."""
    _check(idx, val, params, presign_dbg)
    n = params.numel() if n is None else n
    entries = payload_entries(cfg, n)
    vs = entries if val_replica_stride is None else val_replica_stride
    istr = entries if idx_replica_stride is None else idx_replica_stride
    _check_decompress(cfg, n, R, idx, istr, val, vs, params, presign_dbg, packed=False)
    rc = load().detonation_decompress_step(ctypes.byref(cfg.c()), n, R, _ptr(idx), istr, _ptr(val),
                                           vs, _ptr(params), _dtype(params), _ptr(presign_dbg),
                                           _stream(stream))
    if rc != 0:
        raise DetonationError(rc)


def detonation_accumulate(cfg: Config, grad, momentum, stream=None, n: int | None = None) -> None:
    """momentum <- beta*momentum + grad (Algorithm 1's first line alone; the steps of a DiLoCo
    cycle that do not synchronise)."""
    import torch
    _check(grad, momentum)
    n = momentum.numel() if n is None else n
    _need(grad, "grad", (torch.float32, torch.bfloat16), n)
    _need(momentum, "momentum", (torch.float32,), n)
    rc = load().detonation_accumulate(ctypes.byref(cfg.c()), n, _ptr(grad), _dtype(grad),
                                      _ptr(momentum), _stream(stream))
    if rc != 0:
        raise DetonationError(rc)


def detonation_compress_packed(cfg: Config, grad, momentum, idx_out, val_out, coeff_dbg=None,
                               stream=None, n: int | None = None) -> None:
    """Compress half with the payload format given by the output tensors' dtypes: indices
    int32 or uint8, values float32, bfloat16, float16, or int32 words of the ternary payload."""
    _check(grad, momentum, idx_out, val_out, coeff_dbg)
    n = momentum.numel() if n is None else n
    _check_compress(cfg, n, grad, momentum, idx_out, val_out, coeff_dbg, packed=True)
    rc = load().detonation_compress_packed(ctypes.byref(cfg.c()), n, _ptr(grad), _dtype(grad),
                                           _ptr(momentum), _ptr(idx_out), _idx_dtype(idx_out),
                                           _ptr(val_out), _val_dtype(val_out), _ptr(coeff_dbg),
                                           _stream(stream))
    if rc != 0:
        raise DetonationError(rc)


def detonation_decompress_step_packed(cfg: Config, R: int, idx, val, params, presign_dbg=None,
                                      stream=None, n: int | None = None,
                                      idx_replica_stride: int | None = None,
                                      val_replica_stride: int | None = None) -> None:
    """Decompress-and-update half for payloads in the format given by the tensors' dtypes."""
    _check(idx, val, params, presign_dbg)
    n = params.numel() if n is None else n
    entries = payload_entries(cfg, n)
    vdt = _val_dtype(val)
    vs = val_replica_stride
    if vs is None:
        vs = ternary_words(cfg, n) if vdt == TERNARY else entries
    istr = entries if idx_replica_stride is None else idx_replica_stride
    _check_decompress(cfg, n, R, idx, istr, val, vs, params, presign_dbg, packed=True)
    rc = load().detonation_decompress_step_packed(ctypes.byref(cfg.c()), n, R, _ptr(idx),
                                                  _idx_dtype(idx), istr, _ptr(val), vdt, vs,
                                                  _ptr(params), _dtype(params), _ptr(presign_dbg),
                                                  _stream(stream))
    if rc != 0:
        raise DetonationError(rc)


def detonation_decompress_adamw_step(cfg: Config, opt: AdamW, R: int, idx, val, params, exp_avg,
                                     exp_avg_sq, max_exp_avg_sq=None, presign_dbg=None,
                                     stream=None, n: int | None = None,
                                     idx_replica_stride: int | None = None,
                                     val_replica_stride: int | None = None) -> None:
    """Decompress half with Decoupled AdamW as the underlying optimizer; params and the moment
    tensors are updated in place."""
    _check(idx, val, params, exp_avg, exp_avg_sq, max_exp_avg_sq, presign_dbg)
    n = params.numel() if n is None else n
    entries = payload_entries(cfg, n)
    vs = entries if val_replica_stride is None else val_replica_stride
    istr = entries if idx_replica_stride is None else idx_replica_stride
    _check_decompress(cfg, n, R, idx, istr, val, vs, params, presign_dbg, packed=False,
                      moments=(("exp_avg", exp_avg, False), ("exp_avg_sq", exp_avg_sq, False),
                               ("max_exp_avg_sq", max_exp_avg_sq, not opt.amsgrad)))
    rc = load().detonation_decompress_adamw_step(ctypes.byref(cfg.c()), ctypes.byref(opt.c()), n, R,
                                                 _ptr(idx), istr, _ptr(val), vs, _ptr(params),
                                                 _dtype(params), _ptr(exp_avg), _ptr(exp_avg_sq),
                                                 _ptr(max_exp_avg_sq), _ptr(presign_dbg),
                                                 _stream(stream))
    if rc != 0:
        raise DetonationError(rc)


def detonation_decompress_adamw_step_packed(cfg: Config, opt: AdamW, R: int, idx, val, params,
                                            exp_avg, exp_avg_sq, max_exp_avg_sq=None,
                                            presign_dbg=None, stream=None, n: int | None = None,
                                            idx_replica_stride: int | None = None,
                                            val_replica_stride: int | None = None) -> None:
    """Decoupled AdamW on payloads in the format given by the tensors' dtypes."""
    _check(idx, val, params, exp_avg, exp_avg_sq, max_exp_avg_sq, presign_dbg)
    n = params.numel() if n is None else n
    entries = payload_entries(cfg, n)
    vdt = _val_dtype(val)
    vs = val_replica_stride
    if vs is None:
        vs = ternary_words(cfg, n) if vdt == TERNARY else entries
    istr = entries if idx_replica_stride is None else idx_replica_stride
    _check_decompress(cfg, n, R, idx, istr, val, vs, params, presign_dbg, packed=True,
                      moments=(("exp_avg", exp_avg, False), ("exp_avg_sq", exp_avg_sq, False),
                               ("max_exp_avg_sq", max_exp_avg_sq, not opt.amsgrad)))
    rc = load().detonation_decompress_adamw_step_packed(
        ctypes.byref(cfg.c()), ctypes.byref(opt.c()), n, R, _ptr(idx), _idx_dtype(idx), istr,
        _ptr(val), vdt, vs, _ptr(params), _dtype(params), _ptr(exp_avg), _ptr(exp_avg_sq),
        _ptr(max_exp_avg_sq), _ptr(presign_dbg), _stream(stream))
    if rc != 0:
        raise DetonationError(rc)
