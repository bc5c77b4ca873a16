"""The C-ABI library loads, exports every symbol include/detonation.h declares, and its
host-side validation answers without touching a GPU (these calls return before any launch)."""
import ctypes
import os
import re

import pytest

from paper_2502_06728_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2502_06728_amd import build
        build.build()
    return binding.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "detonation.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(detonation_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_version_and_status_strings(lib):
    assert binding.version() == 1007
    assert binding.status_string(0) == "ok"
    assert len({binding.status_string(i) for i in range(6)}) == 6


def test_config_struct_layout_matches_header():
    assert ctypes.sizeof(binding.deto_config) == 48
    assert binding.deto_config.seed.offset == 32 and binding.deto_config.step.offset == 40


def test_payload_entries(lib):
    cfg = binding.Config(chunk=32, topk=4)
    assert binding.payload_entries(cfg, 10_820_957) == 338_155 * 4
    assert binding.payload_entries(cfg, 0) == 0
    assert binding.payload_entries(binding.Config(chunk=64, topk=65), 100) == -1


def _compress(lib, cfg, n, grad=1024, mom=1024, idx=1024, val=1024, dtype=0):
    vp = ctypes.c_void_p
    return lib.detonation_compress(ctypes.byref(cfg.c()) if cfg else None, n, vp(grad), dtype,
                                   vp(mom), vp(idx), vp(val), None, None)


def test_host_side_validation(lib):
    ok = binding.Config(chunk=64, topk=8)
    assert _compress(lib, None, 10) == 1
    assert _compress(lib, ok, 10, grad=None) == 1
    assert _compress(lib, ok, 10, idx=None) == 1                      # top-k needs idx_out
    assert _compress(lib, binding.Config(chunk=0, topk=1), 10) == 2
    assert _compress(lib, binding.Config(chunk=257, topk=1), 10) == 2
    assert _compress(lib, binding.Config(chunk=64, topk=0), 10) == 2
    assert _compress(lib, binding.Config(chunk=64, topk=8, scheme=3), 10) == 2
    assert _compress(lib, ok, -1) == 2
    assert _compress(lib, ok, 10, dtype=9) == 2
    assert _compress(lib, ok, 10, mom=1026) == 4                      # fp32 buffer off by 2 bytes
    assert _compress(lib, ok, 0, grad=None, mom=None, idx=None, val=None) == 0   # n = 0: no-op
    vp = ctypes.c_void_p
    d = lib.detonation_decompress_step
    c = ctypes.byref(ok.c())
    assert d(c, 10, 0, vp(1024), 8, vp(1024), 8, vp(1024), 0, None, None) == 2   # R < 1
    assert d(c, 10, 65, vp(1024), 8, vp(1024), 8, vp(1024), 0, None, None) == 3  # R > 64: unsupported
    assert d(c, 10, 2, vp(1024), 4, vp(1024), 8, vp(1024), 0, None, None) == 2   # stride < C*k
    assert d(c, 10, 1, None, 8, vp(1024), 8, vp(1024), 0, None, None) == 1       # top-k needs idx
    assert d(c, 10, 1, vp(1024), 8, vp(1024), 8, vp(1025), 1, None, None) == 4   # bf16 off by 1
    assert d(c, 0, 1, None, 0, None, 0, None, 0, None, None) == 0


def test_binding_refuses_host_tensors(lib):
    import torch
    cfg = binding.Config()
    t = torch.zeros(64)
    with pytest.raises(ValueError):
        binding.detonation_compress(cfg, t, t, t.int(), t)


def test_binding_refuses_wrong_dtypes_and_short_buffers():
    """A wrong element type or a buffer shorter than the call needs would be an out-of-bounds
    access on the device; the binding's host-side checks turn it into a ValueError."""
    import torch
    cfg = binding.Config(chunk=64, topk=8)
    n = 64 * 10 + 3                       # 11 chunks, 88 entries
    f32 = lambda m: torch.zeros(m)
    i32 = lambda m: torch.zeros(m, dtype=torch.int32)
    ok = dict(grad=f32(n), momentum=f32(n), idx_out=i32(88), val_out=f32(88), coeff_dbg=f32(704))
    binding._check_compress(cfg, n, packed=False, **ok)
    for name, bad in [("grad", f32(n - 1)), ("grad", torch.zeros(n, dtype=torch.float16)),
                      ("momentum", torch.zeros(n, dtype=torch.bfloat16)),
                      ("idx_out", i32(87)), ("idx_out", torch.zeros(88, dtype=torch.int64)),
                      ("idx_out", None), ("val_out", f32(87)),
                      ("val_out", torch.zeros(88, dtype=torch.bfloat16)),
                      ("coeff_dbg", f32(703))]:
        with pytest.raises(ValueError):
            binding._check_compress(cfg, n, packed=False, **{**ok, name: bad})
    # narrow formats are for the *_packed calls only; ternary words: ceil(k/16) per chunk
    binding._check_compress(cfg, n, packed=True, **{**ok, "idx_out": torch.zeros(88, dtype=torch.uint8),
                                                    "val_out": torch.zeros(88, dtype=torch.float16)})
    binding._check_compress(cfg, n, packed=True, **{**ok, "val_out": i32(11)})
    with pytest.raises(ValueError):
        binding._check_compress(cfg, n, packed=True, **{**ok, "val_out": i32(10)})
    # Striding / Random need no index array
    binding._check_compress(binding.Config(chunk=64, topk=8, scheme=binding.SCHEME_RANDOM), n,
                            packed=False, **{**ok, "idx_out": None})
    # decompress: R replicas at the given strides
    R, stride = 3, 96
    okd = dict(idx=i32(2 * stride + 88), val=f32(2 * stride + 88), params=f32(n), presign_dbg=f32(n))
    binding._check_decompress(cfg, n, R, okd["idx"], stride, okd["val"], stride, okd["params"],
                              okd["presign_dbg"], packed=False)
    with pytest.raises(ValueError):       # last replica's entries would run past the buffer
        binding._check_decompress(cfg, n, R, okd["idx"], stride, f32(2 * stride + 87), stride,
                                  okd["params"], okd["presign_dbg"], packed=False)
    with pytest.raises(ValueError):       # stride shorter than a replica's payload
        binding._check_decompress(cfg, n, R, okd["idx"], 80, okd["val"], stride, okd["params"],
                                  okd["presign_dbg"], packed=False)
    with pytest.raises(ValueError):
        binding._check_decompress(cfg, n, R, okd["idx"], stride, okd["val"], stride, f32(n - 1),
                                  None, packed=False)
    with pytest.raises(ValueError):       # AdamW moments must be fp32 and cover the shard
        binding._check_decompress(cfg, n, R, okd["idx"], stride, okd["val"], stride, okd["params"],
                                  None, packed=False,
                                  moments=(("exp_avg", f32(n), False),
                                           ("exp_avg_sq", f32(n - 1), False)))


def test_packed_entry_points_validate_formats(lib):
    vp = ctypes.c_void_p
    ok = ctypes.byref(binding.Config(chunk=64, topk=8).c())
    c = lib.detonation_compress_packed
    assert c(ok, 10, vp(1024), 0, vp(1024), vp(1024), 7, vp(1024), 0, None, None) == 2   # idx dtype
    assert c(ok, 10, vp(1024), 0, vp(1024), vp(1024), 0, vp(1024), 4, None, None) == 2   # val dtype
    assert c(ok, 10, vp(1024), 0, vp(1024), vp(1024), 0, vp(1026), 3, None, None) == 4   # ternary words
    assert c(ok, 10, vp(1024), 0, vp(1024), vp(1025), 0, vp(1024), 0, None, None) == 4   # int32 idx
    assert c(ok, 10, vp(1024), 0, vp(1024), vp(1024), 1, vp(1025), 2, None, None) == 4   # fp16 val
    d = lib.detonation_decompress_step_packed
    assert d(ok, 10, 1, vp(1024), 2, 8, vp(1024), 0, 8, vp(1024), 0, None, None) == 2
    assert d(ok, 0, 1, None, 1, 0, None, 2, 0, None, 0, None, None) == 0
    # ternary payload: replica stride counted in 32-bit words, ceil(k/16) per chunk
    assert d(ok, 128, 2, vp(1024), 0, 16, vp(1024), 3, 1, vp(1024), 0, None, None) == 2
    assert lib.detonation_ternary_words(ok, 128) == 2
    assert lib.detonation_ternary_words(ctypes.byref(binding.Config(chunk=64, topk=33).c()), 65) == 6


def test_accumulate_validation(lib):
    vp = ctypes.c_void_p
    ok = ctypes.byref(binding.Config(chunk=64, topk=8).c())
    f = lib.detonation_accumulate
    assert f(None, 10, vp(1024), 0, vp(1024), None) == 1
    assert f(ok, 10, None, 0, vp(1024), None) == 1
    assert f(ok, 10, vp(1024), 7, vp(1024), None) == 2
    assert f(ok, -1, vp(1024), 0, vp(1024), None) == 2
    assert f(ok, 10, vp(1025), 1, vp(1024), None) == 4
    assert f(ok, 0, None, 0, None, None) == 0


def test_adamw_entry_point_validation(lib):
    vp = ctypes.c_void_p
    ok = ctypes.byref(binding.Config(chunk=64, topk=8).c())
    f = lib.detonation_decompress_adamw_step
    good = ctypes.byref(binding.AdamW(step=1).c())

    def call(opt, m=1024, v=1024, vm=None, n=10):
        return f(ok, opt, n, 1, vp(1024), 8, vp(1024), 8, vp(1024), 0, vp(m) if m else None,
                 vp(v) if v else None, vp(vm) if vm else None, None, None)
    assert call(None) == 1
    assert call(ctypes.byref(binding.AdamW(step=0).c())) == 2
    assert call(ctypes.byref(binding.AdamW(beta1=1.0).c())) == 2
    assert call(good, m=None) == 1
    assert call(ctypes.byref(binding.AdamW(amsgrad=True).c())) == 1       # needs max_exp_avg_sq
    assert call(good, m=1026) == 4
    assert call(good, n=0) == 0
    assert ctypes.sizeof(binding.deto_adamw) == 24
    # the same update on narrow payloads
    fp = lib.detonation_decompress_adamw_step_packed

    def callp(opt, idx_dtype=1, val_dtype=3, val=1024, m=1024, n=10):
        return fp(ok, opt, n, 1, vp(1024), idx_dtype, 8, vp(val), val_dtype, 8, vp(1024), 0,
                  vp(m) if m else None, vp(1024), None, None, None)
    assert callp(None) == 1
    assert callp(good, idx_dtype=5) == 2
    assert callp(good, val_dtype=4) == 2
    assert callp(good, val=1026) == 4                                     # ternary words
    assert callp(good, m=None) == 1
    assert callp(good, n=0) == 0


def test_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 with no C++ or HIP types
    import subprocess
    src = tmp_path / "use.c"
    src.write_text('#include "detonation.h"\n'
                   'int use(void) { deto_config c = {64, 8, DETO_SCHEME_TOPK, DETO_FLAG_SIGN, 0.9f, '
                   '1e-3f, 0.0f, 0u, 0u}; deto_adamw a = {0.9f, 0.999f, 1e-8f, 0, 1u};\n'
                   '  (void)a; return (int)detonation_payload_entries(&c, 128) + '
                   'detonation_compress(&c, 0, 0, DETO_F32, 0, 0, 0, 0, 0); }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                    "-I", os.path.join(ROOT, "include"), str(src)], check=True)
