"""Writes tests/golden/oracle_small_case.json from the CPU oracle alone.

A regression pin: the stored integers are the oracle's own outputs (indices, and the
bit patterns of fp32 results) for one small seeded case per scheme, so an accidental
change to the oracle's arithmetic shows up as a diff.  It calls nothing but `oracle/`
and the input generator.  Run:  python -m tests.golden.make_golden
"""
import json
import os
import zlib

import numpy as np

import oracle
from oracle import Config, SCHEME_RANDOM, SCHEME_STRIDE, SCHEME_TOPK
from paper_2502_06728_amd import synth


def _crc(a: np.ndarray) -> int:
    return zlib.crc32(np.ascontiguousarray(a).tobytes())


def small_case() -> dict:
    out = {}
    n, s, k = 64 * 9 + 17, 64, 8
    g = synth.normal(0, synth.TAG_GRAD, n, 1e-3)
    m = synth.normal(0, synth.TAG_MOMENTUM, n, 1e-3)
    th = synth.normal(0, synth.TAG_PARAMS, n, 0.02)
    for name, scheme, dct in [("topk", SCHEME_TOPK, False), ("stride", SCHEME_STRIDE, False),
                              ("random", SCHEME_RANDOM, False), ("random_dct", SCHEME_RANDOM, True)]:
        cfg = Config(chunk=s, topk=k, scheme=scheme, dct=dct, seed=11, step=3)
        m_new, idx, val = oracle.compress(cfg, g, m)
        th_new = oracle.decompress_step(cfg, idx, val, th)
        out[name + "_idx_first_chunks"] = [int(v) for v in idx[:2 * k]]
        out[name + "_idx_crc"] = _crc(idx)
        out[name + "_val_crc"] = _crc(val)
        out[name + "_m_crc"] = _crc(m_new)
        out[name + "_theta_crc"] = _crc(th_new)
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_case.json")
    with open(path, "w") as f:
        json.dump(small_case(), f, indent=1, sort_keys=True)
    print("wrote", path)
