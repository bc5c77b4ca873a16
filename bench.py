#!/usr/bin/env python3
"""Benchmark of the fused optimizer step (compress + decompress-and-update) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload olmo-1b-1of8]

A step is one pass of the whole hot path over the shard: detonation_compress (momentum
accumulate, chunked DCT, selection, residual, payload) followed by
detonation_decompress_step (scatter R payloads, average, inverse DCT, sign, parameter
update).  All inputs are resident in HBM before the timed region; debug outputs are off.
Prints ONE JSON line: throughput in parameters per second, the roofline of the slower
kernel (algorithmic bytes / measured duration against the 8 TB/s HBM peak) and the CPU
oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak


def kernel_sources_sha16() -> str:
    """Fingerprint of the HIP sources (every file under csrc/, comments and blank lines left
    out): the counter-measured traffic recorded under profiles/ is only quoted for the code it
    was measured on."""
    import hashlib
    import re
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2502_06728_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name == "membench.hip":
            continue
        text = open(os.path.join(d, name), encoding="utf-8").read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        code = "\n".join(l.rstrip() for l in text.splitlines() if l.strip())
        h.update(name.encode())
        h.update(code.encode())
    return h.hexdigest()[:16]


def algorithmic_bytes(n: int, s: int, k: int, R: int, grad_bytes: int, param_bytes: int,
                      with_idx: bool, val_bytes: float = 4, idx_bytes: int = 4) -> dict:
    """Bytes the method itself must move per launch: compress reads g and m, writes m and
    the payload; decompress reads R payloads, reads and writes the parameters."""
    C = -(-n // s)
    pay = int(C * k * (val_bytes + (idx_bytes if with_idx else 0)))
    return {"compress": n * (grad_bytes + 8) + pay, "decompress": R * pay + 2 * n * param_bytes}


def _oracle_step_rate(w, cfg_kwargs: dict, sample_params: int, every: int):
    """Parameters per second of the oracle on the leading `sample_params` of the shard with the
    thread count it is currently set to; returns (rate, n, seconds)."""
    import numpy as np
    import oracle
    from paper_2502_06728_amd import synth
    cfg = oracle.Config(**cfg_kwargs)
    n = min(sample_params, w.n)
    n -= n % cfg.chunk
    g, m, th = synth.shard(w, stop=n)
    C = n // cfg.chunk
    R = w.replicas
    idx = np.empty((R, C * cfg.topk), np.int32)
    val = np.empty((R, C * cfg.topk), np.float32)
    for r in range(1, R):   # replica payloads, untimed (as on the GPU side)
        idx[r], val[r] = synth.structured_payload(w.seed + r, C, cfg.chunk, cfg.topk, w.momentum_std)
    oracle.lib()
    t0 = time.perf_counter()
    for _ in range(every - 1):
        m = oracle.fold(cfg, g, m)
    m_new, idx0, val0 = oracle.compress(cfg, g, m)
    idx[0], val[0] = idx0, val0
    oracle.decompress_step(cfg, idx if cfg.scheme == 0 else None, val, th)
    dt = time.perf_counter() - t0
    return every * n / dt, n, dt


def cpu_baseline(w, cfg_kwargs: dict, sample_params: int, every: int = 1,
                 one_core_sample: int = 1 << 23) -> dict:
    """The oracle as it stands, on the host cores, on the leading `sample_params` of the shard,
    and on one core on a smaller leading sample.
    every > 1 (DiLoCo): every-1 accumulate-only steps, then the synchronising step."""
    import oracle
    rate, n, dt = _oracle_step_rate(w, cfg_kwargs, sample_params, every)
    cores = oracle.threads()
    oracle.set_threads(1)
    try:
        rate1, n1, dt1 = _oracle_step_rate(w, cfg_kwargs, one_core_sample, every)
    finally:
        oracle.set_threads(cores)
    R = w.replicas
    what = "one full step" if every == 1 else f"{every - 1} accumulate-only steps and one full step"
    return {"value": rate, "unit": "params/s", "cores": cores, "kind": "oracle",
            "sample": f"leading {n} of {w.n} parameters of the same shard, {what} "
                      f"(compress + decompress, R={R}), {dt:.1f} s, gcc -O2 + OpenMP",
            "value_1core": rate1,
            "sample_1core": f"leading {n1} parameters, same step, one thread, {dt1:.1f} s"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="olmo-1b-1of8")
    ap.add_argument("--scheme", default="topk", choices=["topk", "stride", "random", "diloco"],
                    help="diloco: accumulate only, and every --diloco-every'th step extract and "
                         "average the whole momentum (Striding with k = chunk)")
    ap.add_argument("--diloco-every", type=int, default=4)
    ap.add_argument("--dct", action="store_true", help="coefficient domain for stride/random")
    ap.add_argument("--payload", default="f32i32", choices=["f32i32", "bf16u8", "f16u8", "ternaryu8"],
                    help="payload format: value dtype + index width (top-k)")
    ap.add_argument("--optimizer", default="sgd", choices=["sgd", "adamw"],
                    help="underlying optimizer of the update: DeMo-SGD or Decoupled AdamW")
    ap.add_argument("--chunk", type=int, default=0, help="override the workload's chunk size")
    ap.add_argument("--topk", type=int, default=0, help="override the workload's k")
    ap.add_argument("--replicas", type=int, default=0,
                    help="override the workload's R, the size of the replication group")
    ap.add_argument("--no-sign", action="store_true", help="update with Q itself, not sign(Q)")
    ap.add_argument("--graph", action="store_true",
                    help="time the step as replays of one captured HIP graph (compress + decompress "
                         "with the step counter frozen): no launch gap between the two kernels")
    ap.add_argument("--cpu-sample", type=int, default=1 << 28)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--sources-sha", action="store_true",
                    help="print the fingerprint of the HIP sources (recorded with counter runs)")
    ap.add_argument("--report", action="store_true",
                    help="run every benchmark configuration and print a markdown report "
                         "(GPU rate, HBM GB/s, oracle on 1 and all host cores, paper context)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the one-GPU hot path only: the payload all_gather across the "
              "replication group is not part of this build, so --gpus must be 1.", file=sys.stderr)
        return 2
    if args.sources_sha:
        print(kernel_sources_sha16())
        return 0
    if args.report:
        return report(args)
    print(json.dumps(run(args)))
    return 0


def run(args) -> dict:
    """One benchmark configuration; returns the record bench.py prints as its JSON line."""
    import numpy as np
    import torch
    from paper_2502_06728_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.load()
    dev = torch.device("cuda:0")
    w = synth.workloads()[args.workload]
    if args.chunk or args.topk:
        import dataclasses
        w = dataclasses.replace(w, chunk=args.chunk or w.chunk, topk=args.topk or w.topk)
    if getattr(args, "replicas", 0):
        import dataclasses
        w = dataclasses.replace(w, replicas=args.replicas)
    if getattr(args, "no_sign", False):
        import dataclasses
        w = dataclasses.replace(w, sign=False)
    diloco = args.scheme == "diloco"
    every = max(1, args.diloco_every) if diloco else 1
    if diloco:
        import dataclasses
        w = dataclasses.replace(w, topk=w.chunk)
    scheme = {"topk": binding.SCHEME_TOPK, "stride": binding.SCHEME_STRIDE,
              "random": binding.SCHEME_RANDOM, "diloco": binding.SCHEME_STRIDE}[args.scheme]
    cfg_kwargs = dict(chunk=w.chunk, topk=w.topk, scheme=scheme, sign=w.sign, dct=args.dct,
                      decay=w.decay, lr=w.lr, weight_decay=w.weight_decay, seed=w.seed, step=0)
    cfg = binding.Config(**cfg_kwargs)
    n, s, k, R = w.n, w.chunk, w.topk, w.replicas
    entries = binding.payload_entries(cfg, n)
    with_idx = scheme == binding.SCHEME_TOPK

    # ---- resident inputs: the shard itself from the seeded recipe ...
    g_np, m_np, th_np = synth.shard(w)

    def up(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    grad, mom, params = up(g_np), up(m_np), up(th_np)
    del g_np, m_np, th_np
    packed = args.payload != "f32i32"
    ternary = args.payload == "ternaryu8"     # signs only: int32 words of 16 two-bit codes
    val_t = {"f32i32": torch.float32, "bf16u8": torch.bfloat16, "f16u8": torch.float16,
             "ternaryu8": torch.int32}[args.payload]
    idx_t = torch.uint8 if packed else torch.int32
    idx = torch.zeros((R, entries), dtype=idx_t, device=dev) if with_idx else None
    val = torch.zeros((R, binding.ternary_words(cfg, n) if ternary else entries), dtype=val_t,
                      device=dev)
    compress = binding.detonation_compress_packed if packed else binding.detonation_compress
    decompress = (binding.detonation_decompress_step_packed if packed
                  else binding.detonation_decompress_step)
    # ... and R-1 other replicas' payloads: the library's compress run, untimed, on
    # independently seeded shards of the same recipe (what an all_gather would deliver).
    gen = torch.Generator(device=dev)
    for r in range(1, R):
        gen.manual_seed(w.seed + r)
        gr = torch.randn(n, generator=gen, device=dev, dtype=torch.float32) * w.grad_std
        if w.outlier_frac > 0:
            u = torch.rand(n, generator=gen, device=dev)
            gr = torch.where(u < w.outlier_frac, gr * w.outlier_scale, gr)
        gr = gr.to(grad.dtype)
        mr = torch.randn(n, generator=gen, device=dev, dtype=torch.float32) * w.momentum_std
        compress(cfg, gr, mr, None if idx is None else idx[r], val[r])
        torch.cuda.synchronize()
        del gr, mr
    torch.cuda.empty_cache()

    adamw = args.optimizer == "adamw"
    if adamw:
        exp_avg = torch.zeros(n, dtype=torch.float32, device=dev)
        exp_avg_sq = torch.zeros(n, dtype=torch.float32, device=dev)
        opt = binding.AdamW(0.9, 0.95, 1e-8, False, 0)

    def step(ev=None):
        cfg.step += 1
        if ev:
            ev[0].record()
        if cfg.step % every:                 # DiLoCo: a step that only accumulates
            binding.detonation_accumulate(cfg, grad, mom)
            if ev:
                ev[1].record()
                ev[2].record()
            return
        compress(cfg, grad, mom, None if idx is None else idx[0], val[0])
        if ev:
            ev[1].record()
        if adamw:
            opt.step += 1
            (binding.detonation_decompress_adamw_step_packed if packed
             else binding.detonation_decompress_adamw_step)(cfg, opt, R, idx, val, params,
                                                            exp_avg, exp_avg_sq)
        else:
            decompress(cfg, R, idx, val, params)
        if ev:
            ev[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    if getattr(args, "graph", False):
        # the same step as one HIP graph, replayed: what is left is the kernels' own time
        assert not diloco, "--graph times the plain step"
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

    # ms per launch; with DiLoCo only every `every`-th step runs compress + decompress
    first = cfg.step - args.steps + 1
    sync = [e for i, e in enumerate(events) if (first + i) % every == 0] or events
    t_c = sum(e[0].elapsed_time(e[1]) for e in sync) / len(sync)
    t_d = sum(e[1].elapsed_time(e[2]) for e in sync) / len(sync)
    acc = [e for i, e in enumerate(events) if (first + i) % every != 0]
    t_a = sum(e[0].elapsed_time(e[1]) for e in acc) / len(acc) if acc else None
    ms_per_step = wall * 1e3 / args.steps
    ab = algorithmic_bytes(n, s, k, R, grad.element_size(), params.element_size(), with_idx,
                           4.0 * -(-k // 16) / k if ternary else val.element_size(),   # whole words per chunk
                           idx.element_size() if with_idx else 0)
    if adamw:
        ab["decompress"] += 16 * n          # exp_avg and exp_avg_sq, fp32, read and written
    gbs_c = ab["compress"] / (t_c * 1e-3) / 1e9
    gbs_d = ab["decompress"] / (t_d * 1e-3) / 1e9
    dom = "compress" if t_c >= t_d else "decompress"
    dom_gbs = gbs_c if dom == "compress" else gbs_d

    # HBM bytes per launch of the dominant kernel as rocprofv3's FETCH_SIZE + WRITE_SIZE counters
    # measured them for this workload.  Counters need a profiler run of their own, so the figure
    # comes from the summary under profiles/; the record says which file, at which commit it
    # was measured, and the figure is withheld if the kernels' sources have changed since.
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload}_{args.scheme}.txt")
    if os.path.exists(tpath) and not packed and not adamw and not (args.chunk or args.topk or args.dct
                                                                  or args.replicas):
        meta, rows = {}, {}
        for line in open(tpath):
            f = line.split()
            if len(f) == 3 and f[0] == "#" and f[1] in ("commit", "kernel_sources_sha16"):
                meta[f[1]] = f[2]
            elif len(f) == 2 and not line.startswith("#"):
                rows[f[0]] = float(f[1])
        now = kernel_sources_sha16()
        stale = meta.get("kernel_sources_sha16") != now
        traffic = None if stale else rows.get(dom)
        traffic_source = {"file": os.path.relpath(tpath, ROOT), "measured_at_commit": meta.get("commit"),
                          "kernel_sources_sha16": meta.get("kernel_sources_sha16"),
                          "kernel_sources_sha16_now": now, "stale": stale}

    # bytes of an average step (DiLoCo: every-1 accumulations of g and m per synchronisation)
    ab_acc = n * (grad.element_size() + 8)
    step_bytes = (ab["compress"] + ab["decompress"] + (every - 1) * ab_acc) / every
    out = {
        "metric": "optimizer_step_params_per_sec", "value": n * args.steps / wall,
        "unit": "params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "params": n, "chunk": s, "topk": k, "replicas": R,
                   "scheme": args.scheme, "payload": args.payload,
                   "optimizer": args.optimizer, "dct_domain": bool(cfg.scheme == 0 or args.dct),
                   "grad_dtype": str(grad.dtype).split(".")[-1],
                   "param_dtype": str(params.dtype).split(".")[-1], "momentum_dtype": "float32",
                   "sign": w.sign, "decay": w.decay, "lr": w.lr,
                   "hip_graph": bool(getattr(args, "graph", False))},
        "step_hbm_gbs": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_hbm_frac_of_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kernels": {
            "compress": {"ms": t_c, "algorithmic_bytes": ab["compress"], "gbs": gbs_c,
                         "frac": gbs_c / HBM_PEAK_GBS},
            "decompress": {"ms": t_d, "algorithmic_bytes": ab["decompress"], "gbs": gbs_d,
                           "frac": gbs_d / HBM_PEAK_GBS}},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": dom_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": dom_gbs / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": traffic_source},
    }
    if diloco:
        out["config"]["diloco_every"] = every
        if t_a:
            out["kernels"]["accumulate"] = {"ms": t_a, "algorithmic_bytes": ab_acc,
                                            "gbs": ab_acc / (t_a * 1e-3) / 1e9,
                                            "frac": ab_acc / (t_a * 1e-3) / 1e9 / HBM_PEAK_GBS}
    del grad, mom, params, idx, val
    torch.cuda.empty_cache()
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, cfg_kwargs, args.cpu_sample, every)
    return out


PAPER_CONTEXT = """\
Context only — what the paper reports (whole-training or network figures, other hardware; it gives no
number for this kernel path):
- FlexDeMo (any replicator) vs Hybrid-FSDP + AdamW: about 2.6x faster wall-clock, OLMo2-1B on Dolma
  v1.6, 10K steps, 2 nodes x 4 NVIDIA A100 64 GB, InfiniBand 200 Gb/s ("OLMo2: Causal Language
  Modeling", Discussion).
- Random replicator vs conventional Hybrid-FSDP + AdamW at 64 nodes x 4 GPUs, rate 1/32: about 64 %
  faster; DeMo much slower there, which the paper puts down to the all_gather ("OLMo2: Scaling Up").
- Average inter-node bandwidth, T5-small, 2 nodes x 4 RTX A6000, 10 GbE, rate 1/16: 1070 Mbps full
  replication, 291 Mbps DeMo, 152 Mbps Random ("Replicator bandwidth usage").
- Time per optimizer step at 10 Mbps, ViT-B, 2 x 4 RTX A6000: Random about 3.33x faster than DeMo
  and about 18x faster than Decoupled AdamW with full replication ("Performance in congested
  networks").
"""


def report(args) -> int:
    """All benchmark configurations, one row each, with the CPU oracle timed in the same run."""
    import copy
    rows = []
    plan = [("flat-1m", "topk", False), ("t5-base-1of8", "topk", False),
            ("vit-b16-1of8", "topk", False), ("olmo-1b-1of8", "topk", False),
            ("olmo-7b-1of8", "topk", False), ("olmo-7b-1of8", "stride", False),
            ("olmo-7b-1of8", "random", False), ("olmo-7b-1of8", "random", True),
            ("olmo-1b-1of8", "diloco", False)]
    for workload, scheme, dct in plan:
        a = copy.copy(args)
        a.workload, a.scheme, a.dct = workload, scheme, dct
        a.steps, a.warmup, a.no_cpu = min(args.steps, 20), 3, False
        a.cpu_sample = 1 << 26           # oracle on at most 67 M leading parameters (labelled)
        rec = run(a)
        all_cores = rec["cpu_baseline"]
        one = {"value": all_cores["value_1core"]}
        rows.append((rec, all_cores, one))
        print(f"# done {workload} {scheme}{' dct' if dct else ''}", file=sys.stderr, flush=True)
    print("| workload | scheme | params | step ms | GPU params/s | step GB/s (% of 8 TB/s) | "
          "compress GB/s | decompress GB/s | oracle params/s, 1 core | oracle params/s, all cores "
          "| GPU / oracle (all cores) |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for rec, allc, one in rows:
        c = rec["config"]
        name = c["scheme"] + (" (coefficients)" if c["scheme"] != "topk" and c["dct_domain"] else "")
        if c["scheme"] == "diloco":
            name = f"diloco (sync every {c['diloco_every']})"
        print(f"| {c['workload']} | {name} | {c['params']:,} | {rec['ms_per_step']:.3f} | "
              f"{rec['value'] / 1e9:.1f} G | {rec['step_hbm_gbs']:.0f} "
              f"({100 * rec['step_hbm_frac_of_peak']:.0f} %) | {rec['kernels']['compress']['gbs']:.0f} | "
              f"{rec['kernels']['decompress']['gbs']:.0f} | {one['value'] / 1e6:.1f} M | "
              f"{allc['value'] / 1e6:.1f} M ({allc['cores']} cores) | "
              f"{rec['value'] / allc['value']:.0f}x |")
    print()
    # the small shards again as replays of a captured HIP graph (no launch gap between the kernels)
    small = []
    for workload in ("t5-base-1of8", "vit-b16-1of8"):
        a = copy.copy(args)
        a.workload, a.scheme, a.dct, a.graph = workload, "topk", False, True
        a.steps, a.warmup, a.no_cpu = min(args.steps, 50), 5, True
        small.append(run(a))
    print("Small shards, the step captured in a HIP graph and replayed (kernel columns: eager run of the same step):")
    print()
    print("| workload | compress ms | decompress ms | step ms (graph replay) | GPU params/s | step GB/s (% of 8 TB/s) |")
    print("|---|---|---|---|---|---|")
    for rec in small:
        c = rec["config"]
        print(f"| {c['workload']} | {rec['kernels']['compress']['ms']:.4f} | {rec['kernels']['decompress']['ms']:.4f} | "
              f"{rec['ms_per_step']:.4f} | {rec['value'] / 1e9:.1f} G | {rec['step_hbm_gbs']:.0f} "
              f"({100 * rec['step_hbm_frac_of_peak']:.0f} %) |")
    print()
    # the ViT-B/16 sweep of the benchmark configurations: chunk x top-k x sign, R = 2, on the
    # 10.8 M-parameter shard (fp32, ragged length)
    vit = []
    for s_ in (32, 64, 128):
        for k_ in sorted({1, 4, 16, s_ // 2}):
            for sign in (True, False):
                a = copy.copy(args)
                a.workload, a.scheme, a.dct = "vit-b16-1of8", "topk", False
                a.chunk, a.topk, a.no_sign = s_, k_, not sign
                a.steps, a.warmup, a.no_cpu = min(args.steps, 50), 5, True
                vit.append(run(a))
        print(f"# done vit chunk {s_}", file=sys.stderr, flush=True)
    print("ViT-B/16 sweep (vit-b16-1of8: 10,820,957 parameters, fp32, R = 2; the whole step moves "
          "0.2 - 0.4 GB, so launch and tail effects weigh more than on the larger shards):")
    print()
    print("| chunk | top-k | sign | compress ms | decompress ms | step ms | GPU params/s | "
          "step GB/s (% of 8 TB/s) |")
    print("|---|---|---|---|---|---|---|---|")
    for rec in vit:
        c = rec["config"]
        print(f"| {c['chunk']} | {c['topk']} | {'on' if c['sign'] else 'off'} | "
              f"{rec['kernels']['compress']['ms']:.4f} | {rec['kernels']['decompress']['ms']:.4f} | "
              f"{rec['ms_per_step']:.4f} | {rec['value'] / 1e9:.1f} G | {rec['step_hbm_gbs']:.0f} "
              f"({100 * rec['step_hbm_frac_of_peak']:.0f} %) |")
    print()
    # chunk-size sweep of Appendix B ("DeMo Chunk Size": 16 ... 256 at compression rates 1/8 and
    # 1/16) on the OLMo-1B shard, GPU only
    sweep = []
    for rate in (8, 16):
        for s_ in (16, 32, 64, 96, 128, 192, 256):
            a = copy.copy(args)
            a.workload, a.scheme, a.dct = "olmo-1b-1of8", "topk", False
            a.chunk, a.topk = s_, s_ // rate
            a.steps, a.warmup, a.no_cpu = min(args.steps, 20), 3, True
            sweep.append(run(a))
            print(f"# done chunk {s_} rate 1/{rate}", file=sys.stderr, flush=True)
    print("Chunk-size sweep (Appendix B, \"DeMo Chunk Size\"), olmo-1b-1of8, top-k, R = 4:")
    print()
    print("| chunk | top-k | rate | compress ms | decompress ms | step ms | GPU params/s | "
          "step GB/s (% of 8 TB/s) |")
    print("|---|---|---|---|---|---|---|---|")
    for rec in sweep:
        c = rec["config"]
        print(f"| {c['chunk']} | {c['topk']} | 1/{c['chunk'] // c['topk']} | "
              f"{rec['kernels']['compress']['ms']:.3f} | {rec['kernels']['decompress']['ms']:.3f} | "
              f"{rec['ms_per_step']:.3f} | {rec['value'] / 1e9:.1f} G | {rec['step_hbm_gbs']:.0f} "
              f"({100 * rec['step_hbm_frac_of_peak']:.0f} %) |")
    print()
    # the setting of the paper's experiments ("Overall Setup": chunk size 32, only the signs
    # synchronised, top-k varied to set the compression rate), plain and Decoupled AdamW update
    setting = []
    for scheme, k_, optimizer in (("topk", 16, "sgd"), ("topk", 4, "sgd"), ("topk", 1, "sgd"),
                                  ("random", 4, "sgd"), ("random", 1, "sgd"), ("stride", 1, "sgd"),
                                  ("topk", 4, "adamw"), ("random", 4, "adamw")):
        a = copy.copy(args)
        a.workload, a.scheme, a.dct = "olmo-1b-1of8", scheme, False
        a.chunk, a.topk, a.payload, a.optimizer = 32, k_, "ternaryu8", optimizer
        a.steps, a.warmup, a.no_cpu = min(args.steps, 20), 3, True
        setting.append(run(a))
        print(f"# done chunk 32 k {k_} {scheme} signs {optimizer}", file=sys.stderr, flush=True)
    print("The paper's experimental setting (chunk size 32, signs only on the wire: two bits per "
          "entry, byte indices under top-k, none under Striding / Random), olmo-1b-1of8, R = 4:")
    print()
    print("| scheme | top-k | rate | optimizer | compress ms | decompress ms | step ms | "
          "GPU params/s | step GB/s (% of 8 TB/s) |")
    print("|---|---|---|---|---|---|---|---|---|")
    for rec in setting:
        c = rec["config"]
        print(f"| {c['scheme']} | {c['topk']} | 1/{c['chunk'] // c['topk']} | {c['optimizer']} | "
              f"{rec['kernels']['compress']['ms']:.3f} | {rec['kernels']['decompress']['ms']:.3f} | "
              f"{rec['ms_per_step']:.3f} | {rec['value'] / 1e9:.1f} G | {rec['step_hbm_gbs']:.0f} "
              f"({100 * rec['step_hbm_frac_of_peak']:.0f} %) |")
    print()
    print("Oracle: the CPU reference as it stands (plain C, double arithmetic, gcc -O2, OpenMP over "
          "chunks), one full step on the leading parameters of the same shard (all cores: up to "
          "67 M parameters; 1 core: 8 M), rate scaled per parameter.  flat-1m fits the caches "
          "and is a correctness configuration, not a bandwidth one.")
    print()
    print(PAPER_CONTEXT)
    return 0


if __name__ == "__main__":
    sys.exit(main())
