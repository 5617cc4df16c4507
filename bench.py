#!/usr/bin/env python3
"""Benchmark of the Tandem hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

Prints ONE JSON line.  A "step" is one pass of the selected workload over one batch of
seeded synthetic inputs that are resident in HBM before the timed region starts.  Timing uses
HIP events recorded on the stream the kernels are launched on (torch's current stream, whose
handle is what the C ABI receives).  Working sets smaller than 512 MB are rotated over enough
distinct copies that the 256 MB Infinity Cache cannot serve the stream.

The line also carries
  roofline     - the dominant kernel against the MI355X HBM peak (8 TB/s), from its algorithmic
                 bytes and its live-measured average duration;
  cpu_baseline - the fp64 oracle timed on this machine's host cores on a bounded sample of the same
                 workload (a reported baseline, not a target).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MALL_BYTES = 256 << 20


def _rotations(bytes_per_copy):
    return max(1, math.ceil(2 * MALL_BYTES / bytes_per_copy))


def _time_calls(torch, fn, n_copies, steps, warmup, use_graph=True):
    """Average milliseconds per call over exactly `steps` calls.  The calls are recorded once into a
    HIP graph (on a side stream, which is the stream the kernels are then launched on) and the
    graph is replayed between two HIP events, so host launch overhead does not bound short kernels."""
    for i in range(warmup):
        fn(i % n_copies)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if use_graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(steps):
                fn(i % n_copies)
        g.replay()  # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        e0.record()
        g.replay()
        e1.record()
    else:
        e0.record()
        for i in range(steps):
            fn(i % n_copies)
        e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps  # ms per call


def _cpu_threads():
    try:
        from threadpoolctl import threadpool_info

        n = [p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"]
        return max(n) if n else 1
    except Exception:
        return 1


# ------------------------------------------------------------------ attention workloads
def draft_workload(torch, binding, inputs, B, H, Hkv, dh, n_large, n_cur, gmax, seed):
    T_max = n_large
    bytes_alg = B * Hkv * (n_large + n_cur) * dh * 2 * 2
    R = _rotations(bytes_alg)
    sets = []
    for i in range(R):
        sets.append(dict(
            q=inputs.device_normal((B, H, dh), seed * 100 + 5 * i, 1.0),
            khat=inputs.device_normal((B, Hkv, T_max, dh), seed * 100 + 5 * i + 1, 1.0 / math.sqrt(dh)),
            vhat=inputs.device_normal((B, Hkv, T_max, dh), seed * 100 + 5 * i + 2, 1.0 / math.sqrt(dh)),
            kcur=inputs.device_normal((B, Hkv, gmax, dh), seed * 100 + 5 * i + 3, 1.0 / math.sqrt(dh)),
            vcur=inputs.device_normal((B, Hkv, gmax, dh), seed * 100 + 5 * i + 4, 1.0 / math.sqrt(dh)),
        ))
    nl = torch.full((B,), n_large, dtype=torch.int32, device="cuda")
    nc = torch.full((B,), n_cur, dtype=torch.int32, device="cuda")
    out = torch.empty((B, H, dh), dtype=torch.bfloat16, device="cuda")
    d = binding.attn_desc(B, H, Hkv, dh, T_max, gmax, 1.0 / math.sqrt(dh), binding.BF16)
    ws = torch.empty(max(256, binding.tandem_draft_attn_workspace(d)), dtype=torch.uint8, device="cuda")

    def call(i):
        s = sets[i]
        binding.tandem_draft_attn(s["q"], s["khat"], s["vhat"], nl, s["kcur"], s["vcur"], nc, out=out, ws=ws)

    def oracle_sample(n_seq):
        from oracle import tandem_oracle as orc

        s = sets[0]
        f = lambda t: inputs.torch_to_f64(t[:n_seq])
        args = (f(s["q"]), f(s["khat"]), f(s["vhat"]), nl[:n_seq].cpu().numpy(), f(s["kcur"]), f(s["vcur"]),
                nc[:n_seq].cpu().numpy(), 1.0 / math.sqrt(dh))
        t0 = time.perf_counter()
        want = orc.draft_attn(*args)
        dt = time.perf_counter() - t0
        call(0)
        torch.cuda.synchronize()
        return dt, want, inputs.torch_to_f64(out[:n_seq])

    return call, R, bytes_alg, oracle_sample


def block_workload(torch, binding, inputs, B, q_len, Hq, Hkv, dh, n_prefix, seed):
    T_max = n_prefix + q_len
    bytes_alg = B * Hkv * T_max * dh * 2 * 2
    R = _rotations(bytes_alg)
    sets = []
    for i in range(R):
        sets.append(dict(
            q=inputs.device_normal((B, q_len, Hq, dh), seed * 100 + 3 * i, 1.0),
            k=inputs.device_normal((B, Hkv, T_max, dh), seed * 100 + 3 * i + 1, 1.0),
            v=inputs.device_normal((B, Hkv, T_max, dh), seed * 100 + 3 * i + 2, 1.0),
        ))
    n = torch.full((B,), n_prefix, dtype=torch.int32, device="cuda")
    out = torch.empty((B, q_len, Hq, dh), dtype=torch.bfloat16, device="cuda")
    d = binding.attn_desc(B, Hq, Hkv, dh, T_max, 0, 1.0 / math.sqrt(dh), binding.BF16)
    ws = torch.empty(max(256, binding.tandem_block_attn_workspace(d, q_len)), dtype=torch.uint8, device="cuda")

    def call(i):
        s = sets[i]
        binding.tandem_block_attn(s["q"], s["k"], s["v"], n, out=out, ws=ws)

    def oracle_sample(n_seq):
        from oracle import tandem_oracle as orc

        s = sets[0]
        f = lambda t: inputs.torch_to_f64(t[:n_seq])
        args = (f(s["q"]), f(s["k"]), f(s["v"]), n[:n_seq].cpu().numpy(), 1.0 / math.sqrt(dh))
        t0 = time.perf_counter()
        want = orc.block_attn(*args)
        dt = time.perf_counter() - t0
        call(0)
        torch.cuda.synchronize()
        return dt, want, inputs.torch_to_f64(out[:n_seq])

    return call, R, bytes_alg, oracle_sample


WORKLOADS = {
    # name: (kind, kwargs, oracle sample sequences, description)
    "c1_draft": ("draft", dict(B=8, H=8, Hkv=8, dh=128, n_large=2044, n_cur=4, gmax=4, seed=1), 8,
                 "tandem_draft_attn bf16 B=8 H=8 dh=128 ctx=2044+4"),
    "c2_block": ("block", dict(B=16, q_len=4, Hq=32, Hkv=8, dh=128, n_prefix=4096, seed=2), 4,
                 "tandem_block_attn bf16 B=16 Hq/Hkv=32/8 dh=128 prefix=4096 gamma=4"),
    "c4_draft": ("draft", dict(B=64, H=8, Hkv=8, dh=128, n_large=32760, n_cur=8, gmax=8, seed=4), 1,
                 "tandem_draft_attn bf16 B=64 H=8 dh=128 ctx=32760+8"),
    "c4_block": ("block", dict(B=64, q_len=8, Hq=32, Hkv=8, dh=128, n_prefix=32760, seed=4), 1,
                 "tandem_block_attn bf16 B=64 Hq/Hkv=32/8 dh=128 prefix=32760 gamma=8"),
    "c3_draft": ("draft", dict(B=32, H=8, Hkv=8, dh=128, n_large=8188, n_cur=4, gmax=4, seed=3), 2,
                 "tandem_draft_attn bf16 B=32 H=8 dh=128 ctx=8188+4 (one small layer of the decode step)"),
    "c3_block": ("block", dict(B=32, q_len=4, Hq=32, Hkv=8, dh=128, n_prefix=8188, seed=3), 2,
                 "tandem_block_attn bf16 B=32 Hq/Hkv=32/8 dh=128 prefix=8188 gamma=4 (one large layer of the decode step)"),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c1_draft", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2402_08644_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.lib()  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)

    kind, kw, n_seq, desc = WORKLOADS[args.workload]
    maker = draft_workload if kind == "draft" else block_workload
    call, n_copies, bytes_alg, oracle_sample = maker(torch, binding, inputs, **kw)
    torch.cuda.synchronize()
    ms = _time_calls(torch, call, n_copies, args.steps, args.warmup, use_graph=not args.no_graph)
    gbs = bytes_alg / (ms * 1e-3) / 1e9

    cpu = None
    if not args.no_cpu_baseline:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from parity import row_errors

        dt, want, got = oracle_sample(n_seq)
        e_inf, _ = row_errors(got, want)
        frac = n_seq / kw["B"]
        cpu = {"value": bytes_alg * frac / dt / 1e9, "unit": "GB/s", "cores": _cpu_threads(), "kind": "oracle",
               "sample": f"{n_seq} of {kw['B']} sequences of the same call, fp64 numpy, {dt:.2f} s",
               "gpu_max_rel_err_on_sample": float(e_inf.max())}

    line = {
        "metric": "Tandem attention HBM GB/s (algorithmic KV bytes / time)",
        "value": gbs,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc}", "rotated_copies": n_copies},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                     "traffic": None},
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
