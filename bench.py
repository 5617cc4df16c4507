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
        # K and V as a TandemState lays them out for the block attention (V out of phase with K, see the binding)
        seeds = iter((seed * 100 + 3 * i + 1, seed * 100 + 3 * i + 2))
        k, v = binding.kv_pair_out_of_phase(lambda *s: inputs.device_normal(s, next(seeds), 1.0), (B, Hkv, T_max, dh),
                                            torch.bfloat16, "cuda")
        sets.append(dict(q=inputs.device_normal((B, q_len, Hq, dh), seed * 100 + 3 * i, 1.0), k=k, v=v))
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


def shared_workload(torch, binding, inputs, B, samples, q_len, Hq, Hkv, dh, n_shared, n_own, seed, copied=False):
    """Block-mode attention with `samples` continuations per prompt.  copied=False: the prompt rows stored and
    read once per prompt (tandem_block_attn_shared).  copied=True: the form it replaces - every sample holds a
    copy of the prompt rows in its own cache (tandem_block_attn) - on the same values."""
    T_own = n_own + q_len
    nseq = B * samples
    if copied:
        bytes_alg = nseq * Hkv * (n_shared + T_own) * dh * 2 * 2
    else:
        bytes_alg = (B * n_shared + nseq * T_own) * Hkv * dh * 2 * 2
    R = _rotations(bytes_alg)
    sets = []
    for i in range(R):
        c = dict(
            q=inputs.device_normal((B, samples, q_len, Hq, dh), seed * 100 + 5 * i, 1.0),
            ks=inputs.device_normal((B, Hkv, n_shared, dh), seed * 100 + 5 * i + 1, 1.0),
            vs=inputs.device_normal((B, Hkv, n_shared, dh), seed * 100 + 5 * i + 2, 1.0),
            ko=inputs.device_normal((nseq, Hkv, T_own, dh), seed * 100 + 5 * i + 3, 1.0),
            vo=inputs.device_normal((nseq, Hkv, T_own, dh), seed * 100 + 5 * i + 4, 1.0),
        )
        if copied:
            rep = lambda t: t.repeat_interleave(samples, dim=0)
            c["k"] = torch.cat([rep(c["ks"]), c["ko"]], dim=2).contiguous()
            c["v"] = torch.cat([rep(c["vs"]), c["vo"]], dim=2).contiguous()
            if i > 0:
                del c["ks"], c["vs"], c["ko"], c["vo"]
        sets.append(c)
    ns_t = torch.full((B,), n_shared, dtype=torch.int32, device="cuda")
    no_t = torch.full((nseq,), n_own, dtype=torch.int32, device="cuda")
    n_t = torch.full((nseq,), n_shared + n_own, dtype=torch.int32, device="cuda")
    out = torch.empty((B, samples, q_len, Hq, dh), dtype=torch.bfloat16, device="cuda")
    if copied:
        d = binding.attn_desc(nseq, Hq, Hkv, dh, n_shared + T_own, 0, 1.0 / math.sqrt(dh), binding.BF16)
        ws = binding.workspace(binding.tandem_block_attn_workspace(d, q_len))
    else:
        d = binding.attn_desc(B, Hq, Hkv, dh, n_shared, 0, 1.0 / math.sqrt(dh), binding.BF16)
        ws = binding.workspace(binding.tandem_block_attn_shared_workspace(d, samples, T_own, q_len))

    def call(i):
        s = sets[i]
        if copied:
            binding.tandem_block_attn(s["q"].view(nseq, q_len, Hq, dh), s["k"], s["v"], n_t,
                                      out=out.view(nseq, q_len, Hq, dh), ws=ws)
        else:
            binding.tandem_block_attn_shared(s["q"], s["ks"], s["vs"], ns_t, s["ko"], s["vo"], no_t, out=out, ws=ws)

    def oracle_sample(n_prompts):
        from oracle import tandem_oracle as orc

        s = sets[0]
        f = inputs.torch_to_f64
        args = (f(s["q"][:n_prompts]), f(s["ks"][:n_prompts]), f(s["vs"][:n_prompts]), ns_t[:n_prompts].cpu().numpy(),
                f(s["ko"][:n_prompts * samples]), f(s["vo"][:n_prompts * samples]),
                no_t[:n_prompts * samples].cpu().numpy(), 1.0 / math.sqrt(dh))
        t0 = time.perf_counter()
        want = orc.block_attn_shared(*args)
        dt = time.perf_counter() - t0
        call(0)
        torch.cuda.synchronize()
        return dt, want.reshape(-1, Hq, dh), inputs.torch_to_f64(out[:n_prompts]).reshape(-1, Hq, dh)

    return call, R, bytes_alg, oracle_sample


def shared_draft_workload(torch, binding, inputs, B, samples, H, Hkv, dh, n_shared, n_own, n_cur, gmax, seed, copied=False):
    """Draft attention with `samples` continuations per prompt: the prompt's K_hat / V_hat rows stored and read once per
    prompt (tandem_draft_attn_shared), or - copied - tandem_draft_attn on per-sample caches that each hold a copy."""
    nseq = B * samples
    rows_own = n_own + n_cur
    bytes_alg = ((nseq * (n_shared + rows_own)) if copied else (B * n_shared + nseq * rows_own)) * Hkv * dh * 2 * 2
    R = _rotations(bytes_alg)
    sets = []
    for i in range(R):
        mk = lambda j, *sh: inputs.device_normal(sh, seed * 100 + 7 * i + j, 1.0)
        c = dict(q=mk(0, B, samples, H, dh), khs=mk(1, B, Hkv, n_shared, dh), vhs=mk(2, B, Hkv, n_shared, dh),
                 kho=mk(3, nseq, Hkv, n_own, dh), vho=mk(4, nseq, Hkv, n_own, dh),
                 kc=mk(5, nseq, Hkv, gmax, dh), vc=mk(6, nseq, Hkv, gmax, dh))
        if copied:
            rep = lambda t: t.repeat_interleave(samples, dim=0)
            c["k"] = torch.cat([rep(c["khs"]), c["kho"]], dim=2).contiguous()
            c["v"] = torch.cat([rep(c["vhs"]), c["vho"]], dim=2).contiguous()
            if i > 0:
                del c["khs"], c["vhs"], c["kho"], c["vho"]
        sets.append(c)
    i32 = lambda n, v: torch.full((n,), v, dtype=torch.int32, device="cuda")
    ns_t, no_t, nc_t, n_t = i32(B, n_shared), i32(nseq, n_own), i32(nseq, n_cur), i32(nseq, n_shared + n_own)
    out = torch.empty((B, samples, H, dh), dtype=torch.bfloat16, device="cuda")
    ws = binding.workspace(1 << 26)

    def call(i):
        s = sets[i]
        if copied:
            binding.tandem_draft_attn(s["q"].view(nseq, H, dh), s["k"], s["v"], n_t, s["kc"], s["vc"], nc_t,
                                      out=out.view(nseq, H, dh), ws=ws)
        else:
            binding.tandem_draft_attn_shared(s["q"], s["khs"], s["vhs"], ns_t, s["kho"], s["vho"], no_t, s["kc"], s["vc"],
                                             nc_t, out=out, ws=ws)

    def oracle_sample(n_prompts):
        from oracle import tandem_oracle as orc

        s = sets[0]
        f = inputs.torch_to_f64
        m = n_prompts * samples
        args = (f(s["q"][:n_prompts]), f(s["khs"][:n_prompts]), f(s["vhs"][:n_prompts]), ns_t[:n_prompts].cpu().numpy(),
                f(s["kho"][:m]), f(s["vho"][:m]), no_t[:m].cpu().numpy(), f(s["kc"][:m]), f(s["vc"][:m]),
                nc_t[:m].cpu().numpy(), 1.0 / math.sqrt(dh))
        t0 = time.perf_counter()
        want = orc.draft_attn_shared(*args)
        dt = time.perf_counter() - t0
        call(0)
        torch.cuda.synchronize()
        return dt, want.reshape(-1, H, dh), inputs.torch_to_f64(out[:n_prompts]).reshape(-1, H, dh)

    return call, R, bytes_alg, oracle_sample


def mixed_workload(torch, binding, inputs, B, q_len, H, Hkv, dh, n_prefix, gamma, seed):
    """All-positions small-model attention on q_len consecutive positions at the end of a context: the keys are the
    rows derived from the large model up to each query's block boundary plus a few own rows."""
    T_max = n_prefix + q_len
    bytes_alg = B * Hkv * T_max * dh * 2 * 2  # every visible position's K and V row once, from one cache or the other
    R = _rotations(bytes_alg)
    sets = []
    for i in range(R):
        sets.append({k: inputs.device_normal(sh, seed * 100 + 5 * i + j, 1.0) for j, (k, sh) in enumerate((
            ("q", (B, q_len, H, dh)), ("khat", (B, Hkv, T_max, dh)), ("vhat", (B, Hkv, T_max, dh)),
            ("kown", (B, Hkv, T_max, dh)), ("vown", (B, Hkv, T_max, dh))))})
    n = torch.full((B,), n_prefix, dtype=torch.int32, device="cuda")
    out = torch.empty((B, q_len, H, dh), dtype=torch.bfloat16, device="cuda")
    d = binding.attn_desc(B, H, Hkv, dh, T_max, 0, 1.0 / math.sqrt(dh), binding.BF16)
    ws = binding.workspace(binding.tandem_mixed_attn_workspace(d, q_len))

    def call(i):
        s = sets[i]
        binding.tandem_mixed_attn(s["q"], s["khat"], s["vhat"], s["kown"], s["vown"], n, gamma, out=out, ws=ws)

    def oracle_sample(n_seq):
        from oracle import tandem_oracle as orc

        s = sets[0]
        f = lambda t: inputs.torch_to_f64(t[:n_seq])
        args = (f(s["q"]), f(s["khat"]), f(s["vhat"]), f(s["kown"]), f(s["vown"]), n[:n_seq].cpu().numpy(), gamma,
                1.0 / math.sqrt(dh))
        t0 = time.perf_counter()
        want = orc.mixed_attn(*args)
        dt = time.perf_counter() - t0
        call(0)
        torch.cuda.synchronize()
        return dt, want.reshape(-1, H, dh), inputs.torch_to_f64(out[:n_seq]).reshape(-1, H, dh)

    return call, R, bytes_alg, oracle_sample


# ------------------------------------------------------------------ whole decode step
C3 = dict(
    B=32, gamma=4, ctx=8192, vocab=32768,
    large=dict(d=4096, n_layers=32, Hq=32, Hkv=8, dh=128, d_ff=16384),
    small=dict(d=1024, n_layers=8, Hq=8, Hkv=8, dh=128, d_ff=4096),
    d_hidden=8192,
)


def device_tandem_weights(inputs, cfg, seed):
    """Random-init Tandem pair generated directly in HBM: weights N(0, 0.02), gains 1, biases 0."""
    import torch

    ctr = [seed * 100000]

    def nrm(*shape):
        ctr[0] += 1
        return inputs.device_normal(shape, ctr[0], 0.02)

    def dec(c):
        def lay():
            return {"g_attn": torch.ones(c["d"], dtype=torch.bfloat16, device="cuda"),
                    "Wq": nrm(c["Hq"] * c["dh"], c["d"]), "Wk": nrm(c["Hkv"] * c["dh"], c["d"]),
                    "Wv": nrm(c["Hkv"] * c["dh"], c["d"]), "Wo": nrm(c["d"], c["Hq"] * c["dh"]),
                    "g_mlp": torch.ones(c["d"], dtype=torch.bfloat16, device="cuda"),
                    "W1": nrm(c["d_ff"], c["d"]), "b1": torch.zeros(c["d_ff"], dtype=torch.bfloat16, device="cuda"),
                    "W2": nrm(c["d"], c["d_ff"]), "b2": torch.zeros(c["d"], dtype=torch.bfloat16, device="cuda")}

        return {"emb": nrm(cfg["vocab"], c["d"]), "layers": [lay() for _ in range(c["n_layers"])],
                "g_final": torch.ones(c["d"], dtype=torch.bfloat16, device="cuda"), "W_out": nrm(cfg["vocab"], c["d"]),
                "Hq": c["Hq"], "Hkv": c["Hkv"], "dh": c["dh"]}

    L, S = dec(cfg["large"]), dec(cfg["small"])
    every = cfg["large"]["n_layers"] // cfg["small"]["n_layers"]
    ff = [{"W1": nrm(cfg["d_hidden"], cfg["large"]["d"]), "b1": torch.zeros(cfg["d_hidden"], dtype=torch.bfloat16, device="cuda"),
           "W2": nrm(cfg["small"]["d"], cfg["d_hidden"]), "b2": torch.zeros(cfg["small"]["d"], dtype=torch.bfloat16, device="cuda"),
           "act": "gelu"} for _ in range(cfg["small"]["n_layers"])]
    return {"L": L, "S": S, "ell": [every * (j + 1) for j in range(cfg["small"]["n_layers"])], "ff": ff, "eps": 1e-6}


def step_bytes(cfg):
    """Algorithmic HBM bytes of one decode step: every weight once per model run, every visible KV row once."""
    B, g, ctx = cfg["B"], cfg["gamma"], cfg["ctx"]

    def dec_w(c):
        per = (c["Hq"] + 2 * c["Hkv"]) * c["dh"] * c["d"] + c["d"] * c["Hq"] * c["dh"] + 2 * c["d"] * c["d_ff"]
        return 2 * (c["n_layers"] * per + cfg["vocab"] * c["d"])

    def kv(c, rows):
        return c["n_layers"] * B * c["Hkv"] * rows * c["dh"] * 2 * 2

    L, S = cfg["large"], cfg["small"]
    n = ctx - g
    draft = sum(dec_w(S) + kv(S, n + r + 1) for r in range(g))
    verify = dec_w(L) + kv(L, ctx)
    ff = S["n_layers"] * 2 * (cfg["d_hidden"] * L["d"] + S["d"] * cfg["d_hidden"] + 2 * S["Hkv"] * S["dh"] * S["d"])
    return draft + verify + ff


def step_workload(torch, binding, inputs, cfg, seed=3, pack_weights=True, free_token=False, adaptive=False):
    B, g, ctx = cfg["B"], cfg["gamma"], cfg["ctx"]
    W = device_tandem_weights(inputs, cfg, seed)
    model = binding.TandemModel(W, pack_weights=pack_weights)
    del W
    k = [seed * 7919]

    def fill(*shape):
        k[0] += 1
        return inputs.device_normal(shape, k[0], 1.0)

    state = binding.TandemState(model, B, ctx, g, fill=fill)
    q = g + 1 if free_token else g
    n0 = ctx - q
    state.n.fill_(n0)
    state.pending.fill_(1)
    ws = torch.empty(binding.tandem_decode_step_workspace(model, B, g), dtype=torch.uint8, device="cuda")
    out = {"tokens": torch.empty((B, q), dtype=torch.int32, device="cuda"),
           "n_accepted": torch.empty((B,), dtype=torch.int32, device="cuda")}
    router = None
    if adaptive:
        # random-init router of the adaptive block length (k = 4, 256 hidden units); the threshold 0.5 sits in
        # the middle of what such a router puts out, so the sequences stop at different block lengths
        S = cfg["small"]
        router = {"k": 4, "W1": inputs.device_normal((256, 1 + 4 * (S["d"] + 1)), seed * 31 + 1, 0.05),
                  "b1": inputs.device_normal((256,), seed * 31 + 2, 0.05),
                  "w2": inputs.device_normal((256,), seed * 31 + 3, 0.5),
                  "b2": inputs.device_normal((1,), seed * 31 + 4, 0.05)}
        out["n_drafted"] = torch.empty((B,), dtype=torch.int32, device="cuda")
        out["router_p"] = torch.empty((B, g), dtype=torch.float32, device="cuda")

    def call(_i):
        state.n.fill_(n0)       # keep the context at ctx: the step itself advances n
        state.pending.fill_(1)
        binding.tandem_decode_step(model, state, g, ws=ws, out=out, free_token=free_token, router=router, tau=0.5)

    return call, model, state, out


def run_prefill_workload(torch, binding, inputs, args):
    """One tandem_prefill call: 128 prompt tokens of each of 32 sequences appended at context 4096 (C3 pair)."""
    cfg = dict(C3)
    B, q, n0 = cfg["B"], 128, 4096
    W = device_tandem_weights(inputs, cfg, 3)
    model = binding.TandemModel(W, pack_weights=not args.plain_weights)
    del W
    k = [5]

    def fill(*shape):
        k[0] += 1
        return inputs.device_normal(shape, k[0], 1.0)

    state = binding.TandemState(model, B, cfg["ctx"], 4, fill=fill)
    toks = torch.randint(0, cfg["vocab"], (B, q), dtype=torch.int32, device="cuda", generator=torch.Generator("cuda").manual_seed(9))
    ws = torch.empty(binding.tandem_prefill_workspace(model, B, q), dtype=torch.uint8, device="cuda")

    def call(_i):
        state.n.fill_(n0)
        binding.tandem_prefill(model, state, toks, ws=ws)

    torch.cuda.synchronize()
    ms = _time_calls(torch, call, 1, args.steps, args.warmup, use_graph=not args.no_graph)
    L, S = cfg["large"], cfg["small"]
    M = B * q
    per_layer = (L["Hq"] + 2 * L["Hkv"]) * L["dh"] * L["d"] + L["d"] * L["Hq"] * L["dh"] + 2 * L["d"] * L["d_ff"]
    ff = S["n_layers"] * (cfg["d_hidden"] * L["d"] + S["d"] * cfg["d_hidden"] + 2 * S["Hkv"] * S["dh"] * S["d"])
    flops_dense = 2.0 * M * (L["n_layers"] * per_layer + ff)
    flops_attn = 4.0 * B * q * L["Hq"] * L["dh"] * (n0 + q / 2) * L["n_layers"]
    tflops = (flops_dense + flops_attn) / (ms * 1e-3) / 1e12
    return {
        "metric": "Tandem prompt ingestion tokens/sec (tandem_prefill, 128 tokens x 32 sequences per call)",
        "value": M / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "c3_prefill: tandem_prefill bf16 B=32, 128 rows per sequence at context 4096, C3 model pair "
                               "(M_L block pass + FF_Tandem + K_hat/V_hat rows; M_S does not run)",
                   "dense_TFLOP": flops_dense / 1e12, "attention_TFLOP": flops_attn / 1e12},
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / MFMA_PEAK_TFLOPS, "traffic": None},
        "cpu_baseline": None,
    }


def run_shared_step_workload(torch, binding, inputs, args):
    """tandem_decode_step_shared at the C3 pair: 8 prompts x 4 samples = 32 sequences, prompt 7936 rows (once per prompt),
    252 rows per sequence after it, gamma = 4."""
    cfg = dict(C3)
    P, ns, g = 8, 4, cfg["gamma"]
    B, Tp, To = P * ns, 7936, 256
    W = device_tandem_weights(inputs, cfg, 3)
    model = binding.TandemModel(W, pack_weights=not args.plain_weights)
    del W
    k = [11]

    def fill(*shape):
        k[0] += 1
        return inputs.device_normal(shape, k[0], 1.0)

    pst = binding.TandemState(model, P, Tp, g, fill=fill)
    pst.n.fill_(Tp)
    state = binding.TandemState(model, B, To, g, fill=fill)
    q = g + 1 if args.free_token else g
    n0 = To - q
    prompt = binding.TandemPrompt(pst, ns)
    ws = torch.empty(binding.tandem_decode_step_shared_workspace(model, B, ns, g), dtype=torch.uint8, device="cuda")
    out = {"tokens": torch.empty((B, q), dtype=torch.int32, device="cuda"),
           "n_accepted": torch.empty((B,), dtype=torch.int32, device="cuda")}

    def call(_i):
        state.n.fill_(n0)
        state.pending.fill_(1)
        binding.tandem_decode_step(model, state, g, ws=ws, out=out, free_token=args.free_token, prompt=prompt)

    torch.cuda.synchronize()
    ms = _time_calls(torch, call, 1, args.steps, args.warmup, use_graph=not args.no_graph)
    L, S = cfg["large"], cfg["small"]
    weights = step_bytes(dict(cfg, B=0))  # B = 0: no KV rows, the weights of every model run
    kv = lambda c, rows_p, rows_o: c["n_layers"] * c["Hkv"] * c["dh"] * 2 * 2 * (P * rows_p + B * rows_o)
    total = weights + kv(L, Tp, To) + sum(kv(S, Tp, n0 + r + 1) for r in range(g))
    gbs = total / (ms * 1e-3) / 1e9
    return {
        "metric": "Tandem decode steps/sec at gamma=4, 4 samples per prompt (prompt rows shared)",
        "value": 1e3 / ms, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c3_step_shared: tandem_decode_step_shared bf16, 8 prompts x 4 samples (B=32), prompt 7936 rows "
                               "once per prompt + 256 rows per sequence, gamma=4, C3 model pair"
                               + (", free token" if args.free_token else ""),
                   "step_algorithmic_GB": total / 1e9},
        "roofline": {"bound": "hbm", "kernel": "whole step (weights of every model run + every visible cache row once)",
                     "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None},
        "cpu_baseline": None,
    }


def run_score_workload(torch, binding, inputs, args):
    """One tandem_score call: the small model teacher-forced on 32 tokens of each of 32 sequences at context 4096 (C3
    pair; the large model's K_hat / V_hat rows are already in the state)."""
    cfg = dict(C3)
    B, q, n0, gamma = cfg["B"], 32, 4096, cfg["gamma"]
    W = device_tandem_weights(inputs, cfg, 3)
    model = binding.TandemModel(W, pack_weights=not args.plain_weights)
    del W
    k = [5]

    def fill(*shape):
        k[0] += 1
        return inputs.device_normal(shape, k[0], 1.0)

    state = binding.TandemState(model, B, cfg["ctx"], 4, fill=fill)
    S = cfg["small"]
    ko = [fill(B, S["Hkv"], cfg["ctx"], S["dh"]) for _ in range(S["n_layers"])]
    vo = [fill(B, S["Hkv"], cfg["ctx"], S["dh"]) for _ in range(S["n_layers"])]
    toks = torch.randint(0, cfg["vocab"], (B, q), dtype=torch.int32, device="cuda", generator=torch.Generator("cuda").manual_seed(9))
    pos = torch.full((B,), n0, dtype=torch.int32, device="cuda")
    ws = torch.empty(binding.tandem_score_workspace(model, B, q), dtype=torch.uint8, device="cuda")

    def call(_i):
        binding.tandem_score(model, state, ko, vo, pos, toks, gamma, ws=ws)

    torch.cuda.synchronize()
    ms = _time_calls(torch, call, 1, args.steps, args.warmup, use_graph=not args.no_graph)
    M = B * q
    # per layer the visible K_hat / V_hat and own rows cross HBM once; the weights are small (25 MB per layer)
    kv_bytes = S["n_layers"] * B * S["Hkv"] * (n0 + q) * S["dh"] * 2 * 2
    w_bytes = 2 * (S["n_layers"] * ((S["Hq"] + 2 * S["Hkv"]) * S["dh"] * S["d"] + S["d"] * S["Hq"] * S["dh"] + 2 * S["d"] * S["d_ff"])
                   + 2 * cfg["vocab"] * S["d"])
    gbs = (kv_bytes + w_bytes) / (ms * 1e-3) / 1e9
    return {
        "metric": "Tandem teacher-forced small-model scoring tokens/sec (tandem_score, 32 tokens x 32 sequences per call)",
        "value": M / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "c3_score: tandem_score bf16 B=32, 32 positions per sequence at context 4096, gamma=4, C3 small "
                               "model (8 layers, all-positions mixed attention, head over 32768 tokens)",
                   "kv_GB": kv_bytes / 1e9, "weight_GB": w_bytes / 1e9},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                     "traffic": None},
        "cpu_baseline": None,
    }


def run_deep_step_workload(torch, binding, inputs, args):
    """One tandem_deep_step call (Sec. 5): 32 sequences at context 8192, gamma = 4, C3 model pair plus an FF_DeepTandem of
    the configuration's FF_Tandem shape: M_L's block pass over the next 4 rows, then 4 runs of M_S."""
    cfg = dict(C3)
    B, g, ctx = cfg["B"], cfg["gamma"], cfg["ctx"]
    W = device_tandem_weights(inputs, cfg, 3)
    model = binding.TandemModel(W, pack_weights=not args.plain_weights)
    del W
    L, S = cfg["large"], cfg["small"]
    ffd = {"W1": inputs.device_normal((cfg["d_hidden"], L["d"]), 901, 0.02),
           "b1": torch.zeros(cfg["d_hidden"], dtype=torch.bfloat16, device="cuda"),
           "W2": inputs.device_normal((S["d"], cfg["d_hidden"]), 902, 0.02),
           "b2": torch.zeros(S["d"], dtype=torch.bfloat16, device="cuda"), "act": "gelu"}
    if not args.plain_weights:
        ffd["W1p"], ffd["W2p"] = binding.tandem_pack_weight(ffd["W1"]), binding.tandem_pack_weight(ffd["W2"])
    st = binding.DeepState(model, B, ctx)
    k = [17]
    for caches in (st.KL, st.VL, st.KS, st.VS):
        for j in range(len(caches)):
            k[0] += 1
            caches[j].copy_(inputs.device_normal(tuple(caches[j].shape), k[0], 1.0))
    n0 = ctx - g
    toks = torch.randint(0, cfg["vocab"], (B, ctx), dtype=torch.int32, device="cuda", generator=torch.Generator("cuda").manual_seed(9))
    length = torch.empty((B,), dtype=torch.int32, device="cuda")
    d = binding.ff_desc(ffd)
    ws = torch.empty(int(binding.lib().tandem_deep_score_workspace(model.handle, d, B, g)), dtype=torch.uint8, device="cuda")

    def call(_i):
        length.fill_(n0)  # keep the context at ctx: the step itself advances the lengths
        binding.tandem_deep_step(model, ffd, st, toks, length, g, ws=ws)

    torch.cuda.synchronize()
    ms = _time_calls(torch, call, 1, args.steps, args.warmup, use_graph=not args.no_graph)
    per = lambda c: (c["Hq"] + 2 * c["Hkv"]) * c["dh"] * c["d"] + c["d"] * c["Hq"] * c["dh"] + 2 * c["d"] * c["d_ff"]
    kv = lambda c, rows: c["n_layers"] * B * c["Hkv"] * rows * c["dh"] * 2 * 2
    seen_L = (n0 // g) * g  # rows of the blocks completed before the new rows' block
    total = (2 * L["n_layers"] * per(L) + kv(L, seen_L) + 2 * (cfg["d_hidden"] * L["d"] + S["d"] * cfg["d_hidden"])
             + sum(2 * (S["n_layers"] * per(S) + cfg["vocab"] * S["d"]) + kv(S, n0 + t) for t in range(g)))
    gbs = total / (ms * 1e-3) / 1e9
    return {
        "metric": "Deep Tandem decoding steps/sec at gamma=4 (tandem_deep_step)",
        "value": 1e3 / ms, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c3_deep_step: tandem_deep_step bf16 B=32, context 8192, gamma=4, C3 model pair with an "
                               "FF_DeepTandem MLP 4096-8192-1024 (M_L block pass with block-prefix attention, 4 runs of M_S "
                               "with causal attention over its own rows)",
                   "step_algorithmic_GB": total / 1e9},
        "roofline": {"bound": "hbm", "kernel": "whole step (weights of every model run + every visible cache row once)",
                     "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None},
        "cpu_baseline": None,
    }


def cpu_step_estimate(torch, inputs, cfg, state, model):
    """Oracle pieces of one step timed on sampled slices (one sequence / one layer each), extrapolated by
    the layer, run and batch counts.  The full fp64 step is ~2 TFLOP and is not run."""
    import numpy as np

    from oracle import tandem_oracle as orc

    B, g, ctx = cfg["B"], cfg["gamma"], cfg["ctx"]
    L, S = cfg["large"], cfg["small"]
    n = ctx - g
    rng = np.random.default_rng(0)
    t = {}
    f = lambda x: inputs.torch_to_f64(x)
    # attention: one sequence of one layer each
    kc, vc = f(state.Khat[0][:1]), f(state.Vhat[0][:1])
    q = rng.standard_normal((1, S["Hq"], S["dh"]))
    kcur = rng.standard_normal((1, S["Hkv"], g, S["dh"]))
    t0 = time.perf_counter()
    orc.draft_attn(q, kc, vc, [n], kcur, kcur, [g], S["dh"] ** -0.5)
    t["draft_attn_1seq"] = time.perf_counter() - t0
    kc, vc = f(state.KL[0][:1]), f(state.VL[0][:1])
    q = rng.standard_normal((1, g, L["Hq"], L["dh"]))
    t0 = time.perf_counter()
    orc.block_attn(q, kc, vc, [n], L["dh"] ** -0.5)
    t["block_attn_1seq"] = time.perf_counter() - t0
    del kc, vc

    # dense: products of the right shape on a quarter of the output features, scaled by 4
    def dense(rows, c):
        per = (c["Hq"] + 2 * c["Hkv"]) * c["dh"] * c["d"] + c["d"] * c["Hq"] * c["dh"] + 2 * c["d"] * c["d_ff"]
        nq = per // c["d"] // 4
        Wq = rng.standard_normal((nq, c["d"]))
        x = rng.standard_normal((rows, c["d"]))
        t0 = time.perf_counter()
        orc.linear(x, Wq)
        return (time.perf_counter() - t0) * 4

    t["large_layer_dense"] = dense(B * g, L)
    t["small_layer_dense"] = dense(B, S)
    ffW = {"W1": rng.standard_normal((cfg["d_hidden"] // 4, L["d"])), "W2": rng.standard_normal((S["d"], cfg["d_hidden"] // 4))}
    x = rng.standard_normal((B * g, L["d"]))
    t0 = time.perf_counter()
    orc.project(x, ffW)
    t["project"] = (time.perf_counter() - t0) * 4
    Wh = rng.standard_normal((cfg["vocab"] // 4, L["d"]))
    t0 = time.perf_counter()
    orc.linear(x, Wh)
    t["large_head"] = (time.perf_counter() - t0) * 4
    est = (L["n_layers"] * (t["large_layer_dense"] + B * t["block_attn_1seq"])
           + g * S["n_layers"] * (t["small_layer_dense"] + B * t["draft_attn_1seq"])
           + S["n_layers"] * t["project"] + t["large_head"] * (1 + g * S["d"] / L["d"] * B / (B * g)))
    return est, t


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
    # the latency evaluation's 4 samples per prompt at the C3 layer shape: 8 prompts of 7936 rows, each sample
    # 251 rows past the prompt, a block of gamma + 1 = 5 rows
    "s4_shared": ("shared", dict(B=8, samples=4, q_len=5, Hq=32, Hkv=8, dh=128, n_shared=7936, n_own=251, seed=5), 1,
                  "tandem_block_attn_shared bf16 8 prompts x 4 samples, Hq/Hkv=32/8 dh=128, prompt 7936 rows read once "
                  "per prompt + 256 own rows per sample, 5 query rows"),
    "s4_draft_shared": ("shared_draft", dict(B=8, samples=4, H=8, Hkv=8, dh=128, n_shared=7936, n_own=248, n_cur=4, gmax=4,
                                             seed=7), 1,
                        "tandem_draft_attn_shared bf16 8 prompts x 4 samples, H=8 dh=128, prompt 7936 K_hat rows read once per "
                        "prompt + 248 own + 4 current rows per sample"),
    "s4_draft_copied": ("shared_draft", dict(B=8, samples=4, H=8, Hkv=8, dh=128, n_shared=7936, n_own=248, n_cur=4, gmax=4,
                                             seed=7, copied=True), 1,
                        "tandem_draft_attn bf16 on 32 per-sample caches that each hold a copy of the 7936 prompt rows (the "
                        "form tandem_draft_attn_shared replaces; same values)"),
    # teacher-forced scoring with the small model: 32 consecutive positions of every sequence at the end of an 8192
    # context, C3's small-layer shape, block length 4
    "c3_mixed": ("mixed", dict(B=32, q_len=32, H=8, Hkv=8, dh=128, n_prefix=8160, gamma=4, seed=6), 1,
                 "tandem_mixed_attn bf16 B=32 H=8 dh=128, 32 query positions at context 8160+32, gamma=4"),
    "s4_copied": ("shared", dict(B=8, samples=4, q_len=5, Hq=32, Hkv=8, dh=128, n_shared=7936, n_own=251, seed=5,
                                 copied=True), 1,
                  "tandem_block_attn bf16 on 32 per-sample caches that each hold a copy of the 7936 prompt rows "
                  "(the form tandem_block_attn_shared replaces; same values)"),
}


# ------------------------------------------------------------------ FF_Tandem projection
MFMA_PEAK_TFLOPS = 2500.0
PROJECT_WORKLOADS = {
    # the benchmark's projection 4096 -> 8192 -> 1024 (GELU) on M rows
    "c2_project": (64, "tandem_project bf16 M=64 (batch 16 x gamma 4) 4096->8192->1024"),
    "c3_project": (128, "tandem_project bf16 M=128 (batch 32 x gamma 4) 4096->8192->1024"),
    "project_m512": (512, "tandem_project bf16 M=512 (batch 64 x gamma 8) 4096->8192->1024"),
    "project_m4096": (4096, "tandem_project bf16 M=4096 (prompt-time, one 4096-token prompt) 4096->8192->1024"),
    "project_m65536": (65536, "tandem_project bf16 M=65536 (prompt-time, 16 prompts of 4096 tokens) 4096->8192->1024"),
}


def run_project_workload(torch, binding, inputs, args):
    M, desc = PROJECT_WORKLOADS[args.workload]
    d_L, d_h, d_S = 4096, 8192, 1024
    wbytes = 2 * (d_h * d_L + d_S * d_h)
    R = _rotations(wbytes)
    ffs = [{"W1": inputs.device_normal((d_h, d_L), 700 + 2 * i, 0.02), "b1": torch.zeros(d_h, dtype=torch.bfloat16, device="cuda"),
            "W2": inputs.device_normal((d_S, d_h), 701 + 2 * i, 0.02), "b2": torch.zeros(d_S, dtype=torch.bfloat16, device="cuda"),
            "act": "gelu"} for i in range(R)]
    if not args.plain_weights:  # weights are static: packed once, outside the timed region, as a deployed model holds them
        for ff in ffs:
            ff["W1p"], ff["W2p"] = binding.tandem_pack_weight(ff["W1"]), binding.tandem_pack_weight(ff["W2"])
    x = inputs.device_normal((M, d_L), 699, 1.0)
    y = torch.empty((M, d_S), dtype=torch.bfloat16, device="cuda")
    ws = binding.workspace(binding.tandem_project_workspace(binding.ff_desc(ffs[0]), M))
    call = lambda i: binding.tandem_project(ffs[i], x, out=y, ws=ws)
    torch.cuda.synchronize()
    ms = _time_calls(torch, call, R, args.steps, args.warmup, use_graph=not args.no_graph)
    flops = 2.0 * M * (d_L * d_h + d_h * d_S)
    bytes_alg = wbytes + 2 * M * (d_L + 2 * d_h + d_S)  # weights once; x read, hidden written and read, y written
    tflops = flops / (ms * 1e-3) / 1e12
    gbs = bytes_alg / (ms * 1e-3) / 1e9
    hbm_bound = flops / bytes_alg < MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    cpu = None
    if not args.no_cpu_baseline:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from oracle import tandem_oracle as orc
        from parity import row_errors

        rows = min(M, 64)
        ff64 = {k: (inputs.torch_to_f64(v) if hasattr(v, "shape") else v) for k, v in ffs[0].items() if not k.endswith("p")}
        xs = inputs.torch_to_f64(x[:rows])
        t0 = time.perf_counter()
        want = orc.project(xs, ff64)
        dt = time.perf_counter() - t0
        call(0)
        torch.cuda.synchronize()
        e_inf, _ = row_errors(inputs.torch_to_f64(y[:rows]), want)
        cpu = {"value": flops * rows / M / dt / 1e12, "unit": "TFLOP/s", "cores": _cpu_threads(), "kind": "oracle",
               "sample": f"first {rows} of {M} rows, fp64 numpy, {dt:.2f} s", "gpu_max_rel_err_on_sample": float(e_inf.max())}
    roof = ({"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}
            if hbm_bound else
            {"bound": "mfma", "achieved": tflops, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops / MFMA_PEAK_TFLOPS})
    roof["traffic"] = _traffic(args.workload)
    return {
        "metric": "FF_Tandem projection TFLOP/s (bf16 MFMA)", "value": tflops, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc}", "rotated_weight_sets": R, "packed_weights": not args.plain_weights, "frac_of_mfma_peak": tflops / MFMA_PEAK_TFLOPS,
                   "weight_stream_GBps": wbytes / (ms * 1e-3) / 1e9},
        "roofline": roof, "cpu_baseline": cpu,
    }


def _traffic(name):
    """HBM traffic per launch measured offline with rocprofv3 counters (profiles/measured.json), or None."""
    m = _measured(name)
    return m.get("hbm_bytes_per_launch") if m else None


def run_kernel_workload(torch, binding, inputs, args):
    kind, kw, n_seq, desc = WORKLOADS[args.workload]
    maker = {"draft": draft_workload, "block": block_workload, "shared": shared_workload, "mixed": mixed_workload,
             "shared_draft": shared_draft_workload}[kind]
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
    return {
        "metric": "Tandem attention HBM GB/s (algorithmic KV bytes / time)",
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {desc}", "rotated_copies": n_copies},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                     "traffic": _traffic(args.workload)},
        "cpu_baseline": cpu,
    }


def _quick_extra(torch, binding, inputs, args):
    """Short timings of the other configurations' entry points, so that one default run shows every number the
    target names: C1 / C2 / C4 attention (HBM-bound) and FF_Tandem at decode and prompt sizes."""
    import gc

    extra = {}
    for name in ("c1_draft", "c2_block", "c4_draft", "c4_block"):
        kind, kw, _n, _desc = WORKLOADS[name]
        maker = {"draft": draft_workload, "block": block_workload}[kind]
        call, n_copies, bytes_alg, _oracle = maker(torch, binding, inputs, **kw)
        torch.cuda.synchronize()
        ms = _time_calls(torch, call, n_copies, 60 if name.startswith("c4") else 200, 10, use_graph=not args.no_graph)
        gbs = bytes_alg / (ms * 1e-3) / 1e9
        extra[name] = {"us": ms * 1e3, "GBps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
        del call, _oracle
        gc.collect()
        torch.cuda.empty_cache()
    for name in ("c2_project", "c3_project", "project_m4096"):
        sub = argparse.Namespace(**vars(args))
        sub.workload, sub.no_cpu_baseline = name, True
        sub.steps, sub.warmup = (20, 5) if name == "project_m4096" else (200, 20)
        line = run_project_workload(torch, binding, inputs, sub)
        extra[name] = {"us": line["ms_per_step"] * 1e3, "TFLOPs": line["value"], "roofline": {k: line["roofline"][k] for k in ("bound", "frac")}}
        gc.collect()
        torch.cuda.empty_cache()
    return extra


def _read_ceiling(torch, binding, tensors, use_graph):
    """Rate of the library's plain read-only stream kernel over the given (large, distinct) device tensors."""
    sink = torch.empty(binding.READ_STREAM_BLOCKS, dtype=torch.int32, device="cuda")
    call = lambda i: binding.tandem_read_stream(tensors[i], sink)
    ms = _time_calls(torch, call, len(tensors), 4 * len(tensors), 4, use_graph=use_graph)
    nbytes = tensors[0].numel() * tensors[0].element_size()
    return nbytes / (ms * 1e-3) / 1e9


def _measured(name):
    """Figures taken offline with rocprofv3 and kept under profiles/ (measured.json names the summary each comes from)."""
    path = os.path.join(ROOT, "profiles", "measured.json")
    try:
        with open(path) as f:
            return json.load(f).get(name)
    except Exception:
        return None


def run_step_workload(torch, binding, inputs, args):
    cfg = C3
    B, g, ctx = cfg["B"], cfg["gamma"], cfg["ctx"]
    call, model, state, out = step_workload(torch, binding, inputs, cfg, pack_weights=not args.plain_weights,
                                            free_token=args.free_token, adaptive=args.adaptive)
    torch.cuda.synchronize()
    ms = _time_calls(torch, call, 1, args.steps, args.warmup, use_graph=not args.no_graph)

    # dominant kernels, timed alone in the launch configuration the step uses (same caches, one layer
    # after the other, so every launch streams 1.07 GB that is not in the Infinity Cache)
    L, S = cfg["large"], cfg["small"]
    n_dev = torch.full((B,), ctx - g, dtype=torch.int32, device="cuda")
    qL = inputs.device_normal((B, g, L["Hq"], L["dh"]), 991, 1.0)
    oL = torch.empty_like(qL)
    dL = binding.attn_desc(B, L["Hq"], L["Hkv"], L["dh"], ctx, 0, L["dh"] ** -0.5, binding.BF16)
    wsL = torch.empty(max(256, binding.tandem_block_attn_workspace(dL, g)), dtype=torch.uint8, device="cuda")
    blk = lambda i: binding.tandem_block_attn(qL, state.KL[i], state.VL[i], n_dev, out=oL, ws=wsL)
    ms_blk = _time_calls(torch, blk, L["n_layers"], 2 * L["n_layers"], 4, use_graph=not args.no_graph)
    qS = inputs.device_normal((B, S["Hq"], S["dh"]), 992, 1.0)
    oS = torch.empty_like(qS)
    nc = torch.full((B,), g, dtype=torch.int32, device="cuda")
    dS = binding.attn_desc(B, S["Hq"], S["Hkv"], S["dh"], ctx, g, S["dh"] ** -0.5, binding.BF16)
    wsS = torch.empty(max(256, binding.tandem_draft_attn_workspace(dS)), dtype=torch.uint8, device="cuda")
    drf = lambda i: binding.tandem_draft_attn(qS, state.Khat[i], state.Vhat[i], n_dev, state.Kcur[i], state.Vcur[i], nc,
                                              out=oS, ws=wsS)
    ms_drf = _time_calls(torch, drf, S["n_layers"], 8 * S["n_layers"], 4, use_graph=not args.no_graph)
    bytes_blk = B * L["Hkv"] * ctx * L["dh"] * 2 * 2
    bytes_drf = B * S["Hkv"] * ctx * S["dh"] * 2 * 2
    gbs_blk = bytes_blk / (ms_blk * 1e-3) / 1e9
    gbs_drf = bytes_drf / (ms_drf * 1e-3) / 1e9
    total_bytes = step_bytes(cfg)
    # the box's read ceiling: the plain read-only stream kernel over the same caches (537 MB each, one after the other)
    ceiling = _read_ceiling(torch, binding, state.KL[:8], not args.no_graph)

    def roof(kernel, gbs, ms_launch, key):
        prof = _measured(key) or {}
        r = {"bound": "hbm", "kernel": kernel, "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
             "frac_is": "kernel launched alone in the step's launch configuration (live HIP events, this run)",
             "ms_per_launch": ms_launch, "read_stream_ceiling_GBps": ceiling, "frac_of_read_ceiling": gbs / ceiling,
             "traffic": prof.get("hbm_bytes_per_launch"), "traffic_source": prof.get("traffic_source")}
        if prof.get("in_step_us"):
            bytes_alg = bytes_blk if key == "c3_block" else bytes_drf
            r["in_step"] = {"us": prof["in_step_us"], "frac": bytes_alg / (prof["in_step_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS,
                            "source": prof.get("in_step_source")}
        return r

    cpu = None
    if not args.no_cpu_baseline:
        est, parts = cpu_step_estimate(torch, inputs, cfg, state, model)
        cpu = {"value": 1.0 / est, "unit": "steps/s", "cores": _cpu_threads(), "kind": "oracle",
               "sample": "fp64 numpy oracle pieces timed on the step's own caches (sequence 0 of layer 0 for the draft and the "
                         "block attention: single-threaded loops over heads and rows around BLAS calls) and on a quarter of one "
                         "layer's dense products (BLAS, `cores` threads), extrapolated by layer, run and batch counts: "
                         + ", ".join(f"{k}={v:.3f}s" for k, v in parts.items())
                         + "; no parity is taken on these slices (parity at this configuration: tests/test_gpu_full_size.py)"}
    extra = None if args.no_extra else _quick_extra(torch, binding, inputs, args)
    return {
        "metric": "Tandem decode steps/sec at gamma=4 (draft/verify attention HBM GB/s in roofline)",
        "value": 1e3 / ms, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c3_step: tandem_decode_step bf16 B=32 ctx=8192 gamma=4, large 32L d=4096 32/8x128, "
                               "small 8L d=1024 8x128, FF_Tandem 4096->8192->1024, vocab 32768"
                               + (", free token (5 verified rows)" if args.free_token else "")
                               + (", adaptive block length (random-init router, k=4, 256 units, tau=0.5; block lengths "
                                  f"drafted in the last step: {sorted(out['n_drafted'].cpu().tolist())})" if args.adaptive else ""),
                   "step_algorithmic_GB": total_bytes / 1e9, "step_GBps": total_bytes / (ms * 1e-3) / 1e9,
                   "step_frac_of_hbm_peak": total_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "roofline": roof("attn_block_kernel (tandem_block_attn, one large layer of the step)", gbs_blk, ms_blk, "c3_block"),
        "roofline_draft": roof("attn_rows_kernel (tandem_draft_attn, one small layer of the step)", gbs_drf, ms_drf, "c3_draft"),
        "cpu_baseline": cpu,
        "extra": extra,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c3_step", choices=sorted(WORKLOADS) + sorted(PROJECT_WORKLOADS) + ["c3_step", "c3_prefill", "c3_score", "c3_step_shared", "c3_deep_step"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--plain-weights", action="store_true",
                    help="read weights in the caller's row-major layout only (no packed copies)")
    ap.add_argument("--no-extra", action="store_true",
                    help="c3_step: skip the short timings of the other configurations (C1, C2, C4, FF_Tandem)")
    ap.add_argument("--adaptive", action="store_true",
                    help="c3_step: run the step with the adaptive block length (tandem_decode_step_adaptive)")
    ap.add_argument("--free-token", action="store_true",
                    help="c3_step only: verify gamma + 1 rows and emit the bonus token (Fig. 2)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run three plain 1 GiB device copies (known traffic) so that rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings of the same run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    step = args.workload == "c3_step"
    if args.steps is None:
        args.steps = 20 if step else 200
    if args.warmup is None:
        args.warmup = 3 if step else 20

    import torch

    from paper_2402_08644_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.lib()  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    runner = run_step_workload if step else (run_project_workload if args.workload in PROJECT_WORKLOADS else run_kernel_workload)
    if args.workload == "c3_prefill":
        runner = run_prefill_workload
        args.steps = min(args.steps, 10)
    if args.workload == "c3_step_shared":
        runner = run_shared_step_workload
        args.steps = min(args.steps, 20)
    if args.workload == "c3_deep_step":
        runner = run_deep_step_workload
        args.steps = min(args.steps, 20)
    if args.workload == "c3_score":
        runner = run_score_workload
        args.steps = min(args.steps, 20)
    if args.workload in ("project_m4096", "project_m65536"):
        args.steps = min(args.steps, 20)
    line = runner(torch, binding, inputs, args)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
