#!/usr/bin/env python3
"""Benchmark of the generation hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input: prefill of B prompts
of P tokens plus G-1 decode steps (B*G generated tokens), free-running greedy generation with on-device
token feedback.  Prints ONE JSON line: `value` = generated tokens/s of the whole step (weight re-layout + prefill + decode),
`phases` = prefill TFLOP/s and decode algorithmic GB/s with their fractions of the published peaks, `roofline` = the dominant
kernel (decode attention) timed with HIP events on the launch stream against its algorithmic bytes, `cpu_baseline` = the CPU
oracle timed on a bounded sample of the same model.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama7b] [--no-cpu-baseline] [--no-roofline] [--mbs N]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

DTYPE = "f16 x bf16 -> fp32 on the matrix cores (f16 activations, as two-term sums where the precision level asks; 16-bit KV cache)"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense 16-bit matrix cores (bf16 and fp16), published
# HBM bytes per decode-attention launch (mean over the launches of one generation) as rocprofv3 counters saw them in a
# separate profiling run of this benchmark: FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for the
# library's 1 GiB copy_kernel.  A RECORDED figure (the counters cannot be read from inside this process): it is reported
# with its source file, and only for the unmodified workload it was recorded on.
RECORDED_TRAFFIC = {"llama7b": {"bytes": 537160 * 1024, "source": "profiles/decode_attention_llama7b_hbm_traffic.md"}}


def kv_row_bytes(shape, block_scaled):
    """Bytes of one cache row (head_dim 16-bit elements, plus the fp32 scale of a block-scaled row)."""
    return shape.head_dim * 2 + (4 if block_scaled else 0)


def decode_bytes(shape, B, t, block_scaled=False):
    """Algorithmic HBM bytes of one decode step at position t (the new token attends to t+1 cache rows):
    every weight once, the KV cache rows read, the appended K/V rows, the fp32 logits, the embedding rows."""
    d, hd, Hq, Hkv, F, V, L = shape.hidden, shape.head_dim, shape.n_heads, shape.n_kv_heads, shape.ffn, shape.vocab, shape.n_layers
    w = 2 * (L * ((Hq + 2 * Hkv) * hd * d + Hq * hd * d + 3 * d * F + 2 * d) + d + V * d)
    kv_row = 2 * L * Hkv * kv_row_bytes(shape, block_scaled)
    return w + B * (t + 1) * kv_row + B * kv_row + B * V * 4 + B * d * 2


def attention_bytes(shape, B, t, block_scaled=False):
    """Algorithmic bytes of ONE decode-attention launch (one layer) at position t: K and V rows 0..t of every
    (sequence, kv head), the fp32 queries and the 16-bit outputs."""
    hd, Hq, Hkv = shape.head_dim, shape.n_heads, shape.n_kv_heads
    return B * (t + 1) * 2 * Hkv * kv_row_bytes(shape, block_scaled) + B * Hq * hd * (4 + 2)


def decode_kernel_models(shape, B, P, G, block_scaled, level):
    """Per kernel class of a decode step: algorithmic bytes per launch (weights once + activations in + results out; for
    attention the mean over the positions of the generation) and executed flops per launch (second activation terms
    included).  M = B rows."""
    d, hd, Hq, Hkv, F, V = shape.hidden, shape.head_dim, shape.n_heads, shape.n_kv_heads, shape.ffn, shape.vocab
    qd, kvd, M = Hq * hd, Hkv * hd, B
    nqkv = qd + 2 * kvd
    t_o, t_act, t_ffn = (2 if level >= 2 else 1), (2 if level >= 2 else 1), (2 if level >= 3 else 1)
    att = sum(attention_bytes(shape, B, t, block_scaled) for t in range(P, P + G - 1)) / max(G - 1, 1)
    return {
        "gemm_qkv": {"bytes": nqkv * d * 2 + 2 * M * d * 2 + M * nqkv * 4, "flops": 2 * 2 * M * nqkv * d},
        "gemm_o": {"bytes": d * qd * 2 + t_o * M * qd * 2 + M * d * 4, "flops": 2 * t_o * M * d * qd},
        "gemm_gate_up": {"bytes": 2 * F * d * 2 + t_ffn * M * d * 2 + t_act * M * F * 2, "flops": 2 * t_ffn * M * 2 * F * d},
        "gemm_down": {"bytes": d * F * 2 + t_act * M * F * 2 + M * d * 4, "flops": 2 * t_act * M * d * F},
        # free-running greedy decode: the LM head leaves per-pass candidates (value + column per 128 columns) instead of logits
        "gemm_lm_head": {"bytes": V * d * 2 + t_ffn * M * d * 2 + M * ((V + 127) // 128) * 8, "flops": 2 * t_ffn * M * V * d},
        "add_rmsnorm": {"bytes": M * d * (4 + 4 + 2 * 2), "flops": 0},
        "rope_append": {"bytes": M * nqkv * 4 + M * qd * 4 + 2 * M * Hkv * kv_row_bytes(shape, block_scaled), "flops": 0},
        "decode_attention": {"bytes": att, "flops": 0},
        "argmax": {"bytes": M * ((V + 127) // 128) * 8 + M * 4, "flops": 0},
        "embed": {"bytes": M * d * (2 + 4), "flops": 0},
    }


def prefill_flops(shape, B, P):
    d, hd, Hq, Hkv, F, V, L = shape.hidden, shape.head_dim, shape.n_heads, shape.n_kv_heads, shape.ffn, shape.vocab, shape.n_layers
    return 2 * B * P * L * ((Hq + 2 * Hkv) * hd * d + Hq * hd * d + 3 * d * F) + 2 * B * V * d + 4 * L * B * Hq * hd * P * (P + 1) // 2


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llama7b")
    ap.add_argument("--layers", type=int, default=0, help="debug: truncate the model depth (the result is then not the benchmark)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--call", default="generation", choices=["generation", "logprobs"],
                    help="generation (the benchmark) or the inference call that scores every token of [B, P+G] sequences")
    ap.add_argument("--pack-gate-up", default="auto", choices=["auto", "on", "off"],
                    help="fragment-order copies of the gate/up pair too (auto: where the library prefers them and memory allows)")
    ap.add_argument("--mbs", type=int, default=1,
                    help="generation only: run the batch as this many sequential portions through rl_gen_generate on a "
                         "generator (and KV cache) of batch/mbs sequences; not the headline configuration")
    ap.add_argument("--precision", type=int, default=0, choices=[0, 1, 2, 3],
                    help="rl_gen_shape.precision: 0 = the library's default for the shape (the benchmark; what the parity tests "
                         "cover at full depth), 1-3 force a level (1 is faster and misses the parity bar at full depth)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (copy_kernel: a known-size kernel to scale profiler byte counters by)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the data-parallel hot path of one GPU's share); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2406_14088_amd import Generator, kv_block_scaled, precision_level
    from workload import PRESETS, make_prompts, make_weights

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = "cuda:0"
    wl = PRESETS[args.workload]
    shape = wl.shape.with_layers(args.layers) if args.layers else wl.shape
    B, P, G = wl.batch, wl.prompt_len, wl.gen_len
    level, bs = precision_level(shape, args.precision), kv_block_scaled(shape, args.precision)

    t0 = time.perf_counter()
    W = make_weights(shape, wl.index, device=dev)
    prompts = make_prompts(wl, device=dev)
    if args.mbs < 1 or B % args.mbs:
        print(f"bench.py: --mbs must divide the batch ({B})", file=sys.stderr)
        sys.exit(2)
    gen = Generator(shape, W, B // args.mbs, P + G, pack_gate_up={"auto": None, "on": True, "off": False}[args.pack_gate_up],
                    precision=args.precision)
    gen.set_graph(not args.no_graph)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t0

    if args.mbs > 1 and args.call == "generation":
        print(json.dumps(bench_portions(args, gen, wl, shape, prompts, setup_s)))
        gen.close()
        return

    if args.call == "logprobs":
        print(json.dumps(bench_logprobs(args, gen, wl, shape, dev, setup_s)))
        gen.close()
        return

    buf = [torch.empty((B,), dtype=torch.int32, device=dev) for _ in range(2)]
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        from paper_2406_14088_amd import ops
        for _ in range(3):
            ops.copy(src, dst)            # copy_kernel of the library: 16 bytes per lane, like the hot kernels
        torch.cuda.synchronize()
        del src, dst

    def generate(timing=None, after_prefill=None):
        """weight re-layout + prefill + (G-1) decode steps; tokens stay on the device.  The fragment-order weight copies
        are rebuilt inside every step: in the RLHF loop each generation phase starts from freshly trained weights."""
        if timing is not None:
            torch.cuda.synchronize()
            tp = time.perf_counter()
        gen.pack_weights()
        if timing is not None:
            torch.cuda.synchronize()
            ta = time.perf_counter()
            timing["pack_s"] = timing.get("pack_s", 0.0) + ta - tp
        gen.prefill(prompts, next_tokens=buf[0])
        if after_prefill is not None:
            after_prefill()
        if timing is not None:
            torch.cuda.synchronize()
            tb = time.perf_counter()
        cur = 0
        marks = {}
        for i in range(G - 1):
            if timing is not None and i in (1, (G - 1) // 2, G - 2):     # single steps early, in the middle and at the end
                marks[i] = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                marks[i][0].record()
            gen.decode_step(buf[cur], next_tokens=buf[1 - cur], want_logits=False)
            if i in marks:
                marks[i][1].record()
            cur = 1 - cur
        if timing is not None:
            torch.cuda.synchronize()
            tc = time.perf_counter()
            timing["step_ms"] = {i: m[0].elapsed_time(m[1]) for i, m in marks.items()}
            timing["prefill_s"] = timing.get("prefill_s", 0.0) + tb - ta
            timing["decode_s"] = timing.get("decode_s", 0.0) + tc - tb
        return buf[cur]

    for _ in range(args.warmup):
        generate()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        last = generate()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    tokens = B * G * args.steps
    value = tokens / elapsed
    last_tokens = last.clone()

    # split of one generation into prefill and decode (separate, synchronised pass; not part of `value`)
    split = {}
    generate(split)
    dec_bytes = sum(decode_bytes(shape, B, t, bs) for t in range(P, P + G - 1))
    pf = prefill_flops(shape, B, P)
    phases = {
        "pack_weights_ms": split["pack_s"] * 1e3,
        "prefill_ms": split["prefill_s"] * 1e3,
        "prefill_tflops": pf / split["prefill_s"] / 1e12,
        "prefill_frac_of_mfma_peak": pf / split["prefill_s"] / 1e12 / MFMA_PEAK_TFLOPS,
        "decode_ms_per_step": split["decode_s"] * 1e3 / max(G - 1, 1),
        "decode_algorithmic_GBs": dec_bytes / split["decode_s"] / 1e9,
        "decode_frac_of_hbm_peak": dec_bytes / split["decode_s"] / 1e9 / HBM_PEAK_GBS,
        "decode_tokens_per_s": B * (G - 1) / split["decode_s"],
        # single decode steps (events on the launch stream): position, ms, algorithmic GB/s
        "decode_steps": [{"position": P + i, "ms": ms, "algorithmic_GBs": decode_bytes(shape, B, P + i, bs) / (ms * 1e-3) / 1e9}
                         for i, ms in sorted(split["step_ms"].items())],
    }

    out = {
        "metric": "generated tokens/sec on 1 GPU + decode-step HBM GB/s (% peak), LLaMA-7B shape" if args.workload == "llama7b"
        else f"generated tokens/sec on 1 GPU + decode-step HBM GB/s (% peak), {args.workload}",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": f"{wl.name}: L{shape.n_layers} d{shape.hidden} H{shape.n_heads}/{shape.n_kv_heads} F{shape.ffn} "
                               f"V{shape.vocab}, batch {B}, prompt {P}, generate {G}",
                   "global_batch": B, "prompt_len": P, "gen_len": G, "hip_graph": not args.no_graph,
                   "packed_gate_up_layers": gen.packed_gate_up_layers(), "precision_level": level,
                   "precision_forced": args.precision != 0,
                   "kv_cache": "int16 rows with one fp32 scale each" if bs else "IEEE half rows"},
        "phases": phases, "setup_s": setup_s,
    }

    if not args.no_roofline:
        # per-kernel durations, measured with HIP events on the launch stream during one more generation
        gen.profile(True)
        gen.profile_read()
        pre = {}
        generate(after_prefill=lambda: pre.update(gen.profile_read()))   # the prefill's launches are read (and reset) apart
        prof = gen.profile_read()
        gen.profile(False)
        att = prof["decode_attention"]
        att_bytes = sum(attention_bytes(shape, B, t, bs) for t in range(P, P + G - 1)) * shape.n_layers
        if att["launches"] > 0 and att["ms"] > 0:
            achieved = att_bytes / (att["ms"] * 1e-3) / 1e9
            rec = RECORDED_TRAFFIC.get(args.workload) if not args.layers and not args.precision else None
            out["roofline"] = {"kernel": "decode_attention", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                               "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                               "traffic": rec["bytes"] if rec else None,
                               "traffic_source": (rec["source"] + " (rocprofv3 counters of a separate run of this command; not "
                                                  "measured by this run)") if rec and rec["bytes"] else None,
                               "launches": att["launches"], "avg_launch_us": att["ms"] * 1e3 / att["launches"],
                               "bytes_per_launch_mean": att_bytes / att["launches"]}
        # every kernel class of the decode step against its own roofline: algorithmic bytes per launch / event-timed duration
        # (HIP events around every launch on the launch stream; graph replay is off in this pass, which adds 2-4 us per launch)
        models = decode_kernel_models(shape, B, P, G, bs, level)
        ra = []
        for k, mdl in models.items():
            v = prof.get(k)
            if not v or not v["launches"] or v["ms"] <= 0:
                continue
            us = v["ms"] * 1e3 / v["launches"]
            e = {"class": k, "bound": "hbm", "launches": v["launches"], "avg_launch_us": us, "bytes_per_launch": mdl["bytes"],
                 "achieved": mdl["bytes"] / us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": mdl["bytes"] / us / 1e3 / HBM_PEAK_GBS,
                 "share_of_decode_kernel_time": None}
            if mdl["flops"]:
                e["executed_tflops"] = mdl["flops"] / us / 1e6
            ra.append(e)
        tot = sum(e["avg_launch_us"] * e["launches"] for e in ra)
        for e in ra:
            e["share_of_decode_kernel_time"] = e["avg_launch_us"] * e["launches"] / tot
        out["roofline_all"] = sorted(ra, key=lambda e: -e["share_of_decode_kernel_time"])
        out["kernels"] = {"prefill": {k: {"launches": v["launches"], "ms": round(v["ms"], 3)} for k, v in pre.items() if v["launches"]},
                          "decode": {k: {"launches": v["launches"], "ms": round(v["ms"], 3)} for k, v in prof.items() if v["launches"]}}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, wl, W)

    out["checksum_last_tokens"] = int(last_tokens.to(torch.int64).sum().item())
    gen.close()
    print(json.dumps(out))


def bench_portions(args, gen, wl, shape, prompts, setup_s):
    """The same generation through the single call rl_gen_generate, the batch cut into --mbs sequential portions (the
    KV cache holds one portion): what the smaller cache costs in throughput, since every portion streams all weights
    again at every decode step."""
    import torch
    B, P, G = wl.batch, wl.prompt_len, wl.gen_len
    out_tokens = torch.empty((B, G), dtype=torch.int32, device=prompts.device)

    def generate():
        gen.pack_weights()
        gen.generate(prompts, G, out=out_tokens)

    for _ in range(args.warmup):
        generate()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        generate()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    return {"metric": f"generated tokens/sec on 1 GPU, {wl.name}, batch in {args.mbs} sequential portions",
            "value": B * G * args.steps / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": elapsed * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": DTYPE, "data": "synthetic",
            "config": {"workload": f"{wl.name}: L{shape.n_layers} d{shape.hidden} H{shape.n_heads}/{shape.n_kv_heads} F{shape.ffn} "
                                   f"V{shape.vocab}, batch {B} as {args.mbs} portions of {B // args.mbs}, prompt {P}, generate {G}",
                       "global_batch": B, "prompt_len": P, "gen_len": G, "mbs": args.mbs, "hip_graph": not args.no_graph},
            "kv_cache_bytes": gen.kv_arena.numel(), "setup_s": setup_s,
            "checksum_last_tokens": int(out_tokens[:, G - 1].to(torch.int64).sum().item())}


def bench_logprobs(args, gen, wl, shape, dev, setup_s):
    """The inference call (log-probability of every following token) over B sequences of P+G tokens: a step is one
    call; value = scored tokens per second.  Bound by the matrix cores: the roofline entry is the tiled projection
    kernel, flops of the calls it served / their summed event-timed duration."""
    import torch
    from workload import Workload, make_prompts
    B, T = wl.batch, wl.prompt_len + wl.gen_len
    toks = make_prompts(Workload(wl.name, wl.index, shape, B, T, 0), device=dev)
    logp = torch.empty((B, T), dtype=torch.float32, device=dev)
    for _ in range(args.warmup):
        gen.logprobs(toks, logp)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        gen.logprobs(toks, logp)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    d, hd, Hq, Hkv, F, V, L = shape.hidden, shape.head_dim, shape.n_heads, shape.n_kv_heads, shape.ffn, shape.vocab, shape.n_layers
    proj_flops = 2 * B * T * (L * ((Hq + 2 * Hkv) * hd * d + Hq * hd * d + 3 * d * F) + V * d)
    flops = proj_flops + 4 * L * B * Hq * hd * T * (T + 1) // 2
    out = {"metric": f"inference call (token log-probabilities), scored tokens/sec on 1 GPU, {wl.name}", "value": B * T * args.steps / elapsed,
           "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed * 1e3 / args.steps,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": DTYPE, "data": "synthetic",
           "config": {"workload": f"{wl.name}: L{L} d{d} H{Hq}/{Hkv} F{F} V{V}, batch {B}, sequence {T}", "global_batch": B, "seq_len": T},
           "phases": {"tflops": flops / (elapsed / args.steps) / 1e12, "frac_of_mfma_peak": flops / (elapsed / args.steps) / 1e12 / MFMA_PEAK_TFLOPS},
           "setup_s": setup_s, "checksum_logp": float(logp.double().sum().item())}
    if not args.no_roofline:
        gen.profile(True)
        gen.profile_read()
        gen.logprobs(toks, logp)
        prof = gen.profile_read()
        gen.profile(False)
        ms = sum(prof[k]["ms"] for k in ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm_head"))
        n = sum(prof[k]["launches"] for k in ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm_head"))
        # executed flops of the projections: the QKV projection runs on both terms of its activations
        executed = proj_flops + 2 * B * T * L * (Hq + 2 * Hkv) * hd * d
        if ms > 0:
            out["roofline"] = {"kernel": "gemm_tiled (all projections)", "bound": "mfma", "achieved": executed / (ms * 1e-3) / 1e12,
                               "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": executed / (ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                               "traffic": None, "launches": n, "avg_launch_us": ms * 1e3 / max(n, 1)}
        out["kernels"] = {k: {"launches": v["launches"], "ms": round(v["ms"], 3)} for k, v in prof.items() if v["launches"]}
    return out


def cpu_baseline(shape, wl, W):
    """The CPU oracle as it stands, timed on this machine's host cores on a bounded sample of the same model shape."""
    import numpy as np
    from oracle import orc
    from workload import make_prompts
    Bs, Ps, Gs = 4, 64, 4      # about 10-20 s of host work at the 7B shape
    Wn = orc.weights_to_numpy(W)            # device -> host copy of the same bf16 values
    om = orc.OracleModel(shape, Wn, Bs, Ps + Gs)
    prompts = make_prompts(wl, batch=Bs, prompt_len=Ps).numpy()
    t0 = time.perf_counter()
    _, nxt = om.prefill(prompts)
    for _ in range(Gs - 1):
        _, nxt = om.decode_step(nxt)
    dt = time.perf_counter() - t0
    om.close()
    return {"value": Bs * Gs / dt, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"same model and weights, batch {Bs}, prompt {Ps}, generate {Gs} tokens (fp64 CPU oracle, {dt:.1f} s)"}


if __name__ == "__main__":
    main()
