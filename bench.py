#!/usr/bin/env python3
"""Benchmark of the D2O hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input, with all inputs
resident in HBM before the timed region: for every layer the prefill attention with per-key
scores and density (a1-a2), the dynamic budget allocation from the measured densities (a3),
for every layer selection / compaction / matching / threshold / merge (a4-a8), then
`decode_steps` generation steps over the compressed caches of all layers (a9-a12).

Prints ONE JSON line.  `value` is the decode throughput in tokens/s (batch * decode steps /
decode time); the same line carries the prefill-compress time per layer, the roofline of the
dominant kernel (matrix-core prefill attention) and of the HBM-bound decode kernel, and the
CPU oracle timed on a bounded sample of the same workload."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2406_13035_amd import binding, synth  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16/fp16 matrix-core peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E peak
MIN_BUDGET = 64
DECODE_TIMING_STRIDE = 16


def generate(w, device):
    """All inputs of one benchmark step, resident on the device."""
    Q, K, V = [], [], []
    for l in range(w.n_layers):
        q, k, v = [], [], []
        for b in range(w.batch):
            ql, kl, vl = synth.layer_inputs(w, b, l, device)
            q.append(ql)
            k.append(kl)
            v.append(vl)
        Q.append(torch.stack(q))
        K.append(torch.stack(k))
        V.append(torch.stack(v))
    return Q, K, V


def generate_decode(w, steps, device):
    qs, ks, vs = [], [], []
    for l in range(w.n_layers):
        ql, kl, vl = [], [], []
        for b in range(w.batch):
            q, k, v = synth.layer_decode_inputs(w, b, l, steps, device)
            ql.append(q)
            kl.append(k)
            vl.append(v)
        qs.append(torch.stack(ql, 1))
        ks.append(torch.stack(kl, 1))
        vs.append(torch.stack(vl, 1))
    # [steps, L, B, H, d]
    return (torch.stack(qs, 1).contiguous(), torch.stack(ks, 1).contiguous(),
            torch.stack(vs, 1).contiguous())


def run_step(ctx, w, Q, K, V, O, dq, dk, dv, dout, decode_steps):
    """One pass of the hot path.  Returns (prefill_ms, decode_ms, budgets [B, L], F [B, L])."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ctx.d2o_reset()
    ev[0].record()
    for l in range(w.n_layers):
        ctx.d2o_prefill_attend(l, Q[l], K[l], V[l], O)
    F = ctx.d2o_get_density()
    n = w.prompt_len
    budgets = np.stack([binding.d2o_allocate_budgets(F[b], n, w.total_budget(), MIN_BUDGET)
                        for b in range(w.batch)])
    for l in range(w.n_layers):
        bud = budgets[:, l]
        ctx.d2o_compress_layer(l, K[l], V[l], bud, bud // 4)
    ev[1].record()
    for t in range(decode_steps):
        ctx.d2o_decode_step(0, w.n_layers, dq[t], dk[t], dv[t], dout)
    ev[2].record()
    torch.cuda.synchronize()
    return ev[0].elapsed_time(ev[1]), ev[1].elapsed_time(ev[2]), budgets, F


def cpu_baseline(w, heads_sample=3, decode_steps_sample=32):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload (about 10-15 s of
    CPU work at configuration 3): for the first KV heads of layer 0, the prompt attention and
    scores of one of their query heads, the token-level stages at the mean budget, and a few
    decode steps; the mean times are scaled to the whole workload."""
    from oracle import d2o_ref as ref
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    n = w.prompt_len
    budget = w.total_budget() // w.n_layers
    heads = list(range(min(heads_sample, w.n_kv_heads)))
    attn_s = comp_s = dec_s = 0.0
    for h in heads:
        Qh, Kh, Vh = synth.kv_head_inputs(w, 0, 0, h, "cpu")
        Qd, Kd, Vd = (binding.tensor_to_f64(t) for t in (Qh, Kh, Vh))
        t0 = time.perf_counter()
        o, s = ref.prefill_attention_head(Qd[0], Kd, Vd)
        var = ref.head_variance(s)
        t1 = time.perf_counter()
        score = s * w.group
        cache, _ = ref.compress_head(Kd, Vd, score, budget, budget // 4, 0, w.dtype)
        t2 = time.perf_counter()
        q, k, v = synth.kv_head_decode_inputs(w, 0, 0, h, decode_steps_sample, "cpu")
        qd, kd, vd = (binding.tensor_to_f64(t) for t in (q, k, v))
        t3 = time.perf_counter()
        for t in range(decode_steps_sample):
            ref.decode_step_head(cache, qd[t], kd[t], vd[t], n + t, budget, budget // 4, 0, w.beta)
        t4 = time.perf_counter()
        attn_s += (t1 - t0) / len(heads)
        comp_s += (t2 - t1) / len(heads)
        dec_s += (t4 - t3) / decode_steps_sample / len(heads)
    heads_q, heads_kv = w.n_q_heads * w.batch, w.n_kv_heads * w.batch
    prefill_ms_layer = (attn_s * heads_q + comp_s * heads_kv) * 1e3
    step_s = dec_s * heads_kv * w.n_layers
    return {
        "value": w.batch / step_s, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
        "prefill_compress_ms_per_layer": prefill_ms_layer,
        "sample": (f"layer 0, {len(heads)} KV heads: attention+scores of one query head each ({attn_s:.1f} s per "
                   f"head), token-level stages at budget {budget} ({comp_s:.1f} s per head), {decode_steps_sample} "
                   f"decode steps per head ({dec_s * 1e3:.1f} ms each); mean times scaled by "
                   f"{heads_q} query heads / {heads_kv} KV heads per layer and {w.n_layers} layers"),
    }


def measured_traffic(cfg: int, kernel: str):
    """HBM bytes per launch (fetch + write) of a kernel from the committed rocprofv3 counter
    summary of this configuration, or None when that summary has no complete entry."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_cfg{cfg}.txt")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) == 4 and parts[0] == "kernel" and parts[1] == kernel:
                return float(int(parts[2]) + int(parts[3]))
    except (OSError, ValueError):
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--cfg", type=int, default=3, help="benchmark configuration 1..5")
    ap.add_argument("--decode-steps", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=None,
                    help="run only this many layers (profiling aid; the metric needs all)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="profiling aid: also run three elementwise copies of 1 GiB (reads 1 GiB, "
                         "writes 1 GiB each), the known traffic that scales the HBM byte counters")
    ap.add_argument("--skip-per-layer-decode", action="store_true",
                    help="profiling aid: leave out the extra decode steps issued as one call per "
                         "layer, so that a kernel trace holds the all-layers launches only")
    ap.add_argument("--zero-data-probe", action="store_true",
                    help="profiling aid: after the measurement, time the two prompt-attention "
                         "kernels of layer 0 on the workload's data and on all-zero Q, K, V (same "
                         "instruction stream; the difference is what the chip's power management "
                         "takes for operands that toggle)")
    ap.add_argument("--no-extras", action="store_true",
                    help="profiling aid: leave out what runs outside the timed region (upstream projection, "
                         "block append, the fp8-cache pass), so that a kernel trace holds the timed path only")
    ap.add_argument("--cache-fp8", action="store_true",
                    help="run the workload with the fp8 cache encoding (E4M3 codes and one power of two "
                         "per row) instead of a cache in the tensors' dtype; the decode roofline then "
                         "counts 2 * d + 2 + 8 bytes per slot")
    ap.add_argument("--split-rows", type=int, default=0,
                    help="tuning aid: the context's split_rows (entries above which a head's closing "
                         "work in a generation step is split over workgroups); 0 = the library's default")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (one GPU's share "
              "of the work is what is measured); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("no GPU visible: the D2O library has no CPU path", file=sys.stderr)
        sys.exit(3)
    w = synth.WORKLOADS[args.cfg]
    if args.layers:
        w = w.scaled(n_layers=args.layers)
    dsteps = args.decode_steps or w.decode_steps
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    print(f"[bench] generating {w.name}: B={w.batch} L={w.n_layers} Hq={w.n_q_heads} "
          f"Hkv={w.n_kv_heads} d={w.head_dim} N={w.prompt_len}", file=sys.stderr, flush=True)
    Q, K, V = generate(w, dev)
    dq, dk, dv = generate_decode(w, dsteps, dev)
    slots = w.total_budget() + w.n_layers + 8
    ctx = binding.D2O(w.batch, w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.prompt_len,
                      slots, dtype=w.dtype, n_sink=0, beta=w.beta, split_rows=args.split_rows,
                      cache_fp8=args.cache_fp8)
    O = torch.empty_like(Q[0])
    dout = torch.empty_like(dq[0])
    torch.cuda.synchronize()
    print("[bench] inputs resident; warm-up", file=sys.stderr, flush=True)
    for _ in range(args.warmup):
        run_step(ctx, w, Q, K, V, O, dq, dk, dv, dout, dsteps)
    # kernel durations by HIP events inside the timed region: every launch of the prompt-phase
    # kernels, every 16th decode step (the events of a decode step cost it 3 %)
    ctx.d2o_timing_enable(DECODE_TIMING_STRIDE)
    for k in binding.KERNEL_IDS:
        ctx.d2o_timing_read(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pre, dec = [], []
    for i in range(args.steps):
        p, d, budgets, F = run_step(ctx, w, Q, K, V, O, dq, dk, dv, dout, dsteps)
        pre.append(p)
        dec.append(d)
        print(f"[bench] step {i}: prefill+compress {p:.1f} ms, decode {d:.1f} ms", file=sys.stderr,
              flush=True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kt = {k: ctx.d2o_timing_read(k) for k in binding.KERNEL_IDS}
    ctx.d2o_timing_enable(False)
    misses = ctx.d2o_candidate_misses()  # of the last pass (d2o_reset clears the counter)
    # the same decode steps issued as one call per layer (a caller that interleaves the layers
    # with its own work), continuing on the caches of the last step; outside the timed region
    per_layer_steps = 0 if (args.layers or args.skip_per_layer_decode) else min(32, dsteps)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for t in range(per_layer_steps):
        for l in range(w.n_layers):
            ctx.d2o_decode_step(l, 1, dq[t][l:l + 1], dk[t][l:l + 1], dv[t][l:l + 1], dout[l:l + 1])
    ev[1].record()
    torch.cuda.synchronize()
    per_layer_ms = ev[0].elapsed_time(ev[1]) / per_layer_steps if per_layer_steps else None

    n, d, L = w.prompt_len, w.head_dim, w.n_layers
    decode_ms = float(np.mean(dec))
    prefill_ms = float(np.mean(pre))
    tokens_per_s = w.batch * dsteps / (decode_ms * 1e-3)
    # dominant kernel: prefill attention pass 1.  Algorithmic work = causal QK^T + PV:
    # 2 * N^2 * d FLOP per (sequence, query head), per launch B * Hq heads.
    attn_ms, attn_n = kt["attn_fwd"]
    flop_per_launch = 2.0 * n * n * d * w.n_q_heads * w.batch
    attn_tflops = flop_per_launch / (attn_ms / attn_n * 1e-3) / 1e12 if attn_n else 0.0
    # decode attention: K and V rows read once (2 * d * esize bytes per slot) + fp64 logits
    # written, per KV head; slots = budget (+1) per layer.
    es = 2 if w.dtype == "bf16" else 4
    slots_b = budgets.sum(axis=1) + L
    row_bytes = 2 * d + 2 if args.cache_fp8 else 2 * d * es  # K and V row (fp8: codes and the two powers of two)
    bytes_per_launch = float(sum(int(s) for s in slots_b) * w.n_kv_heads * (row_bytes + 8))
    da_ms, da_n = kt["decode_attend"]
    da_avg = da_ms / da_n if da_n else None
    dec_gbs = bytes_per_launch / (da_avg * 1e-3) / 1e9 if da_n else 0.0
    step_bytes = bytes_per_launch  # whole decode step, algorithmic (K second touch not counted)
    # the whole prompt phase of a layer: the attention product above plus the evicted-by-retained
    # similarity product of Eq. 9 (2 * Le * Lr * d per (sequence, KV head), mean over the layers);
    # the column sums' second QK^T is overhead of this implementation, not algorithmic work
    match_flop_layer = float(sum(2.0 * (n - int(s)) * int(s) * d for s in budgets.reshape(-1)) * w.n_kv_heads / L)
    layer_flop = flop_per_launch + match_flop_layer
    cs_ms, cs_n = kt["colsum"]
    passes_ms = (attn_ms / attn_n + cs_ms / cs_n) if attn_n and cs_n else None
    out = {
        "metric": "compressed-KV decode tokens/s (+ prefill-compress ms/layer at N=32k)",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"config {w.cfg}: {w.name}", "batch": w.batch, "layers": L,
                   "q_heads": w.n_q_heads, "kv_heads": w.n_kv_heads, "head_dim": d, "prompt_len": n,
                   "decode_steps": dsteps, "total_budget": w.total_budget(),
                   "cache": "fp8 (E4M3 codes + one power of two per row)" if args.cache_fp8 else w.dtype,
                   "layer_budgets_seq0": [int(x) for x in budgets[0]],
                   "density_F_seq0_min_max": [float(F[0].min()), float(F[0].max())]},
        "prefill_compress_ms_per_layer": prefill_ms / L,
        "decode_ms_per_step": decode_ms / dsteps,
        "decode_ms_per_step_one_call_per_layer": per_layer_ms,
        "decode_step_hbm_frac": step_bytes / (decode_ms / dsteps * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "roofline": {"kernel": "attn_fwd (prefill attention pass 1)", "bound": "mfma",
                     "achieved": attn_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": attn_tflops / PEAK_BF16_TFLOPS,
                     "traffic": measured_traffic(w.cfg, "attn_fwd_bf16"),
                     "algorithmic_flop_per_launch": flop_per_launch,
                     "avg_launch_ms": attn_ms / attn_n if attn_n else None},
        "roofline_prefill_compress": {
            "what": "one layer's whole prompt phase (attention, column sums, selection, matching, merge)",
            "bound": "mfma", "algorithmic_flop_per_layer": layer_flop,
            "achieved": layer_flop / (prefill_ms / L * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": layer_flop / (prefill_ms / L * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "attention_and_column_sums_ms": passes_ms,
            "attention_and_column_sums_frac": (flop_per_launch / (passes_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS
                                               if passes_ms else None)},
        "roofline_decode": {"kernel": "decode_attend", "bound": "hbm", "achieved": dec_gbs,
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": dec_gbs / PEAK_HBM_GBS,
                            "traffic": measured_traffic(w.cfg, "decode_attend"),
                            "algorithmic_bytes_per_launch": bytes_per_launch,
                            "avg_launch_ms": da_avg},
        "kernel_ms_per_launch": {k: (v[0] / v[1] if v[1] else None) for k, v in kt.items()},
        # evictions of the last pass whose token was not among the candidates predicted a step ahead
        "decode_candidate_misses": {"misses": int(misses), "head_steps": int(L * w.batch * w.n_kv_heads * dsteps)},
    }
    # ---- outside the timed region: the upstream step (Sec. 3 Eq. 1 + rotary embedding) at the
    #      workload's shape with the hidden size of the model the shape comes from (heads * d)
    if w.dtype == "bf16" and w.head_dim == 128 and not args.layers and not args.no_extras:
        hidden = w.n_q_heads * w.head_dim
        gx = torch.Generator(device=dev)
        gx.manual_seed(synth.BASE_SEED + 17)
        X = torch.randn(w.batch, n, hidden, generator=gx, device=dev, dtype=torch.float32).to(torch.bfloat16)
        Wm = (torch.randn((w.n_q_heads + 2 * w.n_kv_heads) * d, hidden, generator=gx, device=dev,
                          dtype=torch.float32) / hidden ** 0.5).to(torch.bfloat16)
        binding.d2o_qkv_project(X, Wm, w.n_q_heads, w.n_kv_heads, d)
        evq = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        evq[0].record()
        for _ in range(5):
            binding.d2o_qkv_project(X, Wm, w.n_q_heads, w.n_kv_heads, d)
        evq[1].record()
        torch.cuda.synchronize()
        q_ms = evq[0].elapsed_time(evq[1]) / 5
        q_flop = 2.0 * w.batch * n * hidden * (w.n_q_heads + 2 * w.n_kv_heads) * d
        out["qkv_project"] = {"ms_per_layer": q_ms, "hidden": hidden, "tflops": q_flop / (q_ms * 1e-3) / 1e12,
                              "frac_of_bf16_peak": q_flop / (q_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        del X, Wm
    # ---- outside the timed region: a block of new tokens on one layer's compressed cache
    #      (d2o_append_chunk) in the shape of the multi-turn experiment of the appendix: budget
    #      2048 = 48 heavy hitters + 2000 recent, turns of 256 tokens, the workload's heads
    if w.dtype == "bf16" and not args.layers and not args.no_extras:
        m, a_budget, a_recent, a_n = 256, 2048, 2000, 4096
        actx = binding.D2O(w.batch, 1, w.n_q_heads, w.n_kv_heads, d, a_n, a_budget + m + 8, dtype=w.dtype,
                           beta=w.beta, max_append=m)
        ga = torch.Generator(device=dev)
        ga.manual_seed(synth.BASE_SEED + 23)
        mk = lambda *shape: torch.randn(*shape, generator=ga, device=dev, dtype=torch.float32).to(torch.bfloat16)
        Qa, Ka, Va = mk(w.batch, w.n_q_heads, a_n, d), mk(w.batch, w.n_kv_heads, a_n, d), mk(w.batch, w.n_kv_heads, a_n, d)
        actx.d2o_prefill_compress(0, Qa, Ka, Va, a_budget, a_recent)
        Qb, Kb, Vb = mk(w.batch, w.n_q_heads, m, d), mk(w.batch, w.n_kv_heads, m, d), mk(w.batch, w.n_kv_heads, m, d)
        Ob = torch.empty_like(Qb)
        actx.d2o_append_chunk(0, Qb, Kb, Vb, Ob)          # warm-up turn
        eva = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        eva[0].record()
        turns = 3
        for _ in range(turns):
            actx.d2o_append_chunk(0, Qb, Kb, Vb, Ob)
        eva[1].record()
        torch.cuda.synchronize()
        a_ms = eva[0].elapsed_time(eva[1]) / turns
        out["append_chunk"] = {"ms_per_layer_and_block": a_ms, "block_tokens": m, "budget": a_budget,
                               "recent": a_recent, "tokens_per_s_one_layer": w.batch * m / (a_ms * 1e-3)}
        actx.close()
        del Qa, Ka, Va, Qb, Kb, Vb, Ob
    # ---- outside the timed region: the same workload's decode steps on the fp8 cache encoding
    if w.dtype == "bf16" and not args.layers and not args.cache_fp8 and not args.no_extras:
        fctx = binding.D2O(w.batch, w.n_layers, w.n_q_heads, w.n_kv_heads, w.head_dim, w.prompt_len,
                           slots, dtype=w.dtype, n_sink=0, beta=w.beta, split_rows=args.split_rows, cache_fp8=True)
        run_step(fctx, w, Q, K, V, O, dq, dk, dv, dout, dsteps)
        _, fdec, _, _ = run_step(fctx, w, Q, K, V, O, dq, dk, dv, dout, dsteps)
        f_bytes = float(sum(int(s) for s in slots_b) * w.n_kv_heads * (2 * d + 2 + 8))
        out["fp8_cache"] = {"decode_ms_per_step": fdec / dsteps, "tokens_per_s": w.batch * dsteps / (fdec * 1e-3),
                            "algorithmic_bytes_per_step": f_bytes,
                            "decode_step_hbm_frac": f_bytes / (fdec / dsteps * 1e-3) / 1e9 / PEAK_HBM_GBS,
                            "candidate_misses": int(fctx.d2o_candidate_misses())}
        fctx.close()
    if args.zero_data_probe:
        probe = {}
        for tag, (q, k, v) in (("workload_data", (Q[0], K[0], V[0])),
                               ("zero_data", tuple(torch.zeros_like(t) for t in (Q[0], K[0], V[0])))):
            ctx.d2o_reset()
            ctx.d2o_timing_enable(False)
            ctx.d2o_prefill_attend(0, q, k, v, O)
            ctx.d2o_timing_enable(True)
            for kk in ("attn_fwd", "colsum"):
                ctx.d2o_timing_read(kk)
            for _ in range(5):
                ctx.d2o_prefill_attend(0, q, k, v, O)
            torch.cuda.synchronize()
            for kk in ("attn_fwd", "colsum"):
                ms, cnt = ctx.d2o_timing_read(kk)
                probe[f"{kk}_ms_{tag}"] = ms / cnt
            ctx.d2o_timing_enable(False)
        out["zero_data_probe"] = probe
    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        print("[bench] timing the CPU oracle on a bounded sample", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
