#!/usr/bin/env python3
"""Benchmark of the diffusion-forcing sampler hot path on one MI355X.

A "step" is one sampler iteration (Alg. 1): prelude on the in-flight tokens, r' recurrences of
the core block over the window, coda + LM head + Sample on every window row, freeze / append
bookkeeping -- all inside librdlm.so.  Default workload: the 3.5B-shaped model, 512-token prompt,
32 recurrences, window 32, batch 1, greedy (steady state freezes one token per step).

Prints ONE JSON line: tokens/s (inputs resident in HBM, prefill not timed), the roofline of the
dominant kernel (the weight-streaming GEMM of the gate/up projection, timed per launch with HIP
events inside the timed region) and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as S  # noqa: E402

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_weights(shape, seed, keep_f64: bool, threads: int):
    """Upload the seeded weights tensor by tensor; optionally keep float64 host copies (oracle)."""
    import torch
    import paper_2510_14961_amd as R
    dev, host = {}, {}
    pool = ThreadPoolExecutor(max_workers=4)
    futs = []
    t0 = time.time()
    for name, arr in S.iter_weights(shape, seed, threads=threads):
        dev.update(R.upload_weights(shape, [(name, arr)]))
        if keep_f64:
            futs.append((name, pool.submit(lambda a: a.astype(np.float64), arr)))
        del arr
    for name, f in futs:
        host[name] = f.result()
    pool.shutdown()
    torch.cuda.synchronize()
    log(f"[bench] weights generated and uploaded in {time.time() - t0:.1f}s")
    return dev, host


def cpu_baseline(shape, w64, prompt_len, window, budget_s=20.0):
    """Time the oracle (as it is) on steady-state sampler steps of the same shape: window rows
    behind a context of prompt_len positions.  Cache content is random (only timing is read)."""
    from oracle import rdlm_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    m = O.RecurrentDepthLM(shape, w64)
    max_steps = 24                       # about 15 s on the 16 host threads of a GPU machine
    cache = m.new_cache(prompt_len + window + max_steps + 2)
    rng = np.random.default_rng(0)
    for d in (cache.k, cache.v):
        for name in d:
            d[name][: prompt_len] = rng.standard_normal((prompt_len, shape.n_heads, shape.head_dim))
    y = np.concatenate([S.make_prompt(shape.vocab, prompt_len, 1), np.zeros(window + max_steps + 2, dtype=np.int32)])
    p0 = prompt_len - 1
    z = np.stack([O.init_state(shape.hidden, p0 + j, 0, 1.0, 1) for j in range(window)])
    times = []
    for t in range(1, max_steps + 1):
        t0 = time.time()
        pos = np.arange(p0, p0 + window)
        e = m.prelude(y[pos], pos, cache)
        z = m.core(e, z, pos, cache)
        logits = m.coda(z, pos, cache)
        for i, p in enumerate(pos):
            y[p + 1] = O.sample(logits[i], 0.0, int(p), 0, t, 1)
        # steady state: the oldest state leaves, a fresh one enters
        z = np.concatenate([z[1:], O.init_state(shape.hidden, p0 + window, 0, 1.0, 1)[None]])
        p0 += 1
        times.append(time.time() - t0)
        if sum(times) > budget_s:
            break
    per_step = float(np.mean(times))
    return {"value": 1.0 / per_step, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{len(times)} steady-state sampler steps (window {window}, context {prompt_len}+, float64 numpy; "
                      f"cache prefix filled with random values, prefill not run), {per_step:.2f} s/step, 1 token/step"}


def machine_reference(ctx, shape):
    """What the machine does beside the kernels: a plain streaming read of the gate/up weights in the
    dominant kernel's own launch shape (and a wider one), and the matrix instruction from registers."""
    names = __import__("paper_2510_14961_amd").weight_names(shape)
    gu = names.index("R0.wg")
    out = {}
    best = 0.0
    for wgs, waves in ((224, 4), (256, 4), (512, 4), (1024, 4)):
        ms, nbytes = ctx.time_stream_read(gu, wgs, waves, 40)
        gbs = nbytes / (ms * 1e-3) / 1e9
        out[f"stream_read_{wgs}x{waves}_GBps"] = gbs
        best = max(best, gbs)
    out["hbm_stream_GBps"] = best
    ms, fl = ctx.time_mfma_loop(1024, 20000, 1)            # a short burst: the clock has not dropped yet
    out["mfma_bf16_burst_TFLOPs"] = fl / (ms * 1e-3) / 1e12
    ms, fl = ctx.time_mfma_loop(1024, 20000, 40)           # about a third of a second: the sustained clock
    out["mfma_bf16_sustained_TFLOPs"] = fl / (ms * 1e-3) / 1e12
    out["note"] = ("plain nontemporal streaming read of one layer's packed gate/up weights (layers in turn), "
                   "workgroups x waves as named; v_mfma_f32_32x32x16_bf16 from registers, 1024 workgroups x 4 waves x "
                   "4 accumulators")
    return out


def gemm_probe(args):
    """Every projection alone (the kernel and launch shape the model path picks for that row count), going
    round the layers' weights; flops = 2 x rows x N x K, bytes = the weights once."""
    import torch
    import paper_2510_14961_amd as R
    shape = S.BIG
    rows_list = [int(x) for x in args.gemm_probe.split(",")]
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    dev, _ = build_weights(shape, 1, False, args.threads)
    ctx = R.Context(shape, dev, 1, max(rows_list) + 64, max(rows_list))
    del dev
    torch.cuda.empty_cache()
    names = R.weight_names(shape)
    h, F, V = shape.hidden, shape.mlp, shape.vocab
    projs = {"gate_up": ("R0.wg", 2 * F, h), "qkv": ("R0.wqkv", 3 * h, h), "out": ("R0.wo", h, h),
             "down": ("R0.wd", h, F), "adapter": ("wa", h, 2 * h), "lm_head": ("emb", V, h)}
    out = []
    for rows in rows_list:
        for pname, (wname, N, K) in projs.items():
            ms = ctx.time_linear(names.index(wname), rows, 8 if rows > 256 else 24)
            out.append({"projection": pname, "rows": rows, "us": ms * 1e3, "TFLOPs": 2.0 * rows * N * K / (ms * 1e-3) / 1e12,
                        "weight_GBps": N * K * 2 / (ms * 1e-3) / 1e9})
            log(f"[probe] {pname:8s} rows {rows:5d}: {ms * 1e3:8.1f} us")
    print(json.dumps({"gemm_probe": out}), flush=True)
    ctx.close()


def core_sweep(args):
    """Core step (adapter + core layers + closing norm, r' = 1) over window rows x cached context."""
    import torch
    import paper_2510_14961_amd as R
    shape = S.BIG
    rows_grid = [1, 4, 16, 32, 64, 128, 256, 512, 1024, 2048, 4095]
    ctx_grid = [0, 512, 4096]
    dev, _ = build_weights(shape, 1, False, args.threads)
    ctx = R.Context(shape, dev, 1, max(ctx_grid) + max(rows_grid) + 1, max(rows_grid))
    del dev
    torch.cuda.empty_cache()
    h, F = shape.hidden, shape.mlp
    core_params = shape.n_core * (4 * h * h + 3 * h * F) + 2 * h * h
    table = []
    for c in ctx_grid:
        for rows in rows_grid:
            iters = 20 if rows <= 256 else 5 if rows <= 1024 else 3
            ms = ctx.time_core_step(0, c, rows, iters)
            kv = shape.n_core * 2 * (c + rows) * h * 2
            table.append({"rows": rows, "context": c, "ms": ms,
                          "weight_GBps": core_params * 2 / (ms * 1e-3) / 1e9,
                          "kv_bytes": kv, "TFLOPs": 2.0 * core_params * rows / (ms * 1e-3) / 1e12})
            log(f"[sweep] rows {rows:5d} context {c:5d}: {ms:8.3f} ms")
    ref = machine_reference(ctx, shape)
    # ridge: the flat (weight-streaming) time of the narrow windows against the slope of the wide ones
    ridge = {}
    for c in ctx_grid:
        t = {r["rows"]: r["ms"] for r in table if r["context"] == c}
        flat = min(t[1], t[4], t[16], t[32])
        slope = (t[4095] - t[1024]) / (4095 - 1024)
        ridge[str(c)] = {"flat_ms": flat, "ms_per_row_wide": slope, "ridge_rows": flat / slope}
    print(json.dumps({"core_step_sweep": table, "ridge": ridge, "machine": ref,
                      "model_ridge_rows": MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9),
                      "shape": "3.5B: 5280 x 55 x 96, mlp 17920, 4 core layers + adapter, bf16"}), flush=True)
    ctx.close()


def batch_sweep(args):
    """Batches of sequences with short windows (App. "Larger batch sizes"): sampler steps of n sequences x
    window w (fixed exit, r' = 1, r = w) at the 3.5B shape behind 512-token prompts, with the rows of the
    sequences packed into shared row tiles and with one row tile per sequence."""
    import torch
    import paper_2510_14961_amd as R
    shape = S.BIG
    grid = [(1, 32), (2, 16), (4, 8), (8, 4), (16, 2), (8, 32)]
    dev, _ = build_weights(shape, 1, False, args.threads)
    out = []
    for n_seqs, w in grid:
        row = {"sequences": n_seqs, "window": w, "rows": n_seqs * w}
        for packed in (True, False):
            ctx = R.Context(shape, dev, n_seqs, 512 + 256, 512)
            ctx.set_tuning("no_pack", "0" if packed else "1")
            for q in range(n_seqs):
                ctx.set_tokens(q, S.make_prompt(shape.vocab, 512, 5, seq=q))
                ctx.prefill(q, 511, 1, 1.0, 1)         # (timing only: one recurrence fills the caches)
            ctx.sampler_begin(n_seqs, n_new=200, r_inner=1, r_total=w, seed=1)
            for _ in range(w + 4):
                ctx.sample_step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            K = 40
            for _ in range(K):
                ctx.sample_step()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) / K * 1e3
            key = "packed" if packed else "tile_per_sequence"
            row[key + "_ms_per_step"] = ms
            row[key + "_tokens_per_s"] = n_seqs / ms * 1e3
            log(f"[batch] {n_seqs:2d} x window {w:2d} {key}: {ms:.3f} ms/step")
            ctx.close()
        out.append(row)
    print(json.dumps({"batch_sweep": out, "shape": "3.5B: 5280 x 55 x 96, mlp 17920, P2/R4/C2, bf16, prompt 512, greedy"}),
          flush=True)


def window_sweep(args):
    """Tokens in flight against throughput (Sec. 4.2: wavefront size and headway; the paper finds its optimum
    at 64-128 tokens on A100 and calls it accelerator-specific).  3.5B shape, batch 1, prompt 512, r = 32, fixed
    exit, greedy.  (a) headway h = 1..16 at r' = 1: window 32 h, h tokens frozen per step; (b) inner recurrences
    r' = 1..32 at headway 1: window 32 / r', down to the autoregressive sampler at r' = r (end of Sec. 3.3)."""
    import torch
    import paper_2510_14961_amd as R
    shape = S.BIG
    r = 32
    dev, _ = build_weights(shape, 1, False, args.threads)
    lead_cap = 160                                          # untimed lead-in after the wave fill (see --settle-ms)
    ctx = R.Context(shape, dev, 1, 512 + 16 * (32 + lead_cap + 40 + 8) + 640, 512)
    del dev
    torch.cuda.empty_cache()
    prompt = S.make_prompt(shape.vocab, 512, 5, seq=0)
    out = []
    for r_inner, headway in [(1, 1), (1, 2), (1, 3), (1, 4), (1, 6), (1, 8), (1, 12), (1, 16),
                             (2, 1), (4, 1), (8, 1), (16, 1), (32, 1)]:
        fill = -(-r // r_inner)
        K = 40 if r_inner <= 4 else 12
        ctx.set_tokens(0, prompt)
        ctx.prefill(0, 511, 1, 1.0, 1)                 # (timing only: one recurrence fills the caches)
        ctx.sampler_begin(1, n_new=(fill + lead_cap + K + 8) * headway, r_inner=r_inner, r_total=r, headway=headway,
                          seed=1)
        for _ in range(fill + 4):
            ctx.sample_step()
        torch.cuda.synchronize()
        lead, t_lead = 0, time.perf_counter()
        while lead < lead_cap - 4 and (time.perf_counter() - t_lead) * 1e3 < args.settle_ms:
            for _ in range(4):
                ctx.sample_step()
            torch.cuda.synchronize()
            lead += 4
        n0 = ctx.read_tokens(0, 1)[1]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            ctx.sample_step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        tokens = ctx.read_tokens(0, 1)[1] - n0
        row = {"r_inner": r_inner, "headway": headway, "window": fill * headway, "ms_per_step": dt / K * 1e3,
               "tokens_per_step": tokens / K, "tokens_per_s": tokens / dt}
        out.append(row)
        log(f"[window] r' {r_inner:2d} headway {headway:2d} window {row['window']:4d}: {row['ms_per_step']:.3f} ms/step, "
            f"{row['tokens_per_s']:.0f} tokens/s")
    print(json.dumps({"window_sweep": out, "shape": "3.5B: 5280 x 55 x 96, mlp 17920, P2/R4/C2, bf16, prompt 512, "
                      "r 32, fixed exit, greedy, batch 1"}), flush=True)
    ctx.close()


def attention_paths(args):
    """Windows of several row tiles: the core step (four layers) with the grouped attention kernel and with the
    one-tile kernel launched per segment, each forced through the "att_group_keys" knob, over rows x context --
    the measurement behind the rule the host applies (row tiles of a sequence x visible keys)."""
    import torch
    import paper_2510_14961_amd as R
    shape = S.BIG
    dev, _ = build_weights(shape, 1, False, args.threads)
    ctx = R.Context(shape, dev, 1, 8192 + 600, 512)
    del dev
    torch.cuda.empty_cache()
    ctx.time_core_step(0, 512, 64, 5)
    out = []
    for rows in (64, 128, 256, 512):
        for c in (512, 1024, 2048, 4096, 8192):
            row = {"rows": rows, "context": c, "tiles_x_keys": (rows // 32) * (c + rows)}
            for key, lim in (("grouped_us", "0"), ("per_segment_us", "1000000000")):
                ctx.set_tuning("att_group_keys", lim)
                row[key] = ctx.time_core_step(0, c, rows, 10) * 1e3
            ctx.set_tuning("att_group_keys", "")
            row["default_us"] = ctx.time_core_step(0, c, rows, 10) * 1e3
            out.append(row)
            log(f"[attention] rows {rows:4d} context {c:5d}: grouped {row['grouped_us']:8.1f} us, per segment "
                f"{row['per_segment_us']:8.1f} us, default {row['default_us']:8.1f} us")
    print(json.dumps({"attention_paths": out, "shape": "3.5B: 5280 x 55 x 96, four core layers + adapter, bf16"}),
          flush=True)
    ctx.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=511)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="cfg3", choices=["cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--ar-tokens", type=int, default=8,
                    help="tokens of the autoregressive (r' = r) run timed for comparison; 0 = skip")
    ap.add_argument("--headway", type=int, default=0,
                    help="override the workload's headway (states appended per step, Sec. 4.2): the window "
                         "becomes r/r' x headway; 0 = the workload's own")
    ap.add_argument("--paper-default-steps", type=int, default=48,
                    help="sampler steps timed with the paper's default sampler settings (r'=4, wavefront limit 128, "
                         "eps 0.03, momentum 0.1, temperature 0.2, top-p 0.95); 0 = skip")
    ap.add_argument("--settle-ms", type=float, default=200.0,
                    help="untimed sampler steps (in chunks of 8) for this long after the wave fill and before "
                         "--warmup (at most 256 steps), so that the timed steps see the machine's steady state; 0 = none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--large-window-rows", type=int, default=4095,
                    help="rows of the large-window core step timed against the MFMA peak (0 = skip)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (known HBM traffic) to scale rocprofv3 --pmc counters")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="instead of the benchmark: sampler steps of batches of sequences with short windows, rows "
                         "packed into shared row tiles against one row tile per sequence")
    ap.add_argument("--window-sweep", action="store_true",
                    help="tokens/s against the number of tokens in flight: headway 1..16 and r' 1..32 (Sec. 4.2)")
    ap.add_argument("--attention-paths", action="store_true",
                    help="core step with the grouped and with the per-segment attention kernel over rows x context")
    ap.add_argument("--core-sweep", action="store_true",
                    help="instead of the benchmark: time one core step (r' = 1) at the 3.5B shape over a grid of window "
                         "rows x cached context, print the table and the measured ridge (rows at which the step "
                         "turns from weight-streaming bound to matrix-core bound) as JSON")
    ap.add_argument("--gemm-probe", default="",
                    help="instead of the benchmark: time every projection of the 3.5B shape alone at these row counts "
                         "(comma separated), print JSON; the command to run under rocprofv3 --pmc for per-kernel counters")
    ap.add_argument("--threads", type=int, default=int(os.environ.get("OMP_NUM_THREADS", "8")))
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2510_14961_amd as R
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.window_sweep:
        window_sweep(args)
        return
    if args.attention_paths:
        attention_paths(args)
        return
    if args.batch_sweep:
        batch_sweep(args)
        return
    if args.core_sweep:
        core_sweep(args)
        return
    if args.gemm_probe:
        gemm_probe(args)
        return
    wl = S.WORKLOADS[args.workload]
    shape, sp = wl.shape, wl.sampler
    if args.headway > 0:
        import dataclasses
        sp = dataclasses.replace(sp, headway=args.headway)
    K, W = args.steps, args.warmup
    wave = -(-sp.r // sp.r_inner) * sp.headway
    window = sp.w_max if (sp.adaptive and sp.w_max > 0) else wave
    n_seqs = wl.n_seqs
    # steps before the first freeze: ceil(r / r') under the fixed exit rule and, at worst (no state
    # converges before the cap), under the adaptive one
    fill_steps = -(-sp.r // sp.r_inner)
    K2_max = 64
    # untimed lead-in after the wave fill (see --settle-ms), at most this many steps
    settle_cap = 256 if args.settle_ms > 0 else 0
    n_new = max(sp.n_new, (fill_steps + settle_cap + K + W + K2_max + 1) * sp.headway)   # never finish inside the timed steps
    max_positions = wl.prompt_len + n_new + window + sp.headway + 8
    max_rows = max(wl.prompt_len, n_seqs * (-(-window // 32) * 32))
    want_cpu = not args.no_cpu_baseline and args.workload in ("cfg2", "cfg3")

    if args.copy_calibration:       # 2^30 bytes read + 2^30 bytes written per copy
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    dev, w64 = build_weights(shape, wl.weight_seed, want_cpu, args.threads)
    t0 = time.time()
    ctx = R.Context(shape, dev, n_seqs, max_positions, max_rows)
    want_large = args.large_window_rows > 0 and args.workload == "cfg3"
    if not want_large:
        del dev
    torch.cuda.empty_cache()
    log(f"[bench] context created in {time.time() - t0:.1f}s, {ctx.device_bytes() / 2**30:.1f} GiB on device")

    prompts = [S.make_prompt(shape.vocab, wl.prompt_len, wl.prompt_seed, seq=q) for q in range(n_seqs)]
    t0 = time.time()
    for q, prompt in enumerate(prompts):
        ctx.set_tokens(q, prompt)
        ctx.prefill(q, wl.prompt_len - 1, sp.r, sp.alpha, sp.seed)
    torch.cuda.synchronize()
    log(f"[bench] prefill of {n_seqs} x {wl.prompt_len - 1} positions x {sp.r} recurrences: {time.time() - t0:.2f}s")
    sampler_kw = dict(r_inner=sp.r_inner, r_total=sp.r, headway=sp.headway, alpha=sp.alpha, w_max=sp.w_max,
                      adaptive=sp.adaptive, eps=sp.eps, temperature=sp.temperature, seed=sp.seed,
                      pad_token=sp.pad_token)
    ctx.sampler_begin(n_seqs, n_new=n_new, **sampler_kw)
    frozen = lambda: sum(ctx.read_tokens(q, 1)[1] for q in range(n_seqs))
    # wave fill (untimed, not part of --warmup): a position stays in flight for ceil(r / r') steps, so
    # nothing is frozen before that many steps have run; after them every step freezes tokens
    for _ in range(fill_steps):
        ctx.sample_step()
    # lead-in (untimed, not part of --warmup either): the headline is the steady-state rate of a generation.
    # For 100-150 ms after a prefill every weight-streaming kernel runs about 5 % slower on this machine
    # (its memory side takes that long to come back up after the matrix-core-heavy phase); the rate of
    # that phase is measured on its first steps and reported beside the headline, not hidden.
    torch.cuda.synchronize()
    settle_steps, first_ms, t_settle, chunk_ms = 0, None, time.perf_counter(), []
    while settle_steps < settle_cap and (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        t1 = time.perf_counter()
        for _ in range(8):
            ctx.sample_step()
        torch.cuda.synchronize()
        chunk_ms.append((time.perf_counter() - t1) / 8 * 1e3)
        if first_ms is None:
            first_ms = chunk_ms[0]
        settle_steps += 8
    if chunk_ms:
        log("[bench] lead-in, ms/step by chunks of 8 steps: " + " ".join(f"{x:.3f}" for x in chunk_ms))
    for _ in range(W):
        ctx.sample_step()
    torch.cuda.synchronize()
    nf0 = frozen()
    # headline: K steps, nothing but the sampler's own launches on the stream
    t0 = time.perf_counter()
    for _ in range(K):
        ctx.sample_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    nf1 = frozen()
    tokens = nf1 - nf0
    ms_per_step = dt / K * 1e3
    if tokens <= 0:
        print(f"bench.py: no token was frozen in the {K} timed steps (fill {fill_steps}, warmup {W}): "
              "the metric cannot be computed", file=sys.stderr)
        sys.exit(3)
    # roofline leg (second, short pass, not part of the headline): every launch of the gate/up
    # projection bracketed by a HIP event pair on the library's stream
    n_gu, k_gu = 2 * shape.mlp, shape.hidden
    per_step_launches = shape.n_prelude + sp.r_inner * shape.n_core + shape.n_coda     # one per layer pass
    K2 = min(K, 64)
    ctx.profile_gemm_begin(n_gu, k_gu, K2 * per_step_launches)
    torch.cuda.synchronize()
    for _ in range(K2):
        ctx.sample_step()
    torch.cuda.synchronize()
    gemm_ms, gemm_launches = ctx.profile_gemm_read()
    nf2 = frozen()

    # dominant kernel: gate/up projection over the rows of a step (each sequence's window padded to 32)
    rows = n_seqs * (-(-window // 32) * 32)
    # weights once + the packed bf16 operand + the bf16 SwiGLU output (width F = n_gu / 2)
    algo_bytes = n_gu * k_gu * 2 + rows * k_gu * 2 + rows * (n_gu // 2) * 2
    achieved = algo_bytes / (gemm_ms * 1e-3) / 1e9 if gemm_ms > 0 else 0.0
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(f"gemm_gu_{args.workload}")
        except Exception:
            traffic = None
    core_ms = ctx.time_core_step(0, wl.prompt_len, min(window, max_rows), 20)
    machine = machine_reference(ctx, shape) if shape.dtype == "bf16" and shape.hidden >= 2048 else None
    h, F, V = shape.hidden, shape.mlp, shape.vocab
    layer_b = (4 * h * h + 3 * h * F) * 2
    core_bytes = shape.n_core * layer_b + 2 * h * h * 2
    step_bytes = shape.n_layers * layer_b + 2 * h * h * 2 + V * h * 2

    # the same path run as the autoregressive sampler (r' = r: one token at a time, end of Sec. 3.3)
    ar = None
    if args.ar_tokens > 0 and not sp.adaptive:
        ctx.set_tokens(0, prompts[0])          # caches of the prompt prefix are still in place
        ar_kw = dict(sampler_kw, r_inner=sp.r, headway=1, w_max=0)
        ar_lead = 16 if args.settle_ms > 0 else 0          # same untimed lead-in as the headline leg
        ctx.sampler_begin(1, n_new=args.ar_tokens + 2 + ar_lead, **ar_kw)
        ctx.sample_step()
        ctx.sample_step()
        torch.cuda.synchronize()
        t_settle = time.perf_counter()
        while ar_lead > 0 and (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
            ctx.sample_step()
            torch.cuda.synchronize()
            ar_lead -= 1
        t0 = time.perf_counter()
        for _ in range(args.ar_tokens):
            ctx.sample_step()
        torch.cuda.synchronize()
        ar_dt = time.perf_counter() - t0
        ar = {"value": args.ar_tokens / ar_dt, "unit": "tokens/s", "tokens_timed": args.ar_tokens,
              "speedup_of_diffusion_forcing": (tokens / dt) / (args.ar_tokens / ar_dt),
              "note": "autoregressive sampling (r' = r) through the same library; the paper reports 4.4-4.8x "
                      "for r'=4 on A100-40GB"}

    # and as the token-per-token adaptive-compute sampler (Alg. 2 with a wavefront of one, Sec. 3.5);
    # with random weights the exit pattern is not a trained model's: the cap and the mean are reported
    ada = None
    if args.ar_tokens > 0 and not sp.adaptive:
        ctx.set_tokens(0, prompts[0])
        ada_kw = dict(sampler_kw, r_inner=4, headway=1, w_max=1, adaptive=True, eps=0.03)
        ctx.sampler_begin(1, n_new=4 * args.ar_tokens, **ada_kw)
        ctx.generate(4)                                     # the first steps, untimed
        torch.cuda.synchronize()
        f0 = ctx.read_tokens(0, 1)[1]
        t0 = time.perf_counter()
        steps = ctx.generate(10 * sp.r)
        torch.cuda.synchronize()
        ada_dt = time.perf_counter() - t0
        f1 = ctx.read_tokens(0, 1)[1]
        if f1 > f0:
            cnt = ctx.read_counts(0, wl.prompt_len - 1, f1 - wl.prompt_len) * 4
            ada = {"value": (f1 - f0) / ada_dt, "unit": "tokens/s", "tokens_timed": int(f1 - f0),
                   "mean_recurrences_per_token": float(np.mean(cnt)), "r_inner": 4, "eps": 0.03, "cap": sp.r,
                   "note": "Alg. 2 with wavefront 1 (adaptive-compute autoregression) through the same library"}

    # the paper's default sampler settings (Sec. 5 "Hyperparameters" and App. "Dataset details"):
    # Alg. 2, r' = 4, wavefront limit 128, eps = 0.03, momentum 0.1, temperature 0.2 with top-p 0.95.
    # Random weights: the exit pattern is this model's, not a trained one's -- the mean is reported.
    pd = None
    if args.paper_default_steps > 0 and not sp.adaptive and max_rows >= 128:
        n_pd = args.paper_default_steps
        ctx.set_tokens(0, prompts[0])
        pd_new = min(n_pd + 16, max_positions - wl.prompt_len - 128 - 2)
        pd_kw = dict(sampler_kw, r_inner=4, headway=1, w_max=128, adaptive=True, eps=0.03, eta=0.1,
                     temperature=0.2, top_p=0.95)
        ctx.sampler_begin(1, n_new=pd_new, **pd_kw)
        ctx.generate(12)                                    # fill the wave, untimed
        torch.cuda.synchronize()
        f0 = ctx.read_tokens(0, 1)[1]
        t0 = time.perf_counter()
        steps = ctx.generate(n_pd)
        torch.cuda.synchronize()
        pd_dt = time.perf_counter() - t0
        f1 = ctx.read_tokens(0, 1)[1]
        if f1 > f0 and steps > 0:
            cnt = ctx.read_counts(0, wl.prompt_len - 1, f1 - wl.prompt_len) * 4
            pd = {"value": (f1 - f0) / pd_dt, "unit": "tokens/s", "tokens_timed": int(f1 - f0), "steps_timed": int(steps),
                  "ms_per_step": pd_dt / steps * 1e3, "mean_recurrences_per_token": float(np.mean(cnt)),
                  "settings": "Alg. 2, r'=4, wavefront limit 128, eps 0.03, eta 0.1, temperature 0.2, top-p 0.95, "
                              f"cap r={sp.r}"}

    out = {
        "metric": "generated tokens/sec @batch1 (3.5B-shaped)" if args.workload == "cfg3" else f"generated tokens/sec ({args.workload})",
        "value": tokens / dt, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {h}x{shape.n_heads}x{shape.head_dim}, mlp {F}, vocab {V}, "
                               f"P{shape.n_prelude}/R{shape.n_core}/C{shape.n_coda}, prompt {wl.prompt_len}, "
                               f"r={sp.r}, r'={sp.r_inner}, window {window}, batch {n_seqs}, "
                               + ("greedy" if sp.temperature == 0 else f"temperature {sp.temperature}")
                               + (f", adaptive exit eps={sp.eps}" if sp.adaptive else "")
                               + (f", headway {sp.headway}" if sp.headway > 1 else ""),
                   "tokens_in_timed_region": int(tokens), "fill_steps": int(fill_steps),
                   "lead_in_steps": int(settle_steps), "ms_per_step_right_after_prefill": first_ms,
                   "context_at_end": int(nf2)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "achievable": machine["hbm_stream_GBps"] if machine else None,
                     "frac_of_achievable": achieved / machine["hbm_stream_GBps"] if machine else None,
                     "traffic_source": "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier "
                                       "run of this command, scaled by a 1 GiB copy; not measured by this run)"
                                       if traffic is not None else None,
                     "timing": f"HIP event pair around each launch, second pass of {K2} steps after the headline steps",
                     "kernel": f"gemm_bf16_k (gate/up projection with fused SwiGLU, [2F x h] weights, {rows} rows)",
                     "bytes_per_launch": algo_bytes, "avg_ms_per_launch": gemm_ms, "launches_timed": gemm_launches},
        "whole_step": {"weight_bytes": step_bytes, "GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
                       "frac_of_hbm_peak": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "core_step": {"ms": core_ms, "weight_bytes": core_bytes, "GBps": core_bytes / (core_ms * 1e-3) / 1e9},
        "machine_reference": machine,
        "autoregressive_same_path": ar,
        "adaptive_autoregressive_same_path": ada,
        "paper_default_settings": pd,
    }
    ctx.close()
    torch.cuda.empty_cache()
    if want_large:
        # the same core step over a prefill-sized window: every GEMM runs many row tiles per weight
        # tile, the regime bounded by the matrix cores (algorithmic flops: the GEMMs only)
        rows = args.large_window_rows
        ctx2 = R.Context(shape, dev, 1, rows + 64, rows)
        del dev
        ms = ctx2.time_core_step(0, 0, rows, 3)
        core_params = shape.n_core * (4 * h * h + 3 * h * F) + 2 * h * h
        flops = 2.0 * core_params * rows
        out["core_step_large_window"] = {"rows": rows, "ms": ms, "TFLOPs": flops / (ms * 1e-3) / 1e12,
                                         "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
                                         "frac_of_mfma_peak": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                         "flops_counted": "2 x core weights x rows (attention not counted)"}
        ctx2.close()
        torch.cuda.empty_cache()
    if want_cpu:
        t0 = time.time()
        out["cpu_baseline"] = cpu_baseline(shape, w64, wl.prompt_len, window)
        log(f"[bench] cpu baseline took {time.time() - t0:.1f}s")
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
