"""Benchmark of the mixed-batch serving step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg1|cfg2|grid|...] [--no-cpu-baseline]

A step is one pass of the whole layer stack (per layer: RMSNorm, QKV, rotary + KV append, paged attention,
O-projection, SwiGLU feed-forward) over one batch of synthetic input that is already resident
in HBM.  The default workload is the largest configuration that fits one GPU: the 70B-shaped stack of 80
layers on a mixed batch (1024-token prefill chunk at prefix 4096 + 256 decodes).  The two single-layer
8B-shaped configurations (64 decodes; 512-token chunk + 128 decodes) ride along as secondary records in the
same line.  Step time = median of per-step HIP event pairs on the step's stream.  Prints ONE JSON line.

--workload grid times the latency-profile grid instead (prefill chunk sizes x decode counts, five
draws of the lengths per cell, median step time): the (batch size, KV cache size) -> iteration
time table that the paper's router consumes (Sec. 4.5).  It prints one JSON object with the cells.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0
NOMINAL_CLOCK_MHZ = 2400.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-secondary", action="store_true", help="cfg4: leave out the secondary cfg1 / cfg2 records")
    ap.add_argument("--workload", default="cfg4", choices=["cfg1", "cfg2", "grid", "cfg4", "model8b", "prefill", "profile", "sim"])
    ap.add_argument("--requests", type=int, default=20000, help="sim: requests per simulated run")
    ap.add_argument("--table", default=None, help="sim: JSON written by an earlier --workload sim run; its table is used instead of measuring")
    ap.add_argument("--layers", type=int, default=80, help="cfg4: number of decoder layers")
    ap.add_argument("--kv-slots", type=int, default=8, help="cfg4: physical KV layer slots (layer l uses slot l mod this)")
    ap.add_argument("--check-layers", default="", help="cfg4: comma-separated layers to check against the oracle, teacher-forced")
    ap.add_argument("--vocab", type=int, default=128256, help="model8b: vocabulary size")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="library tuning knob passed to ps_set_option (repeatable); the defaults are what is reported")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--null-stream", action="store_true", help="run on the default stream instead of a dedicated one")
    ap.add_argument("--device-info", action="store_true", help="only print what the runtime reports about the device")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy a few times (reference for HBM byte counters)")
    return ap.parse_args()


def mfma_clock(ctx, tflops):
    """Sec. 2.2's compute-bound side priced twice: against the nominal matrix peak and against what the matrix pipes sustain at
    the clock the device holds under dense MFMA load (read after the timed region with ps_clock_under_load)."""
    r = ctx.clock_under_load(400000, 2)
    peak_at_clock = MFMA_BF16_PEAK_TFLOPS * r["shader_mhz"] / NOMINAL_CLOCK_MHZ
    return {"shader_mhz_under_mfma_load": round(r["shader_mhz"], 1), "mfma_only_loop_tflops": round(r["mfma_tflops"], 1),
            "ticks_per_mfma": round(r["ticks_per_mfma"], 2), "nominal_clock_mhz": NOMINAL_CLOCK_MHZ,
            "mfma_peak_at_that_clock_tflops": round(peak_at_clock, 1), "frac_mfma_at_that_clock": tflops / peak_at_clock}


def cpu_baseline(batch, weights, n_runs=2):
    """The oracle as it stands, timed on the host cores on the same workload (whole step)."""
    import numpy as np
    from oracle import run as orun
    from paper_2507_17769_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    model = W.MODELS[batch.model]
    pool = orun.make_pool(model, batch.n_pool_pages)
    for i, s in enumerate(batch.seqs):
        if s.prefix > 0:
            k, v = batch.prefix_kv(i)
            pool.write_bits(0, [int(p) for p in s.pages], 0, k, v)
    x = batch.activations()
    times = []
    for _ in range(n_runs):
        t0 = time.perf_counter()
        orun.run_step(model, [weights], batch.seqs, x, pool)
        times.append(time.perf_counter() - t0)
    t = sorted(times)[len(times) // 2] if len(times) % 2 else min(times)
    return {"value": batch.n_tokens / t, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"the whole {batch.name} step (all {batch.n_tokens} tokens, {batch.total_kv} KV tokens), "
                      f"best of {n_runs} runs, {t * 1e3:.0f} ms per step, numpy fp32",
            "ms_per_step": t * 1e3}


def measured_traffic(workload, seed):
    """HBM bytes per launch of the workload's dominant kernel from the committed rocprofv3 counter runs
    (FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a plain copy).  None when
    there is no record for this workload or the kernel source has changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "paper_2507_17769_amd", "measured_traffic.json")
    try:
        for rec in json.load(open(path))["records"]:
            if rec.get("workload") != f"{workload} seed {seed}":
                continue
            for rel, sha in rec["source_sha256"].items():
                if hashlib.sha256(open(os.path.join(ROOT, rel), "rb").read()).hexdigest() != sha:
                    return None
            return float(rec["fetch_bytes"]) + float(rec["write_bytes"])
    except Exception:
        pass
    return None


def run_grid(a):
    import numpy as np
    import torch
    from paper_2507_17769_amd import workloads as W
    from paper_2507_17769_amd.binding import STAGE_NAMES
    from paper_2507_17769_amd.runner import Engine, bits_to_dev

    model = "8b"
    m = W.MODELS[model]
    cells, worst_pages, worst_tokens = [], 0, 0
    for chunk in W.GRID_CHUNKS:
        for n_dec in W.GRID_DECODES:
            draws = [W.grid_cell_lengths(chunk, n_dec, s) for s in W.GRID_SEEDS]
            prefixes = [d[0] for d in draws]
            dkv = np.array([d[1] for d in draws], dtype=np.int32).reshape(len(draws), n_dec)
            cells.append((chunk, n_dec, prefixes, dkv))
            for off, kv in draws:
                pages = sum((int(L) + 15) // 16 for L in kv) + ((off + chunk + 15) // 16 if chunk else 0)
                worst_pages = max(worst_pages, pages)
            worst_tokens = max(worst_tokens, chunk + n_dec)
    n_pool = worst_pages + worst_pages // 8 + 64
    eng = Engine(model, n_pool, max_position=8192 + 4096 + 2048 + 16)
    for kv in a.option:
        eng.ctx.set_option(kv.split("=")[0], int(kv.split("=")[1]))
    eng.load_layer(0, W.layer_weights(model, a.seed, 0))
    # fill every page with N(0,1) keys and values (timing must not run on an all-zero cache)
    rng = np.random.Generator(np.random.PCG64([a.seed, 2718281]))
    blk = 8192
    k = bits_to_dev(W.normal_bf16(rng, (blk, m["n_kv"], m["head_dim"])), eng.device)
    v = bits_to_dev(W.normal_bf16(rng, (blk, m["n_kv"], m["head_dim"])), eng.device)
    rid = 0
    while eng.ctx.kv_free_pages() > 0:
        n_tok = min(blk, eng.ctx.kv_free_pages() * 16)
        pages = eng.ctx.kv_reserve(10_000 + rid, n_tok)
        eng.ctx.kv_write(0, pages, 0, n_tok, k.data_ptr(), v.data_ptr())
        rid += 1
    eng.ctx.sync()
    for r in range(rid):
        eng.ctx.kv_release(10_000 + r)
    x = bits_to_dev(W.normal_bf16(rng, (max(worst_tokens, 1), m["hidden"])), eng.device)
    y = torch.empty_like(x)
    t0 = time.perf_counter()
    res = eng.ctx.profile_grid(cells, x.data_ptr(), y.data_ptr(), warmup=a.warmup if a.warmup < 20 else 3, iters=min(a.steps, 10))
    wall = time.perf_counter() - t0
    out = []
    for c in res:
        out.append({"chunk": c.chunk, "n_decode": c.n_decode, "n_tokens": c.n_tokens, "total_kv": int(c.total_kv),
                    "median_ms": round(float(c.median_ms), 4),
                    "draw_ms": [round(float(c.draw_ms[i]), 4) for i in range(c.n_draws)],
                    "draw_total_kv": [int(c.draw_total_kv[i]) for i in range(c.n_draws)],
                    "stage_ms": {n: round(float(c.stage_ms[i]), 4) for i, n in enumerate(STAGE_NAMES)}})
    eng.close()
    print(json.dumps({"metric": "latency_profile_grid", "unit": "ms", "model": "8B-shaped layer", "seeds": list(W.GRID_SEEDS),
                      "pool_pages": n_pool, "wall_s": round(wall, 2), "cells": out}))


def percentiles(ms):
    import numpy as np
    return {"p10": round(float(np.percentile(ms, 10)), 4), "p50": round(float(np.percentile(ms, 50)), 4),
            "p90": round(float(np.percentile(ms, 90)), 4), "mean": round(float(np.mean(ms)), 4)}


def timed_steps(eng, call, steps, warmup):
    """W untimed steps, then K steps with an event at every step boundary on the stream the library launches on (torch's
    current stream, handed to ps_create), the whole region bracketed by synchronisations.  call(i) enqueues step i.
    Returns per-step GPU times (ms; consecutive pairs tile the stream's timeline, so an idle GPU waiting for the host
    counts against the step), per-call host times (us) and the wall time of the region."""
    import torch
    for i in range(warmup):
        call(i)
    eng.ctx.sync()
    torch.cuda.synchronize()
    # one event per step boundary: the end of step i is the start of step i + 1 (a record costs the stream a few
    # microseconds, which is part of what is measured)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    host_us = []
    t0 = time.perf_counter()
    evs[0].record(eng.stream)
    for i in range(steps):
        h0 = time.perf_counter()
        call(warmup + i)
        host_us.append((time.perf_counter() - h0) * 1e6)
        evs[i + 1].record(eng.stream)
    eng.ctx.sync()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)], host_us, wall_ms


def cpu_baseline_cfg4(batch, seed, n_layers):
    """The oracle on ONE layer of the 70B-shaped stack at the full batch, times the number of layers (extrapolated:
    the whole fp32 stack is 175 TFLOP and 137 GB of weights)."""
    import numpy as np
    from oracle import run as orun
    from paper_2507_17769_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    m = W.MODELS[batch.model]
    w = W.layer_weights(batch.model, seed, 0)
    pool = orun.make_pool(m, batch.n_pool_pages)
    rng = np.random.Generator(np.random.PCG64([seed, 31415926]))
    mp = max(s.prefix for s in batch.seqs)
    k = W.normal_bf16(rng, (mp, m["n_kv"], m["head_dim"]))
    v = W.normal_bf16(rng, (mp, m["n_kv"], m["head_dim"]))
    for s in batch.seqs:
        if s.prefix > 0:
            pool.write_bits(0, [int(p) for p in s.pages], 0, k[:s.prefix], v[:s.prefix])
    x = batch.activations()
    t0 = time.perf_counter()
    orun.run_step(m, [w], batch.seqs, x, pool)
    t = time.perf_counter() - t0
    return {"value": batch.n_tokens / (t * n_layers), "unit": "tokens/s", "cores": int(threads), "kind": "oracle", "extrapolated": True,
            "sample": f"one layer of the {n_layers} at the full batch ({batch.n_tokens} tokens, {batch.total_kv} KV tokens), one run, "
                      f"{t:.1f} s, numpy fp32; the step is taken as {n_layers} x that",
            "ms_per_step": t * 1e3 * n_layers}


def run_cfg4(a):
    """70B-shaped stack on one GPU: 80 layers (137 GB of bf16 weights, generated on the device),
    1024-token chunk at prefix 4096 + 256 decodes, KV slots aliased across layers.  Returns the result record."""
    import numpy as np
    import torch
    from paper_2507_17769_amd import workloads as W
    from paper_2507_17769_amd.binding import STAGE_NAMES, SeqArray
    from paper_2507_17769_amd.runner import Engine, bits_to_dev

    def log(msg):
        print(msg, file=sys.stderr, flush=True)

    model, L, slots = "70b", a.layers, min(a.kv_slots, a.layers)
    m = W.MODELS[model]
    H, F, nq, nkv, d = m["hidden"], m["ffn"], m["n_q"], m["n_kv"], m["head_dim"]
    check = sorted({int(v) for v in a.check_layers.split(",") if v.strip() != ""})
    batch = W.config_batch(4, a.seed)
    T, total_kv = batch.n_tokens, batch.total_kv
    eng = Engine(model, batch.n_pool_pages, L, slots, max_position=max(s.kv_len for s in batch.seqs) + 16)
    for kv in a.option:
        eng.ctx.set_option(kv.split("=")[0], int(kv.split("=")[1]))
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(1000 + a.seed)
    shapes = {"w_qkv": (H, (nq + 2 * nkv) * d), "w_o": (nq * d, H), "w_gate": (H, F), "w_up": (H, F), "w_down": (F, H)}
    ones = torch.ones(H, dtype=torch.bfloat16, device="cuda:0")
    cpu_weights = {}
    t0 = time.perf_counter()
    for l in range(L):
        if l in check:          # these layers' weights must also exist on the host for the oracle
            cpu_weights[l] = W.layer_weights(model, a.seed, l)
            eng.load_layer(l, cpu_weights[l])
        else:
            dev = {k: (torch.randn(s, generator=gen, device="cuda:0", dtype=torch.float32) * W.WEIGHT_STD).to(torch.bfloat16)
                   for k, s in shapes.items()}
            dev["g_attn"], dev["g_ffn"] = ones, ones
            eng.ctx.init_layer(l, **{k: t.data_ptr() for k, t in dev.items()})
            eng.ctx.sync()
            del dev
        if l % 8 == 7 or l == L - 1:
            log(f"cfg4: {l + 1}/{L} layers loaded ({time.perf_counter() - t0:.0f} s)")
    # cached prefixes: one block of N(0,1) keys/values reused for every sequence, written to every slot
    rng = np.random.Generator(np.random.PCG64([a.seed, 31415926]))
    max_prefix = max(s.prefix for s in batch.seqs)
    kblk = bits_to_dev(W.normal_bf16(rng, (max_prefix, nkv, d)), eng.device)
    vblk = bits_to_dev(W.normal_bf16(rng, (max_prefix, nkv, d)), eng.device)
    for slot in range(slots):
        for s in batch.seqs:
            if s.prefix > 0:
                eng.ctx.kv_write(slot, s.pages, 0, s.prefix, kblk.data_ptr(), vblk.data_ptr())
        eng.ctx.sync()
    log(f"cfg4: KV prefixes written to {slots} slots")
    x_bits = batch.activations()
    x = bits_to_dev(x_bits, eng.device)
    out = torch.empty_like(x)
    seqs = SeqArray(batch.seqs)
    # The timed region: every 5th step also carries event pairs around its attention and projection launches (the
    # kernel durations behind `roofline`); the step time reported is the median, which those few steps do not move.
    eng.ctx.set_option("time_gemm", 5)
    eng.ctx.set_option("time_attention", 5)
    ms, host_us, wall_ms = timed_steps(eng, lambda i: eng.ctx.step(seqs, x.data_ptr(), out.data_ptr()), a.steps, a.warmup)
    # The host's own work per step (plan, metadata, 800 launches): a call into an empty queue, three times.  Inside the timed
    # region the host runs one step ahead and then waits for room in the launch queue, so its time per call there equals
    # the device's.
    idle_us = []
    for i in range(3):
        eng.ctx.sync()
        h0 = time.perf_counter()
        eng.ctx.step(seqs, x.data_ptr(), out.data_ptr())
        idle_us.append((time.perf_counter() - h0) * 1e6)
    eng.ctx.sync()
    gemm_recs = np.array(eng.ctx.gemm_times(), dtype=np.float64).reshape(-1, 4)
    attn_ms = eng.ctx.attention_times()
    eng.ctx.set_option("time_gemm", 0)
    eng.ctx.set_option("time_attention", 0)
    med = float(np.median(ms))
    st = eng.ctx.step(seqs, x.data_ptr(), out.data_ptr(), want_stats=True)
    stage = {n: round(float(st.ms_stage[i]), 3) for i, n in enumerate(STAGE_NAMES)}
    params = H * (nq + 2 * nkv) * d + nq * d * H + 3 * H * F
    finite = bool(torch.isfinite(out.view(torch.bfloat16).float()).all().item())
    # dominant kernels of this step: the four projection launches of a layer (compute-bound at 1280 tokens)
    gemm_layer_ms = float(gemm_recs.sum(axis=1).mean()) if len(gemm_recs) else float("nan")
    flop_layer = 2.0 * params * T
    tflops = flop_layer / (gemm_layer_ms * 1e-3) / 1e12
    attn_avg = float(np.mean(attn_ms)) if attn_ms else float("nan")
    res = {"metric": "mixed_batch_step_throughput", "value": T / (med * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps,
           "warmup": a.warmup, "ms_per_step": med, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"cfg4: 70B-shaped stack (hidden 8192, 64 q / 8 kv heads, d 128, ffn 28672), {L} layers, {slots} KV slots, "
                                  f"{T} new tokens (1024-token chunk at prefix 4096 + 256 decodes), {total_kv} KV tokens per layer, "
                                  f"16-token pages, seed {a.seed}", "n_tokens": T, "total_kv": total_kv, "n_layers": L},
           "ms_per_step_events": percentiles(ms), "wall_ms_per_step": wall_ms / a.steps,
           "host_us_per_step": round(float(np.median(host_us)), 1),
           "host_us_per_step_into_an_empty_queue": round(float(np.median(idle_us)), 1),
           "roofline": {"bound": "mfma", "kernel": "gemm_sk_kernel: the four projection launches of one layer (QKV, O, gate/up + SwiGLU, down)",
                        "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops / MFMA_BF16_PEAK_TFLOPS,
                        "traffic": measured_traffic("cfg4", a.seed),
                        "traffic_note": "HBM bytes of the four launches of one layer: stored reading of the rocprofv3 FETCH_SIZE / WRITE_SIZE "
                                        "counters on a two-layer stack of this workload (null once the kernel source has changed since)",
                        "algorithmic_flop_per_launch_group": flop_layer, "avg_launch_group_ms": gemm_layer_ms,
                        "avg_launch_ms": {n: round(float(v), 4) for n, v in zip(("qkv", "o", "gate_up", "down"), gemm_recs.mean(axis=0))} if len(gemm_recs) else None,
                        "launch_groups_timed": int(len(gemm_recs)),
                        "note": "event pairs on the step's stream around each launch, in every 5th step of the timed region"},
           "attention": {"avg_launch_ms": attn_avg, "launches_timed": len(attn_ms),
                         "kv_GBs": 2 * nkv * d * 2 * total_kv / (attn_avg * 1e-3) / 1e9,
                         "note": "chunk and decode attention in one launch; the KV bytes of the decodes over the whole launch time"},
           "stage_ms_all_layers": stage, "output_finite": finite}
    res["roofline"]["clock"] = mfma_clock(eng.ctx, tflops)
    if check:
        from oracle import bf16 as obf
        from oracle import run as orun
        eng.ctx.set_option("out_f32", 1)
        out32 = torch.empty((T, H), dtype=torch.float32, device=eng.device)
        xin_t = torch.zeros((T, H), dtype=torch.float32, device=eng.device)
        xout_t = torch.zeros((T, H), dtype=torch.float32, device=eng.device)
        res["layer_checks"] = []
        for l in check:
            eng.ctx.set_taps(l, x_in=xin_t.data_ptr(), x_out=xout_t.data_ptr())
            eng.ctx.step(seqs, x.data_ptr(), out32.data_ptr())
            eng.ctx.sync()
            eng.ctx.set_taps(0)
            x_in = obf.from_bits(x_bits) if l == 0 else xin_t.cpu().numpy()
            got = xout_t.cpu().numpy()
            pool = orun.make_pool(m, batch.n_pool_pages, 1)
            for s in batch.seqs:                      # the slot's cached prefixes, read back from the device
                if s.prefix > 0:
                    k, v = eng.read_kv(l % slots, s.pages, 0, s.prefix)
                    pool.write_bits(0, [int(p) for p in s.pages], 0, k, v)
            log(f"cfg4: layer {l}: oracle running")
            import copy
            pool_b = copy.deepcopy(pool)
            w64 = orun.run_layer_from(m, cpu_weights[l], batch.seqs, x_in, pool, 0).astype(np.float64)
            wb64 = orun.run_layer_from(m, cpu_weights[l], batch.seqs, x_in, pool_b, 0, bf16_activations=True).astype(np.float64)
            rms = float(np.sqrt(np.mean(w64 * w64)))
            err = float(np.max(np.abs(got - w64))) / rms
            err_b = float(np.max(np.abs(got - wb64))) / rms
            gap = float(np.max(np.abs(wb64 - w64))) / rms
            d_b = np.abs(got - wb64)
            worst_row = int(np.argmax(d_b.max(axis=1)))
            rms_err_b = float(np.sqrt(np.mean(d_b * d_b))) / rms
            # One rule for every layer: within the bar of the definition evaluated with bf16 contraction operands,
            # hence within the bar plus the CPU-only distance between the two evaluations of the plain definition.
            ok = err_b <= 2e-2 and err <= 2e-2 + gap
            res["layer_checks"].append({"layer": l, "out_rms": rms, "max_err_over_rms_vs_bf16_operand_definition": err_b,
                                        "max_err_over_rms_vs_plain_definition": err, "cpu_only_gap_between_the_two": gap, "pass": bool(ok),
                                        "rms_err_over_rms_vs_bf16_operand_definition": rms_err_b, "worst_row": worst_row,
                                        "worst_row_is_prefill": bool(worst_row < batch.seqs[0].n_new)})
            log(f"cfg4: layer {l}: out rms {rms:.3f}; max|err|/rms = {err_b:.4f} (bf16-operand definition; rms of the error {rms_err_b:.5f}, "
                f"worst row {worst_row}), {err:.4f} (plain definition); the two differ by {gap:.4f} on the CPU alone")
    eng.close()
    del eng, kblk, vblk, x, out
    torch.cuda.empty_cache()
    if not a.no_cpu_baseline and not check:
        log("cfg4: timing the oracle on one layer")
        res["cpu_baseline"] = cpu_baseline_cfg4(batch, a.seed, L)
    return res


def run_model8b(a):
    """8B-shaped full model on one GPU (Sec. 2.1: tokens in, next token out): embedding gather, 32 layers,
    final norm, output projection over the whole vocabulary, greedy token.  Two batches: a single decode
    request (the per-token latency the paper quotes for its engine, Sec. 5.1) and the 64-decode batch."""
    import numpy as np
    import torch
    from paper_2507_17769_amd import workloads as W
    from paper_2507_17769_amd.binding import STAGE_NAMES, SeqArray
    from paper_2507_17769_amd.runner import Engine

    def log(msg):
        print(msg, file=sys.stderr, flush=True)

    model, L, V = "8b", a.layers if a.layers != 80 else 32, a.vocab
    m = W.MODELS[model]
    H, F, nq, nkv, d = m["hidden"], m["ffn"], m["n_q"], m["n_kv"], m["head_dim"]
    batches = {"1 decode, KV 1024": W.custom_batch(model, a.seed, 0, 0, [1024], name="b1"),
               "64 decodes, KV U[512,4096]": W.config_batch(1, a.seed)}
    n_pool = max(b.n_pool_pages for b in batches.values())
    eng = Engine(model, n_pool, L, L, max_position=4096 + 16)
    for kv in a.option:
        eng.ctx.set_option(kv.split("=")[0], int(kv.split("=")[1]))
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(2000 + a.seed)
    rnd = lambda shape, std: (torch.randn(shape, generator=gen, device="cuda:0", dtype=torch.float32) * std).to(torch.bfloat16)
    ones = torch.ones(H, dtype=torch.bfloat16, device="cuda:0")
    shapes = {"w_qkv": (H, (nq + 2 * nkv) * d), "w_o": (nq * d, H), "w_gate": (H, F), "w_up": (H, F), "w_down": (F, H)}
    for l in range(L):
        dev = {k: rnd(s, W.WEIGHT_STD) for k, s in shapes.items()}
        dev["g_attn"], dev["g_ffn"] = ones, ones
        eng.ctx.init_layer(l, **{k: t.data_ptr() for k, t in dev.items()})
        eng.ctx.sync()
        del dev
    emb, w_out = rnd((V, H), 1.0), rnd((H, V), W.WEIGHT_STD)
    eng.ctx.init_head(emb.data_ptr(), ones.data_ptr(), w_out.data_ptr(), V)
    eng.ctx.sync()
    eng.vocab = V
    log(f"model8b: {L} layers + head (vocab {V}) loaded")
    params_layer = H * (nq + 2 * nkv) * d + nq * d * H + 3 * H * F
    weight_bytes = 2 * (L * params_layer + H * V)          # streamed per step: all layers + output matrix
    res = {"metric": "full_model_step", "unit": "ms", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"model8b: 8B-shaped model, {L} layers, vocabulary {V}, greedy token", "n_layers": L, "vocab": V},
           "weight_bytes_per_step": weight_bytes, "batches": []}
    for name, batch in batches.items():
        # cached prefixes: one block of N(0,1) keys/values reused for every sequence and layer
        rng = np.random.Generator(np.random.PCG64([a.seed, 27182818]))
        from paper_2507_17769_amd.runner import bits_to_dev
        mp = max(s.prefix for s in batch.seqs)
        kblk = bits_to_dev(W.normal_bf16(rng, (mp, nkv, d)), eng.device)
        vblk = bits_to_dev(W.normal_bf16(rng, (mp, nkv, d)), eng.device)
        for slot in range(L):
            for s in batch.seqs:
                eng.ctx.kv_write(slot, s.pages, 0, s.prefix, kblk.data_ptr(), vblk.data_ptr())
        eng.ctx.sync()
        ids = W.token_ids(V, batch.n_tokens, a.seed, 1)
        seqs = SeqArray(batch.seqs)
        nxt = torch.empty(len(batch.seqs), dtype=torch.int32, device="cuda:0")
        for _ in range(max(2, min(a.warmup, 5))):
            eng.ctx.step_tokens(seqs, ids, nxt.data_ptr())
        eng.ctx.sync()
        steps = max(5, min(a.steps, 50))
        t0 = time.perf_counter()
        for _ in range(steps):
            eng.ctx.step_tokens(seqs, ids, nxt.data_ptr())
        eng.ctx.sync()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        st, parts = eng.ctx.step_tokens(seqs, ids, nxt.data_ptr(), want_stats=True, want_parts=True)
        rec = {"batch": name, "n_tokens": batch.n_tokens, "total_kv_per_layer": batch.total_kv, "ms_per_step": ms,
               "tokens_per_s": batch.n_tokens / (ms * 1e-3),
               "parts_ms": {"embedding": round(parts[0], 4), "layers": round(parts[1], 3), "head": round(parts[2], 4)},
               "stage_ms_all_layers": {n: round(float(st.ms_stage[i]), 3) for i, n in enumerate(STAGE_NAMES)},
               "hbm_GBs": (weight_bytes + 2 * nkv * d * 2 * batch.total_kv * L) / (ms * 1e-3) / 1e9}
        # head check, teacher-forced: the oracle's head applied to the device's own final hidden states
        if not a.no_cpu_baseline:
            from oracle import bf16 as obf
            from oracle import head as oh
            from oracle import run as orun
            out = {"logits": torch.empty((len(batch.seqs), V), dtype=torch.float32, device="cuda:0"),
                   "hidden": torch.empty((batch.n_tokens, H), dtype=torch.float32, device="cuda:0")}
            eng.ctx.step_tokens(seqs, ids, nxt.data_ptr(), out["logits"].data_ptr(), out["hidden"].data_ptr())
            eng.ctx.sync()
            hid, lg, tok = out["hidden"].cpu().numpy(), out["logits"].cpu().numpy(), nxt.cpu().numpy()
            w_host = w_out.float().cpu().numpy()
            want = oh.logits(hid, orun.to_seqs(batch.seqs), np.ones(H, np.float32), w_host, W.RMS_EPS)
            rms = float(np.sqrt(np.mean(want.astype(np.float64) ** 2)))
            err = float(np.max(np.abs(lg - want))) / rms
            first_max = np.argmax(lg, axis=1)
            lead_ok = all(want[i, tok[i]] >= want[i].max() - 4e-2 * rms for i in range(len(tok)))
            rec["head_check"] = {"logits_max_err_over_rms": err, "greedy_is_first_max_of_device_logits": bool(np.array_equal(tok, first_max)),
                                 "greedy_within_rounding_of_oracle_best": bool(lead_ok), "finite": bool(np.isfinite(hid).all()),
                                 "pass": bool(err <= 2e-2 and np.array_equal(tok, first_max) and lead_ok)}
            log(f"model8b: {name}: head check max|err|/rms = {err:.4f}")
        res["batches"].append(rec)
        log(f"model8b: {name}: {ms:.3f} ms/step")
    eng.close()
    print(json.dumps(res))


def run_prefill(a):
    """Prefill-only steps of an 8B-shaped layer, as a prefill instance of a prefill-decode disaggregated
    deployment runs them (Sec. 3.4: its token batch reaches 2048): one request or several sharing the step."""
    import numpy as np
    import torch
    from paper_2507_17769_amd import workloads as W
    from paper_2507_17769_amd.binding import STAGE_NAMES, SeqArray
    from paper_2507_17769_amd.runner import Engine, bits_to_dev

    model = "8b"
    m = W.MODELS[model]
    H, F, nq, nkv, d = m["hidden"], m["ffn"], m["n_q"], m["n_kv"], m["head_dim"]
    params = H * (nq + 2 * nkv) * d + nq * d * H + 3 * H * F
    specs = {"1 x 2048": [(2048, 0)], "4 x 512": [(512, 0)] * 4, "16 x 128": [(128, 0)] * 16,
             "2 x 1024 at prefix 1024": [(1024, 1024)] * 2, "1023 + 1 + 1024 (budget boundary)": [(1023, 0), (1, 2049), (1024, 0)]}
    batches = {k: W.multi_batch(model, a.seed, v, []) for k, v in specs.items()}
    n_copies = 4
    eng = Engine(model, max(b.n_pool_pages for b in batches.values()), n_copies, 1, max_position=4096 + 16)
    for kv in a.option:
        eng.ctx.set_option(kv.split("=")[0], int(kv.split("=")[1]))
    weights = W.layer_weights(model, a.seed, 0)
    for l in range(n_copies):
        eng.load_layer(l, weights)
    res = {"metric": "prefill_step", "unit": "ms", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "prefill-only steps, 8B-shaped layer, four weight copies in rotation"}, "batches": []}
    for name, b in batches.items():
        eng.load_prefixes(b)
        x = bits_to_dev(b.activations(), eng.device)
        out = torch.empty_like(x)
        seqs = SeqArray(b.seqs)
        for i in range(5):
            eng.ctx.set_option("only_layer", i % n_copies)
            eng.ctx.step(seqs, x.data_ptr(), out.data_ptr())
        eng.ctx.sync()
        steps = max(10, min(a.steps, 100))
        t0 = time.perf_counter()
        for i in range(steps):
            eng.ctx.set_option("only_layer", i % n_copies)
            eng.ctx.step(seqs, x.data_ptr(), out.data_ptr())
        eng.ctx.sync()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        stage = np.zeros(len(STAGE_NAMES))
        for i in range(5):
            eng.ctx.set_option("only_layer", i % n_copies)
            st = eng.ctx.step(seqs, x.data_ptr(), out.data_ptr(), want_stats=True)
            stage += np.array(list(st.ms_stage)) / 5
        T = b.n_tokens
        gemm_ms = float(stage[1] + stage[4] + stage[6] + stage[7])
        # causal (query, key) pairs of the step, 4 * d * n_q flop each
        pairs = sum(s.n_new * s.prefix + s.n_new * (s.n_new + 1) // 2 for s in b.seqs)
        res["batches"].append({"batch": name, "n_tokens": T, "ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3),
                               "stage_ms": {n: round(float(v), 4) for n, v in zip(STAGE_NAMES, stage)},
                               "gemm_tflops": 2 * params * T / (gemm_ms * 1e-3) / 1e12,
                               "gemm_frac_mfma": 2 * params * T / (gemm_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                               "attention_tflops": 4 * d * nq * pairs / (float(stage[3]) * 1e-3) / 1e12})
    clk = mfma_clock(eng.ctx, 0.0)
    del clk["frac_mfma_at_that_clock"]
    res["clock"] = clk
    for r in res["batches"]:
        r["gemm_frac_mfma_at_measured_clock"] = r["gemm_tflops"] / clk["mfma_peak_at_that_clock_tflops"]
    eng.close()
    print(json.dumps(res))


def measure_profile(a, batch_sizes, kv_sizes, n_decodes_in_mixed=256, extra_batches=None):
    """Measure the map (batch size, KV cache size) -> iteration time of the whole 8B-shaped model (Sec. 4.5) with
    ps_step_tokens.  Rows up to n_decodes_in_mixed tokens are decode batches (the KV size split evenly over the requests);
    larger rows are the co-located kind of batch (Sec. 2.4): n_decodes_in_mixed decodes plus one prefill chunk with the
    remaining tokens at prefix 0, the decodes sharing the KV size that the chunk does not attend.  Returns
    (measured table with NaN where a cell cannot exist, table with those cells filled from the nearest measured cell of the
    row, layers, vocabulary, KV capacity in tokens of one 288 GB instance); with extra_batches (a dict name -> batch) also
    the measured step time of each of those, as a last element."""
    import numpy as np
    import torch
    from paper_2507_17769_amd import workloads as W
    from paper_2507_17769_amd.binding import SeqArray
    from paper_2507_17769_amd.runner import Engine, bits_to_dev

    model, L, V = "8b", a.layers if a.layers != 80 else 32, a.vocab
    m = W.MODELS[model]
    H, F, nq, nkv, d = m["hidden"], m["ffn"], m["n_q"], m["n_kv"], m["head_dim"]
    cells = {}
    for bs in batch_sizes:
        for kv in kv_sizes:
            if bs <= n_decodes_in_mixed:
                per = kv // bs
                if 16 <= per:
                    cells[(bs, kv)] = W.custom_batch(model, a.seed, 0, 0, [per] * bs, name=f"b{bs}_kv{kv}", tag=bs * 7 + 1)
            else:
                chunk = bs - n_decodes_in_mixed
                per = (kv - chunk) // n_decodes_in_mixed
                if 16 <= per:
                    cells[(bs, kv)] = W.custom_batch(model, a.seed, chunk, 0, [per] * n_decodes_in_mixed, name=f"b{bs}_kv{kv}", tag=bs * 7 + 1)
    todo = dict(cells)
    todo.update(extra_batches or {})
    n_pool = max(b.n_pool_pages for b in todo.values())
    eng = Engine(model, n_pool, L, L, max_position=max(s.kv_len for b in todo.values() for s in b.seqs) + 16)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(3000 + a.seed)
    rnd = lambda shape, std: (torch.randn(shape, generator=gen, device="cuda:0", dtype=torch.float32) * std).to(torch.bfloat16)
    ones = torch.ones(H, dtype=torch.bfloat16, device="cuda:0")
    shapes = {"w_qkv": (H, (nq + 2 * nkv) * d), "w_o": (nq * d, H), "w_gate": (H, F), "w_up": (H, F), "w_down": (F, H)}
    for l in range(L):
        dev = {k: rnd(s, W.WEIGHT_STD) for k, s in shapes.items()}
        dev["g_attn"], dev["g_ffn"] = ones, ones
        eng.ctx.init_layer(l, **{k: t.data_ptr() for k, t in dev.items()})
        eng.ctx.sync()
        del dev
    emb, w_out = rnd((V, H), 1.0), rnd((H, V), W.WEIGHT_STD)
    eng.ctx.init_head(emb.data_ptr(), ones.data_ptr(), w_out.data_ptr(), V)
    eng.ctx.sync()
    # the cache content does not matter for timing: the pool is filled once with N(0,1) values through one sequence-sized block
    rng = np.random.Generator(np.random.PCG64([a.seed, 16180339]))
    blk = bits_to_dev(W.normal_bf16(rng, (4096, nkv, d)), eng.device)
    table = np.full((len(batch_sizes), len(kv_sizes)), np.nan, dtype=np.float32)
    steps = max(3, min(a.steps, 10))
    extra_ms = {}
    for key, b in todo.items():
        for s in b.seqs:          # keys and values of every cached position, block by block
            for p0 in range(0, s.prefix, 4096):
                n = min(4096, s.prefix - p0)
                for slot in range(L):
                    eng.ctx.kv_write(slot, s.pages, p0, n, blk.data_ptr(), blk.data_ptr())
        eng.ctx.sync()
        ids = W.token_ids(V, b.n_tokens, a.seed, 2)
        seqs = SeqArray(b.seqs)
        nxt = torch.empty(len(b.seqs), dtype=torch.int32, device="cuda:0")
        for _ in range(2):
            eng.ctx.step_tokens(seqs, ids, nxt.data_ptr())
        eng.ctx.sync()
        t0 = time.perf_counter()
        for _ in range(steps):
            eng.ctx.step_tokens(seqs, ids, nxt.data_ptr())
        eng.ctx.sync()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        if key in cells:
            bs, kv = key
            table[batch_sizes.index(bs), kv_sizes.index(kv)] = ms
            print(f"profile: batch {bs} kv {kv}: {ms:.3f} ms", file=sys.stderr, flush=True)
        else:
            extra_ms[key] = ms
    eng.close()
    filled = table.copy()
    for i in range(len(batch_sizes)):
        for j in range(len(kv_sizes)):
            if np.isnan(filled[i, j]):
                js = [jj for jj in range(len(kv_sizes)) if not np.isnan(table[i, jj])]
                filled[i, j] = table[i, min(js, key=lambda jj: abs(jj - j))]
    # KV capacity of what is left of 288 GB beside the weights and 8 GB of workspace
    weights_gb = 2 * (L * (H * (nq + 2 * nkv) * d + nq * d * H + 3 * H * F) + 2 * H * V) / 1e9
    capacity = (288 - weights_gb - 8) * 1e9 / (2 * nkv * d * 2 * L)
    if extra_batches is not None:
        return table, filled, L, V, capacity, extra_ms
    return table, filled, L, V, capacity


def run_profile(a):
    """The map (batch size, KV cache size) -> iteration time of the whole 8B-shaped model (Sec. 4.5), measured on
    decode batches, and the router's decisions taken with it through polysched (Sec. 3.4, 4.5-4.7) for the paper's
    TPOT tiers (Sec. 5.1: 20, 30, 50, 100 ms; TTFT 300, 500, 1000 ms)."""
    import numpy as np
    from paper_2507_17769_amd import binding as B

    batch_sizes = [1, 4, 16, 64, 256]
    kv_sizes = [4096, 32768, 131072, 524288]          # total KV tokens of the batch
    table, filled, L, V, capacity = measure_profile(a, batch_sizes, kv_sizes)
    prof = B.Profile(batch_sizes, kv_sizes, filled)
    res = {"metric": "iteration_time_profile", "unit": "ms", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"profile: 8B-shaped model, {L} layers + head, decode batches", "n_layers": L, "vocab": V},
           "batch_sizes": batch_sizes, "kv_sizes": kv_sizes,
           "ms": [[None if np.isnan(v) else round(float(v), 4) for v in row] for row in table], "decisions": {}}
    dec = res["decisions"]
    # Sec. 3.4: largest decode batch per TPOT tier for a request shape (p, d), KV capacity of what is left of 288 GB
    dec["kv_capacity_tokens"] = int(capacity)
    dec["batch_limit_pd"] = {f"p={p},d={dd},tpot={t}": prof.batch_limit_pd(p, dd, t, capacity, 4096)
                             for (p, dd) in ((512, 512), (4096, 1024)) for t in (20, 30, 50, 100)}
    dec["batch_limit_co"] = {f"p={p},d={dd},tpot={t},ttft={tt}": prof.batch_limit_co(p, dd, t, tt, capacity, 4096)
                             for (p, dd) in ((512, 512), (4096, 1024)) for t in (20, 50, 100) for tt in (300, 1000)}
    # Sec. 4.5/4.6: a server with 63 running requests (KV 2000, 100 tokens generated), average output 512
    run = [(2000, 100)] * 63
    dec["admit_64th_request"] = {f"tpot={t},wait={w}": list(prof.predict_admit(run, 1000, 512, t, w)) for t in (20, 30) for w in (0.0, 15.0)}
    # Sec. 4.7: the worked example, and a co-located prefill
    sizes = lambda plan: [sum(t for _, t in it) for it in plan]
    dec["chunk_plan_2050_budget_1024"] = {"chunked": sizes(B.chunk_plan([2050], 1024, False)), "chunked_after_1023": sizes(B.chunk_plan([2050], 1024, False, 1023)),
                                          "dynamic": sizes(B.chunk_plan([2050], 1024, True)), "dynamic_after_1023": sizes(B.chunk_plan([2050], 1024, True, 1023))}
    dec["chunked_prefill_2000_tokens_beside_63_decodes"] = {f"tpot={t},ttft={tt}": list(prof.predict_chunked_prefill(run, 2000, 512, t, tt)) for t in (20, 50) for tt in (300, 1000)}
    prof.close()
    print(json.dumps(res))


def run_sim(a):
    """The paper's evaluation method (Sec. 5.1) on the table measured here: a cluster of 20 instances simulated in 1 ms steps
    under the router of Sec. 4, co-located and disaggregated, on the two synthetic traces the paper fully specifies
    (uniform_512_512, uniform_4096_1024: Sec. 5.1 / Table of trace statistics) and on the tier-flip workload of Sec. 5.3,
    with the SLO tiers of Sec. 5.1.  Reports DSLO attainment per request rate and per TPOT tier, the goodput at 90 %
    attainment, instance-seconds per request, and how many requests per second of wall time the C++ router places."""
    import numpy as np
    from paper_2507_17769_amd import binding as B
    from paper_2507_17769_amd import workloads as W

    batch_sizes = [1, 16, 64, 256, 512, 1024, 2048, 4096]
    kv_sizes = [4096, 32768, 131072, 524288]
    if a.table:
        rec = json.load(open(a.table))
        batch_sizes, kv_sizes = rec["batch_sizes"], rec["kv_sizes"]
        table = np.array([[np.nan if v is None else v for v in row] for row in rec["ms"]], dtype=np.float32)
        filled = np.array(rec["ms_filled"], dtype=np.float32)
        L, V, capacity = rec["n_layers"], rec["vocab"], rec["kv_capacity_tokens"]
    else:
        # besides the table's cells: random batches of the kind an instance runs (decodes with log-normal KV lengths, with
        # or without a prefill chunk at some prefix), to see how well a lookup by (tokens, KV size) predicts their time
        rng = np.random.Generator(np.random.PCG64([a.seed, 314159]))
        check = {}
        for i in range(24):
            n_dec = int(np.exp(rng.uniform(0.0, np.log(512.0))))
            chunk = 0 if rng.random() < 0.4 else int(np.exp(rng.uniform(np.log(16.0), np.log(1536.0))))
            kvs = W.lognormal_lengths(rng, n_dec, 1024, 0.8, 16, 8192)
            check[f"check{i}"] = W.custom_batch("8b", a.seed, chunk, int(rng.integers(0, 4096)) if chunk else 0, kvs, name=f"check{i}", tag=900 + i)
        table, filled, L, V, capacity, check_ms = measure_profile(a, batch_sizes, kv_sizes, extra_batches=check)
    prof = B.Profile(batch_sizes, kv_sizes, filled)
    tpots = list(W.SIM_TPOTS_MS)
    n, n_servers = a.requests, 20
    res = {"metric": "cluster_simulation_dslo_goodput", "unit": "requests/s at >= 90 % DSLO attainment", "n_gpus": 1, "dtype": "bf16",
           "data": "synthetic", "higher_is_better": True, "vs_baseline": None,
           "config": {"workload": f"sim: {n_servers} simulated instances of the 8B-shaped model ({L} layers + head), iteration times from the "
                                  f"table measured on this GPU, {n} requests per run, TPOT tiers {tpots} ms, TTFT 300/500/1000 ms"},
           "batch_sizes": batch_sizes, "kv_sizes": kv_sizes, "n_layers": L, "vocab": V, "kv_capacity_tokens": int(capacity),
           "ms": [[None if np.isnan(v) else round(float(v), 4) for v in row] for row in table],
           "ms_filled": [[round(float(v), 4) for v in row] for row in filled], "runs": [], "goodput": {}}
    if not a.table:
        rows = []
        for name, b in check.items():
            pred = prof.lookup(b.n_tokens, b.total_kv)
            rows.append({"decodes": sum(1 for s in b.seqs if s.n_new == 1), "chunk": max(s.n_new for s in b.seqs) if any(s.n_new > 1 for s in b.seqs) else 0,
                         "tokens": b.n_tokens, "kv": b.total_kv, "measured_ms": round(check_ms[name], 3), "looked_up_ms": round(pred, 3),
                         "ratio": round(pred / check_ms[name], 3)})
        ratios = np.array([r["ratio"] for r in rows])
        res["table_check"] = {"batches": rows, "looked_up_over_measured": {"min": float(ratios.min()), "median": float(np.median(ratios)), "max": float(ratios.max())}}
    # request rates: from the start value up in steps of 30 % until the attainment falls below 90 % (at most 16 steps)
    traces = {"uniform_512_512": (1024, 1024, False, 100.0), "uniform_4096_1024": (8192, 2048, False, 20.0),
              "tier_flip_4096_1024": (8192, 2048, True, 20.0)}
    wall_total, placed_total, tests_total = 0.0, 0, 0
    res["optimal"] = {}
    for name, (max_p, max_o, burst, rate0) in traces.items():
        for mode in ("co-located", "disaggregated"):
            # Sec. 3.5: the minimal cost of every request at its batch limits -> the request rate 20 instances could carry at best
            tr = W.sim_trace(a.seed, n, 1.0, max_p, max_o, burst=burst)
            costs = []
            for i in range(min(n, 2000)):
                p_, d_, tp_, tt_ = tr["prompt"][i], tr["output"][i], tpots[tr["tier"][i]], tr["ttft"][i]
                costs.append(prof.optimal_cost_co(p_, d_, tp_, tt_, capacity, 4096) if mode == "co-located"
                             else prof.optimal_cost_pd(p_, d_, tp_, capacity, 2048, 4096))
            finite = [c for c in costs if np.isfinite(c)]
            res["optimal"][f"{name} {mode}"] = {"instance_ms_per_request": round(float(np.mean(finite)), 3),
                                                "rate_per_s": round(n_servers * 1e3 / float(np.mean(finite)), 1),
                                                "requests_without_a_feasible_batch": len(costs) - len(finite)}
            best, att = 0.0, 1.0
            for step in range(16):
                if att < 0.9:
                    break
                rate = round(rate0 * 1.3 ** step, 1)
                tr = W.sim_trace(a.seed, n, rate / 1e3, max_p, max_o, burst=burst)
                t0 = time.perf_counter()
                r = prof.simulate(tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], tpots, n_servers, (1 + max_o) // 2, capacity,
                                  1000, disaggregated=(mode == "disaggregated"), prefill_budget=2048)
                wall = time.perf_counter() - t0
                wall_total, placed_total, tests_total = wall_total + wall, placed_total + n, tests_total + r["admission_tests"]
                tier = np.array(tr["tier"])
                att = float(r["attained"].mean())
                if att >= 0.9:
                    best = max(best, rate * att)
                res["runs"].append({"trace": name, "mode": mode, "rate_per_s": rate, "attained": round(att, 4),
                                    "attained_by_tier": [round(float(r["attained"][tier == t].mean()), 4) for t in range(len(tpots))],
                                    "dropped": int(r["dropped"]), "promotions": int(r["promotions"]), "scale_ups": int(r["scale_ups"]),
                                    "instance_seconds_per_request": round(r["cost_ms"] / 1e3 / n, 4),
                                    "simulated_s": round(r["end_ms"] / 1e3, 1), "wall_s": round(wall, 3)})
                print(f"sim: {name} {mode} {rate}/s attained {att:.3f} wall {wall:.2f}s", file=sys.stderr, flush=True)
            res["goodput"][f"{name} {mode}"] = round(best, 1)
            res["optimal"][f"{name} {mode}"]["goodput_over_optimal"] = round(best / res["optimal"][f"{name} {mode}"]["rate_per_s"], 3)
    # Sec. 5.4: an unlimited pool (200 instances), auto-scaling decides how many are used; cost = instance time per request
    res["cost_with_unlimited_pool"] = []
    for name, (max_p, max_o, burst, rate0) in traces.items():
        for mode in ("co-located", "disaggregated"):
            for frac in (0.25, 1.0):
                rate = max(1.0, round(frac * res["goodput"][f"{name} {mode}"], 1))
                tr = W.sim_trace(a.seed, n, rate / 1e3, max_p, max_o, burst=burst)
                t0 = time.perf_counter()
                r = prof.simulate(tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], tpots, 200, (1 + max_o) // 2, capacity,
                                  1000, disaggregated=(mode == "disaggregated"), prefill_budget=2048)
                wall_total, placed_total, tests_total = wall_total + time.perf_counter() - t0, placed_total + n, tests_total + r["admission_tests"]
                res["cost_with_unlimited_pool"].append({
                    "trace": name, "mode": mode, "rate_per_s": rate, "attained": round(float(r["attained"].mean()), 4),
                    "instance_ms_per_request": round(r["cost_ms"] / n, 2), "mean_instances_in_use": round(r["cost_ms"] / r["end_ms"], 2),
                    "optimal_instance_ms_per_request": res["optimal"][f"{name} {mode}"]["instance_ms_per_request"]})
                print(f"sim: cost {name} {mode} {rate}/s: {r['cost_ms'] / n:.1f} instance-ms per request", file=sys.stderr, flush=True)
    # Sec. 5.5: goodput per instance as the number of instances grows (uniform_4096_1024; rate from 60 % of the optimum
    # of Sec. 3.5 upwards in steps of 15 % until the attainment falls below 90 %)
    res["goodput_per_instance"] = []
    n5 = min(n, 50000)
    for mode in ("co-located", "disaggregated"):
        opt20 = res["optimal"][f"uniform_4096_1024 {mode}"]["rate_per_s"] / n_servers
        for servers in (8, 16, 32, 64):
            best, att = 0.0, 1.0
            for step in range(8):
                if att < 0.9:
                    break
                rate = round(0.6 * opt20 * servers * 1.15 ** step, 1)
                tr = W.sim_trace(a.seed, n5, rate / 1e3, 8192, 2048)
                t0 = time.perf_counter()
                r = prof.simulate(tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], tpots, servers, 1024, capacity,
                                  1000, disaggregated=(mode == "disaggregated"), prefill_budget=2048)
                wall_total, placed_total, tests_total = wall_total + time.perf_counter() - t0, placed_total + n5, tests_total + r["admission_tests"]
                att = float(r["attained"].mean())
                if att >= 0.9:
                    best = max(best, rate * att)
            res["goodput_per_instance"].append({"mode": mode, "instances": servers, "goodput_per_s": round(best, 1),
                                                "per_instance": round(best / servers, 2)})
            print(f"sim: {mode} {servers} instances: {best / servers:.2f} requests/s per instance", file=sys.stderr, flush=True)
    prof.close()
    res["value"] = res["goodput"]["uniform_512_512 co-located"]
    res["router"] = {"requests_per_wall_second": round(placed_total / wall_total, 1), "admission_tests_per_wall_second": round(tests_total / wall_total, 1),
                     "note": "whole simulation (instances stepped in 1 ms steps included), one host thread"}
    if not a.no_cpu_baseline:
        # the oracle simulator on a bounded sample, on a table of the same shape that does not come from the GPU path
        from oracle import policy as opol
        from oracle import sim as osim
        ms = np.array([[4.0 + 0.013 * b + 2.2e-5 * k for k in kv_sizes] for b in batch_sizes], dtype=np.float32)
        tr = W.sim_trace(a.seed, 2000, 0.1, 1024, 1024)
        args = (tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], tpots, n_servers, 512, capacity, 1000)
        t0 = time.perf_counter()
        want = osim.simulate(opol.Profile(batch_sizes, kv_sizes, ms.astype(np.float64).tolist()), *args)
        t_oracle = time.perf_counter() - t0
        gp = B.Profile(batch_sizes, kv_sizes, ms)
        t0 = time.perf_counter()
        got = gp.simulate(*args)
        t_cpp = time.perf_counter() - t0
        gp.close()
        assert got["attained"].tolist() == want["attained"] and got["finish_ms"].tolist() == want["finish_ms"]
        res["cpu_baseline"] = {"value": round(2000 / t_oracle, 1), "unit": "simulated requests per wall second", "cores": 1, "kind": "oracle",
                               "sample": "uniform_512_512, 2000 requests at 100/s, co-located, analytic table 4 + 0.013 B + 2.2e-5 KV ms",
                               "same_sample_cpp": round(2000 / t_cpp, 1), "identical_outputs": True}
    print(json.dumps(res))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2507_17769_amd import workloads as W
    from paper_2507_17769_amd.binding import STAGE_NAMES, SeqArray
    from paper_2507_17769_amd.runner import Engine, bits_to_dev

    if a.device_info:
        p = torch.cuda.get_device_properties(0)
        info = {k: getattr(p, k) for k in dir(p) if not k.startswith("_") and isinstance(getattr(p, k), (int, float, str))}
        info["torch"], info["hip"] = torch.__version__, torch.version.hip
        print(json.dumps(info))
        return
    if a.calibrate_copy:
        n = 1 << 30
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n, "copies": 3}))
        return
    if a.workload == "sim" and a.table:   # host only: the table was measured by an earlier run
        run_sim(a)
        return
    if not a.null_stream:   # a stream of our own (default priority); torch only allocates and copies
        torch.cuda.set_stream(torch.cuda.Stream(device="cuda:0"))
    if a.workload == "grid":
        run_grid(a)
        return
    if a.workload == "cfg4":
        # The headline: the largest single-GPU configuration.  One JSON line; the single-layer 8B-shaped configurations
        # ride along as secondary records (decode attention against the HBM roofline, mixed-batch GEMMs against MFMA).
        res = run_cfg4(a)
        if not a.no_secondary and not a.check_layers:
            res["secondary"] = {}
            for name, cfg in (("cfg1", 1), ("cfg2", 2)):
                print(f"bench: secondary record {name}", file=sys.stderr, flush=True)
                res["secondary"][name] = run_layer_cfg(a, cfg, 200, 20, cpu=not a.no_cpu_baseline)
            res["secondary"]["host_cost_700_short_decodes"] = host_cost_many_sequences(a)
        print(json.dumps(res))
        return
    if a.workload == "model8b":
        run_model8b(a)
        return
    if a.workload == "prefill":
        run_prefill(a)
        return
    if a.workload == "sim":
        run_sim(a)
        return
    if a.workload == "profile":
        run_profile(a)
        return
    print(json.dumps(run_layer_cfg(a, {"cfg1": 1, "cfg2": 2}[a.workload], a.steps, a.warmup, cpu=not a.no_cpu_baseline)))


def host_cost_many_sequences(a):
    """Host side of a step with many sequences (700 one-token requests with 1..50 cached tokens, 8B-shaped layer):
    validation, planning, metadata fill and the enqueue of the step's launches, per ps_step call with the stream busy."""
    import numpy as np
    import torch
    from paper_2507_17769_amd import workloads as W
    from paper_2507_17769_amd.binding import SeqArray
    from paper_2507_17769_amd.runner import Engine, bits_to_dev
    kv = 1 + (np.arange(700) * 37) % 50
    b = W.custom_batch("8b", a.seed, 0, 0, kv, name="many")
    eng = Engine(b.model, b.n_pool_pages, 1, 1, max_position=128)
    eng.load_layer(0, W.layer_weights(b.model, a.seed, 0))
    eng.load_prefixes(b)
    x = bits_to_dev(b.activations(), eng.device)
    out = torch.empty_like(x)
    seqs = SeqArray(b.seqs)
    ms, host_us, wall_ms = timed_steps(eng, lambda i: eng.ctx.step(seqs, x.data_ptr(), out.data_ptr()), 100, 10)
    eng.close()
    return {"n_seqs": 700, "n_tokens": b.n_tokens, "total_kv": b.total_kv, "host_us_per_step": round(float(np.median(host_us)), 1),
            "ms_per_step": round(float(np.median(ms)), 4), "wall_ms_per_step": round(wall_ms / 100, 4)}


def run_layer_cfg(a, cfg, steps, warmup, cpu=True):
    """One 8B-shaped layer: the decode-only batch (cfg 1) or the mixed batch (cfg 2).  Returns the result record."""
    import numpy as np
    import torch
    from paper_2507_17769_amd import workloads as W
    from paper_2507_17769_amd.binding import STAGE_NAMES, SeqArray
    from paper_2507_17769_amd.runner import Engine, bits_to_dev

    name = f"cfg{cfg}"
    batch = W.config_batch(cfg, a.seed)
    model = W.MODELS[batch.model]
    weights = W.layer_weights(batch.model, a.seed, 0)
    # Four device copies of the layer (1.7 GB, several times the 256 MB last-level cache), one per step in
    # rotation: every step streams its weights from HBM, as a layer inside a 32-layer model would.
    n_copies = 4
    eng = Engine(batch.model, batch.n_pool_pages, n_copies, 1, max_position=max(s.kv_len for s in batch.seqs) + 16)
    for kv in a.option:
        eng.ctx.set_option(kv.split("=")[0], int(kv.split("=")[1]))
    for l in range(n_copies):
        eng.load_layer(l, weights)
    eng.load_prefixes(batch)
    x = bits_to_dev(batch.activations(), eng.device)
    out = torch.empty_like(x)
    seqs = SeqArray(batch.seqs)
    T, total_kv = batch.n_tokens, batch.total_kv

    def call(i):
        eng.ctx.set_option("only_layer", i % n_copies)
        eng.ctx.step(seqs, x.data_ptr(), out.data_ptr())

    # the timed region carries no instrumentation: at a quarter of a millisecond per step two event records show
    ms, host_us, wall_ms = timed_steps(eng, call, steps, warmup)
    med = float(np.median(ms))
    # kernel durations for the roofline: event pairs around the attention launch and the projection launches, in
    # 32 further steps of the same loop
    eng.ctx.set_option("time_attention", 1)
    eng.ctx.set_option("time_gemm", 1)
    for i in range(32):
        call(i)
    attn_ms = eng.ctx.attention_times()
    gemm_recs = np.array(eng.ctx.gemm_times(), dtype=np.float64).reshape(-1, 4)
    eng.ctx.set_option("time_attention", 0)
    eng.ctx.set_option("time_gemm", 0)

    # per-stage split (separate, synchronous passes; not part of the timed region)
    stage = np.zeros(len(STAGE_NAMES))
    n_stat = 10
    for i in range(n_stat):
        eng.ctx.set_option("only_layer", i % n_copies)
        st = eng.ctx.step(seqs, x.data_ptr(), out.data_ptr(), want_stats=True)
        stage += np.array(list(st.ms_stage))
    stage /= n_stat

    H, F = model["hidden"], model["ffn"]
    nq, nkv, d = model["n_q"], model["n_kv"], model["head_dim"]
    params = H * (nq + 2 * nkv) * d + nq * d * H + 3 * H * F
    kv_bytes_per_token = 2 * nkv * d * 2
    attn_avg_ms = float(np.mean(attn_ms)) if attn_ms else float("nan")
    attn_bytes = kv_bytes_per_token * total_kv
    achieved = attn_bytes / (attn_avg_ms * 1e-3) / 1e9
    gemm_ms = float(gemm_recs.sum(axis=1).mean())
    gemm_tflops = 2 * params * T / (gemm_ms * 1e-3) / 1e12
    hbm_roof = {"bound": "hbm", "kernel": "attn_kernel (paged attention, split merge excluded)",
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": measured_traffic(name, a.seed),
                "traffic_note": "stored reading of the rocprofv3 FETCH_SIZE / WRITE_SIZE counters of an earlier run of this command "
                                "(null once the kernel source has changed since)",
                "algorithmic_bytes_per_launch": attn_bytes, "avg_launch_ms": attn_avg_ms, "launches_timed": len(attn_ms)}
    mfma_roof = {"bound": "mfma", "kernel": "the four projection launches of the layer (QKV, O, gate/up + SwiGLU, down)",
                 "achieved": gemm_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": gemm_tflops / MFMA_BF16_PEAK_TFLOPS,
                 "traffic": None, "algorithmic_flop_per_launch_group": 2.0 * params * T, "avg_launch_group_ms": gemm_ms,
                 "avg_launch_ms": {n: round(float(v), 4) for n, v in zip(("qkv", "o", "gate_up", "down"), gemm_recs.mean(axis=0))},
                 "launch_groups_timed": int(len(gemm_recs))}
    res = {
        "metric": "mixed_batch_step_throughput", "value": T / (med * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": med,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{batch.name}: 8B-shaped layer (hidden 4096, 32 q / 8 kv heads, d 128, ffn 14336), "
                               f"{T} new tokens ({sum(1 for s in batch.seqs if s.n_new == 1)} decodes"
                               f"{', 512-token chunk at prefix 2048' if cfg == 2 else ''}), {total_kv} KV tokens, "
                               f"16-token pages, seed {a.seed}",
                   "n_tokens": T, "total_kv": total_kv, "n_layers": 1},
        "ms_per_step_events": percentiles(ms), "wall_ms_per_step": wall_ms / steps, "host_us_per_step": round(float(np.median(host_us)), 1),
        # the decode-only step is bound by the bytes it streams, the mixed step by its projections
        "roofline": hbm_roof if cfg == 1 else mfma_roof,
        "roofline_other": mfma_roof if cfg == 1 else hbm_roof,
        "step_hbm_GBs": (2 * params + attn_bytes) / (med * 1e-3) / 1e9,
        "stage_ms": {n: round(float(v), 4) for n, v in zip(STAGE_NAMES, stage)},
        "gemm": {"ms": gemm_ms, "weight_GBs": 2 * params / (gemm_ms * 1e-3) / 1e9, "tflops": gemm_tflops,
                 "frac_hbm": 2 * params / (gemm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "frac_mfma": gemm_tflops / MFMA_BF16_PEAK_TFLOPS},
    }
    res["gemm"]["clock"] = mfma_clock(eng.ctx, gemm_tflops)
    # the same fraction against what plain loads stream out of HBM on this device (2 GiB buffer, read after the timed region)
    stream_gbs = eng.ctx.hbm_read_rate(2 << 30, 4)
    hbm_roof["measured_stream_read_GBs"] = round(stream_gbs, 1)
    hbm_roof["frac_of_measured_stream_read"] = achieved / stream_gbs
    eng.close()
    del eng, x, out
    torch.cuda.empty_cache()
    if cpu:
        res["cpu_baseline"] = cpu_baseline(batch, weights)
    return res


if __name__ == "__main__":
    main()
