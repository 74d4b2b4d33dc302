#!/usr/bin/env python3
"""Benchmark of the SiDA-MoE layer hot path on one MI355X.

A step is one pass of the whole path over one batch: for each of the workload's L MoE layers,
plan (host) -> expert prefetch host->HBM pool on the copy stream -> counting sort + gather ->
grouped expert FFN per wave -> gate-weighted combine.  Token activations, ids and gate values are
resident in HBM before the timed region; expert weights live in pinned host memory and stream
through the S-slot pool, as the workload states.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
H2D_PEAK_GBS = 64.0            # PCIe Gen5 x16, one direction

COUNTER_PROFILE = os.path.join("profiles", "grouped_ffn_switch-base-128.counters.txt")


def load_counter_profile(path=None):
    """Figures that only separate rocprofv3 --pmc runs can give (HBM bytes per launch from FETCH_SIZE /
    WRITE_SIZE, matrix-core busy share and issued / algorithmic MFMA work from the SQ counters), read
    from the committed summary of those runs: its lines `DATA <mode> <kernel> <field> <value>`.
    Returns {(mode, kernel): {field: value}}; empty when the file is missing."""
    path = path or os.path.join(ROOT, COUNTER_PROFILE)
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        p = line.split()
        if len(p) == 5 and p[0] == "DATA":
            out.setdefault((p[1], p[2]), {})[p[3]] = float(p[4])
    return out


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_steps(r, wl, dev, ids_host, steps, warmup, reset_each_step=False):
    import torch
    xs, idss, alphas, ys = ([d[i] for d in dev] for i in range(4))

    def one_step():
        plans = r.plan_all(ids_host)
        r.run(plans, xs, idss, alphas, ys)
        return plans

    for _ in range(warmup):
        one_step()
    r.sync()
    r.ctx.profile_read(reset=True)
    t0 = time.perf_counter()
    plans = None
    for _ in range(steps):
        plans = one_step()
    r.sync()
    dt = time.perf_counter() - t0
    prof = r.ctx.profile_read(reset=True)
    return dt, prof, plans


def kernel_report(wl, prof, steps, n_miss_per_step):
    """Average launch duration and achieved rate per kernel class."""
    d, F, T, L = wl.d_model, wl.d_ff, wl.T, wl.L
    tok = float(L * T * steps)             # tokens processed by each class over the timed region
    out = {}
    for k, (ms, n) in prof.items():
        if n == 0:
            continue
        e = {"launches": int(n), "avg_us": 1e3 * ms / n, "total_ms": ms}
        s = ms * 1e-3
        if k == "sort":
            e["GBps"] = tok * 16 / s / 1e9
        elif k == "gather":
            e["GBps"] = tok * (4 + 4 * d) / s / 1e9
        elif k == "combine":
            e["GBps"] = tok * (8 + 4 * d) / s / 1e9
        elif k in ("gemm1", "gemm2"):
            e["TFLOPs"] = tok * 2 * d * F / s / 1e12
            # bytes the launch must move at least: its experts' matrix once + activations in/out
            w_bytes = n_miss_per_step["active_experts"] * steps * 2 * d * F
            act = tok * (2 * d + 2 * F)
            e["GBps_min_traffic"] = (w_bytes + act) / s / 1e9
            e["bytes_per_launch"] = (w_bytes + act) / n
            e["flops_per_launch"] = tok * 2 * d * F / n
        elif k == "copy":
            e["GBps"] = n_miss_per_step["loads"] * steps * 4 * d * F / s / 1e9
        out[k] = e
    return out


def cpu_baseline(wl, r, ins, budget_tokens):
    """The oracle as it stands, timed on the host's cores over whole layers until the token budget is used."""
    import oracle
    hw = r.host_weights.numpy()
    done, layers = 0, 0
    t0 = time.perf_counter()
    for l in range(wl.L):
        if done >= budget_tokens:
            break
        x_bits, ids, alpha = ins[l]
        n = min(budget_tokens - done, wl.T)
        blocks = [hw[l * wl.E + e] for e in range(wl.E)]
        oracle.token_counts(ids[:n], wl.E)
        oracle.moe_forward(x_bits[:n], ids[:n], alpha[:n], blocks, wl.d_model, wl.d_ff)
        done += n
        layers += 1
    dt = time.perf_counter() - t0
    return {"value": done / dt, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{done} tokens = the first {layers} layer(s) of {wl.name} (grouping + Eq. 1 per token), {dt:.1f} s"}


def serve_leg(wl, hw, S, W, policy, look, n_batches, warm, T_b):
    """Algorithm 1 in full on a stream of small batches: a producer thread pushes hash tables, the
    main thread pops, plans and runs them; the slot pool persists across batches.  Steady state:
    the first `warm` batches fill the pool and are not timed."""
    import threading

    import numpy as np
    import torch
    from paper_2310_18859_amd.runner import MoERunner
    from workloads import gen_batch_ids, gen_gate, gen_x

    r = MoERunner(wl.L, wl.E, wl.d_model, wl.d_ff, S, W, T_b)
    r.host_weights = hw
    base = hw.data_ptr()
    r.ctx.bind_host_weights([base + i * r.expert_bytes for i in range(wl.L * wl.E)], keep=hw)
    r.ctx.set_policy(policy, look)
    tables = [gen_batch_ids(wl, b, T_b) for b in range(n_batches)]
    shared = [r.to_device(gen_x(wl, l, T_b), tables[0][l], gen_gate(wl, l, T_b)) for l in range(wl.L)]
    xs, alphas, ys = [t[0] for t in shared], [t[2] for t in shared], [t[3] for t in shared]
    ids_dev = [[torch.from_numpy(t[l]).to(r.dev) for l in range(wl.L)] for t in tables]
    r.sync()

    def producer():                                   # the hash-building thread: always ahead
        for b, t in enumerate(tables):
            r.push_table(b, t)
        r.ctx.queue_close()

    th = threading.Thread(target=producer)
    th.start()
    th.join()                                         # n_batches <= queue capacity: the look-ahead is always full
    misses = active = 0
    t0 = None
    for b in range(n_batches):
        if b == warm:
            r.sync()
            t0 = time.perf_counter()
        tag, plans = r.serve_next(lambda t: (xs, ids_dev[t], alphas, ys), 1000)
        if b >= warm:
            misses += sum(p.n_miss for p in plans)
            active += sum(p.n_active for p in plans)
    r.sync()
    dt = time.perf_counter() - t0
    timed = n_batches - warm
    r.close()
    return {"policy": policy, "lookahead_batches": look, "pool_slots": S, "wave_experts": W,
            "tokens_per_s": timed * wl.L * T_b / dt, "ms_per_batch": 1e3 * dt / timed,
            "hit_rate": 1.0 - misses / max(active, 1), "expert_loads_per_batch": misses / timed,
            "activated_per_batch": active / timed, "h2d_GBps": misses * wl.expert_bytes / dt / 1e9}


def hash_leg(wl, C=128, seq_len=128):
    """Times sida_hash_forward (Section 3.4.2) with random parameters on 1, 8 and 64 sequences."""
    import numpy as np
    import torch
    from paper_2310_18859_amd.binding import SidaHashConfig, hash_forward, hash_param_count, hash_workspace_bytes
    from workloads import f32_to_bf16_bits

    cfg = SidaHashConfig(wl.d_model, C, wl.L, wl.E, 1, seq_len)
    rng = np.random.default_rng(20231018)
    params = torch.from_numpy((0.1 * rng.standard_normal(hash_param_count(cfg))).astype(np.float32)).cuda()
    st = torch.cuda.Stream()
    rows = []
    for n_seq in (1, 8, 64):
        n = n_seq * seq_len
        x = torch.from_numpy(f32_to_bf16_bits(rng.standard_normal((n, wl.d_model)).astype(np.float32))).cuda()
        ids = torch.empty((wl.L, n, 1), dtype=torch.int32, device="cuda")
        alpha = torch.empty((wl.L, n, 1), dtype=torch.float32, device="cuda")
        ws = torch.empty(hash_workspace_bytes(cfg, n), dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        for timed in (False, True):
            t0 = time.perf_counter()
            for _ in range(20):
                hash_forward(cfg, params, x, n_seq, seq_len, ids, alpha, ws, st)
            st.synchronize()
            dt = (time.perf_counter() - t0) / 20
        rows.append({"sequences": n_seq, "seq_len": seq_len, "ms": 1e3 * dt, "tokens_per_s": n / dt})
    return {"config": {"d": wl.d_model, "C": C, "L": wl.L, "E": wl.E, "top_k": 1}, "rows": rows}


def roofline_of(wl, kern, mode, counters, prefer=None):
    """Roofline entry of the slower grouped GEMM of a run: the binding bound is the one with the larger
    time floor, max(flops / MFMA peak, algorithmic bytes / HBM peak); the other one is reported beside
    it, and what the rocprofv3 counter runs say about the same kernel and mode (when a summary for
    this workload is committed)."""
    if not kern or "gemm1" not in kern or "gemm2" not in kern:
        return None
    k = "gemm1" if kern["gemm1"]["total_ms"] >= kern["gemm2"]["total_ms"] else "gemm2"
    tf, gb = kern[k]["TFLOPs"], kern[k]["GBps_min_traffic"]
    mfma = {"achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS}
    hbm = {"achieved": gb, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gb / HBM_PEAK_GBS}
    bound = prefer or ("hbm" if hbm["frac"] >= mfma["frac"] else "mfma")   # larger fraction = larger floor
    e = {"kernel": f"grouped_gemm_nt ({k}: {'x W_in^T, ReLU' if k == 'gemm1' else 'h W_out^T'})", "bound": bound}
    e.update(hbm if bound == "hbm" else mfma)
    e["avg_launch_us"] = kern[k]["avg_us"]
    e["algorithmic_bytes_per_launch"] = kern[k]["bytes_per_launch"]
    e["algorithmic_flops_per_launch"] = kern[k]["flops_per_launch"]
    e["other_bound"] = dict(mfma if bound == "hbm" else hbm, bound="mfma" if bound == "hbm" else "hbm")
    c = counters.get((mode, k)) if wl.index == 2 and wl.T == 16384 else None
    e["traffic"] = c["fetch_bytes"] + c["write_bytes"] if c and "fetch_bytes" in c else None
    if c:
        e["traffic_source"] = f"{COUNTER_PROFILE} ({mode} {k}: FETCH_SIZE and WRITE_SIZE of separate rocprofv3 --pmc runs, scaled by a plain copy)"
        if "mfma_busy_frac" in c:
            e["mfma_counters"] = {"busy_frac": c["mfma_busy_frac"], "issued_over_algorithmic": c.get("mfma_issued_over_algorithmic"),
                                  "source": COUNTER_PROFILE,
                                  "note": "SQ_VALU_MFMA_BUSY_CYCLES / (4 * SQ_BUSY_CU_CYCLES); SQ_INSTS_VALU_MFMA_MOPS_BF16 * 512 / (2 d F rows)"}
    return e


def measure_workload(wl, hw_cache, steps, warmup, resident_steps, profile, prefetch="auto", copy_cus=-1, extra=None):
    """Streaming (the workload's own pool, when it is smaller than L*E) and resident (a pool of L*E
    slots, filled by a first pass) runs of one workload; the resident run also with separate gather /
    combine passes, which is where their rates come from.  Returns (summary dict, context for extras)."""
    import torch
    from paper_2310_18859_amd.runner import MoERunner
    from workloads import fill_host_weights, gen_gate, gen_ids, gen_x

    counters = load_counter_profile()
    out = {"workload": wl.name, "L": wl.L, "E": wl.E, "d": wl.d_model, "F": wl.d_ff, "T": wl.T,
           "ids": f"zipf(s={wl.zipf_s})" if wl.zipf_s else "uniform", "pool_slots": wl.S, "wave_experts": wl.W}
    log(f"[bench] workload {wl.name}: L={wl.L} E={wl.E} d={wl.d_model} F={wl.d_ff} T={wl.T} S={wl.S} W={wl.W}")
    ins = [(gen_x(wl, l), gen_ids(wl, l), gen_gate(wl, l)) for l in range(wl.L)]
    ids_host = [i[1] for i in ins]
    tokens_per_step = wl.L * wl.T
    streams = wl.S < wl.L * wl.E
    r = MoERunner(wl.L, wl.E, wl.d_model, wl.d_ff, wl.S, wl.W, wl.T, copy_cus=None if copy_cus < 0 else copy_cus)
    t0 = time.perf_counter()
    fill_host_weights(wl, r.alloc_host_weights(), progress=lambda i, n: log(f"[bench] weights {i}/{n}"))
    log(f"[bench] host weights: {wl.L * wl.E * wl.expert_bytes / 1e9:.2f} GB pinned in {time.perf_counter() - t0:.1f} s")
    hw = r.host_weights
    ctx = {"ins": ins, "hw": hw, "runner": r}
    if streams:
        r.ctx.set_prefetch_mode(prefetch)
        dev = [r.to_device(*i) for i in ins]
        r.sync()
        r.ctx.profile_enable(profile)
        dt, prof, plans = time_steps(r, wl, dev, ids_host, steps, warmup)
        loads = sum(p.n_miss for p in plans)
        kern = kernel_report(wl, prof, steps, {"loads": loads, "active_experts": sum(p.n_active for p in plans)})
        h2d = loads * wl.expert_bytes * steps / dt / 1e9
        out["streaming"] = {"tokens_per_s": tokens_per_step * steps / dt, "ms_per_step": 1e3 * dt / steps, "steps": steps,
                            "expert_loads_per_step": loads, "waves_per_step": sum(p.n_waves for p in plans),
                            "h2d": {"achieved": h2d, "peak": H2D_PEAK_GBS, "unit": "GB/s", "frac": h2d / H2D_PEAK_GBS,
                                    "note": "expert bytes copied per step / wall time per step"},
                            "kernels": kern, "roofline": roofline_of(wl, kern, "streaming", counters)}
        log(f"[bench] streaming: {1e3 * dt / steps:.2f} ms/step, {loads} expert loads/step, {h2d:.1f} GB/s host to HBM")
        if extra:
            extra("after_streaming", ctx)
    else:
        if extra:
            extra("after_streaming", ctx)
    r.close()                                                    # also destroys its streams

    # ---- resident: same kernels with every expert already in HBM (pool of L*E slots) -----------
    r2 = MoERunner(wl.L, wl.E, wl.d_model, wl.d_ff, wl.L * wl.E, wl.E, wl.T)
    r2.host_weights = hw
    base = hw.data_ptr()
    r2.ctx.bind_host_weights([base + i * r2.expert_bytes for i in range(wl.L * wl.E)], keep=hw)
    dev2 = [r2.to_device(*i) for i in ins]
    r2.ctx.profile_enable(False)
    time_steps(r2, wl, dev2, ids_host, 1, 1)                     # first pass loads every activated expert
    for mode, fused in (("resident", True), ("resident_separate_passes", False)):
        r2.ctx.set_fusion(fused)
        r2.ctx.profile_enable(profile)
        dt2, prof2, plans2 = time_steps(r2, wl, dev2, ids_host, resident_steps, 2)
        assert sum(p.n_miss for p in plans2) == 0
        kern2 = kernel_report(wl, prof2, resident_steps, {"loads": 0, "active_experts": sum(p.n_active for p in plans2)})
        e = {"tokens_per_s": tokens_per_step * resident_steps / dt2, "ms_per_step": 1e3 * dt2 / resident_steps,
             "steps": resident_steps, "kernels": kern2, "roofline": roofline_of(wl, kern2, mode, counters)}
        if profile:                                              # the same steps without the timing events
            r2.ctx.profile_enable(False)
            dtu, _, _ = time_steps(r2, wl, dev2, ids_host, resident_steps, 2)
            e["ms_per_step_without_timing_events"] = 1e3 * dtu / resident_steps
            e["tokens_per_s_without_timing_events"] = tokens_per_step * resident_steps / dtu
        out[mode] = e
        log(f"[bench] {mode}: {e['ms_per_step']:.3f} ms/step"
            + (f" ({e['ms_per_step_without_timing_events']:.3f} without timing events)" if profile else ""))
    r2.ctx.set_fusion(True)
    ctx["resident_runner"] = r2
    if extra:
        extra("resident", ctx)
    r2.close()
    return out


def brief(w):
    """The per-workload row of the `workloads` array: rates and fractions of peak."""
    row = {k: w[k] for k in ("workload", "L", "E", "d", "F", "T", "ids", "pool_slots", "wave_experts")}
    if "streaming" in w:
        s = w["streaming"]
        row["streaming"] = {"tokens_per_s": s["tokens_per_s"], "ms_per_step": s["ms_per_step"],
                            "h2d_GBps": s["h2d"]["achieved"], "h2d_frac_of_64": s["h2d"]["frac"]}
    res, sep = w["resident"], w["resident_separate_passes"]
    row["resident"] = {"tokens_per_s": res.get("tokens_per_s_without_timing_events", res["tokens_per_s"]),
                       "ms_per_step": res.get("ms_per_step_without_timing_events", res["ms_per_step"])}
    kb = {}
    for g in ("gemm1", "gemm2"):
        k = res["kernels"].get(g)
        if k:
            kb[g] = {"avg_us": k["avg_us"], "hbm_frac": k["GBps_min_traffic"] / HBM_PEAK_GBS, "mfma_frac": k["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS,
                     "GBps": k["GBps_min_traffic"], "TFLOPs": k["TFLOPs"]}
    row["grouped_ffn_resident"] = kb
    for name in ("sort", "gather", "combine"):
        k = sep["kernels"].get(name)
        if k:
            row[name] = {"avg_us": k["avg_us"], "GBps": k["GBps"], "hbm_frac": k["GBps"] / HBM_PEAK_GBS}
    return row


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", type=int, default=2, help="index into workloads.WORKLOADS (2 = Switch-base-128)")
    ap.add_argument("--resident-steps", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket launches with timing events")
    ap.add_argument("--cpu-tokens", type=int, default=0, help="tokens of the oracle sample (0 = four layers, ~10-15 s)")
    ap.add_argument("--only", choices=["all", "main", "large_m"], default="all",
                    help="main: the one workload's streaming and resident runs, none of the other legs; "
                         "large_m: only the grouped FFN on many-token experts (for profiling)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--tokens", type=int, default=0, help="override T of the workload (sweeps; 0 = as defined)")
    ap.add_argument("--zipf", type=float, default=None, help="override the Zipf exponent (0 = uniform ids)")
    ap.add_argument("--copy-cus", type=int, default=-1,
                    help="compute units set aside for the copy stream in the streaming legs (-1: the runner's default)")
    ap.add_argument("--prefetch", choices=["auto", "copy_engine", "kernel"], default="auto")
    ap.add_argument("--serve", choices=["off", "short", "sweep"], default="short",
                    help="stream-of-batches leg: a few pool sizes and policies (short) or the full table (sweep)")
    ap.add_argument("--serve-tokens", type=int, default=128, help="tokens per batch of the stream")
    ap.add_argument("--serve-batches", type=int, default=120)
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (no sharding, no collectives); run with --gpus 1")

    import numpy as np
    import torch
    from paper_2310_18859_amd.runner import MoERunner
    from workloads import WORKLOADS, fill_host_weights, gen_gate, gen_ids, gen_x

    wl = WORKLOADS[a.workload]
    if a.tokens:
        wl = wl.scaled(T=a.tokens, name=f"{wl.name}-T{a.tokens}")
    if a.zipf is not None:
        wl = wl.scaled(zipf_s=(a.zipf or None), name=f"{wl.name}-zipf{a.zipf}")
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    full = a.only == "all" and not a.tokens and a.zipf is None
    profile = not a.no_profile
    legs = {}

    if a.calibrate_copy:                     # a plain copy kernel of known size: 1 GiB read, 1 GiB written
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(7)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def extra(stage, ctx):
        """Legs that reuse the main workload's pinned weights."""
        if stage == "after_streaming" and not a.no_cpu_baseline:
            n = a.cpu_tokens or min(wl.L, 4) * wl.T
            log(f"[bench] timing the CPU oracle on {n} tokens ...")
            legs["cpu"] = cpu_baseline(wl, ctx["runner"], ctx["ins"], n)
            log(f"[bench] oracle: {legs['cpu']['value']:.1f} tokens/s on {legs['cpu']['cores']} threads")
        if stage == "resident" and full:
            # k = 3 experts per token (the paper's setting on two of its datasets): T / 3 tokens, so the
            # grouped GEMMs see the same number of rows; the combine adds a token's three rows
            r2, k = ctx["resident_runner"], 3
            tok = wl.T // k
            r2.ctx.set_top_k(k)
            ins_k = [(gen_x(wl, l, tok), gen_ids(wl, l, tok * k), gen_gate(wl, l, tok * k)) for l in range(wl.L)]
            dev_k = [r2.to_device(*i) for i in ins_k]
            ids_k = [i[1] for i in ins_k]
            wl_k = wl.scaled(T=tok * k)
            top_k = {"experts_per_token": k, "tokens": tok}
            for fused in (False, True):
                r2.ctx.set_fusion(fused)
                r2.ctx.profile_enable(False)
                time_steps(r2, wl_k, dev_k, ids_k, 1, 1)         # may activate experts the top-1 ids did not
                dtk, _, plans_k = time_steps(r2, wl_k, dev_k, ids_k, a.resident_steps, 2)
                assert sum(p.n_miss for p in plans_k) == 0
                top_k["fused_gather" if fused else "separate"] = {
                    "ms_per_step": 1e3 * dtk / a.resident_steps,
                    "tokens_per_s": wl.L * tok * a.resident_steps / dtk,
                    "expert_rows_per_s": wl.L * tok * k * a.resident_steps / dtk}
            log(f"[bench] resident, 3 experts per token ({tok} tokens): "
                f"{top_k['separate']['ms_per_step']:.3f} ms/step, gather folded in: {top_k['fused_gather']['ms_per_step']:.3f}")
            legs["top_k"] = top_k
            r2.ctx.set_top_k(1)
            r2.ctx.set_fusion(True)
            # ---- the cross-batch serving loop (Algorithm 1 in full) on sentence-sized batches
            if a.serve != "off" and wl.L * wl.E > wl.S:
                hw = ctx["hw"]
                LE = wl.L * wl.E
                sizes = [LE // 8, LE // 4, LE // 2] if a.serve == "short" else [LE // 16, LE // 8, LE // 4, 3 * LE // 8, LE // 2, 3 * LE // 4, LE]
                rows = []
                for S in sizes:
                    for policy, look in (("fifo", 0), ("lru", 0), ("belady", 8)):
                        W = max(1, min(wl.E, S // 2))
                        row = serve_leg(wl, hw, S, W, policy, look, a.serve_batches, a.serve_batches // 3, a.serve_tokens)
                        rows.append(row)
                        log(f"[bench] serve S={S} {policy}: {row['tokens_per_s']:.3e} tok/s, hit rate {row['hit_rate']:.3f}, "
                            f"{row['expert_loads_per_batch']:.1f} loads/batch")
                legs["serving"] = {"workload": f"{wl.name}: stream of {a.serve_batches} batches of {a.serve_tokens} tokens, "
                                               f"first {a.serve_batches // 3} untimed", "rows": rows}

    main_w = None
    if a.only != "large_m":
        main_w = measure_workload(wl, None, a.steps, a.warmup, a.resident_steps, profile, a.prefetch, a.copy_cus, extra)

    # ---- K-b on many-token experts alone (every expert far above the MFMA/HBM ridge) ---------
    if full or a.only == "large_m":
        wt = WORKLOADS[0].scaled(d_model=wl.d_model, d_ff=wl.d_ff, T=16384, name=f"{WORKLOADS[0].name}-T16384")
        r3 = MoERunner(wt.L, wt.E, wt.d_model, wt.d_ff, wt.L * wt.E, wt.E, wt.T)
        fill_host_weights(wt, r3.alloc_host_weights())
        ins3 = [(gen_x(wt, l), gen_ids(wt, l), gen_gate(wt, l)) for l in range(wt.L)]
        dev3 = [r3.to_device(*i) for i in ins3]
        ids3 = [i[1] for i in ins3]
        r3.ctx.set_fusion(False)
        r3.ctx.profile_enable(False)
        time_steps(r3, wt, dev3, ids3, 1, 1)
        r3.ctx.profile_enable(profile)
        dt3, prof3, plans3 = time_steps(r3, wt, dev3, ids3, a.resident_steps, 2)
        kern3 = kernel_report(wt, prof3, a.resident_steps, {"loads": 0, "active_experts": sum(p.n_active for p in plans3)})
        legs["kb_large_m"] = {"workload": wt.name, "rows_per_expert": wt.T // wt.E,
                              "kernels": {k: kern3[k] for k in ("gemm1", "gemm2") if k in kern3},
                              "roofline": roofline_of(wt, kern3, "resident", {}, prefer="mfma")}
        r3.close()
        if "gemm1" in kern3:
            log(f"[bench] large-M experts alone: gemm1 {kern3['gemm1']['avg_us']:.1f} us, gemm2 {kern3['gemm2']['avg_us']:.1f} us")
    if a.only == "large_m":
        print(json.dumps({"kb_large_m": legs["kb_large_m"]}), flush=True)
        return
    if full:
        # ---- the hash function's forward pass (predicts the ids / alpha table of a batch)
        legs["hash_fn"] = hash_leg(wl)
        log("[bench] hash function: " + ", ".join(f"{r['sequences']} x {r['seq_len']} tokens {r['ms']:.3f} ms" for r in legs["hash_fn"]["rows"]))

    # ---- the other four configurations: streaming and resident rates, fractions of peak --------
    rows = {wl.index: brief(main_w)}
    if full:
        for other in WORKLOADS:
            if other.index == wl.index:
                continue
            big = other.L * other.E * other.expert_bytes > 10e9
            w = measure_workload(other, None, 2 if big else 3, 1, 20, profile)
            rows[other.index] = brief(w)

    main_mode = "streaming" if "streaming" in main_w else "resident"
    main = main_w[main_mode]
    line = {
        "metric": "moe_layer_tokens_per_sec",
        "value": main["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": main["steps"], "warmup": a.warmup,
        "ms_per_step": main["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "L": wl.L, "E": wl.E, "d": wl.d_model, "F": wl.d_ff,
                   "T": wl.T, "ids": f"zipf(s={wl.zipf_s})" if wl.zipf_s else "uniform",
                   "pool_slots": wl.S if main_mode == "streaming" else wl.L * wl.E,
                   "wave_experts": wl.W if main_mode == "streaming" else wl.E, "mode": main_mode,
                   "dispatch_combine": "folded into the grouped GEMMs (the library's default)"},
    }
    roof = dict(main["roofline"]) if main.get("roofline") else None
    if roof and main_mode == "streaming":
        # what binds the timed step is not this kernel but the host link the experts stream over
        copy = main["kernels"].get("copy")
        total_kernel_ms = sum(k["total_ms"] for k in main["kernels"].values())
        h2d = main["h2d"]
        roof["step_bound"] = {"kernel": "copy_experts (expert prefetch, pinned host memory -> pool slots)", "bound": "host_link",
                              "achieved": h2d["achieved"], "peak": h2d["peak"], "unit": "GB/s", "frac": h2d["frac"],
                              "share_of_kernel_time": (copy["total_ms"] / total_kernel_ms) if copy and total_kernel_ms else None,
                              "note": "the grouped GEMMs of a wave run hidden behind the next wave's copies; "
                                      "their quality shows in the resident run"}
        roof["resident"] = main_w["resident"]["roofline"]
    line["roofline"] = roof
    line["cpu_baseline"] = legs.get("cpu")
    for mode in ("streaming", "resident", "resident_separate_passes"):
        if mode in main_w:
            line[mode] = main_w[mode]
    for k in ("top_k", "hash_fn", "serving", "kb_large_m"):
        if k in legs:
            line[k] = legs[k]
    line["workloads"] = [rows[i] for i in sorted(rows)]
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
