#!/usr/bin/env python3
"""Benchmark of the ChunkWise LoRA hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: score_tokens -> partition_chunks -> select_ranks -> chunkwise_lora_linear
(packed weights).  Prints ONE JSON line.  Besides the headline tokens/s it reports the roofline
position of the dominant kernel (the main MFMA GEMM, timed with HIP events around its launches
inside the timed region), the scoring kernel's HBM rate, the same linear at fixed r_max and at
rank 0, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--spin-up", type=int, default=64,
                    help="untimed whole-path steps before the warm-up steps.  After its first few launches out of "
                         "idle the part drops its clocks for some 25 launches (~15 ms) before settling; these steps "
                         "take the run past that, so that the timed region measures the sustained rate")
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--proj", type=int, default=0)
    ap.add_argument("--group-rows", type=int, default=0)
    ap.add_argument("--form", choices=("two_phase", "calls"), default="two_phase",
                    help="two_phase (default): score_tokens, cwl_schedule_chunks (chunker + selector in one call, "
                         "with x A riding in the chunker's launch), cwl_chunkwise_lora_linear_packed_shrunk (gate + "
                         "main GEMM): five launches.  calls: the four calls of the boundary one after the other "
                         "(seven launches).  Same results bit for bit; --group-rows 1 needs 'calls'")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-variants", action="store_true")
    ap.add_argument("--all-projections", action="store_true",
                    help="also time the linear of every projection of the workload (own x, W, A, B; the same "
                         "chunk table) and report the sum")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the compact block on the other bf16 workloads (cfg2, cfg3 with all seven projections "
                         "on one chunk table, cfg4)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-size kernel to scale "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings against)")
    return ap.parse_args()


def read_traffic(tag):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a
    plain copy of known size), from the committed summary profiles/pmc_traffic_<tag>.txt."""
    out = {}
    path = os.path.join(ROOT, "profiles", f"pmc_traffic_{tag}.txt")
    if os.path.exists(path):
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch."):
                key, val = line.split(":", 1)
                out[key.split(".", 1)[1].strip()] = float(val.split()[0])
    return out


def tail_stage_ratio(r_eff, r_max, rows=256, step=64):
    """Adapter stages the main GEMM's row tiles run (token order), over what they run at fixed r_max."""
    import numpy as np
    n = len(r_eff)
    pad = (-n) % rows
    r = np.concatenate([r_eff, np.zeros(pad, dtype=r_eff.dtype)]).reshape(-1, rows).max(axis=1)
    run = np.ceil(r / step).sum()
    full = np.ceil(r_max / step) * len(r)
    return float(run / full) if full else 1.0


def other_workload(name, steps, warmup):
    """Compact figures of one of the other bf16 workloads: one whole step = score_tokens, partition_chunks,
    select_ranks once and the linear of EVERY projection of the workload on that one chunk table (own x, W, A,
    B each, weights prepacked).  Returns step time, the scoring kernel's HBM rate and, per projection, the whole
    call and its main GEMM against the bf16 MFMA peak."""
    import numpy as np
    import torch
    from paper_2601_21109_amd import binding as B
    from paper_2601_21109_amd import workloads as W
    dev = "cuda:0"
    wl = W.WORKLOADS[name]
    N, K = wl.n_rows, len(wl.ladder)
    so = W.seq_offsets(wl)
    sod = torch.from_numpy(so).to(dev)
    h = torch.empty(N, dtype=torch.float32, device=dev)
    tile = wl.logit_tile_rows or N
    n_tiles = N // tile
    sig = W.token_sigmas(wl)
    for t in range(n_tiles):                        # scores of the real logits, tile by tile through one buffer
        logits = W.logits_rows(wl, t * tile, (t + 1) * tile, dev, sigmas=sig)
        B.score_tokens(logits, out=h[t * tile:(t + 1) * tile])
    h_sink = torch.empty(tile, dtype=torch.float32, device=dev)
    table = B.partition_chunks(h, sod, wl.l_min, wl.l_max, wl.theta(), wl.delta())
    ri = B.select_ranks(table, wl.taus(), K)
    projs = []
    for p_i, (p_name, p_in, p_out) in enumerate(wl.projections):
        xp, Wp, Ap, Bp = W.linear_operands(wl, p_i, dev)
        pk = B.prepack_weights(Wp, Ap, Bp)
        del Wp, Ap, Bp
        projs.append((p_name, p_in, p_out, xp, pk, torch.empty((N, p_out), dtype=wl.dtype, device=dev),
                      B.linear_workspace((N, p_in), wl.dtype, p_out, wl.r_max, wl.ladder, wl.scales, wl.blend_w, dev)))
    torch.cuda.synchronize()

    def linear(pr):
        B.chunkwise_lora_linear(pr[3], pr[4], None, None, wl.ladder, wl.scales, wl.blend_w, sod, table, ri,
                                out=pr[5], workspace=pr[6])

    def step():
        for t in range(n_tiles):                    # with tiles: the last tile's buffer stands in for all of them
            B.score_tokens(logits, out=h_sink if n_tiles > 1 else h)
        B.partition_chunks(h, sod, wl.l_min, wl.l_max, wl.theta(), wl.delta(), out=table)
        B.select_ranks(table, wl.taus(), K, out=ri)
        for pr in projs:
            linear(pr)

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ms_step = timed(step, steps)
    # effective ranks of the rows, for the algorithmic flops
    n_chunks = int(table["chunk_offsets"][-1].item())
    cl = table["chunk_len"][:n_chunks].cpu().numpy()
    cs = table["chunk_start"][:n_chunks].cpu().numpy()
    co = table["chunk_offsets"].cpu().numpy()
    rk = np.asarray(wl.ladder)[ri[:n_chunks].cpu().numpy()]
    r_sum = 0.0
    for b in range(wl.n_seqs):
        for c in range(co[b], co[b + 1]):
            r_sum += float(rk[c]) * float(cl[c])
            if c > co[b] and wl.blend_w:
                r_sum += float(max(rk[c], rk[c - 1]) - rk[c]) * float(min(wl.blend_w, cl[c]))
    B.profile_enable((B.PROF_SCORE,))
    for _ in range(steps):
        for t in range(n_tiles):
            B.score_tokens(logits, out=h_sink if n_tiles > 1 else h)
    torch.cuda.synchronize()
    t_s, n_s = B.profile_read(B.PROF_SCORE)
    B.profile_enable(False)
    score_ms = t_s / max(n_s, 1)
    score_gbs = tile * (wl.vocab * 2 + 4.0) / (score_ms * 1e-3) / 1e9
    calls, fl_all, ms_all = {}, 0.0, 0.0
    for pr in projs:
        p_name, p_in, p_out = pr[0], pr[1], pr[2]
        call_ms = timed(lambda: linear(pr), max(steps // 2, 2))
        B.profile_enable((B.PROF_MAIN,))
        for _ in range(max(steps // 2, 2)):
            linear(pr)
        torch.cuda.synchronize()
        t_m, n_m = B.profile_read(B.PROF_MAIN)
        B.profile_enable(False)
        main_ms = t_m / max(n_m, 1)
        fl_call = 2.0 * N * p_in * p_out + 2.0 * r_sum * (p_in + p_out)
        fl_main = 2.0 * N * p_in * p_out + 2.0 * r_sum * p_out
        calls[p_name if p_name not in calls else f"{p_name}_{len(calls)}"] = {
            "d_in": p_in, "d_out": p_out, "call_ms": call_ms,
            "call_frac_of_bf16_peak": fl_call / (call_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "main_ms": main_ms, "main_frac_of_bf16_peak": fl_main / (main_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        fl_all += fl_call
        ms_all += call_ms
    # the first projection at fixed r_max (one rung, every chunk on it) next to its chunk-wise call, in
    # interleaved blocks so that clock drift hits both alike
    pr0 = projs[0]
    zero_idx = torch.zeros(max(n_chunks, 1), dtype=torch.int32, device=dev)

    def linear_fixed():
        B.chunkwise_lora_linear(pr0[3], pr0[4], None, None, [wl.r_max], [wl.alpha / wl.r_max], wl.blend_w, sod, table,
                                zero_idx, out=pr0[5], workspace=pr0[6])
    linear_fixed()
    torch.cuda.synchronize()
    t_cw = t_fx = 0.0
    n_blk = max(steps // 2, 2)
    for _ in range(3):
        t_cw += timed(lambda: linear(pr0), n_blk)
        t_fx += timed(linear_fixed, n_blk)
    fixed = {"projection": pr0[0], "chunkwise_ms": t_cw / 3, "fixed_r_max_ms": t_fx / 3,
             "speedup_vs_fixed_r_max": t_fx / t_cw,
             "adapter_stage_share_of_main": ((wl.r_max + 63) // 64 * 64) / (pr0[1] + (wl.r_max + 63) // 64 * 64)}
    # the projections that read the same activations (q/k/v; gate/up) as grouped calls: one gate table and one
    # shrink pass over x per group, every projection still on its own rungs
    grouped = None
    names = [pr[0] for pr in projs]
    groups = [g for g in (["q_proj", "k_proj", "v_proj"], ["gate_proj", "up_proj"], ["up_proj", "gate_proj"])
              if all(n in names for n in g)]
    if groups:
        groups = groups[:2] if len(groups) > 2 else groups
        seen, calls_g = set(), []
        for g in groups:
            if seen & set(g):
                continue
            seen |= set(g)
            idx = [names.index(n) for n in g]
            ops = [W.linear_operands(wl, i, dev) for i in idx]
            pg = B.prepack_weights_grouped([o[1] for o in ops], [o[2] for o in ops], [o[3] for o in ops])
            del ops
            xg = projs[idx[0]][3]                  # the group reads the activations of its first projection
            yg = torch.empty((N, pg.d_out), dtype=wl.dtype, device=dev)
            wsg = B.grouped_workspace(N, pg, wl.ladder, wl.scales, wl.blend_w, dev)
            calls_g.append((g, idx, pg, xg, yg, wsg))
        rest = [pr for i, pr in enumerate(projs) if names[i] not in seen]

        def step_grouped():
            for t in range(n_tiles):
                B.score_tokens(logits, out=h_sink if n_tiles > 1 else h)
            B.partition_chunks(h, sod, wl.l_min, wl.l_max, wl.theta(), wl.delta(), out=table)
            B.select_ranks(table, wl.taus(), K, out=ri)
            for _, _, pg, xg, yg, wsg in calls_g:
                B.chunkwise_lora_linear_grouped(xg, pg, wl.ladder, wl.scales, wl.blend_w, sod, table, ri, out=yg,
                                                workspace=wsg)
            for pr in rest:
                linear(pr)

        step_grouped()
        torch.cuda.synchronize()
        ms_g = timed(step_grouped, steps)
        grouped = {"groups": ["+".join(g) for g, *_ in calls_g], "step_ms": ms_g,
                   "tokens_per_s": N / (ms_g * 1e-3),
                   "group_call_ms": {"+".join(g): timed(lambda pg=pg, xg=xg, yg=yg, wsg=wsg: B.chunkwise_lora_linear_grouped(
                       xg, pg, wl.ladder, wl.scales, wl.blend_w, sod, table, ri, out=yg, workspace=wsg), max(steps // 2, 2))
                       for g, _, pg, xg, yg, wsg in calls_g},
                   "separate_calls_ms": {"+".join(g): sum(calls[names[i]]["call_ms"] for i in idx)
                                         for g, idx, *_ in calls_g}}
        del calls_g
    out = {"n_rows": N, "vocab": wl.vocab, "ladder": wl.ladder, "chunks": n_chunks, "mean_r_eff": r_sum / N,
           "steps": steps, "step_ms": ms_step, "tokens_per_s": N / (ms_step * 1e-3),
           "score": {"ms_per_launch": score_ms, "launches_per_step": n_tiles, "GBps": score_gbs,
                     "frac_of_hbm_peak": score_gbs / PEAK_HBM_GBS},
           "linear_calls": calls,
           "all_calls_frac_of_bf16_peak": fl_all / (ms_all * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           "first_projection_vs_fixed_r_max": fixed}
    if grouped:
        out["with_grouped_calls"] = grouped
    del projs, logits
    torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2601_21109_amd import binding as B
    from paper_2601_21109_amd import workloads as W

    dev = "cuda:0"
    wl = W.WORKLOADS[args.workload]
    pname, d_in, d_out = wl.projections[args.proj]
    N, K = wl.n_rows, len(wl.ladder)
    bf16 = wl.dtype == torch.bfloat16

    # ---- resident inputs --------------------------------------------------------------------
    so = W.seq_offsets(wl)
    sod = torch.from_numpy(so).to(dev)
    logits = W.logits(wl, dev)
    x, Wm, A, Bm = W.linear_operands(wl, args.proj, dev)
    packed = B.prepack_weights(Wm, A, Bm)          # static weights: re-laid out once, untimed
    y = torch.empty((N, d_out), dtype=wl.dtype, device=dev)
    h = torch.empty(N, dtype=torch.float32, device=dev)
    ws = B.linear_workspace((N, d_in), wl.dtype, d_out, wl.r_max, wl.ladder, wl.scales, wl.blend_w, dev)
    table = B.partition_chunks(B.score_tokens(logits, out=h), sod, wl.l_min, wl.l_max, wl.theta(), wl.delta())
    ri = B.select_ranks(table, wl.taus(), K)
    torch.cuda.synchronize()

    def step_calls():
        B.score_tokens(logits, out=h)
        B.partition_chunks(h, sod, wl.l_min, wl.l_max, wl.theta(), wl.delta(), out=table)
        B.select_ranks(table, wl.taus(), K, out=ri)
        B.chunkwise_lora_linear(x, packed, None, None, wl.ladder, wl.scales, wl.blend_w, sod, table, ri,
                                out=y, group_rows=args.group_rows, workspace=ws)

    two_phase = args.form == "two_phase" and args.group_rows == 0
    u = B.lora_shrink(x, packed, wl.ladder, wl.scales, wl.blend_w) if two_phase else None

    def step_two_phase():
        # x A needs no chunk table: it rides in the chunker's launch, whose chain of look-ups occupies one
        # wavefront per sequence; the linear call is then the gate on that product and the main GEMM
        B.score_tokens(logits, out=h)
        B.schedule_chunks(h, sod, wl.l_min, wl.l_max, wl.theta(), wl.delta(), wl.taus(), K, out=table, rank_idx=ri,
                          shrink=(x, packed, wl.ladder, wl.scales, wl.blend_w, u))
        B.chunkwise_lora_linear_shrunk(x, packed, u, wl.ladder, wl.scales, wl.blend_w, sod, table, ri, out=y,
                                       workspace=ws)

    step = step_two_phase if two_phase else step_calls

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        return max(e0.elapsed_time(e1), 0.0) / steps, wall / steps

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)              # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region: K whole-path steps ---------------------------------------------------
    # HIP events are recorded on the launch stream around the two kernels whose rooflines are
    # reported (the main GEMM and score_tokens).  Every event record leaves the stream idle for a
    # few microseconds, so the other kernels are timed in a second pass of K steps right after.
    slots = (("score", B.PROF_SCORE), ("partition", B.PROF_PARTITION), ("select", B.PROF_SELECT),
             ("meta", B.PROF_META), ("shrink", B.PROF_SHRINK), ("main", B.PROF_MAIN))
    # first exactly what the flags say, out of idle: W warm-up steps, K timed steps (reported as
    # "first_pass"); then the spin-up steps and the sustained measurement that the headline uses
    first_ms, _ = timed(step, args.steps, args.warmup)
    for _ in range(max(args.spin_up, 0)):
        step()
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.profile_enable((B.PROF_MAIN, B.PROF_SCORE))
    ms_step, ms_wall = timed(step, args.steps, 0)
    timed_prof = {name: B.profile_read(slot) for name, slot in slots if name in ("main", "score")}
    B.profile_enable(True)
    timed(step, args.steps, 0)
    prof = {name: B.profile_read(slot) for name, slot in slots}
    B.profile_enable(False)
    ms_step = max(ms_step, ms_wall) if ms_step <= 0 else ms_step
    kern_ms = {k: (v[0] / v[1] if v[1] else None) for k, v in prof.items()}
    breakdown_ms = dict(kern_ms)                      # all six, from the second pass
    for k, v in timed_prof.items():                   # the roofline kernels: from the timed region
        if v[1]:
            kern_ms[k] = v[0] / v[1]
    # the other form of the step, same region length, and its kernels (the one-call linear is what the
    # whole-call roofline figure is stated on)
    ms_calls, calls_ms = None, None
    if two_phase and not args.no_variants:
        for _ in range(args.warmup):
            step_calls()
        torch.cuda.synchronize()
        ms_calls, _ = timed(step_calls, args.steps, 0)
        B.profile_enable((B.PROF_MAIN,))
        timed(step_calls, args.steps, 0)
        main_calls = B.profile_read(B.PROF_MAIN)
        B.profile_enable(True)
        timed(step_calls, args.steps, 0)
        calls_prof = {name: B.profile_read(slot) for name, slot in slots}
        B.profile_enable(False)
        calls_ms = {k: (v[0] / v[1] if v[1] else None) for k, v in calls_prof.items()}
        if main_calls[1]:
            calls_ms["main"] = main_calls[0] / main_calls[1]

    # ---- chunk statistics and algorithmic work --------------------------------------------------
    n_chunks = int(table["chunk_offsets"][-1].item())
    cl = table["chunk_len"][:n_chunks].cpu().numpy()
    cs = table["chunk_start"][:n_chunks].cpu().numpy()
    co = table["chunk_offsets"].cpu().numpy()
    rk = np.asarray(wl.ladder)[ri[:n_chunks].cpu().numpy()]
    r_eff = np.zeros(N, dtype=np.int64)
    for b in range(wl.n_seqs):
        for c in range(co[b], co[b + 1]):
            r_eff[cs[c]:cs[c] + cl[c]] = rk[c]
            if c > co[b] and wl.blend_w:
                w = min(wl.blend_w, cl[c])
                r_eff[cs[c]:cs[c] + w] = max(rk[c], rk[c - 1])
    flops_base = 2.0 * N * d_in * d_out
    flops_alg = flops_base + 2.0 * float(r_eff.sum()) * (d_in + d_out)     # whole linear
    flops_main = flops_base + 2.0 * float(r_eff.sum()) * d_out             # what the main kernel runs
    flops_fixed = flops_base + 2.0 * N * wl.r_max * (d_in + d_out)
    esz = 2 if bf16 else 4

    out = {
        "metric": "chunkwise_lora_hot_path_tokens_per_s",
        "value": N / (ms_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "spin_up_steps": max(args.spin_up, 0),
        "ms_per_step": ms_step,
        "first_pass": {"note": "the same K steps after the W warm-up steps only, straight out of idle (inside the "
                               "clock dip that follows the first launches); the headline is measured after "
                               "spin_up_steps more untimed steps",
                       "ms_per_step": first_ms, "value": N / (first_ms * 1e-3)},
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}:{pname}", "n_rows": N, "n_seqs": wl.n_seqs,
                   "seq_len": wl.seq_len, "vocab": wl.vocab, "d_in": d_in, "d_out": d_out,
                   "ladder": wl.ladder, "l_min": wl.l_min, "l_max": wl.l_max, "blend_w": wl.blend_w,
                   "group_rows": args.group_rows, "weights": "prepacked"},
        "form": ("two_phase: score_tokens, schedule_chunks (chunker + x A in one launch, compact + selector in a "
                 "second), chunkwise_lora_linear_packed_shrunk (gate, main GEMM): 5 launches" if two_phase else
                 "calls: score_tokens, partition_chunks, select_ranks, chunkwise_lora_linear_packed: 7 launches"),
        "kernel_ms": kern_ms,
        "kernel_ms_note": "main and score: HIP events in the timed region; the rest: a second pass of the same "
                          "steps with events around every kernel" + (
                              "; two_phase form: 'partition' = the chunker's launch with x A in it + compact/selector, "
                              "'meta' = the gate kernel, 'shrink' and 'select' have no launch of their own" if two_phase else ""),
        "kernel_ms_all_events_pass": breakdown_ms,
        "chunks": {"count": n_chunks, "mean_len": float(cl.mean()) if n_chunks else 0.0,
                   "tokens_by_rank": {str(r): int(cl[rk == r].sum()) for r in wl.ladder},
                   "mean_r_eff": float(r_eff.mean())},
    }
    traffic = read_traffic(f"{wl.name}_{pname}")
    if kern_ms["main"]:
        ach = flops_main / (kern_ms["main"] * 1e-3) / 1e12
        out["roofline"] = {"kernel": "main_bf16_kernel (x W + uhat B)" if bf16 else "gemm_f32_tn_kernel",
                           "bound": "mfma" if bf16 else "alu", "achieved": ach,
                           "peak": PEAK_BF16_TFLOPS if bf16 else 157.3, "unit": "TFLOP/s",
                           "frac": ach / (PEAK_BF16_TFLOPS if bf16 else 157.3), "traffic": traffic.get("main"),
                           "avg_launch_ms": kern_ms["main"], "flops_per_launch": flops_main}
    if kern_ms["score"]:
        bytes_score = N * (wl.vocab * esz + 4.0)
        gbs = bytes_score / (kern_ms["score"] * 1e-3) / 1e9
        out["roofline_score_tokens"] = {"kernel": "score_tokens_kernel", "bound": "hbm", "achieved": gbs,
                                        "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                                        "traffic": traffic.get("score"), "avg_launch_ms": kern_ms["score"],
                                        "bytes_per_launch": bytes_score}
    if calls_ms is not None:
        out["calls_form"] = {"note": "the same step as the four calls of the boundary one after the other "
                                     "(7 launches), same run", "ms_per_step": ms_calls,
                             "value": N / (ms_calls * 1e-3), "kernel_ms": calls_ms}
    lin_src = calls_ms if two_phase else kern_ms
    lin_ms = sum(lin_src[k] or 0.0 for k in ("meta", "shrink", "main")) if lin_src is not None else 0.0
    if lin_ms and "roofline" in out and bf16:
        # the benchmark spec's target is stated for the whole call: gate table + shrink + main GEMM, priced with
        # the whole layer's algorithmic flops
        out["roofline"]["whole_call"] = {"kernels": "token_meta + shrink + main", "ms": lin_ms,
                                         "flops": flops_alg, "achieved": flops_alg / (lin_ms * 1e-3) / 1e12,
                                         "frac": flops_alg / (lin_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        if two_phase and calls_ms is not None and kern_ms["meta"] and kern_ms["main"]:
            ms2 = kern_ms["meta"] + kern_ms["main"]
            sched_alone = sum(calls_ms[k] or 0.0 for k in ("partition", "select"))
            out["roofline"]["two_phase"] = {
                "note": "the layer as cwl_lora_shrink_packed + cwl_chunkwise_lora_linear_packed_shrunk: x A runs in "
                        "the chunker's launch, what is left on the step's critical path is the gate kernel and the "
                        "main GEMM; 'frac' prices the whole layer's flops against that time plus what the chunker's "
                        "launch grew by",
                "second_phase_ms": ms2,
                "schedule_with_product_ms": kern_ms["partition"],
                "schedule_alone_ms": sched_alone,
                "added_to_schedule_ms": max((kern_ms["partition"] or 0.0) - sched_alone, 0.0),
                "flops": flops_alg,
                "frac": flops_alg / ((ms2 + max((kern_ms["partition"] or 0.0) - sched_alone, 0.0)) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                "frac_second_phase_alone": flops_alg / (ms2 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    out["linear"] = {"ms": lin_ms, "tokens_per_s": N / (lin_ms * 1e-3) if lin_ms else None,
                     "effective_tflops": flops_alg / (lin_ms * 1e-3) / 1e12 if lin_ms else None,
                     "frac_of_bf16_peak": flops_alg / (lin_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS if lin_ms else None}

    # ---- same kernels at fixed r_max and at rank 0 (launches interleaved so that clock and
    #      temperature drift hit the three variants alike) ----------------------------------------
    if not args.no_variants:
        zero_idx = torch.zeros(max(n_chunks, 1), dtype=torch.int32, device=dev)

        def make(ranks, scales, rid, group_rows=args.group_rows):
            return lambda: B.chunkwise_lora_linear(x, packed, None, None, ranks, scales, wl.blend_w, sod,
                                                   table, rid, out=y, group_rows=group_rows,
                                                   workspace=ws)
        fns = {"chunkwise": make(wl.ladder, wl.scales, ri),
               "fixed_r_max": make([wl.r_max], [wl.alpha / wl.r_max], zero_idx),
               "rank_0": make([0], [0.0], zero_idx),
               # the other setting of group_rows: rows sorted by effective rank before the GEMMs
               "chunkwise_other_group_rows": make(wl.ladder, wl.scales, ri, 1 - args.group_rows)}
        for fn in fns.values():
            for _ in range(args.warmup):
                fn()
        torch.cuda.synchronize()
        tot = {k: 0.0 for k in fns}
        block = 5
        rounds = max(1, args.steps // block)
        for _ in range(rounds):
            for k, fn in fns.items():
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(block):
                    fn()
                e1.record()
                e1.synchronize()
                tot[k] += e0.elapsed_time(e1)
        ms_v = {k: v / (rounds * block) for k, v in tot.items()}
        out["linear_variants"] = {
            "chunkwise": {"ms": ms_v["chunkwise"], "effective_tflops": flops_alg / ms_v["chunkwise"] / 1e9},
            "fixed_r_max": {"ms": ms_v["fixed_r_max"], "effective_tflops": flops_fixed / ms_v["fixed_r_max"] / 1e9},
            "rank_0": {"ms": ms_v["rank_0"], "effective_tflops": flops_base / ms_v["rank_0"] / 1e9},
            "speedup_vs_fixed_r_max": ms_v["fixed_r_max"] / ms_v["chunkwise"],
            "group_rows_%d" % (1 - args.group_rows): {"ms": ms_v["chunkwise_other_group_rows"],
                                                      "effective_tflops": flops_alg / ms_v["chunkwise_other_group_rows"] / 1e9},
            # what skipping can save at most: the share of the main GEMM's reduction stages that belong
            # to the adapter part, and the share of those that the tiles' largest ranks leave out
            "adapter_stage_share_of_main": ((wl.r_max + 63) // 64 * 64) / (d_in + (wl.r_max + 63) // 64 * 64),
            "adapter_stages_run_over_fixed_r_max": tail_stage_ratio(r_eff, wl.r_max),
            "note": "the main GEMM walks ceil(r_tile / 64) adapter stages per 256-row tile (r_tile = largest "
                    "effective rank in the tile) after d_in / 64 base stages, so what rank skipping can save "
                    "of the main GEMM is adapter_stage_share_of_main x (1 - adapter_stages_run_over_fixed_r_max); "
                    "tiles are assigned to compute units statically, so the unit whose tiles skip least sets the kernel time",
            "lora_flop_share_at_r_max": wl.r_max * (d_in + d_out) / (d_in * d_out),
        }

    # ---- the same projection on a few rows (decode steps, short prompts): bound by streaming the
    #      weights once; the two kernels of that path are timed with their event pairs -----------
    if not args.no_variants and bf16:
        few = {}
        R_pad = (max(wl.r_max, 1) + 63) // 64 * 64
        w_bytes = 2.0 * d_in * (d_out + R_pad)

        def graph_call_us(fn, reps=10):
            """microseconds per call of fn, ten calls recorded into a HIP graph and replayed (no event pairs between
            the kernels: for launches of a few microseconds an event pair costs as much as the kernel)"""
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                fn()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                for _ in range(reps):
                    fn()
            gr.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                gr.replay()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / (args.steps * reps) * 1e3

        for rows in (1, 8, 64, 512):
            tb = W.random_chunk_table(1, [rows], min(wl.l_min, rows), max(min(wl.l_max, rows), 1), K, 11)
            sod_f, tab_f, rid_f = B.table_from_host(*tb, dev)
            ws_f = B.linear_workspace((rows, d_in), wl.dtype, d_out, wl.r_max, wl.ladder, wl.scales,
                                      wl.blend_w, dev)
            y_f = torch.empty((rows, d_out), dtype=wl.dtype, device=dev)
            fn = lambda: B.chunkwise_lora_linear(x[:rows], packed, None, None, wl.ladder, wl.scales,
                                                 wl.blend_w, sod_f, tab_f, rid_f, out=y_f, workspace=ws_f)
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            B.profile_enable((B.PROF_MAIN, B.PROF_META))
            for _ in range(args.steps):
                fn()
            torch.cuda.synchronize()
            t_p, n_p = B.profile_read(B.PROF_MAIN)
            t_f, n_f = B.profile_read(B.PROF_META)
            B.profile_enable(False)
            if n_p:
                us_p = t_p / n_p * 1e3
                us_f = t_f / n_f * 1e3 if n_f else 0.0
                few[str(rows)] = {"path": ("one row: x A (+ gate entry) in a first launch ('fixup_us'), then every output column "
                                           "as one dot product over [x | uhat] ('products_us')") if rows == 1 and d_in <= 8192
                                  else "partial products over slices of d_in ('products_us') + fix-up kernel ('fixup_us')",
                                  "products_us": us_p, "fixup_us": us_f, "launches": 2 if n_f else 1,
                                  "events_weight_stream_GBps": w_bytes / ((us_p + us_f) * 1e-6) / 1e9}
                try:
                    us_call = graph_call_us(fn)
                    few[str(rows)].update({"call_us_from_graph": us_call,
                                           "weight_stream_GBps": w_bytes / (us_call * 1e-6) / 1e9,
                                           "frac_of_hbm_peak": w_bytes / (us_call * 1e-6) / 1e9 / PEAK_HBM_GBS})
                except RuntimeError as err:        # graph capture unavailable: fall back to the event pairs
                    few[str(rows)].update({"graph_error": str(err)[:120],
                                           "weight_stream_GBps": w_bytes / ((us_p + us_f) * 1e-6) / 1e9,
                                           "frac_of_hbm_peak": w_bytes / ((us_p + us_f) * 1e-6) / 1e9 / PEAK_HBM_GBS})
        # one decode step of the scheduler for 64 sequences (one thread per sequence: launch latency)
        st_f = B.stream_state(64, dev)
        h_f = h[:64].contiguous()
        so_f = None
        for _ in range(args.warmup):
            so_f = B.stream_step(h_f, st_f, wl.l_min, wl.l_max, wl.theta(), wl.delta(), wl.taus(), wl.ladder,
                                 wl.scales, wl.blend_w, out=so_f)
        torch.cuda.synchronize()
        B.profile_enable((B.PROF_PARTITION,))
        for _ in range(args.steps):
            B.stream_step(h_f, st_f, wl.l_min, wl.l_max, wl.theta(), wl.delta(), wl.taus(), wl.ladder, wl.scales,
                          wl.blend_w, out=so_f)
        torch.cuda.synchronize()
        t_s, n_s = B.profile_read(B.PROF_PARTITION)
        B.profile_enable(False)
        if n_s:
            few["stream_step_us_64_sequences"] = t_s / n_s * 1e3
        # a decode step for 64 sequences replayed from a HIP graph (the calls only enqueue kernels): ten
        # copies of [scores of 64 new tokens + scheduler step] and of [the projection on 64 gated rows]
        try:
            nd, reps = 64, 10
            lg_d = logits[:nd].contiguous()
            x_d = x[:nd].contiguous()
            h_d = torch.empty(nd, dtype=torch.float32, device=dev)
            st_d = B.stream_state(nd, dev)
            so_d = B.stream_step(h_f, st_d, wl.l_min, wl.l_max, wl.theta(), wl.delta(), wl.taus(), wl.ladder,
                                 wl.scales, wl.blend_w)
            y_d = torch.empty((nd, d_out), dtype=wl.dtype, device=dev)
            ws_d = B.linear_workspace((nd, d_in), wl.dtype, d_out, wl.r_max, wl.ladder, wl.scales, wl.blend_w, dev)

            def sched():
                B.score_tokens(lg_d, out=h_d)
                B.stream_step(h_d, st_d, wl.l_min, wl.l_max, wl.theta(), wl.delta(), wl.taus(), wl.ladder,
                              wl.scales, wl.blend_w, out=so_d)

            def proj():
                B.gated_lora_linear(x_d, packed, so_d["gate"], wl.ladder, wl.scales, out=y_d, workspace=ws_d)

            def graph_us(fn):
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    fn()
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize()
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr, stream=side):
                    for _ in range(reps):
                        fn()
                gr.replay()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(args.steps):
                    gr.replay()
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / (args.steps * reps) * 1e3

            us_sched, us_proj = graph_us(sched), graph_us(proj)
            few["decode_step_graph_64_sequences"] = {
                "scores_and_scheduler_us": us_sched, "projection_us": us_proj,
                "projection_weight_stream_GBps": w_bytes / (us_proj * 1e-6) / 1e9,
                "projection_frac_of_hbm_peak": w_bytes / (us_proj * 1e-6) / 1e9 / PEAK_HBM_GBS}
        except RuntimeError as err:           # graph capture unavailable: report, do not fail the bench
            few["decode_step_graph_64_sequences"] = {"error": str(err)[:200]}
        out["few_rows"] = {"note": "rows <= 512: two launches per call (see 'path'); weight bytes = 2 d_in (d_out + R); the rate is "
                                   "taken from whole calls replayed from a HIP graph ('call_us_from_graph'); 'products_us' and "
                                   "'fixup_us' are the two launches by their event pairs, each of which adds a few microseconds",
                           "weight_bytes": w_bytes, **few}

    # ---- chunk-level KV-cache policy: one of K / V of a layer with 32 heads x 128 on this batch, the lower half
    #      of the ladder's rungs stored in INT8 (HBM-bound streaming; event-timed back-to-back calls) ----------
    if not args.no_variants and bf16:
        kv_h, kv_d, k_keep = 32, 128, max(K // 2, 1)
        gk = torch.Generator(device=dev)
        gk.manual_seed(77)
        kv = torch.randn((N, kv_h * kv_d), generator=gk, device=dev).to(wl.dtype)
        cache = B.kv_quantise_chunks(kv, kv_h, kv_d, k_keep, table, ri)
        kv_back = B.kv_dequantise(cache, N)
        torch.cuda.synchronize()
        nq, nf = cache["counts"].cpu().tolist()
        reps = max(args.steps, 10)
        B.profile_enable((B.PROF_KV,))
        for _ in range(reps):
            B.kv_quantise_chunks(kv, kv_h, kv_d, k_keep, table, ri, out=cache)
        torch.cuda.synchronize()
        t_k, n_k = B.profile_read(B.PROF_KV)
        B.profile_enable(False)
        us_q = t_k / max(n_k, 1) * 1e3
        us_d = timed(lambda: B.kv_dequantise(cache, N, out=kv_back), reps, 3)[0] * 1e3
        wid = kv_h * kv_d
        bytes_q = N * wid * 2.0 + nq * (wid + 4.0 * kv_h) + nf * wid * 2.0 + 4.0 * N
        bytes_d = nq * (wid + 4.0 * kv_h) + nf * wid * 2.0 + 4.0 * N + N * wid * 2.0
        out["kv_cache"] = {"note": "cwl_kv_quantise_chunks / cwl_kv_dequantise on one K (or V) tensor of the batch: rows of "
                                   "chunks whose rung is below k_keep in INT8 (one fp32 scale per row and head), the rest "
                                   "bf16; bytes = rows read + pools and slots written (quantise), the reverse (dequantise)",
                           "n_heads": kv_h, "head_dim": kv_d, "k_keep": k_keep, "rows_int8": nq, "rows_full": nf,
                           "cache_bytes_over_bf16": (nq * (wid + 4.0 * kv_h) + nf * wid * 2.0) / (N * wid * 2.0),
                           "quantise_us": us_q, "quantise_GBps": bytes_q / (us_q * 1e-6) / 1e9,
                           "quantise_frac_of_hbm_peak": bytes_q / (us_q * 1e-6) / 1e9 / PEAK_HBM_GBS,
                           "dequantise_us": us_d, "dequantise_GBps": bytes_d / (us_d * 1e-6) / 1e9,
                           "dequantise_frac_of_hbm_peak": bytes_d / (us_d * 1e-6) / 1e9 / PEAK_HBM_GBS}
        del kv, cache, kv_back

    # ---- scheduler variants: budget of high-capacity chunks, percentile buckets, aligned chunker ---
    if not args.no_variants:
        n_b = max(1, min(4, wl.n_seqs // 2))
        bk = B.bucket_sequences(h, sod, n_b, 2)
        tab_a = B.partition_chunks_aligned(h, sod, bk["bucket"], n_b, wl.l_min, wl.l_max, wl.theta(), wl.delta())
        ri_b, asked = B.select_ranks_budget(table, wl.taus(), K, K - 1, 4)
        # composite score: entropy + 3-gram novelty in a window of 256 tokens + positional prior over 512 positions
        gt = torch.Generator(device=dev)
        gt.manual_seed(5)
        tok = torch.randint(0, 8, (N,), generator=gt, device=dev, dtype=torch.int32)    # small alphabet: n-grams do repeat
        sc_c, nov_c = B.compose_scores(h, tok, sod, 3, 256, 1.0, 0.5, 0.25, 512.0)
        torch.cuda.synchronize()
        reps = max(args.steps, 10)
        us = lambda fn: timed(fn, reps, 3)[0] * 1e3
        out["scheduler_variants"] = {
            "note": "event-timed back-to-back launches of one call each, microseconds; integer work, launch-bound",
            "n_buckets": n_b,
            "partition_chunks_us": us(lambda: B.partition_chunks(h, sod, wl.l_min, wl.l_max, wl.theta(), wl.delta(),
                                                                out=table)),
            "bucket_sequences_us": us(lambda: B.bucket_sequences(h, sod, n_b, 2, out=bk)),
            "partition_chunks_aligned_us": us(lambda: B.partition_chunks_aligned(
                h, sod, bk["bucket"], n_b, wl.l_min, wl.l_max, wl.theta(), wl.delta(), out=tab_a)),
            "select_ranks_us": us(lambda: B.select_ranks(table, wl.taus(), K, out=ri)),
            "select_ranks_budget_us": us(lambda: B.select_ranks_budget(table, wl.taus(), K, K - 1, 4, out=ri_b,
                                                                       n_asked=asked)),
            "compose_scores_us": us(lambda: B.compose_scores(h, tok, sod, 3, 256, 1.0, 0.5, 0.25, 512.0, out=sc_c,
                                                             novelty=nov_c)),
            "compose_scores_new_ngrams": float(nov_c.float().mean().item()),
            "stream_step_aligned_us_64_sequences": None,
            "chunks_plain": int(table["chunk_offsets"][-1].item()),
            "chunks_aligned": int(tab_a["chunk_offsets"][-1].item()),
        }

        # the decode step of a batch of 64 sequences in 4 buckets with a budget
        st64 = B.stream_state(64, dev)
        bst4 = B.bucket_state(4, dev)
        bk64 = (torch.arange(64, device=dev, dtype=torch.int32) % 4).contiguous()
        nh64 = torch.zeros(64, dtype=torch.int32, device=dev)
        h64 = h[:64].contiguous()
        so64 = B.stream_step_aligned(h64, st64, wl.l_min, wl.l_max, wl.theta(), wl.delta(), wl.taus(), wl.ladder,
                                     wl.scales, wl.blend_w, bucket=bk64, bucket_st=bst4, k_high=K - 1, budget=4,
                                     n_high=nh64)
        out["scheduler_variants"]["stream_step_aligned_us_64_sequences"] = us(lambda: B.stream_step_aligned(
            h64, st64, wl.l_min, wl.l_max, wl.theta(), wl.delta(), wl.taus(), wl.ladder, wl.scales, wl.blend_w,
            bucket=bk64, bucket_st=bst4, k_high=K - 1, budget=4, n_high=nh64, out=so64))

    # ---- set-up work: the ladder of this projection's adapter by one SVD (offline in the paper) ----
    if not args.no_variants:
        B.build_ladder(A, Bm)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.build_ladder(A, Bm)
        torch.cuda.synchronize()
        out["ladder_build"] = {"note": "cwl_build_ladder on this projection's adapter, once per adapter, wall clock",
                               "d_in": d_in, "d_out": d_out, "r": wl.r_max,
                               "ms": (time.perf_counter() - t0) * 1e3}

    # ---- projections that share x (q/k/v): three calls against ONE grouped call (each projection on its own
    #      rungs: the same layers), and against one call on the fused weights with the ladder of the fused
    #      adapter (the joint best truncation below full rank: NOT the same layers) ----------------------
    if not args.no_variants and bf16 and d_in == d_out:
        gq = torch.Generator(device=dev)
        gq.manual_seed(1234)
        mk = lambda shape, scale: (torch.randn(shape, generator=gq, device=dev) * scale).to(wl.dtype)
        Ws3 = [Wm] + [mk((d_in, d_out), d_in ** -0.5) for _ in range(2)]
        As3 = [A] + [mk((d_in, wl.r_max), d_in ** -0.5) for _ in range(2)]
        Bs3 = [Bm] + [mk((wl.r_max, d_out), wl.r_max ** -0.5) for _ in range(2)]
        pk3 = [packed] + [B.prepack_weights(w_, a_, b_) for w_, a_, b_ in zip(Ws3[1:], As3[1:], Bs3[1:])]
        pg3 = B.prepack_weights_grouped(Ws3, As3, Bs3)
        joint = 3 * wl.r_max <= B.MAX_RANK
        if joint:
            Bf = torch.zeros((3 * wl.r_max, 3 * d_out), dtype=wl.dtype, device=dev)
            for i in range(3):
                Bf[i * wl.r_max:(i + 1) * wl.r_max, i * d_out:(i + 1) * d_out] = Bs3[i]
            A2f, B2f, _ = B.build_ladder(torch.cat(As3, dim=1).contiguous(), Bf)
            pkf = B.prepack_weights(torch.cat(Ws3, dim=1).contiguous(), A2f, B2f)
            del Bf, A2f, B2f
        del Ws3, As3, Bs3
        lad3 = [3 * v for v in wl.ladder]
        fused = {}
        for rows in (64, N):
            if rows == N:
                sod_q, tab_q, rid_q, x_q = sod, table, ri, x
            else:
                tb = W.random_chunk_table(1, [rows], min(wl.l_min, rows), max(min(wl.l_max, rows), 1), K, 11)
                sod_q, tab_q, rid_q = B.table_from_host(*tb, dev)
                x_q = x[:rows]
            ws1 = B.linear_workspace((rows, d_in), wl.dtype, d_out, wl.r_max, wl.ladder, wl.scales, wl.blend_w, dev)
            wsg = B.grouped_workspace(rows, pg3, wl.ladder, wl.scales, wl.blend_w, dev)
            y1 = torch.empty((rows, d_out), dtype=wl.dtype, device=dev)
            yf = torch.empty((rows, 3 * d_out), dtype=wl.dtype, device=dev)

            def three():
                for pk in pk3:
                    B.chunkwise_lora_linear(x_q, pk, None, None, wl.ladder, wl.scales, wl.blend_w, sod_q, tab_q,
                                            rid_q, out=y1, workspace=ws1)

            def grouped():
                B.chunkwise_lora_linear_grouped(x_q, pg3, wl.ladder, wl.scales, wl.blend_w, sod_q, tab_q, rid_q,
                                                out=yf, workspace=wsg)

            reps = max(args.steps // 2, 5)
            fused[str(rows)] = {"three_calls_us": timed(three, reps, 3)[0] * 1e3,
                                "one_grouped_call_us": timed(grouped, reps, 3)[0] * 1e3}
            if joint:
                wsf = B.linear_workspace((rows, d_in), wl.dtype, 3 * d_out, 3 * wl.r_max, lad3, wl.scales,
                                         wl.blend_w, dev)

                def one():
                    B.chunkwise_lora_linear(x_q, pkf, None, None, lad3, wl.scales, wl.blend_w, sod_q, tab_q, rid_q,
                                            out=yf, workspace=wsf)

                fused[str(rows)]["one_call_on_jointly_truncated_weights_us"] = timed(one, reps, 3)[0] * 1e3
                del wsf
            del ws1, wsg, y1, yf
        del pk3, pg3
        if joint:
            del pkf
        torch.cuda.empty_cache()
        out["grouped_qkv"] = {"note": "three d_in -> d_out projections of the same x: three calls against one "
                                      "grouped call (cwl_chunkwise_lora_linear_grouped_packed: the same three "
                                      "layers, each on its own rungs); 'jointly_truncated': one call on [Wq|Wk|Wv] "
                                      "with the ladder rebuilt on the fused adapter (ranks x 3), which below full "
                                      "rank is a different, jointly truncated layer and is listed for its timing "
                                      "only", **fused}

    # ---- every projection of the workload with the same chunk table -------------------------------
    if args.all_projections:
        per = {}
        for p_i, (p_name, p_in, p_out) in enumerate(wl.projections):
            xp, Wp, Ap, Bp = W.linear_operands(wl, p_i, dev)
            pk = B.prepack_weights(Wp, Ap, Bp)
            del Wp, Ap, Bp
            yp = torch.empty((N, p_out), dtype=wl.dtype, device=dev)
            wsp = B.linear_workspace((N, p_in), wl.dtype, p_out, wl.r_max, wl.ladder, wl.scales, wl.blend_w, dev)
            fn = lambda: B.chunkwise_lora_linear(xp, pk, None, None, wl.ladder, wl.scales, wl.blend_w, sod, table,
                                                 ri, out=yp, workspace=wsp)
            ms_p, _ = timed(fn, max(args.steps // 2, 1), 2)
            fl = 2.0 * N * p_in * p_out + 2.0 * float(r_eff.sum()) * (p_in + p_out)
            per[f"{p_i}:{p_name}"] = {"d_in": p_in, "d_out": p_out, "ms": ms_p, "effective_tflops": fl / ms_p / 1e9}
            del xp, pk, yp, wsp
            torch.cuda.empty_cache()
        tot = sum(v["ms"] for v in per.values())
        out["all_projections"] = {"linear_ms_sum": tot, "linear_tokens_per_s": N / (tot * 1e-3),
                                  "whole_path_tokens_per_s": N / ((tot + sum((kern_ms[k] or 0.0) for k in
                                                                   ("score", "partition", "select"))) * 1e-3),
                                  "per_projection": per}

    # ---- the CPU oracle on a bounded sample of the same workload ---------------------------------
    if not args.no_cpu_baseline:
        import oracle as O
        # bounded sample, sized for roughly 10-20 s of host work: entropy on every row when the logits
        # are at most ~1 GB (else 4096 rows), the linear on about 2.7e11 multiply-adds worth of rows
        n_ent = N if N * wl.vocab * esz <= 1.1e9 else min(N, 4096)
        n_lin = int(max(64, min(N, 2.7e11 // (d_in * d_out))))
        rows_e = np.linspace(0, N - 1, n_ent).astype(np.int64)
        rows_l = np.unique(np.linspace(0, N - 1, n_lin).astype(np.int64))
        lg = logits[torch.from_numpy(rows_e).to(dev)].float().cpu().numpy()
        xh, Wh, Ah, Bh = (t.float().cpu().numpy() for t in (x, Wm, A, Bm))
        hh = h.cpu().numpy()
        t0 = time.perf_counter(); O.entropy(lg); t_ent = time.perf_counter() - t0
        t0 = time.perf_counter()
        q, _ = O.quantise(hh)
        st, tab = O.partition(q, so, wl.l_min, wl.l_max, O.quantise_threshold(wl.theta()),
                              O.quantise_threshold(wl.delta()))
        rid = O.select(tab["chunk_sum"], tab["chunk_len"], [O.quantise_threshold(t) for t in wl.taus()])
        t_part = time.perf_counter() - t0
        t0 = time.perf_counter()
        O.linear(xh, Wh, Ah, Bh, wl.ladder, wl.scales, wl.blend_w, so, tab["chunk_offsets"],
                 tab["chunk_start"], tab["chunk_len"], rid, rows=rows_l)
        t_lin = time.perf_counter() - t0
        per_tok = t_ent / n_ent + t_part / N + t_lin / len(rows_l)
        out["cpu_baseline"] = {"value": 1.0 / per_tok, "unit": "tokens/s", "cores": O.num_threads(),
                               "kind": "oracle",
                               "sample": f"entropy on {n_ent} rows ({t_ent:.2f} s), partition+select on all "
                                         f"{N} rows ({t_part:.3f} s), linear on {len(rows_l)} rows "
                                         f"({t_lin:.2f} s); tokens/s extrapolated from the per-row times"}
    # ---- the other bf16 workloads, compact (whole step with every projection on one chunk table) ---
    if not args.no_other_workloads and not args.no_variants and args.workload == "cfg1":
        del logits, x, Wm, A, Bm, packed, y, ws
        torch.cuda.empty_cache()
        n_other = max(3, min(args.steps // 4, 10))
        out["other_workloads"] = {"note": "one step = scoring, partition and select once + the linear of every "
                                          "projection of the workload on that chunk table; call = gate table + "
                                          "shrink + main GEMM of one projection; fractions against the 2.5 PFLOP/s "
                                          "bf16 peak with the method's own flops (r_eff, not r_max)"}
        for other in ("cfg2", "cfg3", "cfg4"):
            out["other_workloads"][other] = other_workload(other, n_other, 3)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
