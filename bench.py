#!/usr/bin/env python3
"""Benchmark of the layerwise-offloaded DiT block path on one MI355X.

A "step" is one denoising step of the workload: one pass of the whole hot path (prefetch issue,
per-chunk waits, modulation, LayerNorm, GEMMs, relayout, attention, gated residual) over all
blocks of the configuration, in steady state (the prefetch of block 0 for the next step is issued
during the last block).  Two arms are timed with the same kernels: fully resident (r = 1) and
chunked offload (r = --resident, default 0 = every weight byte streamed from pinned host memory).

Headline workload (no --config): the HunyuanVideo-like large-workload share, all 20 double-stream
blocks with distinct seeded weights -- the regime in which the prefetch has to hide (Sec. 4.2).  The
Flux-like small-workload share (8 blocks) and the Wan-like share (30 DiT blocks) are measured in
the same run and carried as `other_workloads` of the same JSON line.

Prints ONE JSON line: the offloaded step time as `value`, the resident step time beside it, the
roofline of the dominant kernel (measured with HIP events on the compute stream, per launch) and
the CPU oracle timed on this host's cores.
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

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
PEAK_LINK_GBS = 64.0           # PCIe Gen5 x16, one direction

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# scaled by a copy kernel of known size (see profiles/); None until measured for a workload.
TRAFFIC = {("flux", "gemm_lin1/256x256"): 607860396,      # profiles/hbm_traffic_flux_kernels.md
           ("flux", "gemm_lin2/128x128"): 528712950,
           ("flux", "attention"): 66248782,               # profiles/hbm_traffic_attention_all_shares.md
           ("wan", "attention"): 950651315,
           ("hunyuan", "attention"): 11949446179}
HEADLINE = "hunyuan"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default=None, help="one workload only (default: the headline workload plus the others as sub-records)", choices=["toy", "flux", "wan", "hunyuan", "flux_mm", "hunyuan_mm", "toy_mm"])
    ap.add_argument("--blocks", type=int, default=0, help="override the number of blocks (0 = the config's)")
    ap.add_argument("--shared-weights", action="store_true",
                    help="one seeded host blob per block kind, registered for every block of that kind: lets the full "
                         "57/60-block stacks run (every block still has its own resident copy and its own transfers)")
    ap.add_argument("--batch", type=int, default=1, help="samples per forward (B of App. B); the headline workload is 1")
    ap.add_argument("--resident", type=float, default=0.0, help="resident fraction of the offloaded arm")
    ap.add_argument("--chunk-mib", type=float, default=0.0, help="chunk size in MiB (0 = the config's chunk count)")
    ap.add_argument("--contention", choices=["off", "on", "pause", "pause2"], default="off",
                    help="emulated all-to-all traffic on a third stream; 'pause' adds pause/resume with one chunk in flight, "
                         "'pause2' with two")
    ap.add_argument("--sweep", action="store_true", help="memory-latency grid (r x chunk x contention) to stderr")
    ap.add_argument("--tune-budget-frac", type=float, default=0.5,
                    help="with --sweep: weight-memory budget, as a fraction of the stack's weights, handed to the tuner")
    ap.add_argument("--scale-sweep", action="store_true",
                    help="vary the sequence length of the config (frames for wan, image tokens for flux) and locate "
                         "the workload at which the prefetch becomes hidden (Eq. 3-4); prints its own JSON line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="headline workload only, no sub-records")
    ap.add_argument("--profile-steps", type=int, default=0,
                    help="steps of the pass that times every kernel with an event pair (0: --steps, at most 3 on the video shares)")
    ap.add_argument("--only", choices=["both", "resident", "offload"], default="both")
    return ap.parse_args()


def time_steps(run, ios, steps, warmup, torch):
    for _ in range(warmup):
        run.step(ios)
    run.ctx.cf_sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run.step(ios)
    run.ctx.cf_sync()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def block_times(run, ios, torch, reps=5):
    """Per-block compute time with everything resident: events on the compute stream around each
    block forward, median over `reps` passes."""
    import numpy as np
    L = len(ios)
    run.ctx.set_resident_fraction(1.0)
    ms = np.zeros((reps, L))
    for rep in range(reps + 1):                       # first pass warms up
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(L + 1)]
        evs[0].record(run.compute)
        for l in range(L):
            run.begin(l)
            run.fwd(l, ios[l])
            evs[l + 1].record(run.compute)
        run.ctx.cf_sync()
        torch.cuda.synchronize()
        if rep:
            ms[rep - 1] = [evs[l].elapsed_time(evs[l + 1]) for l in range(L)]
    return np.median(ms, axis=0)


def chain_residual_buffers(cfg, run, tens, torch, wl):
    """Chained residual stream: block l writes the buffer block l+1 reads.  One [B, n_local, d]
    buffer per block boundary, a sample's rows being this rank's text rows then its image rows;
    a double-stream block takes the two row ranges as two tensors, strided between samples."""
    L, tl, nl, d = cfg.n_blocks, cfg.n_txt_local, cfg.n_local, cfg.d
    lead = (cfg.batch,) if cfg.batch > 1 else ()
    bufs = [torch.randn(lead + (nl, d), device=run.device).to(torch.bfloat16).float() for _ in range(L + 1)]
    for b in range(L):
        t = tens[b]
        if cfg.kind_of(b) == wl.KIND_DOUBLE:
            s0 = lambda buf: buf[0] if cfg.batch > 1 else buf
            t["x_txt"], t["x"] = s0(bufs[b])[:tl], s0(bufs[b])[tl:]
            t["y_txt"], t["y"] = s0(bufs[b + 1])[:tl], s0(bufs[b + 1])[tl:]
            if cfg.batch > 1:
                t["x_sample_stride"] = t["x_txt_sample_stride"] = nl * d
        else:
            t["x"], t["y"] = bufs[b], bufs[b + 1]
    return bufs


def scale_sweep(args):
    """Sec. 4's scaling experiments on this machine: the same blocks at growing sequence lengths.
    Per size: FLOPs of the share (library counters), per-block time resident and fully offloaded,
    the first-order verdict (Eq. 3: hidden iff T_comp >= T_pref) and the measured one; then F* (Eq. 4)
    from the measured compute and link rates and the size at which the measured exposure vanishes."""
    import numpy as np
    import torch
    import workload as wl
    from paper_2605_11335_amd.runner import BlockRunner, chunk_bytes_for

    base = wl.CONFIGS[args.config]
    L = args.blocks or 3
    if base.kind == wl.KIND_DIT:
        # Wan-like video: S = 220 (n + 3) tokens for n frames (App. C, Table 2); n = 121 gives 27280
        sizes = [(f"{n} frames", 220 * (n + 3)) for n in (21, 41, 61, 81, 121, 161)]
    else:
        # Flux-like image model: the workload grows with the batch size B (Sec. 4.2)
        sizes = [(f"batch {k}", k) for k in (1, 2, 4, 8, 12, 16)]
    rows = []
    streams = None                      # every size runs on the same three streams
    for label, size in sizes:
        if base.kind == wl.KIND_DIT:
            n_total, batch = size // (2 * base.sp_degree) * (2 * base.sp_degree), 1
        else:
            n_total, batch = base.n_total, size
        cfg = base.with_(n_total=n_total, n_blocks=L, n_double=0, batch=batch)
        run = BlockRunner(cfg, chunk_bytes=chunk_bytes_for(cfg), streams=streams)
        streams = (run.compute, run.copy, run.comm)
        try:
            for b in range(L):
                run.register_params(b, wl.gen_block_params(cfg, b))
            tens = [run.make_io(wl.gen_block_inputs(cfg.with_(n_blocks=1), b)) for b in range(L)]
            bufs = chain_residual_buffers(cfg, run, tens, torch, wl)
            ios = [run.io_struct(t) for t in tens]

            def arm(r, profile=False):
                run.ctx.set_resident_fraction(r)
                run.ctx.cf_kernel_times_reset()
                run.ctx.cf_set_profiling(profile)
                run.begin(0)
                ms = time_steps(run, ios, args.steps if not profile else 2, max(3, args.warmup), torch)
                run.fwd(0, ios[0])
                run.ctx.cf_sync()
                kt = run.ctx.cf_kernel_times() if profile else None
                run.ctx.cf_set_profiling(False)
                return ms, kt
            _, kt = arm(1.0, profile=True)
            launches_steps = (2 + max(3, args.warmup)) * L + 1      # blocks run while profiling
            flops_blk = sum(k["flops"] for k in kt if not k["name"].startswith("modvec")) / launches_steps
            res_ms, _ = arm(1.0)
            off_ms, _ = arm(0.0)
            rows.append({"size": label, "n_total": n_total, "batch": batch, "flops_per_block": flops_blk,
                         "resident_ms_per_block": res_ms / L, "offload_ms_per_block": off_ms / L,
                         "exposed_ms_per_block": (off_ms - res_ms) / L, "blob_bytes": run.blob_bytes})
            print("[scale] " + json.dumps(rows[-1]), file=sys.stderr)
        finally:
            run.close()
            del run
            torch.cuda.empty_cache()
    # machine rates: compute rate from the largest size, link rate from the smallest (fully exposed) one
    blob = rows[0]["blob_bytes"]
    link = blob / (rows[0]["offload_ms_per_block"] * 1e-3)
    comp_rate = rows[-1]["flops_per_block"] / (rows[-1]["resident_ms_per_block"] * 1e-3)
    f_star = comp_rate * blob / link                               # Eq. 4 with measured eta_c * P_peak and eta_p * BW
    for r in rows:
        r["t_pref_ms"] = blob / link * 1e3
        r["hidden_by_eq3"] = bool(r["resident_ms_per_block"] >= r["t_pref_ms"])
        r["exposed_fraction_of_prefetch"] = r["exposed_ms_per_block"] / r["t_pref_ms"]
        r["hidden_measured"] = bool(r["exposed_fraction_of_prefetch"] <= 0.15)
        r["flops_over_f_star"] = r["flops_per_block"] / f_star
    out = {"metric": "prefetch exposure vs workload size (Eq. 3-4)", "config": {"workload": f"{base.name}: {L} blocks per size"},
           "n_gpus": 1, "dtype": "bf16", "data": "synthetic", "link_gbs": link / 1e9, "compute_tflops_at_largest": comp_rate / 1e12,
           "f_star_tflop": f_star / 1e12, "i_star_flop_per_byte": comp_rate / link, "sizes": rows}
    print(json.dumps(out))


def gen_params_parallel(cfg, blocks, wl, workers=8):
    """Seeded weights of several blocks, drawn tensor by tensor on a few host threads (NumPy's
    generators fill large arrays without holding the interpreter lock).  Same values as
    workload.gen_block_params: each tensor has its own counter-based stream."""
    from concurrent.futures import ThreadPoolExecutor
    jobs = [(b, spec) for b in blocks for spec in wl.param_specs(cfg.block_cfg(b))]
    def draw(job):
        b, (name, shape, std, mean) = job
        return b, name, wl.normal_bf16(cfg.name, b, name, shape, std, mean)
    out = {b: {} for b in blocks}
    with ThreadPoolExecutor(max_workers=workers) as ex:
        for b, name, arr in ex.map(draw, jobs):
            out[b][name] = arr
    return out


def measure(args, name, steps, warmup, *, blocks=0, shared_weights=False, shared_inputs=False, prof_steps=0,
            cpu_baseline=True, sweeps=False, streams=None):
    """Both arms of one workload; returns the fields of the JSON line that describe it."""
    import numpy as np
    import torch
    import workload as wl
    from paper_2605_11335_amd.runner import BlockRunner, chunk_bytes_for

    cfg = wl.CONFIGS[name].with_(batch=max(1, args.batch))
    if cfg.n_double and cfg.n_blocks > 12 and not blocks and not shared_weights:
        blocks = 6               # the full MMDiT stack holds 24 GB of distinct seeded weights; keep its 1:2 mix
    if blocks:
        # a mixed stack keeps its proportion of double-stream blocks
        cfg = cfg.with_(n_blocks=blocks,
                        n_double=(max(1, round(blocks * cfg.n_double / cfg.n_blocks)) if cfg.n_double else 0))
    L = cfg.n_blocks
    chunk_bytes = int(args.chunk_mib * (1 << 20)) if args.chunk_mib else chunk_bytes_for(cfg)
    video = cfg.n_total > 8192
    prof_steps = prof_steps or (min(steps, 3) if video else steps)
    prof_warmup = min(warmup, 1) if video else warmup

    t_setup = time.perf_counter()
    run = BlockRunner(cfg, chunk_bytes=chunk_bytes, streams=streams)
    first_of_kind = {}
    for b in range(L):
        first_of_kind.setdefault(cfg.kind_of(b), b)
    own = [b for b in range(L) if not shared_weights or first_of_kind[cfg.kind_of(b)] == b]
    # distinct seeded weights, a few blocks at a time so that the unpacked tensors never pile up
    for i in range(0, len(own), 4):
        for b, params in gen_params_parallel(cfg, own[i:i + 4], wl).items():
            run.register_params(b, params)
    for b in range(L):
        if b not in own:
            run.register_blob(b, run.blobs[first_of_kind[cfg.kind_of(b)]])
    if shared_weights or shared_inputs:
        # one seeded set of inputs per kind (peer tensors of a video share are 0.2-0.5 GB each); the
        # residual stream is chained through the blocks either way
        per_kind = {k: run.make_io(wl.gen_block_inputs(cfg.block_cfg(b), b)) for k, b in first_of_kind.items()}
        tens = [dict(per_kind[cfg.kind_of(b)]) for b in range(L)]
    else:
        tens = [run.make_io(wl.gen_block_inputs(cfg.block_cfg(b), b)) for b in range(L)]
    bufs = chain_residual_buffers(cfg, run, tens, torch, wl)
    ios = [run.io_struct(t) for t in tens]
    blob_total = run.total_blob_bytes                      # weight bytes of the whole stack
    print(f"[bench] {cfg.name}: {L} blocks, blobs {blob_total/1e6:.1f} MB in all, chunks of "
          f"{chunk_bytes/1e6:.2f} MB ({[run.ctx.cf_n_chunks(b) for b in range(L)]} per block), "
          f"setup {time.perf_counter()-t_setup:.1f}s", file=sys.stderr, flush=True)

    comm_host = None
    def set_contention(mode):
        nonlocal comm_host
        if mode == "off":
            run.ctx.cf_set_contention(None, None, 0, False)
            return
        nbytes = cfg.batch * cfg.n_local * cfg.d * 2          # one [B, n_local, d] bf16 tensor per all-to-all
        nbytes = nbytes // 512 * 512
        if comm_host is None:
            comm_host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
        run.ctx.cf_set_contention(run.comm, comm_host, nbytes, {"pause": 1, "pause2": 2}.get(mode, 0))

    def arm(r, n_steps, n_warmup):
        actual = run.ctx.set_resident_fraction(r)
        run.ctx.cf_stats_reset()
        run.begin(0)
        ms = time_steps(run, ios, n_steps, n_warmup, torch)
        st = run.ctx.cf_stats()
        run.fwd(0, ios[0])                         # consume the pending prefetch
        run.ctx.cf_sync()
        return ms, actual, st

    def table(ktimes, n_steps):
        out = {}
        for k in ktimes:
            e = {"launches": k["launches"], "launches_per_step": k["launches"] / n_steps,
                 "avg_ms": k["total_ms"] / k["launches"], "total_ms": k["total_ms"]}
            if k["flops"] > 0 and not k["name"].startswith("modvec"):
                e["tflops"] = k["flops"] / k["total_ms"] / 1e9
                e["frac_mfma_peak"] = e["tflops"] / PEAK_BF16_TFLOPS
            elif k["bytes"] > 0:
                e["gbs"] = k["bytes"] / k["total_ms"] / 1e6
                e["frac_hbm_peak"] = e["gbs"] / PEAK_HBM_GBS
            out[k["name"]] = e
        return out

    def breakdown(ktimes, n_steps, step_ms):
        """Step-time breakdown in the form of Sec. 4.3: kernels, time parked on chunk events (the
        exposed prefetch), time parked on emulated collectives, and the rest (launch gaps, event
        overhead), per step of the profiled pass."""
        waits = {"prefetch_stall": 0.0, "collective_wait": 0.0}
        comp = 0.0
        per_step = L / (n_steps * L + 1.0)          # the counters also hold the one block that drains the last prefetch
        for k in ktimes:
            if k["name"] in waits:
                waits[k["name"]] += k["total_ms"] * per_step
            else:
                comp += k["total_ms"] * per_step
        return {"step_ms_profiled": step_ms, "compute_ms": comp, "prefetch_stall_ms": waits["prefetch_stall"],
                "collective_wait_ms": waits["collective_wait"],
                "other_ms": step_ms - comp - waits["prefetch_stall"] - waits["collective_wait"]}

    set_contention(args.contention)
    total_steps = steps + warmup
    prof_total = prof_steps + prof_warmup
    do_res, do_off = args.only in ("both", "resident"), args.only in ("both", "offload")
    res_ms = off_ms = None
    kt_res, kt_off, st, actual_r = [], [], None, None
    if do_res:
        # resident arm: timed without event pairs, then once more with a hipEvent pair around
        # every kernel launch on the compute stream (the per-kernel table and the roofline)
        res_ms, _, _ = arm(1.0, steps, warmup)
        run.ctx.cf_kernel_times_reset()
        run.ctx.cf_set_profiling(True)
        res_prof_ms, _, _ = arm(1.0, prof_steps, prof_warmup)
        kt_res = run.ctx.cf_kernel_times()
        run.ctx.cf_set_profiling(False)
        print(f"[bench] {cfg.name}: resident {res_ms:.3f} ms/step", file=sys.stderr, flush=True)
    if do_off:
        off_ms, actual_r, st = arm(args.resident, steps, warmup)
        run.ctx.cf_kernel_times_reset()
        run.ctx.cf_set_profiling(True)
        off_prof_ms, _, _ = arm(args.resident, prof_steps, prof_warmup)
        kt_off = run.ctx.cf_kernel_times()
        run.ctx.cf_set_profiling(False)
        h2d_per_step = st["model_blob_bytes"] - st["model_resident_bytes"]
        # the drain block's streamed bytes: all but its leading round(r * n_chunks) chunks
        n_res0 = int(np.floor(args.resident * run.ctx.cf_n_chunks(0) + 0.5))
        first = run.blob_bytes_of[0] - min(run.blob_bytes_of[0], n_res0 * chunk_bytes)
        assert st["h2d_bytes"] == total_steps * h2d_per_step + first, "I/O volume changed"
        h2d_gbs = h2d_per_step / (off_ms * 1e-3) / 1e9
        print(f"[bench] {cfg.name}: chunked offload {off_ms:.3f} ms/step", file=sys.stderr, flush=True)
    else:
        h2d_per_step, h2d_gbs = 0, 0.0

    is_mfma = lambda k: k["flops"] > 0 and not k["name"].startswith("modvec")
    kt_main = kt_res if do_res else kt_off
    arm_name = "resident" if do_res else "offload"
    # the profiled arm ran prof_total steps plus one drain block: FLOPs per step from the counters
    total_flops = sum(k["flops"] for k in kt_main if is_mfma(k)) * L / (prof_total * L + 1)
    dom = max([k for k in kt_main if is_mfma(k)], key=lambda k: k["total_ms"])
    dom_ms = dom["total_ms"] / dom["launches"]
    dom_flops = dom["flops"] / dom["launches"]
    value = off_ms if do_off else res_ms

    weights_note = ("one seeded blob per block kind, registered for every block of that kind" if shared_weights
                    else "distinct seeded weights per block")
    inputs_note = ("one seeded set of activations and peer tensors per block kind, residual stream chained"
                   if (shared_weights or shared_inputs) else "distinct seeded inputs per block, residual stream chained")
    result = {
        "value": value, "unit": "ms", "steps": steps, "warmup": warmup, "ms_per_step": value,
        "config": {"workload": f"{cfg.name}: {L} blocks" + (f" ({cfg.n_double} double-stream + {L - cfg.n_double} single-stream)" if cfg.n_double else "") + f", d={cfg.d}, H={cfg.n_heads}x{cfg.head_dim}, f={cfg.f}, "
                               f"N={cfg.n_total}, Ulysses P={cfg.sp_degree} share (GEMMs on {cfg.n_local} tokens, "
                               f"attention {cfg.h_local} heads over {cfg.n_total})" + (f", batch {cfg.batch}" if cfg.batch > 1 else ""),
                   "arm": "chunked offload" if do_off else "resident",
                   "chunk_bytes": chunk_bytes, "chunks_per_block": run.n_chunks, "blob_bytes": run.blob_bytes,
                   "blob_bytes_all_blocks": blob_total, "shared_weights": bool(shared_weights),
                   "weights": weights_note, "inputs": inputs_note,
                   "resident_fraction": actual_r if do_off else 1.0, "contention": args.contention},
        "offload_ms": off_ms, "resident_ms": res_ms,
        "offload_over_resident": (off_ms / res_ms) if (do_res and do_off) else None,
        "step_tflops": total_flops / ((res_ms if do_res else off_ms) * 1e-3) / 1e12,
        "eta_comp_measured": (total_flops / (res_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS) if do_res else None,
        "h2d_gbs": h2d_gbs, "h2d_frac_link_peak": h2d_gbs / PEAK_LINK_GBS,
        "h2d_bytes_per_step": h2d_per_step,
        # block forwards of the offloaded arm that waited once for all their chunks (prefetch observed hidden)
        "blocks_one_wait": st["blocks_one_wait"] if st else None,
        "exposed_prefetch_ms": (off_ms - res_ms) if (do_res and do_off) else None,
        "weight_memory_bytes": st["weight_memory_bytes"] if st else blob_total,
        "roofline": {"bound": "mfma", "kernel": dom["name"], "arm": arm_name,
                     "achieved": dom_flops / dom_ms / 1e9,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": dom_flops / dom_ms / 1e9 / PEAK_BF16_TFLOPS,
                     "avg_launch_ms": dom_ms, "flops_per_launch": dom_flops, "launches": dom["launches"],
                     "traffic": TRAFFIC.get((cfg.name, dom["name"]))},
        "profiled_steps": prof_steps,
        "kernels_resident_arm": table(kt_res, prof_total), "kernels_offload_arm": table(kt_off, prof_total),
        "breakdown_resident_arm": breakdown(kt_res, prof_total, res_prof_ms) if do_res else None,
        "breakdown_offload_arm": breakdown(kt_off, prof_total, off_prof_ms) if do_off else None,
    }

    # ---- overlap-model view of this machine (Eq. 1-4 with the measured eta's)
    blob = blob_total / L                 # per block, averaged over the stack (App. B, block-averaged)
    t_comp_blk = (res_ms if do_res else off_ms) / L
    t_pref_blk = (blob / (h2d_gbs * 1e9) * 1e3) if h2d_gbs > 0 else None
    result["model"] = {"t_comp_block_ms": t_comp_blk, "t_pref_block_ms_at_measured_rate": t_pref_blk,
                       "t_pref_block_ms_at_link_peak": blob / (PEAK_LINK_GBS * 1e9) * 1e3,
                       "hidden": bool(do_res and do_off and off_ms <= 1.05 * res_ms),
                       "i_block_flop_per_byte": total_flops / L / blob,
                       "i_star_flop_per_byte": (total_flops / L / (t_comp_blk * 1e-3)) / (h2d_gbs * 1e9) if h2d_gbs else None}

    if sweeps:
        grid = []
        link = None                       # H2D rate of the fully offloaded, uncontended point
        # per-kind block compute time for the chunk-level model
        bt = block_times(run, ios, torch)
        t_comp = {k: float(np.mean([bt[b] for b in range(L) if cfg.kind_of(b) == k])) for k in set(cfg.kinds)}
        for mode in ("off", "on", "pause"):
            set_contention(mode)
            base_ms = None                # r = 1 step time of this contention mode
            pts = []
            for r in (1.0, 0.75, 0.5, 0.25, 0.0):
                ms, act, s2 = arm(r, steps, max(2, warmup))
                pts.append((r, ms, act, s2))
                if r == 1.0:
                    base_ms = ms
            if mode == "off":
                link = blob_total / (pts[-1][1] * 1e-3)
            for r, ms, act, s2 in reversed(pts):
                # first-order prediction (Eq. 1-3 applied per block): max(compute window, prefetch time);
                # chunk-level prediction: the library's walk of the two streams (uncontended link)
                pred = L * max(base_ms / L, (1.0 - act) * blob_total / L / link * 1e3)
                sim = run.ctx.cf_simulate(r, t_comp, link / 1e9)
                grid.append({"contention": mode, "r": r, "actual_r": act, "step_ms": ms, "model_step_ms": pred,
                             "sim_step_ms": sim["step_ms"] if mode == "off" else None,
                             "weight_memory_bytes": s2["weight_memory_bytes"],
                             "h2d_gbs": (s2["model_blob_bytes"] - s2["model_resident_bytes"]) / (ms * 1e-3) / 1e9,
                             "pauses": s2["pauses"]})
                print("[sweep] " + json.dumps(grid[-1]), file=sys.stderr)
        set_contention("off")
        result["sweep"] = grid
        # the dial (Sec. 3.3): fastest resident fraction under a weight-memory budget, then measured
        budget = int(args.tune_budget_frac * blob_total)
        choice = run.ctx.cf_tune(t_comp, link / 1e9, [chunk_bytes], 16, memory_budget_bytes=budget)
        ms, act, s2 = arm(choice["r"], steps, max(2, warmup))
        result["tune"] = {"budget_bytes": budget, "t_comp_ms_per_block": t_comp, "link_gbs": link / 1e9,
                          "chosen_r": choice["r"], "feasible": choice["feasible"],
                          "predicted_step_ms": choice["step_ms"], "measured_step_ms": ms,
                          "predicted_weight_memory_bytes": choice["weight_memory_bytes"],
                          "measured_weight_memory_bytes": s2["weight_memory_bytes"]}
        print("[tune] " + json.dumps(result["tune"]), file=sys.stderr)

    streams_used = (run.compute, run.copy, run.comm)
    run.close()
    del run, tens, bufs, ios
    torch.cuda.empty_cache()

    # ---- CPU oracle on this host, bounded sample (the GPU is idle meanwhile)
    if cpu_baseline:
        from oracle import block as ob
        import threadpoolctl
        rows = None
        sample = "1 full block of each kind"
        n_rows = 0
        if video:                                 # exact row sample: full attention would take hours
            # a few hundred rows keep the sample to some tens of seconds: K and V of all tokens are always built
            n_rows = 256
            rng = np.random.default_rng(1)
            rows = np.sort(rng.choice(cfg.n_local, n_rows, replace=False))
            sample = "%d of %d local rows of 1 block (keys and values of all %d tokens)" % (n_rows, cfg.n_local, cfg.n_total)
        total = 0.0
        measured = 0.0
        for b in sorted({cfg.kinds.index(k) for k in set(cfg.kinds)}):      # first block of each kind
            cb = cfg.block_cfg(b).with_(batch=1)          # one sample; a batch is that many independent samples
            params, inputs = wl.gen_block_params(cb, b), wl.gen_block_inputs(cb, b)
            t0 = time.perf_counter()
            ob.block_forward(cb, params, inputs, rows=rows, send_rows=(None if rows is None else np.arange(0)))
            dt = time.perf_counter() - t0
            measured += dt
            total += dt * cfg.kinds.count(cb.kind) * cfg.batch
        threads = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
        scale = 1.0 if rows is None else cfg.n_local / float(n_rows)
        result["cpu_baseline"] = {"value": total * 1e3 * scale, "unit": "ms", "cores": threads, "kind": "oracle",
                                  "measured_s": measured,
                                  "sample": f"{sample}, float64 NumPy, times the number of blocks of that kind per step"
                                            + ("" if rows is None else
                                               f"; row-sample extrapolation: measured time x {cfg.n_local}/{n_rows} rows, which "
                                               "overstates the share of the key/value projections that every row shares")}
    return result, streams_used


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding): use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.scale_sweep:
        args.config = args.config or "flux"
        return scale_sweep(args)
    contract = {"metric": "denoise step ms (chunked offload vs resident)", "n_gpus": 1, "higher_is_better": False,
                "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic"}
    if args.config:
        res, _ = measure(args, args.config, args.steps, args.warmup, blocks=args.blocks, shared_weights=args.shared_weights,
                         prof_steps=args.profile_steps, cpu_baseline=not args.no_cpu_baseline, sweeps=args.sweep)
        print(json.dumps({**contract, **res}))
        return
    # Headline: the large-workload share with all its blocks; K timed steps per arm as asked.
    res, streams = measure(args, HEADLINE, args.steps, args.warmup, blocks=args.blocks, shared_weights=args.shared_weights,
                           shared_inputs=True, prof_steps=args.profile_steps, cpu_baseline=not args.no_cpu_baseline)
    out = {**contract, **res}
    if not args.no_others:
        others = {}
        # the small-workload regime (link-bound by construction: the memory-latency curve lives here) and
        # the Wan-like share; the same three streams serve every runner (hardware queues are few)
        r2, _ = measure(args, "flux", args.steps, args.warmup, cpu_baseline=False, streams=streams)
        others["flux"] = r2
        r3, _ = measure(args, "wan", min(args.steps, 8), min(args.warmup, 2), shared_weights=True, cpu_baseline=False,
                        streams=streams)
        others["wan"] = r3
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
