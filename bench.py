#!/usr/bin/env python3
"""Benchmark of the biased multi-channel beam-search decoder on one MI355X.

A step is one pass of the whole hot path over one synthetic workload: context upload,
utterance start, every chunk's advance, partial best paths where the workload asks for
them, final best paths.  Inputs are resident in HBM before the timed region starts.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published

# HBM bytes per advance launch (fetched + written) from rocprofv3's FETCH_SIZE / WRITE_SIZE counters, each scaled by
# what the same counter reads for a plain 1 GiB device copy (2.000 and 1.000); the runs and their commands are
# summarised under profiles/.  Counters cannot be read from inside this process, so the figure is carried here for the
# default configuration of the workloads that were profiled, each with the kernel's average launch time in the
# profiled build: a run whose own launch time is more than 5 % away from it is another kernel (or another machine
# state) and reports no traffic instead of a stale one.
MEASURED_TRAFFIC = {  # workload: (bytes per launch, ms per launch that bench.py reported in the profiled runs)
    "large": (1250044412, 0.6156),
    "stress": (14224662745, 4.9539),
    "dynamic": (4625691914, 1.8659),
    "medium": (438157735, 2.2768),
    "words": (523528186, 0.5160),
    "e2e": (4250525025, 4.0906),   # teams of four workgroups per channel
}
TRAFFIC_TOLERANCE = 0.05


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(inp, n_channels, budget_frames):
    """The CPU checker, as it stands, on a bounded sample of the same workload: the first
    n_channels channels of segment 0, all host cores, one channel per task."""
    from oracle import OracleGraph, OracleChannel
    w, g = inp.w, inp.g
    cores = min(len(os.sched_getaffinity(0)), n_channels)
    frames = min(w.frames, budget_frames)
    og = OracleGraph.from_graph(g)
    Lh = inp.loglikes[0][:n_channels, :frames].cpu().numpy()
    lists, offs = inp.contexts[0]
    chans = []
    for c in range(n_channels):
        ch = OracleChannel(og, w.beam, w.max_active)
        ch.set_context(lists[c], offs[c])
        chans.append(ch)

    def work(c):
        ch = chans[c]
        ch.reset()
        t = 0
        while t < frames:
            n = min(w.chunk, frames - t)
            ch.advance(Lh[c, t:t + n])
            t += n
            if w.partial_every_chunk:
                ch.best_path(False)
        ch.best_path(True)
        return ch.emit_arcs

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as ex:
        arcs = list(ex.map(work, range(n_channels)))
    dt = time.perf_counter() - t0
    audio = n_channels * frames * 0.030
    # one channel on one core, for the per-core figure
    t1 = time.perf_counter()
    work(0)
    dt1 = time.perf_counter() - t1
    return {"value": audio / dt, "unit": "x real time (RTFx)", "cores": cores, "kind": "oracle",
            "sample": f"{n_channels} of {w.channels} channels x {frames} of {w.frames} frames of segment 0, "
                      f"one channel per task on {cores} threads, {dt:.2f} s",
            "emit_arcs_per_s": sum(arcs) / dt,
            "single_core_value": frames * 0.030 / dt1}


def phase_report(B, sess, w, team=1):
    """Diagnostic build only: where thread 0 of each workgroup spent the lean frames of the last pass (sums kept per
    channel by the kernel, 100 MHz counter), per lean frame, averaged over the channels."""
    import ctypes as C
    L = B.lib()
    L.cbd_debug_profile.restype = C.c_int32
    L.cbd_debug_profile.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    v = np.zeros((w.channels, 19), np.int64)
    for c in range(w.channels):
        assert L.cbd_debug_profile(sess.dh, c, v[c].ctypes.data_as(C.c_void_p)) == 0
    timeline = None if team > 1 or not v[:, 16].any() else launch_timeline(v[:, 15:19])
    lean, frames = float(max(v[:, 10].sum(), 1)), float(max(v[:, 11].sum(), 1))
    us = lambda k: float(v[:, k].sum()) * 0.01 / lean
    launches = (w.frames + w.chunk - 1) // w.chunk
    run = v[:, 9] * 0.01 / launches
    return {"unit": "us per lean frame (thread 0 of the workgroup)", "lean_frames": int(lean), "frames": int(frames),
            "frames_sent_back_to_general_code": int(v[:, 8].sum()),
            "sent_back_because": {"closure_stage_over_64_records": int(((v[:, 14] >> 0) & 0xFFFF).sum()),
                                  "commit_log_full": int(((v[:, 14] >> 16) & 0xFFFF).sum()),
                                  "too_many_tokens": int(((v[:, 14] >> 32) & 0xFFFF).sum()),
                                  "other": int(((v[:, 14] >> 48) & 0xFFFF).sum()),
                                  "note": "events, several can fall into one frame"},
            "us_per_frame_sent_back_second_run": float(v[:, 7].sum()) * 0.01 / max(float(v[:, 8].sum()), 1.0),
            "sent_back_per_channel_max": int(v[:, 8].max()),
            "emit": us(0), "wait_barrier_1": us(1), "commit": us(6) + us(12) + us(13) + us(2),
            "commit_parts": {"slots_and_closure_reads": us(6), "emitting_min_and_log": us(12), "closure_levels_and_commit": us(13),
                             "next_row_and_rest": us(2)},
            "wait_barrier_2": us(3), "lookup_and_token_writes": us(4), "close_and_wait_barrier_3": us(5),
            "workgroup_us_per_launch": {"mean": float(run.mean()), "median": float(np.median(run)),
                                        "p90": float(np.percentile(run, 90)), "max": float(run.max())},
            "last_launch": timeline}


def launch_timeline(t):
    """The pass's last advance launch, from each workgroup's start and end stamp (one 100 MHz counter for the whole
    device) and hardware ids: how long the workgroups ran, how busy the compute units were until the launch ended,
    how long they stood between two workgroups and after their last one. Times in us."""
    st, en, hw = t[:, 0], t[:, 1], t[:, 2]
    t0 = st.min()
    st, en = (st - t0) * 0.01, (en - t0) * 0.01
    die, hwid = (hw >> 32) & 0xF, hw & 0xFFFFFFFF
    unit = die * 4096 + ((hwid >> 13) & 7) * 256 + ((hwid >> 12) & 1) * 16 + ((hwid >> 8) & 0xF)  # die, engine, array, CU
    dur, span = en - st, float(en.max())
    gaps, last_end = [], []
    for u in np.unique(unit):
        m = unit == u
        o = np.argsort(st[m])
        s, e = st[m][o], en[m][o]
        gaps += list(s[1:] - e[:-1])
        last_end.append(e.max())
    n_units = len(last_end)
    gaps, last_end = np.array(gaps if gaps else [0.0]), np.array(last_end)
    busy = float(dur.sum()) / n_units
    return {"span": span, "workgroups": int(len(dur)), "compute_units": n_units,
            "workgroup_us": {"mean": float(dur.mean()), "median": float(np.median(dur)), "p90": float(np.percentile(dur, 90)),
                             "max": float(dur.max())},
            "busy_per_compute_unit": busy, "busy_share": busy / span,
            "gap_between_workgroups": {"median": float(np.median(gaps)), "p90": float(np.percentile(gaps, 90)),
                                       "max": float(gaps.max()), "sum_per_compute_unit": float(gaps.sum()) / n_units,
                                       "share": float(gaps.sum()) / n_units / span},
            "compute_unit_last_end": {"min": float(last_end.min()), "mean": float(last_end.mean()), "max": float(last_end.max())},
            "tail_share": float(span - last_end.mean()) / span,
            "workgroups_per_die": [int((die == x).sum()) for x in np.unique(die)]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="large", choices=["tiny", "medium", "large", "dynamic", "stress", "e2e", "words"])
    ap.add_argument("--channels", type=int, default=0, help="override the channel count (smaller trial runs)")
    ap.add_argument("--frames", type=int, default=0, help="override the utterance length in frames")
    ap.add_argument("--chunk", type=int, default=0, help="override the frames per advance call")
    ap.add_argument("--compact-records-above", type=int, default=0,
                    help="compact a channel's back-pointer records once it holds more than this many new ones")
    ap.add_argument("--tail-partials", action="store_true",
                    help="partial results through cbd_best_tails_* (the part of the path above what compactions fixed)")
    ap.add_argument("--record-frames", type=int, default=0,
                    help="size the back-pointer buffer for this many frames (default: the utterance)")
    ap.add_argument("--hash-log2", type=int, default=0)
    ap.add_argument("--table-location", type=int, default=0)
    ap.add_argument("--lds-token-cap", type=int, default=0)
    ap.add_argument("--workgroups-per-cu", type=int, default=0)
    ap.add_argument("--block-threads", type=int, default=0)
    ap.add_argument("--workgroups-per-channel", type=int, default=-1,
                    help="team of workgroups per channel (2, 4, 8); default: the workload's (e2e: 4, others: 1)")
    ap.add_argument("--frame-code", type=int, default=0, help="0: lean frame code where it applies; 1: general code only")
    ap.add_argument("--lookup-mode", type=int, default=-1, help="0 binary search, 1 Bloom filter + search; default: the workload's")
    ap.add_argument("--unbiased", action="store_true", help="decode with empty contexts (switch-overhead comparison)")
    ap.add_argument("--sync-partials", action="store_true",
                    help="partial results with the blocking call instead of begin/finish requests")
    ap.add_argument("--context-mode", default="upload", choices=["upload", "pool"],
                    help="upload every segment's lists, or pre-load all of them and switch by id")
    ap.add_argument("--phases", action="store_true",
                    help="run the diagnostic build (python paper_2306_15685_amd/build.py --profile) and report the time "
                         "thread 0 of each workgroup spent in each phase of the lean frames (the stamps cost a few %%)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-channels", type=int, default=256, help="channels of the workload the CPU checker is timed on")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="BYTES",
                    help="only run a plain device copy of BYTES, ten times (scale for the profiler's HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build decodes on one GPU only; channels are independent, so more GPUs would each "
            "hold the graph and a share of the channels (no exchange). Run with --gpus 1.")
        sys.exit(2)

    import torch
    from paper_2306_15685_amd import synth, runner
    from paper_2306_15685_amd import binding as B

    if args.phases:
        from paper_2306_15685_amd import build as _build
        if not os.path.exists(_build.LIB_PROFILE):
            log(f"bench.py: {_build.LIB_PROFILE} is missing: python paper_2306_15685_amd/build.py --profile")
            sys.exit(2)
        B.LIB_PATH = _build.LIB_PROFILE
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = args.calibrate_copy // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n * 4, "copies": 10}))
        return
    w = synth.WORKLOADS[args.workload]
    if args.channels:
        w = synth.scaled(w, channels=args.channels)
    if args.lookup_mode >= 0:
        w = synth.scaled(w, lookup_mode=args.lookup_mode)
    if args.frames:
        w = synth.scaled(w, frames=args.frames)
    if args.chunk:
        w = synth.scaled(w, chunk=args.chunk)
    team = args.workgroups_per_channel if args.workgroups_per_channel >= 0 else runner.default_team(w)
    t0 = time.perf_counter()
    inp = runner.make_inputs(w)
    torch.cuda.synchronize()
    log(f"inputs: graph {inp.g.num_states} states {inp.g.num_arcs} arcs, {w.channels} channels x "
        f"{w.segments} x {w.frames} frames x {w.num_pdfs} pdfs in {time.perf_counter() - t0:.1f} s")
    sess = runner.Session(inp, hash_log2=args.hash_log2 or None, table_location=args.table_location,
                          biased=not args.unbiased, lds_token_cap=args.lds_token_cap, context_mode=args.context_mode,
                          async_partials=not args.sync_partials, workgroups_per_cu=args.workgroups_per_cu,
                          compact_records_above=args.compact_records_above, record_frames=args.record_frames,
                          tail_partials=args.tail_partials, block_threads=args.block_threads, frame_code=args.frame_code,
                          workgroups_per_channel=team)
    info = B.cbd_decoder_info(sess.dh)
    log(f"decoder: {info}")

    for _ in range(max(args.warmup, 0)):
        sess.step()
    torch.cuda.synchronize()
    # one untimed pass with counters (they do not change between passes: the decode is deterministic)
    sess.step(collect_stats=True)
    st = sess.step_stats
    if st["status"] != 0:
        log(f"bench.py: a channel ended in error state {st['status']} ({B.cbd_strerror(st['status'])})")
        sys.exit(1)

    sess.time_kernels = True
    sess.advance_events = []
    # The interpreter's cyclic garbage collector is kept out of the timed region: a full collection over the input
    # lists takes 30-70 ms once per process, and whether it lands in a timed pass is a matter of allocation counts.
    gc.collect()
    gc.disable()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sess.step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gc.enable()
    kms = sess.kernel_ms()
    sess.time_kernels = False

    ms_per_step = wall / args.steps * 1e3
    audio_s = w.channels * w.segments * w.frames * synth.FRAME_SHIFT_S
    rtfx = audio_s / (wall / args.steps)
    arcs = st["emit_arcs"] + st["eps_arcs"]
    launches_per_step = len(kms) // args.steps
    ctx_ints = sum(int(sum(len(x) for x in lists)) for lists, _ in inp.contexts) * ((w.frames + w.chunk - 1) // w.chunk)
    alg_bytes_step = runner.algorithmic_bytes(st, w, ctx_ints if not args.unbiased else 0)
    avg_launch_ms = float(np.mean(kms))
    achieved = alg_bytes_step / launches_per_step / (avg_launch_ms * 1e-3) / 1e9

    default_cfg = (not args.unbiased and args.context_mode == "upload" and not args.channels and not args.hash_log2
                   and not args.table_location and not args.lds_token_cap and not args.workgroups_per_cu and not args.block_threads and not args.frame_code and args.workgroups_per_channel < 0
                   and args.lookup_mode < 0 and not args.sync_partials and not args.frames and not args.chunk
                   and not args.compact_records_above and not args.record_frames and not args.tail_partials)
    traffic, traffic_at_ms = None, None
    if default_cfg and w.name in MEASURED_TRAFFIC:
        t_bytes, t_ms = MEASURED_TRAFFIC[w.name]
        traffic_at_ms = t_ms
        if abs(avg_launch_ms - t_ms) <= TRAFFIC_TOLERANCE * t_ms:
            traffic = t_bytes
        else:
            log(f"bench.py: launch time {avg_launch_ms:.4f} ms is more than {TRAFFIC_TOLERANCE:.0%} from the "
                f"{t_ms:.4f} ms the traffic figure was measured at: roofline.traffic = null")

    out = {
        "metric": "RTFx and arcs expanded/sec (1 MI355X, N channels) + % peak HBM BW",
        "value": rtfx, "unit": "x real time (RTFx)", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "channels": w.channels, "segments": w.segments, "frames": w.frames,
                   "chunk": w.chunk, "states": inp.g.num_states, "arcs": inp.g.num_arcs, "pdfs": w.num_pdfs,
                   "beam": w.beam, "max_active": w.max_active, "biased": not args.unbiased,
                   "context_mode": args.context_mode, "async_partials": not args.sync_partials,
                   "lookup_mode": w.lookup_mode, "lds_token_cap": info["lds_token_cap"],
                   "lds_bytes": info["lds_bytes"], "block_threads": info["block_threads"], "workgroups_per_channel": max(team, 1),
                   "compact_records_above": args.compact_records_above, "tail_partials": args.tail_partials, "device_bytes": info["device_bytes"]},
        "arcs_per_s": arcs / (wall / args.steps),
        "frames_per_s": w.channels * w.segments * w.frames / (wall / args.steps),
        "tokens_per_frame": st["tokens"] / max(st["frames"], 1),
        "counters": {k: int(v) for k, v in st.items()},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_measured_at_launch_ms": traffic_at_ms,
                     "achieved_is": "a model: per-unit bytes x the decoder's counters / measured kernel time "
                                    "(counts table and candidate traffic that this design keeps in LDS)",
                     "kernel": "advance_team_kernel" if team > 1 else "advance_kernel",
                     "kernel_note": None if team > 1 else "launches that start while result walks of earlier calls are in flight run "
                                    "as advance_beside_kernel (the same code held to 120 vector registers); both are timed here",
                     "launches_per_step": launches_per_step,
                     "avg_launch_ms": avg_launch_ms, "algorithmic_bytes_per_launch": alg_bytes_step / launches_per_step,
                     "kernel_time_share": sum(kms) / (wall * 1e3)},
    }
    out["config"]["device_bytes"] = B.cbd_decoder_info(sess.dh)["device_bytes"]   # (buffers allocated on first use included)
    if args.phases:
        out["phases"] = phase_report(B, sess, w, team)
    if inp.context_build is not None:   # Algorithm 1 on the host, outside the timed region (lists arrive rarely)
        out["context_build"] = inp.context_build
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, min(args.cpu_channels, w.channels), w.frames)
    sess.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
