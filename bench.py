#!/usr/bin/env python3
"""Benchmark of the CommFuse rank step on one MI355X.

``python bench.py --gpus 1 --steps K --warmup W`` prints ONE JSON line.

A "step" is one emulated rank step of the Llama-70B-shape MLP pair (p = 8):
the all-gather + GEMM up-projection (Alg. 1: 8 chunk GEMMs, 7 slice deliveries)
followed by the GEMM + reduce-scatter down-projection (Alg. 2 / Alg. 3: 8 chunk
GEMMs with the fused B_in add, 7 partial-sum deliveries), i.e. every row of the
hot path except the gradient reduce, which is reported next to it
(``dp_reduce``), as are the two Llama-7B-shape rank steps (``other_configs``).
All inputs are seeded, synthetic and resident in HBM before the timed region.
Everything runs on one GPU; ``--gpus N`` with N > 1 is refused.
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

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
SETTLE_S = 0.06               # untimed load before every timed region (see time_calls)
# HBM-side bytes per launch of the dominant kernel from rocprofv3 counters (FETCH_SIZE x 2.00 + WRITE_SIZE): a constant
# taken from TRAFFIC_SOURCE, not measured in this run -- to be re-derived there whenever that kernel changes
TRAFFIC_DOWN_RANK_STEP = 1226.4e6
TRAFFIC_DOWN_RANK_STEP_CARRIED = 1461.4e6    # the same launch carrying its deliveries: 955.5 MB read + 505.9 MB written
TRAFFIC_SOURCE = "profiles/gemm_bf16_dl_kernel_70b_pair_counters.md"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--skip-dp", action="store_true", help="leave out the 1e9-element gradient bucket")
    ap.add_argument("--skip-cpu", action="store_true", help="leave out the CPU-oracle baseline")
    ap.add_argument("--only-pair", action="store_true", help="time the headline workload only")
    ap.add_argument("--sections", default="", help="comma-separated subset of the secondary measurements to run "
                    "(7b, pairwise, granularity, backward, attention, dp; and, on request only, power); default: all.  With --skip-pair the headline "
                    "workload is left out and the JSON line carries only what was measured (profiling runs)")
    ap.add_argument("--skip-pair", action="store_true", help="leave the headline workload out (profiling runs of one section)")
    ap.add_argument("--skip-kernel-probe", action="store_true",
                    help="do not time the dominant kernel alone (profiling runs of one schedule mode: the probe launches the "
                         "same kernel without its deliveries); the line then carries no roofline")
    ap.add_argument("--modes", default="", help="comma-separated subset of the schedule modes to time (default: all)")
    ap.add_argument("--power-data", default="both", choices=("random", "zero", "both"),
                    help="operands of the section 'power' (--sections power: the up-projection kernel on random and on "
                         "all-zero operands, and on grids capped below the chip)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (known bytes, for scaling hardware counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (peer traffic is emulated in HBM); --gpus must be 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2604_24013_amd import binding as cf
    from paper_2604_24013_amd import inputs
    from paper_2604_24013_amd import emulated_rank as H

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if "power" in args.sections.split(","):          # that probe switches a tuning override between its launches
        os.environ["COMMFUSE_TUNING_LIVE"] = "1"
    cf.load()
    K, W = args.steps, args.warmup
    ALL_SECTIONS = ("7b", "pairwise", "granularity", "backward", "attention", "dp")
    sections = set(args.sections.split(",")) if args.sections else set(ALL_SECTIONS)
    power_probe = "power" in sections                # on request only: not one of the default sections
    sections.discard("power")
    if args.only_pair:
        sections = set()
    if args.skip_dp:
        sections.discard("dp")
    assert sections <= set(ALL_SECTIONS), f"unknown section in {sorted(sections)}"

    def time_calls(fn, stream, steps, warmup):
        """Average milliseconds of fn() over `steps` back-to-back calls, HIP events on `stream`.
        Untimed calls first: `warmup` of them, and as many more as it takes to keep the GPU busy for
        SETTLE_S seconds (after an idle stretch -- input generation on the host -- the shader clock
        takes some tens of milliseconds of load to settle; shorter warm-ups time the ramp)."""
        t0, n = time.perf_counter(), 0
        while n < warmup or time.perf_counter() - t0 < SETTLE_S:
            fn()
            n += 1
            if n % 4 == 0:
                stream.synchronize()
        stream.synchronize()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            fn()
        e1.record(stream)
        e1.synchronize()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def schedule_times(run, kind, steps, warmup):
        """Rank-step time overlapped / compute-only / copy-only: the best mode of each, and every mode's own
        three times under "by_mode" (the overlap figures compare a mode with ITS compute-only and copy-only times)."""
        out = {"by_mode": {}}
        for name, fl in (("overlapped", 0), ("compute_only", cf.CF_NO_COPY), ("copy_only", cf.CF_NO_COMPUTE)):
            best = None
            pers_pair = kind == cf.CF_KIND_RS_PAIR and getattr(run, "each", None) is not None
            for mode, extra in MODES if (kind in (cf.CF_KIND_RS, cf.CF_KIND_AG) and (fl == 0 or "persistent" in mode or mode in BASIC_NAMES)) \
                    else (BASIC + tuple(m for m in MODES if "persistent" in m[0] and "groups" not in m[0]) if pers_pair else BASIC):
                if fl != 0 and (extra & (cf.CF_FUSED_COPY | cf.CF_DEVICE_WAIT)):
                    continue
                if (extra & cf.CF_PERSISTENT) and getattr(run, "each", None) is None:
                    continue                              # needs a landing buffer per hop
                t = time_calls(lambda: cf.run_schedule(run.desc, kind, run.bufs, run.cs, run.xs, fl | extra),
                               run.cs, steps, warmup)
                out["by_mode"].setdefault(mode, {})[name] = t
                if best is None or t < best[0]:
                    best = (t, mode)
            out[name] = best
        return out

    # how the emulated deliveries are enqueued: hipMemcpyAsync on the copy stream ordered by events
    # (eager or as a captured graph), or carried by extra workgroups of the step kernels (one stream)
    # or not overlapped at all (one stream, each delivery after the kernel before it: the copies then run
    # at full speed and disturb no GEMM -- a reference point for what the overlap buys); "persistent": all
    # steps of a rank step in one kernel launch, the deliveries enqueued before it; "persistent+carried": no copy is
    # enqueued, the kernel's own waves read B_in from the neighbour's buffer under the main loop and store it to the
    # landing buffer; "persistent-groups": two streams again -- a few launches per layer, each a group of steps that fills
    # the chip about once, the deliveries of a group on the copy stream under the launches of the groups before it
    MODES = (("streams", 0), ("graph", cf.CF_GRAPH), ("fused-copy", cf.CF_FUSED_COPY),
             ("fused-copy+graph", cf.CF_FUSED_COPY | cf.CF_GRAPH), ("device-wait", cf.CF_DEVICE_WAIT),
             ("serial", cf.CF_SERIAL), ("serial+graph", cf.CF_SERIAL | cf.CF_GRAPH),
             ("persistent", cf.CF_PERSISTENT | cf.CF_SERIAL),
             ("persistent+graph", cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_GRAPH),
             ("persistent+carried", cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY),
             ("persistent-groups", cf.CF_PERSISTENT), ("persistent-groups+graph", cf.CF_PERSISTENT | cf.CF_GRAPH))

    BASIC_NAMES = ("streams", "graph", "serial", "serial+graph")
    BASIC = tuple(m for m in MODES if m[0] in BASIC_NAMES)   # work for every kind and flag
    if args.modes:
        keep = set(args.modes.split(","))
        MODES = tuple(m for m in MODES[:2]) + tuple(m for m in MODES[2:] if m[0] in keep) if not keep & {"streams", "graph"} \
            else tuple(m for m in MODES if m[0] in keep)

    def overlap_of(step, compute, copy):
        """Overlap efficiency max(compute, copy) / step and hidden fraction (compute + copy - step) / copy of ONE
        mode: all three times are that mode's own.  A mode that enqueues the deliveries in front of the kernels
        (serial, persistent) hides nothing: its hidden fraction is ~0 whatever its efficiency figure says."""
        return {"overlap_eff": round(max(compute, copy) / step, 3),
                "hidden_fraction": round((compute + copy - step) / copy, 3) if copy > 0 else None}

    def overlap_eff(t):
        """Overlap figures of the mode whose step time is reported (its own compute-only / copy-only times;
        the fused-copy and device-wait modes have no such variants and take the stream mode's)."""
        m = t["by_mode"].get(t["overlapped"][1], {})
        ref = t["by_mode"].get("persistent" if "persistent" in t["overlapped"][1] else "streams", {})
        comp = m.get("compute_only", ref.get("compute_only", t["compute_only"][0]))
        cpy = m.get("copy_only", ref.get("copy_only", t["copy_only"][0]))
        return overlap_of(t["overlapped"][0], comp, cpy)

    def overlap_by_mode(t):
        out = {}
        for mode, v in t["by_mode"].items():
            ref = t["by_mode"].get("persistent" if "persistent" in mode else "streams", {})
            if "overlapped" in v:
                comp = v.get("compute_only", ref.get("compute_only"))
                cpy = v.get("copy_only", ref.get("copy_only"))
                if comp and cpy:
                    out[mode] = dict(us_per_step=round(v["overlapped"] * 1e3, 1), **overlap_of(v["overlapped"], comp, cpy))
        return out

    # split-K workspace for the layers whose per-step grids are small (sized for the largest layer here)
    ws_bytes = max(cf.workspace_bytes(H.desc_of(inputs.CONFIGS[n], 0), cf.CF_KIND_AG if inputs.CONFIGS[n].kind == "ag" else cf.CF_KIND_RS)
                   for n in ("c2_rs_7b", "c3_ag_7b", "c4_ag_70b_up", "c4_rs_70b_down"))
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=H.DEV)
    cf.set_workspace(workspace, ws_bytes)
    torch.cuda.synchronize()

    # ---------------- headline: 70B MLP pair ----------------
    up, dn = inputs.CONFIGS["c4_ag_70b_up"], inputs.CONFIGS["c4_rs_70b_down"]
    flops_pair = up.flops + dn.flops
    value = ms_step = None
    roofline = vanilla = None
    pair_t, pair_modes, pair_overlap, pair_by_mode = {}, {}, {}, {}
    if not args.skip_pair:
        log("generating 70B-shape inputs ...")
        # every hop's delivery has a landing buffer of its own (cf_buffers.recv_each): nothing is reused inside a
        # rank step, so the copy stream never waits for a kernel
        ag = H.AgRun(up, inputs.make_ag(up), 0, each=True)
        ddn = inputs.make_rs(dn)
        rs = H.RsRun(dn, ddn, 0, each=True)
        rs.A = ag.O                                   # H is handed over on the device, in bf16
        rs.bufs = cf.make_buffers(rs.A, rs.W, rs.O, rs.stage, rs.slot, rs.send, None, rs.each, rs.send_each)
        rs.cs, rs.xs = ag.cs, ag.xs                   # one compute stream, one copy stream for the pair

        def pair(flags):
            cf.run_schedule(ag.desc, cf.CF_KIND_AG, ag.bufs, ag.cs, ag.xs, flags)
            cf.run_schedule(rs.desc, cf.CF_KIND_RS, rs.bufs, rs.cs, rs.xs, flags)

        for name, fl in (("overlapped", 0), ("compute_only", cf.CF_NO_COPY), ("copy_only", cf.CF_NO_COMPUTE)):
            best = None
            for mode, extra in MODES:
                if fl != 0 and (extra & (cf.CF_FUSED_COPY | cf.CF_DEVICE_WAIT)):
                    continue
                t = time_calls(lambda: pair(fl | extra), ag.cs, K, W)
                log(f"  pair {name} [{mode}]: {t*1e3:.1f} us")
                pair_by_mode.setdefault(mode, {})[name] = t
                if fl == 0:
                    pair_modes[mode] = round(t * 1e3, 1)
                if best is None or t < best[0]:
                    best = (t, mode)
            pair_t[name] = best
            log(f"pair {name}: {best[0]*1e3:.1f} us ({best[1]})")
        ms_step = pair_t["overlapped"][0]
        value = flops_pair / (ms_step * 1e-3) / 1e12

        # dominant kernel: the down-projection rank-step kernel (one persistent launch = the eight chunk GEMMs
        # of the rank step with their B_in adds and B_out / O stores), launched alone: CF_NO_COPY enqueues nothing else
        PS = cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_NO_COPY
        if not args.skip_kernel_probe:
            t_kernel = time_calls(lambda: cf.run_schedule(rs.desc, cf.CF_KIND_RS, rs.bufs, rs.cs, rs.xs, PS), ag.cs, max(K, 50), W)
            ach = dn.flops / (t_kernel * 1e-3) / 1e12
            t_kernel_up = time_calls(lambda: cf.run_schedule(ag.desc, cf.CF_KIND_AG, ag.bufs, ag.cs, ag.xs, PS), ag.cs, max(K, 50), W)
            # the same GEMMs as one kernel per step (what every mode but "persistent" launches), step 1 alone
            t_chunk = time_calls(lambda: cf.rs_step(rs.desc, 1, rs.A, rs.W, rs.stage[0], rs.send[0], ag.cs), ag.cs, max(K, 50), W)
            t_chunk_up = time_calls(lambda: cf.ag_step(ag.desc, 1, ag.stage[0], ag.W, ag.O, ag.cs), ag.cs, max(K, 50), W)
            chunk_flops = 2.0 * dn.m_chunk * dn.n * dn.k
            # the same launch as the headline mode issues it: carrying its deliveries (it reads the seven B_in from the
            # neighbours' buffers and also stores them to the landing buffers -- the emulated transfers' 234.9 MB of
            # writes, which are no part of the method's own bytes)
            # (only where that mode is among the modes of this run: a counter pass over one mode must not mix the two)
            PC = cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_FUSED_COPY
            carried_too = any(m == "persistent+carried" for m, _ in MODES)
            t_carry = time_calls(lambda: cf.run_schedule(rs.desc, cf.CF_KIND_RS, rs.bufs, rs.cs, rs.xs, PC), ag.cs, max(K, 50), W) if carried_too else None
            t_carry_up = time_calls(lambda: cf.run_schedule(ag.desc, cf.CF_KIND_AG, ag.bufs, ag.cs, ag.xs, PC), ag.cs, max(K, 50), W) if carried_too else None
            roofline = {"bound": "mfma",
                        "kernel": "gemm_bf16_dl_kernel<256,256,...,persistent,B_in through LDS> (down-projection rank step: 8 chunk GEMMs, "
                                  "fused B_in adds, every step's B_out stored)",
                        "achieved": round(ach, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                        # bytes through the L2s' memory side per launch from rocprofv3 counters: FETCH_SIZE x 2.00 (scale
                        # from a plain 256 MiB copy) + WRITE_SIZE; algorithmic bytes: A 58.7 + W 58.7 + B_in 7 x 33.55 +
                        # B_out/O 8 x 33.55 MB
                        "traffic": TRAFFIC_DOWN_RANK_STEP, "traffic_source": TRAFFIC_SOURCE, "algorithmic_bytes": 620.7e6,
                        "us_per_launch": round(t_kernel * 1e3, 2),
                        "carrying_its_deliveries": None if t_carry is None else {
                            "us_per_launch": round(t_carry * 1e3, 2),
                            "achieved": round(dn.flops / (t_carry * 1e-3) / 1e12, 1),
                            "frac": round(dn.flops / (t_carry * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                            "traffic": TRAFFIC_DOWN_RANK_STEP_CARRIED,
                            "up_projection_us_per_launch": round(t_carry_up * 1e3, 2)},
                        "up_projection_rank_step_kernel": {"us_per_launch": round(t_kernel_up * 1e3, 2),
                                                           "tflops": round(up.flops / (t_kernel_up * 1e-3) / 1e12, 1)},
                        "one_kernel_per_step": {"down_us": round(t_chunk * 1e3, 2), "down_tflops": round(chunk_flops / (t_chunk * 1e-3) / 1e12, 1),
                                                "up_us": round(t_chunk_up * 1e3, 2), "up_tflops": round(chunk_flops / (t_chunk_up * 1e-3) / 1e12, 1)}}
            log(f"rank-step kernel down {t_kernel*1e3:.1f} us = {ach:.0f} TFLOP/s, up {t_kernel_up*1e3:.1f} us; "
                f"chunk GEMM down {t_chunk*1e3:.1f} us, up {t_chunk_up*1e3:.1f} us")
        # comparator, same kernels: the layer pair WITHOUT the fusion ("vanilla": the collective, then / after the whole GEMM).
        # up: all-gather first, then the GEMM over all 8192 rows -- which is what the persistent arrangement does anyway;
        # down: the GEMM over all 8192 rows into a full fp32 partial (the same persistent kernel, no B_in adds), then the
        # reduce-scatter: seven deliveries, each added to its slice in a pass of its own (the gradient kernel).
        # One stream, nothing overlaps: what the paper's method starts from.
        if sections:
            H_all = ag.O                                              # [8192 x 3584] bf16, written by the up-projection
            Y_all = torch.empty((dn.p * dn.m_chunk, dn.n), dtype=torch.float32, device=H.DEV)
            blk = lambda c: H_all[c * dn.m_chunk:(c + 1) * dn.m_chunk]
            rows = [blk((0 - i) % dn.p) for i in range(1, dn.p)]      # slice of step i where Alg. 1 expects it: no copies needed
            d_whole = cf.layer_desc(dn.p, 0, dn.m_chunk, dn.n, dn.k, "bf16", "f32")
            b_whole = cf.make_buffers(blk(0), rs.W, Y_all, rows, (None, None), (None, None), None, rows)
            chunk_elems = dn.m_chunk * dn.n
            PS_ = cf.CF_PERSISTENT | cf.CF_SERIAL

            def vanilla_up():
                cf.run_schedule(ag.desc, cf.CF_KIND_AG, ag.bufs, ag.cs, ag.xs, PS_)

            def vanilla_down():
                cf.run_schedule(d_whole, cf.CF_KIND_AG, b_whole, ag.cs, ag.xs, PS_ | cf.CF_NO_COPY)
                cf.run_schedule(rs.desc, cf.CF_KIND_RS, rs.bufs, rs.cs, rs.xs, PS_ | cf.CF_NO_COMPUTE)   # the seven deliveries
                for i in range(1, dn.p):
                    cf.dp_reduce_step(dn.p, 0, i, Y_all, chunk_elems, rs.each[i - 1], ag.cs)

            t_vu = time_calls(vanilla_up, ag.cs, K, W)
            t_vd = time_calls(vanilla_down, ag.cs, K, W)
            t_vp = time_calls(lambda: (vanilla_up(), vanilla_down()), ag.cs, K, W)
            vanilla = {"us_up_gather_then_gemm": round(t_vu * 1e3, 1), "us_down_gemm_then_reduce_scatter": round(t_vd * 1e3, 1),
                       "us_pair": round(t_vp * 1e3, 1), "tflops_pair": round(flops_pair / (t_vp * 1e-3) / 1e12, 1),
                       "vanilla_over_fused": round(t_vp / ms_step, 3)}
            log("vanilla", vanilla)
            del Y_all, b_whole, rows
        del ag, rs, ddn
        torch.cuda.empty_cache()

    # ---------------- the two 7B-shape rank steps ----------------
    others = {}
    if "7b" in sections:
        for name, Run, make, kind in (("c2_rs_7b", H.RsRun, inputs.make_rs, cf.CF_KIND_RS),
                                      ("c3_ag_7b", H.AgRun, inputs.make_ag, cf.CF_KIND_AG)):
            w = inputs.CONFIGS[name]
            run = Run(w, make(w), 0, each=True)
            t = schedule_times(run, kind, max(K, 100), W)
            others[name] = {"tflops": round(w.flops / (t["overlapped"][0] * 1e-3) / 1e12, 1),
                            "frac_mfma_peak": round(w.flops / (t["overlapped"][0] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                            "us_per_rank_step": round(t["overlapped"][0] * 1e3, 1), "mode": t["overlapped"][1],
                            **overlap_eff(t),
                            "us_compute_only": round(t["compute_only"][0] * 1e3, 1),
                            "us_copy_only": round(t["copy_only"][0] * 1e3, 1),
                            "tflops_compute_only": round(w.flops / (t["compute_only"][0] * 1e-3) / 1e12, 1),
                            "overlap_by_mode": overlap_by_mode(t)}
            log(name, others[name])
            del run
            torch.cuda.empty_cache()

    # ---------------- GEMM + reduce-scatter under the pairwise bidirectional schedule ----------------
    pairwise = {}
    if "pairwise" in sections:
        for name in ("c2_rs_7b", "c4_rs_70b_down"):
            w = inputs.CONFIGS[name]
            data = inputs.make_rs(w)
            run = H.RsPairRun(w, data, 0)
            t_inc = schedule_times(run, cf.CF_KIND_RS_PAIR, max(K, 50), W)
            del run
            run = H.RsPairRun(w, data, 0, keep_all=True)        # every arrival kept, summed by the last step
            t = schedule_times(run, cf.CF_KIND_RS_PAIR, max(K, 50), W)
            pairwise[name] = {"us_per_rank_step_incremental_aggregation": round(t_inc["overlapped"][0] * 1e3, 1),"tflops": round(w.flops / (t["overlapped"][0] * 1e-3) / 1e12, 1),
                              "us_per_rank_step": round(t["overlapped"][0] * 1e3, 1), "mode": t["overlapped"][1],
                              **overlap_eff(t),
                              "us_compute_only": round(t["compute_only"][0] * 1e3, 1),
                              "us_copy_only": round(t["copy_only"][0] * 1e3, 1),
                              "us_per_rank_step_by_mode": {m_: round(v["overlapped"] * 1e3, 1) for m_, v in t["by_mode"].items() if "overlapped" in v}}
            log("pairwise", name, pairwise[name])
            del run
            torch.cuda.empty_cache()

    # ---------------- slicing granularity m = 2 (two sub-steps per ring hop) ----------------
    granularity = {}
    if "granularity" in sections:
        for name, Run, make, kind in (("c4_rs_70b_down", H.RsRun, inputs.make_rs, cf.CF_KIND_RS),
                                      ("c4_ag_70b_up", H.AgRun, inputs.make_ag, cf.CF_KIND_AG)):
            w = inputs.CONFIGS[name]
            data = make(w)
            entry = {}
            for m in (1, 2):
                run = Run(w, data, 0, m=m, each=True)
                t = schedule_times(run, kind, max(K, 50), W)
                entry[f"m{m}"] = {"tflops": round(w.flops / (t["overlapped"][0] * 1e-3) / 1e12, 1),
                                  "us_per_rank_step": round(t["overlapped"][0] * 1e3, 1), "mode": t["overlapped"][1],
                                  **overlap_eff(t),
                                  "us_compute_only": round(t["compute_only"][0] * 1e3, 1)}
                del run
                torch.cuda.empty_cache()
            granularity[name] = entry
            log("granularity", name, entry)

    # ---------------- backward pass of the 70B pair: two data gradients, two weight gradients ----------------
    backward = {}
    if "backward" in sections:
        rng = np.random.default_rng(inputs.BASE_SEED + 77)
        def bf16_dev(shape, sigma):
            return H.to_dev(inputs.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32) * sigma), "bf16")
        p8, mc8, d_model, d_ff = up.p, up.m_chunk, up.k, up.n           # 8, 1024, 8192, 3584
        cs, xs = torch.cuda.Stream(), torch.cuda.Stream()
        def timed(desc, kind, bufs, modes=BASIC):
            best = None
            for mode, extra in modes:
                t = time_calls(lambda: cf.run_schedule(desc, kind, bufs, cs, xs, extra), cs, max(K, 30), W)
                if best is None or t < best[0]:
                    best = (t, mode)
            return best
        flops = 2.0 * p8 * mc8 * d_model * d_ff
        mk32 = lambda r, c: torch.empty((r, c), dtype=torch.float32, device=H.DEV)
        # up-projection layer (all-gather layer, W [d_model x d_ff]): dX = RS(G W^T), dW = AG(X)^T G
        G_up = bf16_dev((p8 * mc8, d_ff), 1.0)
        W_up = bf16_dev((d_model, d_ff), 0.01)
        stage32 = [mk32(mc8, d_model).normal_() for _ in range(p8 - 1)]
        PERS = tuple(m for m in MODES if m[0] in BASIC_NAMES or ("persistent" in m[0] and "groups" not in m[0]))
        each32 = [mk32(mc8, d_model) for _ in range(p8 - 1)]
        keep = [mk32(mc8, d_model), [mk32(mc8, d_model) for _ in range(2)], [mk32(mc8, d_model) for _ in range(2)],
                [mk32(mc8, d_model) for _ in range(p8 - 1)]]
        bufs = cf.make_buffers(G_up, W_up, keep[0], stage32, keep[1], keep[2], None, each32, keep[3])   # (the tensors must outlive bufs)
        t = timed(cf.layer_desc(p8, 0, mc8, d_model, d_ff, "bf16", "f32", cf.CF_W_NK), cf.CF_KIND_RS, bufs, PERS)
        backward["up_dgrad_rs"] = {"us": round(t[0] * 1e3, 1), "tflops": round(flops / (t[0] * 1e-3) / 1e12, 1), "mode": t[1]}
        # the arriving slices land in ONE gathered buffer (own slice in row block rank = 0, hop i in row block
        # (rank - i) mod p): with CF_PERSISTENT the eight chunk GEMMs are then one GEMM over all its rows
        stage16 = [bf16_dev((mc8, d_model), 1.0) for _ in range(p8 - 1)]
        mk16 = lambda r, c: torch.empty((r, c), dtype=torch.bfloat16, device=H.DEV)
        gathered = mk16(p8 * mc8, d_model)
        blk = lambda c: gathered[c * mc8:(c + 1) * mc8]
        blk(0).copy_(bf16_dev((mc8, d_model), 1.0))
        land = [blk((0 - i) % p8) for i in range(1, p8)]
        dW_up = mk32(d_model, d_ff)
        slots16 = [mk16(mc8, d_model) for _ in range(2)]
        bufs = cf.make_buffers(blk(0), G_up, dW_up, stage16, slots16, (None, None), None, land)
        t = timed(cf.layer_desc(p8, 0, mc8, d_ff, d_model, "bf16", "f32"), cf.CF_KIND_WGRAD_X, bufs, PERS)
        backward["up_wgrad"] = {"us": round(t[0] * 1e3, 1), "tflops": round(flops / (t[0] * 1e-3) / 1e12, 1), "mode": t[1]}
        del G_up, stage32, stage16, bufs, dW_up, each32, keep
        torch.cuda.empty_cache()
        # down-projection layer (reduce-scatter layer, W [d_ff x d_model]): dA = AG(G) W^T, dW = A^T AG(G)
        W_dn = bf16_dev((d_ff, d_model), 0.01)
        G_own = bf16_dev((mc8, d_model), 1.0)
        stage16 = [bf16_dev((mc8, d_model), 1.0) for _ in range(p8 - 1)]
        each16 = [mk16(mc8, d_model) for _ in range(p8 - 1)]
        keep = [mk32(p8 * mc8, d_ff)]
        bufs = cf.make_buffers(G_own, W_dn, keep[0], stage16, slots16, (None, None), None, each16)
        t = timed(cf.layer_desc(p8, 0, mc8, d_ff, d_model, "bf16", "f32", cf.CF_W_NK), cf.CF_KIND_AG, bufs, PERS)
        backward["down_dgrad_ag"] = {"us": round(t[0] * 1e3, 1), "tflops": round(flops / (t[0] * 1e-3) / 1e12, 1), "mode": t[1]}
        A_loc = bf16_dev((p8 * mc8, d_ff), 1.0)
        blk(0).copy_(G_own)
        keep = [mk32(d_ff, d_model)]
        bufs = cf.make_buffers(blk(0), A_loc, keep[0], stage16, slots16, (None, None), None, land)
        t = timed(cf.layer_desc(p8, 0, mc8, d_model, d_ff, "bf16", "f32"), cf.CF_KIND_WGRAD_G, bufs, PERS)
        backward["down_wgrad"] = {"us": round(t[0] * 1e3, 1), "tflops": round(flops / (t[0] * 1e-3) / 1e12, 1), "mode": t[1]}
        total = sum(v["us"] for v in backward.values())
        backward["all_four_rank_steps"] = {"us": round(total, 1), "tflops": round(4 * flops / (total * 1e-6) / 1e12, 1)}
        log("backward", backward)
        del A_loc, stage16, bufs, W_dn, W_up, gathered, land, keep, slots16, each16
        torch.cuda.empty_cache()

    # ---------------- query-split attention FuseRS (Alg. 4), 70B shape: 8 of 64 heads per rank ----------------
    attention = {}
    if "attention" in sections:
        rng = np.random.default_rng(inputs.BASE_SEED + 78)
        pa, Ba, ha, Sa, Da = 8, 1, 8, 8192, 8192
        mca = Ba * Sa // pa
        def bf16_dev(shape, sigma):
            return H.to_dev(inputs.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32) * sigma), "bf16")
        Qa, Ka, Va = (bf16_dev((Ba, ha, Sa, 128), 1.0) for _ in range(3))
        Woa = bf16_dev((ha * 128, Da), 0.01)
        adesc = cf.attn_desc(pa, 0, Ba, ha, Sa, 128, Da, 1.0 / 128 ** 0.5)
        attn_out = torch.empty((pa * mca, ha * 128), dtype=torch.bfloat16, device=H.DEV)   # all p slices (persistent mode)
        mk32 = lambda: torch.empty((mca, Da), dtype=torch.float32, device=H.DEV)
        stage_a = [mk32().normal_() for _ in range(pa - 1)]
        keep = [mk32(), [mk32(), mk32()], [mk32(), mk32()], [mk32() for _ in range(pa - 1)], [mk32() for _ in range(pa - 1)]]
        abufs = cf.make_attn_buffers(Qa, Ka, Va, Woa, attn_out, keep[0], stage_a, keep[1], keep[2], None, keep[3], keep[4])
        cs, xs = torch.cuda.Stream(), torch.cuda.Stream()
        t_attn = time_calls(lambda: cf.attn_slice(adesc, 1, Qa, Ka, Va, attn_out, cs), cs, 50, W)
        fl_attn = 4.0 * Ba * ha * (Sa // pa) * Sa * 128
        fl_proj = 2.0 * mca * Da * ha * 128
        best = None
        attn_by_mode = {}
        for mode, extra in MODES:
            if "groups" in mode:                         # (the grouped launches exist for the plain RS / AG kinds)
                continue
            t = time_calls(lambda: cf.run_attn_schedule(adesc, abufs, cs, xs, extra), cs, max(K, 30), W)
            attn_by_mode[mode] = round(t * 1e3, 1)
            if best is None or t < best[0]:
                best = (t, mode)
        attention = {"attention_kernel_us": round(t_attn * 1e3, 1),
                     "attention_kernel_tflops": round(fl_attn / (t_attn * 1e-3) / 1e12, 1),
                     "frac_mfma_peak_attention_kernel": round(fl_attn / (t_attn * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                     "rank_step_us": round(best[0] * 1e3, 1), "mode": best[1], "rank_step_us_by_mode": attn_by_mode,
                     "rank_step_tflops": round(pa * (fl_attn + fl_proj) / (best[0] * 1e-3) / 1e12, 1),
                     "shape": "p=8, 8 of 64 heads per rank, head_dim 128, seq 8192, batch 1, W_o [1024 x 8192]"}
        log("attention", attention)
        del Qa, Ka, Va, Woa, abufs, stage_a, keep
        torch.cuda.empty_cache()

    # ---------------- gradient reduce-scatter step, 1e9 fp32 elements ----------------
    dp = None
    if "dp" in sections:
        w5 = inputs.CONFIGS["c5_dp"]
        log("generating the 1e9-element gradient bucket on the host (about half a minute) ...")
        t0 = time.time()
        run = H.DpRun(w5, inputs.make_dp(w5), 0)
        log(f"  done in {time.time()-t0:.0f} s")
        c = w5.m_chunk
        t_k = time_calls(lambda: cf.dp_reduce_step(w5.p, 0, 1, run.bucket, c, run.stage[0], run.cs), run.cs, 50, 5)
        gbs = 12.0 * c / (t_k * 1e-3) / 1e9
        t = schedule_times(run, cf.CF_KIND_DP, 10, 2)
        # CF_PERSISTENT: a landing buffer per hop, the seven deliveries as one batched copy, then the seven adds
        pers = H.DpRun.__new__(H.DpRun)
        pers.__dict__.update(run.__dict__)
        pers.each = [torch.empty((c,), dtype=torch.float32, device=H.DEV) for _ in range(w5.p - 1)]
        pers.bufs = cf.make_buffers(None, None, run.bucket, run.stage, run.slot, (None, None), None, pers.each)
        for name, fl in (("overlapped", 0), ("copy_only", cf.CF_NO_COMPUTE)):
            for mode, extra in (m_ for m_ in MODES if "persistent" in m_[0] and "groups" not in m_[0]):
                if fl != 0 and "carried" in mode:     # (the add kernels land what they read: no copy-only variant)
                    continue
                tp = time_calls(lambda: cf.run_schedule(pers.desc, cf.CF_KIND_DP, pers.bufs, pers.cs, pers.xs, fl | extra),
                                pers.cs, 10, 2)
                t["by_mode"].setdefault(mode, {})[name] = tp
                if tp < t[name][0]:
                    t[name] = (tp, mode)
        # pairwise schedule on the same bucket: seven arrivals for the own slice, summed in one pass (36 B per element)
        t_pw, pw_mode = min((time_calls(lambda: cf.run_schedule(pers.desc, cf.CF_KIND_DP_PAIR, pers.bufs, pers.cs, pers.xs, extra),
                                        pers.cs, 10, 2), mode) for mode, extra in MODES if "persistent" in mode and "groups" not in mode)
        t_pw_c = time_calls(lambda: cf.run_schedule(pers.desc, cf.CF_KIND_DP_PAIR, pers.bufs, pers.cs, pers.xs,
                                                    cf.CF_PERSISTENT | cf.CF_NO_COPY), pers.cs, 10, 2)
        steps_with_add = w5.p - 1
        dp = {"kernel_GBps": round(gbs, 1), "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4),
              "us_per_reduce_kernel": round(t_k * 1e3, 1), "bytes_per_elem": 12,
              "rank_step_us": round(t["overlapped"][0] * 1e3, 1), "rank_step_mode": t["overlapped"][1],
              "rank_step_GBps_algorithmic": round(12.0 * c * steps_with_add / (t["overlapped"][0] * 1e-3) / 1e9, 1),
              # bytes moved per element and hop: a copy (8) plus the add (12), or 16 where the add kernel reads the
              # neighbour's buffer and lands what it reads ("persistent+carried")
              "rank_step_bytes_per_elem_moved": 16 if "carried" in t["overlapped"][1] else 20,
              "rank_step_GBps_with_copies": round((16.0 if "carried" in t["overlapped"][1] else 20.0) * c * steps_with_add /
                                                  (t["overlapped"][0] * 1e-3) / 1e9, 1),
              "rank_step_us_by_mode": {m_: round(v["overlapped"] * 1e3, 1) for m_, v in t["by_mode"].items() if "overlapped" in v},
              **overlap_eff(t),
              "us_compute_only": round(t["compute_only"][0] * 1e3, 1), "us_copy_only": round(t["copy_only"][0] * 1e3, 1),
              "pairwise_rank_step_us": round(t_pw * 1e3, 1), "pairwise_rank_step_mode": pw_mode, "pairwise_us_compute_only": round(t_pw_c * 1e3, 1),
              "pairwise_add_GBps": round(4.0 * (w5.p + 1) * c / (t_pw_c * 1e-3) / 1e9, 1)}
        log("dp", dp)
        del run, pers
        torch.cuda.empty_cache()

    # ---------------- what bounds the main loop: the up-projection rank-step kernel under less electrical load ----------------
    # The same launch (same instructions, same memory traffic) on operands that are all zero toggles far fewer wires in
    # the matrix pipe; a grid capped below the chip leaves compute units idle.  If the launch were bound by its
    # instruction schedule or by memory, neither would change the time per unit of work.
    power = None
    if power_probe:
        up_w = inputs.CONFIGS["c4_ag_70b_up"]
        PSK = cf.CF_PERSISTENT | cf.CF_SERIAL | cf.CF_NO_COPY
        d_up = H.desc_of(up_w, 0)
        mk = lambda *shape: torch.randn(shape, dtype=torch.float32, device=H.DEV).to(torch.bfloat16)
        Xp = mk(up_w.m_chunk, up_w.k)
        each_p = [mk(up_w.m_chunk, up_w.k) for _ in range(up_w.p - 1)]
        slot_p = [torch.empty((up_w.m_chunk, up_w.k), dtype=torch.bfloat16, device=H.DEV) for _ in range(2)]
        Wp = mk(up_w.k, up_w.n) * 0.02
        Op = torch.empty((up_w.p * up_w.m_chunk, up_w.n), dtype=torch.bfloat16, device=H.DEV)
        bufs_p = cf.make_buffers(Xp, Wp, Op, each_p, slot_p, (None, None), None, each_p)
        cs_p, xs_p = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        launch = lambda: cf.run_schedule(d_up, cf.CF_KIND_AG, bufs_p, cs_p, xs_p, PSK)
        power = {"kernel": "up-projection rank-step kernel alone (8 x 1024x3584x8192, one persistent launch)", "random_data_us": {}}
        which = args.power_data
        if which in ("random", "both"):
            for wgs in (256, 224, 192, 160, 128):
                os.environ["COMMFUSE_PERSIST_WGS"] = str(wgs)
                t = time_calls(launch, cs_p, max(K, 30), W)
                power["random_data_us"][str(wgs) + "_workgroups"] = round(t * 1e3, 1)
                log(f"power probe: random data, {wgs} workgroups: {t*1e3:.1f} us = {up_w.flops/(t*1e-3)/1e12:.0f} TFLOP/s")
            os.environ.pop("COMMFUSE_PERSIST_WGS", None)
        if which in ("zero", "both"):
            for t_ in [Xp, Wp] + each_p:
                t_.zero_()
            torch.cuda.synchronize()
            t = time_calls(launch, cs_p, max(K, 30), W)
            power["zero_data_us"] = {"256_workgroups": round(t * 1e3, 1)}
            log(f"power probe: all-zero operands, 256 workgroups: {t*1e3:.1f} us = {up_w.flops/(t*1e-3)/1e12:.0f} TFLOP/s")
        del Xp, each_p, slot_p, Wp, Op, bufs_p
        torch.cuda.empty_cache()
        # Context, not a target and not part of the path: the vendor library's plain GEMM (torch.matmul) on the two whole
        # layers (no slicing, no B_in, no deliveries, bf16 output) under the same two kinds of operands, on this machine, in
        # this run; weights stored [k x n] as the path stores them, and [n x k].  On torch's current stream: on another
        # stream the library may pick a different kernel for want of a workspace.
        power["library_gemm_us"] = {}
        cur = torch.cuda.current_stream()
        for data in (("random",) if which == "random" else ("zero",) if which == "zero" else ("random", "zero")):
            for name, (gm, gn, gk) in (("down_8192x8192x3584", (dn.p * dn.m_chunk, dn.n, dn.k)), ("up_8192x3584x8192", (up_w.p * up_w.m_chunk, up_w.n, up_w.k))):
                Al = mk(gm, gk) if data == "random" else torch.zeros((gm, gk), dtype=torch.bfloat16, device=H.DEV)
                Wl = mk(gk, gn) * 0.02 if data == "random" else torch.zeros((gk, gn), dtype=torch.bfloat16, device=H.DEV)
                Wt = Wl.t().contiguous()              # the same weights stored [n x k]
                Ol = torch.empty((gm, gn), dtype=torch.bfloat16, device=H.DEV)
                for order, fn in (("w_kn", lambda: torch.matmul(Al, Wl, out=Ol)), ("w_nk", lambda: torch.matmul(Al, Wt.t(), out=Ol))):
                    t = time_calls(fn, cur, max(K, 30), W)
                    power["library_gemm_us"][f"{name}_{order}_{data}"] = round(t * 1e3, 1)
                    log(f"power probe: torch.matmul {name}, weights {order}, {data} operands: {t*1e3:.1f} us = {2.0*gm*gn*gk/(t*1e-3)/1e12:.0f} TFLOP/s")
                del Al, Wl, Wt, Ol
        torch.cuda.empty_cache()

    cf.device_status(None)                            # no step kernel gave up a device-side wait

    # ---------------- CPU oracle on a bounded sample of the headline workload ----------------
    cpu = None
    if not args.skip_cpu:
        import oracle
        # the GEMM work of one whole headline rank step: 8 down-projection and 8 up-projection chunk GEMMs
        dsm = inputs.make_rs(inputs.scaled(dn, p=1, m_chunk=dn.p * dn.m_chunk))
        usm = inputs.make_ag(inputs.scaled(up, p=1, m_chunk=up.p * up.m_chunk))
        A64, W64 = inputs.as_f64(dsm["A"], "bf16"), inputs.as_f64(dsm["W"], "bf16")
        X64, U64 = inputs.as_f64(usm["X"], "bf16"), inputs.as_f64(usm["W"], "bf16")
        oracle.gemm(A64[:64], W64)                                   # page in, spin up threads
        t0 = time.time()
        oracle.gemm(A64, W64)
        oracle.gemm(X64, U64)
        dt = time.time() - t0
        cpu = {"value": round(flops_pair / dt / 1e12, 5), "unit": "TFLOP/s", "cores": oracle.num_threads(),
               "kind": "oracle", "seconds": round(dt, 2),
               "sample": "the 16 chunk GEMMs of one headline rank step as two fp64 triple-loop products "
                         f"({dn.p * dn.m_chunk}x{dn.n}x{dn.k} and {up.p * up.m_chunk}x{up.n}x{up.k}), epilogue adds left out"}
        log("cpu", cpu)

    if args.calibration_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device=H.DEV)
        b = torch.empty(256 << 20, dtype=torch.uint8, device=H.DEV)
        a.fill_(1)
        b.copy_(a)                                                   # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()

    if args.skip_pair:                                # profiling run of one section: no headline, no contract line
        print(json.dumps({"sections": sorted(sections), "power_probe": power, "dp_reduce": dp, "other_configs": others, "pairwise_schedule": pairwise,
                          "slicing_granularity": granularity, "backward_pass": backward,
                          "query_split_attention": attention}), flush=True)
        return 0
    # overlap figures: every mode against ITS OWN compute-only and copy-only times (the fused-copy and
    # device-wait modes have no such variants and take the stream mode's)
    for mode, v in pair_by_mode.items():
        ref = pair_by_mode.get("persistent" if "persistent" in mode else "streams", {})
        comp, cpy = v.get("compute_only", ref.get("compute_only")), v.get("copy_only", ref.get("copy_only"))
        if "overlapped" in v and comp and cpy:
            pair_overlap[mode] = dict(us_per_step=round(v["overlapped"] * 1e3, 1), **overlap_of(v["overlapped"], comp, cpy))
    head_mode = pair_t["overlapped"][1]
    head = pair_by_mode[head_mode]
    head_comp = head.get("compute_only", pair_t["compute_only"][0])
    head_copy = head.get("copy_only", pair_t["copy_only"][0])
    line = {
        "metric": "rank-step TFLOP/s (% bf16 MFMA peak) + overlap efficiency; grad-reduce GB/s",
        "value": round(value, 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "Llama-70B-shape MLP pair rank step, p=8: AG-GEMM up [8x(1024x8192)]x[8192x3584] -> bf16 H, "
                               "GEMM-RS down [8x(1024x3584)]x[3584x8192] + fp32 partials; emulated ring on one GPU",
                   "p": 8, "rank": 0, "mode": head_mode, "us_per_step_by_mode": pair_modes,
                   "mode_note": "persistent = every delivery enqueued in front of ONE kernel per layer (nothing is hidden: "
                                "hidden_fraction ~ 0); persistent+carried = no copy is enqueued, that one kernel reads what the "
                                "neighbours send from their buffers under its main loop and stores it to this rank's landing "
                                "buffers; streams / graph / fused-copy / device-wait overlap each delivery with the step kernel "
                                "before it"},
        "frac_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4),
        # of the headline mode, against its own compute-only and copy-only times
        **overlap_of(ms_step, head_comp, head_copy),
        "overlap_by_mode": pair_overlap,
        "ms_compute_only": round(head_comp, 4), "ms_copy_only": round(head_copy, 4),
        "roofline": roofline, "cpu_baseline": cpu, "dp_reduce": dp, "other_configs": others,
        "vanilla_comparator": vanilla, "power_probe": power,
        "pairwise_schedule": pairwise, "slicing_granularity": granularity, "backward_pass": backward, "query_split_attention": attention,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
