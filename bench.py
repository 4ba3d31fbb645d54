#!/usr/bin/env python3
"""Benchmark of the GaussWS hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gpt2_124m|llama_1b]

A step is one pass of the whole hot path over every linear weight of the workload:
gws_sample_fwd (paper Eq. 3 + FP8-E4M3 cast) followed by gws_sample_bwd (Eq. 4, dL/dw
passed through as an alias).  Inputs are seeded synthetic tensors already resident in
HBM.  The last line printed is one JSON object (metric, roofline, cpu_baseline, extras).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense BF16, published
FWD_BYTES_PER_PARAM = 4.0      # read w (2) + write w_hat (2); + 8 B per 1024-param block (b_t, scale)
BWD_BYTES_PER_PARAM = 2.0      # read dL/dw_hat (2); dL/dw aliased; + 8 B per block (scale, db_t)
BLOCK_BYTES = 8.0
EVENT_EVERY = 4             # steps between event-bracketed steps in the timed region


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="llama_1b", choices=["gpt2_124m", "llama_1b"],
                    help="llama_1b (968.9 M params, the largest single-GPU configuration) or gpt2_124m (84.9 M)")
    ap.add_argument("--sets", type=int, default=0, help="distinct buffer sets rotated through (0 = auto)")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="run only the precision x format sweep of config 4 and print its JSON")
    ap.add_argument("--only-layer", action="store_true",
                    help="run only the decoder-layer comparison (five GEMMs per layer, sampling separate / riding) and print its JSON")
    ap.add_argument("--only-bases", action="store_true",
                    help="run only the noise-basis comparison (forward unit benchmark) and print its JSON")
    ap.add_argument("--only-linear", action="store_true",
                    help="run only the fused-linear comparison (config 5) and print its JSON (for profiling)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a plain 1 GiB device copy (reference dispatch for the HBM byte counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the GaussWS hot path needs no exchange "
              "between GPUs: blocks are independent and shards reproduce the noise from their origin). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2505_11170_amd as gws
    from paper_2505_11170_amd import binding, synth

    if not os.path.exists(binding.library_path()):
        from paper_2505_11170_amd.build import build_library
        build_library()
    gws.load_library()
    if not torch.cuda.is_available():
        raise RuntimeError("bench.py needs a GPU: the HIP path has no fallback")
    dev = "cuda:0"
    torch.cuda.set_device(0)

    def make_sets(shapes, n_sets, bt=None):
        """n_sets independent copies of (W, w_hat, b_t, scale, g, db_t) for every shape."""
        sets = []
        idx = 0
        for s in range(n_sets):
            descs = []
            for i, sh in enumerate(shapes):
                t = synth.make_tensor(idx, sh.rows, sh.cols, bt=bt, device=dev)
                idx += 1
                nbr, nbc = synth.n_blocks(sh.rows, sh.cols)
                descs.append(gws.TensorDesc(
                    rows=sh.rows, cols=sh.cols, seed=gws.gws_derive_seed(0, i), w=t["w"], w_hat=torch.empty_like(t["w"]),
                    bt=t["bt"], scale=torch.empty(nbr, nbc, device=dev), g=t["g"], dw=t["g"],
                    dbt=torch.empty(nbr, nbc, device=dev)))
            sets.append((descs, gws.pack(descs)))
        return sets

    def run_workload(shapes, steps, warmup, n_sets, fmt=gws.FMT_FP8_E4M3, bt=None, bitwidth=None):
        """bitwidth: a gws.Bitwidth turns the buffers named bt / dbt into b_i / db_i (paper Eq. 11, Eq. 12)."""
        params = sum(s.rows * s.cols for s in shapes)
        blocks = sum(synth.n_blocks(s.rows, s.cols)[0] * synth.n_blocks(s.rows, s.cols)[1] for s in shapes)
        sets = make_sets(shapes, n_sets, bt=bt)
        n_launch = (len(shapes) + 55) // 56
        if bitwidth is None:
            def fwd(p, step): gws.gws_sample_fwd(p, fmt, step)
            def bwd(p, step): gws.gws_sample_bwd(p, step)
        else:
            bws = gws.pack_bitwidth([bitwidth] * len(shapes))
            for descs, _ in sets:             # b_i ~ U[0, 1] from the U[4, 9] the generator gives for b_t
                for d in descs:
                    d.bt.sub_(4.0).div_(5.0)
            def fwd(p, step): gws.gws_sample_fwd_bi(p, bws, fmt, step)
            def bwd(p, step): gws.gws_sample_bwd_bi(p, bws, step)
        for s in range(warmup):
            _, p = sets[s % n_sets]
            fwd(p, s)
            bwd(p, s)
        # HIP events bracket the forward and the backward call of every EVENT_EVERY-th step of the
        # timed region (an event costs a few microseconds of stream time, which would otherwise
        # weigh on every step of a 0.1 ms step)
        sampled = [s for s in range(steps) if s % EVENT_EVERY == 0]
        ev = {s: [torch.cuda.Event(enable_timing=True) for _ in range(3)] for s in sampled}
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            _, p = sets[s % n_sets]
            e = ev.get(s)
            if e is None:
                fwd(p, warmup + s)
                bwd(p, warmup + s)
            else:
                e[0].record()
                fwd(p, warmup + s)
                e[1].record()
                bwd(p, warmup + s)
                e[2].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        fwd_all = sorted(ev[s][0].elapsed_time(ev[s][1]) for s in sampled)
        bwd_all = sorted(ev[s][1].elapsed_time(ev[s][2]) for s in sampled)
        fwd_ms, bwd_ms = sum(fwd_all) / len(fwd_all), sum(bwd_all) / len(bwd_all)
        return dict(params=params, blocks=blocks, n_launch=n_launch, wall_s=t1 - t0, fwd_ms=fwd_ms, bwd_ms=bwd_ms,
                    fwd_ms_median=fwd_all[len(fwd_all) // 2], fwd_ms_min=fwd_all[0],
                    bwd_ms_median=bwd_all[len(bwd_all) // 2], bwd_ms_min=bwd_all[0], sets=sets)

    if args.only_linear:
        print(json.dumps({"fused_linear": linear_bench(torch, gws, synth, dev)}))
        return
    if args.only_layer:
        print(json.dumps({"decoder_layer_forward": layer_bench(torch, gws, synth, dev)}))
        return
    if args.only_bases:
        sh = synth.llama_1b_shapes()
        print(json.dumps({"noise_bases_forward_unit_benchmark": basis_bench(torch, gws, synth, dev),
                          "noise_bases_fwd_bwd_llama_1b": basis_step_bench(torch, gws, synth, dev, sh, sum(s.rows * s.cols for s in sh))}))
        return

    if args.sweep:
        # config 4: noise precision {4..9, U[4,9]} x target {FP6-E3M2, FP8-E4M3, BF16} on the 1B weights
        shapes4 = synth.llama_1b_shapes()
        p4 = sum(s.rows * s.cols for s in shapes4)
        cells = {}
        for fmt_name, fmt in (("fp6_e3m2", gws.FMT_FP6_E3M2), ("fp8_e4m3", gws.FMT_FP8_E4M3), ("bf16", gws.FMT_BF16)):
            for bt in (4.0, 5.0, 6.0, 7.0, 8.0, 9.0, None):
                r4 = run_workload(shapes4, 40, 20, 1, fmt=fmt, bt=bt)
                fb = FWD_BYTES_PER_PARAM * p4 + BLOCK_BYTES * r4["blocks"]
                bb = BWD_BYTES_PER_PARAM * p4 + BLOCK_BYTES * r4["blocks"]
                cells[f"{fmt_name}/bt={'U[4,9]' if bt is None else int(bt)}"] = {
                    "params_per_s": p4 * 40 / r4["wall_s"], "fwd_ms": r4["fwd_ms"], "bwd_ms": r4["bwd_ms"],
                    "fwd_GBps": fb / r4["fwd_ms"] / 1e6, "bwd_GBps": bb / r4["bwd_ms"] / 1e6,
                    "step_frac_of_hbm_peak": (fb + bb) / (r4["wall_s"] / 40) / 1e9 / HBM_PEAK_GBS}
                del r4
                torch.cuda.empty_cache()
        print(json.dumps({"config4_sweep": cells}))
        return

    shapes = synth.gpt2_124m_shapes() if args.workload == "gpt2_124m" else synth.llama_1b_shapes()
    params = sum(s.rows * s.cols for s in shapes)
    # Rotate through enough distinct buffer sets that no operand can still sit in the 256 MB
    # last-level cache when it is touched again (each set is 6 bytes per parameter per step).
    n_sets = args.sets or max(1, min(8, int(1.5e9 // (6 * params)) + 1))
    res = run_workload(shapes, args.steps, args.warmup, n_sets)
    ms_per_step = res["wall_s"] * 1e3 / args.steps
    value = params * args.steps / res["wall_s"]
    fwd_bytes = FWD_BYTES_PER_PARAM * params + BLOCK_BYTES * res["blocks"]
    bwd_bytes = BWD_BYTES_PER_PARAM * params + BLOCK_BYTES * res["blocks"]
    pair_ms = empty_event_pair_ms(torch)
    out = {
        "metric": "GaussWS fwd+bwd sampled params/s",
        "value": value,
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: all {len(shapes)} linear weights, {params} params, W~N(0,0.02) BF16, "
                               "b_t~U[4,9] per 32x32 block, dW~N(0,1e-3), FP8-E4M3 cast, fwd+bwd (dW aliased), "
                               f"{n_sets} buffer sets rotated",
                   "params": params, "buffer_sets": n_sets, "launches_per_pass": res["n_launch"]},
        "step_GBps": (fwd_bytes + bwd_bytes) / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": (fwd_bytes + bwd_bytes) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": roofline_block(res, fwd_bytes, bwd_bytes, pair_ms, args.workload),
        "paper_context": "paper reports 1.40% end-to-end tokens/s overhead (Llama2-134M, A100-40G, Table 1); "
                         "no params/s or GB/s figure exists for this path",
    }
    ceilings(torch, gws, res, params, n_sets, pair_ms, out["roofline"])
    # ---- cpu_baseline: the oracle, as it stands, on a bounded sample of the same workload ----
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(synth, res["sets"][0][0], args.workload)
    del res

    # ---- extras: other configurations, outside the timed region ----
    if not args.no_extras:
        extras = {}
        torch.cuda.empty_cache()
        try:
            other = synth.llama_1b_shapes() if args.workload == "gpt2_124m" else synth.gpt2_124m_shapes()
            name = "llama_1b" if args.workload == "gpt2_124m" else "gpt2_124m"
            op = sum(s.rows * s.cols for s in other)
            o_sets = max(1, min(8, int(1.5e9 // (6 * op)) + 1))
            r2 = run_workload(other, 60, 20, o_sets)
            fb = FWD_BYTES_PER_PARAM * op + BLOCK_BYTES * r2["blocks"]
            bb = BWD_BYTES_PER_PARAM * op + BLOCK_BYTES * r2["blocks"]
            extras[name] = {"params": op, "params_per_s": op * 60 / r2["wall_s"], "ms_per_step": r2["wall_s"] * 1e3 / 60,
                            "fwd_ms": r2["fwd_ms"], "bwd_ms": r2["bwd_ms"], "buffer_sets": o_sets,
                            "step_frac_of_hbm_peak": (fb + bb) / (r2["wall_s"] / 60) / 1e9 / HBM_PEAK_GBS,
                            "roofline": roofline_block(r2, fb, bb, pair_ms, name)}
            del r2
            torch.cuda.empty_cache()
        except Exception as e:  # pragma: no cover
            extras["other_workload_error"] = repr(e)
        try:
            # the same step with the bitwidth given through b_i (Eq. 11) and the loss term of Eq. 12
            # (timed next to a control run of the plain entry points with the same step counts)
            r3 = run_workload(shapes, 100, 50, n_sets, bitwidth=gws.Bitwidth(6.0, 4.0, 1e-3))
            rc = run_workload(shapes, 100, 50, n_sets)
            extras["parametrised_bitwidth"] = {"params_per_s": params * 100 / r3["wall_s"], "fwd_ms": r3["fwd_ms"],
                                               "bwd_ms": r3["bwd_ms"], "b_init": 6.0, "b_target": 4.0, "lambda": 1e-3,
                                               "control_plain": {"params_per_s": params * 100 / rc["wall_s"],
                                                                 "fwd_ms": rc["fwd_ms"], "bwd_ms": rc["bwd_ms"]}}
            del rc
            del r3
            torch.cuda.empty_cache()
        except Exception as e:  # pragma: no cover
            extras["parametrised_bitwidth_error"] = repr(e)
        try:
            # config 1: one 768x768 weight, forward only; a latency-bound launch
            t1 = synth.make_tensor(0, 768, 768, bt=6.0, device=dev, with_grad=False)
            d1 = gws.pack([gws.TensorDesc(rows=768, cols=768, seed=gws.gws_derive_seed(0, 0), w=t1["w"],
                                          w_hat=torch.empty_like(t1["w"]), bt=t1["bt"],
                                          scale=torch.empty(24, 24, device=dev))])
            ms1 = _time_ms(torch, lambda: gws.gws_sample_fwd(d1, gws.FMT_FP8_E4M3, 0), 200, warmup=20)
            extras["config1_768x768_fwd"] = {"us_per_call_back_to_back": ms1 * 1e3,
                                             "GBps": (4.0 * 768 * 768 + 8 * 576) / ms1 / 1e6}
            # the same 20 calls recorded once into a HIP graph and replayed
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for _ in range(20):
                    gws.gws_sample_fwd(d1, gws.FMT_FP8_E4M3, 0)
            msg = _time_ms(torch, graph.replay, 20, warmup=3) / 20
            extras["config1_768x768_fwd"]["us_per_call_in_a_graph_of_20"] = msg * 1e3
            del graph
        except Exception as e:  # pragma: no cover
            extras["config1_error"] = repr(e)
        try:
            extras["mx_output"] = mx_bench(torch, gws, synth, dev, shapes, params)
        except Exception as e:  # pragma: no cover
            extras["mx_output_error"] = repr(e)
        try:
            extras["noise_bases_forward_unit_benchmark"] = basis_bench(torch, gws, synth, dev)
            extras["noise_bases_fwd_bwd_" + args.workload] = basis_step_bench(torch, gws, synth, dev, shapes, params)
        except Exception as e:  # pragma: no cover
            extras["noise_bases_error"] = repr(e)
        try:
            extras["copy_ceiling"] = copy_ceiling(torch)
            extras["fused_linear"] = linear_bench(torch, gws, synth, dev)
        except Exception as e:  # pragma: no cover
            extras["linear_error"] = repr(e)
        try:
            extras["decoder_layer_forward"] = layer_bench(torch, gws, synth, dev)
        except Exception as e:  # pragma: no cover
            extras["decoder_layer_error"] = repr(e)
        # Context only, derived from the figures above (nothing here is measured end to end): what share
        # of a training step the sampling of every weight would take if the step's GEMMs (6 FLOP per
        # parameter and token) ran at the plain BF16 GEMM rate measured above.
        try:
            l1b = extras["llama_1b"] if "llama_1b" in extras else None
            tf = extras["fused_linear"]["plain_torch_TFLOPs"]
            if l1b is not None:
                sample_ms = 1e3 * l1b["params"] / l1b["params_per_s"]
                est = {}
                for tokens in (16384, 49152):
                    gemm_ms = 6.0 * l1b["params"] * tokens / (tf * 1e12) * 1e3
                    est[str(tokens)] = {"gemm_ms_at_plain_rate": gemm_ms, "sampling_fwd_bwd_ms": sample_ms,
                                        "sampling_share_pct": 100.0 * sample_ms / gemm_ms}
                extras["amortised_estimate_llama_1b"] = {
                    "per_tokens_per_step": est,
                    "note": "derived, not measured: sampling fwd+bwd of all 154 weights once per optimizer step against "
                            "6*params*tokens FLOP at the measured plain BF16 GEMM rate; the paper's Table 1 reports 1.92 % "
                            "tokens/s overhead for Llama2-1B on an A100 at 16384 tokens per GPU and step"}
        except Exception as e:  # pragma: no cover
            extras["amortised_estimate_error"] = repr(e)
        out["extras"] = extras

    if args.calibrate:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()

    print(json.dumps(out))


def empty_event_pair_ms(torch):
    """What an event pair with nothing between reads (the second event's own stream time), median of 50."""
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
    for a, b in pairs:
        a.record()
        b.record()
    torch.cuda.synchronize()
    return sorted(a.elapsed_time(b) for a, b in pairs)[len(pairs) // 2]


def traffic_from_profile(workload, kernel=r"sample_fwd\w*_kernel"):
    """HBM bytes per launch of `kernel` as the committed rocprofv3 --pmc summary of this workload states them
    (FETCH_SIZE and WRITE_SIZE runs of this script, each scaled by a 1 GiB plain device copy of the same run).
    Returns (bytes or None, where the figure comes from)."""
    import re
    path = os.path.join(ROOT, "profiles", f"sample_kernels_{workload}.md")
    try:
        text = open(path).read()
    except OSError:
        return None, None
    mb = re.findall(rf"{kernel}: raw \d+ KiB/dispatch -> ([0-9.]+) MB/dispatch", text)
    if len(mb) != 2:
        return None, None
    at = re.search(r"measured at: *(.+)", text)
    return (float(mb[0]) + float(mb[1])) * 1e6, (f"profiles/sample_kernels_{workload}.md: rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE per dispatch, scaled "
                                                  "by a 1 GiB device copy of the same run" + (f"; measured at {at.group(1).strip()}" if at else "")
                                                  + " (a figure of that profiling run, not of this one)")


def roofline_block(res, fwd_bytes, bwd_bytes, pair_ms, workload):
    """Roofline of the dominant kernel (forward) and, inside it, of the backward kernel.  `achieved` / `frac`
    use the time between the HIP events that bracket the call, as read; the *_event_overhead_removed figures
    take off what an empty event pair reads, which is what agrees with rocprofv3 --kernel-trace durations."""
    nl = res["n_launch"]

    def one(call_ms, nbytes):
        raw = call_ms / nl
        corr = max(call_ms - pair_ms, 0.5 * call_ms) / nl
        return raw, corr, (nbytes / nl) / (raw * 1e-3) / 1e9, (nbytes / nl) / (corr * 1e-3) / 1e9

    f_raw, f_corr, f_gbs, f_gbs_corr = one(res["fwd_ms"], fwd_bytes)
    b_raw, b_corr, b_gbs, b_gbs_corr = one(res["bwd_ms"], bwd_bytes)
    traffic, source = traffic_from_profile(workload)
    return {"kernel": "sample_fwd_full_kernel<FP8_E4M3>", "bound": "hbm", "achieved": f_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": f_gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": source,
            "launch_ms": f_raw, "bytes_per_launch": fwd_bytes / nl,
            "achieved_event_overhead_removed": f_gbs_corr, "frac_event_overhead_removed": f_gbs_corr / HBM_PEAK_GBS,
            "launch_ms_event_overhead_removed": f_corr,
            "timing": f"HIP events around the call on every {EVENT_EVERY}th step of the timed region, divided by the launches per "
                      "call; the *_event_overhead_removed figures subtract the reading of an empty event pair first",
            "call_ms_between_events": res["fwd_ms"], "call_ms_between_events_median": res["fwd_ms_median"],
            "call_ms_between_events_min": res["fwd_ms_min"], "empty_event_pair_ms": pair_ms,
            "bwd": {"kernel": "sample_bwd_full_kernel", "launch_ms": b_raw, "bytes_per_launch": bwd_bytes / nl,
                    "call_ms_between_events": res["bwd_ms"], "call_ms_between_events_median": res["bwd_ms_median"],
                    "call_ms_between_events_min": res["bwd_ms_min"], "achieved": b_gbs, "frac": b_gbs / HBM_PEAK_GBS,
                    "achieved_event_overhead_removed": b_gbs_corr, "frac_event_overhead_removed": b_gbs_corr / HBM_PEAK_GBS,
                    "launch_ms_event_overhead_removed": b_corr}}


def ceilings(torch, gws, res, params, n_sets, pair_ms, roof):
    """The same bytes moved by kernels with the sampling kernels' launch shape, loads and stores and no
    arithmetic (include/gws_bench.h): the rates the memory system allows for the two access patterns."""
    nl = res["n_launch"]

    def timed(call):
        for _ in range(20):
            call()
        ev = []
        for _ in range(25):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            call()
            e1.record()
            for _ in range(3):
                call()
            ev.append((e0, e1))
        torch.cuda.synchronize()
        return max(sum(a.elapsed_time(b) for a, b in ev) / len(ev) - pair_ms, 1e-6) / nl

    k = [0]

    def copy_call():
        k[0] += 1
        gws.gws_copy_tiles(res["sets"][k[0] % n_sets][1])
    copy_ms = timed(copy_call)
    copy_gbps = (FWD_BYTES_PER_PARAM * params / nl) / (copy_ms * 1e-3) / 1e9   # 2 B read + 2 B written
    # the backward pass's ceiling: its launch shape, the same gradient buffers read once, 4 bytes written per block
    absmax_sets = [gws.pack([gws.TensorDesc(rows=d.rows, cols=d.cols, seed=0, w=d.g, scale=d.dbt) for d in descs])
                   for descs, _ in res["sets"]]

    def read_call():
        k[0] += 1
        gws.gws_block_absmax(absmax_sets[k[0] % n_sets])
    read_ms = timed(read_call)
    read_gbps = ((2.0 * params + 4.0 * res["blocks"]) / nl) / (read_ms * 1e-3) / 1e9
    roof["bwd"]["read_same_pattern"] = {"kernel": "block_absmax_kernel", "launch_ms": read_ms, "GBps": read_gbps,
                                        "frac_of_hbm_peak": read_gbps / HBM_PEAK_GBS,
                                        "bwd_frac_of_this_ceiling": roof["bwd"]["achieved_event_overhead_removed"] / read_gbps}
    roof["copy_same_pattern"] = {"kernel": "copy_tiles_kernel", "launch_ms": copy_ms, "GBps": copy_gbps,
                                 "frac_of_hbm_peak": copy_gbps / HBM_PEAK_GBS,
                                 "fwd_frac_of_this_ceiling": roof["achieved_event_overhead_removed"] / copy_gbps}


def cpu_baseline(synth, descs, workload):
    """The oracle (oracle/gws_oracle.c, never tuned for this) timed on the host cores: all threads on a prefix of
    the workload of at most ~1.7e8 parameters, and one thread on the first decoder layer / transformer block."""
    import oracle
    cores = oracle.set_threads(0)
    sample, sp = [], 0
    for d in descs:
        if sample and sp + d.rows * d.cols > 170_000_000:
            break
        sample.append(d)
        sp += d.rows * d.cols
    host = [(synth.bits(d.w), d.bt.cpu().numpy(), synth.bits(d.g), d.seed) for d in sample]
    passes, dt = 0, 0.0
    t0 = time.perf_counter()
    while passes < 8 and dt < 1.0:        # about 1-2 s on all host threads: 15-30 s of CPU work
        for (w, bt, g, seed) in host:
            _, sc = oracle.sample_fwd(w, bt, oracle.FMT_FP8_E4M3, seed, passes)
            oracle.sample_bwd(g, sc, seed, passes)
        passes += 1
        dt = time.perf_counter() - t0
    out = {"value": sp * passes / dt, "unit": "params/s", "cores": cores, "kind": "oracle",
           "sample": f"first {len(sample)} tensors of {workload} ({sp} params), {passes} fwd+bwd steps, "
                     f"{dt:.2f} s wall on {cores} threads"}
    # the same oracle on one thread: one layer of the model (7 weights of the 1B decoder, 4 of GPT2-124M)
    per_layer = 7 if workload == "llama_1b" else 4
    oracle.set_threads(1)
    lp = sum(d.rows * d.cols for d in sample[:per_layer])
    t0 = time.perf_counter()
    for (w, bt, g, seed) in host[:per_layer]:
        _, sc = oracle.sample_fwd(w, bt, oracle.FMT_FP8_E4M3, seed, 0)
        oracle.sample_bwd(g, sc, seed, 0)
    dt1 = time.perf_counter() - t0
    oracle.set_threads(0)
    out["single_thread"] = {"value": lp / dt1, "unit": "params/s", "cores": 1,
                            "sample": f"first layer of {workload} ({per_layer} weights, {lp} params), one fwd+bwd step, {dt1:.2f} s"}
    return out


def _time_ms(torch, fn, iters, warmup=3):
    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def bwd_w_shapes_bench(torch, gws, synth, dev, tokens=8192):
    """Weight gradient + dL/db_t of the four weight shapes of a 1B decoder layer: the one-kernel form, the form with
    the tokens split into parts through a workspace (weights of few tiles), and torch.matmul(x.T, dy) (no dL/db_t)."""
    out = {}
    for name, K, N in (("qkv", 2048, 2560), ("o", 2048, 2048), ("gate_up", 2048, 5632), ("down", 5632, 2048)):
        x = synth.make_activation(90, tokens, K, device=dev)
        dy = (synth.make_activation(91, tokens, N, device=dev).float() * 1e-3).to(torch.bfloat16)
        dw = torch.zeros(K, N, dtype=torch.bfloat16, device=dev)
        d = gws.TensorDesc(rows=K, cols=N, seed=1, scale=torch.full((K // 32, N // 32), 1e-3, device=dev), dw=dw,
                           dbt=torch.zeros(K // 32, N // 32, device=dev))
        need = gws.gws_linear_bwd_w_workspace_bytes(d, tokens)
        ws = torch.empty(need // 4, device=dev) if need else None
        xt = x.t()
        variants = {"one_kernel_ms": lambda: gws.gws_linear_bwd_w(x, dy, d, 3),
                    "split_ms": lambda: gws.gws_linear_bwd_w_ws(x, dy, d, 3, ws),
                    "torch_matmul_ms": lambda: torch.matmul(xt, dy, out=dw)}
        bursts = {k: [] for k in variants}
        for _ in range(5):
            for k, fn in variants.items():
                bursts[k].append(_time_ms(torch, fn, 6, warmup=1))
        r = {k: sorted(v)[len(v) // 2] for k, v in bursts.items()}
        r["tiles"] = (K // 256) * (N // 256)
        r["workspace_MiB"] = need / 2 ** 20
        r["parts"] = need // (r["tiles"] * 256 * 256 * 4) if need else 1
        out[f"{name}_{K}x{N}"] = r
    return out


def mx_bench(torch, gws, synth, dev, shapes, params):
    """Forward pass writing MX element codes + E8M0 block scales instead of the BF16 container."""
    out = {}
    blocks = sum(synth.n_blocks(s.rows, s.cols)[0] * synth.n_blocks(s.rows, s.cols)[1] for s in shapes)
    for name, fmt, bpp in (("fp8_e4m3", gws.FMT_FP8_E4M3, 1.0), ("fp6_e3m2", gws.FMT_FP6_E3M2, 0.75)):
        sets = []
        for k in range(3):      # rotate three buffer sets, as the main measurement does
            descs, outs = [], []
            for i, sh in enumerate(shapes):
                t = synth.make_tensor(100 * k + i, sh.rows, sh.cols, device=dev, with_grad=False)
                nbr, nbc = synth.n_blocks(sh.rows, sh.cols)
                ldc = sh.cols if fmt == gws.FMT_FP8_E4M3 else sh.cols * 6 // 8
                descs.append(gws.TensorDesc(rows=sh.rows, cols=sh.cols, seed=gws.gws_derive_seed(0, i), w=t["w"],
                                            bt=t["bt"], scale=torch.empty(nbr, nbc, device=dev)))
                outs.append(gws.MxOut(torch.empty(sh.rows, ldc, dtype=torch.uint8, device=dev),
                                      torch.empty(nbr, nbc, dtype=torch.uint8, device=dev), ldc))
            sets.append((gws.pack(descs), gws.pack_mx(outs)))
        step = [0]

        def fn():
            p, o = sets[step[0] % 3]
            gws.gws_sample_fwd_mx(p, o, fmt, step[0])
            step[0] += 1
        ms = _time_ms(torch, fn, 60, warmup=20)
        nbytes = (2.0 + bpp) * params + 9.0 * blocks
        out[name] = {"fwd_ms": ms, "params_per_s": params / ms * 1e3, "bytes_per_param": 2.0 + bpp,
                     "GBps": nbytes / ms / 1e6, "frac_of_hbm_peak": nbytes / ms / 1e6 / HBM_PEAK_GBS}
        del sets
        torch.cuda.empty_cache()
    return out


def basis_bench(torch, gws, synth, dev):
    """The shape of the paper's forward unit benchmark (Sec. 4 "Overhead", Fig. 7: Eq. 3 on a matrix w_(M,N), in
    10^9 elements/s, "ours" against a Box-Muller rounded normal) on this hardware, plus the BF16 uniform basis of
    the paper's DiffQ extension: gws_sample_fwd against gws_sample_fwd_basis, BF16 target as in the paper's runs.
    Shapes: the ends of the ranges the paper names for Llama 3.2 1B and Llama 3.1 405B weights."""
    out = {}
    bases = (("ours_bits", gws.BASIS_BITS), ("box_muller", gws.BASIS_BOX_MULLER), ("uniform_bf16", gws.BASIS_UNIFORM_BF16))
    for rows, cols in ((2048, 512), (2048, 2048), (2048, 8192), (16384, 1024), (16384, 16384)):
        n_buf = max(2, min(8, int(6e8 // (rows * cols * 4)) + 1))        # rotate past the last-level cache where that is cheap
        packs = []
        for k in range(n_buf):
            t = synth.make_tensor(40 + k, rows, cols, device=dev, with_grad=False)
            packs.append(gws.pack([gws.TensorDesc(rows=rows, cols=cols, seed=gws.gws_derive_seed(1, k), w=t["w"],
                                                  w_hat=torch.empty_like(t["w"]), bt=t["bt"],
                                                  scale=torch.empty(rows // 32, cols // 32, device=dev))]))
        cell = {}
        for name, basis in bases:
            k = [0]

            def fn():
                k[0] += 1
                gws.gws_sample_fwd_basis(packs[k[0] % n_buf], basis, gws.FMT_BF16, k[0])
            iters = 200 if rows * cols < 1 << 24 else 30
            ms = _time_ms(torch, fn, iters, warmup=10)
            cell[name] = {"us_per_call": ms * 1e3, "gelem_per_s": rows * cols / ms / 1e6}
        cell["box_muller_over_ours"] = cell["box_muller"]["us_per_call"] / cell["ours_bits"]["us_per_call"]
        cell["uniform_over_ours"] = cell["uniform_bf16"]["us_per_call"] / cell["ours_bits"]["us_per_call"]
        out[f"{rows}x{cols}"] = cell
        del packs
        torch.cuda.empty_cache()
    return out


def basis_step_bench(torch, gws, synth, dev, shapes, params):
    """fwd+bwd over a whole workload per noise basis (what the paper's Table 1 contrasts as GaussWS against DiffQ,
    there inside a training step)."""
    out = {}
    descs = []
    for i, sh in enumerate(shapes):
        t = synth.make_tensor(i, sh.rows, sh.cols, device=dev)
        nbr, nbc = synth.n_blocks(sh.rows, sh.cols)
        descs.append(gws.TensorDesc(rows=sh.rows, cols=sh.cols, seed=gws.gws_derive_seed(0, i), w=t["w"], w_hat=torch.empty_like(t["w"]),
                                    bt=t["bt"], scale=torch.empty(nbr, nbc, device=dev), g=t["g"], dw=t["g"],
                                    dbt=torch.empty(nbr, nbc, device=dev)))
    pk = gws.pack(descs)
    for name, basis in (("ours_bits", gws.BASIS_BITS), ("box_muller", gws.BASIS_BOX_MULLER), ("uniform_bf16", gws.BASIS_UNIFORM_BF16)):
        k = [0]

        def fn():
            k[0] += 1
            gws.gws_sample_fwd_basis(pk, basis, gws.FMT_FP8_E4M3, k[0])
            gws.gws_sample_bwd_basis(pk, basis, k[0])
        ms = _time_ms(torch, fn, 30, warmup=10)
        out[name] = {"ms_per_step": ms, "params_per_s": params / ms * 1e3}
    out["box_muller_over_ours"] = out["box_muller"]["ms_per_step"] / out["ours_bits"]["ms_per_step"]
    out["uniform_over_ours"] = out["uniform_bf16"]["ms_per_step"] / out["ours_bits"]["ms_per_step"]
    return out


def layer_bench(torch, gws, synth, dev, tokens=8192, layers=4):
    """The sampled-weight linear at the level the method is used: the five GEMMs of a Llama-style 1B decoder layer
    (hidden 2048, fused q/k/v of 2560 outputs, SwiGLU intermediate 5632) over `tokens` tokens, `layers` layers in a
    row.  Plain BF16 GEMMs on the stored weights against the same GEMMs on sampled weights, the sampling done
      separate: by gws_linear_fwd (sampling kernel, then GEMM) for every weight;
      riding:   inside the launch of an earlier GEMM wherever that GEMM's last round of tiles leaves compute units
                idle (gws_gemm_bf16_sample_next_n): q/k/v's GEMM (320 tiles, 192 units idle in its second round)
                carries w_o, w_gate and the next layer's w_qkv; gate's and up's GEMMs (704 tiles, 64 idle) carry
                w_up and w_down; o's and down's GEMMs fill the chip exactly (256 tiles) and carry nothing.
    Attention and the activation function are left out: every GEMM runs on a fixed input of its shape."""
    H, QKV, FF = 2048, 2560, 5632
    fmt = gws.FMT_FP8_E4M3
    shapes = {"qkv": (H, QKV), "o": (H, H), "gate": (H, FF), "up": (H, FF), "down": (FF, H)}   # stored [K x N]
    order = ["qkv", "o", "gate", "up", "down"]
    x_h = synth.make_activation(60, tokens, H, device=dev)
    x_ff = synth.make_activation(61, tokens, FF, device=dev)
    outs = {n: torch.empty(tokens, shapes[n][1], dtype=torch.bfloat16, device=dev) for n in order}
    inp = {"qkv": x_h, "o": x_h, "gate": x_h, "up": x_h, "down": x_ff}
    W = []
    for l in range(layers):
        lw = {}
        for k, n in enumerate(order):
            r, c = shapes[n]
            t = synth.make_tensor(70 + 5 * l + k, r, c, bt=6.0, device=dev, with_grad=False)
            lw[n] = gws.TensorDesc(rows=r, cols=c, seed=gws.gws_derive_seed(2, 5 * l + k), w=t["w"], w_hat=torch.empty_like(t["w"]),
                                   bt=t["bt"], scale=torch.empty(r // 32, c // 32, device=dev))
        W.append(lw)
    step = [0]

    def plain():
        for l in range(layers):
            for n in order:
                gws.gws_gemm_bf16(inp[n], W[l][n].w, outs[n])

    def plain_torch():
        for l in range(layers):
            for n in order:
                torch.matmul(inp[n], W[l][n].w, out=outs[n])

    def plain_on_w_hat():            # the same GEMMs on weights sampled beforehand: what the sampling itself adds is
        for l in range(layers):      # the difference to this (GEMM time depends on the operand values: fewer bits toggle)
            for n in order:
                gws.gws_gemm_bf16(inp[n], W[l][n].w_hat, outs[n])

    def torch_on_w_hat():
        for l in range(layers):
            for n in order:
                torch.matmul(inp[n], W[l][n].w_hat, out=outs[n])

    def separate():
        step[0] += 1
        for l in range(layers):
            for n in order:
                gws.gws_linear_fwd(inp[n], W[l][n], outs[n], fmt, step[0])

    # what each GEMM is asked to carry (the library decides what fits; the rest follows the GEMM as a launch)
    def carried(l):
        nxt_qkv = [W[l + 1]["qkv"]] if l + 1 < layers else []
        return {"qkv": [W[l]["o"], W[l]["gate"]] + nxt_qkv, "o": [], "gate": [W[l]["up"]], "up": [W[l]["down"]], "down": []}

    def riding():
        step[0] += 1
        gws.gws_sample_fwd([W[0]["qkv"]], fmt, step[0])
        for l in range(layers):
            c = carried(l)
            for n in order:
                gws.gws_gemm_bf16_sample_next_n(inp[n], W[l][n].w_hat, outs[n], c[n], fmt, step[0])

    plan = {n: f"{gws.gws_ride_plan(tokens, shapes[n][0], shapes[n][1], carried(0)[n]) if carried(0)[n] else 0} of {len(carried(0)[n])} ride"
            for n in order}
    # the riding schedule produces the same sampled weights as gws_sample_fwd
    riding()
    ref = gws.TensorDesc(rows=H, cols=FF, seed=W[1]["up"].seed, w=W[1]["up"].w, w_hat=torch.empty_like(W[1]["up"].w),
                         bt=W[1]["up"].bt, scale=torch.empty(H // 32, FF // 32, device=dev))
    gws.gws_sample_fwd([ref], fmt, step[0])
    torch.cuda.synchronize()
    same = bool(torch.equal(ref.w_hat.view(torch.int16), W[1]["up"].w_hat.view(torch.int16)))
    # ---- the layer's backward GEMMs: dX = dY * W^T (on w_hat in the sampled run) and dW = X^T dY (+ dL/db_t) ----
    dys = {n: (synth.make_activation(62 + k, tokens, shapes[n][1], device=dev).float() * 1e-3).to(torch.bfloat16) for k, n in enumerate(order)}
    dxs = {n: torch.empty(tokens, shapes[n][0], dtype=torch.bfloat16, device=dev) for n in order}
    G = []                                    # per layer and weight: descriptors of the gradient, plain and with dL/db_t
    ws_bytes = 0
    for l in range(layers):
        lg = {}
        for n in order:
            r, c = shapes[n]
            dw = torch.empty(r, c, dtype=torch.bfloat16, device=dev)
            lg[n] = (gws.TensorDesc(rows=r, cols=c, seed=W[l][n].seed, dw=dw),
                     gws.TensorDesc(rows=r, cols=c, seed=W[l][n].seed, dw=dw, scale=W[l][n].scale, dbt=torch.empty(r // 32, c // 32, device=dev)))
            ws_bytes = max(ws_bytes, gws.gws_linear_bwd_w_workspace_bytes(lg[n][0], tokens))
        G.append(lg)
    ws = torch.empty(ws_bytes // 4, device=dev) if ws_bytes else None

    def bwd_plain():
        for l in reversed(range(layers)):
            for n in reversed(order):
                gws.gws_gemm_bf16(dys[n], W[l][n].w, dxs[n], w_is_nk=True)          # the [K x N] weight read as [N' x K'] = dY * W^T
                gws.gws_linear_bwd_w_ws(inp[n], dys[n], G[l][n][0], 0, ws)

    def bwd_torch():
        for l in reversed(range(layers)):
            for n in reversed(order):
                torch.matmul(dys[n], W[l][n].w.t(), out=dxs[n])
                torch.matmul(inp[n].t(), dys[n], out=G[l][n][0].dw)

    def bwd_sampled():
        for l in reversed(range(layers)):
            for n in reversed(order):
                gws.gws_gemm_bf16(dys[n], W[l][n].w_hat, dxs[n], w_is_nk=True)
                gws.gws_linear_bwd_w_ws(inp[n], dys[n], G[l][n][1], step[0], ws)      # dW and dL/db_t (Eq. 4) in one pass

    variants = {"plain": plain, "plain_torch": plain_torch, "plain_on_w_hat": plain_on_w_hat, "torch_on_w_hat": torch_on_w_hat,
                "separate": separate, "riding": riding, "bwd_plain": bwd_plain, "bwd_torch": bwd_torch, "bwd_sampled": bwd_sampled}
    for fn in variants.values():
        for _ in range(2):
            fn()
    bursts = {k: [] for k in variants}
    for _ in range(9):
        for k, fn in variants.items():
            bursts[k].append(_time_ms(torch, fn, 3, warmup=1) / layers)
    med = {k: sorted(v)[len(v) // 2] for k, v in bursts.items()}
    fb_plain, fb_torch, fb_sampled = med["plain"] + med["bwd_plain"], med["plain_torch"] + med["bwd_torch"], med["riding"] + med["bwd_sampled"]
    best_plain = min(med["plain"], med["plain_torch"])
    flop = 2.0 * tokens * sum(r * c for r, c in shapes.values())
    return {"tokens": tokens, "layers_in_a_row": layers, "gemms_per_layer": {n: [tokens, shapes[n][0], shapes[n][1]] for n in order},
            "ms_per_layer": med, "plain_TFLOPs": flop / med["plain"] / 1e9,
            "separate_overhead_pct_vs_own_plain": 100.0 * (med["separate"] - med["plain"]) / med["plain"],
            "riding_overhead_pct_vs_own_plain": 100.0 * (med["riding"] - med["plain"]) / med["plain"],
            "separate_overhead_pct_vs_best_plain": 100.0 * (med["separate"] - best_plain) / best_plain,
            "riding_overhead_pct_vs_best_plain": 100.0 * (med["riding"] - best_plain) / best_plain,
            "riding_overhead_pct_vs_same_gemms_on_w_hat": 100.0 * (med["riding"] - med["plain_on_w_hat"]) / med["plain_on_w_hat"],
            "separate_overhead_pct_vs_same_gemms_on_w_hat": 100.0 * (med["separate"] - med["plain_on_w_hat"]) / med["plain_on_w_hat"],
            "forward_and_backward": {
                "ms_per_layer": {"plain_own": fb_plain, "plain_torch": fb_torch, "sampled": fb_sampled},
                "sampled_overhead_pct_vs_own_plain": 100.0 * (fb_sampled - fb_plain) / fb_plain,
                "sampled_overhead_pct_vs_best_plain": 100.0 * (fb_sampled - min(fb_plain, fb_torch)) / min(fb_plain, fb_torch),
                "backward_overhead_pct_vs_own_plain": 100.0 * (med["bwd_sampled"] - med["bwd_plain"]) / med["bwd_plain"],
                "note": "forward: the riding schedule; backward per weight: dX = dY * w_hat^T (gws_gemm_bf16) and dW = X^T dY with "
                        "dL/db_t from the GEMM's epilogue (gws_linear_bwd_w_ws; the tokens split into parts for the weights of few "
                        "tiles); plain: the same GEMMs on W without sampling and without dL/db_t; torch: torch.matmul for all 15 GEMMs",
                "paper_context": "the paper's Table 1 reports 1.40 % (134M) to 5.30 % (3B) tokens/s overhead of a whole training "
                                 "step on A100; this is the linear layers' GEMMs of one decoder layer alone, the part that overhead "
                                 "is added to"},
            "carried_by_each_gemm": plan, "riding_matches_gws_sample_fwd": same,
            "sampled_params_per_layer": sum(r * c for r, c in shapes.values())}


def copy_ceiling(torch):
    """A plain device copy of 2 x 1 GiB (torch's copy kernel): what a streaming read+write reaches here."""
    a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    b = torch.empty_like(a)
    ms = _time_ms(torch, lambda: b.copy_(a), 10)
    return {"GBps": 2 * a.numel() / ms / 1e6, "frac_of_hbm_peak": 2 * a.numel() / ms / 1e6 / HBM_PEAK_GBS}


def linear_bench(torch, gws, synth, dev):
    """Fused sampled-weight linear vs unfused (sample kernel + plain GEMM) vs plain BF16 GEMM."""
    M, K, N = 8192, 2048, 5632
    x = synth.make_activation(5, M, K, device=dev)
    t = synth.make_tensor(5, K, N, bt=6.0, device=dev, with_grad=False)
    w, bt = t["w"], t["bt"]
    w_hat = torch.empty_like(w)
    scale = torch.empty(K // 32, N // 32, device=dev)
    y = torch.empty(M, N, dtype=torch.bfloat16, device=dev)
    seed = gws.gws_derive_seed(0, 5)
    d_full = gws.TensorDesc(rows=K, cols=N, seed=seed, w=w, w_hat=w_hat, bt=bt, scale=scale)
    pk = gws.pack([d_full])
    fmt = gws.FMT_FP8_E4M3
    # without w_hat / scale outputs the sampling sits in the operand load of every M-tile
    d_inop = gws.TensorDesc(rows=K, cols=N, seed=seed, w=w, bt=bt)
    ws = torch.empty(gws.gws_linear_fwd_workspace_bytes(d_inop), dtype=torch.uint8, device=dev)

    def unfused():
        gws.gws_sample_fwd(pk, fmt, 0)
        gws.gws_gemm_bf16(x, w_hat, y)

    def unfused_torch():
        gws.gws_sample_fwd(pk, fmt, 0)
        torch.matmul(x, w_hat, out=y)

    # backward of the same linear: dW = X^T dY [K x N], with dL/db_t from the GEMM's epilogue or from the
    # separate backward kernel on the stored dW
    dy = (synth.make_activation(6, M, N, device=dev).float() * 1e-3).to(torch.bfloat16)
    dw = torch.empty_like(w)
    dbt = torch.empty_like(scale)
    d_bwd = gws.TensorDesc(rows=K, cols=N, seed=seed, scale=scale, dw=dw, dbt=dbt)
    d_bwd_plain = gws.TensorDesc(rows=K, cols=N, seed=seed, dw=dw)
    pk_bwd = gws.pack([gws.TensorDesc(rows=K, cols=N, seed=seed, scale=scale, g=dw, dw=dw, dbt=dbt)])

    def bwd_unfused():
        gws.gws_linear_bwd_w(x, dy, d_bwd_plain, 0)
        gws.gws_sample_bwd(pk_bwd, 0)

    dx = torch.empty_like(x)
    # eight layers in a row, as a forward pass issues them
    # ... and with the sampling of the next layer's weight riding in the GEMM's launch (two w_hat buffers)
    w_hat_b, scale_b = torch.empty_like(w_hat), torch.empty_like(scale)
    whs = (w_hat, w_hat_b)
    nxt = [gws.TensorDesc(rows=K, cols=N, seed=seed, w=w, w_hat=wh, bt=bt, scale=sc)
           for wh, sc in ((w_hat, scale), (w_hat_b, scale_b))]

    # a smaller next weight (the 1B model's 2048 x 2048 projections): its sampling fits beside the GEMM's last round
    tq = synth.make_tensor(7, 2048, 2048, bt=6.0, device=dev, with_grad=False)
    d_q = gws.TensorDesc(rows=2048, cols=2048, seed=seed, w=tq["w"], w_hat=torch.empty_like(tq["w"]), bt=tq["bt"],
                         scale=torch.empty(64, 64, device=dev))
    pk_q = gws.pack([d_q])

    def gemm_then_sample_q():
        gws.gws_gemm_bf16(x, w_hat, y)
        gws.gws_sample_fwd(pk_q, fmt, 1)

    def next_loop(layers=8):
        gws.gws_sample_fwd(pk, fmt, 0)                                   # the first layer's weight
        for l in range(layers):
            gws.gws_gemm_bf16_sample_next(x, whs[l % 2], y, nxt[(l + 1) % 2], fmt, l + 1)

    def plain_loop(layers=8):
        for _ in range(layers):
            gws.gws_gemm_bf16(x, w, y)

    def auto_loop(layers=8):
        for l in range(layers):
            gws.gws_linear_fwd(x, d_full, y, fmt, l)

    variants = {
        "plain8": plain_loop,
        "next8": next_loop,
        "gemm_next": lambda: gws.gws_gemm_bf16_sample_next(x, w_hat, y, nxt[1], fmt, 1),
        "gemm_next_q": lambda: gws.gws_gemm_bf16_sample_next(x, w_hat, y, d_q, fmt, 1),
        "gemm_then_q": gemm_then_sample_q,
        "auto8": auto_loop,
        "bwd_x": lambda: gws.gws_gemm_bf16(dy, w_hat, dx, w_is_nk=True),          # dX = dY * w_hat^T
        "bwd_x_torch": lambda: torch.matmul(dy, w_hat.t(), out=dx),
        "bwd_w_fused": lambda: gws.gws_linear_bwd_w(x, dy, d_bwd, 0),
        "bwd_w_plain": lambda: gws.gws_linear_bwd_w(x, dy, d_bwd_plain, 0),
        "bwd_w_unfused": bwd_unfused,
        "bwd_w_torch": lambda: torch.matmul(x.t(), dy, out=dw),
        "staged": lambda: gws.gws_linear_fwd_ws(x, d_inop, y, fmt, 0, ws),
        "auto": lambda: gws.gws_linear_fwd(x, d_full, y, fmt, 0),
        "unfused": unfused,
        "plain": lambda: gws.gws_gemm_bf16(x, w, y),
        "plain_what": lambda: gws.gws_gemm_bf16(x, w_hat, y),
        "torch": lambda: torch.matmul(x, w, out=y),
        "torch_what": lambda: torch.matmul(x, w_hat, out=y),
        "unfused_torch": unfused_torch,
        "sample": lambda: gws.gws_sample_fwd(pk, fmt, 0),
    }
    # GEMM times move with the clock and temperature state the preceding work leaves, so the
    # variants are timed in short bursts taken in turn, and the median burst is reported
    gws.gws_sample_fwd(pk, fmt, 0)
    for fn in variants.values():
        for _ in range(3):
            fn()
    bursts = {k: [] for k in variants}
    for _ in range(9):
        for k, fn in variants.items():
            bursts[k].append(_time_ms(torch, fn, 6, warmup=1))
    med = {k: sorted(v)[len(v) // 2] for k, v in bursts.items()}
    t_unfused, t_plain, t_plain_what = med["unfused"], med["plain"], med["plain_what"]
    t_torch, t_torch_what, t_unfused_torch, t_sample = med["torch"], med["torch_what"], med["unfused_torch"], med["sample"]
    t_inop = _time_ms(torch, lambda: gws.gws_linear_fwd_mode(x, d_inop, y, fmt, 0, gws.LINEAR_IN_OPERAND), 10)
    t_auto = med["auto"]
    flop = 2.0 * M * K * N
    best_plain = min(t_plain, t_torch)
    return {"shape": [M, K, N],
            "linear_fwd_auto_ms": t_auto, "auto_overhead_pct_vs_own_plain": 100.0 * (t_auto - t_plain) / t_plain,
            "auto_overhead_pct_vs_best_plain": 100.0 * (t_auto - best_plain) / best_plain,
            "linear_fwd_ws_ms": med["staged"], "fused_in_operand_ms": t_inop, "unfused_own_gemm_ms": t_unfused,
            "unfused_torch_gemm_ms": t_unfused_torch, "sample_only_ms": t_sample,
            "plain_own_ms": t_plain, "plain_own_on_w_hat_ms": t_plain_what,
            "plain_torch_ms": t_torch, "plain_torch_on_w_hat_ms": t_torch_what,
            "eight_layers": {"plain_gemm_ms_per_layer": med["plain8"] / 8, "linear_fwd_ms_per_layer": med["auto8"] / 8,
                             "linear_fwd_overhead_pct": 100.0 * (med["auto8"] - med["plain8"]) / med["plain8"],
                             "gemm_sample_next_ms_per_layer": med["next8"] / 8,
                             "gemm_sample_next_overhead_pct": 100.0 * (med["next8"] - med["plain8"]) / med["plain8"],
                             "note": "gemm_sample_next: one gws_sample_fwd for the first layer, then per layer one "
                                     "gws_gemm_bf16_sample_next (GEMM on w_hat of layer l, sampling of layer l+1 in the same launch)"},
            "gemm_sample_next": {"same_shape_next_ms": med["gemm_next"], "next_2048x2048_riding_ms": med["gemm_next_q"],
                                 "gemm_then_sample_2048x2048_ms": med["gemm_then_q"], "gemm_on_w_hat_alone_ms": t_plain_what,
                                 "note": "the GEMM's 704 tiles leave 64 of 256 compute units idle in the last round; a 2048 x 5632 or a "
                                         "2048 x 2048 next weight is sampled there, in the GEMM's launch"},
            "bwd_x": {"gemm_on_w_hat_ms": med["bwd_x"], "torch_matmul_ms": med["bwd_x_torch"],
                      "TFLOPs": 2.0 * M * K * N / med["bwd_x"] / 1e9},
            "bwd_w": {"gemm_with_dbt_epilogue_ms": med["bwd_w_fused"], "gemm_plain_ms": med["bwd_w_plain"],
                      "gemm_plain_then_sample_bwd_ms": med["bwd_w_unfused"], "torch_matmul_ms": med["bwd_w_torch"],
                      "epilogue_overhead_pct": 100.0 * (med["bwd_w_fused"] - med["bwd_w_plain"]) / med["bwd_w_plain"],
                      "separate_kernel_overhead_pct": 100.0 * (med["bwd_w_unfused"] - med["bwd_w_plain"]) / med["bwd_w_plain"],
                      "TFLOPs_with_epilogue": 2.0 * M * K * N / med["bwd_w_fused"] / 1e9},
            "bwd_w_layer_shapes": bwd_w_shapes_bench(torch, gws, synth, dev),
            "fused_in_operand_overhead_pct_vs_best_plain": 100.0 * (t_inop - best_plain) / best_plain,
            "unfused_overhead_pct_vs_own_plain": 100.0 * (t_unfused - t_plain) / t_plain,
            "unfused_overhead_pct_vs_best_plain": 100.0 * (min(t_unfused, t_unfused_torch) - best_plain) / best_plain,
            "linear_fwd_TFLOPs": flop / t_auto / 1e9, "plain_own_TFLOPs": flop / t_plain / 1e9,
            "plain_torch_TFLOPs": flop / t_torch / 1e9,
            "mfma_frac_of_peak_linear_fwd": flop / t_auto / 1e9 / MFMA_BF16_PEAK_TFLOPS,
            "mfma_frac_of_peak_plain_own": flop / t_plain / 1e9 / MFMA_BF16_PEAK_TFLOPS,
            "paper_context": "paper: 1.40% tokens/s overhead end to end (Llama2-134M, A100), sampling amortised over "
                             "49152 tokens per step; here one forward GEMM over 8192 tokens"}


if __name__ == "__main__":
    main()
