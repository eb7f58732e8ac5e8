#!/usr/bin/env python3
"""Benchmark of the shard-GEMM hot path on one MI355X.

A step is one pass of the hot path over one workload: the forward, dgrad and wgrad local
products of a 3D-tensor-parallel FC layer shard (for the chain workloads: of every layer), through
axo_layer_step (default; the benchmark's layers have buffers of their own, so the library finds one
dependence level and runs all products in one grouped launch) or axo_layer_step_ordered (--step
ordered: one launch per product, in program order).  Inputs are seeded synthetic bf16 shards, resident
in HBM before the timed region.

The headline workload (`value`) is config 3, the MLP up-projection shard with the bias + GELU epilogue:
with config 4 the largest single-GPU workload of the benchmark.  The same run also times configs
2, 4 and 5 and reports them under `configs`, each with a roofline object of its own.

Prints one JSON line: TFLOP/s of the step (2*M*Kl*Nl flop per product), a roofline object for the
dominant kernel (HIP-event timed on the launch stream) and the CPU oracle timed on a bounded sample of
the headline workload.

Pre-heat: the chip leaves idle at a low clock and needs some hundred milliseconds of load before its power
controller has settled; a run of `--warmup 5 --steps 20` is 7 ms of GPU time and would be timed on that
ramp.  Every timed loop is therefore preceded by a time-based pre-heat of the very launch that is
timed (`--preheat-ms`, default 500 ms of GPU time, reported as `preheat`), then the counted warm-up steps,
then the timed steps.  The chunk times of the timed region are reported in time order.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak (published)
PEAK_HBM_GBPS = 8000.0

# HBM-side traffic per launch of the tuned kernels, as (FETCH_SIZE, WRITE_SIZE) counter readings from
# rocprofv3 --pmc runs of this script (profiles/gemm_kernels_cfg*.md give the commands and the tables),
# scaled by the same counters' readings for a plain 1 GiB copy: 2.000 KiB per FETCH_SIZE count, 1.000 KiB
# per WRITE_SIZE count.  Keyed by (workload, product); "group" is the single launch of the grouped step.
FETCH_KIB_PER_COUNT, WRITE_KIB_PER_COUNT = 2.0, 1.0
MEASURED_TRAFFIC_COUNTS = {
    ("cfg2", "group"): (304881.7, 90117.6), ("cfg2", "fwd"): (82089.3, 49152.0),
    ("cfg2", "dgrad"): (98376.9, 16385.4), ("cfg2", "wgrad"): (82012.0, 24585.7),
    ("cfg3", "group"): (782891.4, 213002.6), ("cfg3", "fwd"): (196822.5, 131105.4),
    ("cfg3", "dgrad"): (269250.1, 16394.7), ("cfg3", "wgrad"): (196700.0, 65536.4),
    ("cfg4", "group"): (782160.2, 213008.2), ("cfg4", "fwd"): (272950.8, 16386.0),
    ("cfg4", "dgrad"): (196708.5, 131092.2), ("cfg4", "wgrad"): (196700.0, 65536.2),
    ("cfg5", "group"): (1087142.1, 251960.1), ("cfg5", "fwd"): (61667.2, 49152.0),
    ("cfg5", "dgrad"): (86080.5, 12288.0), ("cfg5", "wgrad"): (83036.0, 18440.0),
}
MEASURED_TRAFFIC_BYTES = {k: int((f * FETCH_KIB_PER_COUNT + w * WRITE_KIB_PER_COUNT) * 1024)
                          for k, (f, w) in MEASURED_TRAFFIC_COUNTS.items()}

HEADLINE = "cfg3"
ALSO = ("cfg2", "cfg4", "cfg5")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", default=HEADLINE,
                    help="headline workload: cfg1..cfg5 or gpt20b (default cfg3, the MLP up-projection shard)")
    ap.add_argument("--only", action="store_true",
                    help="time the headline workload only (default: the other benchmark configs too, under 'configs')")
    ap.add_argument("--with-gpt20b", action="store_true",
                    help="also time the (2,2,4) shards of the paper's GPT-20B running example")
    ap.add_argument("--preheat-ms", type=float, default=500.0,
                    help="GPU time of the untimed pre-heat in front of every timed loop (same launches as the loop)")
    ap.add_argument("--step", choices=("layer_step", "ordered"), default="layer_step",
                    help="entry point of the timed step: axo_layer_step (dependence levels, grouped launches; the "
                         "default) or axo_layer_step_ordered (one launch per product, in program order)")
    ap.add_argument("--no-per-op", action="store_true", help="skip the separate per-product launch loops")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", action="store_true",
                    help="also time the backward-side extras on the largest layer: dgrad through GELU, fp32-accumulating "
                         "wgrad, bias gradient (reported under 'extras')")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share of the work on one GPU; "
              "--gpus must be 1 (no collectives or multi-GPU path exist here).", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import axo_synth as syn
    import paper_2305_13525_amd as axo

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    axo.library()  # fails loudly if the HIP library is not built
    st = torch.cuda.current_stream().cuda_stream
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to("cuda:0")

    def setup(cfg_name):
        layers = syn.configs()[cfg_name]
        objs, keep, flop = [], [], 0
        for L in layers:
            d = syn.layer_inputs(L)
            p = axo.Problem.make(L.grid, (0, 0, 0), L.T, L.K, L.N)
            M, Kl, Nl = L.shard
            t = {k: dev(v) for k, v in d.items()}
            t["Y"] = torch.zeros((M, Nl), dtype=torch.int16, device="cuda:0")
            t["dX"] = torch.zeros((M, Kl), dtype=torch.int16, device="cuda:0")
            t["dW"] = torch.zeros((Kl, Nl), dtype=torch.int16, device="cuda:0")
            keep.append(t)
            epi = L.epilogue
            objs.append(axo.Layer(p, epi, 0, t["X"].data_ptr(), Kl, t["W"].data_ptr(), Nl,
                                  t["bias"].data_ptr() if epi else None, t["Y"].data_ptr(), Nl,
                                  t["dY"].data_ptr(), Nl, t["dX"].data_ptr(), Kl, t["dW"].data_ptr(), Nl))
            flop += 3 * L.flop_per_gemm
        nws = axo.axo_layer_step_workspace_bytes(objs)
        ws = torch.empty(max(nws, 16), dtype=torch.uint8, device="cuda:0")
        keep.append(ws)
        return layers, objs, keep, flop, ws.data_ptr(), nws

    step_fn = axo.axo_layer_step_ordered if args.step == "ordered" else axo.axo_layer_step

    def preheat(fn):
        """Runs fn back to back until --preheat-ms of GPU time have passed; returns what it did."""
        info = {"ms": 0.0, "steps": 0}
        if args.preheat_ms <= 0:
            return info
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        batch, first = 4, None
        while info["ms"] < args.preheat_ms and info["steps"] < 1_000_000:
            e0.record()
            for _ in range(batch):
                fn()
            e1.record()
            torch.cuda.synchronize()
            dt = e0.elapsed_time(e1)
            if first is None:
                first = dt / batch
            info["ms"] += dt
            info["steps"] += batch
            last = dt / batch
            # batches of about 25 ms: few synchronisation gaps, and the loop stops close to the target
            batch = max(1, min(4096, int(25.0 / max(last, 1e-3))))
        info["ms"] = round(info["ms"], 1)
        info["first_batch_ms_per_step"] = round(first, 5)
        info["last_batch_ms_per_step"] = round(last, 5)
        return info

    def time_loop(fn, steps, warmup):
        """Pre-heat, `warmup` untimed calls, then exactly `steps` timed calls between two events on the
        launch stream.  An event per eighth of the run as well (no synchronisation inside the timed
        region): the chunk times, in time order, show clock drift that the mean hides."""
        heat = preheat(fn)
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        chunk = max(1, steps // 8)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps // chunk + 1)]
        e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(steps):
            fn()
            if (i + 1) % chunk == 0:
                marks[(i + 1) // chunk].record()
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        per_chunk = [marks[k].elapsed_time(marks[k + 1]) / chunk for k in range(steps // chunk)]
        srt = sorted(per_chunk)
        chunks = {"steps_per_chunk": chunk, "in_time_order_ms": [round(c, 5) for c in per_chunk],
                  "median_ms": round(srt[len(srt) // 2], 5), "best_ms": round(srt[0], 5),
                  "worst_ms": round(srt[-1], 5)}
        return max(marks[0].elapsed_time(e1), 0.0) / steps, wall / steps, chunks, heat

    def per_op(o, wsp, nws, steps, warmup):
        res = {}
        res["fwd"] = time_loop(lambda: axo.axo_fc_fwd(o.p, o.X, o.ldx, o.W, o.ldw, o.bias, o.epilogue, o.Y, o.ldy,
                                                      wsp, nws, st), steps, warmup)[0]
        res["dgrad"] = time_loop(lambda: axo.axo_fc_dgrad(o.p, o.dY, o.lddy, o.W, o.ldw, o.dX, o.lddx, wsp, nws, st),
                                 steps, warmup)[0]
        res["wgrad"] = time_loop(lambda: axo.axo_fc_wgrad(o.p, o.X, o.ldx, o.dY, o.lddy, o.dW, o.lddw, wsp, nws, st),
                                 steps, warmup)[0]
        return res

    def measure(cfg_name, with_per_op):
        """Times one workload; returns (result dict, state kept for the extras / cpu baseline)."""
        layers, objs, keep, flop, wsp, nws = setup(cfg_name)
        ms, wall_ms, chunks, heat = time_loop(lambda: step_fn(objs, wsp, nws, st), args.steps, args.warmup)
        tflops = flop / (ms * 1e-3) / 1e12
        li = max(range(len(layers)), key=lambda i: layers[i].flop_per_gemm)
        gflop = layers[li].flop_per_gemm
        alg_bytes = sum(2 * (L.shard[0] * L.shard[1] + L.shard[1] * L.shard[2] + L.shard[0] * L.shard[2])
                        for L in layers)
        ops = per_op(objs[li], wsp, nws, args.steps, args.warmup) if with_per_op else None
        grouped = args.step == "layer_step" and 3 * len(layers) <= 12
        if grouped or ops is None:
            # the whole step is ONE launch of gemm_group_kernel: its duration is the step's
            roofline = {"bound": "mfma", "kernel": "gemm_group_kernel (all products of the step in one launch)"
                        if grouped else "gemm_mixed_kernel (all launches of the step)",
                        "achieved": round(tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(tflops / PEAK_BF16_TFLOPS, 4),
                        "traffic": MEASURED_TRAFFIC_BYTES.get((cfg_name, "group")) if grouped else None,
                        "flop_per_launch": flop, "avg_launch_ms": round(ms, 5),
                        "algorithmic_bytes_per_launch": 3 * alg_bytes}
        else:
            # one launch per product: the dominant kernel is the slowest product of the largest layer
            dom = max(ops, key=ops.get)
            ach = gflop / (ops[dom] * 1e-3) / 1e12
            M, Kl, Nl = layers[li].shard
            roofline = {"bound": "mfma", "kernel": f"gemm_mixed_kernel ({layers[li].name}.{dom})",
                        "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                        "traffic": MEASURED_TRAFFIC_BYTES.get((cfg_name, dom)), "flop_per_launch": gflop,
                        "avg_launch_ms": round(ops[dom], 5),
                        "algorithmic_bytes_per_launch": 2 * (M * Kl + Kl * Nl + M * Nl)}
        if ops is not None:
            roofline["separate_launches"] = {
                "layer": layers[li].name, "per_op_ms": {k: round(v, 5) for k, v in ops.items()},
                "per_op_tflops": {k: round(gflop / (v * 1e-3) / 1e12, 2) for k, v in ops.items()}}
        res = {"value": round(tflops, 2), "unit": "TFLOP/s", "frac_of_bf16_mfma_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
               "ms_per_step": round(ms, 5), "wall_ms_per_step": round(wall_ms, 5), "ms_per_step_chunks": chunks,
               "preheat": heat,
               "config": {"workload": cfg_name,
                          "step": "axo_layer_step_ordered" if args.step == "ordered" else "axo_layer_step",
                          "layers": [{"name": L.name, "grid": list(L.grid), "shard_MKN": list(L.shard),
                                      "epilogue": L.epilogue} for L in layers],
                          "flop_per_step": flop},
               "roofline": roofline}
        state = {"layers": layers, "objs": objs, "keep": keep, "li": li, "wsp": wsp, "nws": nws, "ops": ops}
        return res, state

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")   # 1 GiB read + 1 GiB write per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    head, state = measure(args.config, not args.no_per_op)
    out = {"metric": "TFLOP/s for fwd+dgrad+wgrad shard GEMMs, 1 MI355X", "value": head["value"],
           "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": head["ms_per_step"], "wall_ms_per_step": head["wall_ms_per_step"],
           "ms_per_step_chunks": head["ms_per_step_chunks"], "preheat": head["preheat"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "frac_of_bf16_mfma_peak": head["frac_of_bf16_mfma_peak"],
           "config": head["config"], "roofline": head["roofline"]}

    layers, objs, li, wsp, nws, ops = (state[k] for k in ("layers", "objs", "li", "wsp", "nws", "ops"))
    if args.extras:
        L, o = layers[li], objs[li]
        gflop = L.flop_per_gemm
        M, Kl, Nl = L.shard
        pre = torch.randn((M, Kl), device="cuda:0").to(torch.bfloat16).view(torch.int16)
        dW32 = torch.zeros((Kl, Nl), dtype=torch.float32, device="cuda:0")
        db = torch.zeros((Nl,), dtype=torch.float32, device="cuda:0")
        t_fw = ops["fwd"] if ops else time_loop(
            lambda: axo.axo_fc_fwd(o.p, o.X, o.ldx, o.W, o.ldw, o.bias, o.epilogue, o.Y, o.ldy, wsp, nws, st),
            args.steps, args.warmup)[0]
        t_da = time_loop(lambda: axo.axo_fc_dgrad_act(o.p, o.dY, o.lddy, o.W, o.ldw, pre.data_ptr(), Kl,
                                                      axo.AXO_EPI_BIAS_GELU_TANH, o.dX, o.lddx, wsp, nws, st),
                         args.steps, args.warmup)[0]
        t_wa = time_loop(lambda: axo.axo_fc_wgrad_acc(o.p, o.X, o.ldx, o.dY, o.lddy, dW32.data_ptr(), Nl, wsp, nws, st),
                         args.steps, args.warmup)[0]
        t_bg = time_loop(lambda: axo.axo_bias_grad(o.p, o.dY, o.lddy, db.data_ptr(), 0, st), args.steps, args.warmup)[0]
        bg_bytes = 2 * M * Nl + 4 * Nl
        nbw = axo.axo_bias_grad_workspace_bytes(o.p)
        bws = torch.zeros(max(nbw, 16), dtype=torch.uint8, device="cuda:0")   # arrival counters start at zero
        t_bs = time_loop(lambda: axo.axo_bias_grad_ws(o.p, o.dY, o.lddy, db.data_ptr(), 0, bws.data_ptr(), nbw, st),
                         args.steps, args.warmup)[0]
        # the whole local step of that layer with all extras, through the scheduled chain entry point
        ext = [axo.LayerExt.make(o, pre=pre.data_ptr(), ldpre=Kl, act_below=axo.AXO_EPI_BIAS_GELU_TANH,
                                 dW32=dW32.data_ptr(), lddw32=Nl, db=db.data_ptr(), accumulate_db=0)]
        t_ext = time_loop(lambda: axo.axo_layer_step_ext(ext, wsp, nws, st), args.steps, args.warmup)[0]
        out["extras"] = {
            "layer_step_ext": {"ms": round(t_ext, 5), "tflops": round(3 * gflop / (t_ext * 1e-3) / 1e12, 2),
                               "what": "fwd + dgrad through GELU + fp32-accumulating wgrad + bias gradient, one call",
                               "separate_calls_ms": round(t_fw + t_da + t_wa + t_bg, 5)},
            "layer": L.name,
            "dgrad_gelu_tanh": {"ms": round(t_da, 5), "tflops": round(gflop / (t_da * 1e-3) / 1e12, 2)},
            "wgrad_acc_f32": {"ms": round(t_wa, 5), "tflops": round(gflop / (t_wa * 1e-3) / 1e12, 2)},
            "bias_grad": {"ms": round(t_bg, 5), "bound": "hbm", "algorithmic_bytes": bg_bytes,
                          "achieved_GBps": round(bg_bytes / (t_bg * 1e-3) / 1e9, 1), "peak_GBps": PEAK_HBM_GBPS,
                          "frac": round(bg_bytes / (t_bg * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)},
            "bias_grad_ws": {"ms": round(t_bs, 5), "bound": "hbm", "algorithmic_bytes": bg_bytes,
                             "workspace_bytes": nbw,
                             "achieved_GBps": round(bg_bytes / (t_bs * 1e-3) / 1e9, 1), "peak_GBps": PEAK_HBM_GBPS,
                             "frac": round(bg_bytes / (t_bs * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)}}
        del pre, dW32, db, ext

    head_layer = layers[li]
    del state, objs, layers
    if not args.only:
        names = [n for n in ALSO + (("gpt20b",) if args.with_gpt20b else ()) if n != args.config]
        others = {}
        for name in names:
            torch.cuda.empty_cache()
            res, s2 = measure(name, False)
            del s2
            others[name] = {k: res[k] for k in ("value", "unit", "frac_of_bf16_mfma_peak", "ms_per_step",
                                                "ms_per_step_chunks", "preheat", "config", "roofline")}
        out["configs"] = others

    if not args.no_cpu_baseline:
        import oracle  # test infrastructure; only this baseline leg uses it
        L = head_layer
        d = syn.layer_inputs(L)
        M, Kl, Nl = L.shard
        # the oracle runs about 60 GFLOP/s on 16 cores: bound the sample to roughly 10-20 s of CPU work
        budget_flop = 0.9e12
        frac = min(1.0, budget_flop / (3.0 * L.flop_per_gemm))
        n_act = max(1, int(M * frac))
        n_w = max(1, int(Kl * frac))
        rows = np.linspace(0, M - 1, n_act).astype(np.int64)
        krows = np.linspace(0, Kl - 1, n_w).astype(np.int64)
        t0 = time.perf_counter()
        oracle.fc_fwd(d["X"], d["W"], d["bias"] if L.epilogue else None, L.epilogue, rows=rows)
        oracle.fc_dgrad(d["dY"], d["W"], rows=rows)
        oracle.fc_wgrad(d["X"], d["dY"], rows=krows)
        dt = time.perf_counter() - t0
        cflop = 2.0 * (2 * n_act * Kl * Nl + n_w * M * Nl)
        out["cpu_baseline"] = {"value": round(cflop / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"{args.config} {L.name}: {n_act} of {M} output rows of fwd and of dgrad, "
                                         f"{n_w} of {Kl} rows of dW (fp64 plain loops)"}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
