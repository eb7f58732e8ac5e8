#!/usr/bin/env python3
"""Benchmark of the shard-GEMM hot path on one MI355X.

A step is one pass of the hot path over one workload: the forward, dgrad and wgrad local
products of a 3D-tensor-parallel FC layer shard (for the chain workloads: of every layer), through
axo_layer_step (default; the benchmark's layers have buffers of their own, so the library finds one
dependence level and runs all products in one grouped launch) or axo_layer_step_ordered (--step
ordered: one launch per product, in program order).  Inputs are seeded synthetic bf16 shards, resident
in HBM before the timed region.  Prints one JSON line: TFLOP/s of the step (2*M*Kl*Nl flop per
product), a roofline object for the dominant kernel (HIP-event timed on the launch stream) and the
CPU oracle timed on a bounded sample of the same workload.
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

# HBM-side bytes per launch (fetched + written) of the tuned kernel, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs of this script, scaled by the same counters' readings for a plain 1 GiB copy
# (2.000 KiB per FETCH_SIZE count, 1.000 KiB per WRITE_SIZE count).  Keyed by (workload, product);
# "group" is the single launch of the grouped step.
MEASURED_TRAFFIC_BYTES = {
    ("cfg2", "fwd"): int((82100.9 * 2.0 + 49152.0) * 1024),
    ("cfg2", "dgrad"): int((98372.0 * 2.0 + 16385.4) * 1024),
    ("cfg2", "wgrad"): int((82012.6 * 2.0 + 24581.5) * 1024),
    ("cfg2", "group"): int((305489.7 * 2.0 + 90116.2) * 1024),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", default="cfg2", help="cfg1..cfg5 (default cfg2, the QKV shard)")
    ap.add_argument("--all-configs", action="store_true",
                    help="also time cfg2..cfg5 and gpt20b and report them under 'configs'")
    ap.add_argument("--step", choices=("layer_step", "ordered"), default="layer_step",
                    help="entry point of the timed step: axo_layer_step (dependence levels, grouped launches; the "
                         "default) or axo_layer_step_ordered (one launch per product, in program order)")
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

    def time_step(objs, wsp, nws, steps, warmup):
        for _ in range(warmup):
            step_fn(objs, wsp, nws, st)
        torch.cuda.synchronize()
        # one event per eighth of the run as well (no synchronisation inside the timed region): the
        # spread between the chunks shows clock drift that the mean hides
        chunk = max(1, steps // 8)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps // chunk + 1)]
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(steps):
            step_fn(objs, wsp, nws, st)
            if (i + 1) % chunk == 0:
                marks[(i + 1) // chunk].record()
        e1 = torch.cuda.Event(enable_timing=True)
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        per_chunk = sorted(marks[k].elapsed_time(marks[k + 1]) / chunk for k in range(steps // chunk))
        time_step.chunks = {"steps_per_chunk": chunk, "median_ms": round(per_chunk[len(per_chunk) // 2], 5),
                            "best_ms": round(per_chunk[0], 5), "worst_ms": round(per_chunk[-1], 5)}
        return max(marks[0].elapsed_time(e1), 0.0) / steps, wall / steps

    def time_op(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    def per_op(L, o, wsp, nws, steps, warmup):
        res = {}
        res["fwd"] = time_op(lambda: axo.axo_fc_fwd(o.p, o.X, o.ldx, o.W, o.ldw, o.bias, o.epilogue, o.Y, o.ldy,
                                                    wsp, nws, st), steps, warmup)
        res["dgrad"] = time_op(lambda: axo.axo_fc_dgrad(o.p, o.dY, o.lddy, o.W, o.ldw, o.dX, o.lddx, wsp, nws, st),
                               steps, warmup)
        res["wgrad"] = time_op(lambda: axo.axo_fc_wgrad(o.p, o.X, o.ldx, o.dY, o.lddy, o.dW, o.lddw, wsp, nws, st),
                               steps, warmup)
        return res

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")   # 1 GiB read + 1 GiB write per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    layers, objs, keep, flop, wsp, nws = setup(args.config)
    ms, wall_ms = time_step(objs, wsp, nws, args.steps, args.warmup)
    chunk_stats = dict(time_step.chunks)
    tflops = flop / (ms * 1e-3) / 1e12

    # per-product launches of the largest layer, each timed in a loop of its own
    li = max(range(len(layers)), key=lambda i: layers[i].flop_per_gemm)
    ops = per_op(layers[li], objs[li], wsp, nws, args.steps, args.warmup)
    gflop = layers[li].flop_per_gemm
    per_op_info = {"layer": layers[li].name,
                   "per_op_ms": {k: round(v, 5) for k, v in ops.items()},
                   "per_op_tflops": {k: round(gflop / (v * 1e-3) / 1e12, 2) for k, v in ops.items()}}
    alg_bytes = sum(2 * (L.shard[0] * L.shard[1] + L.shard[1] * L.shard[2] + L.shard[0] * L.shard[2]) for L in layers)
    if args.step == "layer_step" and len(layers) <= 4:
        # the whole step is ONE launch of gemm_group_kernel: its duration is the step's
        roofline = {"bound": "mfma", "kernel": "gemm_group_kernel (all products of the step)",
                    "achieved": round(tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tflops / PEAK_BF16_TFLOPS, 4),
                    "traffic": MEASURED_TRAFFIC_BYTES.get((args.config, "group")), "flop_per_launch": flop,
                    "avg_launch_ms": round(ms, 5), "algorithmic_bytes_per_launch": 3 * alg_bytes}
    else:
        # one launch per product: the dominant kernel is the slowest product of the largest layer
        dom = max(ops, key=ops.get)
        ach = gflop / (ops[dom] * 1e-3) / 1e12
        M, Kl, Nl = layers[li].shard
        roofline = {"bound": "mfma", "kernel": f"gemm_mixed_kernel ({layers[li].name}.{dom})", "achieved": round(ach, 2),
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                    "traffic": MEASURED_TRAFFIC_BYTES.get((args.config, dom)), "flop_per_launch": gflop,
                    "avg_launch_ms": round(ops[dom], 5),
                    "algorithmic_bytes_per_launch": 2 * (M * Kl + Kl * Nl + M * Nl)}
    roofline["separate_launches"] = per_op_info

    out = {"metric": "TFLOP/s for fwd+dgrad+wgrad shard GEMMs, 1 MI355X", "value": round(tflops, 2),
           "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms, 5), "wall_ms_per_step": round(wall_ms, 5), "ms_per_step_chunks": chunk_stats,
           "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "frac_of_bf16_mfma_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
           "config": {"workload": args.config,
                      "step": "axo_layer_step_ordered" if args.step == "ordered" else "axo_layer_step", "layers": [
               {"name": L.name, "grid": list(L.grid), "shard_MKN": list(L.shard), "epilogue": L.epilogue}
               for L in layers], "flop_per_step": flop},
           "roofline": roofline}

    if args.extras:
        L, o = layers[li], objs[li]
        M, Kl, Nl = L.shard
        pre = torch.randn((M, Kl), device="cuda:0").to(torch.bfloat16).view(torch.int16)
        dW32 = torch.zeros((Kl, Nl), dtype=torch.float32, device="cuda:0")
        db = torch.zeros((Nl,), dtype=torch.float32, device="cuda:0")
        t_da = time_op(lambda: axo.axo_fc_dgrad_act(o.p, o.dY, o.lddy, o.W, o.ldw, pre.data_ptr(), Kl,
                                                    axo.AXO_EPI_BIAS_GELU_TANH, o.dX, o.lddx, wsp, nws, st),
                       args.steps, args.warmup)
        t_wa = time_op(lambda: axo.axo_fc_wgrad_acc(o.p, o.X, o.ldx, o.dY, o.lddy, dW32.data_ptr(), Nl, wsp, nws, st),
                       args.steps, args.warmup)
        t_bg = time_op(lambda: axo.axo_bias_grad(o.p, o.dY, o.lddy, db.data_ptr(), 0, st), args.steps, args.warmup)
        bg_bytes = 2 * M * Nl + 4 * Nl
        # the whole local step of that layer with all extras, through the scheduled chain entry point
        ext = [axo.LayerExt.make(o, pre=pre.data_ptr(), ldpre=Kl, act_below=axo.AXO_EPI_BIAS_GELU_TANH,
                                 dW32=dW32.data_ptr(), lddw32=Nl, db=db.data_ptr(), accumulate_db=0)]
        t_ext = time_op(lambda: axo.axo_layer_step_ext(ext, wsp, nws, st), args.steps, args.warmup)
        out["extras"] = {
            "layer_step_ext": {"ms": round(t_ext, 5), "tflops": round(3 * gflop / (t_ext * 1e-3) / 1e12, 2),
                               "what": "fwd + dgrad through GELU + fp32-accumulating wgrad + bias gradient, one call",
                               "separate_calls_ms": round(ops["fwd"] + t_da + t_wa + t_bg, 5)},
            "layer": L.name,
            "dgrad_gelu_tanh": {"ms": round(t_da, 5), "tflops": round(gflop / (t_da * 1e-3) / 1e12, 2),
                                "plain_dgrad_ms": round(ops["dgrad"], 5)},
            "wgrad_acc_f32": {"ms": round(t_wa, 5), "tflops": round(gflop / (t_wa * 1e-3) / 1e12, 2),
                              "plain_wgrad_ms": round(ops["wgrad"], 5)},
            "bias_grad": {"ms": round(t_bg, 5), "bound": "hbm", "algorithmic_bytes": bg_bytes,
                          "achieved_GBps": round(bg_bytes / (t_bg * 1e-3) / 1e9, 1), "peak_GBps": 8000.0,
                          "frac": round(bg_bytes / (t_bg * 1e-3) / 1e9 / 8000.0, 4)}}

    if args.all_configs:
        extra = {}
        for name in ("cfg2", "cfg3", "cfg4", "cfg5", "gpt20b"):
            if name == args.config:
                extra[name] = {"tflops": round(tflops, 2), "ms_per_step": round(ms, 5)}
                continue
            del keep
            torch.cuda.empty_cache()
            l2, o2, keep, f2, w2, n2 = setup(name)
            m2, _ = time_step(o2, w2, n2, args.steps, args.warmup)
            extra[name] = {"tflops": round(f2 / (m2 * 1e-3) / 1e12, 2), "ms_per_step": round(m2, 5),
                           "frac_of_peak": round(f2 / (m2 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        out["configs"] = extra

    if not args.no_cpu_baseline:
        import oracle  # test infrastructure; only this baseline leg uses it
        L = layers[li]
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
                               "sample": f"{L.name}: {n_act} of {M} output rows of fwd and of dgrad, "
                                         f"{n_w} of {Kl} rows of dW (fp64 plain loops)"}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
