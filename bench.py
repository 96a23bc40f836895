#!/usr/bin/env python3
"""Benchmark of the kFkB stage engine on one MI355X.

One step = one whole kFkB iteration of the stage (all micro-batches forward and backward in
kFkB order, gradient accumulation, transfers) on synthetic data already resident in pinned
host / device memory.  Workload: the GPT-2-medium-shaped stage (6 blocks, hidden 1024, 16 heads,
seq 1024, micro-batch 4, 16 micro-batches, bf16 with fp32 gradient accumulation).

Prints ONE JSON line: whole-job samples/s at the best group size k, the per-k table, the roofline
of the kernel the iteration spends most time in (measured live with HIP events on the library's
compute stream) and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: L, H, heads, T, b, M, dtype, ks, default delay model, activation limit (bytes, 0 = none)
    "gpt2-medium-stage": dict(L=6, H=1024, heads=16, T=1024, b=4, M=16, dtype="bf16", ks=(1, 2, 4), delay="none", limit=0),
    "tiny-stage": dict(L=2, H=128, heads=4, T=64, b=2, M=4, dtype="f32", ks=(1, 2), delay="none", limit=0),
    # the larger configurations: timing only (weights are one seeded 4M-element draw tiled over every tensor,
    # two seeded micro-batches reused cyclically); parity at these shapes is covered kernel by kernel in tests/
    "gpt-1.3b-stage": dict(L=6, H=2048, heads=16, T=2048, b=2, M=32, dtype="bf16", ks=(1, 2, 4, 8), delay="lognormal",
                           limit=0, tiled=True),
    "wide-stage": dict(L=4, H=4096, heads=32, T=2048, b=1, M=32, dtype="bf16", ks=(1, 2, 4, 8, 0), delay="bimodal",
                       limit=200e9, tiled=True),
    "very-wide-stage": dict(L=2, H=8192, heads=64, T=4096, b=1, M=64, dtype="bf16", ks=(1, 2, 4, 8), delay="drift",
                            limit=250e9, tiled=True),
}
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0
PEAK_F32_TFLOPS = 157.3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt2-medium-stage", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic, used to scale "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command)")
    ap.add_argument("--wgrad-stream", type=int, default=1, choices=[0, 1],
                    help="1 (the library's default): weight and bias gradients run on a stream of their own beside the "
                         "input-gradient chain; 0: everything on the compute stream")
    ap.add_argument("--lanes", type=int, default=2, choices=[1, 2],
                    help="compute lanes (the library's default is 2): ops in flight at once, within the plan's peak of live "
                         "micro-batches")
    ap.add_argument("--adaptive", action="store_true",
                    help="also time the same steps under the tuner (run_kFkB_adaptive: moving averages of the measured "
                         "transfer times, k re-chosen every 2 iterations among the workload's k values)")
    ap.add_argument("--pipeline-stages", type=int, default=0,
                    help="also time the same iteration run as a pipeline of this many virtual stages on the one GPU "
                         "(run_pipeline_kFkB: every stage under its own kFkB plan, boundary crossings delayed by the "
                         "workload's delay model); reported under \"pipeline_sim\", the headline value is unchanged")
    ap.add_argument("--candidates-gb", type=float, default=0.0,
                    help="also time every candidate plan (k, b) on the memory-limit curve (paper Section 4.2): the global "
                         "batch stays fixed, for each k the largest micro-batch size b whose (w+1) k live micro-batches fit "
                         "this many GB of stashed activations; the stage is set up anew for every b; reported under "
                         "\"candidates\", the headline value is unchanged")
    ap.add_argument("--recompute", action="store_true",
                    help="activation recomputation: LayerNorm and GELU outputs are formed again in the backward pass "
                         "instead of being stashed (10 instead of 16 activation tensors per block)")
    ap.add_argument("--dtype", default=None, choices=["bf16", "f16"],
                    help="storage type of a 16-bit workload (default: the workload's own, bf16; f16 is the paper's "
                         "precision and runs the same kernels)")
    ap.add_argument("--delay", default=None, choices=["none", "lognormal", "bimodal", "drift"],
                    help="per-transfer injected delay; default: the workload's own (lognormal: mean 2 ms, sigma 0.5; "
                         "bimodal: 0.5 ms w.p. 0.7 / 10 ms w.p. 0.3; drift: 0 -> 20 ms over the timed steps)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build drives one pipeline stage on ONE GPU; --gpus %d is not supported "
              "(how the path shards over stages is described in DESIGN.md)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import kfkb_synth as synth
    import paper_2303_01675_amd as kf

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    kf.load_library()                      # fails loudly if libkfkb.so was not built

    w = dict(WORKLOADS[args.workload])
    if args.dtype is not None and w["dtype"] != "f32":
        w["dtype"] = args.dtype
    L, H, heads, T, b, M = w["L"], w["H"], w["heads"], w["T"], w["b"], w["M"]
    dt = {"bf16": kf.BF16, "f16": kf.F16, "f32": kf.F32}[w["dtype"]]
    delay_model = args.delay or w["delay"]
    t0 = time.time()
    if w.get("tiled"):
        base = synth.normal(1234, 1 << 22, 0.0, 0.02)

        def tensor(name, shp):
            v = np.resize(base, int(np.prod(shp)))
            v = v + 1.0 if name in ("ln1_g", "ln2_g") else v
            return (synth.round_to_bf16(v) if w["dtype"] == "bf16" else v.astype(np.float16).astype(np.float32)).reshape(shp)
        one = {n: tensor(n, shp) for n, shp in synth.param_shapes(H, 4 * H).items()}
        blocks = [one] * L
    else:
        blocks = synth.stage_weights(L, H, 4 * H, w["dtype"])
    st = kf.StageBuffers(blocks, dt, heads, T, b, M, M if (0 in w["ks"] or args.pipeline_stages > 1) else max(w["ks"]),
                         recompute=int(args.recompute))
    distinct = 2 if w.get("tiled") else M
    cache = {}
    for mb in range(M):
        src = mb % distinct
        if src not in cache:
            cache[src] = (synth.microbatch_inputs(src, b, T, H, w["dtype"]), synth.microbatch_upstream_grads(src, b, T, H, w["dtype"]))
        st.set_inputs_one(mb, *cache[src])
    del cache
    if w.get("tiled"):
        del blocks
    t_setup = time.time() - t0
    overlap = kf.stage_side_streams_overlap()
    kf.stage_set_wgrad_stream(args.wgrad_stream)
    kf.stage_set_compute_lanes(args.lanes)

    def set_delays(step_index, n_steps):
        """Delays of one iteration, the same for every k: drawn per (iteration, direction, micro-batch)."""
        if delay_model == "none":
            return
        if delay_model == "lognormal":
            d = [synth.delays_lognormal(M, 2.0, 0.5, seed=4242 + 4 * step_index + i) for i in range(4)]
        elif delay_model == "bimodal":
            d = [synth.delays_bimodal(M, 0.5, 10.0, 0.7, seed=4242 + 4 * step_index + i) for i in range(4)]
        else:
            d = [synth.delays_drift(M, step_index, n_steps, 20.0)] * 4
        kf.stage_set_delays(*d)

    from oracle import stage_math as osm        # only for the FLOP model and the CPU-baseline leg
    flops_iter = M * osm.stage_flops(L, b, T, H, causal=True)
    flops_iter_megatron = M * osm.stage_flops(L, b, T, H, causal=True, megatron=True)

    limit = int(w["limit"])

    def step(k, i=0):
        set_delays(i, args.steps)
        kf.stage_zero_grads()
        kf.run_kFkB(k, M, limit)

    per_k = {}
    for k_req in w["ks"]:
        for _ in range(args.warmup):
            step(k_req)
        kf.stage_sync()
        k = kf.stage_last_k()                      # k_req = 0 asks for the largest k that fits the activation limit
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(k_req, i)
        kf.stage_sync()
        torch.cuda.synchronize()
        dt_s = time.perf_counter() - t0
        per_k[k] = dict(ms_per_step=1e3 * dt_s / args.steps, samples_per_s=M * b * args.steps / dt_s,
                        tflops=flops_iter * args.steps / dt_s / 1e12,
                        tflops_megatron=flops_iter_megatron * args.steps / dt_s / 1e12,
                        activation_gb=kf.stage_activation_bytes(k, M) / 1e9)
    best_k = max(per_k, key=lambda k: per_k[k]["samples_per_s"])

    pipeline_sim = None
    if args.pipeline_stages > 1:
        S = args.pipeline_stages
        wire = torch.empty(kf.stage_pipeline_bytes(S, M), dtype=torch.uint8, device="cuda")
        kf.stage_sync()
        kf.stage_pipeline_bind(wire, S, M)

        def boundary_delays(step_index, n_steps):
            n = (S - 1) * M
            if delay_model == "none":
                return None, None
            if delay_model == "lognormal":
                return tuple(synth.delays_lognormal(n, 2.0, 0.5, seed=9000 + 2 * step_index + i) for i in range(2))
            if delay_model == "bimodal":
                return tuple(synth.delays_bimodal(n, 0.5, 10.0, 0.7, seed=9000 + 2 * step_index + i) for i in range(2))
            d = np.tile(synth.delays_drift(M, step_index, n_steps, 20.0), S - 1)
            return d, d

        def pstep(k, i=0):
            set_delays(i, args.steps)
            kf.stage_set_pipeline_delays(*boundary_delays(i, args.steps))
            kf.stage_zero_grads()
            kf.run_pipeline_kFkB(k)

        pk = {}
        for k in sorted({k for k in per_k} | {M}):
            for _ in range(args.warmup):
                pstep(k)
            kf.stage_sync()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(args.steps):
                pstep(k, i)
            kf.stage_sync()
            dt_s = time.perf_counter() - t0
            peaks = [kf.kfkb_peak_live(k, M, min(S - 1 - v, -(-M // k))) for v in range(S)]
            pk[str(k)] = dict(ms_per_step=1e3 * dt_s / args.steps, samples_per_s=M * b * args.steps / dt_s,
                              peak_live_per_stage=peaks)
        kf.stage_set_pipeline_delays(None, None)
        pipeline_sim = dict(stages=S, blocks_per_stage=L // S, delay=delay_model, per_k=pk,
                            note="S virtual stages share the one GPU: total work equals the single stage's, so the "
                                 "figures show what the schedule and the boundary delays cost, not a pipeline speed-up")

    adaptive = None
    if args.adaptive:
        cands = sorted(k for k in per_k)
        kf.stage_sync()
        kf.kfkb_tuner_config(2, 2, cands)
        kf.stage_set_delays(None, None, None, None)
        kf.stage_tuner_calibrate(M, 2)
        chosen = []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            set_delays(i, args.steps)
            kf.stage_zero_grads()
            chosen.append(kf.run_kFkB_adaptive(M, limit))
        kf.stage_sync()
        dt_s = time.perf_counter() - t0
        adaptive = dict(ms_per_step=1e3 * dt_s / args.steps, samples_per_s=M * b * args.steps / dt_s, k_per_step=chosen,
                        window=2, interval=2, candidates=cands)

    # per-kernel timing of the same steps at the best k: HIP start/stop events on the stream of each launch.
    # Kernels that share the chip stretch each other's durations, so this pass runs on one lane with the W steps
    # behind their chains: every duration below is that of a kernel running alone.
    kf.stage_sync()
    kf.stage_set_wgrad_stream(0)
    kf.stage_set_compute_lanes(1)
    kf.stage_set_delays(None, None, None, None)
    delay_model_saved, delay_model = delay_model, "none"
    kf.kfkb_profile(True)
    for _ in range(args.steps):
        step(best_k)
    kf.stage_sync()
    kf.kfkb_profile(False)
    kf.stage_set_wgrad_stream(args.wgrad_stream)
    kf.stage_set_compute_lanes(args.lanes)
    delay_model = delay_model_saved
    stats = kf.kfkb_profile_report()
    tot_ms = sum(s["total_ms"] for s in stats) or 1.0
    kernels = []
    for s in sorted(stats, key=lambda s: -s["total_ms"]):
        rate = s["work"] / (s["total_ms"] * 1e-3) if s["total_ms"] > 0 else 0.0
        kernels.append(dict(name=s["name"], bound=s["bound"], launches_per_step=s["launches"] / args.steps,
                            avg_us=1e3 * s["total_ms"] / max(s["launches"], 1), share=s["total_ms"] / tot_ms,
                            achieved=(rate / 1e12 if s["bound"] != "hbm" else rate / 1e9),
                            unit="TFLOP/s" if s["bound"] != "hbm" else "GB/s"))
    dom = kernels[0]
    peak = {"mfma": PEAK_BF16_TFLOPS, "hbm": PEAK_HBM_GBS, "alu": PEAK_F32_TFLOPS}[dom["bound"]]
    roofline = dict(bound=dom["bound"], kernel=dom["name"], achieved=dom["achieved"], peak=peak, unit=dom["unit"],
                    frac=dom["achieved"] / peak, traffic=None, avg_us=dom["avg_us"], share_of_kernel_time=dom["share"])
    # HBM traffic of that kernel, where a rocprofv3 --pmc measurement of this workload is on file
    try:
        with open(os.path.join(ROOT, "profiles", "stage_%s_hbm_traffic.json" % args.workload.replace("-stage", "").replace("-", ""))) as f:
            tj = json.load(f)
        key = dom["name"].replace(" ", "")
        hit = [v for k, v in tj["kernels"].items() if k.startswith(key.rstrip(">")) or key.startswith(k.rstrip(">"))]
        if hit:
            roofline["traffic"] = hit[0]["read_bytes"] + hit[0]["write_bytes"]
            roofline["traffic_source"] = "profiles/stage_%s_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a 1 GiB copy)" % args.workload.replace("-stage", "").replace("-", "")
    except (OSError, ValueError, KeyError):
        pass
    gemm = [s for s in stats if s["name"].startswith("gemm_bf16")]
    if gemm:
        roofline["all_gemm_tflops"] = sum(s["work"] for s in gemm) / (sum(s["total_ms"] for s in gemm) * 1e-3) / 1e12
        roofline["all_gemm_frac"] = roofline["all_gemm_tflops"] / PEAK_BF16_TFLOPS

    cpu = None
    if not args.no_cpu_baseline and not w.get("tiled"):
        from oracle import stage_math as sm
        x = synth.microbatch_inputs(0, b, T, H, w["dtype"])
        dy = synth.microbatch_upstream_grads(0, b, T, H, w["dtype"])
        nsamp = b
        # bounded sample: one whole micro-batch of the iteration's 16 (about 15 s of float64 numpy on the machine's cores)
        t0 = time.perf_counter()
        y, caches = sm.stage_fwd(x, blocks, heads, True)
        sm.stage_bwd(dy, blocks, caches, heads)
        dt_s = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        cpu = dict(value=nsamp / dt_s, unit="samples/s", cores=cores, kind="oracle",
                   sample="forward+backward of %d sample(s) of micro-batch 0 (of %d samples per iteration), float64 numpy"
                          % (nsamp, M * b), seconds=dt_s)

    best = per_k[best_k]
    out = {
        "metric": "stage fwd+bwd samples/sec (kFkB iteration, best k)", "value": best["samples_per_s"],
        "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": best["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w["dtype"],
        "data": "synthetic" + (" (one seeded draw tiled over the weights, 2 micro-batches reused)" if w.get("tiled") else ""),
        "config": {"workload": args.workload, "layers": L, "hidden": H, "heads": heads, "seq_len": T, "micro_batch": b,
                   "num_microbatches": M, "global_batch": M * b, "k": best_k, "delay": delay_model,
                   "activation_limit_bytes": limit,
                   "side_streams_overlap": bool(overlap), "wgrad_stream": bool(args.wgrad_stream), "compute_lanes": args.lanes,
                   "recompute": bool(args.recompute)},
        "tflops": best["tflops"], "tflops_megatron_convention": best["tflops_megatron"],
        "frac_of_bf16_peak": best["tflops"] / PEAK_BF16_TFLOPS if w["dtype"] != "f32" else None,   # fp16 has the same peak
        "per_k": {str(k): v for k, v in per_k.items()},
        "adaptive": adaptive, "pipeline_sim": pipeline_sim, "roofline": roofline, "kernels": kernels[:12], "cpu_baseline": cpu, "setup_seconds": t_setup,
    }
    st.close()
    if args.candidates_gb > 0:
        per_sample = kf.kfkb_activation_bytes_per_microbatch(L, 1, T, H, heads, 4 * H, 2 if w["dtype"] != "f32" else 4,
                                                             recompute=int(args.recompute))
        cands = kf.kfkb_enumerate_candidates(M * b, int(args.candidates_gb * 1e9), per_sample)
        rows = []
        for ck, cb in cands:
            cM = M * b // cb
            cst = kf.StageBuffers(blocks if not w.get("tiled") else [one] * L, dt, heads, T, cb, cM, ck, recompute=int(args.recompute))
            pair = [(synth.microbatch_inputs(j, cb, T, H, w["dtype"]), synth.microbatch_upstream_grads(j, cb, T, H, w["dtype"])) for j in range(2)]
            for mb in range(cM):
                cst.set_inputs_one(mb, *pair[mb % 2])
            kf.stage_set_wgrad_stream(args.wgrad_stream)
            kf.stage_set_compute_lanes(args.lanes)

            def cstep(i):
                if delay_model == "lognormal":
                    kf.stage_set_delays(*[synth.delays_lognormal(cM, 2.0, 0.5, seed=4242 + 4 * i + j) for j in range(4)])
                elif delay_model == "bimodal":
                    kf.stage_set_delays(*[synth.delays_bimodal(cM, 0.5, 10.0, 0.7, seed=4242 + 4 * i + j) for j in range(4)])
                elif delay_model == "drift":
                    kf.stage_set_delays(*([synth.delays_drift(cM, i, args.steps, 20.0)] * 4))
                kf.stage_zero_grads()
                kf.run_kFkB(ck, cM, int(args.candidates_gb * 1e9))
            for _ in range(args.warmup):
                cstep(0)
            kf.stage_sync()
            t0 = time.perf_counter()
            for i in range(args.steps):
                cstep(i)
            kf.stage_sync()
            dt_s = time.perf_counter() - t0
            rows.append(dict(k=ck, micro_batch=cb, num_microbatches=cM, ms_per_step=1e3 * dt_s / args.steps,
                             samples_per_s=M * b * args.steps / dt_s, activation_gb=kf.stage_activation_bytes(ck, cM) / 1e9))
            cst.close()
        out["candidates"] = dict(global_batch=M * b, activation_limit_gb=args.candidates_gb, delay=delay_model, plans=rows)
    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        c = torch.empty_like(a)
        c.copy_(a)
        torch.cuda.synchronize()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
