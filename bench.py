#!/usr/bin/env python3
"""Benchmark of the kFkB stage engine on one MI355X.

One step = one whole kFkB iteration of the stage (all micro-batches forward and backward in kFkB order, gradient
accumulation, delayed transfers) on synthetic data already resident in pinned host / device memory.

Default workload: the very wide stage (2 blocks, hidden 8192, 64 heads, seq 4096, micro-batch 1, 64 micro-batches,
bf16 with fp32 gradient accumulation, transfer delay drifting from 0 to 20 ms over the timed steps, 250 GB
activation limit), the largest of the five configurations and the one the metric "vs k (1, 2, 4, 8)" is quoted on.

What a run does:
  1. per-k scan: every group size k of the workload is timed over a few steps under the workload's delay model
     (`per_k`, with its own step count), which shows what larger groups gain over 1F1B (k = 1);
  2. headline: W warm-up steps, then EXACTLY K timed steps at the best k of the scan -> `value` (samples/s);
  3. per-kernel pass: a few steps at that k on one compute lane with per-kernel HIP events -> `roofline`, `kernels`;
  4. the CPU oracle timed on a bounded sample of the same workload -> `cpu_baseline`;
  5. (default run only) the GPT-2-medium-shaped stage, timed the same way -> `secondary`.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    # name: L, H, heads, T, b, M, dtype, ks (0 = largest k that fits the limit), delay model, activation limit in bytes
    "tiny-stage": dict(L=2, H=128, heads=4, T=64, b=2, M=4, dtype="f32", ks=(1, 2), delay="none", limit=0),
    "gpt2-medium-stage": dict(L=6, H=1024, heads=16, T=1024, b=4, M=16, dtype="bf16", ks=(1, 2, 4), delay="none", limit=0),
    # the larger configurations: weights are one seeded draw repeated cyclically over every tensor
    # (kfkb_synth.stage_weights_tiled), two seeded micro-batches are reused cyclically
    "gpt-1.3b-stage": dict(L=6, H=2048, heads=16, T=2048, b=2, M=32, dtype="bf16", ks=(1, 2, 4, 8), delay="lognormal",
                           limit=0, tiled=True),
    "wide-stage": dict(L=4, H=4096, heads=32, T=2048, b=1, M=32, dtype="bf16", ks=(1, 2, 4, 8, 0), delay="bimodal",
                       limit=200e9, tiled=True),
    "very-wide-stage": dict(L=2, H=8192, heads=64, T=4096, b=1, M=64, dtype="bf16", ks=(1, 2, 4, 8), delay="drift",
                            limit=250e9, tiled=True),
}
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 / fp16 MFMA peak
PEAK_HBM_GBS = 8000.0
PEAK_F32_TFLOPS = 157.3


def stage_flops(L, b, T, H, causal=True, megatron=False):
    """Model FLOPs of forward + backward of one micro-batch: 3 L m (24 H^2 + 4 T H c), m = b T tokens, c = 1/2 under
    a causal mask (the masked half need not be computed), c = 1 in the Megatron convention the paper's throughput
    plots use (Section 6.2.2).  Bias, LayerNorm, GELU and softmax arithmetic is not counted."""
    c = 0.5 if (causal and not megatron) else 1.0
    return 3.0 * L * (b * T) * (24.0 * H * H + 4.0 * T * H * c)


_T0 = time.time()


def progress(msg):
    """Phase lines on stderr (the result is the one JSON line on stdout): a run of minutes is not silent."""
    print("[bench %6.1f s] %s" % (time.time() - _T0, msg), file=sys.stderr, flush=True)


def delays_for(synth, model, M, step_index, n_steps, seed0=4242):
    """Delays of one iteration, the same for every k: drawn per (iteration, direction, micro-batch)."""
    if model == "none":
        return (None, None, None, None)
    if model == "lognormal":
        return tuple(synth.delays_lognormal(M, 2.0, 0.5, seed=seed0 + 4 * step_index + i) for i in range(4))
    if model == "bimodal":
        return tuple(synth.delays_bimodal(M, 0.5, 10.0, 0.7, seed=seed0 + 4 * step_index + i) for i in range(4))
    if model.startswith("fixed:"):                              # every transfer delayed by the same time, in ms
        import numpy as np
        return (np.full(M, int(float(model[6:]) * 1e6), dtype=np.int64),) * 4
    return (synth.delays_drift(M, step_index, n_steps, 20.0),) * 4


class Run:
    """One workload set up on the GPU: weights, inputs, the bound stage."""

    def __init__(self, name, w, args, kf, synth, np):
        self.name, self.w, self.kf, self.synth, self.np = name, w, kf, synth, np
        L, H, heads, T, b, M = w["L"], w["H"], w["heads"], w["T"], w["b"], w["M"]
        self.dt = {"bf16": kf.BF16, "f16": kf.F16, "f32": kf.F32}[w["dtype"]]
        t0 = time.time()
        if w.get("tiled"):
            blocks = synth.stage_weights_tiled(L, H, 4 * H, w["dtype"], out=np.float32)
        else:
            blocks = synth.stage_weights(L, H, 4 * H, w["dtype"])
        k_max = M if (0 in w["ks"] or args.pipeline_stages > 1) else max(w["ks"])
        self.st = kf.StageBuffers(blocks, self.dt, heads, T, b, M, k_max, recompute=int(args.recompute))
        self.block0 = blocks[0] if w.get("tiled") else None       # the CPU-baseline leg times the oracle on one block
        self.blocks = None if w.get("tiled") else blocks
        del blocks
        distinct = 2 if w.get("tiled") else M
        cache = {}
        for mb in range(M):
            src = mb % distinct
            if src not in cache:
                cache[src] = (synth.microbatch_inputs(src, b, T, H, w["dtype"]), synth.microbatch_upstream_grads(src, b, T, H, w["dtype"]))
            self.st.set_inputs_one(mb, *cache[src])
        self.setup_seconds = time.time() - t0
        self.overlap = kf.stage_side_streams_overlap()
        # the library picks lanes and W-step placement from the stage's shape; the flags override it
        self.lanes = kf.stage_set_compute_lanes(1)
        self.wgrad_stream = kf.stage_set_wgrad_stream(0)
        if args.lanes:
            self.lanes = args.lanes
        if args.wgrad_stream >= 0:
            self.wgrad_stream = args.wgrad_stream
        kf.stage_set_compute_lanes(self.lanes)
        kf.stage_set_wgrad_stream(self.wgrad_stream)
        if args.inputs_ahead >= 0:
            kf.kfkb_set_inputs_ahead(args.inputs_ahead)
        if args.mid_tiles >= 0:
            kf.kfkb_set_mid_tiles(args.mid_tiles)
        if args.send_copy_blocks >= 0:
            kf.stage_set_send_copy_blocks(args.send_copy_blocks)
        if args.wstep_window > 0:
            kf.stage_set_wstep_window(args.wstep_window)
        self.delay_model = args.delay or w["delay"]
        self.limit = int(w["limit"])
        self.flops_iter = M * stage_flops(L, b, T, H)
        self.flops_iter_megatron = M * stage_flops(L, b, T, H, megatron=True)

    def step(self, k, i, n_steps):
        self.kf.stage_set_delays(*delays_for(self.synth, self.delay_model, self.w["M"], i, n_steps))
        self.kf.stage_zero_grads()
        self.kf.run_kFkB(k, self.w["M"], self.limit)

    def timed(self, k_req, warmup, steps, torch):
        """`warmup` untimed steps, then `steps` timed ones bracketed by synchronisation; returns (k used, row)."""
        kf, w = self.kf, self.w
        for _ in range(warmup):
            self.step(k_req, 0, steps)
        kf.stage_sync()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(k_req, i, steps)
        kf.stage_sync()
        torch.cuda.synchronize()
        dt_s = time.perf_counter() - t0
        k = kf.stage_last_k()                      # k_req = 0 asks for the largest k that fits the activation limit
        M, b = w["M"], w["b"]
        return k, dict(steps=steps, warmup=warmup, ms_per_step=1e3 * dt_s / steps, samples_per_s=M * b * steps / dt_s,
                       tflops=self.flops_iter * steps / dt_s / 1e12,
                       tflops_megatron=self.flops_iter_megatron * steps / dt_s / 1e12,
                       activation_gb=kf.stage_activation_bytes(k, M) / 1e9)


def kernel_pass(run, k, steps, args):
    """The same steps at group size k with per-kernel timing on: HIP start/stop events on the stream of each launch.
    Kernels that share the chip stretch each other's durations, so this pass runs on one lane with the W steps
    behind their chains and without injected delays: every duration is that of a kernel running alone."""
    kf = run.kf
    kf.stage_sync()
    kf.stage_set_wgrad_stream(0)
    kf.stage_set_compute_lanes(1)
    saved, run.delay_model = run.delay_model, "none"
    run.step(k, 0, 1)                                       # one untimed step in this configuration
    kf.stage_sync()
    kf.kfkb_profile(True)
    for _ in range(steps):
        run.step(k, 0, 1)
    kf.stage_sync()
    kf.kfkb_profile(False)
    kf.stage_set_wgrad_stream(run.wgrad_stream)
    kf.stage_set_compute_lanes(run.lanes)
    run.delay_model = saved
    stats = kf.kfkb_profile_report()
    tot_ms = sum(s["total_ms"] for s in stats) or 1.0
    kernels = []
    for s in sorted(stats, key=lambda s: -s["total_ms"]):
        rate = s["work"] / (s["total_ms"] * 1e-3) if s["total_ms"] > 0 else 0.0
        hbm = s["bound"] == "hbm"
        peak = {"mfma": PEAK_BF16_TFLOPS, "hbm": PEAK_HBM_GBS, "alu": PEAK_F32_TFLOPS}[s["bound"]]
        ach = rate / 1e9 if hbm else rate / 1e12
        kernels.append(dict(name=s["name"], bound=s["bound"], launches_per_step=s["launches"] / steps,
                            avg_us=1e3 * s["total_ms"] / max(s["launches"], 1), share=s["total_ms"] / tot_ms,
                            achieved=ach, unit="GB/s" if hbm else "TFLOP/s", frac=ach / peak,
                            work_per_launch=s["work"] / max(s["launches"], 1)))
    dom = kernels[0]
    peak = {"mfma": PEAK_BF16_TFLOPS, "hbm": PEAK_HBM_GBS, "alu": PEAK_F32_TFLOPS}[dom["bound"]]
    roofline = dict(bound=dom["bound"], kernel=dom["name"], achieved=dom["achieved"], peak=peak, unit=dom["unit"],
                    frac=dom["achieved"] / peak, traffic=None, avg_us=dom["avg_us"], share_of_kernel_time=dom["share"],
                    algorithmic_work_per_launch=dom["work_per_launch"], launches_per_step=dom["launches_per_step"])
    # HBM traffic of that kernel, where a rocprofv3 --pmc measurement of this workload is on file (same kernel names)
    tag = run.name.replace("-stage", "").replace("-", "").replace(".", "")
    try:
        with open(os.path.join(ROOT, "profiles", "stage_%s_hbm_traffic.json" % tag)) as f:
            tj = json.load(f)
        hit = tj["kernels"].get(dom["name"])
        if hit:
            # per launch of THIS run: a W-step launch covers as many micro-batches as the group size allows, so the
            # measured bytes are scaled by the algorithmic work of a launch here over that of a launch in the counter run
            scale = dom["work_per_launch"] / hit["work_per_launch"] if hit.get("work_per_launch") else 1.0
            roofline["traffic"] = (hit["read_bytes"] + hit["write_bytes"]) * scale
            roofline["traffic_source"] = ("profiles/stage_%s_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, "
                                          "scaled by a 1 GiB copy; x %.2f for the work of a launch in this run)" % (tag, scale))
            roofline["traffic_level"] = ("bytes between the eight L2s and the fabric: every XCD streams the operand panels of its "
                                         "own tiles through its own 4 MiB L2, and hits in the memory-side cache are not subtracted")
    except (OSError, ValueError, KeyError):
        pass
    gemm = [s for s in stats if s["name"].startswith("gemm_")]
    if gemm and run.w["dtype"] != "f32":
        roofline["all_gemm_tflops"] = sum(s["work"] for s in gemm) / (sum(s["total_ms"] for s in gemm) * 1e-3) / 1e12
        roofline["all_gemm_frac"] = roofline["all_gemm_tflops"] / PEAK_BF16_TFLOPS
    return roofline, kernels


def cpu_baseline(run, np):
    """The oracle (float64 numpy, as it stands) on the machine's host cores, on a bounded sample of the workload.
    Small workloads: forward + backward of one whole micro-batch.  Large ones: ONE block and ONE sample with the
    sequence cut to `tokens`, extrapolated to the stage by model FLOPs and labelled so.  A one-thread figure on a
    smaller sample goes with it."""
    from oracle import stage_math as sm
    synth, w = run.synth, run.w
    L, H, heads, T, b, M = w["L"], w["H"], w["heads"], w["T"], w["b"], w["M"]
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threadpool_limits, cores = None, os.cpu_count()

    def once(blocks, bs, Ts):
        x = synth.microbatch_inputs(0, bs, Ts, H, w["dtype"])
        dy = synth.microbatch_upstream_grads(0, bs, Ts, H, w["dtype"])
        t0 = time.perf_counter()
        _, caches = sm.stage_fwd(x, blocks, heads, True)
        sm.stage_bwd(dy, blocks, caches, heads)
        return time.perf_counter() - t0

    flops_sample = stage_flops(L, 1, T, H)                       # one sample of the real workload, whole stage
    if not w.get("tiled"):
        secs = once(run.blocks, b, T)
        out = dict(value=b / secs, unit="samples/s", cores=cores, kind="oracle", seconds=secs, extrapolated=False,
                   sample="forward+backward of the %d sample(s) of micro-batch 0 (of %d samples per iteration), whole stage, "
                          "float64 numpy" % (b, M * b))
        one_blocks, one_T, one_L = run.blocks[:1], min(T, 256), 1
    else:
        blk = {n: np.asarray(v, dtype=np.float64) for n, v in run.block0.items()}
        # tokens (and, where one sample's whole sequence is not enough, samples) so that the sample is about
        # 12 TFLOP of float64 work: 10 - 30 s on the machine's cores
        target = 1.2e13
        Ts = int(min(T, max(32, 2 ** int(np.log2(target / (3.0 * 24.0 * H * H))))))
        ns = int(min(8, max(1, target // stage_flops(1, 1, Ts, H))))
        secs = once([blk], ns, Ts)
        f_meas = ns * stage_flops(1, 1, Ts, H)
        out = dict(value=(f_meas / secs) / flops_sample, unit="samples/s", cores=cores, kind="oracle", seconds=secs,
                   extrapolated=True, measured_gflops=f_meas / secs / 1e9,
                   sample="EXTRAPOLATED by model FLOPs from forward+backward of ONE block on %d sample(s) cut to %d of %d "
                          "tokens (%.2f TFLOP of float64 numpy) to the %d-block stage at full sequence length "
                          "(%.1f TFLOP per sample)" % (ns, Ts, T, f_meas / 1e12, L, flops_sample / 1e12))
        one_blocks, one_T, one_L = [blk], max(16, Ts // 8), 1
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            s1 = once(one_blocks, 1, one_T)
        f1 = stage_flops(one_L, 1, one_T, H)
        out["one_thread"] = dict(value=(f1 / s1) / flops_sample, unit="samples/s", seconds=s1, extrapolated=True,
                                 sample="one block, one sample of %d tokens, BLAS limited to 1 thread, extrapolated by model FLOPs" % one_T)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="very-wide-stage", choices=sorted(WORKLOADS))
    ap.add_argument("--ks", default=None,
                    help="comma-separated group sizes to scan instead of the workload's own (e.g. 4 for a short profiling run)")
    ap.add_argument("--microbatches", type=int, default=0,
                    help="run the workload with this many micro-batches per iteration instead of its own (same kernels and "
                         "launch shapes, shorter iteration: for profiling runs)")
    ap.add_argument("--scan-steps", type=int, default=0,
                    help="timed steps per k of the per-k scan (after one warm-up step each); 0 = max(3, steps / 5)")
    ap.add_argument("--profile-steps", type=int, default=0, help="steps of the per-kernel pass; 0 = 2 for the large workloads, else steps")
    ap.add_argument("--secondary", default=None, choices=sorted(WORKLOADS) + ["none"],
                    help="a second workload timed after the first, reported under \"secondary\" (default: gpt2-medium-stage "
                         "when the first is the default workload, else none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--inputs-ahead", type=int, default=-1, help="receive order (kfkb_set_inputs_ahead): 0 consumption order, 1 stage inputs one schedule unit ahead, 2 by k; -1 keeps the library default")
    ap.add_argument("--mid-tiles", type=int, default=-1, help="128 x 256 tiles for the forward / input-gradient products (kfkb_set_mid_tiles): 0 never, 1 where they rate best, 2 wherever they fit; -1 keeps the library default")
    ap.add_argument("--send-copy-blocks", type=int, default=-1, help="sends: 0 the runtime's device-to-host copy, n > 0 the library's copy kernel with n workgroups (stage_set_send_copy_blocks); -1 keeps the library default")
    ap.add_argument("--wstep-window", type=int, default=0,
                    help="most micro-batches whose gradient accumulation goes into one W step (stage_set_wstep_window); "
                         "1: every backward accumulates by itself; 0 (default): the library's default, 8")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic, used to scale "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command)")
    ap.add_argument("--wgrad-stream", type=int, default=-1, choices=[-1, 0, 1],
                    help="1: weight and bias gradients run on the other lane's stream beside the input-gradient chain; "
                         "0: everything on the op's own stream; -1 (default): the library's own choice for the stage's shape")
    ap.add_argument("--lanes", type=int, default=0, choices=[0, 1, 2],
                    help="compute lanes: ops in flight at once, within the plan's peak of live micro-batches; 0 (default): "
                         "the library's own choice for the stage's shape (2 for small blocks, 1 for large ones)")
    ap.add_argument("--adaptive", dest="adaptive", action="store_true", default=None,
                    help="also time the same steps under the tuner (run_kFkB_adaptive: moving averages of the measured "
                         "transfer times, k re-chosen every 2 iterations among the workload's k values); on by default for "
                         "the very wide stage under its drifting delays (the configuration that names an adaptive k)")
    ap.add_argument("--no-adaptive", dest="adaptive", action="store_false")
    ap.add_argument("--pipeline-stages", type=int, default=0,
                    help="also time the same iteration run as a pipeline of this many virtual stages on the one GPU "
                         "(run_pipeline_kFkB); reported under \"pipeline_sim\", the headline value is unchanged")
    ap.add_argument("--candidates-gb", type=float, default=0.0,
                    help="also time every candidate plan (k, b) on the memory-limit curve (paper Section 4.2) at this many GB "
                         "of stashed activations; reported under \"candidates\", the headline value is unchanged")
    ap.add_argument("--recompute", action="store_true",
                    help="activation recomputation: LayerNorm and GELU outputs are formed again in the backward pass")
    ap.add_argument("--dtype", default=None, choices=["bf16", "f16"],
                    help="storage type of a 16-bit workload (default bf16; f16 is the paper's precision, same kernels)")
    ap.add_argument("--delay", default=None,
                    help="per-transfer injected delay: none | lognormal | bimodal | drift | fixed:MS; default: the workload's "
                         "own (lognormal: mean 2 ms, sigma 0.5; bimodal: 0.5 ms w.p. 0.7 / 10 ms w.p. 0.3; drift: 0 -> 20 ms "
                         "over the timed steps; fixed:MS: every transfer MS milliseconds)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build drives one pipeline stage on ONE GPU; --gpus %d is not supported "
              "(a pipeline puts one such stage on every GPU; no collective is involved)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import kfkb_synth as synth
    import paper_2303_01675_amd as kf

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    kf.load_library()                      # fails loudly if libkfkb.so was not built
    t_start = time.time()

    def workload(name):
        w = dict(WORKLOADS[name])
        if args.dtype is not None and w["dtype"] != "f32":
            w["dtype"] = args.dtype
        if args.ks and name == args.workload:
            w["ks"] = tuple(int(k) for k in args.ks.split(","))
        if args.microbatches and name == args.workload:
            w["M"] = args.microbatches
        return w

    def measure(name, steps, warmup, with_extras):
        w = workload(name)
        progress("%s: setting up weights, inputs and the stage" % name)
        run = Run(name, w, args, kf, synth, np)
        scan_steps = args.scan_steps or max(3, steps // 5)
        per_k = {}
        for k_req in w["ks"]:
            k, row = run.timed(k_req, 0 if w.get("tiled") else 1, scan_steps, torch)   # iterations of seconds need no warm-up step
            per_k[k] = row
            progress("%s: scan k = %d: %.1f ms per iteration (%d steps, delay %s)" % (name, k, row["ms_per_step"], scan_steps, run.delay_model))
        best_k = max(per_k, key=lambda k: per_k[k]["samples_per_s"])
        _, head = run.timed(best_k, warmup, steps, torch)
        progress("%s: k = %d, %d warm-up + %d timed steps: %.1f ms per iteration" % (name, best_k, warmup, steps, head["ms_per_step"]))
        k1 = per_k.get(1)
        res = dict(run=run, w=w, per_k=per_k, best_k=best_k, head=head,
                   best_k_over_k1=(head["samples_per_s"] / k1["samples_per_s"]) if k1 else None)
        return res

    res = measure(args.workload, args.steps, args.warmup, True)
    run, w, per_k, best_k, best = res["run"], res["w"], res["per_k"], res["best_k"], res["head"]
    L, H, heads, T, b, M = w["L"], w["H"], w["heads"], w["T"], w["b"], w["M"]

    pipeline_sim = None
    if args.pipeline_stages > 1:
        S = args.pipeline_stages
        wire = torch.empty(kf.stage_pipeline_bytes(S, M), dtype=torch.uint8, device="cuda")
        kf.stage_sync()
        kf.stage_pipeline_bind(wire, S, M)

        def boundary_delays(step_index, n_steps):
            n = (S - 1) * M
            if run.delay_model == "none":
                return None, None
            if run.delay_model == "lognormal":
                return tuple(synth.delays_lognormal(n, 2.0, 0.5, seed=9000 + 2 * step_index + i) for i in range(2))
            if run.delay_model == "bimodal":
                return tuple(synth.delays_bimodal(n, 0.5, 10.0, 0.7, seed=9000 + 2 * step_index + i) for i in range(2))
            d = np.tile(synth.delays_drift(M, step_index, n_steps, 20.0), S - 1)
            return d, d

        def pstep(k, i=0):
            kf.stage_set_delays(*delays_for(synth, run.delay_model, M, i, args.steps))
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
        pipeline_sim = dict(stages=S, blocks_per_stage=L // S, delay=run.delay_model, per_k=pk,
                            note="S virtual stages share the one GPU: total work equals the single stage's, so the "
                                 "figures show what the schedule and the boundary delays cost, not a pipeline speed-up")

    adaptive = None
    if args.adaptive if args.adaptive is not None else (args.workload == "very-wide-stage" and run.delay_model == "drift" and len(per_k) > 1):
        cands = sorted(k for k in per_k)
        kf.stage_sync()
        kf.kfkb_tuner_config(2, 2, cands)
        kf.stage_set_delays(None, None, None, None)
        kf.stage_tuner_calibrate(M, 1)
        progress("tuner calibrated (every candidate k run once without delay)")
        chosen = []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            kf.stage_set_delays(*delays_for(synth, run.delay_model, M, i, args.steps))
            kf.stage_zero_grads()
            chosen.append(kf.run_kFkB_adaptive(M, run.limit))
        kf.stage_sync()
        dt_s = time.perf_counter() - t0
        adaptive = dict(ms_per_step=1e3 * dt_s / args.steps, samples_per_s=M * b * args.steps / dt_s, k_per_step=chosen,
                        window=2, interval=2, candidates=cands)
        progress("adaptive k: %.1f ms per iteration, k per step %s" % (adaptive["ms_per_step"], chosen))

    prof_steps = args.profile_steps or (2 if w.get("tiled") else args.steps)
    roofline, kernels = kernel_pass(run, best_k, prof_steps, args)
    progress("per-kernel pass done (%d steps on one lane)" % prof_steps)

    cpu = None if args.no_cpu_baseline else cpu_baseline(run, np)
    if cpu is not None:
        progress("CPU baseline (the oracle) timed")

    out = {
        "metric": "stage fwd+bwd samples/sec (kFkB iteration, best k of 1,2,4,8 under the workload's transfer delays)",
        "value": best["samples_per_s"],
        "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": best["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w["dtype"],
        "data": "synthetic" + (" (one seeded draw repeated over the weights, 2 micro-batches reused)" if w.get("tiled") else ""),
        "config": {"workload": args.workload, "layers": L, "hidden": H, "heads": heads, "seq_len": T, "micro_batch": b,
                   "num_microbatches": M, "global_batch": M * b, "k": best_k, "delay": run.delay_model,
                   "activation_limit_bytes": run.limit,
                   "side_streams_overlap": bool(run.overlap), "wgrad_stream": bool(run.wgrad_stream), "compute_lanes": run.lanes,
                   "recompute": bool(args.recompute)},
        "tflops": best["tflops"], "tflops_megatron_convention": best["tflops_megatron"],
        "frac_of_bf16_peak": best["tflops"] / PEAK_BF16_TFLOPS if w["dtype"] != "f32" else None,   # fp16 has the same peak
        "per_k": {str(k): v for k, v in per_k.items()},
        "best_k_over_k1": res["best_k_over_k1"],
        "adaptive": adaptive, "pipeline_sim": pipeline_sim, "roofline": roofline, "kernels": kernels[:14], "cpu_baseline": cpu,
        "setup_seconds": run.setup_seconds,
    }
    blocks_small = run.blocks
    run.st.close()
    if args.candidates_gb > 0:
        per_sample = kf.kfkb_activation_bytes_per_microbatch(L, 1, T, H, heads, 4 * H, 2 if w["dtype"] != "f32" else 4,
                                                             recompute=int(args.recompute))
        cands = kf.kfkb_enumerate_candidates(M * b, int(args.candidates_gb * 1e9), per_sample)
        cblocks = blocks_small if blocks_small is not None else synth.stage_weights_tiled(L, H, 4 * H, w["dtype"], out=np.float32)
        rows = []
        for ck, cb in cands:
            cM = M * b // cb
            cst = kf.StageBuffers(cblocks, run.dt, heads, T, cb, cM, ck, recompute=int(args.recompute))
            pair = [(synth.microbatch_inputs(j, cb, T, H, w["dtype"]), synth.microbatch_upstream_grads(j, cb, T, H, w["dtype"])) for j in range(2)]
            for mb in range(cM):
                cst.set_inputs_one(mb, *pair[mb % 2])
            if args.lanes:
                kf.stage_set_compute_lanes(args.lanes)
            if args.wgrad_stream >= 0:
                kf.stage_set_wgrad_stream(args.wgrad_stream)

            def cstep(i):
                kf.stage_set_delays(*delays_for(synth, run.delay_model, cM, i, args.steps))
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
        out["candidates"] = dict(global_batch=M * b, activation_limit_gb=args.candidates_gb, delay=run.delay_model, plans=rows)

    sec_name = args.secondary if args.secondary is not None else ("gpt2-medium-stage" if args.workload == "very-wide-stage" else "none")
    if sec_name != "none" and sec_name != args.workload:
        del run, res
        torch.cuda.empty_cache()
        r2 = measure(sec_name, args.steps, args.warmup, False)
        w2, h2 = r2["w"], r2["head"]
        rl2, k2 = kernel_pass(r2["run"], r2["best_k"], args.profile_steps or (2 if w2.get("tiled") else min(args.steps, 5)), args)
        out["secondary"] = dict(workload=sec_name, k=r2["best_k"], delay=r2["run"].delay_model, value=h2["samples_per_s"],
                                unit="samples/s", ms_per_step=h2["ms_per_step"], tflops=h2["tflops"],
                                frac_of_bf16_peak=h2["tflops"] / PEAK_BF16_TFLOPS if w2["dtype"] != "f32" else None,
                                per_k={str(k): v for k, v in r2["per_k"].items()}, roofline=rl2, kernels=k2[:8])
        r2["run"].st.close()
    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        c = torch.empty_like(a)
        c.copy_(a)
        torch.cuda.synchronize()
    out["wall_seconds"] = time.time() - t_start
    print(json.dumps(out))


if __name__ == "__main__":
    main()
