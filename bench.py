#!/usr/bin/env python3
"""Benchmark of one n-wise interlocking-backprop training step on one MI355X.

A step is the whole hot path: K x (il_stage_forward + il_head_xent) and the n-wise
truncated backward il_stage_backward_nwise for k = K..1, all parameter gradients final,
on seeded synthetic tokens already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps 20] [--warmup 5] [--workload small] [--n N] [--also medium]

`value` is the workload named by --workload (default: the Small configuration); the workloads
named by --also are measured the same way and reported under "other_workloads".
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# HBM-side bytes per GEMM kernel launch (average over the launches of one step), from two
# rocprofv3 --pmc runs of this script (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same
# counter reads for a 256 MiB device-to-device copy (--calibration-copy-mib 256): see
# profiles/traffic_small_bf16_n2.md.  bench.py cannot run the profiler on itself, so the
# figure is carried here for the workload it was measured on and is null for any other.
MEASURED_TRAFFIC = {
    "small_bf16_n2": 41.88e6,   # 32.18 MB read + 9.70 MB written per launch, 768 launches
}


def minimal_flops(w):
    """Algorithmic flops of one step, not counting recomputation: per block forward
    GEMMs 24 N d^2 (for m = 4d; general: 2N(4d^2 + 2dm)) and causal attention 2 B T^2 d;
    backward per distinct stream: dgrad = forward GEMM flops, attention backward 2.5x;
    one weight-gradient pass per block; head 3 x 2 N d V."""
    from paper_2010_04116_amd import binding
    N, d, m = w.N, w.d, w.m
    G = 2.0 * N * (4 * d * d + 2 * d * m)
    At = 2.0 * w.B * w.T * w.T * d
    live, _ = binding.il_routing_plan(w.K, w.n, "window_sum")
    tot = 0.0
    for k in range(w.K):
        tot += w.L * (G + At)                                   # forward
        tot += w.L * ((live[k] + 1) * G + 2.5 * live[k] * At)   # dgrad per stream + one wgrad
        tot += 3 * 2.0 * N * d * w.V                            # head fwd + dx + dW
        tot += w.Lh * ((G + At) + (2 * G + 2.5 * At))           # the head's own blocks: forward, one stream back
    return tot


def time_steps(st, steps, warmup):
    import torch
    for _ in range(warmup):
        st.run()
    st.stream.synchronize()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(st.stream)
    for _ in range(steps):
        st.run()
    e1.record(st.stream)
    st.stream.synchronize()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall / steps


def kernel_table(w, flat, steps):
    """Per-kernel-class HIP-event times from the library's own profiling hooks."""
    from paper_2010_04116_amd import binding
    st = binding.Step(w, flat, profile=True)
    st.set_inputs(*INPUTS)
    st.run()
    binding.il_profile_read(st.ctx)             # discard warm-up
    for _ in range(steps):
        st.run()
    prof = binding.il_profile_read(st.ctx)
    st.close()
    for v in prof.values():
        v["steps"] = steps
        v["ms_per_step"] = v["ms"] / steps
        v["flops_per_step"] = v["flops"] / steps
        v["bytes_per_step"] = v["bytes"] / steps
        v["launches_per_step"] = v["launches"] / steps
    return prof


def cpu_baseline(w, params, x0, tgt):
    """The float64 oracle, as it stands, on the host cores, on a bounded sample: the
    first `b` sequences of the batch through the whole model (every per-token cost is
    the same as in the full batch, so tokens/s is directly comparable)."""
    from oracle import interlock as O
    # aim at ~10-30 s: assume ~100 GFLOP/s float64 on the host
    full = minimal_flops(w)
    b = int(max(1, min(w.B, np.floor(w.B * 2.0e12 / full))))
    ws = w.with_(B=b)
    xs = x0[: b * w.T]
    ts = tgt[:b]
    t0 = time.perf_counter()
    O.nwise_streams(params, xs, ts, ws.B, ws.T, ws.H, ws.n)
    dt = time.perf_counter() - t0
    return {"value": b * w.T / dt, "unit": "tokens/s", "cores": len(os.sched_getaffinity(0)),
            "kind": "oracle", "seconds": dt,
            "sample": f"first {b} of {w.B} sequences ({b * w.T} tokens), all {w.K} components and heads, "
                      f"n={w.n}, float64 numpy stream path, one run"}


INPUTS = None


def measure(w, steps, warmup):
    """Time `steps` whole steps of workload w, then the per-class table in a profiling context."""
    global INPUTS
    from paper_2010_04116_amd import binding, synth
    params = synth.make_params(w)                      # N(0,0.02) weights, biases 0, LN 1/0
    inp, tgt = synth.make_tokens(w)
    x0 = synth.make_x0(w, inp)
    flat = binding.pack_params(w, params)
    INPUTS = (x0, tgt)

    st = binding.Step(w, flat)
    st.set_inputs(x0, tgt)
    ms, wall_ms = time_steps(st, steps, warmup)
    losses = st.results()["losses"]
    st.close()
    # uniform random tokens: every loss sits at ln V plus half the logit variance, which grows with depth
    assert np.all(np.isfinite(losses)) and np.all(losses > np.log(w.V) - 0.5) and np.all(losses < 4 * np.log(w.V)), losses

    prof = kernel_table(w, flat, max(2, min(steps, 5)))
    flops = minimal_flops(w)
    gemm = [k for k in prof if k.startswith("gemm")]
    g_fl = sum(prof[k]["flops_per_step"] for k in gemm)
    g_by = sum(prof[k]["bytes_per_step"] for k in gemm)
    g_n = sum(prof[k]["launches_per_step"] for k in gemm)
    if w.dtype == "bf16":
        # events attached to each MFMA GEMM dispatch: the kernel's own execution time
        g_ms = sum(prof[k]["kernel_ms"] for k in gemm) / prof[gemm[0]]["steps"]
        peak, how = PEAK_BF16_TFLOPS, "HIP events attached to each GEMM kernel dispatch"
    else:
        g_ms = sum(prof[k]["ms_per_step"] for k in gemm)
        peak, how = PEAK_F32_TFLOPS, "HIP events recorded around each GEMM launch"
    achieved = g_fl / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    res = {
        "ms_per_step": ms, "wall_ms_per_step": wall_ms, "tokens_per_s": w.N / (ms * 1e-3),
        "mfma_utilisation_pct_of_bf16_peak": 100.0 * flops / (ms * 1e-3) / (PEAK_BF16_TFLOPS * 1e12),
        "algorithmic_tflop_per_step": flops / 1e12,
        "roofline": {"bound": "mfma" if w.dtype == "bf16" else "alu",
                     "kernel": "gemm_dma_kernel / gemm_persist_kernel: every GEMM launch of one step (forward, dgrad, wgrad, head)"
                     if w.dtype == "bf16" else "gemm_simt_kernel: every GEMM launch of one step",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": MEASURED_TRAFFIC.get(f"{w.name}_{w.dtype}_n{w.n}"),
                     "launches_per_step": g_n, "avg_launch_ms": g_ms / max(g_n, 1),
                     "algorithmic_gflop_per_launch": g_fl / max(g_n, 1) / 1e9,
                     "algorithmic_bytes_per_launch": g_by / max(g_n, 1), "timing": how},
        "kernels": {k: {"ms_per_step": round(v["ms_per_step"], 4), "launches": v["launches_per_step"],
                        "tflops": (v["flops_per_step"] / (v["ms_per_step"] * 1e-3) / 1e12)
                        if v["ms_per_step"] > 0 and v["flops_per_step"] else None,
                        "gbs": (v["bytes_per_step"] / (v["ms_per_step"] * 1e-3) / 1e9)
                        if v["ms_per_step"] > 0 and v["bytes_per_step"] else None}
                    for k, v in prof.items()},
        "losses": [float(x) for x in losses],
    }
    res["optimizer"] = optimizer_line(w)
    res["embedding"] = embedding_line(w)
    return res, params, x0, tgt


def optimizer_line(w, reps=10):
    """The Adam update (App. B) over this workload's parameters: an HBM-bound kernel, timed on its own
    with HIP events on the current stream and reported beside the step (it is not part of `value`,
    which is the gradient step the metric names)."""
    import torch
    from paper_2010_04116_amd import binding
    count = binding.param_count(w)
    dev = "cuda:0"
    master = torch.zeros(count, device=dev)
    grads = torch.full((count,), 1e-3, device=dev)
    m = torch.zeros(count, device=dev)
    v = torch.zeros(count, device=dev)
    bf = w.dtype == "bf16"
    params = torch.zeros(count, dtype=torch.bfloat16, device=dev) if bf else master
    st = torch.cuda.current_stream()
    def go(step):
        binding.il_adam_step(w.dtype, params, master if bf else None, grads, m, v, count, step,
                             binding.il_lr_schedule(step, w.d, 4000), stream=st.cuda_stream)
    go(1)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for i in range(reps):
        go(2 + i)
    e1.record(st)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    per = 30 if bf else 28          # g, m, v, w read; m, v, w written; + the bf16 image
    gbs = count * per / (ms * 1e-3) / 1e9
    return {"kernel": "adam_step_kernel", "parameters": count, "ms": ms, "bound": "hbm", "achieved": gbs,
            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "bytes_per_parameter": per}


def embedding_line(w, reps=10):
    """Input embedding (App. B: module 1 holds the embedding matrix) and its gradient at this workload's
    shape, timed on their own; HBM-bound kernels, not part of `value`."""
    import torch
    from paper_2010_04116_amd import binding, synth
    dev = "cuda:0"
    tt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    eb = 2 if w.dtype == "bf16" else 4
    wte, wpe = synth.make_embeddings(w)
    inp, _ = synth.make_tokens(w)
    d_wte, d_wpe = torch.from_numpy(wte).to(tt).to(dev), torch.from_numpy(wpe).to(tt).to(dev)
    tok = torch.from_numpy(inp.reshape(-1).astype(np.int32)).to(dev)
    x0 = torch.empty(w.N, w.d, device=dev)
    dx0 = torch.randn(w.N, w.d, device=dev)
    dwte, dwpe = torch.empty(w.V, w.d, device=dev), torch.empty(w.T, w.d, device=dev)
    st = torch.cuda.current_stream()
    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(reps):
            fn()
        e1.record(st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    f_ms = timed(lambda: binding.il_embed_forward(w.dtype, d_wte, d_wpe, tok, w.B, w.T, w.d, w.V, x0,
                                                  stream=st.cuda_stream))
    b_ms = timed(lambda: binding.il_embed_backward(dx0, tok, w.B, w.T, w.d, w.V, dwte, dwpe, stream=st.cuda_stream))
    f_bytes = w.N * w.d * (eb + 4) + w.T * w.d * eb            # gathered rows + positions read, x0 written
    b_bytes = 2 * w.N * w.d * 4 + (w.V + w.T) * w.d * 4         # dx0 read by both kernels, both tables written
    return {"forward_ms": f_ms, "forward_gbs": f_bytes / (f_ms * 1e-3) / 1e9,
            "backward_ms": b_ms, "backward_gbs": b_bytes / (b_ms * 1e-3) / 1e9, "bound": "hbm",
            "peak": PEAK_HBM_GBS, "unit": "GB/s"}


def config_of(w):
    from paper_2010_04116_amd import synth
    return {"workload": f"{w.name}_{w.dtype}_n{w.n}", "K": w.K, "blocks_per_component": w.L,
            "d_model": w.d, "n_heads": w.H, "d_mlp": w.m, "vocab": w.V, "batch": w.B, "seq": w.T,
            "head_blocks": w.Lh,
            "n": w.n, "route": "window_sum", "param_seed": synth.PARAM_SEED, "token_seed": synth.TOKEN_SEED}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="small")
    ap.add_argument("--n", type=int, default=0, help="override the workload's window")
    ap.add_argument("--also", default="medium",
                    help="comma-separated further workloads reported under other_workloads ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="first run one device-to-device copy of this many MiB (a kernel of known HBM "
                         "traffic, against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (--gpus 1); depthwise sharding "
                 "across GPUs (one component per GPU, point-to-point activations and gradient streams) is not built")
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: launched with WORLD_SIZE > 1; this build runs on exactly one GPU")

    from paper_2010_04116_amd import synth
    if a.calibration_copy_mib > 0:
        import torch
        src = torch.ones(a.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    w = synth.WORKLOADS[a.workload]
    if a.n:
        w = w.with_(n=a.n)
    res, params, x0, tgt = measure(w, a.steps, a.warmup)
    out = {
        "metric": "tokens/sec per n-wise train step at 1 GPU",
        "value": res.pop("tokens_per_s"), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic", "config": config_of(w),
    }
    out.update(res)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, params, x0.astype(np.float64), tgt)
    del params, x0, tgt
    others = {}
    for name in [x for x in a.also.split(",") if x and x != "none" and x != a.workload]:
        wo = synth.WORKLOADS[name]
        ro = measure(wo, min(a.steps, 10), min(a.warmup, 3))[0]
        ro.pop("kernels"); ro.pop("losses")
        ro["config"] = config_of(wo)
        others[wo.name] = ro
    if others:
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
