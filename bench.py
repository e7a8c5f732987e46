#!/usr/bin/env python3
"""Benchmark of one n-wise interlocking-backprop training step on one MI355X.

A step is the whole hot path: K x (il_stage_forward + il_head_xent) and the n-wise
truncated backward il_stage_backward_nwise for k = K..1, all parameter gradients final,
on seeded synthetic tokens already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps 20] [--warmup 5] [--workload large] [--n N] [--also large:6,medium,many_head,small]

`value` is the workload named by --workload (default: Large, n = 2 - the largest single-GPU
configuration, the one the MFMA-utilisation target is about); the workloads named by --also (default: Large with n = K,
Medium, Many-head, Small) are measured the same way and reported under "other_workloads".
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

# HBM-side bytes per GEMM kernel launch (average over the GEMM launches of one step), from two
# rocprofv3 --pmc runs of this script (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same
# counter reads for the library's streaming copy of known size (--calibration-copy-mib 256): see
# profiles/traffic_<workload>.md.  bench.py cannot run the profiler on itself, so the figures are
# carried here for the workloads they were measured on and are null for any other.
MEASURED_TRAFFIC = {
    "small_bf16_n2": 41.98e6,   # 32.190 MB read + 9.788 MB written per launch, 1536 launches (1.85 x)
    "large_bf16_n2": 478.98e6,  # 390.00 MB read + 88.97 MB written per launch, 4320 launches (2.15 x algorithmic)
    "medium_bf16_n2": 179.40e6,  # 140.98 + 38.42 MB, 2880 launches (1.88 x)
    "many_head_bf16_n3": 238.28e6,  # 190.65 + 47.63 MB, 2880 launches (1.99 x)
}

# which roofline bounds a kernel class, and the peak its fraction is taken against
CLASS_BOUND = {"gemm_fwd": "mfma", "gemm_dgrad": "mfma", "gemm_wgrad": "mfma", "gemm_head": "mfma",
               "attn_fwd": "mfma", "attn_bwd": "mfma", "ln_fwd": "hbm", "ln_bwd": "hbm", "colsum": "hbm",
               "xent": "hbm", "misc": "hbm"}


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


def time_graph_replays(st, steps, warmup):
    """One whole step (both of the library's streams, their event fork / joins) captured into a HIP graph
    after an eager step has created the library's stream and events; K replays timed like K eager steps."""
    import torch
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st.stream):
        st.run()
    torch.cuda.synchronize()
    with torch.cuda.stream(st.stream):
        for _ in range(warmup):
            g.replay()
        st.stream.synchronize()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(st.stream)
        for _ in range(steps):
            g.replay()
        e1.record(st.stream)
        st.stream.synchronize()
        torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    losses = st.results()["losses"]
    del g
    return ms, losses


def class_table(w, dev_params, steps, mode):
    """Per-kernel-class figures from the library's own timers.  mode 1: everything in line on one
    stream, HIP events around each launch group and attached to each GEMM dispatch.  mode 2: the step
    as it is timed (two streams), timers attached to the GEMM dispatches only."""
    from paper_2010_04116_amd import binding
    st = binding.Step(w, dev_params, profile=mode)
    st.set_inputs(*INPUTS)
    st.run()
    binding.il_profile_read(st.ctx)             # discard warm-up
    for _ in range(steps):
        st.run()
    prof = binding.il_profile_read(st.ctx)
    st.close()
    for v in prof.values():
        for key in ("ms", "flops", "bytes", "launches", "kernel_ms"):
            v[key + "_per_step"] = v[key] / steps
    return prof


def cpu_baseline(w, params, x0, tgt):
    """The float64 oracle, as it stands, on the host cores, on a bounded sample of the workload
    (about 10-30 s of CPU work at the ~0.1 TFLOP/s the numpy oracle reaches).  Small workloads: the
    first b sequences of the batch through the whole model (every per-token cost is the same as in the
    full batch, so tokens/s is directly comparable).  Workloads whose single sequence costs more than
    that budget: sequence 0 through component 1 and head 1 alone (forward, loss, local backward), scaled
    to the whole step by the ratio of algorithmic flops - the sample line says so."""
    from oracle import interlock as O
    per_seq = minimal_flops(w.with_(B=1))
    cores = len(os.sched_getaffinity(0))
    if per_seq <= 3.0e12:
        b = int(max(1, min(w.B, np.floor(2.0e12 / per_seq))))
        ws = w.with_(B=b)
        t0 = time.perf_counter()
        O.nwise_streams(params, x0[: b * w.T], tgt[:b], ws.B, ws.T, ws.H, ws.n)
        dt = time.perf_counter() - t0
        return {"value": b * w.T / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle", "seconds": dt,
                "extrapolated": False,
                "sample": f"first {b} of {w.B} sequences ({b * w.T} tokens), all {w.K} components and heads, "
                          f"n={w.n}, float64 numpy stream path, one run"}
    ws = w.with_(B=1, K=1, n=1)
    sub = {"components": params["components"][:1], "heads": params["heads"][:1],
           "head_blocks": params["head_blocks"][:1]}
    t0 = time.perf_counter()
    O.nwise_streams(sub, x0[: w.T], tgt[:1], 1, w.T, w.H, 1)
    dt = time.perf_counter() - t0
    ratio = per_seq / minimal_flops(ws)
    return {"value": w.T / (dt * ratio), "unit": "tokens/s", "cores": cores, "kind": "oracle", "seconds": dt,
            "extrapolated": True, "flop_ratio_step_over_sample": ratio,
            "sample": f"sequence 0 ({w.T} tokens) through component 1 ({w.L} blocks) and head 1 only, n=1 "
                      f"(forward, loss, local backward), float64 numpy stream path, one run of {dt:.1f} s; scaled to "
                      f"the whole step (all {w.K} components and heads, n={w.n}) by the ratio of algorithmic "
                      f"flops, {ratio:.2f}"}


INPUTS = None
PARAMS = {}


def measure(w, steps, warmup, peaks):
    """Time `steps` whole steps of workload w, then the GEMM kernels inside the same two-stream step,
    then the per-class table in a single-stream profiling context."""
    global INPUTS
    import torch
    from paper_2010_04116_amd import binding, synth
    key = (w.name, w.dtype, w.K, w.L, w.d, w.H, w.m, w.V, w.Lh)        # (the window does not enter the parameters)
    if key not in PARAMS:
        PARAMS.clear()
        params = synth.make_params(w)                  # N(0,0.02) weights, biases 0, LN 1/0
        flat = torch.from_numpy(binding.pack_params(w, params))
        PARAMS[key] = (params, (flat.to(torch.bfloat16) if w.dtype == "bf16" else flat).to("cuda:0").contiguous())
        del flat
    params, dev_params = PARAMS[key]
    inp, tgt = synth.make_tokens(w)
    x0 = synth.make_x0(w, inp)
    INPUTS = (x0, tgt)

    stream = torch.cuda.Stream()                       # (a capture cannot run on the default stream)
    st = binding.Step(w, dev_params, stream=stream)
    with torch.cuda.stream(stream):
        st.set_inputs(x0, tgt)
        eager_ms, wall_ms = time_steps(st, steps, warmup)
        losses = st.results()["losses"]
    graph_ms, glosses = time_graph_replays(st, steps, warmup)
    assert np.array_equal(losses, glosses), (losses, glosses)   # a replay is the same step, bit for bit
    st.close()
    del st
    ms = min(eager_ms, graph_ms)
    # uniform random tokens: every loss sits at ln V plus half the logit variance, which grows with depth
    assert np.all(np.isfinite(losses)) and np.all(losses > np.log(w.V) - 0.5) and np.all(losses < 4 * np.log(w.V)), losses

    psteps = max(2, min(steps, 5))
    flops = minimal_flops(w)
    bf = w.dtype == "bf16"
    prof = class_table(w, dev_params, psteps, 1)
    gemm = [k for k in prof if k.startswith("gemm")]
    g_fl = sum(prof[k]["flops_per_step"] for k in gemm)
    g_by = sum(prof[k]["bytes_per_step"] for k in gemm)
    g_n = sum(prof[k]["launches_per_step"] for k in gemm)
    peak = PEAK_BF16_TFLOPS if bf else PEAK_F32_TFLOPS
    if bf:
        # events attached to each MFMA GEMM dispatch: the kernel's own execution time
        iso_ms = sum(prof[k]["kernel_ms_per_step"] for k in gemm)
        instep = class_table(w, dev_params, psteps, 2)
        g_ms = sum(instep[k]["kernel_ms_per_step"] for k in gemm)
        how = ("HIP events attached to each GEMM kernel dispatch (hipExtLaunchKernelGGL) inside the two-stream step "
               "as it is timed for `value`: other kernels run beside the GEMMs; `isolated` is the same launches "
               "with the whole step in line on one stream")
    else:
        iso_ms = g_ms = sum(prof[k]["ms_per_step"] for k in gemm)
        instep = None
        how = "HIP events recorded around each GEMM launch, single stream"
    achieved = g_fl / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    iso = g_fl / (iso_ms * 1e-3) / 1e12 if iso_ms > 0 else 0.0
    traffic = MEASURED_TRAFFIC.get(f"{w.name}_{w.dtype}_n{w.n}")
    roof = {"bound": "mfma" if bf else "alu",
            "kernel": "gemm_dma_kernel / gemm_persist_kernel: every GEMM launch of one step (forward, dgrad, wgrad, head)"
            if bf else "gemm_simt_kernel: every GEMM launch of one step",
            "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
            "traffic": traffic, "launches_per_step": g_n, "avg_launch_ms": g_ms / max(g_n, 1),
            "algorithmic_gflop_per_launch": g_fl / max(g_n, 1) / 1e9,
            "algorithmic_bytes_per_launch": g_by / max(g_n, 1),
            "traffic_over_algorithmic_bytes": (traffic / (g_by / max(g_n, 1))) if traffic else None,
            "hbm_gbs_from_traffic": (traffic / (g_ms / max(g_n, 1) * 1e-3) / 1e9) if traffic and g_ms > 0 else None,
            "frac_is": "in-step" if bf else "single stream",
            "isolated": {"achieved": iso, "frac": iso / peak, "avg_launch_ms": iso_ms / max(g_n, 1)},
            "timing": how}
    if bf and peaks:
        roof["measured_peak"] = peaks["mfma_only_tflops"]
        roof["frac_of_measured_peak"] = achieved / peaks["mfma_only_tflops"]

    kernels = {}
    for k, v in prof.items():
        bound = CLASS_BOUND.get(k, "hbm")
        if not bf and bound == "mfma":
            bound = "alu"
        t = v["ms_per_step"] * 1e-3
        e = {"ms_per_step": round(v["ms_per_step"], 4), "launches": v["launches_per_step"], "bound": bound}
        if bound in ("mfma", "alu"):
            e["tflops"] = v["flops_per_step"] / t / 1e12 if t > 0 and v["flops_per_step"] else None
            e["frac"] = e["tflops"] / peak if e["tflops"] else None
            if bf and k in gemm:                       # the kernel alone, and inside the two-stream step
                tk, ti = v["kernel_ms_per_step"] * 1e-3, instep[k]["kernel_ms_per_step"] * 1e-3
                e["kernel_tflops"] = v["flops_per_step"] / tk / 1e12 if tk > 0 else None
                e["kernel_frac"] = e["kernel_tflops"] / peak if e["kernel_tflops"] else None
                e["in_step_kernel_tflops"] = v["flops_per_step"] / ti / 1e12 if ti > 0 else None
                e["in_step_kernel_frac"] = e["in_step_kernel_tflops"] / peak if e["in_step_kernel_tflops"] else None
        else:
            e["gbs"] = v["bytes_per_step"] / t / 1e9 if t > 0 and v["bytes_per_step"] else None
            e["frac"] = e["gbs"] / PEAK_HBM_GBS if e["gbs"] else None
            if e["gbs"] and peaks:
                e["frac_of_measured_copy"] = e["gbs"] / peaks["stream_copy_gbs"]
        kernels[k] = e
    res = {
        "ms_per_step": ms, "wall_ms_per_step": wall_ms, "tokens_per_s": w.N / (ms * 1e-3),
        "launch": {"timed_as": "hip_graph_replay" if graph_ms <= eager_ms else "eager_calls",
                   "eager_ms_per_step": eager_ms, "graph_replay_ms_per_step": graph_ms,
                   "note": "one whole step (five C-ABI calls per component, both library streams) captured once "
                           "into a HIP graph and replayed; the eager figure issues the same calls from Python"},
        "mfma_utilisation_pct_of_bf16_peak": 100.0 * flops / (ms * 1e-3) / (PEAK_BF16_TFLOPS * 1e12),
        "algorithmic_tflop_per_step": flops / 1e12,
        "algorithmic_hbm_gbs": (sum(v["bytes_per_step"] for v in prof.values()) / (ms * 1e-3) / 1e9),
        "roofline": roof,
        "kernels": kernels,
        "kernels_note": "single-stream profiling context; ms_per_step brackets each launch group with HIP events "
                        "(upper bounds: an event costs a few microseconds between launches)",
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


def gemm_reference(w, iters=10, rot=6):
    """Context for the GEMM rates: the library's kernel (il_test_gemm, epilogue = plain store) and the vendor
    library (torch.matmul, which dispatches to hipBLASLt / rocBLAS) on the headline workload's main GEMM
    shapes, both timed the same way - HIP events around `iters` launches that rotate through `rot` operand sets,
    so operands come from HBM / Infinity Cache as they do inside a step.  The vendor library is not part of the
    product path; this is a yardstick for what a tuned kernel reaches on this board."""
    import torch
    from paper_2010_04116_amd import binding as b
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream()
    N, d, m, V = w.N, w.d, w.m, w.V
    live = max(b.il_routing_plan(w.K, w.n)[0])
    nc = min(N // 2, 2048)
    shapes = [("fwd_qkv", N, 3 * d, d, 0, 1, 0), ("fwd_o", N, d, d, 0, 1, 0), ("fwd_fc1", N, m, d, 0, 1, 0),
              ("fwd_fc2", N, d, m, 0, 1, 0), (f"dgrad_fc2_{live}streams", live * N, m, d, 0, 0, 0),
              (f"dgrad_fc1_{live}streams", live * N, d, m, 0, 0, 0), ("wgrad_fc1", d, m, N, 1, 1, 6),
              ("head_logits", nc, V, d, 0, 1, 0), ("head_dx", nc, d, V, 0, 0, 5)]
    out = {}
    def timed(fn):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for i in range(iters):
            fn(i)
        e1.record(st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters
    for name, M, Nn, K, akm, bkm, epi in shapes:
        As = [(torch.randn((K, M) if akm else (M, K), device=dev) * 0.5).to(torch.bfloat16) for _ in range(rot)]
        Bs = [(torch.randn((K, Nn) if bkm else (Nn, K), device=dev) * 0.5).to(torch.bfloat16) for _ in range(rot)]
        C = torch.zeros((M, Nn), device=dev, dtype=torch.float32 if epi in (5, 6) else torch.bfloat16)
        ours = timed(lambda i: b.il_test_gemm(b.IL_BF16, As[i % rot], Bs[i % rot], M, Nn, K, M if akm else K,
                                              Nn if bkm else K, akm, bkm, epi, C, stream=st.cuda_stream))
        lib = timed(lambda i: torch.matmul(As[i % rot].t() if akm else As[i % rot],
                                           Bs[i % rot] if bkm else Bs[i % rot].t()))
        fl = 2.0 * M * Nn * K
        out[name] = {"M": M, "N": Nn, "K": K, "this_library_tflops": fl / ours / 1e9,
                     "vendor_library_tflops": fl / lib / 1e9}
        del As, Bs, C
    return out


def measured_peaks(copy_mib=1024):
    """What the board itself reaches: a matrix-unit-only loop and a streaming copy (the library's
    micro-benchmarks), reported beside the nominal peaks the roofline fractions use."""
    import torch
    from paper_2010_04116_amd import binding
    n = copy_mib << 20
    src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    st = torch.cuda.current_stream().cuda_stream
    mf = max(binding.il_measure_mfma_peak(dst, 20000, stream=st) for _ in range(2))
    cp = max(binding.il_measure_copy_peak(dst, src, n, 10, stream=st) for _ in range(2))
    del src, dst
    return {"mfma_only_tflops": mf, "mfma_only_frac_of_nominal": mf / PEAK_BF16_TFLOPS,
            "stream_copy_gbs": cp, "stream_copy_frac_of_nominal": cp / PEAK_HBM_GBS,
            "how": f"il_measure_mfma_peak (512 workgroups x 4 wavefronts x 80000 MFMAs 32x32x16 bf16, registers only); "
                   f"il_measure_copy_peak ({copy_mib} MiB device-to-device, read + written bytes, the better of a plain 16-byte-per-lane copy "
                   f"and one with four vectors in flight and non-temporal accesses, best of 2 x 10 launches each)"}


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
    ap.add_argument("--workload", default="large")
    ap.add_argument("--n", type=int, default=0, help="override the workload's window")
    ap.add_argument("--also", default="large:6,medium,many_head,small",
                    help="comma-separated further workloads reported under other_workloads ('none' = none); "
                         "name:n overrides the window, e.g. large:6")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the MFMA-only / streaming-copy micro-benchmarks")
    ap.add_argument("--peaks-only", action="store_true",
                    help="run only the MFMA-only / streaming-copy micro-benchmarks and print their JSON line")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="first run two launches of the library's streaming copy kernel over this many MiB "
                         "(a kernel of known HBM traffic, against which rocprofv3's FETCH_SIZE / WRITE_SIZE "
                         "counters are scaled)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (--gpus 1); depthwise sharding "
                 "across GPUs (one component per GPU, point-to-point activations and gradient streams) is not built")
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: launched with WORLD_SIZE > 1; this build runs on exactly one GPU")

    from paper_2010_04116_amd import binding, synth
    if a.calibration_copy_mib > 0:
        import torch
        src = torch.ones(a.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        binding.il_measure_copy_peak(dst, src, a.calibration_copy_mib << 20, 1,
                                     stream=torch.cuda.current_stream().cuda_stream)
        del src, dst
    peaks = None if a.no_peaks else measured_peaks()
    if a.peaks_only:
        print(json.dumps({"measured_peaks": peaks, "nominal": {"bf16_mfma_tflops": PEAK_BF16_TFLOPS,
                                                                "hbm_gbs": PEAK_HBM_GBS}}))
        return
    w = synth.WORKLOADS[a.workload]
    if a.n:
        w = w.with_(n=a.n)
    res, params, x0, tgt = measure(w, a.steps, a.warmup, peaks)
    out = {
        "metric": "tokens/sec per n-wise train step at 1 GPU",
        "value": res.pop("tokens_per_s"), "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic", "config": config_of(w),
    }
    out.update(res)
    if peaks:
        out["measured_peaks"] = peaks
    if w.dtype == "bf16" and not a.no_peaks:
        out["gemm_reference"] = gemm_reference(w)
    out["target"] = {"mfma_utilisation_pct": 50.0, "met": out["mfma_utilisation_pct_of_bf16_peak"] >= 50.0,
                     "note": "north star: >= 50 % of bf16 MFMA peak on the GEMM-dominated configurations"}
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, params, x0.astype(np.float64), tgt)
    del params, x0, tgt
    others = {}
    for spec in [x for x in a.also.split(",") if x and x != "none"]:
        name, _, nn = spec.partition(":")
        wo = synth.WORKLOADS[name]
        if nn:
            wo = wo.with_(n=int(nn))
        if (wo.name, wo.n) == (w.name, w.n):
            continue
        ro = measure(wo, min(a.steps, 10), min(a.warmup, 3), peaks)[0]
        ro.pop("losses")
        ro["config"] = config_of(wo)
        others[f"{wo.name}_{wo.dtype}_n{wo.n}"] = ro
    if others:
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
