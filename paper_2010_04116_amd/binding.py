"""ctypes binding of libinterlock (include/interlock.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch supplies device memory and the stream.  The library must be built first
(`python __graft_entry__.py`); loading fails loudly when it is missing - there is no
CPU or eager fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional

import numpy as np

from . import synth

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libinterlock.so")
_lib = None

IL_OK, IL_E_ARG, IL_E_SHAPE, IL_E_STATE, IL_E_WORKSPACE, IL_E_HIP = 0, -1, -2, -3, -4, -5
IL_F32, IL_BF16 = 0, 1
ROUTES = {"window_sum": 0, "far_head": 1, "mean_local_far": 2}
SYMBOLS = ("il_init", "il_stage_forward", "il_head_xent", "il_stage_backward_nwise", "il_free",
           "il_routing_plan", "il_profile_read", "il_status_string", "il_test_gemm", "il_lr_schedule",
           "il_adam_step", "il_embed_forward", "il_embed_backward", "il_set_accumulation",
           "il_time_per_batch", "il_optimal_microbatches", "il_measure_mfma_peak", "il_measure_copy_peak",
           "il_head_xent_static")


class il_config(C.Structure):
    _fields_ = [("K", C.c_int32), ("blocks_per_component", C.c_int32), ("d_model", C.c_int32),
                ("n_heads", C.c_int32), ("d_mlp", C.c_int32), ("vocab", C.c_int32),
                ("batch", C.c_int32), ("seq", C.c_int32), ("n", C.c_int32), ("dtype", C.c_int32),
                ("route", C.c_int32), ("ln_eps", C.c_float), ("head_chunk", C.c_int32),
                ("profile", C.c_int32), ("head_blocks", C.c_int32), ("reserved", C.c_int32),
                ("params", C.c_void_p), ("params_bytes", C.c_size_t),
                ("grads", C.c_void_p), ("grads_bytes", C.c_size_t), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p)]


class InterlockError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {il_status_string(status)}")


def load():
    """Load libinterlock.so and declare the prototypes.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python __graft_entry__.py` "
                          "(there is no fallback path)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32 = C.c_void_p, C.c_int32
    lib.il_init.argtypes = [C.POINTER(il_config), C.POINTER(vp)]
    lib.il_stage_forward.argtypes = [vp, i32, vp, vp]
    lib.il_head_xent.argtypes = [vp, i32, vp, vp, vp]
    lib.il_head_xent_static.argtypes = [vp, i32, vp, vp, vp]
    lib.il_stage_backward_nwise.argtypes = [vp, i32, vp]
    lib.il_free.argtypes = [vp]
    lib.il_routing_plan.argtypes = [i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.il_profile_read.argtypes = [vp, i32, C.POINTER(C.c_char_p), C.POINTER(C.c_int64),
                                    C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double),
                                    C.POINTER(C.c_double)]
    lib.il_test_gemm.argtypes = [i32, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, i32, vp, vp, vp,
                                 i32, C.c_float, i32, i32, vp]
    lib.il_lr_schedule.argtypes = [C.c_int64, i32, i32]
    lib.il_lr_schedule.restype = C.c_double
    lib.il_adam_step.argtypes = [i32, vp, vp, vp, vp, vp, C.c_size_t, C.c_int64, C.c_float, C.c_float, C.c_float,
                                 C.c_float, vp]
    lib.il_embed_forward.argtypes = [i32, vp, vp, vp, i32, i32, i32, i32, vp, vp]
    lib.il_embed_backward.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp]
    lib.il_set_accumulation.argtypes = [vp, i32, C.c_float]
    lib.il_time_per_batch.argtypes = [i32, i32, i32, C.c_double, C.c_double]
    lib.il_time_per_batch.restype = C.c_double
    lib.il_optimal_microbatches.argtypes = [i32, i32, C.c_double, C.c_double, i32]
    lib.il_measure_mfma_peak.argtypes = [vp, i32, vp, C.POINTER(C.c_double)]
    lib.il_measure_copy_peak.argtypes = [vp, vp, C.c_size_t, i32, vp, C.POINTER(C.c_double)]
    lib.il_status_string.argtypes = [C.c_int]
    lib.il_status_string.restype = C.c_char_p
    for name in SYMBOLS:
        if name not in ("il_status_string", "il_lr_schedule", "il_time_per_batch"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def il_status_string(status: int) -> str:
    return load().il_status_string(status).decode()


def il_routing_plan(K: int, n: int, route: str = "window_sum"):
    """(live streams, backward passes) per component, from the library's host planner."""
    live = (C.c_int32 * K)()
    passes = (C.c_int32 * K)()
    rc = load().il_routing_plan(K, n, ROUTES[route] if isinstance(route, str) else route, live, passes)
    if rc:
        raise InterlockError(rc, "il_routing_plan")
    return list(live), list(passes)


def make_config(w: synth.Workload, route: str = "window_sum", head_chunk: int = 0,
                profile: int = 0, ln_eps: float = 1e-5) -> il_config:
    cfg = il_config()
    cfg.K, cfg.blocks_per_component, cfg.d_model, cfg.n_heads = w.K, w.L, w.d, w.H
    cfg.d_mlp, cfg.vocab, cfg.batch, cfg.seq, cfg.n = w.m, w.V, w.B, w.T, w.n
    cfg.dtype = IL_F32 if w.dtype == "f32" else IL_BF16
    cfg.route = ROUTES[route]
    cfg.ln_eps = ln_eps
    cfg.head_chunk = head_chunk
    cfg.profile = int(profile)
    cfg.head_blocks = w.Lh
    return cfg


def il_init(cfg: il_config):
    """Returns an opaque context handle (c_void_p).  With cfg.workspace unset the call is
    a size query: the *_bytes fields are filled and InterlockError(IL_E_WORKSPACE) raised
    unless `query=True` semantics are wanted - use query_sizes() for that."""
    ctx = C.c_void_p()
    rc = load().il_init(C.byref(cfg), C.byref(ctx))
    if rc:
        raise InterlockError(rc, "il_init")
    return ctx


def query_sizes(cfg: il_config):
    ctx = C.c_void_p()
    save = cfg.workspace
    cfg.workspace = None
    rc = load().il_init(C.byref(cfg), C.byref(ctx))
    cfg.workspace = save
    if rc != IL_E_WORKSPACE:
        raise InterlockError(rc if rc else IL_E_ARG, "il_init(size query)")
    return cfg.params_bytes, cfg.grads_bytes, cfg.workspace_bytes


def _check(rc: int, where: str):
    if rc:
        raise InterlockError(rc, where)


def il_stage_forward(ctx, k: int, x_in, x_out):
    _check(load().il_stage_forward(ctx, k, x_in.data_ptr(), x_out.data_ptr()), f"il_stage_forward({k})")


def il_head_xent(ctx, k: int, x_k, targets, loss_out):
    _check(load().il_head_xent(ctx, k, x_k.data_ptr(), targets.data_ptr(), loss_out.data_ptr()),
           f"il_head_xent({k})")


def il_head_xent_static(ctx, k: int, x_k, targets, loss_out):
    _check(load().il_head_xent_static(ctx, k, x_k.data_ptr(), targets.data_ptr(), loss_out.data_ptr()),
           f"il_head_xent_static({k})")


def il_stage_backward_nwise(ctx, k: int, dx0_out=None):
    _check(load().il_stage_backward_nwise(ctx, k, dx0_out.data_ptr() if dx0_out is not None else None),
           f"il_stage_backward_nwise({k})")


def il_free(ctx):
    _check(load().il_free(ctx), "il_free")


def il_test_gemm(dtype, A, B, M, N, K, lda, ldb, a_kmajor, b_kmajor, epi, Cout, C2=None, ldc=None, bias=None,
                 res=None, aux=None, aux_wrap=1, scale=1.0, beta=0, tile=0, stream=None):
    """One GEMM launch of the library's kernels on torch device tensors (test hook)."""
    p = lambda t: t.data_ptr() if t is not None else None
    rc = load().il_test_gemm(dtype, p(A), p(B), M, N, K, lda, ldb, a_kmajor, b_kmajor, epi, p(Cout), p(C2),
                             ldc if ldc is not None else N, p(bias), p(res), p(aux), aux_wrap, scale, beta,
                             tile, stream)
    _check(rc, "il_test_gemm")


def il_profile_read(ctx) -> Dict[str, dict]:
    cap = 32
    names = (C.c_char_p * cap)()
    n = (C.c_int64 * cap)()
    ms = (C.c_double * cap)()
    fl = (C.c_double * cap)()
    by = (C.c_double * cap)()
    kms = (C.c_double * cap)()
    cnt = load().il_profile_read(ctx, cap, names, n, ms, fl, by, kms)
    if cnt < 0:
        raise InterlockError(cnt, "il_profile_read")
    return {names[i].decode(): dict(launches=n[i], ms=ms[i], flops=fl[i], bytes=by[i], kernel_ms=kms[i])
            for i in range(cnt)}


def _ptr(x):
    return None if x is None else (x.data_ptr() if hasattr(x, "data_ptr") else x)


def il_embed_forward(dtype, wte, wpe, tokens, batch: int, seq: int, d_model: int, vocab: int, x0, stream=None):
    dt = {"f32": IL_F32, "bf16": IL_BF16}[dtype] if isinstance(dtype, str) else dtype
    _check(load().il_embed_forward(dt, _ptr(wte), _ptr(wpe), _ptr(tokens), batch, seq, d_model, vocab, _ptr(x0),
                                   stream), "il_embed_forward")


def il_embed_backward(dx0, tokens, batch: int, seq: int, d_model: int, vocab: int, dwte, dwpe, stream=None):
    _check(load().il_embed_backward(_ptr(dx0), _ptr(tokens), batch, seq, d_model, vocab, _ptr(dwte), _ptr(dwpe),
                                    stream), "il_embed_backward")


def il_set_accumulation(ctx, accumulate: bool, grad_scale: float = 1.0):
    _check(load().il_set_accumulation(ctx, int(accumulate), grad_scale), "il_set_accumulation")


def il_time_per_batch(A: int, M: int, N: int, c0: float = 0.025, c1: float = 1.279) -> float:
    return float(load().il_time_per_batch(A, M, N, c0, c1))


def il_optimal_microbatches(A: int, N: int, c0: float = 0.025, c1: float = 1.279, max_m: int = 64) -> int:
    rc = load().il_optimal_microbatches(A, N, c0, c1, max_m)
    if rc < 0:
        raise InterlockError(rc, "il_optimal_microbatches")
    return rc


def il_measure_mfma_peak(scratch, iters: int = 20000, stream=None) -> float:
    """Achieved TFLOP/s of the matrix-unit-only loop (synchronises)."""
    out = C.c_double()
    _check(load().il_measure_mfma_peak(_ptr(scratch), iters, stream, C.byref(out)), "il_measure_mfma_peak")
    return out.value


def il_measure_copy_peak(dst, src, nbytes: int, reps: int = 10, stream=None) -> float:
    """Achieved GB/s (read + written) of the streaming copy kernel (synchronises)."""
    out = C.c_double()
    _check(load().il_measure_copy_peak(_ptr(dst), _ptr(src), nbytes, reps, stream, C.byref(out)),
           "il_measure_copy_peak")
    return out.value


def il_lr_schedule(step: int, d_model: int, warmup_steps: int = 4000) -> float:
    return float(load().il_lr_schedule(step, d_model, warmup_steps))


def il_adam_step(dtype, params, master, grads, m, v, count: int, step: int, lr: float,
                 beta1: float = 0.9, beta2: float = 0.98, eps: float = 1e-9, stream=None):
    """Device tensors (or raw pointers) in, one fused Adam update enqueued on `stream`."""
    def p(x):
        return None if x is None else (x.data_ptr() if hasattr(x, "data_ptr") else x)
    dt = {"f32": IL_F32, "bf16": IL_BF16}[dtype] if isinstance(dtype, str) else dtype
    _check(load().il_adam_step(dt, p(params), p(master), p(grads), p(m), p(v), count, step, lr, beta1, beta2,
                               eps, stream), "il_adam_step")


# --------------------------------------------------------------------------------------
# flat parameter layout (see include/interlock.h) <-> named tensors
# --------------------------------------------------------------------------------------

def param_count(w: synth.Workload) -> int:
    per_block = sum(int(np.prod(s)) for s in synth.block_shapes(w).values())
    return w.K * (w.L + w.Lh) * per_block + w.K * w.d * w.V


def pack_params(w: synth.Workload, params: dict) -> np.ndarray:
    """Named float32 tensors -> one flat float32 array in the library's order."""
    out = np.empty(param_count(w), np.float32)
    o = 0
    for blocks in params["components"]:
        for b in blocks:
            for name in synth.BLOCK_TENSORS:
                a = b[name].ravel()
                out[o:o + a.size] = a
                o += a.size
    hblocks = params.get("head_blocks") or [[] for _ in params["heads"]]
    for h, hb in zip(params["heads"], hblocks):
        assert len(hb) == w.Lh
        for b in hb:                                   # the head's own blocks come before its matrix
            for name in synth.BLOCK_TENSORS:
                a = b[name].ravel()
                out[o:o + a.size] = a
                o += a.size
        out[o:o + h.size] = h.ravel()
        o += h.size
    assert o == out.size
    return out


def unpack_grads(w: synth.Workload, flat: np.ndarray) -> dict:
    shapes = synth.block_shapes(w)
    o = 0
    comps: List[List[Dict[str, np.ndarray]]] = []
    for _ in range(w.K):
        blocks = []
        for _ in range(w.L):
            b = {}
            for name in synth.BLOCK_TENSORS:
                n = int(np.prod(shapes[name]))
                b[name] = flat[o:o + n].reshape(shapes[name])
                o += n
            blocks.append(b)
        comps.append(blocks)
    heads, hblocks = [], []
    for _ in range(w.K):
        blocks = []
        for _ in range(w.Lh):
            b = {}
            for name in synth.BLOCK_TENSORS:
                n = int(np.prod(shapes[name]))
                b[name] = flat[o:o + n].reshape(shapes[name])
                o += n
            blocks.append(b)
        hblocks.append(blocks)
        heads.append(flat[o:o + w.d * w.V].reshape(w.d, w.V))
        o += w.d * w.V
    return {"components": comps, "heads": heads, "head_blocks": hblocks}


class Step:
    """Device buffers + context for one workload; `run()` performs one whole n-wise step
    through the five library calls."""

    def __init__(self, w: synth.Workload, flat_params, route: str = "window_sum",
                 head_chunk: int = 0, profile: int = 0, device: str = "cuda:0", stream=None):
        import torch
        self.torch = torch
        self.w = w
        self.dev = torch.device(device if ":" in device else device + ":0")
        load()
        cfg = make_config(w, route, head_chunk, profile)
        pb, gb, wb = query_sizes(cfg)
        tt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        if isinstance(flat_params, torch.Tensor):      # already on the device in the run's element type: shared
            if flat_params.device != self.dev or flat_params.dtype != tt or not flat_params.is_contiguous():
                raise ValueError("device parameters must be a contiguous tensor of the workload's dtype on " + device)
            self.params = flat_params
        else:
            self.params = torch.from_numpy(flat_params).to(tt).to(self.dev).contiguous()
        assert self.params.numel() * self.params.element_size() == pb
        self.grads = torch.empty(gb // 4, dtype=torch.float32, device=self.dev)
        self.workspace = torch.empty(wb, dtype=torch.uint8, device=self.dev)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.dev)
        cfg.params, cfg.params_bytes = self.params.data_ptr(), pb
        cfg.grads, cfg.grads_bytes = self.grads.data_ptr(), gb
        cfg.workspace, cfg.workspace_bytes = self.workspace.data_ptr(), wb
        cfg.stream = self.stream.cuda_stream
        self.cfg = cfg
        self.ctx = il_init(cfg)
        N, d = w.N, w.d
        self.x = [torch.empty(N, d, dtype=torch.float32, device=self.dev) for _ in range(w.K + 1)]
        self.losses = torch.zeros(w.K, dtype=torch.float32, device=self.dev)
        self.dx0 = torch.empty(N, d, dtype=torch.float32, device=self.dev)
        self.targets = torch.zeros(N, dtype=torch.int32, device=self.dev)

    def set_inputs(self, x0: np.ndarray, targets: np.ndarray):
        t = self.torch
        self.x[0].copy_(t.from_numpy(np.ascontiguousarray(x0, dtype=np.float32)))
        self.targets.copy_(t.from_numpy(np.ascontiguousarray(targets.reshape(-1), dtype=np.int32)))

    def run(self, static_heads: bool = False):
        w = self.w
        head = il_head_xent_static if static_heads else il_head_xent
        for k in range(1, w.K + 1):
            il_stage_forward(self.ctx, k, self.x[k - 1], self.x[k])
            head(self.ctx, k, self.x[k], self.targets, self.losses[k - 1:])
        for k in range(w.K, 0, -1):
            il_stage_backward_nwise(self.ctx, k, self.dx0 if k == 1 else None)

    def results(self) -> dict:
        self.stream.synchronize()
        g = unpack_grads(self.w, self.grads.cpu().numpy())
        return dict(losses=self.losses.cpu().numpy().astype(np.float64), comp_grads=g["components"],
                    head_grads=g["heads"], head_block_grads=g["head_blocks"], dx0=self.dx0.cpu().numpy(),
                    x=[t.cpu().numpy() for t in self.x])

    def close(self):
        if self.ctx is not None:
            self.stream.synchronize()
            il_free(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def run_step(w: synth.Workload, params: dict, x0: np.ndarray, targets: np.ndarray,
             route: str = "window_sum", head_chunk: int = 0) -> dict:
    """One n-wise step on cuda:0 through the C ABI; returns host copies of the results."""
    st = Step(w, pack_params(w, params), route=route, head_chunk=head_chunk)
    st.set_inputs(x0, targets)
    st.run()
    out = st.results()
    st.close()
    return out
