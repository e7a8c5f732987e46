"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, plans routes like the oracle, reports sizes, and turns
misuse into status codes."""
import ctypes as C
import os
import re

import pytest

from oracle import interlock as O
from paper_2010_04116_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    import glob
    hdr = "".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    declared = set(re.findall(r"\b(il_[a-z_]+)\s*\(", hdr))
    assert {"il_init", "il_stage_forward", "il_head_xent", "il_stage_backward_nwise", "il_free"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert set(binding.SYMBOLS) == declared


@pytest.mark.parametrize("route", O.ROUTES)
def test_routing_plan_matches_oracle(route):
    for K in range(1, 9):
        for n in range(1, K + 1):
            live, passes = binding.il_routing_plan(K, n, route)
            plan = O.stream_plan(K, n, route)
            assert passes == [len(plan[k]) for k in range(1, K + 1)], (K, n)
            assert all(1 <= l <= p for l, p in zip(live, passes))
            if route == "window_sum":
                # streams that stop at component 1 (heads 1..n) travel as one
                want = [len([j for j in plan[k] if j > n]) + (1 if k <= n else 0) for k in range(1, K + 1)]
                assert live == want, (K, n)
    with pytest.raises(binding.InterlockError):
        binding.il_routing_plan(4, 5, route)
    with pytest.raises(binding.InterlockError):
        binding.il_routing_plan(4, 0, route)


def test_size_query_and_param_count():
    for name, w in synth.WORKLOADS.items():
        cfg = binding.make_config(w)
        pb, gb, wb = binding.query_sizes(cfg)
        eb = 4 if w.dtype == "f32" else 2
        assert pb == binding.param_count(w) * eb
        assert gb == binding.param_count(w) * 4
        assert wb > 0 and wb % 256 == 0
    assert binding.param_count(synth.WORKLOADS["medium"]) == 24 * (12 * 1024 ** 2 + 13 * 1024) + 4 * 1024 * 32768
    # the paper-shaped workload: 4 heads of two blocks each on top of the 24 trunk blocks
    assert binding.param_count(synth.WORKLOADS["paper"]) == 32 * (12 * 1024 ** 2 + 13 * 1024) + 4 * 1024 * 32768
    # a fp32 head width of 256 has no kernel
    cfg = binding.make_config(synth.WORKLOADS["paper"].with_(dtype="f32"))
    ctx = C.c_void_p()
    assert binding.load().il_init(C.byref(cfg), C.byref(ctx)) == binding.IL_E_SHAPE


def test_misuse_returns_status_codes():
    lib = binding.load()
    w = synth.WORKLOADS["tiny"]
    ctx = C.c_void_p()
    assert lib.il_init(None, C.byref(ctx)) == binding.IL_E_ARG
    for field, val, want in [("n", 0, binding.IL_E_ARG), ("n", 5, binding.IL_E_ARG),
                             ("dtype", 7, binding.IL_E_ARG), ("route", 9, binding.IL_E_ARG),
                             ("n_heads", 3, binding.IL_E_SHAPE), ("d_model", 4096, binding.IL_E_SHAPE),
                             ("K", 0, binding.IL_E_ARG), ("head_blocks", -1, binding.IL_E_ARG),
                             ("reserved", 1, binding.IL_E_ARG)]:
        cfg = binding.make_config(w)
        setattr(cfg, field, val)
        assert lib.il_init(C.byref(cfg), C.byref(ctx)) == want, field
    cfg = binding.make_config(w.with_(dtype="bf16", B=1, T=33))
    assert lib.il_init(C.byref(cfg), C.byref(ctx)) == binding.IL_E_SHAPE
    # buffers too small
    cfg = binding.make_config(w)
    pb, gb, wb = binding.query_sizes(cfg)
    cfg.params, cfg.grads, cfg.workspace = 4096, 4096, 4096
    cfg.params_bytes, cfg.grads_bytes, cfg.workspace_bytes = pb, gb, wb - 1
    assert lib.il_init(C.byref(cfg), C.byref(ctx)) == binding.IL_E_WORKSPACE
    # a context over fake pointers: call-order errors are caught before any launch
    cfg.workspace_bytes = wb
    assert lib.il_init(C.byref(cfg), C.byref(ctx)) == binding.IL_OK
    fake = C.c_void_p(4096)
    fake2 = C.c_void_p(8192)
    assert lib.il_stage_forward(ctx, 2, fake, fake2) == binding.IL_E_STATE
    assert lib.il_stage_forward(ctx, 0, fake, fake2) == binding.IL_E_ARG
    assert lib.il_stage_forward(ctx, 1, fake, fake) == binding.IL_E_ARG
    assert lib.il_stage_forward(ctx, 1, None, fake2) == binding.IL_E_ARG
    assert lib.il_head_xent(ctx, 1, fake, fake, fake) == binding.IL_E_STATE
    assert lib.il_stage_backward_nwise(ctx, 4, None) == binding.IL_E_STATE
    assert lib.il_stage_backward_nwise(ctx, 9, None) == binding.IL_E_ARG
    assert lib.il_free(ctx) == binding.IL_OK
    assert lib.il_free(None) == binding.IL_E_ARG
    assert "IL_E_STATE" in binding.il_status_string(binding.IL_E_STATE)


def test_operands_beyond_the_descriptor_range_are_rejected_up_front():
    """Every GEMM operand is addressed through a 32-bit buffer descriptor: il_init refuses a problem whose
    largest stacked operand, head matrix or logits tile reaches 2 GiB instead of failing in mid-step."""
    lib = binding.load()
    ctx = C.c_void_p()
    ok = synth.Workload("fits", "bf16", K=2, L=1, d=1024, H=16, m=4096, V=32768, B=64, T=2048, n=2)
    for w, want in [(ok.with_(B=128), binding.IL_E_SHAPE),                         # 262144 x 4096 x 2 B = 2 GiB
                    (ok, binding.IL_E_WORKSPACE),                                  # half of it: a size query succeeds
                    (ok.with_(B=1, T=64, V=1 << 21, d=512, H=8), binding.IL_E_SHAPE),    # head matrix d x V x 2 B = 2 GiB
                    (ok.with_(B=16, V=1 << 19, n=1), binding.IL_E_WORKSPACE)]:           # the default chunk shrinks to fit
        cfg = binding.make_config(w)
        assert lib.il_init(C.byref(cfg), C.byref(ctx)) == want, w
    cfg = binding.make_config(ok.with_(B=16, V=1 << 19, n=1), head_chunk=2048)          # logits tile 2048 x 2^19 x 2 B
    assert lib.il_init(C.byref(cfg), C.byref(ctx)) == binding.IL_E_SHAPE
    cfg = binding.make_config(ok.with_(B=16, V=1 << 19, n=1), head_chunk=512)           # a smaller tile fits
    assert lib.il_init(C.byref(cfg), C.byref(ctx)) == binding.IL_E_WORKSPACE
    cfg = binding.make_config(ok.with_(B=8192, T=64, H=8, n=1))                         # attention grid: batch x heads = 65536
    assert lib.il_init(C.byref(cfg), C.byref(ctx)) == binding.IL_E_SHAPE
    cfg = binding.make_config(synth.WORKLOADS["tiny"])
    cfg.profile = 3
    assert lib.il_init(C.byref(cfg), C.byref(ctx)) == binding.IL_E_ARG


def test_pack_unpack_roundtrip():
    import numpy as np
    w = synth.WORKLOADS["tiny"]
    p = synth.make_params(w, random_bias=True)
    flat = binding.pack_params(w, p)
    back = binding.unpack_grads(w, flat)
    for k in range(w.K):
        for name in synth.BLOCK_TENSORS:
            assert np.array_equal(back["components"][k][0][name], p["components"][k][0][name])
        assert np.array_equal(back["heads"][k], p["heads"][k])


def test_lr_schedule_and_adam_misuse_without_a_gpu():
    """il_lr_schedule is a host function; il_adam_step rejects bad arguments before any launch."""
    import math
    from oracle import adam as A
    for step in (1, 7, 3999, 4000, 4001, 123456):
        assert binding.il_lr_schedule(step, 1024, 4000) == pytest.approx(A.lr_schedule(step, 1024, 4000), rel=1e-14)
    assert binding.il_lr_schedule(4000, 1024, 4000) == pytest.approx(1.0 / (32.0 * math.sqrt(4000.0)), rel=1e-14)
    assert binding.il_lr_schedule(0, 1024, 4000) == 0.0
    lib = binding.load()
    fake = C.c_void_p(4096)
    ok = (binding.IL_F32, fake, None, fake, fake, fake, 64, 1, 0.1, 0.9, 0.98, 1e-9, None)
    def call(**kw):
        names = ("dtype", "params", "master", "grads", "m", "v", "count", "step", "lr", "beta1", "beta2", "eps", "stream")
        a = dict(zip(names, ok)); a.update(kw)
        return lib.il_adam_step(*[a[n] for n in names])
    assert call(count=0) == binding.IL_OK                       # nothing to do, nothing launched
    assert call(dtype=7) == binding.IL_E_ARG
    assert call(params=None) == binding.IL_E_ARG
    assert call(step=0) == binding.IL_E_ARG
    assert call(beta2=1.0) == binding.IL_E_ARG
    assert call(lr=-0.1) == binding.IL_E_ARG
    assert call(master=fake) == binding.IL_E_ARG                # fp32 mode takes no master copy
    assert call(dtype=binding.IL_BF16) == binding.IL_E_ARG      # bf16 mode needs one
    assert call(grads=C.c_void_p(4100)) == binding.IL_E_SHAPE   # misaligned


def test_timing_model_host_functions_match_the_oracle():
    from oracle import timing as Tm
    for A in range(1, 33):
        for N in (1, 2, 3, 5, 8, 40):
            for M in (1, 2, 3, 4, 8, 16, 64):
                assert binding.il_time_per_batch(A, M, N) == pytest.approx(Tm.time_per_batch(A, M, N), rel=1e-14)
            assert binding.il_optimal_microbatches(A, N) == Tm.optimal_microbatches(A, N)
    assert binding.il_time_per_batch(4, 8, 2, 0.1, 2.0) == pytest.approx(Tm.time_per_batch(4, 8, 2, 0.1, 2.0))
    import math
    assert math.isnan(binding.il_time_per_batch(0, 1, 1))
    with pytest.raises(binding.InterlockError):
        binding.il_optimal_microbatches(4, 0)
    lib = binding.load()
    assert lib.il_set_accumulation(None, 1, 0.5) == binding.IL_E_ARG
