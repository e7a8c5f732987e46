"""GPU parity of the whole n-wise step against the float64 oracle, through the C ABI."""
import sys

import numpy as np
import pytest

from oracle import interlock as O
from paper_2010_04116_amd import binding, synth
from parity import compare, make_inputs, run_both, summary, check_tensor, record, assert_clean, TOL

pytestmark = pytest.mark.gpu
TINY = synth.WORKLOADS["tiny"]


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_tiny_fp32_window_sum(n):
    w = TINY.with_(n=n)
    say("case tiny fp32 n =", n)
    got, ref = run_both(w)
    say("worst", summary(compare(w, got, ref, f"tiny n={n}")))


@pytest.mark.parametrize("route", ["far_head", "mean_local_far"])
@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_tiny_fp32_paper_routes(n, route):
    w = TINY.with_(n=n)
    say("case tiny fp32 route", route, "n =", n)
    got, ref = run_both(w, route=route)
    say("worst", summary(compare(w, got, ref, f"tiny {route} n={n}")))


def test_fp32_two_blocks_many_components():
    w = TINY.with_(K=6, L=2, n=3, B=3, T=16)
    say("case fp32 K=6 L=2 n=3")
    got, ref = run_both(w, seed=1)
    say("worst", summary(compare(w, got, ref, "K6L2")))
    got, ref = run_both(w, seed=1, route="mean_local_far")
    say("worst", summary(compare(w, got, ref, "K6L2 mean")))


def test_fp32_ragged_shapes():
    """Sizes that are not multiples of any tile: d=48 (3 heads of 16), m=100, V=77, N=39."""
    w = synth.Workload("ragged", "f32", K=3, L=1, d=48, H=3, m=100, V=77, B=3, T=13, n=2)
    say("case ragged fp32")
    got, ref = run_both(w, seed=2, head_chunk=16)     # 39 rows -> chunks 16,16,7
    say("worst", summary(compare(w, got, ref, "ragged")))


def test_fp32_single_component_and_single_token():
    w = synth.Workload("k1", "f32", K=1, L=1, d=32, H=2, m=64, V=16, B=2, T=1, n=1)
    say("case K=1 T=1")
    got, ref = run_both(w, seed=3)
    say("worst", summary(compare(w, got, ref, "K1T1")))


def test_fp32_model_width_256():
    """d = 256 takes the 16-byte LayerNorm paths in fp32 as well."""
    w = synth.Workload("w256", "f32", K=2, L=1, d=256, H=4, m=512, V=96, B=2, T=24, n=2)
    say("case fp32 d=256")
    got, ref = run_both(w, seed=6)
    say("worst", summary(compare(w, got, ref, "w256")))


@pytest.mark.parametrize("route", ["window_sum", "mean_local_far", "far_head"])
@pytest.mark.parametrize("Lh", [1, 2])
def test_fp32_heads_with_blocks(Lh, route):
    """Auxiliary heads of Lh Transformer blocks + output matrix (the paper's Transformer heads, App. B)."""
    w = TINY.with_(Lh=Lh, n=2, K=3)
    say("case fp32 block heads Lh =", Lh, route)
    got, ref = run_both(w, seed=9, route=route)
    say("worst", summary(compare(w, got, ref, f"Lh={Lh} {route}")))


def test_bf16_heads_with_blocks():
    w = synth.Workload("small_qh", "bf16", K=3, L=1, d=256, H=4, m=1024, V=2048, B=2, T=128, n=2, Lh=2)
    say("case bf16 block heads")
    got, ref = run_both(w, seed=10)
    say("worst", summary(compare(w, got, ref, "small_qh")))
    got2, _ = run_both(w, seed=10)                           # heads on the side stream: reproducible
    assert np.array_equal(got["losses"], got2["losses"]) and np.array_equal(got["dx0"], got2["dx0"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_micro_batches_accumulate_to_the_full_batch_gradient(dtype):
    """Two micro-batches of half the sequences each, the second accumulating, both scaled by 1/2:
    the gradients of the whole mini-batch (the loss is a mean over positions, sequences are
    independent), against the oracle on the full batch."""
    if dtype == "f32":
        w = TINY.with_(B=4, n=2, Lh=1)
    else:
        w = synth.Workload("mb", "bf16", K=3, L=1, d=256, H=4, m=512, V=1024, B=4, T=64, n=2)
    say("case micro-batching", dtype)
    params, x0, tgt = make_inputs(w, seed=11)
    ref = O.nwise_streams(params, x0, tgt, w.B, w.T, w.H, w.n)
    half = w.with_(B=w.B // 2)
    st = binding.Step(half, binding.pack_params(w, params))
    losses = []
    for mb in range(2):
        rows = slice(mb * half.N, (mb + 1) * half.N)
        st.set_inputs(x0[rows], tgt[mb * half.B:(mb + 1) * half.B])
        binding.il_set_accumulation(st.ctx, mb > 0, 0.5)
        st.run()
        losses.append(st.results()["losses"])
    got = st.results()
    st.close()
    got["losses"] = 0.5 * (losses[0] + losses[1])
    got["dx0"] = ref["dx0"] * 0                      # belongs to each micro-batch; not compared here
    ref = dict(ref, dx0=ref["dx0"] * 0)
    say("worst", summary(compare(w, got, ref, "micro-batches")))


def test_head_chunking_does_not_change_results():
    w = TINY
    params, x0, tgt = make_inputs(w)
    a = binding.run_step(w, params, x0, tgt, head_chunk=64)
    b = binding.run_step(w, params, x0, tgt, head_chunk=16)
    np.testing.assert_allclose(a["losses"], b["losses"], rtol=1e-6)
    for k in range(w.K):
        np.testing.assert_allclose(a["head_grads"][k], b["head_grads"][k], rtol=1e-4, atol=1e-8)


def test_step_is_bit_reproducible_and_restartable():
    w = TINY
    params, x0, tgt = make_inputs(w)
    st = binding.Step(w, binding.pack_params(w, params))
    st.set_inputs(x0, tgt)
    st.run()
    a = st.results()
    st.run()                      # a second step on the same context: nothing accumulates
    b = st.results()
    st.close()
    assert np.array_equal(a["losses"], b["losses"])
    for k in range(w.K):
        for name in synth.BLOCK_TENSORS:
            assert np.array_equal(a["comp_grads"][k][0][name], b["comp_grads"][k][0][name]), name
        assert np.array_equal(a["head_grads"][k], b["head_grads"][k])


def test_call_order_errors_on_device():
    w = TINY
    params, x0, tgt = make_inputs(w)
    st = binding.Step(w, binding.pack_params(w, params))
    st.set_inputs(x0, tgt)
    with pytest.raises(binding.InterlockError) as e:
        binding.il_stage_backward_nwise(st.ctx, w.K)
    assert e.value.status == binding.IL_E_STATE
    for k in range(1, w.K + 1):
        binding.il_stage_forward(st.ctx, k, st.x[k - 1], st.x[k])
    with pytest.raises(binding.InterlockError) as e:   # head K not evaluated yet
        binding.il_stage_backward_nwise(st.ctx, w.K)
    assert e.value.status == binding.IL_E_STATE
    st.close()


def test_heads_with_blocks_in_descending_order():
    """Heads with their own blocks differentiate them in the backward scratch, on the library's
    second stream; enqueued in descending order (head K first) the backward of component K must
    still wait for all of them."""
    w = TINY.with_(Lh=2, n=2, K=3)
    params, x0, tgt = make_inputs(w, seed=9)
    ref = O.nwise_streams(params, x0, tgt, w.B, w.T, w.H, w.n)
    st = binding.Step(w, binding.pack_params(w, params))
    st.set_inputs(x0, tgt)
    for k in range(1, w.K + 1):
        binding.il_stage_forward(st.ctx, k, st.x[k - 1], st.x[k])
    for k in range(w.K, 0, -1):
        binding.il_head_xent(st.ctx, k, st.x[k], st.targets, st.losses[k - 1:])
    for k in range(w.K, 0, -1):
        binding.il_stage_backward_nwise(st.ctx, k, st.dx0 if k == 1 else None)
    with pytest.raises(binding.InterlockError) as e:     # a head of this step after its backward began
        binding.il_head_xent(st.ctx, 1, st.x[1], st.targets, st.losses)
    assert e.value.status == binding.IL_E_STATE
    got = st.results()
    st.close()
    say("worst", summary(compare(w, got, ref, "descending heads Lh=2")))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_targets_out_of_range_are_ignored_positions(dtype):
    """A target outside [0, V) adds nothing to the loss or to any gradient and nothing is read out of
    bounds.  With the whole second sequence ignored, the batch of two equals half of the oracle's
    result on the first sequence alone (sequences are independent, the mean still divides by N)."""
    if dtype == "f32":
        w = TINY.with_(B=2, n=2)
    else:
        w = synth.Workload("ign", "bf16", K=2, L=1, d=256, H=4, m=512, V=1024, B=2, T=64, n=2)
    params, x0, tgt = make_inputs(w, seed=12)
    bad = tgt.copy()
    bad[1, :] = [-1, w.V, -100, 2 ** 31 - 1] * (w.T // 4)
    got = binding.run_step(w, params, x0, bad)
    ref = O.nwise_streams(params, x0[:w.T], tgt[:1], 1, w.T, w.H, w.n)
    assert np.all(got["dx0"][w.T:] == 0)
    got["dx0"] = got["dx0"][:w.T]
    got["losses"] = got["losses"] * 2
    say("worst", summary(compare(w.with_(B=1), got, ref, f"ignored targets {dtype}", scale=2.0)))
    none = binding.run_step(w, params, x0, np.full_like(tgt, -1))
    assert np.all(none["losses"] == 0) and np.all(none["dx0"] == 0)
    assert all(np.all(h == 0) for h in none["head_grads"])


# ---------------------------------------------------------------- bf16 -------------

def test_bf16_reduced_small():
    """Small's structure (K=4 x 2 blocks, head width 64) at a quarter of its width."""
    w = synth.Workload("small_q", "bf16", K=4, L=2, d=256, H=4, m=1024, V=2048, B=2, T=128, n=2)
    say("case bf16 reduced small")
    got, ref = run_both(w, seed=4)
    say("worst", summary(compare(w, got, ref, "small_q")))


@pytest.mark.parametrize("head_chunk", [64, 192])          # 256 token rows: 4 equal chunks; 192 + a ragged 64
def test_bf16_head_in_several_chunks(head_chunk):
    """The head of the bf16 path over several token chunks: statistics, in-place dlogits and dx per chunk,
    the head matrix's gradient accumulated over the chunks, equal and ragged (the default, half the rows, gives two)."""
    w = _small_q()
    say("case bf16 head_chunk =", head_chunk)
    got, ref = run_both(w, seed=4, head_chunk=head_chunk)
    say("worst", summary(compare(w, got, ref, f"small_q head_chunk={head_chunk}")))


@pytest.mark.parametrize("T,H", [(96, 4), (160, 2), (32, 4), (224, 2), (128, 1), (96, 1)])
def test_bf16_sequence_lengths_off_the_attention_tiles(T, H):
    """Sequence lengths that are not multiples of the 64- / 128-row attention tiles, for both MFMA
    head widths (d = 256: H = 4 -> 64, H = 2 -> 128, H = 1 -> 256, the paper's); N = B*T stays a multiple of 64."""
    w = synth.Workload("seq", "bf16", K=2, L=1, d=256, H=H, m=512, V=512, B=2, T=T, n=2)
    say("case bf16 T =", T, "head width", 256 // H)
    got, ref = run_both(w, seed=7)
    say("worst", summary(compare(w, got, ref, f"T={T} H={H}")))


def test_bf16_attention_grid_with_a_partial_round_of_balanced_tiles():
    """5 causal tiles x 128 (batch, head) pairs: every XCD's list of 80 attention workgroups has one full
    round of 64 (longest first, shortest behind them in opposite order) and a remainder of 16 in plain
    descending order - both branches of the tile assignment, with an odd number of tile lengths."""
    w = synth.Workload("bal", "bf16", K=1, L=1, d=256, H=4, m=256, V=256, B=32, T=640, n=1)
    say("case bf16 balanced attention tiles, grid 5 x 128")
    got, ref = run_both(w, seed=9)
    say("worst", summary(compare(w, got, ref, "attention grid 5x128")))


@pytest.mark.parametrize("route,n", [("mean_local_far", 3), ("far_head", 2)])
def test_bf16_paper_routes(route, n):
    """The paper's two routings in bf16 (stacked streams, several runs per component, scaled sums)."""
    w = synth.Workload("routes", "bf16", K=4, L=1, d=256, H=4, m=512, V=1024, B=2, T=64, n=n)
    say("case bf16 route", route, "n =", n)
    got, ref = run_both(w, seed=8, route=route)
    say("worst", summary(compare(w, got, ref, f"{route} n={n}")))


@pytest.mark.parametrize("n", [1, 2, 4])      # local, the benchmark's window, n = K (global backprop)
def test_small_bf16_full_step(n):
    w = synth.WORKLOADS["small"].with_(n=n)
    say("case small bf16 n =", n)
    got, ref = run_both(w, seed=5, random_ln=False)
    say("worst", summary(compare(w, got, ref, f"small n={n}")))
    assert np.all(np.abs(ref["losses"] - np.log(w.V)) < 0.5)     # uniform tokens: loss near ln V


def _small_q():
    return synth.Workload("small_q", "bf16", K=4, L=2, d=256, H=4, m=1024, V=2048, B=2, T=128, n=2)


def test_losses_final_after_last_head_without_backward():
    """Evaluation-style use: forwards and heads only.  The heads run on the library's internal
    stream; the last head joins it, so synchronising the caller's stream is enough."""
    w = _small_q()
    params, x0, tgt = make_inputs(w, seed=4)
    full = binding.run_step(w, params, x0, tgt)
    st = binding.Step(w, binding.pack_params(w, params))
    st.set_inputs(x0, tgt)
    for k in range(1, w.K + 1):
        binding.il_stage_forward(st.ctx, k, st.x[k - 1], st.x[k])
        binding.il_head_xent(st.ctx, k, st.x[k], st.targets, st.losses[k - 1:])
    st.stream.synchronize()
    losses = st.losses.cpu().numpy().astype(np.float64)
    head_grads = binding.unpack_grads(w, st.grads.cpu().numpy())["heads"]
    st.close()
    assert np.array_equal(losses, full["losses"])
    for k in range(w.K):
        assert np.array_equal(head_grads[k], full["head_grads"][k])


def test_abandoned_step_does_not_disturb_the_next():
    """A step that stops after two heads (their work still queued on the internal stream) is
    followed at once by a complete step with other inputs on the same context."""
    w = _small_q()
    params, x0, tgt = make_inputs(w, seed=4)
    _, x0b, tgtb = make_inputs(w, seed=9)
    st = binding.Step(w, binding.pack_params(w, params))
    st.set_inputs(x0b, tgtb)
    for k in range(1, 3):
        binding.il_stage_forward(st.ctx, k, st.x[k - 1], st.x[k])
        binding.il_head_xent(st.ctx, k, st.x[k], st.targets, st.losses[k - 1:])
    st.stream.synchronize()          # the caller's stream only; the heads may still be running
    st.set_inputs(x0, tgt)
    st.run()
    got = st.results()
    st.close()
    ref = binding.run_step(w, params, x0, tgt)
    assert np.array_equal(got["losses"], ref["losses"])
    assert np.array_equal(got["dx0"], ref["dx0"])
    for k in range(w.K):
        assert np.array_equal(got["head_grads"][k], ref["head_grads"][k])


def test_profiling_mode_same_results_and_sane_times():
    w = _small_q()
    params, x0, tgt = make_inputs(w, seed=4)
    ref = binding.run_step(w, params, x0, tgt)
    st = binding.Step(w, binding.pack_params(w, params), profile=True)
    st.set_inputs(x0, tgt)
    st.run()
    got = st.results()
    prof = binding.il_profile_read(st.ctx)
    st.run()
    prof2 = binding.il_profile_read(st.ctx)
    st.close()
    assert np.array_equal(got["losses"], ref["losses"])
    assert np.array_equal(got["dx0"], ref["dx0"])
    gemm = [k for k in prof if k.startswith("gemm")]
    assert sorted(gemm) == ["gemm_dgrad", "gemm_fwd", "gemm_head", "gemm_wgrad"]
    for k in gemm:
        v = prof[k]
        assert v["launches"] > 0 and v["flops"] > 0 and v["bytes"] > 0
        assert 0 < v["kernel_ms"] <= v["ms"], (k, v)           # the kernel alone is inside its bracket
        assert prof2[k]["launches"] == v["launches"]           # counters restart with each read
    fwd_flops = 2.0 * w.N * (4 * w.d * w.d + 2 * w.d * w.m) * w.K * w.L
    assert abs(prof["gemm_fwd"]["flops"] - fwd_flops) < 1e-6 * fwd_flops
    for k in prof:
        if not k.startswith("gemm"):
            assert prof[k]["kernel_ms"] == 0.0


@pytest.mark.parametrize("n", [2, 1, 3])
def test_bf16_two_stream_mode_is_bitwise_the_single_stream_mode(n):
    """The default mode runs heads, stream sums, column sums and weight gradients on a second stream
    over double-buffered operands; profiling mode 1 runs everything in line on one stream, mode 2 is the
    default mode with timers attached to the GEMM dispatches.  Three
    blocks per component, two live streams, all heads live: EVERY loss, component, head and input
    gradient must come out bit for bit the same in both modes and in a repeated step."""
    # (n = 1 and n = K: every block carries a single stream of weight 1, whose wide data gradients are
    # produced straight into the double-buffered weight-gradient operands)
    w = synth.Workload("bits", "bf16", K=3, L=3, d=256, H=4, m=1024, V=2048, B=2, T=128, n=n)
    params, x0, tgt = make_inputs(w, seed=17)
    flat = binding.pack_params(w, params)
    runs = []
    for profile in (0, 0, 1, 2):
        st = binding.Step(w, flat, profile=profile)
        st.set_inputs(x0, tgt)
        st.run()
        if profile == 0:
            st.run()                              # and a second step on the same context
        runs.append(st.results())
        if profile == 2:                          # two streams, timers on the GEMM dispatches only
            prof = binding.il_profile_read(st.ctx)
            for k, v in prof.items():
                assert v["ms"] == 0.0
                assert (v["kernel_ms"] > 0 and v["launches"] > 0) == k.startswith("gemm"), (k, v)
        st.close()
    a = runs[0]
    for which, b in (("repeat", runs[1]), ("single-stream", runs[2]), ("timed two-stream", runs[3])):
        assert np.array_equal(a["losses"], b["losses"]), which
        assert np.array_equal(a["dx0"], b["dx0"]), which
        for k in range(w.K):
            assert np.array_equal(a["head_grads"][k], b["head_grads"][k]), (which, k)
            for l in range(w.L):
                for name in synth.BLOCK_TENSORS:
                    assert np.array_equal(a["comp_grads"][k][l][name], b["comp_grads"][k][l][name]), (which, k, l, name)


# ------------------------------------------------ real-shape slices (bf16) ---------

def test_medium_shape_one_component_and_head():
    """One block + head at Medium's real shape (N=4096, d=1024, m=4096, V=32768): the
    GEMM tile configurations and head chunking the benchmark uses."""
    w = synth.WORKLOADS["medium"].with_(K=1, L=1, n=1)
    say("case medium slice K=1 L=1")
    got, ref = run_both(w, seed=6, random_ln=False)
    say("worst", summary(compare(w, got, ref, "medium slice")))


def test_medium_shape_stacked_streams():
    """Two live gradient streams through real-shape blocks (K=3, n=2; smaller vocab)."""
    w = synth.WORKLOADS["medium"].with_(K=3, L=1, n=2, V=8192)
    say("case medium stacked K=3 n=2")
    got, ref = run_both(w, seed=7, random_ln=False)
    say("worst", summary(compare(w, got, ref, "medium stacked")))


def test_large_shape_one_component_and_head():
    """One block + head at Large's real shape (d=2048, head width 128, V=50304 = 393*128)."""
    w = synth.WORKLOADS["large"].with_(K=1, L=1, n=1)
    say("case large slice K=1 L=1")
    got, ref = run_both(w, seed=8, random_ln=False)
    say("worst", summary(compare(w, got, ref, "large slice")))


# ------------------------------------------------ real-shape slices with stacked streams ----

def test_many_head_shape_three_stacked_streams():
    """Three live gradient streams (M = 3 x 4096 rows in every backward GEMM, grid.z = 3 in attention
    backward) through blocks of Many-head's real shape: K=5, n=3 -> components 3..5 carry 3, 3, 2 streams
    (smaller vocabulary so that the float64 oracle stays cheap).  Every gradient tensor, every loss."""
    w = synth.WORKLOADS["many_head"].with_(K=5, L=1, n=3, V=8192)
    live, _ = binding.il_routing_plan(w.K, w.n)
    assert max(live) == 3
    say("case many_head stacked K=5 n=3, live", live)
    got, ref = run_both(w, seed=15, random_ln=False)
    say("worst", summary(compare(w, got, ref, "many_head slice K5 n3")))


@pytest.mark.parametrize("n", [2, 3])
def test_large_shape_stacked_and_merged_streams(n):
    """Large's real block shape (d=2048, head width 128, m=8192, N=4096): n=2 stacks two streams
    (M = 8192 rows), n = K = 3 merges all heads into the one stream of global backprop."""
    w = synth.WORKLOADS["large"].with_(K=3, L=1, n=n, V=8192)
    say("case large slice K=3 n =", n)
    got, ref = run_both(w, seed=16, random_ln=False)
    say("worst", summary(compare(w, got, ref, f"large slice K3 n{n}")))


# ------------------------------------------------ full-size workloads -------------------------

def _full_size(name, seed, n=None):
    """The workload exactly as bench.py runs it (all components, heads, routing, tile and chunk
    choices), against ONE oracle run on sequence 0 at full depth and width.

    (1) Distinct sequences (the benchmark's batch): sequences are independent, so the oracle fixes every
        x_k row of sequence 0 and - the batch mean over B*T positions - dL/dx_0 of sequence 0 times B.
    (2) Sequence 0 replicated B times: every row block of every GEMM then carries real data, the mean loss
        of the batch equals the single-sequence loss and EVERY parameter and head gradient of the
        full-size step equals the oracle's single-sequence gradient.  All of them are compared, to the
        same element-level bounds as the small cases."""
    w = synth.WORKLOADS[name]
    if n:
        w = w.with_(n=n)
    label = f"{name}_n{w.n} full size"
    params = synth.make_params(w, synth.PARAM_SEED + seed)
    inp, tgt = synth.make_tokens(w, synth.TOKEN_SEED + seed)
    x0 = synth.make_x0(w, inp, synth.PARAM_SEED + seed)
    flat = binding.pack_params(w, params)
    st = binding.Step(w, flat)
    say("case", label, ": GPU step, distinct sequences")
    st.set_inputs(x0, tgt)
    st.run()
    got = st.results()
    say("GPU step, sequence 0 replicated")
    st.set_inputs(np.tile(x0[:w.T], (w.B, 1)), np.tile(tgt[:1], (w.B, 1)))
    st.run()
    rep = st.results()
    st.close()
    del st, flat
    say("oracle on sequence 0")
    w1 = w.with_(B=1)
    ref = O.nwise_streams(params, x0[:w.T].astype(np.float64), tgt[:1], 1, w.T, w.H, w.n)
    # (1)
    worst = {}
    tol = TOL[w.dtype]["grad"]
    for k in range(w.K):
        check_tensor(got["x"][k + 1][:w.T], ref["x"][k], tol / 2, f"{label}: x_{k + 1} of sequence 0", worst, "x_k")
    check_tensor(got["dx0"][:w.T] * w.B, ref["dx0"], tol, f"{label}: dL/dx_0 of sequence 0", worst, "dx0")
    assert np.all(np.isfinite(got["losses"])) and np.all(got["losses"] > np.log(w.V) - 0.5)
    for k in range(w.K):
        np.testing.assert_allclose(got["head_grads"][k].sum(axis=1), 0, atol=2e-3)   # sum_v dlogits = 0
    bad = worst.pop("violations", [])
    record(label + " (distinct, sequence 0)", w, worst)
    say("distinct:", summary(worst))
    assert_clean({"violations": bad}, label + " (distinct)")
    # (2)
    for t in range(1, w.B):              # the replicas come out alike (same tiles, other row blocks)
        assert np.array_equal(rep["x"][w.K][t * w.T:(t + 1) * w.T], rep["x"][w.K][:w.T]), f"{label}: replica {t}"
    rep["dx0"] = rep["dx0"][:w.T] * w.B
    say("replicated:", summary(compare(w1, rep, ref, label + " (replicated)")))


def test_medium_full_size():
    _full_size("medium", 11)


def test_many_head_full_size():
    _full_size("many_head", 12)


def test_large_full_size():
    _full_size("large", 13)


def test_large_full_size_global_equivalent():
    """Large with n = K = 6: every head's stream merges into the one global backward."""
    _full_size("large", 13, n=6)


def test_paper_shape_full_size():
    """The paper's module shape (head width 256, sequences of 128, 6 blocks per module, 2-block heads)."""
    _full_size("paper", 14)
