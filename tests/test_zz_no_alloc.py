"""il_head_xent_static - the head with its scratch in the library's static device array, for
callers that cannot allocate - against il_head_xent, through the C ABI: two calls in a row on one
GPU, the second with a smaller input (the array keeps the first call's contents)."""
import ctypes as C

import numpy as np
import pytest

from paper_2010_04116_amd import binding, synth
from parity import make_inputs

pytestmark = pytest.mark.gpu


def _both(w, seed):
    """One whole step with il_head_xent and one with il_head_xent_static on separate contexts."""
    params, x0, tgt = make_inputs(w, seed=seed)
    flat = binding.pack_params(w, params)
    out = []
    for static in (False, True):
        st = binding.Step(w, flat)
        st.set_inputs(x0, tgt)
        st.run(static_heads=static)
        out.append(st.results())
        st.close()
    return out


def _same(w, a, b, what):
    # same kernels on the same operands in the same order: bit for bit
    assert np.array_equal(a["losses"], b["losses"]), what
    assert np.array_equal(a["dx0"], b["dx0"]), what
    for k in range(w.K):
        assert np.array_equal(a["head_grads"][k], b["head_grads"][k]), (what, "head", k + 1)
        for l in range(w.L):
            for name in synth.BLOCK_TENSORS:
                assert np.array_equal(a["comp_grads"][k][l][name], b["comp_grads"][k][l][name]), (what, k, l, name)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_head_equals_the_workspace_head_twice_in_a_row(dtype):
    if dtype == "bf16":
        big = synth.Workload("na_big", "bf16", K=3, L=1, d=256, H=4, m=512, V=4096, B=4, T=128, n=2)
        small = synth.Workload("na_small", "bf16", K=2, L=1, d=128, H=2, m=256, V=1000, B=1, T=64, n=1)
    else:
        big = synth.WORKLOADS["tiny"].with_(K=3, V=320, B=3)
        small = synth.WORKLOADS["tiny"].with_(K=2, V=96, B=1, T=16, n=1)
    for w, seed in ((big, 21), (small, 22)):           # the second call finds the first one's leftovers
        a, b = _both(w, seed)
        assert np.all(np.isfinite(a["losses"])) and np.all(a["losses"] > 0)
        _same(w, a, b, f"{dtype} {w.name}")


def test_static_scratch_head_rejects_what_does_not_fit():
    import torch
    # the logits tile alone (2048 x 32768 bf16 = 128 MiB) exceeds the 64 MiB array
    w = synth.Workload("na_huge", "bf16", K=1, L=1, d=256, H=4, m=256, V=32768, B=8, T=512, n=1)
    st = binding.Step(w, np.zeros(binding.param_count(w), np.float32))
    st.set_inputs(np.zeros((w.N, w.d), np.float32), np.zeros((w.B, w.T), np.int32))
    binding.il_stage_forward(st.ctx, 1, st.x[0], st.x[1])
    with pytest.raises(binding.InterlockError) as e:
        binding.il_head_xent_static(st.ctx, 1, st.x[1], st.targets, st.losses)
    assert e.value.status == binding.IL_E_WORKSPACE
    binding.il_head_xent(st.ctx, 1, st.x[1], st.targets, st.losses)      # the workspace variant still serves it
    st.close()
    # heads with blocks of their own are not served by this variant
    w = synth.WORKLOADS["tiny"].with_(Lh=1)
    params, x0, tgt = make_inputs(w, seed=23)
    st = binding.Step(w, binding.pack_params(w, params))
    st.set_inputs(x0, tgt)
    binding.il_stage_forward(st.ctx, 1, st.x[0], st.x[1])
    with pytest.raises(binding.InterlockError) as e:
        binding.il_head_xent_static(st.ctx, 1, st.x[1], st.targets, st.losses)
    assert e.value.status == binding.IL_E_SHAPE
    st.close()
    torch.cuda.synchronize()
