"""GPU parity of il_adam_step against the float64 oracle (App. B), through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import adam as A
from paper_2010_04116_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-5


def rel(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b) / max(np.linalg.norm(b), 1e-300))


def run_steps(dtype, count, nsteps, seed):
    """The same seeded gradients through the library (fp32 arithmetic) and the oracle (float64)."""
    rng = np.random.default_rng(seed)
    th0 = (rng.normal(size=count) * 0.02).astype(np.float32)
    if dtype == "bf16":
        th0 = synth.round_to_bf16(th0)
    w = torch.from_numpy(th0.copy()).to(DEV)                       # fp32 weights (master in bf16 mode)
    p = w.to(torch.bfloat16) if dtype == "bf16" else w
    m = torch.zeros(count, device=DEV)
    v = torch.zeros(count, device=DEV)
    th, mo, vo = th0.astype(np.float64), np.zeros(count), np.zeros(count)
    stream = torch.cuda.current_stream().cuda_stream
    for step in range(1, nsteps + 1):
        # gradient scales from 1e-6 to 1 within one buffer, as across the layers of a deep model
        g = (rng.normal(size=count) * 10.0 ** rng.uniform(-6, 0, size=count)).astype(np.float32)
        lr = binding.il_lr_schedule(step, 512, 10)
        assert lr == pytest.approx(A.lr_schedule(step, 512, 10), rel=1e-14)
        gd = torch.from_numpy(g).to(DEV)
        binding.il_adam_step(dtype, p, w if dtype == "bf16" else None, gd, m, v, count, step, lr, stream=stream)
        th, mo, vo = A.adam_step(th, g.astype(np.float64), mo, vo, step, lr)
    torch.cuda.synchronize()
    return dict(w=w.cpu().numpy(), p=p.float().cpu().numpy(), m=m.cpu().numpy(), v=v.cpu().numpy()), dict(w=th, m=mo, v=vo)


@pytest.mark.parametrize("count", [1, 3, 4, 1021, 262144 + 5, 3_000_001])
def test_fp32_parity(count):
    print("case adam fp32 count", count, flush=True)
    got, ref = run_steps("f32", count, 4, seed=count)
    # fp32 arithmetic: a moment update is four roundings (<= 4 * 2^-24 = 2.4e-7 relative), four
    # steps add up to <= 1e-6; the bar is ten times that, a tenth of the 1e-4 the fp32 step is held to
    assert rel(got["m"], ref["m"]) <= TOL
    assert rel(got["v"], ref["v"]) <= TOL
    assert rel(got["w"], ref["w"]) <= TOL
    # and in absolute terms the weights are off by a small fraction of one update (lr ~ 1e-3 .. 1e-2)
    assert np.abs(ref["w"] - got["w"]).max() <= 1e-6


@pytest.mark.parametrize("count", [2, 1024 + 3, 1_000_003])
def test_bf16_parity(count):
    print("case adam bf16 count", count, flush=True)
    got, ref = run_steps("bf16", count, 4, seed=100 + count)
    assert rel(got["m"], ref["m"]) <= TOL and rel(got["v"], ref["v"]) <= TOL
    assert rel(got["w"], ref["w"]) <= TOL                                # the fp32 master weights
    # the bf16 parameters are exactly the round-to-nearest-even image of the library's own master ...
    assert np.array_equal(got["p"], synth.round_to_bf16(got["w"]))
    # ... and therefore within half a bf16 ulp (2^-9 relative) of the oracle's weights, plus what the
    # fp32 master itself is off by (matters only for weights that sit next to zero)
    bound = np.abs(got["w"]).astype(np.float64) * 2.0 ** -8 + np.abs(got["w"] - ref["w"])
    assert np.all(np.abs(got["p"] - ref["w"]) <= bound + 1e-30)


def test_moves_against_the_gradient_and_is_restartable():
    count = 4096
    g = torch.ones(count, device=DEV)
    w = torch.zeros(count, device=DEV)
    m = torch.zeros(count, device=DEV)
    v = torch.zeros(count, device=DEV)
    binding.il_adam_step("f32", w, None, g, m, v, count, 1, 0.5)
    torch.cuda.synchronize()
    np.testing.assert_allclose(w.cpu().numpy(), -0.5, rtol=1e-6)          # first step: lr * g / |g|
    binding.il_adam_step("f32", w, None, g, m, v, 0, 2, 0.5)              # empty update: nothing happens
    torch.cuda.synchronize()
    np.testing.assert_allclose(w.cpu().numpy(), -0.5, rtol=1e-6)


def test_misuse_on_device_buffers():
    x = torch.zeros(64, device=DEV)
    for kwargs, status in [
        (dict(step=0), binding.IL_E_ARG),
        (dict(beta1=1.0), binding.IL_E_ARG),
        (dict(eps=-1.0), binding.IL_E_ARG),
    ]:
        a = dict(step=1, beta1=0.9, beta2=0.98, eps=1e-9)
        a.update(kwargs)
        with pytest.raises(binding.InterlockError) as e:
            binding.il_adam_step("f32", x, None, x, x, x, 64, a["step"], 0.1, a["beta1"], a["beta2"], a["eps"])
        assert e.value.status == status
    with pytest.raises(binding.InterlockError) as e:                       # fp32 mode takes no master copy
        binding.il_adam_step("f32", x, x, x, x, x, 64, 1, 0.1)
    assert e.value.status == binding.IL_E_ARG
    with pytest.raises(binding.InterlockError) as e:                       # bf16 mode needs one
        binding.il_adam_step("bf16", x, None, x, x, x, 64, 1, 0.1)
    assert e.value.status == binding.IL_E_ARG
    with pytest.raises(binding.InterlockError) as e:                       # misaligned fp32 buffer
        binding.il_adam_step("f32", x[1:], None, x, x, x, 32, 1, 0.1)
    assert e.value.status == binding.IL_E_SHAPE
