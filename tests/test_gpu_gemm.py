"""Kernel-level parity of the bf16 MFMA GEMM (every tile configuration, operand layout and
epilogue the step uses, ragged edges, segmented weight-gradient reduction) against a float64
matrix product of the same bf16-rounded operands.  Through the C ABI's il_test_gemm hook."""
import numpy as np
import pytest

from oracle import interlock as O
from paper_2010_04116_amd import binding as b, synth

pytestmark = pytest.mark.gpu
TILES = [1, 2, 3, 4, 5, 6, 7, 8]
# the (layout, epilogue) pairs the library instantiates: forward, data gradient, weight gradient
# (epilogue 7: the head's logits tile, stored as IEEE half)
_COMBOS = [(0, 1, 0), (0, 1, 1), (0, 1, 2), (0, 1, 3), (0, 0, 0), (0, 0, 4), (0, 0, 5), (1, 1, 6), (0, 1, 7)]


def _bf16(a):
    return synth.round_to_bf16(a.astype(np.float32))


_gelu, _gelu_grad = O.gelu, O.gelu_grad      # the oracle's tanh-GELU (pinned in test_oracle_primitives.py)


def run_case(M, N, K, akm, bkm, epi, tile, seed=0, beta=0, scale=1.0):
    import torch
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(seed)
    A = _bf16(rng.standard_normal((M, K)) * 0.5)
    B = _bf16(rng.standard_normal((K, N)) * 0.5)
    bias = _bf16(rng.standard_normal(N) * 0.5)
    res = rng.standard_normal((M, N)).astype(np.float32)
    aux_rows = max(1, M // 2)
    aux = _bf16(rng.standard_normal((aux_rows, N)))
    c0 = rng.standard_normal((M, N)).astype(np.float32)
    acc = A.astype(np.float64) @ B.astype(np.float64)
    tb = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16).to(dev)
    tf = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    dA = tb(A.T if akm else A)
    dB = tb(B if bkm else B.T)
    f32out = epi in (3, 5, 6)
    C = tf(c0) if f32out else torch.zeros((M, N), dtype=torch.bfloat16, device=dev)
    C2 = torch.zeros((M, N), dtype=torch.bfloat16, device=dev)
    b.il_test_gemm(b.IL_BF16, dA, dB, M, N, K, M if akm else K, N if bkm else K, akm, bkm, epi, C, C2=C2,
                   ldc=N, bias=tb(bias), res=tf(res), aux=tb(aux), aux_wrap=aux_rows, scale=scale, beta=beta,
                   tile=tile, stream=torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = (C.view(torch.float16) if epi == 7 else C).float().cpu().numpy().astype(np.float64)
    if epi == 0:
        want = acc
    elif epi == 1:
        want = acc + bias
    elif epi == 2:
        want = acc + bias
        got2 = C2.float().cpu().numpy().astype(np.float64)
        want2 = _gelu(_bf16(want).astype(np.float64))
        assert np.linalg.norm(got2 - want2) <= 6e-3 * np.linalg.norm(want2)
    elif epi == 3:
        want = acc + bias + res
    elif epi == 4:
        want = acc * _gelu_grad(aux.astype(np.float64))[np.arange(M) % aux_rows]
    elif epi in (5, 7):
        want = acc
    else:
        want = scale * acc + (c0 if beta else 0)
    tol = 1e-5 if f32out else (8e-4 if epi == 7 else 6e-3)   # fp32 outputs: accumulation order only; bf16 / half: one rounding
    err = np.linalg.norm(got - want) / np.linalg.norm(want)
    assert err <= tol, f"M={M} N={N} K={K} akm={akm} bkm={bkm} epi={epi} tile={tile}: rel err {err:.3e}"
    if not f32out:
        assert np.max(np.abs(got - want)) <= (2 ** -10 if epi == 7 else 2 ** -7) * np.max(np.abs(want)) + 1e-6
    # no row, column or tile may hide inside the norm: every row and column to twice the tolerance
    # (on the scale of the RMS row / column for the nearly empty ones), every element to a bf16
    # rounding step of the largest value
    d2 = (got - want) ** 2
    for axis in (0, 1):
        nref = np.sqrt((want ** 2).sum(axis=axis))
        e = np.sqrt(d2.sum(axis=axis)) / np.maximum(nref, np.sqrt((nref ** 2).mean()))
        assert e.max() <= 2 * tol, f"M={M} N={N} K={K} epi={epi} tile={tile}: axis {axis} index {int(e.argmax())} rel err {e.max():.3e}"
    assert np.max(np.abs(got - want)) <= (1e-4 if f32out else 2 ** -7) * np.max(np.abs(want)) + 1e-6


@pytest.mark.parametrize("tile", TILES)
def test_forward_layout_all_epilogues(tile):
    for epi in (0, 1, 2, 3):
        run_case(384, 264, 192, 0, 1, epi, tile, seed=epi)


@pytest.mark.parametrize("tile", TILES)
def test_dgrad_layout_all_epilogues(tile):
    for epi in (0, 4, 5):
        run_case(520, 136, 320, 0, 0, epi, tile, seed=10 + epi)


@pytest.mark.parametrize("tile", TILES)
def test_wgrad_layout(tile):
    run_case(200, 392, 256, 1, 1, 6, tile, seed=20, beta=0, scale=0.5)
    run_case(200, 392, 256, 1, 1, 6, tile, seed=21, beta=1, scale=1.0)


@pytest.mark.parametrize("tile", TILES)
def test_k_tail_and_tiny_sizes(tile):
    run_case(8, 8, 8, 0, 0, 0, tile, seed=30)
    run_case(72, 40, 104, 0, 1, 1, tile, seed=31)      # K not a multiple of 32 or 64
    run_case(72, 40, 104, 0, 0, 5, tile, seed=32)
    run_case(40, 72, 72, 1, 1, 6, tile, seed=33)


@pytest.mark.parametrize("tile", [0] + TILES)
def test_multi_tile_shapes(tile):
    run_case(1024, 768, 512, 0, 1, 1, tile, seed=40)
    run_case(1024, 768, 512, 0, 0, 0, tile, seed=41)
    run_case(512, 1024, 2048, 1, 1, 6, tile, seed=42)


def test_library_choice_at_the_benchmark_shapes():
    """tile = 0 at output shapes of the benchmark workloads, one per branch of the tile choice
    (256x256; 128x128 four-stage; 128x256 / 256x128; 128x128 two-stage; 64x64 four-stage; 64x64),
    with a short K so that the float64 product stays cheap."""
    run_case(4096, 4096, 192, 0, 1, 2, 0, seed=50)      # 256 tiles of 256x256
    run_case(4096, 1024, 192, 0, 1, 3, 0, seed=51)      # 256 tiles of 128x128
    run_case(8192, 1024, 192, 0, 0, 0, 0, seed=52)      # 256 tiles of 128x256
    run_case(1024, 8192, 192, 1, 1, 6, 0, seed=53)      # 256 tiles of 256x128 (k-major operands)
    run_case(4096, 1536, 192, 0, 0, 5, 0, seed=54)      # 384 tiles of 128x128
    run_case(2048, 512, 192, 0, 1, 3, 0, seed=55)       # 256 tiles of 64x64
    run_case(2048, 1536, 192, 0, 1, 1, 0, seed=56)      # 768 tiles of 64x64


@pytest.mark.parametrize("tile", [0, 8])
def test_persistent_kernel_second_round_ragged(tile):
    """More than 256 tiles of 256x256 with ragged M and N (18 x 17 = 306 tiles): workgroups of the
    persistent kernel take a second tile, the loaders run ahead into it while the first tile's epilogue
    is still draining.  Every (layout, epilogue) the step uses."""
    for i, (akm, bkm, epi) in enumerate(_COMBOS):
        M, N = (4360, 4104) if not akm else (4360 - 8, 4104)
        run_case(M, N, 128, akm, bkm, epi, tile, seed=70 + i, beta=int(epi == 6))


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 6, 7, 8])
def test_logits_epilogue_statistics(tile):
    """The head's logits GEMM leaves, beside the half-precision tile, the softmax statistics of every
    64-column group taken from its fp32 accumulators, and each row's target logit: checked against the
    float64 product (ragged M and N, a last group of 40 columns, targets at both ends and out of range)."""
    import torch
    dev = torch.device("cuda:0")
    for M, N, K, seed in ((300, 1000, 192, 90), (520, 4104, 128, 91)):
        rng = np.random.default_rng(seed)
        A = _bf16(rng.standard_normal((M, K)))
        B = _bf16(rng.standard_normal((K, N)) * 0.7)
        acc = A.astype(np.float64) @ B.astype(np.float64)
        tgt = rng.integers(0, N, size=M).astype(np.int32)
        tgt[:4] = [0, N - 1, -1, N]                      # edges, and two ignored positions
        G = (N + 63) // 64
        dA = torch.from_numpy(A).to(torch.bfloat16).to(dev)
        dB = torch.from_numpy(B).to(torch.bfloat16).to(dev)
        C = torch.zeros((M, N), dtype=torch.bfloat16, device=dev)
        S = torch.full((M * G * 2 + M,), -7.0, dtype=torch.float32, device=dev)
        b.il_test_gemm(b.IL_BF16, dA, dB, M, N, K, K, N, 0, 1, 7, C, C2=S, aux=torch.from_numpy(tgt).to(dev), tile=tile,
                       stream=torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        z = C.view(torch.float16).float().cpu().numpy().astype(np.float64)
        assert np.abs(z - acc).max() <= 2 ** -10 * np.abs(acc).max() + 1e-6
        s = S.cpu().numpy().astype(np.float64)
        st, zt = s[:M * G * 2].reshape(M, G, 2), s[M * G * 2:]
        pad = np.full((M, G * 64), -np.inf)
        pad[:, :N] = acc
        grp = pad.reshape(M, G, 64)
        m = grp.max(axis=2)
        se = np.exp(grp - m[:, :, None]).sum(axis=2)
        assert np.abs(st[:, :, 0] - m).max() <= 1e-5 * np.abs(acc).max(), (M, N, tile)
        assert np.abs(st[:, :, 1] / se - 1).max() <= 2e-5, (M, N, tile)
        lse = np.log((st[:, :, 1] * np.exp(st[:, :, 0] - st[:, :, 0].max(axis=1, keepdims=True))).sum(axis=1)) \
            + st[:, :, 0].max(axis=1)
        ref = np.log(np.exp(acc - acc.max(axis=1, keepdims=True)).sum(axis=1)) + acc.max(axis=1)
        assert np.abs(lse - ref).max() <= 2e-5, (M, N, tile)
        ok = (tgt >= 0) & (tgt < N)
        want = acc[np.arange(M)[ok], tgt[ok]]
        assert np.abs(zt[ok] - want).max() <= 1e-5 * np.abs(acc).max(), (M, N, tile)
        assert np.all(zt[~ok] == -7.0)                       # ignored rows are left alone


def test_unsupported_combinations_are_rejected():
    import torch
    dev = torch.device("cuda:0")
    x = torch.zeros((64, 64), dtype=torch.bfloat16, device=dev)
    with pytest.raises(b.InterlockError) as e:       # k-major A with k-contiguous B is not a layout the step uses
        b.il_test_gemm(b.IL_BF16, x, x, 64, 64, 64, 64, 64, 1, 0, 0, x)
    assert e.value.status == b.IL_E_SHAPE
    with pytest.raises(b.InterlockError):            # N not a multiple of 8
        b.il_test_gemm(b.IL_BF16, x, x, 64, 60, 64, 64, 64, 0, 0, 0, x, ldc=64)
    with pytest.raises(b.InterlockError) as e:       # the logits epilogue has no 64x64 tile (32-wide wave tiles)
        b.il_test_gemm(b.IL_BF16, x, x, 64, 64, 64, 64, 64, 0, 1, 7, x, tile=4)
    assert e.value.status == b.IL_E_SHAPE




def test_seeded_random_shapes_every_tile_choice():
    """A seeded sweep over sizes from a single 8-wide sliver to several tiles with ragged edges in
    all three dimensions; tile = 0 lets the library choose, the others force each configuration."""
    rng = np.random.default_rng(20100411)
    dims = [8, 16, 24, 40, 64, 72, 120, 128, 136, 200, 256, 264, 328, 520]
    for case in range(45):
        M, N, K = (int(rng.choice(dims)) for _ in range(3))
        akm, bkm, epi = _COMBOS[case % len(_COMBOS)]
        tile = [0, 1, 2, 3, 4, 5, 6, 7, 0][case % 9]
        print("case", case, M, N, K, akm, bkm, epi, "tile", tile, flush=True)
        run_case(M, N, K, akm, bkm, epi, tile, seed=1000 + case, beta=case & 1, scale=0.5 if case & 2 else 1.0)


def test_long_reduction_and_thin_outputs():
    """The shapes of the head's data gradient (tiny output, very long K) and of a bias-sized sliver."""
    run_case(64, 8, 8192, 0, 0, 5, 0, seed=77)
    run_case(8, 64, 4104, 1, 1, 6, 0, seed=78, beta=1, scale=0.25)
    run_case(72, 8, 520, 0, 1, 3, 0, seed=79)
