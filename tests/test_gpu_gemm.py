"""GPU parity of the projection GEMM on its own: the three layouts, ragged and
tile-straddling extents, float accumulation into an existing output, and the
workload's full-size shapes checked on sampled outputs."""
import numpy as np
import pytest
import torch

from paper_2408_12596_amd import binding as pb
from gpu_util import DEV, assert_close_blockwise, rel_l2, to_np, sync

pytestmark = pytest.mark.gpu


def operands(layout, M, N, K, dtype, seed, pad=0):
    """A, B as the layout stores them, with row strides padded by `pad` elements."""
    g = torch.Generator().manual_seed(seed)
    shape_a = (K, M) if layout == pb.GEMM_TN else (M, K)
    shape_b = (N, K) if layout == pb.GEMM_NT else (K, N)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32

    def mk(shape):
        full = torch.zeros(shape[0], shape[1] + (-shape[1]) % 8 + pad, dtype=td)   # zero-padded rows, stride a multiple of 8
        full[:, :shape[1]] = torch.randn(shape, generator=g).to(td)
        return full.to(DEV)
    return mk(shape_a), mk(shape_b), shape_a, shape_b


def oracle(layout, A, B, shape_a, shape_b):
    """The definition: C = sum_k A(m,k) B(k,n) in float64 on the host."""
    a = A[:, :shape_a[1]].double().cpu().numpy()
    b = B[:, :shape_b[1]].double().cpu().numpy()
    if layout == pb.GEMM_NT:
        return a @ b.T
    if layout == pb.GEMM_NN:
        return a @ b
    return a.T @ b


SHAPES = [(64, 64, 64), (128, 128, 64), (200, 136, 72), (129, 257, 520), (1000, 72, 40), (8, 8, 8), (300, 520, 1288), (1, 8, 16)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("layout", [pb.GEMM_NT, pb.GEMM_NN, pb.GEMM_TN])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_matches_definition(layout, M, N, K, dtype):
    ctx = pb.Context(pb.make_cfg(dtype=dtype))
    A, B, sa, sb = operands(layout, M, N, K, dtype, seed=M + N + K, pad=8)
    ref = oracle(layout, A, B, sa, sb)
    tol = 5e-3 if dtype == "bf16" else 1e-5
    # lowp output
    C = torch.full((M, N + (-N) % 8 + 8), 7.0, dtype=A.dtype, device=DEV)
    ctx.gemm(layout, M, N, K, A, A.shape[1], B, B.shape[1], C, C.shape[1])
    # float output, overwritten then accumulated
    ldc = N + (-N) % 8                      # output stride: a multiple of 8 covering N
    Cf = torch.full((M, ldc), float("nan"), device=DEV)
    ctx.gemm(layout, M, N, K, A, A.shape[1], B, B.shape[1], Cf, ldc, c_float=True, beta=0.0)
    sync()
    assert rel_l2(to_np(C[:, :N]), ref) <= tol
    assert rel_l2(to_np(Cf[:, :N]), ref) <= 1e-5   # float output: only the accumulation order differs
    ctx.gemm(layout, M, N, K, A, A.shape[1], B, B.shape[1], Cf, ldc, c_float=True, beta=1.0)
    sync()
    assert rel_l2(to_np(Cf[:, :N]), 2 * ref) <= 1e-5


FULL = [
    # the GPT-2-small workload at local batch 16 (T = 16384 tokens): QKV, MLP up/down, their gradients, the LM head
    (pb.GEMM_NT, 16384, 2304, 768), (pb.GEMM_NT, 16384, 768, 3072), (pb.GEMM_NN, 16384, 3072, 768),
    (pb.GEMM_TN, 3072, 768, 16384), (pb.GEMM_TN, 768, 3072, 16384), (pb.GEMM_NT, 4096, 50257, 768), (pb.GEMM_TN, 50257, 768, 4096),
    (pb.GEMM_NN, 4096, 768, 50257),
]


# ragged extents at sizes where the launcher picks each of its block shapes (256x256, 256x192, 128x128; the
# small shapes above run on 64x64 blocks): partial tiles on both edges, K tails where the layout allows one
RAGGED = [
    (pb.GEMM_NT, 3000, 2000, 576), (pb.GEMM_NN, 3000, 2000, 520), (pb.GEMM_TN, 3000, 2000, 520),
    (pb.GEMM_NT, 5000, 3000, 576), (pb.GEMM_NN, 5000, 3000, 520), (pb.GEMM_TN, 5000, 3000, 520),
    (pb.GEMM_NT, 16000, 2300, 768), (pb.GEMM_NN, 16000, 2300, 776),
]


@pytest.mark.parametrize("c_float", [True, False])
@pytest.mark.parametrize("layout,M,N,K", RAGGED)
def test_gemm_ragged_mid_size_on_sampled_outputs(layout, M, N, K, c_float):
    check_sampled(layout, M, N, K, c_float)


# contractions of one to four K steps at the sizes of RAGGED: the kernel's pipeline is three tiles deep (the first two
# tiles are requested before the loop, the third inside its first step), so these are its start and its end with
# nothing between
SHORT_K = [(layout, M, N, K) for layout in (pb.GEMM_NT, pb.GEMM_NN, pb.GEMM_TN)
           for (M, N) in ((3000, 2000), (5000, 3000), (16000, 2300)) for K in (64, 128, 192, 256)]


@pytest.mark.parametrize("layout,M,N,K", SHORT_K)
def test_gemm_short_contractions_on_sampled_outputs(layout, M, N, K):
    check_sampled(layout, M, N, K, False)


@pytest.mark.parametrize("layout,M,N,K", FULL)
def test_gemm_full_size_on_sampled_outputs(layout, M, N, K):
    check_sampled(layout, M, N, K, True)


# Every element of the output, tile by tile, at the shapes the benchmark launches: the three GPT-2-small products at
# local batch 16, the LM head at 16384 tokens (all three of its products), the ~1.3B layer's products at local
# batch 13 (26624 tokens: an odd tile count on every axis that carries the tokens) and the Llama-7B shape's at 4.
WHOLE = [
    (pb.GEMM_NT, 16384, 2304, 768, False), (pb.GEMM_NN, 16384, 768, 3072, False), (pb.GEMM_TN, 3072, 768, 16384, True),
    (pb.GEMM_NT, 16384, 50257, 768, False), (pb.GEMM_NN, 16384, 768, 50257, False), (pb.GEMM_TN, 50257, 768, 16384, True),
    (pb.GEMM_NT, 26624, 8192, 2048, False), (pb.GEMM_NN, 26624, 2048, 8192, False), (pb.GEMM_TN, 8192, 2048, 26624, True),
    (pb.GEMM_TN, 2048, 6144, 26624, True),
    (pb.GEMM_NT, 8192, 22016, 4096, False), (pb.GEMM_TN, 4096, 11008, 8192, True),
    # 1376 tiles: the launcher cuts the partial sixth round off along N and runs it on smaller tiles
    (pb.GEMM_NN, 8192, 11008, 4096, False), (pb.GEMM_NT, 8192, 11008, 4096, True),
    # 688 tiles of a lone weight gradient: cut along M, the rest split over K
    (pb.GEMM_TN, 11008, 4096, 8192, True),
]


@pytest.mark.parametrize("layout,M,N,K,c_float", WHOLE)
def test_gemm_full_size_every_tile(layout, M, N, K, c_float):
    """The float64 product of the same operands, compared whole and on every 64 x 64 tile of the output."""
    ctx = pb.Context(pb.make_cfg(dtype="bf16"))
    g = torch.Generator().manual_seed(layout * 11 + 3)
    sa = (K, M) if layout == pb.GEMM_TN else (M, K)
    sb = (N, K) if layout == pb.GEMM_NT else (K, N)
    lda, ldb = sa[1] + (-sa[1]) % 8, sb[1] + (-sb[1]) % 8
    if layout == pb.GEMM_NN and K % 64:
        lda = K + (-K) % 64                                  # the head's input gradient: logits rows padded with zeros
    A = torch.zeros(sa[0], lda, dtype=torch.bfloat16)
    A[:, :sa[1]] = torch.randn(sa, generator=g).to(torch.bfloat16)
    B = torch.zeros(sb[0], ldb, dtype=torch.bfloat16)
    B[:, :sb[1]] = torch.randn(sb, generator=g).to(torch.bfloat16)
    dA, dB = A.to(DEV), B.to(DEV)
    ldc = N + (-N) % 8
    C = torch.full((M, ldc), float("nan"), device=DEV, dtype=torch.float32 if c_float else torch.bfloat16)
    ctx.gemm(layout, M, N, K, dA, lda, dB, ldb, C, ldc, c_float=c_float, beta=0.0)
    sync()
    got = C[:, :N].float().cpu().numpy()
    del C
    a, b = A[:, :sa[1]].double().numpy(), B[:, :sb[1]].double().numpy()
    ref = a @ b.T if layout == pb.GEMM_NT else a @ b if layout == pb.GEMM_NN else a.T @ b
    assert np.isfinite(got).all()
    assert_close_blockwise(got, ref, 1e-5 if c_float else 4e-3, name=(layout, M, N, K))


def check_sampled(layout, M, N, K, c_float):
    ctx = pb.Context(pb.make_cfg(dtype="bf16"))
    pad = (-(N if layout != pb.GEMM_NT else K)) % 8 + 8
    pad_a = (-(M if layout == pb.GEMM_TN else K)) % 8 + 8
    g = torch.Generator().manual_seed(layout * 7 + 1)
    sa = (K, M) if layout == pb.GEMM_TN else (M, K)
    sb = (N, K) if layout == pb.GEMM_NT else (K, N)
    A = torch.zeros(sa[0], sa[1] + pad_a, dtype=torch.bfloat16)
    A[:, :sa[1]] = torch.randn(sa, generator=g).to(torch.bfloat16)
    B = torch.zeros(sb[0], sb[1] + pad, dtype=torch.bfloat16)
    B[:, :sb[1]] = torch.randn(sb, generator=g).to(torch.bfloat16)
    A, B = A.to(DEV), B.to(DEV)
    ldc = N + (-N) % 8
    Cf = torch.full((M, ldc), float("nan"), device=DEV, dtype=torch.float32 if c_float else torch.bfloat16)
    ctx.gemm(layout, M, N, K, A, A.shape[1], B, B.shape[1], Cf, ldc, c_float=c_float, beta=0.0)
    sync()
    rng = np.random.default_rng(0)
    ms = np.unique(np.concatenate([rng.integers(0, M, 40), [0, M - 1, min(M - 1, 255), min(M - 1, 256)]]))
    ns = np.unique(np.concatenate([rng.integers(0, N, 40), [0, N - 1, min(N - 1, 127), min(N - 1, 128)]]))
    a = A[:, :sa[1]].double().cpu()
    b = B[:, :sb[1]].double().cpu()
    rows = a[:, ms].T if layout == pb.GEMM_TN else a[ms]          # [len(ms), K]
    cols = b[ns].T if layout == pb.GEMM_NT else b[:, ns]           # [K, len(ns)]
    ref = (rows @ cols).numpy()
    got = Cf[ms][:, ns].double().cpu().numpy()
    assert rel_l2(got, ref) <= (1e-5 if c_float else 4e-3)   # a bf16 output rounds each element once: 2^-9 at most
    assert torch.isfinite(Cf[:, :N]).all()
