"""GPU: the grouped MFMA GEMM against a float64 numpy product."""
import numpy as np
import pytest

from tests.gpu_util import rel_err, to_bf16_bits, from_bf16_bits

pytestmark = pytest.mark.gpu


def _run(prec, a_k, b_k, c_elem, M, N, K, groups, bias, pad=0, seed=0, tile=-1):
    import torch
    from paper_2110_11199_amd import binding as Bd
    r = np.random.default_rng(seed)
    dev = torch.device("cuda:0")
    r4 = lambda v: (v + 3) // 4 * 4
    lda = r4(K if a_k else M) + pad
    ldb = r4(K if b_k else N) + pad
    ldc = N + pad
    A = r.standard_normal((groups, M if a_k else K, lda)).astype(np.float32)
    B = r.standard_normal((groups, N if b_k else K, ldb)).astype(np.float32)
    bv = r.standard_normal((groups, N)).astype(np.float32) if bias else None
    if prec:
        A, B = from_bf16_bits(to_bf16_bits(A)), from_bf16_bits(to_bf16_bits(B))
        dA = torch.from_numpy(to_bf16_bits(A).view(np.int16)).to(dev)
        dB = torch.from_numpy(to_bf16_bits(B).view(np.int16)).to(dev)
    else:
        dA, dB = torch.from_numpy(A).to(dev), torch.from_numpy(B).to(dev)
    cdt = torch.int16 if (prec and c_elem) else torch.float32
    dC = torch.full((groups, M, ldc), 7, dtype=cdt, device=dev)
    dbias = torch.from_numpy(bv).to(dev) if bias else None
    Bd.adpsgd_gemm(prec, a_k, b_k, c_elem, M, N, K, dA.data_ptr(), lda, dA[0].numel(), dB.data_ptr(), ldb,
                   dB[0].numel(), dC.data_ptr(), ldc, M * ldc, dbias.data_ptr() if bias else None, N, groups,
                   torch.cuda.current_stream().cuda_stream, tile_config=tile)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    if prec and c_elem:
        got = from_bf16_bits(got.view(np.uint16))
    Am = A[:, :, :K] if a_k else A[:, :, :M].transpose(0, 2, 1)
    Bm = B[:, :, :K] if b_k else B[:, :, :N].transpose(0, 2, 1)
    ref = np.einsum("gmk,gnk->gmn", Am.astype(np.float64), Bm.astype(np.float64))
    if bias:
        ref += bv[:, None, :]
    if pad:
        assert (got[:, :, N:] == (from_bf16_bits(np.array([7], np.uint16))[0] if (prec and c_elem) else 7)).all()
    return rel_err(got[:, :, :N], ref)


LAYOUTS = [(1, 1), (1, 0), (0, 0), (0, 1)]


@pytest.mark.parametrize("a_k,b_k", LAYOUTS)
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (200, 136, 100), (80, 256, 40), (257, 129, 260), (4, 4, 4)])
def test_gemm_fp32(a_k, b_k, M, N, K):
    print("gemm fp32", a_k, b_k, M, N, K, flush=True)
    assert _run(0, a_k, b_k, 0, M, N, K, 3, True, pad=4) < 2e-6
    assert _run(0, a_k, b_k, 1, M, N, K, 1, False) < 2e-6


@pytest.mark.parametrize("a_k,b_k", LAYOUTS)
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (200, 136, 100), (80, 256, 40), (257, 132, 260), (4, 8, 12)])
def test_gemm_bf16(a_k, b_k, M, N, K):
    print("gemm bf16", a_k, b_k, M, N, K, flush=True)
    # operands are exactly representable in bf16, so only the fp32 accumulation differs
    assert _run(1, a_k, b_k, 0, M, N, K, 3, True, pad=8) < 2e-6
    assert _run(1, a_k, b_k, 0, M, N, K, 2, False, pad=4) < 2e-6      # 8-byte aligned rows only
    assert _run(1, a_k, b_k, 1, M, N, K, 1, True) < 6e-3             # bf16 output rounding


@pytest.mark.parametrize("a_k,b_k", LAYOUTS)
@pytest.mark.parametrize("M,N,K,pad", [(520, 520, 192, 0), (520, 520, 192, 8), (516, 524, 128, 0), (516, 524, 128, 4),
                                         (264, 776, 100, 0), (520, 520, 64, 0), (520, 516, 448, 8)])
def test_gemm_bf16_large_tiles(a_k, b_k, M, N, K, pad):
    # enough 256x256 tiles (>= 128 over the groups) for the large-tile kernels: direct-to-LDS loads
    # when K is a multiple of 64 and all rows are 16-byte aligned (row counts need not be multiples of 8: pad=4
    # makes the k-rows of a 516-row operand 520 long), else register staging; K = 64 ... 448 is 2 ... 14 stages of
    # the direct-to-LDS main loop (its first, steady-state and last stages are separate code)
    print("gemm bf16 large", a_k, b_k, M, N, K, pad, flush=True)
    groups = 16 if N < 600 else 22
    assert _run(1, a_k, b_k, 0, M, N, K, groups, True, pad=pad) < 2e-6
    assert _run(1, a_k, b_k, 1, M, N, K, groups, False, pad=pad) < 6e-3


@pytest.mark.parametrize("a_k,b_k", LAYOUTS)
@pytest.mark.parametrize("M,N,K,pad", [(520, 516, 512, 0), (776, 520, 576, 8)])
def test_gemm_bf16_long_k_loop(a_k, b_k, M, N, K, pad):
    # 16 and 18 K stages of the hand-pipelined main loop (its steady state)
    print("gemm bf16 long K", a_k, b_k, M, N, K, pad, flush=True)
    assert _run(1, a_k, b_k, 0, M, N, K, 16, True, pad=pad) < 2e-6
    assert _run(1, a_k, b_k, 1, M, N, K, 16, False, pad=pad) < 6e-3


@pytest.mark.parametrize("variant", [11, 12, 13])
@pytest.mark.parametrize("a_k,b_k", LAYOUTS)
@pytest.mark.parametrize("K", [64, 128, 192, 256])
def test_gemm_bf16_forced_large_tile_configurations(variant, a_k, b_k, K):
    # the pipelined main loops (11: 64-k stages, 12 and 13: 32-k stages) have separate code for their first
    # stages, their steady state and their last stages: 1 .. 4 and 2 .. 8 stages here, in every operand layout
    # (the automatic choice uses 11 and 13 for K-contiguous operands only, 12 for the others)
    print("gemm bf16 forced configuration", variant, a_k, b_k, K, flush=True)
    assert _run(1, a_k, b_k, 0, 300, 264, K, 3, True, pad=8, tile=variant) < 2e-6


def test_gemm_rejects_misaligned_rows():
    import torch
    from paper_2110_11199_amd import binding as Bd
    t = torch.zeros(64 * 66, device="cuda:0")
    with pytest.raises(Bd.AdpsgdError) as ei:
        Bd.adpsgd_gemm(0, 1, 1, 0, 8, 8, 8, t.data_ptr(), 10, 0, t.data_ptr(), 8, 0, t.data_ptr(), 8, 0, None, 0, 1, None)
    assert ei.value.code == Bd.EINVAL
    for bad_tile, groups in ((7, 1), (-1, 0), (-1, 129)):     # unknown tile configuration, group counts out of range
        with pytest.raises(Bd.AdpsgdError) as ei:
            Bd.adpsgd_gemm(0, 1, 1, 0, 8, 8, 8, t.data_ptr(), 8, 0, t.data_ptr(), 8, 0, t.data_ptr(), 8, 0, None, 0, groups, None,
                           tile_config=bad_tile)
        assert ei.value.code == Bd.EINVAL
