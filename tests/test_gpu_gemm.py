"""Parity of the weight-streaming skinny GEMM (HIP, through the C ABI) with the
oracle's plain fp64 matrix product on the same seeded inputs."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _check(M, N, K, dtype, seed, tol):
    from paper_2405_19715_amd import binding as B
    g = torch.Generator().manual_seed(seed)
    W = (torch.randn((N, K), generator=g) * 0.05).to(dtype)
    X = torch.randn((M, K), generator=g).to(dtype)
    want = X.double().numpy() @ W.double().numpy().T            # the definition, in fp64
    got = B.sd_gemm_skinny(W.cuda(), X.cuda()).cpu().double().numpy()
    scale = np.abs(want).max()
    err = np.abs(got - want).max() / scale
    assert err < tol, (M, N, K, dtype, err)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 9, 16, 17, 31, 32, 33, 48, 136])
def test_bf16_rows(M):
    # several 64-row workgroup tiles, a ragged last workgroup (N = 16 * 13), several K slices
    _check(M, 16 * 13, 1024, torch.bfloat16, M, 2e-5)
    _check(M, 256, 128, torch.bfloat16, 100 + M, 2e-5)


@pytest.mark.parametrize("shape", [(17, 512, 8192), (17, 1024, 28672 // 4), (1, 4096, 4096), (2, 1024, 11008),
                                   (17, 2560, 2048), (8, 32000, 256)])
def test_bf16_model_shapes(shape):
    _check(*shape, torch.bfloat16, 7, 3e-5)


# Up to 8 rows with K a multiple of 2048 (up to 16384) take the kernel that streams whole 1 KB row pieces and
# multiplies on the vector ALU: every row count (each has its own instantiation and lane reduction), one to eight
# K stripes, row counts N that leave ragged row ranges (fewer rows than wavefronts, a short last range, N odd)
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8])
def test_bf16_row_stripes(M):
    _check(M, 4096 + 16 * 7, 2048, torch.bfloat16, 40 + M, 2e-5)       # one stripe, 2 rows per wavefront + a ragged end
    _check(M, 1001, 4096, torch.bfloat16, 50 + M, 2e-5)                 # two stripes, fewer rows than wavefronts, odd N
    _check(M, 2560, 8192, torch.bfloat16, 60 + M, 3e-5)                 # four stripes (the 70B shape's K)


# 16384: 8 stripes in one workgroup; 28672 (the 70B down projection): 14 stripes, 7 per workgroup (448 threads), two
# partial-sum slices; 18432: 9 stripes, 3 per workgroup, three slices; tiny N: row ranges of one row, idle wavefronts
@pytest.mark.parametrize("shape", [(8, 640, 16384), (3, 5, 2048), (1, 1, 2048), (7, 32000, 2048), (2, 57344, 8192),
                                   (5, 1024 + 8, 28672), (8, 8192, 28672), (4, 2048, 2048 * 9), (6, 300, 2048 * 5)])
def test_bf16_row_stripes_extremes(shape):
    _check(*shape, torch.bfloat16, 9, 3e-5)


def test_bf16_rows_beyond_the_stripe_kernel_take_the_matrix_cores():
    from paper_2405_19715_amd import binding as B
    # the stripes of a row range are added inside the workgroup: one slice up to K = 16384, two for K = 28672
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 8, 8192, 8192) == 8 * 8192 * 4
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 2, 4096, 4096) == 2 * 4096 * 4
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 8, 8192, 28672) == 2 * 8 * 8192 * 4
    # 9 rows, K not a multiple of 2048, or a stripe count that leaves more than 4 slices (11 stripes, prime): MFMA kernel
    _check(9, 2560, 8192, torch.bfloat16, 3, 3e-5)
    _check(4, 4096, 2048 * 11, torch.bfloat16, 3, 3e-5)
    _check(4, 4096, 2048 + 128, torch.bfloat16, 3, 3e-5)


@pytest.mark.parametrize("shape", [(1, 256, 256), (9, 1024, 256), (17, 688 * 2, 256), (32, 256, 688), (3, 7, 5)])
def test_fp32(shape):
    _check(*shape, torch.float32, 11, 2e-6)


def test_rejects_shapes_the_kernel_cannot_take():
    from paper_2405_19715_amd import binding as B
    W = torch.zeros((16, 100), dtype=torch.bfloat16, device="cuda")      # K not a multiple of 128
    X = torch.zeros((1, 100), dtype=torch.bfloat16, device="cuda")
    Y = torch.zeros((1, 16), dtype=torch.float32, device="cuda")
    ws = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.SpecDecError):
        B.sd_gemm_skinny(W, X, out=(Y, ws))


def _check_tile(M, N, K, seed, tol=3e-5):
    from paper_2405_19715_amd import binding as B
    g = torch.Generator().manual_seed(seed)
    W = (torch.randn((N, K), generator=g) * 0.05).to(torch.bfloat16)
    X = torch.randn((M, K), generator=g).to(torch.bfloat16)
    want = X.double().numpy() @ W.double().numpy().T            # the definition, in fp64
    Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    got = B.sd_gemm_tile(W.cuda(), X.cuda(), out=Y).cpu().double().numpy()
    assert np.isfinite(got).all(), (M, N, K)                    # every element of Y was written
    err = np.abs(got - want).max() / np.abs(want).max()
    assert err < tol, (M, N, K, err)


@pytest.mark.parametrize("shape", [
    (1, 64, 32), (64, 128, 32), (128, 256, 64), (130, 640, 512), (257, 1284, 96), (63, 36, 160),
    (512, 2048, 1024), (1024, 1280, 512), (300, 4096, 4096), (1023, 2560, 2048)])
def test_tile_gemm_matches_fp64_matmul(shape):
    """The prompt-pass GEMM: all three tile shapes, ragged M and N tails, one and many
    k steps, grids that do not fill the last group of 8 weight tiles."""
    _check_tile(*shape, seed=sum(shape))


def test_tile_gemm_rejects_bad_shapes():
    from paper_2405_19715_amd import binding as B
    W = torch.zeros((16, 48), dtype=torch.bfloat16, device="cuda")       # K not a multiple of 32
    X = torch.zeros((4, 48), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.SpecDecError):
        B.sd_gemm_tile(W, X)
