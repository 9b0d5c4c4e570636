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
# 9 .. 17 rows (K a multiple of 512) take the same organisation with matrix-core products on LDS-transposed half
# tiles: every row count again (16 and 17 differ in how the 17th row's operands are held)
@pytest.mark.parametrize("M", list(range(1, 18)))
def test_bf16_row_stripes(M):
    _check(M, 4096 + 16 * 7, 2048, torch.bfloat16, 40 + M, 2e-5)       # one stripe, 2 rows per wavefront + a ragged end
    _check(M, 1001, 4096, torch.bfloat16, 50 + M, 2e-5)                 # two stripes, fewer rows than wavefronts, odd N
    _check(M, 2560, 8192, torch.bfloat16, 60 + M, 3e-5)                 # four stripes (the 70B shape's K)


# 16384: 8 stripes in one workgroup; 28672 (the 70B down projection): 14 stripes, 7 wavefronts (448 threads) taking
# two each; 18432: 9 stripes, 3 wavefronts x 3; tiny N: row ranges of one row, idle wavefronts
@pytest.mark.parametrize("shape", [(8, 640, 16384), (3, 5, 2048), (1, 1, 2048), (7, 32000, 2048), (2, 57344, 8192),
                                   (5, 1024 + 8, 28672), (8, 8192, 28672), (4, 2048, 2048 * 9), (6, 300, 2048 * 5),
                                   # 9 .. 17 rows: 32 pieces of K in 4 passes, tiny N (ranges of one half tile, idle
                                   # wavefronts), one piece, the 70B matrices, odd N, 5 pieces (one K slot, 8 row ranges)
                                   (17, 640, 16384), (12, 5, 2048), (9, 1, 512), (17, 57344, 8192), (13, 8192, 28672),
                                   (16, 32000, 8192), (17, 1001, 4096), (11, 3000, 2560), (10, 10240, 8192)])
def test_bf16_row_stripes_extremes(shape):
    _check(*shape, torch.bfloat16, 9, 3e-5)


def test_bf16_rows_beyond_the_stripe_kernel_take_the_matrix_cores():
    from paper_2405_19715_amd import binding as B
    # the stripes of a row range are added inside the workgroup (a wavefront takes several in turn when there are
    # more than 8, or a number 8 wavefronts do not divide): always one slice
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 8, 8192, 8192) == 8 * 8192 * 4
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 2, 4096, 4096) == 2 * 4096 * 4
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 8, 8192, 28672) == 8 * 8192 * 4
    _check(4, 4096, 2048 * 11, torch.bfloat16, 3, 3e-5)          # 11 stripes: one wavefront per row range takes them all
    # K not a multiple of 2048: the last stripe is short (lanes beyond K multiply zeros): 11008 = the 7B down
    # projection (6 stripes, 6 wavefronts), 5632 = the 1.1B one, 2048 + 8 = one 16-byte piece in the last stripe
    for K in (11008, 5632, 2048 + 8, 4096 + 2040):
        _check(5, 1000, K, torch.bfloat16, 3, 3e-5)
        assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 5, 1000, K) == 5 * 1000 * 4
    # 9 .. 17 rows with K not a multiple of 512, more than 17 rows, or few rows with K below 2048: MFMA kernels
    # with K slices
    _check(9, 2560, 8192 + 128, torch.bfloat16, 3, 3e-5)
    _check(18, 2560, 8192, torch.bfloat16, 3, 3e-5)
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 17, 8192, 8192) == 17 * 8192 * 4      # one slice up to 17 rows
    _check(4, 4096, 1024, torch.bfloat16, 3, 3e-5)
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 4, 4096, 1024) > 4 * 4096 * 4


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


def _mlp_case(M, ffn, K, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    W = (torch.randn((2 * ffn, K), generator=g) * (2.0 / K ** 0.5)).to(dtype)
    X = torch.randn((M, K), generator=g).to(dtype)
    return W, X


def _mlp_check(M, ffn, K, dtype, seed, mode):
    """The gated activation against the oracle's fp64 definition of it: one rounding to the storage type at
    the end (2^-9 relative for bf16) plus fp32 accumulation noise relative to the largest product."""
    from oracle.model import silu
    from paper_2405_19715_amd import binding as B
    W, X = _mlp_case(M, ffn, K, dtype, seed)
    x, w = X.double().numpy(), W.double().numpy()
    gate, up = x @ w[:ffn].T, x @ w[ffn:].T
    want = silu(gate) * up
    got_t = B.sd_mlp_act(W.cuda(), X.cuda(), mode=mode).cpu()
    got = got_t.float().double().numpy()
    assert got.shape == want.shape
    rel = 2.0 ** -8 if dtype == torch.bfloat16 else 1e-5
    tol = rel * np.abs(want) + 3e-5 * np.abs(gate).max() * np.abs(up).max()
    bad = np.abs(got - want) > tol
    assert not bad.any(), (M, ffn, K, mode, int(bad.sum()), float(np.abs(got - want).max()))
    return got_t


# one, two, three and four stripes per row range (K = 2048 .. 8192), every row count, ffn that leaves ragged and
# idle row ranges; the one-launch kernel and the product + activation kernel take the same sums in the same order
@pytest.mark.parametrize("M,ffn,K", [(1, 1376, 2048), (2, 5632, 2048), (3, 1376, 6144), (4, 688, 4096), (5, 100, 2048),
                                     (6, 11008, 4096), (7, 3584, 8192), (8, 1001, 8192), (2, 28672, 8192),
                                     (9, 3584, 8192), (12, 28672, 8192), (16, 1001, 4096), (17, 28672, 8192),
                                     (17, 100, 512), (13, 5632, 2048), (10, 11008, 4096)])
def test_mlp_activation_one_launch_kernel(M, ffn, K):
    from paper_2405_19715_amd import binding as B
    assert B.sd_mlp_act_is_fused(torch.bfloat16, M, ffn, K)
    fused = _mlp_check(M, ffn, K, torch.bfloat16, 31 + M, mode=1)
    split = _mlp_check(M, ffn, K, torch.bfloat16, 31 + M, mode=0)
    if M <= 8:
        assert torch.equal(fused.view(torch.int16), split.view(torch.int16))
    # beyond 8 rows the paired launch groups the K pieces over 4 wavefronts per row range where the plain product
    # uses 8: the same sums in another order, each within the tolerance above


@pytest.mark.parametrize("M,ffn,K,dtype", [(17, 688, 256, torch.bfloat16), (40, 1376, 1024, torch.bfloat16),
                                           (18, 3584, 8192, torch.bfloat16), (9, 3584, 8192 + 256, torch.bfloat16),
                                           (4, 512, 16384, torch.bfloat16),
                                           (3, 172, 256, torch.float32)])
def test_mlp_activation_where_the_one_launch_kernel_does_not_apply(M, ffn, K, dtype):
    from paper_2405_19715_amd import binding as B
    assert not B.sd_mlp_act_is_fused(dtype, M, ffn, K)
    _mlp_check(M, ffn, K, dtype, 5, mode=-1)
    W, X = _mlp_case(M, ffn, K, dtype, 5)
    with pytest.raises(B.SpecDecError):
        B.sd_mlp_act(W.cuda(), X.cuda(), mode=1)


# ---------------------------------------------------------------- q|k|v product + rotary embedding + KV append
def _qkv_case(M, Hq, Hkv, hd, K, dtype, seed, n_seq=3, max_seq=64):
    g = torch.Generator().manual_seed(seed)
    N = (Hq + 2 * Hkv) * hd
    W = (torch.randn((N, K), generator=g) * (1.0 / K ** 0.5)).to(dtype)
    X = torch.randn((M, K), generator=g).to(dtype)
    seq = torch.randint(0, n_seq, (M,), generator=g, dtype=torch.int32)
    pos = torch.randperm(max_seq, generator=g)[:M].to(torch.int32)        # distinct cache slots
    if M >= 3:
        seq[M // 2] = -1                                                  # a padding row writes nothing
    return W, X, seq, pos


def _qkv_run(M, Hq, Hkv, hd, K, dtype, seed, mode, n_seq=3, max_seq=64, theta=10000.0):
    """Runs sd_qkv_rope and checks q, the key rows and the value columns it wrote against the oracle's rotary
    embedding of the fp64 product; everything it must not touch keeps its fill value."""
    from oracle import model as OM
    from paper_2405_19715_amd import binding as B
    W, X, seq, pos = _qkv_case(M, Hq, Hkv, hd, K, dtype, seed, n_seq, max_seq)
    half = hd // 2
    ang = np.arange(max_seq, dtype=np.float64)[:, None] * theta ** (-np.arange(half, dtype=np.float64) * 2 / hd)
    cos_sin = torch.from_numpy(np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32))
    fill = 7.0
    q = torch.full((M, Hq * hd), fill, dtype=dtype).cuda()
    kc = torch.full((n_seq, Hkv, max_seq, hd), fill, dtype=dtype).cuda()
    vc = torch.full((n_seq, Hkv, hd, max_seq), fill, dtype=dtype).cuda()
    B.sd_qkv_rope(W.cuda(), X.cuda(), Hq, Hkv, hd, seq.cuda(), pos.cuda(), cos_sin.cuda(), q, kc, vc, mode=mode)
    torch.cuda.synchronize()
    q_t, kc_t, vc_t = q.cpu(), kc.cpu(), vc.cpu()

    y = X.double().numpy() @ W.double().numpy().T
    p = pos.numpy().astype(np.int64)
    want_q = OM.rope(y[:, : Hq * hd].reshape(M, Hq, hd), p, theta).reshape(M, Hq * hd)
    want_k = OM.rope(y[:, Hq * hd: (Hq + Hkv) * hd].reshape(M, Hkv, hd), p, theta)
    want_v = y[:, (Hq + Hkv) * hd:].reshape(M, Hkv, hd)
    rel = 2.0 ** -8 if dtype == torch.bfloat16 else 1e-5
    floor = 3e-5 * np.abs(X.double().numpy()).max() * np.abs(W.double().numpy()).max() * K ** 0.5

    def close(got, want, what):
        bad = np.abs(got - want) > rel * np.abs(want) + floor
        assert not bad.any(), (what, M, Hq, Hkv, hd, K, mode, int(bad.sum()), float(np.abs(got - want).max()))

    exp_k = torch.full_like(kc_t, fill).double().numpy()
    exp_v = torch.full_like(vc_t, fill).double().numpy()
    live = seq.numpy() >= 0
    for m in range(M):
        if not live[m]:
            assert (q_t[m].float() == fill).all()
            continue
        close(q_t[m].double().numpy(), want_q[m], "q")
        exp_k[seq[m], :, p[m], :] = want_k[m]
        exp_v[seq[m], :, :, p[m]] = want_v[m]
    close(kc_t.double().numpy(), exp_k, "k cache")       # untouched entries must equal the fill exactly:
    close(vc_t.double().numpy(), exp_v, "v cache")       # |7 - want| is far outside the tolerance
    written_k = np.zeros(exp_k.shape, bool)
    written_v = np.zeros(exp_v.shape, bool)
    for m in range(M):
        if live[m]:
            written_k[seq[m], :, p[m], :] = True
            written_v[seq[m], :, :, p[m]] = True
    assert (kc_t.float().numpy()[~written_k] == fill).all() and (vc_t.float().numpy()[~written_v] == fill).all()
    return q_t, kc_t, vc_t


# head dimensions 128 and 64, grouped and plain heads, one to four stripes and a ragged last stripe, every row count
@pytest.mark.parametrize("M,Hq,Hkv,hd,K", [(1, 16, 2, 128, 2048), (2, 32, 32, 128, 4096), (3, 8, 1, 128, 8192),
                                           (4, 12, 4, 64, 2048), (5, 5, 5, 64, 6144), (6, 64, 8, 128, 8192),
                                           (7, 3, 1, 32, 4096), (8, 16, 4, 128, 5120), (8, 1, 1, 16, 2048),
                                           (2, 20, 4, 128, 2560), (9, 16, 2, 128, 2048), (12, 64, 8, 128, 8192),
                                           (16, 32, 32, 128, 4096), (17, 64, 8, 128, 8192), (17, 12, 4, 64, 2048),
                                           (13, 3, 1, 32, 1536), (10, 5, 5, 64, 6144)])
def test_qkv_rotary_append_one_launch_kernel(M, Hq, Hkv, hd, K):
    from paper_2405_19715_amd import binding as B
    assert B.sd_qkv_rope_is_fused(torch.bfloat16, M, Hq, Hkv, hd, K)
    fused = _qkv_run(M, Hq, Hkv, hd, K, torch.bfloat16, 77 + M, mode=1)
    split = _qkv_run(M, Hq, Hkv, hd, K, torch.bfloat16, 77 + M, mode=0)
    if M <= 8:
        for a, b in zip(fused, split):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    # beyond 8 rows a row range starts its walk over the K pieces at a piece of its own, and the rotary launch cuts the
    # (permuted) rows into other ranges than the plain product: the same sums in another order, each checked above


@pytest.mark.parametrize("M,Hq,Hkv,hd,K,dtype", [(18, 16, 2, 128, 2048, torch.bfloat16), (4, 8, 2, 96, 2048, torch.bfloat16),
                                                 (17, 8, 2, 64, 256, torch.bfloat16), (3, 4, 2, 16, 64, torch.float32)])
def test_qkv_rotary_append_where_the_one_launch_kernel_does_not_apply(M, Hq, Hkv, hd, K, dtype):
    from paper_2405_19715_amd import binding as B
    assert not B.sd_qkv_rope_is_fused(dtype, M, Hq, Hkv, hd, K)
    _qkv_run(M, Hq, Hkv, hd, K, dtype, 9, mode=-1)
    with pytest.raises(B.SpecDecError):
        _qkv_run(M, Hq, Hkv, hd, K, dtype, 9, mode=1)
