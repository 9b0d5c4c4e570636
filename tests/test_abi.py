"""The C-ABI library loads and exports every symbol the public header declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "specdec.h")
LIB = os.path.join(ROOT, "paper_2405_19715_amd", "libspecdec.so")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b((?:sd_|specdec_)\w+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        from paper_2405_19715_amd import build
        build.build(verbose=False)
    lib = ctypes.CDLL(LIB)
    names = _declared()
    assert {"sd_create", "sd_destroy", "sd_prefill", "specdec_round", "specdec_generate",
            "sd_accept_resample", "sd_gemm_skinny", "sd_forward"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_covers_the_header():
    from paper_2405_19715_amd import binding
    assert sorted(binding.EXPORTS) == _declared()


def test_host_side_argument_checks_need_no_gpu():
    from paper_2405_19715_amd import binding as B
    assert B.lib.sd_strerror(B.SD_ERANGE).decode().startswith("sequence")
    assert B.lib.sd_destroy(None) == B.SD_EINVAL
    assert B.lib.sd_create(None, None, None, None, None) == B.SD_EINVAL
    h = ctypes.c_void_p()
    assert B.lib.sd_create(ctypes.byref(h), None, None, None, ctypes.byref(B.sd_config(1, 64, 4, None))) == B.SD_EINVAL
    assert B.lib.sd_accept_workspace_bytes(4, 16) == 4 * 33 * 16 + 16
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 17, 8192, 8192) % (17 * 8192 * 4) == 0
    assert B.lib.sd_gemm_workspace_bytes(B.SD_BF16, 500, 8192, 8192) == 0
    # the gated activation's one-launch kernel: up to 8 rows with K a multiple of 2048 up to 8192, 9 .. 17 rows
    # with K a multiple of 512
    assert B.lib.sd_mlp_act_is_fused(B.SD_BF16, 1, 28672, 8192) == 1
    assert B.lib.sd_mlp_act_is_fused(B.SD_BF16, 8, 11008, 4096) == 1
    assert B.lib.sd_mlp_act_is_fused(B.SD_BF16, 9, 28672, 8192) == 1
    assert B.lib.sd_mlp_act_is_fused(B.SD_BF16, 17, 28672, 8192) == 1
    assert B.lib.sd_mlp_act_is_fused(B.SD_BF16, 18, 28672, 8192) == 0
    assert B.lib.sd_mlp_act_is_fused(B.SD_BF16, 12, 28672, 8192 + 128) == 0
    assert B.lib.sd_mlp_act_is_fused(B.SD_BF16, 4, 512, 16384) == 0
    assert B.lib.sd_mlp_act_is_fused(B.SD_F32, 1, 688, 256) == 0
    assert B.lib.sd_mlp_act(B.SD_BF16, None, None, 1, 8, 128, None, None, -1, None) == B.SD_EINVAL
    # the q|k|v product that rotates and appends: the same row limits, head dimension a power of two
    assert B.lib.sd_qkv_rope_is_fused(B.SD_BF16, 8, 64, 8, 128, 8192) == 1
    assert B.lib.sd_qkv_rope_is_fused(B.SD_BF16, 1, 32, 32, 128, 4096) == 1
    assert B.lib.sd_qkv_rope_is_fused(B.SD_BF16, 9, 64, 8, 128, 8192) == 1
    assert B.lib.sd_qkv_rope_is_fused(B.SD_BF16, 17, 64, 8, 128, 8192) == 1
    assert B.lib.sd_qkv_rope_is_fused(B.SD_BF16, 18, 64, 8, 128, 8192) == 0
    assert B.lib.sd_qkv_rope_is_fused(B.SD_BF16, 2, 8, 2, 96, 2048) == 0
    assert B.lib.sd_qkv_rope_is_fused(B.SD_BF16, 2, 8, 2, 64, 1024) == 0
    assert B.lib.sd_qkv_rope_is_fused(B.SD_F32, 2, 8, 2, 64, 2048) == 0
    assert B.lib.sd_qkv_rope(B.SD_BF16, None, None, 1, 8, 2, 64, 2048, None, None, None, None, None, None, 64, None,
                             -1, None) == B.SD_EINVAL
    assert B.lib.sd_version().decode().startswith("specdec")
