"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares, and its argument
validation returns error codes (never aborts).  No compute call is made."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include")))
                   if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tm_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    import paper_2508_15601_amd as tm
    if not os.path.exists(tm.lib_path()):
        from paper_2508_15601_amd import build
        build.build()
    return tm.load_library()


def test_header_symbols_are_exported(lib):
    names = _declared_symbols()
    assert "tm_pack_w4" in names and "tm_gemm_w4a16" in names and len(names) >= 15
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/tm_w4.h but not exported"


def test_binding_uses_same_names():
    import paper_2508_15601_amd as tm
    for n in ("tm_pack_w4", "tm_pack_w4_layout", "tm_pack_w8", "tm_group_experts", "tm_gemm_w4a16_grouped", "tm_gemm_w4a16", "tm_gemm_w4a16_ws", "tm_unpack_w4", "tm_packed_raw", "tm_get_plan",
              "tm_set_variant", "tm_gemm_workspace_bytes", "tm_last_error", "tm_version"):
        assert callable(getattr(tm, n))


def test_argument_validation_without_gpu(lib):
    import paper_2508_15601_amd as tm
    assert lib.tm_pack_w4(None, None, None, 128, 16, 128) is None
    assert "null" in tm.tm_last_error()
    fake = ctypes.c_void_p(4096)
    for (K, N, g) in [(100, 16, 128), (128, 24, 128), (128, 16, 48), (0, 16, 128), (128, -16, 128)]:
        assert lib.tm_pack_w4(fake, fake, fake, K, N, g) is None
        assert tm.tm_last_error()
    assert lib.tm_pack_w4(ctypes.c_void_p(4097), fake, fake, 128, 16, 128) is None
    assert "misaligned" in tm.tm_last_error()
    lib.tm_pack_w4_layout.restype = ctypes.c_void_p
    lib.tm_pack_w4_layout.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 4 + [ctypes.c_void_p]
    assert lib.tm_pack_w4_layout(fake, fake, fake, 128, 16, 128, 3, None) is None
    assert "layout" in tm.tm_last_error()
    assert lib.tm_pack_w4_layout(fake, None, fake, 128, 16, 128, 2, None) is None
    assert "null" in tm.tm_last_error()
    assert lib.tm_pack_w4_layout(fake, fake, None, 256, 16, 192, 0, None) is None       # 192 is no multiple of 128
    assert "group" in tm.tm_last_error()
    assert lib.tm_pack_w4_layout(fake, fake, None, 384, 16, 256, 0, None) is None       # 256 does not divide 384
    assert "group" in tm.tm_last_error()
    assert lib.tm_pack_w4_layout(fake, fake, ctypes.c_void_p(4098), 128, 16, 128, 1, None) is None    # u32 zeros
    assert "misaligned" in tm.tm_last_error()
    assert lib.tm_gemm_w4a16(fake, None, fake, 1, None) == -1
    assert lib.tm_pack_w8(fake, None, fake, 128, 16, 128, None) is None and "null" in tm.tm_last_error()
    assert lib.tm_pack_w8(fake, fake, None, 128, 16, 96, None) is None and "group" in tm.tm_last_error()
    assert lib.tm_pack_w8_fp8(fake, None, 128, 16, 128, None) is None and "null" in tm.tm_last_error()
    lib.tm_pack_w4_actorder.restype = ctypes.c_void_p
    lib.tm_pack_w4_actorder.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 4 + [ctypes.c_void_p]
    assert lib.tm_pack_w4_actorder(fake, fake, fake, None, 128, 16, 128, 2, None) is None and "g_idx" in tm.tm_last_error()
    assert lib.tm_pack_w4_actorder(fake, fake, fake, fake, 128, 16, 100, 2, None) is None and "group" in tm.tm_last_error()
    assert lib.tm_packed_bits(None) == -1
    assert lib.tm_kv_create(0, 1, 32, 8) is None and lib.tm_kv_create(1, 1, 32, 4) is None
    assert lib.tm_kv_append(None, fake, fake, fake, 1, None) == -1
    assert lib.tm_attn_decode(fake, None, fake, fake, 8, 0.1, 0, None) == -1
    assert lib.tm_attn_prefill(fake, None, fake, None, 4, fake, 8, ctypes.c_float(0.1), None) == -1
    assert lib.tm_kv_raw(None, None, None, None, None, None) == -1
    lib.tm_kv_free(None)
    assert lib.tm_group_experts(None, 2) is None and lib.tm_group_experts(fake, 0) is None
    assert lib.tm_gemm_w4a16_grouped(fake, None, fake, fake, 4, None) == -1
    assert lib.tm_get_grouped_plan(None, 4, None, None) == -1
    lib.tm_free_expert_group(None)
    assert lib.tm_gemm_workspace_bytes(None, 4) == 0
    assert lib.tm_get_plan_units_per_wave(None, 1) == -1
    assert lib.tm_gemm_w4a16_static(fake, None, fake, 1, None) == -1
    assert lib.tm_reset_workspace(ctypes.c_void_p(4097), None) != 0
    assert lib.tm_packed_info(None, None, None, None, None) == -1
    assert lib.tm_unpack_w4(None, None, None, None, None) == -1
    assert lib.tm_get_plan(None, 1, None, None, None, None) == -1
    lib.tm_free_packed(None)                      # must be a no-op
    assert lib.tm_set_variant(99, 0) == -1 and lib.tm_set_variant(-1, 0) == 0
    assert lib.tm_variant_name(0) == b"skinny16x16" and lib.tm_variant_name(99) == b""
    assert lib.tm_set_launch(5, 0) == -1 and lib.tm_set_launch(0, 3) == -1 and lib.tm_set_launch(0, 0) == 0
    assert lib.tm_set_mfma_shape(8) == -1 and lib.tm_set_mfma_shape(0) == 0 and lib.tm_get_plan_mfma_shape(None, 1) == -1
    assert lib.tm_bench_copy(None, None, 16, None) == -1
    assert lib.tm_bench_mfma(None, 256, 256, 10, 1, None) == -1 and lib.tm_bench_clock(None, 0, 100, None) == -1
    assert tm.tm_version().startswith("tm_w4")


def test_product_package_does_not_touch_the_oracle():
    """The product path must not import, link or read anything under oracle/."""
    pkg = os.path.join(ROOT, "paper_2508_15601_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no fallback", ""), f"{f} mentions the oracle"
