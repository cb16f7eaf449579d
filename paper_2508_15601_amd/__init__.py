"""MI355X-native W4A16 GEMM (offline fragment-order packing + fused dequantise-and-multiply).

Thin binding over the C ABI of ``libtm_w4.so`` (declared in ``include/tm_w4.h``): argument marshalling only;
every step of the method runs in the library's HIP kernels.  PyTorch supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    KvCache, tm_attn_decode, tm_attn_prefill, tm_bench_copy_raw, tm_kv_append, tm_kv_create, tm_kv_download, tm_kv_raw, tm_kv_upload,
    ExpertGroup, PackedW4, TM_LAYOUT_K8, TM_LAYOUT_N8, TM_LAYOUT_N8_INTERLEAVED, TM_READ_NONTEMPORAL, TM_READ_CHUNKED, TM_READ_SHARED, TmError, lib_path, load_library, tm_bench_copy, tm_bench_read, tm_bench_read_shape, tm_bench_mfma, tm_bench_clock, tm_set_mfma_shape, tm_gemm_w4a16, tm_gemm_w4a16_static, tm_gemm_w4a16_ex, tm_pack_w4_gate_up, TM_ACT_NONE, TM_ACT_SILU_MUL, tm_gemm_w4a16_grouped, tm_gemm_w4a16_grouped_act, tm_gemm_w4a16_ws, tm_get_grouped_plan, tm_group_experts,
    tm_gemm_workspace_bytes, tm_reset_workspace, tm_get_plan, tm_last_error, tm_pack_w4, tm_pack_w4_actorder, tm_pack_w4_layout, tm_pack_w8, tm_pack_w8_fp8, tm_packed_raw, tm_set_variant, tm_set_launch, tm_unpack_w4,
    tm_variant_name, tm_version,
)
