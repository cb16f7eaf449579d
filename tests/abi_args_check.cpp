// Argument validation of the C ABI, run as a plain executable so that the host code of the library can be built with the
// address and undefined-behaviour sanitizers (tests/test_sanitizers.py builds and runs it; no GPU is needed: every call
// here must be refused before anything is launched or dereferenced).  Exit status 0 = every call answered as expected.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "tm_attn.h"
#include "tm_w4.h"

static int failures = 0;
#define CHECK(cond)                                                                   \
    do {                                                                              \
        if (!(cond)) {                                                                \
            fprintf(stderr, "abi_args_check: line %d: %s (last error: %s)\n", __LINE__, #cond, tm_last_error()); \
            ++failures;                                                               \
        }                                                                             \
    } while (0)

int main()
{
    const uint32_t* fake32 = (const uint32_t*)(uintptr_t)4096;      // never dereferenced by the host code
    const uint16_t* fake16 = (const uint16_t*)(uintptr_t)4096;
    uint16_t* out16 = (uint16_t*)(uintptr_t)8192;
    CHECK(tm_pack_w4(nullptr, nullptr, nullptr, 128, 16, 128) == nullptr && strstr(tm_last_error(), "null"));
    const int bad[][3] = {{100, 16, 128}, {128, 24, 128}, {128, 16, 48}, {0, 16, 128}, {128, -16, 128}, {256, 16, 192}, {384, 16, 256}};
    for (const auto& b : bad) {
        CHECK(tm_pack_w4(fake32, fake16, fake16, b[0], b[1], b[2]) == nullptr && tm_last_error()[0]);
        CHECK(tm_pack_w8(fake32, fake16, fake16, b[0], b[1], b[2], nullptr) == nullptr);
        CHECK(tm_pack_w8_fp8(fake32, fake16, b[0], b[1], b[2], nullptr) == nullptr);
        CHECK(tm_pack_w4_gate_up(fake32, fake16, fake16, b[0], b[1], b[2], nullptr) == nullptr);
    }
    CHECK(tm_pack_w4((const uint32_t*)(uintptr_t)4097, fake16, fake16, 128, 16, 128) == nullptr && strstr(tm_last_error(), "misaligned"));
    CHECK(tm_pack_w4_layout(fake32, fake16, fake16, 128, 16, 128, 3, nullptr) == nullptr && strstr(tm_last_error(), "layout"));
    CHECK(tm_pack_w4_layout(fake32, nullptr, fake16, 128, 16, 128, 2, nullptr) == nullptr && strstr(tm_last_error(), "null"));
    CHECK(tm_pack_w4_layout(fake32, fake16, (const void*)(uintptr_t)4098, 128, 16, 128, 1, nullptr) == nullptr);
    CHECK(tm_pack_w4_actorder(fake32, fake16, fake16, nullptr, 128, 16, 128, 2, nullptr) == nullptr && strstr(tm_last_error(), "g_idx"));
    CHECK(tm_pack_w4_actorder(fake32, fake16, fake16, (const int32_t*)fake32, 128, 16, 100, 2, nullptr) == nullptr);
    CHECK(tm_pack_w4_gate_up(fake32, fake16, fake16, 128, 48, 128, nullptr) == nullptr);        // N % 32
    CHECK(tm_gemm_w4a16(fake16, nullptr, out16, 1, nullptr) == TM_EINVAL);
    CHECK(tm_gemm_w4a16_ex(fake16, nullptr, out16, 1, nullptr, nullptr) == TM_EINVAL);
    CHECK(tm_gemm_w4a16_ws(fake16, nullptr, out16, 1, out16, 1 << 20, nullptr) == TM_EINVAL);
    CHECK(tm_gemm_w4a16_static(fake16, nullptr, out16, 1, nullptr) == TM_EINVAL);
    // a block of bytes that is not a handle (wrong magic) is refused, not followed
    alignas(16) unsigned char not_a_handle[256];
    memset(not_a_handle, 0x5A, sizeof(not_a_handle));
    CHECK(tm_gemm_w4a16(fake16, (const tm_packed_w4*)not_a_handle, out16, 1, nullptr) == TM_EINVAL);
    CHECK(tm_packed_info((const tm_packed_w4*)not_a_handle, nullptr, nullptr, nullptr, nullptr) == TM_EINVAL);
    CHECK(tm_get_plan((const tm_packed_w4*)not_a_handle, 4, nullptr, nullptr, nullptr, nullptr) == TM_EINVAL);
    tm_free_packed((tm_packed_w4*)not_a_handle);
    tm_free_expert_group((tm_expert_group*)not_a_handle);
    tm_kv_free((tm_kv_cache*)not_a_handle);
    CHECK(tm_gemm_workspace_bytes(nullptr, 4) == 0);
    CHECK(tm_get_plan_units_per_wave(nullptr, 1) == TM_EINVAL);
    CHECK(tm_reset_workspace((void*)(uintptr_t)4097, nullptr) != TM_OK);
    CHECK(tm_packed_bits(nullptr) == TM_EINVAL && tm_packed_info(nullptr, nullptr, nullptr, nullptr, nullptr) == TM_EINVAL);
    CHECK(tm_unpack_w4(nullptr, nullptr, nullptr, nullptr, nullptr) == TM_EINVAL);
    CHECK(tm_packed_raw(nullptr, nullptr, nullptr, nullptr, nullptr) == TM_EINVAL);
    CHECK(tm_get_plan(nullptr, 1, nullptr, nullptr, nullptr, nullptr) == TM_EINVAL);
    tm_free_packed(nullptr);
    CHECK(tm_group_experts(nullptr, 2) == nullptr);
    const tm_packed_w4* none[2] = {nullptr, nullptr};
    CHECK(tm_group_experts(none, 0) == nullptr && tm_group_experts(none, 2) == nullptr && tm_group_experts(none, 70000) == nullptr);
    CHECK(tm_gemm_w4a16_grouped(fake16, nullptr, (const int32_t*)fake32, out16, 4, nullptr) == TM_EINVAL);
    CHECK(tm_gemm_w4a16_grouped_act(fake16, nullptr, (const int32_t*)fake32, out16, 4, 1, nullptr) == TM_EINVAL);
    CHECK(tm_get_grouped_plan(nullptr, 4, nullptr, nullptr) == TM_EINVAL);
    tm_free_expert_group(nullptr);
    CHECK(tm_set_variant(99, 0) == TM_EINVAL && tm_set_variant(-2, 0) == TM_EINVAL && tm_set_variant(0, 1000) == TM_EINVAL);
    CHECK(tm_set_variant(-1, 0) == TM_OK);
    CHECK(tm_set_launch(5, 0) == TM_EINVAL && tm_set_launch(0, 3) == TM_EINVAL && tm_set_launch(0, 0) == TM_OK);
    CHECK(strcmp(tm_variant_name(0), "skinny16x16") == 0 && tm_variant_name(99)[0] == 0 && tm_variant_name(-1)[0] == 0);
    CHECK(tm_bench_copy(nullptr, nullptr, 16, nullptr) == TM_EINVAL && tm_bench_copy(out16, fake16, 24, nullptr) == TM_EINVAL);
    CHECK(tm_bench_read(nullptr, 16, nullptr, nullptr) == TM_EINVAL);
    CHECK(tm_bench_read_shape(fake16, 16, out16, 0, 256, 1, 0, nullptr) == TM_EINVAL);
    CHECK(tm_bench_read_shape(fake16, 16, out16, 1, 100, 1, 0, nullptr) == TM_EINVAL);
    CHECK(tm_bench_read_shape(fake16, 16, out16, 1, 256, 3, 0, nullptr) == TM_EINVAL);
    CHECK(tm_bench_read_shape(fake16, 16, out16, 1, 256, 1, 8, nullptr) == TM_EINVAL);
    CHECK(tm_kv_create(0, 1, 32, 8) == nullptr && tm_kv_create(1, 1, 32, 5) == nullptr && tm_kv_create(1, 70000, 32, 8) == nullptr);
    CHECK(tm_kv_create(1, 1, 1 << 30, 8) == nullptr);
    CHECK(tm_kv_append(nullptr, fake16, fake16, (const int32_t*)fake32, 1, nullptr) == TM_EINVAL);
    CHECK(tm_attn_decode(fake16, nullptr, (const int32_t*)fake32, out16, 8, 0.1f, 0, nullptr) == TM_EINVAL);
    CHECK(tm_attn_prefill(fake16, nullptr, (const int32_t*)fake32, nullptr, 4, out16, 8, 0.1f, nullptr) == TM_EINVAL);
    CHECK(tm_kv_raw(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == TM_EINVAL);
    tm_kv_free(nullptr);
    CHECK(strncmp(tm_version(), "tm_w4", 5) == 0);
    if (failures) {
        fprintf(stderr, "abi_args_check: %d check(s) failed\n", failures);
        return 1;
    }
    printf("abi_args_check: all checks passed\n");
    return 0;
}
