// Host-side declarations shared by the translation units of libtm_w4: kernel launchers and the plan record.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tm_w4_device.h"

namespace tmw4 {

// Kernel variants the dispatcher can choose from (ids are what tm_set_variant / tm_get_plan use).
enum Variant {
    kSkinny16x16 = 0,   // M <= 16, one 16-column tile per wave: weights streamed straight into B-operand registers
    kSkinny16x32 = 1,   // M <= 16, two 16-column tiles per wave
    kSkinny16x64 = 2,   // M <= 16, four
    kSkinny32x32 = 3,   // M <= 32, two
    kSkinny32x64 = 4,   // M <= 32, four
    kTile32x256 = 5,    // CTA tiles, X staged through LDS
    kTile64x256 = 6,
    kTile128x256 = 7,
    kTile256x256 = 8,
    kTile64x128 = 9,
    kTile128x128 = 10,
    kTile192x256 = 11,
    kTile128x512 = 12,
    kTile32x128 = 13,
    kSkinny16x48 = 14,  // M <= 16, up to three / six / eight 16-column tiles per wave
    kSkinny16x96 = 15,
    kSkinny16x128 = 16,
    kSkinny64x32 = 17,  // M <= 64, two / three / four tiles per wave, conversion on the ALU
    kSkinny64x48 = 18,
    kSkinny64x64 = 19,
    kTile32x96 = 20,    // CTA tiles of two waves x three 16-column tiles, always with several wave sets per CTA
    kTile64x96 = 21,
    kTile64x64 = 22,    // CTA tiles of two waves x two 16-column tiles, with several wave sets per CTA: more rows per
    kTile128x64 = 23,   // converted fragment where a wider tile would leave compute units without a CTA
    kNumVariants = 24
};
inline bool is_skinny(int v) { return v <= kSkinny32x64 || (v >= kSkinny16x48 && v <= kSkinny64x64); }
inline int skinny_rows(int v) { return (v == kSkinny32x32 || v == kSkinny32x64) ? 32 : (v >= kSkinny64x32 && v <= kSkinny64x64) ? 64 : 16; }
// widest strip (in 16-column tiles) a skinny variant can take; narrower strips run with the surplus tiles idle
inline int skinny_ntw(int v)
{
    switch (v) {
        case kSkinny16x16: return 1;
        case kSkinny16x32: case kSkinny32x32: case kSkinny64x32: return 2;
        case kSkinny16x48: case kSkinny64x48: return 3;
        case kSkinny16x64: case kSkinny32x64: case kSkinny64x64: return 4;
        case kSkinny16x96: return 6;
        default: return 8;
    }
}
inline int tile_bm(int v) { return (v == kTile32x256 || v == kTile32x128 || v == kTile32x96) ? 32 : ((v == kTile64x256 || v == kTile64x128 || v == kTile64x96 || v == kTile64x64) ? 64 : ((v == kTile128x256 || v == kTile128x128 || v == kTile128x512 || v == kTile128x64) ? 128 : (v == kTile192x256 ? 192 : 256))); }
inline bool tile_two_waves(int v) { return v == kTile32x96 || v == kTile64x96 || v == kTile64x64 || v == kTile128x64; }
inline int tile_threads(int v) { return v == kTile128x512 ? 512 : tile_two_waves(v) ? 128 : 256; }     // of one wave set
// wave sets per CTA (in-CTA split of every K stage) a tile variant is built with, besides 1
inline bool tile_has_kgroups(int v, int kg)
{
    if (tile_two_waves(v)) return kg == 2 || kg == 4;
    return kg == 1 || (kg == 2 && (v == kTile32x128 || v == kTile64x128 || v == kTile128x128 || v == kTile128x256)) || (kg == 4 && (v == kTile32x128 || v == kTile64x128));
}
inline int tile_bn(int v) { return (v == kTile64x64 || v == kTile128x64) ? 64 : (v == kTile32x96 || v == kTile64x96) ? 96 : (v == kTile64x128 || v == kTile128x128 || v == kTile32x128) ? 128 : (v == kTile128x512 ? 512 : 256); }

struct Plan {
    int variant;
    int split;
    int ku_per_split;
    int strips;           // skinny kernels: number of column strips the 16-column tiles are dealt into
    int stage_steps;      // tile kernels: MFMA steps (32 rows of K each) per pipeline stage and wave set: 2, 4 or 8
    int kgroups;          // tile kernels: sets of four waves per CTA, each taking its own slice of every stage
    int stream_ni;        // decode kernels: > 0 = the one-shot kernel with this many packed units per wave (the form
                          // with a ring of X pieces when M > 16)
    int mfma32;           // tile kernels: 1 = the launch runs on the 32x32x16 matrix instruction (tm_w4_tile32.hip)
    int tiles_m, tiles_n;
    unsigned grid;
    unsigned block;
    size_t ws_bytes;      // counters + partial sums
};

hipError_t launch_repack(const uint32_t* qweight, const uint16_t* scales, const void* zeros, uint32_t* w_out,
                         uint32_t* sz_out, int K, int N, int group, int layout, hipStream_t stream);
hipError_t launch_repack8(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros, uint32_t* w_out,
                          uint32_t* sz_out, int K, int N, int group, bool fp8, hipStream_t stream);
hipError_t launch_permute_rows(const uint32_t* in, const int32_t* perm, uint32_t* out, int K, int N, int k_major,
                               hipStream_t stream);
hipError_t launch_permute_x(const uint16_t* X, const int32_t* perm, uint16_t* out, int M, int K, hipStream_t stream);
hipError_t launch_interleave_gate_up(const uint32_t* q, const uint16_t* s, const uint16_t* z, uint32_t* q_out, uint16_t* s_out,
                                     uint16_t* z_out, int K, int N, int G, hipStream_t stream);
hipError_t launch_unpack(const uint32_t* w, const uint32_t* sz, uint32_t* qweight_out, uint16_t* scales_out,
                         uint16_t* zeros_out, int K, int N, int group, hipStream_t stream);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);
hipError_t launch_read(const void* src, size_t bytes, void* sink, hipStream_t stream);
hipError_t launch_clock_probe(void* out, uint32_t delay, uint32_t ticks, int max_rounds, hipStream_t stream);
hipError_t launch_mfma_loop(void* out, unsigned grid, unsigned block, int iters, int pattern, hipStream_t stream);
hipError_t launch_read_shape(const void* src, size_t bytes, void* sink, unsigned grid, unsigned block, int unroll, int flags,
                             hipStream_t stream);

hipError_t launch_kv_append(const AttnCache& kv, const uint16_t* Kn, const uint16_t* Vn, const int32_t* positions,
                            int count, hipStream_t stream);
hipError_t launch_attn_decode(const AttnCache& kv, const uint16_t* Q, const int32_t* lens, uint16_t* O, int q_heads,
                              float scale, int max_len, int num_cu, hipStream_t stream);
hipError_t launch_attn_prefill(const AttnCache& kv, const uint16_t* Q, const int32_t* positions, const int32_t* counts,
                               int count, uint16_t* O, int q_heads, float scale, hipStream_t stream);
hipError_t launch_skinny(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t launch_stream(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t stream_setup();                                             // once per device, outside any capture
hipError_t stream_grouped_setup();                                     // the same for the grouped form
hipError_t launch_stream_grouped(const GroupedParams& gp, int experts, int group, int ni, int block, hipStream_t stream);
int stream_units_per_wave(int ntw, int group, int kus, int waves);     // 0: no one-shot kernel is built for this shape
constexpr size_t kStreamLdsBudget = 156 * 1024;                       // of the 160 KiB of a CU
size_t stream_lds(int ni, int mp_log, int ntw, int waves, int* red_off);
hipError_t launch_rows(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);      // 16 < M <= 64
hipError_t launch_rows32(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t launch_rows64(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
int rows_units_per_wave(int M, int ntw, int group, int kus, int waves);        // 0: no such kernel is built for this shape
hipError_t launch_skinny_w8(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t launch_skinny_f8(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t launch_skinny_grouped(const GroupedParams& gp, int variant, int experts, int group, hipStream_t stream);
hipError_t launch_tile_8bit(const GemmParams& p, const Plan& plan, int group, bool fp8, hipStream_t stream);
hipError_t launch_tile_grouped(const GroupedParams& gp, int variant, int experts, int group, hipStream_t stream);
hipError_t launch_skinny_grouped_w8(const GroupedParams& gp, int variant, int experts, int group, hipStream_t stream);
hipError_t launch_skinny_grouped_f8(const GroupedParams& gp, int variant, int experts, int group, hipStream_t stream);
hipError_t launch_tile_grouped_8bit(const GroupedParams& gp, int variant, int experts, int group, bool fp8, hipStream_t stream);
hipError_t launch_tile(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t launch_tile32(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t launch_tile_small(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t launch_tile_large(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t launch_tile_kgroup(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);

}  // namespace tmw4
