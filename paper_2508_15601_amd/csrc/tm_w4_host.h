// Host-side declarations shared by the translation units of libtm_w4: kernel launchers and the plan record.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tm_w4_device.h"

namespace tmw4 {

// Kernel variants the dispatcher can choose from (ids are what tm_set_variant / tm_get_plan use).
enum Variant {
    kSkinny16 = 0,    // M <= 16: one 16-row MFMA tile, weights streamed straight into B-operand registers
    kSkinny32 = 1,    // M <= 32
    kSkinny64 = 2,    // M <= 64
    kTile128 = 3,     // 128 x 128 CTA tile, X staged through LDS
    kTile256 = 4,     // 256 x 256 CTA tile, X staged through LDS
    kNumVariants = 5
};

struct Plan {
    int variant;
    int split;
    int ku_per_split;
    int tiles_m, tiles_n;
    unsigned grid;
    unsigned block;
    size_t ws_bytes;      // counters + partial sums
};

hipError_t launch_repack(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros, uint32_t* w_out,
                         uint32_t* sz_out, int K, int N, int group, hipStream_t stream);
hipError_t launch_unpack(const uint32_t* w, const uint32_t* sz, uint32_t* qweight_out, uint16_t* scales_out,
                         uint16_t* zeros_out, int K, int N, int group, hipStream_t stream);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);
hipError_t launch_read(const void* src, size_t bytes, void* sink, hipStream_t stream);

hipError_t launch_skinny(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);
hipError_t launch_tile(const GemmParams& p, const Plan& plan, int group, hipStream_t stream);

}  // namespace tmw4
