// The 256 x 256 CTA-tile kernel of the compute-bound (prefill) regime: 256 fp32 accumulators per lane, which only
// fit with the accumulation registers (AGPRs) holding them, one wave per SIMD.
#include "tm_w4_tile_impl.h"

namespace tmw4 {

hipError_t launch_tile_large(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    switch (plan.variant) {
        case kTile256x256: return launch_shape<16, 4, 4, 2>(p, plan, group, stream);
        case kTile192x256: return launch_shape<12, 4, 4, 2>(p, plan, group, stream);
        // eight waves of 128 x 64: one CTA per CU, the X stage loaded once for 512 columns
        case kTile128x512: return launch_shape<8, 4, 8, 2>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_tile(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    if (plan.mfma32) return launch_tile32(p, plan, group, stream);
    if (plan.kgroups > 1) return launch_tile_kgroup(p, plan, group, stream);
    return (plan.variant == kTile256x256 || plan.variant == kTile192x256 || plan.variant == kTile128x512) ? launch_tile_large(p, plan, group, stream)
                                        : launch_tile_small(p, plan, group, stream);
}

}  // namespace tmw4
