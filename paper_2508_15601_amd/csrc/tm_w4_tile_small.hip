// CTA-tile kernels with at most 128 accumulator registers per lane (tiles up to 128 rows).  Built with the MFMA
// accumulators kept in ordinary vector registers (-mllvm -amdgpu-mfma-vgpr-form=1): at this size that avoids the
// copies between the two register files the default allocation inserts into the K loop.
#include "tm_w4_tile_impl.h"

namespace tmw4 {

namespace {

// All variants are four waves wide.  Measured on the mid-M shapes, a 128-column CTA tile made of four waves of 32
// columns beats one made of two waves of 64 columns: at these sizes the number of waves in flight matters more
// than the LDS traffic per MFMA.
template <int TM, int TN>
hipError_t launch_depth(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    switch (plan.stage_steps) {
        case 2: return launch_shape<TM, TN, 4, 2>(p, plan, group, stream);
        case 4:
            // the 128 x 256 tile has no registers left for 128-deep stages
            if constexpr (!(TM == 8 && TN == 4)) return launch_shape<TM, TN, 4, 4>(p, plan, group, stream);
            return hipErrorInvalidValue;
        case 8:
            if constexpr (TM <= 4) return launch_shape<TM, TN, 4, 8>(p, plan, group, stream);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_tile_small(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    switch (plan.variant) {
        case kTile32x256: return launch_depth<2, 4>(p, plan, group, stream);
        case kTile64x256: return launch_depth<4, 4>(p, plan, group, stream);
        case kTile128x256: return launch_depth<8, 4>(p, plan, group, stream);
        case kTile32x128: return launch_depth<2, 2>(p, plan, group, stream);
        case kTile64x128: return launch_depth<4, 2>(p, plan, group, stream);
        case kTile128x128: return launch_depth<8, 2>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
