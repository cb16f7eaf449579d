// CTA-tile kernels with at most 128 accumulator registers per lane (tiles up to 128 rows).  Built with the MFMA
// accumulators kept in ordinary vector registers (-mllvm -amdgpu-mfma-vgpr-form=1): at this size that avoids the
// copies between the two register files the default allocation inserts into the K loop.
#include "tm_w4_tile_impl.h"

namespace tmw4 {

hipError_t launch_tile_small(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    switch (plan.variant) {
        case kTile32x256: return launch_shape<2, 4>(p, plan, group, stream);
        case kTile64x256: return launch_shape<4, 4>(p, plan, group, stream);
        case kTile128x256: return launch_shape<8, 4>(p, plan, group, stream);
        case kTile64x128: return launch_shape<4, 2>(p, plan, group, stream);
        case kTile128x128: return launch_shape<8, 2>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
