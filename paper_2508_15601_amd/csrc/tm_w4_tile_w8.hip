// CTA-tile kernels instantiated for the 8-bit weight formats (integer codes and FP8 E4M3): the same body with two packed
// words per MFMA step and packed units of 64 rows.  Three tile shapes with one or two wave sets (four on the 32-row
// tile), built like the small 4-bit tiles.
#include "tm_w4_tile_impl.h"

namespace tmw4 {

namespace {

template <int FMT>
hipError_t launch_fmt(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    // one, two or four wave sets per CTA (each set multiplies its own slice of every K stage), as for the 4-bit tiles
    if (plan.kgroups == 2) {
        switch (plan.variant) {
            case kTile32x128: return launch_shape<2, 2, 4, 4, 2, FMT>(p, plan, group, stream);
            case kTile64x128: return launch_shape<4, 2, 4, 4, 2, FMT>(p, plan, group, stream);
            case kTile128x256: return launch_shape<8, 4, 4, 2, 2, FMT>(p, plan, group, stream);
            default: return hipErrorInvalidValue;
        }
    }
    if (plan.kgroups == 4) {
        switch (plan.variant) {
            case kTile32x128: return launch_shape<2, 2, 4, 4, 4, FMT>(p, plan, group, stream);
            default: return hipErrorInvalidValue;
        }
    }
    switch (plan.variant) {
        case kTile32x128: return launch_shape<2, 2, 4, 4, 1, FMT>(p, plan, group, stream);
        case kTile64x128: return launch_shape<4, 2, 4, 4, 1, FMT>(p, plan, group, stream);
        case kTile128x256: return launch_shape<8, 4, 4, 2, 1, FMT>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_tile_8bit(const GemmParams& p, const Plan& plan, int group, bool fp8, hipStream_t stream)
{
    return fp8 ? launch_fmt<kFmtFp8>(p, plan, group, stream) : launch_fmt<kFmtInt8>(p, plan, group, stream);
}

}  // namespace tmw4
