// The decode kernels instantiated for 8-bit weight codes (W8A16): same pipeline, packed units of 64 rows, byte-permute
// conversion.  Only the strip widths the dispatcher uses for this format are built.
#include "tm_w4_skinny_impl.h"

namespace tmw4 {

hipError_t launch_skinny_w8(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    const bool w16 = plan.block > 512;
    switch (plan.variant) {
        case kSkinny16x16: return w16 ? launch_cfg<1, 1, 3, 2, 16, 8>(p, plan, group, stream) : launch_cfg<1, 1, 4, 4, 8, 8>(p, plan, group, stream);
        case kSkinny16x32: return w16 ? launch_cfg<1, 2, 2, 2, 16, 8>(p, plan, group, stream) : launch_cfg<1, 2, 4, 4, 8, 8>(p, plan, group, stream);
        case kSkinny16x48: return w16 ? launch_cfg<1, 3, 2, 2, 16, 8>(p, plan, group, stream) : launch_cfg<1, 3, 3, 3, 8, 8>(p, plan, group, stream);
        case kSkinny16x64: return w16 ? launch_cfg<1, 4, 2, 1, 16, 8>(p, plan, group, stream) : launch_cfg<1, 4, 2, 2, 8, 8>(p, plan, group, stream);
        case kSkinny16x96: return w16 ? launch_cfg<1, 6, 1, 1, 16, 8>(p, plan, group, stream) : launch_cfg<1, 6, 3, 2, 8, 8>(p, plan, group, stream);
        case kSkinny16x128: return w16 ? launch_cfg<1, 8, 1, 1, 16, 8>(p, plan, group, stream) : launch_cfg<1, 8, 2, 2, 8, 8>(p, plan, group, stream);
        case kSkinny32x64: return w16 ? hipErrorInvalidValue : launch_cfg<2, 4, 2, 2, 8, 8>(p, plan, group, stream);
        case kSkinny64x64: return w16 ? hipErrorInvalidValue : launch_cfg<4, 4, 2, 1, 8, 8>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
