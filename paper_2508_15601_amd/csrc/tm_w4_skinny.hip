// Fused dequantise-and-multiply for the decode shapes (M <= 64): the HBM-bound regime.
//
// Online stage of the GEMM pipeline (paper Sec. 3.1 steps (i)-(iv), Sec. 4.3).  What differs from the paper's
// design, which stages weights through shared memory for a 32-lane tensor-core fragment load:
//   - the packed buffer is already in matrix-core operand order, so a wave's 128-bit load of one 1 KiB unit lands
//     directly in the B-operand registers of four MFMAs; weights never touch LDS;
//   - every wave issues all weight, scale/zero and activation loads of a batch of units before the first
//     conversion, which is what the memory pipeline depth of the paper's loop achieves with asynchronous copies;
//   - a CTA is 8 or 16 waves that split the K range of one strip of NTW 16-column tiles; their partial tiles meet
//     in LDS.  Only when a shape has too few strips to fill the chip do CTAs also split K among themselves; those
//     partial sums meet in an fp32 workspace that the last-arriving CTA adds in fixed order.
#include "tm_w4_skinny_impl.h"

namespace tmw4 {

hipError_t launch_skinny_grouped(const GroupedParams& gp, int variant, int experts, int group, hipStream_t stream)
{
    return launch_skinny_grouped_fmt<4>(gp, variant, experts, group, stream);
}

hipError_t launch_skinny(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    const bool w16 = plan.block > 512;
    switch (plan.variant) {
        case kSkinny16x16: return w16 ? launch_cfg<1, 1, 3, 2, 16>(p, plan, group, stream) : launch_cfg<1, 1, 4, 4, 8>(p, plan, group, stream);
        case kSkinny16x32: return w16 ? launch_cfg<1, 2, 2, 2, 16>(p, plan, group, stream) : launch_cfg<1, 2, 4, 4, 8>(p, plan, group, stream);
        case kSkinny16x48: return w16 ? launch_cfg<1, 3, 2, 2, 16>(p, plan, group, stream) : launch_cfg<1, 3, 3, 3, 8>(p, plan, group, stream);
        case kSkinny16x64: return w16 ? launch_cfg<1, 4, 2, 1, 16>(p, plan, group, stream) : launch_cfg<1, 4, 2, 2, 8>(p, plan, group, stream);
        case kSkinny16x96: return w16 ? launch_cfg<1, 6, 1, 1, 16>(p, plan, group, stream) : launch_cfg<1, 6, 3, 2, 8>(p, plan, group, stream);
        case kSkinny16x128: return w16 ? launch_cfg<1, 8, 1, 1, 16>(p, plan, group, stream) : launch_cfg<1, 8, 2, 2, 8>(p, plan, group, stream);
        case kSkinny32x32: return w16 ? launch_cfg<2, 2, 2, 1, 16>(p, plan, group, stream) : launch_cfg<2, 2, 2, 2, 8>(p, plan, group, stream);
        case kSkinny32x64: return launch_cfg<2, 4, 2, 2, 8>(p, plan, group, stream);
        case kSkinny64x32: return w16 ? hipErrorInvalidValue : launch_cfg<4, 2, 2, 2, 8>(p, plan, group, stream);
        case kSkinny64x48: return w16 ? hipErrorInvalidValue : launch_cfg<4, 3, 2, 2, 8>(p, plan, group, stream);
        case kSkinny64x64: return w16 ? hipErrorInvalidValue : launch_cfg<4, 4, 2, 1, 8>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
