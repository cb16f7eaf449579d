// CTA-tile kernels whose CTAs hold two or four sets of waves, each set multiplying its own slice of every
// K stage (in-CTA split-K).  A set is four waves of two 16-column tiles (128 columns) or two waves of three
// (96 columns; with two or four sets its waves still cover all four SIMDs evenly, and 96-column tiles divide
// some widths into a number of CTAs closer to a multiple of the CU count).  For the row counts between the decode and the prefill regime, where a shape yields
// fewer CTAs than would give every SIMD a second wave: the sets hide each other's LDS and memory latency, every
// CTA still reads its rows of X once, and the partial tiles meet in LDS instead of global memory.
// Built like the other small tiles with the MFMA accumulators in ordinary vector registers.
#include "tm_w4_tile_impl.h"

namespace tmw4 {

namespace {

template <int TM, int TN, int KG, int NW = 4>
hipError_t launch_depth_kg(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    constexpr int BM = TM * 16;
    constexpr int WAVES = NW * KG;
    // two X buffers of BM rows x (32 * steps * KG + pad) halves must fit the 160 KiB of LDS; CTAs of 16 waves
    // have 128 registers per lane, which bounds the stage depth they are built with (the 128 x 256 tile, 128
    // accumulator registers per lane, is built with 64-deep stages only)
    switch (plan.stage_steps) {
        case 2:
            if constexpr (BM * (64 * KG + 16) * 4 <= 160 * 1024) return launch_shape<TM, TN, NW, 2, KG>(p, plan, group, stream);
            return hipErrorInvalidValue;
        case 4:
            if constexpr ((WAVES < 16 || TM <= 2) && TM * TN <= 16 && BM * (128 * KG + 16) * 4 <= 160 * 1024)
                return launch_shape<TM, TN, NW, 4, KG>(p, plan, group, stream);
            return hipErrorInvalidValue;
        case 8:
            if constexpr (TM <= 4 && TN <= 2 && WAVES <= 8 && BM * (256 * KG + 16) * 4 <= 160 * 1024)
                return launch_shape<TM, TN, NW, 8, KG>(p, plan, group, stream);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_tile_kgroup(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    if (plan.kgroups == 2) {
        switch (plan.variant) {
            case kTile32x128: return launch_depth_kg<2, 2, 2>(p, plan, group, stream);
            case kTile64x128: return launch_depth_kg<4, 2, 2>(p, plan, group, stream);
            case kTile128x128: return launch_depth_kg<8, 2, 2>(p, plan, group, stream);
            case kTile128x256: return launch_depth_kg<8, 4, 2>(p, plan, group, stream);
            case kTile32x96: return launch_depth_kg<2, 3, 2, 2>(p, plan, group, stream);
            case kTile64x96: return launch_depth_kg<4, 3, 2, 2>(p, plan, group, stream);
            case kTile64x64: return launch_depth_kg<4, 2, 2, 2>(p, plan, group, stream);
            case kTile128x64: return launch_depth_kg<8, 2, 2, 2>(p, plan, group, stream);
            default: return hipErrorInvalidValue;
        }
    }
    if (plan.kgroups == 4) {
        switch (plan.variant) {
            case kTile32x128: return launch_depth_kg<2, 2, 4>(p, plan, group, stream);
            case kTile64x128: return launch_depth_kg<4, 2, 4>(p, plan, group, stream);
            case kTile32x96: return launch_depth_kg<2, 3, 4, 2>(p, plan, group, stream);
            case kTile64x96: return launch_depth_kg<4, 3, 4, 2>(p, plan, group, stream);
            case kTile64x64: return launch_depth_kg<4, 2, 4, 2>(p, plan, group, stream);
            case kTile128x64: return launch_depth_kg<8, 2, 4, 2>(p, plan, group, stream);
            default: return hipErrorInvalidValue;
        }
    }
    return hipErrorInvalidValue;
}

}  // namespace tmw4
