// The decode kernels instantiated for FP8 (E4M3) weight codes: the 8-bit packed layout, conversion by the hardware's
// packed FP8 -> fp16 instruction, no zero-point and therefore no bias-cancelling second MFMA.
#include "tm_w4_skinny_impl.h"

namespace tmw4 {

hipError_t launch_skinny_f8(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    return launch_skinny_8bit<kFmtFp8>(p, plan, group, stream);
}

hipError_t launch_skinny_grouped_f8(const GroupedParams& gp, int variant, int experts, int group, hipStream_t stream)
{
    return launch_skinny_grouped_fmt<kFmtFp8>(gp, variant, experts, group, stream);
}

}  // namespace tmw4
