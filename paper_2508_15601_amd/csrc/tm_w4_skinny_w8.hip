// The decode kernels instantiated for 8-bit integer weight codes (W8A16): same pipeline, packed units of 64 rows,
// byte-permute conversion.  Only the strip widths the dispatcher uses for this format are built.
#include "tm_w4_skinny_impl.h"

namespace tmw4 {

hipError_t launch_skinny_w8(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    return launch_skinny_8bit<kFmtInt8>(p, plan, group, stream);
}

hipError_t launch_skinny_grouped_w8(const GroupedParams& gp, int variant, int experts, int group, hipStream_t stream)
{
    return launch_skinny_grouped_fmt<kFmtInt8>(gp, variant, experts, group, stream);
}

}  // namespace tmw4
