// Instantiations of the one-shot decode kernels for 32 < M <= 64 (tm_w4_streamx_impl.h), 4-bit weights.
#include "tm_w4_streamx_impl.h"

namespace tmw4 {

hipError_t launch_rows64(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    return launch_rows_tm<4>(p, plan, group, stream);
}

}  // namespace tmw4
