// Instantiations and launcher of the one-shot decode kernels for 16 < M <= 32 (tm_w4_streamx_impl.h), 4-bit weights.
#include "tm_w4_streamx_impl.h"

namespace tmw4 {

hipError_t launch_rows32(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    return launch_rows_tm<2>(p, plan, group, stream);
}

// Can a launch with strips of ntw column tiles and kus packed units per K slice run as a one-shot kernel for more than
// 16 rows on CTAs of `waves` waves, and with how many units per wave?  Returns 0 if not.
int rows_units_per_wave(int M, int ntw, int group, int kus, int waves)
{
    if (M <= 16 || M > 64) return 0;
    return rows_units(M <= 32 ? 2 : 4, ntw, group, kus, waves);
}

hipError_t launch_rows(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    return p.M <= 32 ? launch_rows32(p, plan, group, stream) : launch_rows64(p, plan, group, stream);
}

}  // namespace tmw4
