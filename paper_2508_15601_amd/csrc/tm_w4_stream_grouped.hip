// Instantiations and launcher of the grouped (mixture-of-experts) form of the one-shot decode kernels
// (tm_w4_stream_impl.h), 4-bit weights, experts with up to sixteen rows per pass.
#include "tm_w4_stream_impl.h"

namespace tmw4 {

namespace {

template <int NTW, int NI>
hipError_t launch_grouped_ni(const GroupedParams& gp, int experts, int group, int block, hipStream_t stream)
{
    return block > 512 ? launch_stream_grouped_cfg<NTW, NI, 16>(gp, experts, group, block, stream)
                       : launch_stream_grouped_cfg<NTW, NI, 8>(gp, experts, group, block, stream);
}

template <int NTW>
hipError_t launch_grouped_ntw(const GroupedParams& gp, int experts, int group, int ni, int block, hipStream_t stream)
{
    switch (ni) {
        case 1: return launch_grouped_ni<NTW, 1>(gp, experts, group, block, stream);
        case 2: return launch_grouped_ni<NTW, 2>(gp, experts, group, block, stream);
        case 3: return launch_grouped_ni<NTW, 3>(gp, experts, group, block, stream);
        case 4: return launch_grouped_ni<NTW, 4>(gp, experts, group, block, stream);
        case 6: return launch_grouped_ni<NTW, 6>(gp, experts, group, block, stream);
        case 8: return launch_grouped_ni<NTW, 8>(gp, experts, group, block, stream);
        default: return hipErrorInvalidValue;
    }
}

template <int NTW, int NI>
hipError_t raise_grouped_ntw_ni()
{
    hipError_t e = hipSuccess;
    auto acc = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    acc(stream_grouped_raise_one<NTW, 1, NI, 16>());
    acc(stream_grouped_raise_one<NTW, 2, NI, 16>());
    acc(stream_grouped_raise_one<NTW, 4, NI, 16>());
    acc(stream_grouped_raise_one<NTW, 1, NI, 8>());
    acc(stream_grouped_raise_one<NTW, 2, NI, 8>());
    acc(stream_grouped_raise_one<NTW, 4, NI, 8>());
    return e;
}

template <int NTW>
hipError_t raise_grouped_ntw()
{
    hipError_t e = raise_grouped_ntw_ni<NTW, 1>();
    if (e == hipSuccess) e = raise_grouped_ntw_ni<NTW, 2>();
    if (e == hipSuccess) e = raise_grouped_ntw_ni<NTW, 3>();
    if (e == hipSuccess) e = raise_grouped_ntw_ni<NTW, 4>();
    if (e == hipSuccess) e = raise_grouped_ntw_ni<NTW, 6>();
    if (e == hipSuccess) e = raise_grouped_ntw_ni<NTW, 8>();
    return e;
}

}  // namespace

hipError_t stream_grouped_setup()
{
    hipError_t e = raise_grouped_ntw<1>();
    if (e == hipSuccess) e = raise_grouped_ntw<2>();
    if (e == hipSuccess) e = raise_grouped_ntw<3>();
    if (e == hipSuccess) e = raise_grouped_ntw<4>();
    if (e == hipSuccess) e = raise_grouped_ntw<5>();
    if (e == hipSuccess) e = raise_grouped_ntw<6>();
    if (e == hipSuccess) e = raise_grouped_ntw<7>();
    if (e == hipSuccess) e = raise_grouped_ntw<8>();
    return e;
}

// ni units per wave and block threads as the single-GEMM plan of one expert at sixteen rows gives them; gp.lds_bytes
// the LDS of that plan.
hipError_t launch_stream_grouped(const GroupedParams& gp, int experts, int group, int ni, int block, hipStream_t stream)
{
    if (experts <= 0 || experts > 65535 || gp.strips <= 0 || (size_t)gp.lds_bytes > kStreamLdsBudget) return hipErrorInvalidValue;
    const int ntw = gp.strip_base + (gp.strip_rem > 0 ? 1 : 0);
    switch (ntw) {
        case 1: return launch_grouped_ntw<1>(gp, experts, group, ni, block, stream);
        case 2: return launch_grouped_ntw<2>(gp, experts, group, ni, block, stream);
        case 3: return launch_grouped_ntw<3>(gp, experts, group, ni, block, stream);
        case 4: return launch_grouped_ntw<4>(gp, experts, group, ni, block, stream);
        case 5: return launch_grouped_ntw<5>(gp, experts, group, ni, block, stream);
        case 6: return launch_grouped_ntw<6>(gp, experts, group, ni, block, stream);
        case 7: return launch_grouped_ntw<7>(gp, experts, group, ni, block, stream);
        case 8: return launch_grouped_ntw<8>(gp, experts, group, ni, block, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
