// Instantiations and launcher of the one-shot decode kernels (tm_w4_stream_impl.h), 4-bit weights, M <= 16.
#include "tm_w4_stream_impl.h"

namespace tmw4 {

namespace {

template <int NTW, int NI>
hipError_t launch_stream_ni(const GemmParams& p, const Plan& plan, int group, size_t lds, hipStream_t stream)
{
    return plan.block > 512 ? launch_stream_cfg<NTW, NI, 16>(p, plan, group, lds, stream)
                            : launch_stream_cfg<NTW, NI, 8>(p, plan, group, lds, stream);
}

template <int NTW>
hipError_t launch_stream_ntw(const GemmParams& p, const Plan& plan, int group, size_t lds, hipStream_t stream)
{
    switch (plan.stream_ni) {
        case 1: return launch_stream_ni<NTW, 1>(p, plan, group, lds, stream);
        case 2: return launch_stream_ni<NTW, 2>(p, plan, group, lds, stream);
        case 3: return launch_stream_ni<NTW, 3>(p, plan, group, lds, stream);
        case 4: return launch_stream_ni<NTW, 4>(p, plan, group, lds, stream);
        case 6: return launch_stream_ni<NTW, 6>(p, plan, group, lds, stream);
        case 8: return launch_stream_ni<NTW, 8>(p, plan, group, lds, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

namespace {

template <int NTW, int NI>
hipError_t raise_ntw_ni()
{
    hipError_t e = hipSuccess;
    auto acc = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    acc(stream_raise_one<NTW, 1, NI, 16>());
    acc(stream_raise_one<NTW, 2, NI, 16>());
    acc(stream_raise_one<NTW, 4, NI, 16>());
    acc(stream_raise_one<NTW, 1, NI, 8>());
    acc(stream_raise_one<NTW, 2, NI, 8>());
    acc(stream_raise_one<NTW, 4, NI, 8>());
    return e;
}

template <int NTW>
hipError_t raise_ntw()
{
    hipError_t e = raise_ntw_ni<NTW, 1>();
    if (e == hipSuccess) e = raise_ntw_ni<NTW, 2>();
    if (e == hipSuccess) e = raise_ntw_ni<NTW, 3>();
    if (e == hipSuccess) e = raise_ntw_ni<NTW, 4>();
    if (e == hipSuccess) e = raise_ntw_ni<NTW, 6>();
    if (e == hipSuccess) e = raise_ntw_ni<NTW, 8>();
    return e;
}

}  // namespace

hipError_t stream_setup()
{
    hipError_t e = raise_ntw<1>();
    if (e == hipSuccess) e = raise_ntw<2>();
    if (e == hipSuccess) e = raise_ntw<3>();
    if (e == hipSuccess) e = raise_ntw<4>();
    if (e == hipSuccess) e = raise_ntw<5>();
    if (e == hipSuccess) e = raise_ntw<6>();
    if (e == hipSuccess) e = raise_ntw<7>();
    if (e == hipSuccess) e = raise_ntw<8>();
    return e;
}

// Can this plan run as a one-shot kernel, and with how many units per wave?  Returns 0 if not.
int stream_units_per_wave(int ntw, int group, int kus, int waves)
{
    const int gpu = 128 / group;
    int ni = (kus + waves - 1) / waves;
    static const int built[] = {1, 2, 3, 4, 6, 8};
    for (int b : built)
        if (b >= ni) {
            ni = b;
            return stream_built(ntw, gpu, ni, waves) ? ni : 0;
        }
    return 0;
}

size_t stream_lds(int ni, int mp_log, int ntw, int waves, int* red_off)
{
    return stream_lds_bytes(ni, mp_log, ntw, waves, kStreamLdsBudget, red_off);
}

hipError_t launch_stream(const GemmParams& p0, const Plan& plan, int group, hipStream_t stream)
{
    GemmParams p = p0;
    const int ntw = p.strip_base + (p.strip_rem > 0 ? 1 : 0);
    const size_t lds = stream_lds_bytes(plan.stream_ni, p.mp_log, ntw, (int)plan.block / 64, kStreamLdsBudget, &p.red_off);
    if (lds > kStreamLdsBudget) return hipErrorInvalidValue;
    switch (ntw) {
        case 1: return launch_stream_ntw<1>(p, plan, group, lds, stream);
        case 2: return launch_stream_ntw<2>(p, plan, group, lds, stream);
        case 3: return launch_stream_ntw<3>(p, plan, group, lds, stream);
        case 4: return launch_stream_ntw<4>(p, plan, group, lds, stream);
        case 5: return launch_stream_ntw<5>(p, plan, group, lds, stream);
        case 6: return launch_stream_ntw<6>(p, plan, group, lds, stream);
        case 7: return launch_stream_ntw<7>(p, plan, group, lds, stream);
        case 8: return launch_stream_ntw<8>(p, plan, group, lds, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
