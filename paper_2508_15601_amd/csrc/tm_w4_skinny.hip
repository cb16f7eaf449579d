// Fused dequantise-and-multiply for the decode shapes (M <= 64): the HBM-bound regime.
//
// Online stage of the GEMM pipeline (paper Sec. 3.1 steps (i)-(iv), Sec. 4.3).  What differs from the paper's
// design, which stages weights through shared memory for a 32-lane tensor-core fragment load:
//   - the packed buffer is already in matrix-core operand order, so a wave's 128-bit load of one 1 KiB unit lands
//     directly in the B-operand registers of four MFMAs; weights never touch LDS;
//   - every wave issues all weight, scale/zero and activation loads of its (up to two) units before the first
//     conversion, which is what the memory pipeline depth of the paper's loop achieves with asynchronous copies;
//   - a CTA is 8 waves that split the K range of one 64-column strip; their partial tiles meet in LDS, and CTAs
//     that split K further meet in an fp32 workspace that the last-arriving CTA sums in fixed order.
#include "tm_w4_host.h"

namespace tmw4 {

namespace {

constexpr int kWaves = 8;       // waves per CTA, splitting K
constexpr int kNTW = 4;         // 16-column tiles per wave (64 columns per CTA)

template <int TM, int GPU>
struct Stage {
    u32x4 wq[kNTW];             // packed weights: 4 words per lane and n-tile
    uint32_t sz[kNTW][GPU];     // scale|zero words of the groups inside the unit
    u32x4 xf[TM][4];            // activation fragments for the four MFMA k-steps
};

template <int TM, int GPU>
__device__ __forceinline__ void load_stage(Stage<TM, GPU>& st, const GemmParams& p, int nt0, int ku, int lane)
{
    const int c = lane & 15, h = lane >> 4;
#pragma unroll
    for (int j = 0; j < kNTW; ++j) {
        int nt = nt0 + j;
        if (nt < p.NT) {
            st.wq[j] = p.W[((size_t)nt * p.KU + ku) * 64 + lane];
#pragma unroll
            for (int g = 0; g < GPU; ++g) st.sz[j][g] = p.SZ[((size_t)nt * p.G + ku * GPU + g) * 16 + c];
        } else {
            st.wq[j] = u32x4{0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < GPU; ++g) st.sz[j][g] = 0;
        }
    }
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
        int row = mt * 16 + c;
        row = row < p.M ? row : p.M - 1;           // rows past M repeat the last row; their outputs are dropped
        const u32x4* xr = (const u32x4*)(p.X + (size_t)row * p.K + (size_t)ku * kUnitK + 8 * h);
#pragma unroll
        for (int t = 0; t < 4; ++t) st.xf[mt][t] = xr[4 * t];   // k = 128*ku + 32*t + 8*h .. +7
    }
}

template <int TM, int GPU>
__device__ __forceinline__ void compute_stage(const Stage<TM, GPU>& st, f32x4 (&acc)[TM][kNTW])
{
#pragma unroll
    for (int j = 0; j < kNTW; ++j) {
        GroupConst gc[GPU];
#pragma unroll
        for (int g = 0; g < GPU; ++g) gc[g] = make_group_const(st.sz[j][g]);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            f16x8 b = dequant8(st.wq[j][t], gc[(t * GPU) / 4]);
#pragma unroll
            for (int mt = 0; mt < TM; ++mt)
                acc[mt][j] = mfma16x16x32(__builtin_bit_cast(f16x8, st.xf[mt][t]), b, acc[mt][j]);
        }
    }
}

template <int TM, int GPU>
__global__ __launch_bounds__(kWaves * 64) void skinny_kernel(GemmParams p)
{
    __shared__ float red[kWaves][kNTW * 4][64];    // one 16 x 64 fp32 tile per wave, in accumulator layout
    __shared__ uint32_t s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int strips = (p.NT + kNTW - 1) / kNTW;
    const int strip = blockIdx.x % strips;
    const int sk = blockIdx.x / strips;
    const int nt0 = strip * kNTW;
    const int ku0 = sk * p.ku_per_split;
    const int ku1 = min(p.KU, ku0 + p.ku_per_split);

    f32x4 acc[TM][kNTW];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int j = 0; j < kNTW; ++j) acc[mt][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int ku = ku0 + wave; ku < ku1; ku += 2 * kWaves) {
        Stage<TM, GPU> a, b;
        const bool two = ku + kWaves < ku1;
        load_stage(a, p, nt0, ku, lane);
        if (two) load_stage(b, p, nt0, ku + kWaves, lane);
        compute_stage(a, acc);
        if (two) compute_stage(b, acc);
    }

    // Reduce the 8 waves' tiles through LDS, one 16-row tile at a time; thread -> (row, two adjacent columns).
    const int row = tid >> 5;
    const int col = (tid & 31) * 2;
    const int src_reg = (col >> 4) * 4 + (row & 3);
    const int src_lane = 16 * (row >> 2) + (col & 15);
    const int n = nt0 * 16 + col;
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
        if (mt) __syncthreads();
#pragma unroll
        for (int j = 0; j < kNTW; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[wave][j * 4 + r][lane] = acc[mt][j][r];
        __syncthreads();
        float v0 = 0.f, v1 = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            v0 += red[w][src_reg][src_lane];
            v1 += red[w][src_reg][src_lane + 1];
        }
        const int m = mt * 16 + row;
        if (m < p.M && n < p.N) {
            if (p.split == 1) {
                uint32_t o = (uint32_t)f32_to_f16_bits(v0) | ((uint32_t)f32_to_f16_bits(v1) << 16);
                *(uint32_t*)(p.Y + (size_t)m * p.N + n) = o;
            } else {
                *(float2*)(p.partial + ((size_t)sk * p.M + m) * p.N + n) = float2{v0, v1};
            }
        }
    }

    if (p.split > 1) {
        // The CTA that arrives last at this strip's counter adds the partial tiles in split order.
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            uint32_t prev = atomicAdd(&p.counters[strip], 1u);
            s_last = (prev == (uint32_t)p.split - 1u) ? 1u : 0u;
        }
        __syncthreads();
        if (s_last) {
            __threadfence();
#pragma unroll
            for (int mt = 0; mt < TM; ++mt) {
                const int m = mt * 16 + row;
                if (m < p.M && n < p.N) {
                    float v0 = 0.f, v1 = 0.f;
                    for (int s = 0; s < p.split; ++s) {
                        float2 t = *(const float2*)(p.partial + ((size_t)s * p.M + m) * p.N + n);
                        v0 += t.x;
                        v1 += t.y;
                    }
                    uint32_t o = (uint32_t)f32_to_f16_bits(v0) | ((uint32_t)f32_to_f16_bits(v1) << 16);
                    *(uint32_t*)(p.Y + (size_t)m * p.N + n) = o;
                }
            }
            if (tid == 0) __hip_atomic_store(&p.counters[strip], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <int TM>
hipError_t launch_tm(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    dim3 grid(plan.grid), block(plan.block);
    switch (group) {
        case 128: hipLaunchKernelGGL((skinny_kernel<TM, 1>), grid, block, 0, stream, p); break;
        case 64: hipLaunchKernelGGL((skinny_kernel<TM, 2>), grid, block, 0, stream, p); break;
        case 32: hipLaunchKernelGGL((skinny_kernel<TM, 4>), grid, block, 0, stream, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_skinny(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    switch (plan.variant) {
        case kSkinny16: return launch_tm<1>(p, plan, group, stream);
        case kSkinny32: return launch_tm<2>(p, plan, group, stream);
        case kSkinny64: return launch_tm<4>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
