// Fused dequantise-and-multiply for the decode shapes (M <= 32): the HBM-bound regime.
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
#include "tm_w4_host.h"

namespace tmw4 {

namespace {

template <int TM, int NTW, int GPU>
struct Stage {
    u32x4 wq[NTW];              // packed weights: 4 words per lane and n-tile
    uint32_t sz[NTW][GPU];      // scale|zero words of the groups inside the unit
    u32x4 xf[TM][4];            // activation fragments for the four MFMA k-steps
};

template <int TM, int NTW, int GPU>
__device__ __forceinline__ void load_stage(Stage<TM, NTW, GPU>& st, const GemmParams& p, int nt0, int ku, int lane)
{
    const int c = lane & 15, h = lane >> 4;
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        int nt = nt0 + j;
        if (nt < p.NT) {
            st.wq[j] = __builtin_nontemporal_load(&p.W[((size_t)nt * p.KU + ku) * 64 + lane]);
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

template <int TM, int NTW, int GPU>
__device__ __forceinline__ void compute_stage(const Stage<TM, NTW, GPU>& st, f32x4 (&acc)[TM][NTW])
{
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
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

// TM 16-row tiles, NTW 16-column tiles per wave, GPU K-groups per 128-row unit, D units in flight per wave.
template <int TM, int NTW, int GPU, int D>
__global__ __launch_bounds__(1024) void skinny_kernel(GemmParams p)
{
    extern __shared__ float red[];                 // [waves][NTW*4][64]: one 16 x 16*NTW fp32 tile per wave
    __shared__ uint32_t s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int waves = blockDim.x >> 6;
    const int strips = (p.NT + NTW - 1) / NTW;
    const int strip = blockIdx.x % strips;
    const int sk = blockIdx.x / strips;
    const int nt0 = strip * NTW;
    const int ku0 = sk * p.ku_per_split;
    const int ku1 = min(p.KU, ku0 + p.ku_per_split);

    f32x4 acc[TM][NTW];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int j = 0; j < NTW; ++j) acc[mt][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int ku = ku0 + wave; ku < ku1; ku += D * waves) {
        Stage<TM, NTW, GPU> st[D];
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (ku + d * waves < ku1) load_stage(st[d], p, nt0, ku + d * waves, lane);
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (ku + d * waves < ku1) compute_stage(st[d], acc);
    }

    // Reduce the waves' tiles through LDS, one 16-row tile at a time; thread -> (row, two adjacent columns).
    constexpr int kPairs = 8 * NTW;                // column pairs per row
    const bool owner = tid < 16 * kPairs;
    const int row = tid / kPairs;
    const int col = (tid % kPairs) * 2;
    const int src_reg = (col >> 4) * 4 + (row & 3);
    const int src_lane = 16 * (row >> 2) + (col & 15);
    const int n = nt0 * 16 + col;
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
        if (mt) __syncthreads();
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[(wave * NTW * 4 + j * 4 + r) * 64 + lane] = acc[mt][j][r];
        __syncthreads();
        const int m = mt * 16 + row;
        if (owner && m < p.M && n < p.N) {
            float v0 = 0.f, v1 = 0.f;
            for (int w = 0; w < waves; ++w) {
                float2 t = *(const float2*)&red[(w * NTW * 4 + src_reg) * 64 + src_lane];
                v0 += t.x;
                v1 += t.y;
            }
            if (p.split == 1) {
                uint32_t o = (uint32_t)f32_to_f16_bits(v0) | ((uint32_t)f32_to_f16_bits(v1) << 16);
                *(uint32_t*)(p.Y + (size_t)m * p.N + n) = o;
            } else {
                st_partial2(p.partial + ((size_t)sk * p.M + m) * p.N + n, v0, v1);
            }
        }
    }

    if (p.split > 1) {
        // The CTA that arrives last at this strip's counter adds the partial tiles in split order.
        wait_stores_done();
        __syncthreads();
        if (tid == 0) {
            uint32_t prev = atomicAdd(&p.counters[strip], 1u);
            s_last = (prev == (uint32_t)p.split - 1u) ? 1u : 0u;
        }
        __syncthreads();
        if (s_last) {
#pragma unroll
            for (int mt = 0; mt < TM; ++mt) {
                const int m = mt * 16 + row;
                if (owner && m < p.M && n < p.N) {
                    float v0 = 0.f, v1 = 0.f;
                    for (int s = 0; s < p.split; ++s) {
                        float a, b;
                        ld_partial2(p.partial + ((size_t)s * p.M + m) * p.N + n, a, b);
                        v0 += a;
                        v1 += b;
                    }
                    uint32_t o = (uint32_t)f32_to_f16_bits(v0) | ((uint32_t)f32_to_f16_bits(v1) << 16);
                    *(uint32_t*)(p.Y + (size_t)m * p.N + n) = o;
                }
            }
            if (tid == 0) __hip_atomic_store(&p.counters[strip], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <int TM, int NTW, int D>
hipError_t launch_cfg(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    dim3 grid(plan.grid), block(plan.block);
    size_t lds = (size_t)(plan.block / 64) * NTW * 4 * 64 * sizeof(float);
    switch (group) {
        case 128: hipLaunchKernelGGL((skinny_kernel<TM, NTW, 1, D>), grid, block, lds, stream, p); break;
        case 64: hipLaunchKernelGGL((skinny_kernel<TM, NTW, 2, D>), grid, block, lds, stream, p); break;
        case 32: hipLaunchKernelGGL((skinny_kernel<TM, NTW, 4, D>), grid, block, lds, stream, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_skinny(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    switch (plan.variant) {
        case kSkinny16x16: return launch_cfg<1, 1, 4>(p, plan, group, stream);
        case kSkinny16x32: return launch_cfg<1, 2, 2>(p, plan, group, stream);
        case kSkinny16x64: return launch_cfg<1, 4, 1>(p, plan, group, stream);
        case kSkinny32x32: return launch_cfg<2, 2, 1>(p, plan, group, stream);
        case kSkinny32x64: return launch_cfg<2, 4, 1>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
