// Decode kernels, one-shot form ("stream"): for M <= 16 and layers whose slice of X fits into LDS.
//
// Same arithmetic as the ring-buffered decode kernels (paper Sec. 3.1 steps (i)-(iv): packed weights straight into
// matrix-core operand registers, bit-manipulation conversion on the vector ALU, conversion bias and zero-point
// cancelled by a second MFMA, group scale on the fp32 group sum), organised for the one thing that bounds a launch of
// 5-15 us: how soon every byte of the weight stream is requested and how little is left to do after the last one lands.
//
//   - A wave owns NI packed units of K (NI is a template parameter) and issues ALL of its weight and scale/zero loads
//     at once, back to back, before anything else happens: straight-line code, so the waits the compiler places are
//     exact per register (a conversion starts when its own 16 bytes per lane have arrived, with the rest of the
//     stream still in flight).  The memory pipeline of paper Sec. 4.3 is here as deep as the whole K range.
//   - Every load is a buffer load: descriptor and K offset in scalar registers, one constant per-lane offset; no
//     vector address arithmetic, no branch around a load.  A wave whose last unit falls outside a ragged K range
//     loads through an empty descriptor (zeros, no memory traffic) and skips that unit's arithmetic.
//   - X does not travel through per-wave registers.  Every wave copies the rows of X that belong to its own units
//     into its own region of LDS, with direct-to-LDS loads of whole 256-byte row pieces issued BEFORE the weight loads
//     (the load counter retires in order, so "at most <weight loads> outstanding" means the rows have landed while
//     the weight stream stays in flight), and reads its fragments from there.  No CTA barrier: a wave starts its
//     arithmetic as soon as its own bytes are there, while younger waves are still issuing loads.  At M = 1 that is
//     one load instruction per wave instead of four per unit; at M = 16 it halves the cache-line requests of the
//     activations, which otherwise outnumber those of the weights.
//   - A strip is exactly NTW column tiles, a template parameter (strips are dealt evenly, so a launch has strips of
//     two adjacent widths: the kernel is instantiated for a width and the one below and the CTA picks).
//
// LDS image of a wave's X region: [unit index i < NI][row r < Mp][16 chunks of 16 bytes], Mp = M rounded up to a power
// of two; chunk q of (i, r) sits in slot q ^ (r & 15), so that the 16 rows a fragment read touches fall into 16
// different bank groups.
#pragma once
#include "tm_w4_skinny_impl.h"

namespace tmw4 {

namespace {

template <int NTW, int GU, int NI>
struct StreamRegs {
    u32x4 wq[NI][NTW];             // packed weights: 4 words per lane, unit and column tile
    uint32_t sz[NI][NTW][GU];      // scale|zero words of the K-groups inside the unit
};

// Cross-wave sum of the one-shot kernels: WAVES partial tiles of 16 x 16*NTW fp32 -> fp16 outputs (or split-K partial
// sums).  Written for latency, because nothing else is left to overlap it with: only the accumulator registers that
// hold rows below M go through LDS, the wave count is a template parameter (every sum is a straight run of 64-bit LDS
// reads), a reading thread owns two neighbouring columns (no cross-lane exchange), and one pass of the CTA covers all
// outputs.  red: [NTW*4 registers][WAVES][64 lanes] floats.
template <int NTW, int WAVES>
__device__ __forceinline__ void stream_reduce(const GemmParams& p, const f32x4 (&acc)[NTW], const int strip, const int sk,
                                              const int nt0, float* __restrict__ red, uint32_t& s_last)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // a lane holds rows 4 * (lane / 16) + r in register r: register r is dead in every lane when r >= M (the test is
    // wave-uniform; lanes whose row is past M write values nobody reads)
#pragma unroll
    for (int j = 0; j < NTW; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (r < p.M) red[((j * 4 + r) * WAVES + wave) * 64 + lane] = acc[j][r];
    __syncthreads();
    // thread -> (register jr = tid / 32 (+ a second pass for wide strips on small CTAs), column pair tid % 32)
    const int pl = (tid & 31) * 2;
    constexpr int kPasses = (NTW * 4 + WAVES * 2 - 1) / (WAVES * 2);
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) {
        const int jr = (tid >> 5) + ps * WAVES * 2;
        const int m = 4 * (pl >> 4) + (jr & 3);
        if (jr < NTW * 4 && m < p.M) {
            const float* src = red + (size_t)jr * WAVES * 64 + pl;
            float2 t[WAVES];                        // all reads in flight at once, then the sum in wave order
#pragma unroll
            for (int w = 0; w < WAVES; ++w) t[w] = *(const float2*)(src + w * 64);
            __builtin_amdgcn_sched_barrier(0);
            float v0 = 0.f, v1 = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) {
                v0 += t[w].x;
                v1 += t[w].y;
            }
            const int n = (nt0 + (jr >> 2)) * 16 + (pl & 15);
            if (p.split == 1) store_pair(p, m, n, v0, v1);
            else st_partial2(p.partial + ((size_t)sk * p.strips + strip) * p.slot_floats + jr * 64 + pl, v0, v1);
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
            for (int ps = 0; ps < kPasses; ++ps) {
                const int jr = (tid >> 5) + ps * WAVES * 2;
                const int m = 4 * (pl >> 4) + (jr & 3);
                if (jr < NTW * 4 && m < p.M) {
                    const int n = (nt0 + (jr >> 2)) * 16 + (pl & 15);
                    float v0, v1;
                    sum_partials2(p.partial + (size_t)strip * p.slot_floats + jr * 64 + pl, (size_t)p.strips * p.slot_floats, p.split, v0, v1);
                    store_pair(p, m, n, v0, v1);
                }
            }
            if (tid == 0) __hip_atomic_store(&p.counters[strip], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// One CTA: column tiles nt0 .. nt0 + NTW - 1, K slice sk.  smem: the waves' X regions, then (or later in the same
// place, see red_off) the reduction tiles.
template <int NTW, int GPU, int NI, int WAVES>
__device__ __forceinline__ void stream_body(const GemmParams& p, const int strip, const int sk, const int nt0,
                                            unsigned char* __restrict__ smem, uint32_t& s_last)
{
    constexpr int GU = GPU;                        // K-groups per 128-row unit
    constexpr int TG = 4 / GU;                     // MFMA k-steps per K-group
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    constexpr int waves = WAVES;                   // the launch uses exactly this many
    const int c = lane & 15, h = lane >> 4;
    const int ku0 = sk * p.ku_per_split;
    const int kus = min(p.KU, ku0 + p.ku_per_split) - ku0;         // packed units in this K slice
    const int mp_log = p.mp_log;
    const Magic mg = make_magic();

    // ---- this wave's rows of X for its own NI units, into its own region of LDS: no other wave reads them, so no
    // CTA barrier stands between a wave and its arithmetic.  One load instruction moves 64 chunks of 16 bytes to
    // 1 KiB of consecutive LDS = four (unit, row) segments of 16 chunks; segment s = unit_index * Mp + row.  Rows
    // r >= M fall outside the descriptor by themselves (r * K * 2 >= M * K * 2) and segments past the wave's units get
    // an offset that does: both write zeros and touch no memory.
    const int x_region = ((((NI << mp_log) + 3) >> 2) << 10);      // bytes per wave: whole load instructions
    unsigned char* const xw = smem + (size_t)wave * x_region;
    {
        const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.X, (uint32_t)p.M * (uint32_t)p.K * 2u);
        const int ninstr = ((NI << mp_log) + 3) >> 2;
        const uint32_t k2 = (uint32_t)p.K * 2u;
#pragma unroll
        for (int i = 0; i < NI * 4; ++i) {                         // NI * 4 = the count for Mp = 16
            if (i < ninstr) {
                const int s = i * 4 + h;
                const int ui = s >> mp_log;                        // which of the wave's units
                const int r = s & ((1 << mp_log) - 1);
                const int ul = wave + ui * waves;
                const bool in = ui < NI && ul < kus;
                const uint32_t off = in ? (uint32_t)r * k2 + (uint32_t)(ku0 + ul) * 256u + (uint32_t)((c ^ (r & 15)) * 16)
                                        : 0x80000000u;
#if defined(__HIP_DEVICE_COMPILE__)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rsrc, (__attribute__((address_space(3))) void*)(xw + i * 1024), 16,
                                                         off, 0, 0, 0);
#else
                (void)off;
                (void)x_rsrc;
#endif
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);             // the count in the wait below is exact only if nothing moves across

    // ---- every weight load of this wave, in the order of use
    StreamRegs<NTW, GU, NI> st;
    {
        const uint32_t w_lane = (uint32_t)lane * 16u, s_lane = (uint32_t)c * 4u;
        const char* wbase = (const char*)p.W + (size_t)nt0 * p.KU * 1024;
        const char* sbase = (const char*)p.SZ + (size_t)nt0 * p.G * 64;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int ul = wave + i * waves;                       // unit of this wave inside the slice (wave-uniform)
            const bool valid = ul < kus;
            const int ku = ku0 + ul;
            const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(wbase, valid ? (uint32_t)(NTW * p.KU) * 1024u : 0u);
            const __amdgpu_buffer_rsrc_t s_rsrc = make_rsrc(sbase, valid ? (uint32_t)(NTW * p.G) * 64u : 0u);
#pragma unroll
            for (int j = 0; j < NTW; ++j) {
#pragma unroll
                for (int g = 0; g < GU; ++g)
                    st.sz[i][j][g] = __builtin_amdgcn_raw_buffer_load_b32(s_rsrc, s_lane, (j * p.G + ku * GU + g) * 64, 0);
                st.wq[i][j] = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, w_lane, (j * p.KU + ku) * 1024, kNonTemporalLoad);
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    {
        // the X loads are older than the NI * NTW * (GU + 1) loads just issued: wait until at most that many are
        // outstanding (the counter field holds up to 63; a smaller bound only waits for a few weight loads as well)
        constexpr int kYounger = NI * NTW * (GU + 1) < 63 ? NI * NTW * (GU + 1) : 63;
        __builtin_amdgcn_s_waitcnt((kYounger & 15) | ((kYounger >> 4) << 14) | (7 << 4) | (15 << 8));
    }
    __builtin_amdgcn_sched_barrier(0);

    f32x4 acc[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- multiply, unit by unit, as the data arrives.  A wave often works alone on its SIMD (the others are still
    // waiting for their bytes), so the order of the MFMAs matters: consecutive ones go to different accumulators.
    const int rr = min(c, p.M - 1);                // rows past M repeat the last row; their results are never stored
    const uint32_t x_lane = (uint32_t)rr * 256u;
    const uint32_t x_swz = (uint32_t)(rr & 15);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int ul = wave + i * waves;
        if (ul < kus) {
            const unsigned char* xu = xw + ((size_t)i << mp_log) * 256 + x_lane;
            f16x8 xf[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) xf[t] = *(const f16x8*)(xu + (((uint32_t)(4 * t + h)) ^ x_swz) * 16u);
            // column tiles in chunks of at most three: the MFMAs of a chunk alternate between its tiles' accumulators,
            // and a chunk starts as soon as its own weights have arrived
#pragma unroll
            for (int j0 = 0; j0 < NTW; j0 += 3) {
                constexpr int kChunkMax = 3;
                const int jn = NTW - j0 < kChunkMax ? NTW - j0 : kChunkMax;     // compile-time after unrolling
                // with one or two tiles in the chunk the products that cancel the conversion bias get accumulators of
                // their own, so that consecutive MFMAs still go to different ones
                const bool SPLITC = jn <= 2;
#pragma unroll
                for (int g = 0; g < GU; ++g) {
                    f32x4 part[kChunkMax], partc[kChunkMax];
                    f16x8 cancel[kChunkMax];
                    float scale[kChunkMax];
#pragma unroll
                    for (int jj = 0; jj < kChunkMax; ++jj) {
                        if (jj < jn) {
                            const f16x2 szp = as_f16x2(st.sz[i][j0 + jj][g]);
                            cancel[jj] = bias_cancel8(szp.y);
                            scale[jj] = (float)szp.x;
                            part[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
                            partc[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
                        }
                    }
#pragma unroll
                    for (int tt = 0; tt < TG; ++tt) {
                        const int t = g * TG + tt;
#pragma unroll
                        for (int jj = 0; jj < kChunkMax; ++jj)
                            if (jj < jn) part[jj] = mfma16x16x32(xf[t], biased8(st.wq[i][j0 + jj][t], mg), part[jj]);
#pragma unroll
                        for (int jj = 0; jj < kChunkMax; ++jj) {
                            if (jj < jn) {
                                if (SPLITC) partc[jj] = mfma16x16x32(xf[t], cancel[jj], partc[jj]);
                                else part[jj] = mfma16x16x32(xf[t], cancel[jj], part[jj]);
                            }
                        }
                    }
#pragma unroll
                    for (int jj = 0; jj < kChunkMax; ++jj) {
                        if (jj < jn) {
                            if (SPLITC) part[jj] += partc[jj];
                            acc[j0 + jj] += scale[jj] * part[jj];
                        }
                    }
                }
            }
        }
    }

    // the reduction tiles lie behind the X regions where both fit; where they share the space, every wave must be done
    // with its X first
    if (p.red_off == 0) __syncthreads();
    stream_reduce<NTW, WAVES>(p, acc, strip, sk, nt0, (float*)(smem + p.red_off), s_last);
}

// NTW = the wider of the two strip widths of the launch (strips of NTW - 1 tiles exist when the tile count is not a
// multiple of the strip count), GPU K-groups per unit, NI units per wave, MAXW the CTA size in waves (8 or 16).
template <int NTW, int GPU, int NI, int MAXW>
__global__ __launch_bounds__(MAXW * 64) void stream_kernel(GemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char stream_smem[];
    __shared__ uint32_t s_last;
    const int strip = blockIdx.x, sk = blockIdx.y;
    const int nt0 = strip * p.strip_base + min(strip, p.strip_rem);
    if constexpr (NTW > 1) {
        if (strip >= p.strip_rem && p.strip_base < NTW) {          // CTA-uniform
            stream_body<NTW - 1, GPU, NI, MAXW>(p, strip, sk, nt0, stream_smem, s_last);
            return;
        }
    }
    stream_body<NTW, GPU, NI, MAXW>(p, strip, sk, nt0, stream_smem, s_last);
}

// Grouped (mixture-of-experts) form of the one-shot kernels: blockIdx.y selects among the experts that have rows, as in
// skinny_grouped_kernel; an expert's rows are taken sixteen at a time, each pass a one-shot GEMM of its own (so the form
// is meant for decode batches, where an expert seldom has more than sixteen rows).  The LDS of the launch is sized for
// sixteen rows; the reduction tiles lie behind the X regions of the pass where both fit.
template <int NTW, int GPU, int NI, int MAXW>
__global__ __launch_bounds__(MAXW * 64) void stream_grouped_kernel(GroupedParams gp)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char stream_smem[];
    __shared__ uint32_t s_last;
    const ExpertRows er = find_expert(gp, blockIdx.y, threadIdx.x & 63);
    if (!er.found) return;                          // fewer experts have rows than the grid is tall
    GemmParams p = expert_params(gp, er);
    const int strip = blockIdx.x;
    const int nt0 = strip * gp.strip_base + min(strip, gp.strip_rem);
    const bool narrow = NTW > 1 && strip >= gp.strip_rem && gp.strip_base < NTW;      // CTA-uniform
    for (int m0 = er.r0; m0 < er.r1; m0 += 16) {
        if (m0 != er.r0) __syncthreads();           // the previous pass is done with LDS
        p.X = gp.X + (size_t)m0 * gp.K;
        p.Y = gp.Y + (size_t)m0 * p.ldy;
        p.M = min(16, er.r1 - m0);
        p.mp_log = p.M > 8 ? 4 : p.M > 4 ? 3 : p.M > 2 ? 2 : p.M > 1 ? 1 : 0;
        const int x_bytes = ((((NI << p.mp_log) + 3) >> 2) << 10) * MAXW;
        const int red_bytes = MAXW * NTW * 4 * 64 * (int)sizeof(float);
        p.red_off = x_bytes + red_bytes <= gp.lds_bytes ? x_bytes : 0;
        if constexpr (NTW > 1) {
            if (narrow) {
                stream_body<NTW - 1, GPU, NI, MAXW>(p, strip, 0, nt0, stream_smem, s_last);
                continue;
            }
        }
        stream_body<NTW, GPU, NI, MAXW>(p, strip, 0, nt0, stream_smem, s_last);
    }
}

// LDS layout of a launch: the waves' X regions (whole 1 KiB load instructions each), and the waves' reduction tiles
// behind them if both fit into `budget` bytes, else in the same place (red_off = 0).
inline size_t stream_lds_bytes(int ni, int mp_log, int ntw, int waves, size_t budget, int* red_off)
{
    const size_t xregion = (size_t)((((ni << mp_log) + 3) >> 2) << 10) * waves;
    const size_t red = (size_t)waves * ntw * 4 * 64 * sizeof(float);
    if (xregion + red <= budget) {
        *red_off = (int)xregion;
        return xregion + red;
    }
    *red_off = 0;
    return xregion > red ? xregion : red;
}

// Which (strip width, K-groups per unit, units per wave, CTA size) combinations exist.  A wave keeps
// NI * NTW * (4 + groups per unit) registers of packed weights and scale/zero words in flight beside 4 * NTW
// accumulators and one unit of activation fragments: CTAs of 16 waves have 128 registers per lane, CTAs of 8 waves 256
// (and are built only where 16 waves do not fit).
constexpr bool stream_built(int ntw, int gpu, int ni, int maxw)
{
    const int inflight = ni * ntw * (4 + gpu);
    return maxw == 16 ? inflight <= 64 : (inflight > 64 && inflight <= 176);
}

template <int NTW, int GPU, int NI, int MAXW>
hipError_t launch_stream_one(const GemmParams& p, const Plan& plan, size_t lds, hipStream_t stream)
{
    if constexpr (stream_built(NTW, GPU, NI, MAXW)) {
        dim3 grid(plan.strips, plan.split), block(plan.block);
        if (plan.block != MAXW * 64 || plan.split > 65535) return hipErrorInvalidValue;
        hipLaunchKernelGGL((stream_kernel<NTW, GPU, NI, MAXW>), grid, block, lds, stream, p);
        return hipGetLastError();
    } else {
        return hipErrorInvalidValue;
    }
}

// More than 64 KiB of dynamic LDS has to be allowed per kernel function; done for every built instantiation at once,
// from the library's set-up path (never from a launch, which may be under stream capture).
template <int NTW, int GPU, int NI, int MAXW>
hipError_t stream_raise_one()
{
    if constexpr (stream_built(NTW, GPU, NI, MAXW)) {
        return hipFuncSetAttribute((const void*)stream_kernel<NTW, GPU, NI, MAXW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)kStreamLdsBudget);
    } else {
        return hipSuccess;
    }
}

template <int NTW, int GPU, int NI, int MAXW>
hipError_t launch_stream_grouped_one(const GroupedParams& gp, int experts, int block, hipStream_t stream)
{
    if constexpr (stream_built(NTW, GPU, NI, MAXW)) {
        dim3 grid(gp.strips, gp.total_rows < experts ? gp.total_rows : experts);
        if (block != MAXW * 64) return hipErrorInvalidValue;
        hipLaunchKernelGGL((stream_grouped_kernel<NTW, GPU, NI, MAXW>), grid, dim3(block), gp.lds_bytes, stream, gp);
        return hipGetLastError();
    } else {
        return hipErrorInvalidValue;
    }
}

template <int NTW, int GPU, int NI, int MAXW>
hipError_t stream_grouped_raise_one()
{
    if constexpr (stream_built(NTW, GPU, NI, MAXW)) {
        return hipFuncSetAttribute((const void*)stream_grouped_kernel<NTW, GPU, NI, MAXW>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStreamLdsBudget);
    } else {
        return hipSuccess;
    }
}

template <int NTW, int NI, int MAXW>
hipError_t launch_stream_cfg(const GemmParams& p, const Plan& plan, int group, size_t lds, hipStream_t stream)
{
    switch (group) {
        case 128: return launch_stream_one<NTW, 1, NI, MAXW>(p, plan, lds, stream);
        case 64: return launch_stream_one<NTW, 2, NI, MAXW>(p, plan, lds, stream);
        case 32: return launch_stream_one<NTW, 4, NI, MAXW>(p, plan, lds, stream);
        default: return hipErrorInvalidValue;
    }
}

template <int NTW, int NI, int MAXW>
hipError_t launch_stream_grouped_cfg(const GroupedParams& gp, int experts, int group, int block, hipStream_t stream)
{
    switch (group) {
        case 128: return launch_stream_grouped_one<NTW, 1, NI, MAXW>(gp, experts, block, stream);
        case 64: return launch_stream_grouped_one<NTW, 2, NI, MAXW>(gp, experts, block, stream);
        case 32: return launch_stream_grouped_one<NTW, 4, NI, MAXW>(gp, experts, block, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

}  // namespace tmw4
