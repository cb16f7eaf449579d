// Templates of the decode ("skinny") kernels, shared by the translation units that instantiate them for 4-bit and
// 8-bit weights.
#pragma once
#include "tm_w4_host.h"

namespace tmw4 {

namespace {

// A packed unit is 1 KiB per 16-column tile whatever the weight width: 128 rows of 4-bit codes or 64 rows of 8-bit
// codes, i.e. T = 4 or 2 matrix-core k-steps.  GPU counts K-groups per 128 rows (1, 2, 4 for groups of 128, 64, 32);
// GU is the number of groups inside one unit, SZDIV the number of units that share a group (8-bit, group 128).
template <int BITS, int GPU>
struct UnitShape {
    static constexpr int T = BITS == 4 ? 4 : 2;
    static constexpr int GU = BITS == 4 ? GPU : (GPU >= 2 ? GPU / 2 : 1);
    static constexpr int SZDIV = (BITS != 4 && GPU == 1) ? 2 : 1;
};

template <int TM, int NTW, int GU, int T>
struct Stage {
    u32x4 wq[NTW];              // packed weights: 4 words per lane and n-tile
    uint32_t sz[NTW][GU];       // scale|zero words of the groups inside the unit
    u32x4 xf[TM][T];            // activation fragments for the unit's MFMA k-steps
};

// Per-lane byte offsets that do not change over the K loop; everything else in an address is wave-uniform and
// stays in scalar registers, so a load costs no vector address arithmetic.
template <int TM>
struct LaneOffsets {
    uint32_t w;                 // lane * 16 inside a 1 KiB unit
    uint32_t sz;                // (lane % 16) * 4 inside a 64-byte scale/zero row
    uint32_t x[TM];             // row(mt, lane) * K * 2 + (lane / 16) * 16 inside X
    bool live[TM];              // row(mt, lane) < M: only these lanes load activations
};

template <int SZDIV, int TM, int NTW, int GU, int T>
__device__ __forceinline__ void load_weights(Stage<TM, NTW, GU, T>& st, const GemmParams& p, const LaneOffsets<TM>& lo,
                                             int nt0, int ntw, int ku)
{
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        const int nt = nt0 + j;                    // wave-uniform
        if (j < ntw) {
            const char* wb = (const char*)p.W + ((size_t)nt * p.KU + ku) * 1024;
            st.wq[j] = __builtin_nontemporal_load((const u32x4*)(wb + lo.w));
            const char* sb = (const char*)p.SZ + ((size_t)nt * p.G + (size_t)(ku / SZDIV) * GU) * 64;
#pragma unroll
            for (int g = 0; g < GU; ++g) st.sz[j][g] = *(const uint32_t*)(sb + g * 64 + lo.sz);
        } else {
            st.wq[j] = u32x4{0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < GU; ++g) st.sz[j][g] = 0;
        }
    }
}

template <int TM, int NTW, int GU, int T>
__device__ __forceinline__ void load_activations(Stage<TM, NTW, GU, T>& st, const GemmParams& p,
                                                 const LaneOffsets<TM>& lo, int ku)
{
    const char* xb = (const char*)p.X + (size_t)ku * (32 * T * 2);
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int t = 0; t < T; ++t) {              // k = 32*T*ku + 32*t + 8*h .. +7
            // Lanes whose row is past M keep an unspecified value instead of loading: row i of an MFMA result
            // depends only on row i of this operand, and rows past M are never stored.
            u32x4 v = __builtin_nondeterministic_value(v);
            if (lo.live[mt]) v = *(const u32x4*)(xb + lo.x[mt] + 64 * t);
            st.xf[mt][t] = v;
        }
}

template <int SZDIV, int TM, int NTW, int GU, int T>
__device__ __forceinline__ void load_stage(Stage<TM, NTW, GU, T>& st, const GemmParams& p, const LaneOffsets<TM>& lo,
                                           int nt0, int ntw, int ku)
{
    load_weights<SZDIV>(st, p, lo, nt0, ntw, ku);
    load_activations(st, p, lo, ku);
}

// One unit of NTW column tiles.  Paper Sec. 3.1 step (iii) / Sec. 4.3 split differently between the units of the
// CU than in the paper: the vector ALU only does the bit manipulation (biased8: 5 instructions per 8 weights);
// the conversion bias and the zero-point are removed by a second MFMA against a constant operand, and the group
// scale multiplies the fp32 group sum.  The decode kernels are bound by HBM and by vector-ALU issue, while the
// matrix cores idle, so moving the subtract and the multiply off the ALU is what brings the per-weight ALU cost
// under the HBM budget.
//
// With four row tiles (M up to 64) the extra MFMAs would cost more matrix-core time than the conversion costs ALU
// time, so that configuration converts on the ALU as the tile kernels do (dequant8: exact subtract, one rounded
// multiply) and accumulates straight into the output tile.
//
// 8-bit codes take the same two routes with their own bit manipulation (one byte permute per two weights).
template <int BITS, int TM, int NTW, int GU, int T>
__device__ __forceinline__ void compute_stage(const Stage<TM, NTW, GU, T>& st, f32x4 (&acc)[TM][NTW], const Magic& mg)
{
    constexpr int TG = T / GU;                     // MFMA k-steps per K-group
    if constexpr (TM >= 4) {
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
            GroupConst gc[GU];
#pragma unroll
            for (int g = 0; g < GU; ++g) gc[g] = make_group_const(st.sz[j][g]);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                f16x8 b;
                if constexpr (BITS == kFmtInt4) {
                    b = dequant8(st.wq[j][t], gc[t / TG], mg);
                } else if constexpr (BITS == kFmtInt8) {
                    b = dequant8_w8(st.wq[j][2 * t], st.wq[j][2 * t + 1], gc[t / TG]);
                } else {                           // FP8: exact conversion, one rounded multiply by the scale
                    const f16x8 v = cvt8_fp8(st.wq[j][2 * t], st.wq[j][2 * t + 1]);
                    const _Float16 sc = gc[t / TG].s2.x;
                    b = v * f16x8{sc, sc, sc, sc, sc, sc, sc, sc};
                }
#pragma unroll
                for (int mt = 0; mt < TM; ++mt)
                    acc[mt][j] = mfma16x16x32(__builtin_bit_cast(f16x8, st.xf[mt][t]), b, acc[mt][j]);
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
#pragma unroll
        for (int g = 0; g < GU; ++g) {
            const f16x2 szp = as_f16x2(st.sz[j][g]);
            const f16x8 cancel = BITS == kFmtInt4 ? bias_cancel8(szp.y) : bias_cancel8_w8(szp.y);   // unused for FP8
            const float scale = (float)szp.x;
            f32x4 part[TM];
#pragma unroll
            for (int mt = 0; mt < TM; ++mt) part[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int tt = 0; tt < TG; ++tt) {
                const int t = g * TG + tt;
                f16x8 b;
                if constexpr (BITS == kFmtInt4) b = biased8(st.wq[j][t], mg);
                else if constexpr (BITS == kFmtInt8) b = biased8_w8(st.wq[j][2 * t], st.wq[j][2 * t + 1]);
                else b = cvt8_fp8(st.wq[j][2 * t], st.wq[j][2 * t + 1]);
#pragma unroll
                for (int mt = 0; mt < TM; ++mt) {
                    const f16x8 a = __builtin_bit_cast(f16x8, st.xf[mt][t]);
                    part[mt] = mfma16x16x32(a, b, part[mt]);
                    if constexpr (BITS != kFmtFp8) part[mt] = mfma16x16x32(a, cancel, part[mt]);
                }
            }
#pragma unroll
            for (int mt = 0; mt < TM; ++mt) acc[mt][j] += scale * part[mt];
        }
    }
}

// The waves of a CTA hold partial tiles of the same outputs (each wave multiplied its own units of K): add them through
// LDS and store, or, when K is also split across CTAs, hand the CTA's sums to the split-K merge.
// red is [waves][NTW*4][64] floats of LDS (one 16 x 16*NTW fp32 tile per wave), s_last one LDS word.
template <int TM, int NTW>
__device__ __forceinline__ void skinny_reduce(const GemmParams& p, f32x4 (&acc)[TM][NTW], const int strip, const int sk,
                                              const int nt0, const int ntw, float* __restrict__ red, uint32_t& s_last)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int waves = blockDim.x >> 6;
    // Reduce the waves' tiles through LDS, one 16-row tile at a time.  A wave stores its accumulator registers as
    // they are (register-major, 64 lanes contiguous), and the readers keep that shape: reader thread e owns
    // accumulator element (register e / 64, lane e % 64), so the 64 lanes of a reading wave fetch 64 consecutive
    // floats per source wave, free of bank conflicts.  In the accumulator layout lane l holds column l % 16 of rows
    // 4*(l / 16) + r; even lanes fetch their right-hand neighbour's sum and store two fp16 columns at once.
    constexpr int kElems = NTW * 4 * 64;
    const int nthreads = blockDim.x;
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
        if (mt) __syncthreads();
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[(wave * NTW * 4 + j * 4 + r) * 64 + lane] = acc[mt][j][r];
        __syncthreads();
        for (int e = tid; e < kElems; e += nthreads) {      // whole waves enter or skip an iteration
            const int reg = e >> 6;
            const int j = reg >> 2;
            const int m = mt * 16 + 4 * (lane >> 4) + (reg & 3);
            const bool mine = m < p.M && j < ntw;
            float v = 0.f;
            if (mine)
                for (int w = 0; w < waves; ++w) v += red[(w * NTW * 4 + reg) * 64 + lane];
            const float vr = __shfl_xor(v, 1);
            if (!mine || (lane & 1)) continue;
            const int n = (nt0 + j) * 16 + (lane & 15);
            if (p.split == 1) {
                store_pair(p, m, n, v, vr);
            } else {
                st_partial2(p.partial + ((size_t)sk * p.strips + strip) * p.slot_floats + (mt * NTW * 4 + reg) * 64 + lane, v, vr);
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
            constexpr int kPairs = 8 * NTW;        // column pairs per row of the 16 x 16*NTW tile
            constexpr int kSlots = 16 * kPairs;
#pragma unroll
            for (int mt = 0; mt < TM; ++mt) {
                for (int slot = tid; slot < kSlots; slot += nthreads) {
                    const int row = slot / kPairs;
                    const int col = (slot % kPairs) * 2;
                    const int m = mt * 16 + row;
                    if (m >= p.M || col >= ntw * 16) continue;
                    const int n = nt0 * 16 + col;
                    float v0, v1;
                    // the slot keeps the accumulator order: register (col / 16) * 4 + row % 4, lane 16 * (row / 4) + col % 16
                    const int at = (mt * NTW * 4 + (col >> 4) * 4 + (row & 3)) * 64 + 16 * (row >> 2) + (col & 15);
                    sum_partials2(p.partial + (size_t)strip * p.slot_floats + at, (size_t)p.strips * p.slot_floats, p.split, v0, v1);
                    store_pair(p, m, n, v0, v1);
                }
            }
            if (tid == 0) __hip_atomic_store(&p.counters[strip], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// TM 16-row tiles, NTW 16-column tiles per wave, GPU K-groups per 128-row unit, D register stages per wave,
// MAXW the largest CTA (in waves) this instantiation is launched with.
//
// One CTA's work on one GEMM: column strip `strip` of p.strips, K slice `sk` of p.split.
// red is [waves][NTW*4][64] floats of LDS (one 16 x 16*NTW fp32 tile per wave), s_last one LDS word.
template <int TM, int NTW, int GPU, int D, int BITS>
__device__ __forceinline__ void skinny_body(const GemmParams& p, const int strip, const int sk, float* __restrict__ red,
                                            uint32_t& s_last)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform by construction
    const int waves = blockDim.x >> 6;
    // The NT column tiles are dealt evenly into p.strips strips (widths differ by at most one tile), so that a
    // shape whose tile count is not a multiple of the CU count still loads every CU almost equally.  Quotient and
    // remainder come from the host: a division here would stand between every wave and its first load.
    const int nt0 = strip * p.strip_base + min(strip, p.strip_rem);
    const int ntw = p.strip_base + (strip < p.strip_rem ? 1 : 0);          // <= NTW (host guarantees)
    const int ku0 = sk * p.ku_per_split;
    const int ku1 = min(p.KU, ku0 + p.ku_per_split);

    const Magic mg = make_magic();
    LaneOffsets<TM> lo;
    lo.w = lane * 16;
    lo.sz = (lane & 15) * 4;
#pragma unroll
    for (int mt = 0; mt < TM; ++mt) {
        const int row = mt * 16 + (lane & 15);
        lo.live[mt] = row < p.M;
        lo.x[mt] = (uint32_t)row * (uint32_t)p.K * 2u + (lane >> 4) * 16;
    }

    f32x4 acc[TM][NTW];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int j = 0; j < NTW; ++j) acc[mt][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Rolling prefetch (the memory pipeline of paper Sec. 4.3): a ring of D register stages; while the unit in
    // stage r is converted and multiplied, the loads of the next D-1 units of this wave are in flight.
    {
        using US = UnitShape<BITS, GPU>;
        Stage<TM, NTW, US::GU, US::T> st[D];
        const int first = ku0 + wave;
#pragma unroll
        for (int r = 0; r < D - 1; ++r)
            if (first + r * waves < ku1) load_stage<US::SZDIV>(st[r], p, lo, nt0, ntw, first + r * waves);
        for (int base = first; base < ku1; base += D * waves) {
#pragma unroll
            for (int r = 0; r < D; ++r) {
                const int cur = base + r * waves;
                if (cur < ku1) {
                    const int pre = cur + (D - 1) * waves;
                    if (pre < ku1) load_stage<US::SZDIV>(st[(r + D - 1) % D], p, lo, nt0, ntw, pre);
                    compute_stage<BITS>(st[r], acc, mg);
                }
            }
        }
    }

    skinny_reduce<TM, NTW>(p, acc, strip, sk, nt0, ntw, red, s_last);
}

template <int TM, int NTW, int GPU, int D, int MAXW, int BITS = 4>
__global__ __launch_bounds__(MAXW * 64) void skinny_kernel(GemmParams p)
{
    extern __shared__ float red[];
    __shared__ uint32_t s_last;
    skinny_body<TM, NTW, GPU, D, BITS>(p, blockIdx.x, blockIdx.y, red, s_last);
}

// The `which`-th expert that has rows: its row range and the addresses of its packed weights and scale/zero words.
// Every wave scans the offsets 64 experts at a time; each lane also fetches its candidate's two table entries, so that the
// scan, the row range and the buffer addresses cost a single round trip to memory.
struct ExpertRows {
    int r0, r1;
    uint64_t w, sz;
    bool found;
};
__device__ __forceinline__ ExpertRows find_expert(const GroupedParams& gp, int which, int lane)
{
    ExpertRows er{0, 0, 0, 0, false};
    int want = which;                               // index among the experts with rows that is still to be skipped
    for (int base = 0; base < gp.experts; base += 64) {
        const int e = base + lane;
        int a = 0, b = 0;
        uint64_t tw = 0, ts = 0;
        if (e < gp.experts) {
            a = gp.offsets[e];
            b = gp.offsets[e + 1];
            tw = gp.table[2 * e];
            ts = gp.table[2 * e + 1];
        }
        a = min(max(a, 0), gp.total_rows);          // rows are clamped to the buffers whatever the offsets hold
        b = min(b, gp.total_rows);
        const bool has_rows = b > a;
        const uint64_t mask = __ballot(has_rows);
        const int count = __popcll(mask);
        if (want < count) {
            const int before = __popcll(mask & ((1ull << lane) - 1ull));
            const uint64_t hit = __ballot(has_rows && before == want);
            const int src = __builtin_ctzll(hit);   // exactly one lane
            er.r0 = __builtin_amdgcn_readlane(a, src);
            er.r1 = __builtin_amdgcn_readlane(b, src);
            er.w = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(tw >> 32), src) << 32) |
                   (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)tw, src);
            er.sz = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(ts >> 32), src) << 32) |
                    (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)ts, src);
            er.found = true;
            break;
        }
        want -= count;
    }
    return er;
}

// What of a launch's parameters is the same for every expert.
__device__ __forceinline__ GemmParams expert_params(const GroupedParams& gp, const ExpertRows& er)
{
    GemmParams p{};
    p.W = (const u32x4*)er.w;
    p.SZ = (const uint32_t*)er.sz;
    p.K = gp.K;
    p.N = gp.N;
    p.ldy = gp.act ? gp.N / 2 : gp.N;
    p.act = gp.act;
    p.epi = gp.act;
    p.KU = gp.KU;
    p.NT = gp.NT;
    p.G = gp.G;
    p.split = 1;
    p.ku_per_split = gp.KU;
    p.strips = gp.strips;
    p.strip_base = gp.strip_base;
    p.strip_rem = gp.strip_rem;
    return p;
}

// Grouped form for mixture-of-experts layers (the paper's evaluation covers MoE models, Sec. 5.1; their expert GEMMs
// are this same GEMM once per expert): rows [offsets[e], offsets[e+1]) of X and Y belong to expert e, whose packed
// weights the pointer table names.  blockIdx.x is the strip, blockIdx.y selects among the experts that have rows
// (the grid is only as tall as the number of experts that can be active, min(experts, rows)).
// Experts with more than 16*TM rows are taken 16*TM rows at a time.
template <int TM, int NTW, int GPU, int D, int MAXW, int BITS = 4>
__global__ __launch_bounds__(MAXW * 64) void skinny_grouped_kernel(GroupedParams gp)
{
    extern __shared__ float red[];
    __shared__ uint32_t s_last;
    const ExpertRows er = find_expert(gp, blockIdx.y, threadIdx.x & 63);
    const int r0 = er.r0, r1 = er.r1;
    const bool found = er.found;
    if (!found) return;                             // fewer experts have rows than the grid is tall
    GemmParams p = expert_params(gp, er);
    for (int m0 = r0; m0 < r1; m0 += 16 * TM) {
        if (m0 != r0) __syncthreads();             // the previous chunk's reads of red are done
        p.X = gp.X + (size_t)m0 * gp.K;
        p.Y = gp.Y + (size_t)m0 * p.ldy;
        p.M = min(16 * TM, r1 - m0);
        skinny_body<TM, NTW, GPU, D, BITS>(p, blockIdx.x, 0, red, s_last);
    }
}

// D128 / DSMALL: register stages per wave for group 128 and for the smaller groups (which carry more scale/zero
// words per unit and would spill with the deeper ring).
template <int TM, int NTW, int D128, int DSMALL, int MAXW, int BITS = 4>
hipError_t launch_cfg(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    dim3 grid(plan.strips, plan.split), block(plan.block);           // x: column strip, y: K slice
    if (plan.block > MAXW * 64 || plan.split > 65535) return hipErrorInvalidValue;
    size_t lds = (size_t)(plan.block / 64) * NTW * 4 * 64 * sizeof(float);
    switch (group) {
        case 128: hipLaunchKernelGGL((skinny_kernel<TM, NTW, 1, D128, MAXW, BITS>), grid, block, lds, stream, p); break;
        case 64: hipLaunchKernelGGL((skinny_kernel<TM, NTW, 2, DSMALL, MAXW, BITS>), grid, block, lds, stream, p); break;
        case 32: hipLaunchKernelGGL((skinny_kernel<TM, NTW, 4, DSMALL, MAXW, BITS>), grid, block, lds, stream, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int TM, int NTW, int D128, int DSMALL, int BITS = 4>
hipError_t launch_grouped_cfg(const GroupedParams& gp, int experts, int group, hipStream_t stream)
{
    dim3 grid(gp.strips, gp.total_rows < experts ? gp.total_rows : experts), block(512);
    size_t lds = (size_t)8 * NTW * 4 * 64 * sizeof(float);
    switch (group) {
        case 128: hipLaunchKernelGGL((skinny_grouped_kernel<TM, NTW, 1, D128, 8, BITS>), grid, block, lds, stream, gp); break;
        case 64: hipLaunchKernelGGL((skinny_grouped_kernel<TM, NTW, 2, DSMALL, 8, BITS>), grid, block, lds, stream, gp); break;
        case 32: hipLaunchKernelGGL((skinny_grouped_kernel<TM, NTW, 4, DSMALL, 8, BITS>), grid, block, lds, stream, gp); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Eight-wave CTAs only: with one grid row per expert there are several CTAs per CU to overlap.
template <int BITS>
hipError_t launch_skinny_grouped_fmt(const GroupedParams& gp, int variant, int experts, int group, hipStream_t stream)
{
    if (experts <= 0 || experts > 65535 || gp.strips <= 0) return hipErrorInvalidValue;
    switch (variant) {
        case kSkinny16x16: return launch_grouped_cfg<1, 1, 4, 4, BITS>(gp, experts, group, stream);
        case kSkinny16x32: return launch_grouped_cfg<1, 2, 4, 4, BITS>(gp, experts, group, stream);
        case kSkinny16x64: return launch_grouped_cfg<1, 4, 2, 2, BITS>(gp, experts, group, stream);
        case kSkinny16x128: return launch_grouped_cfg<1, 8, 2, BITS == 4 ? 1 : 2, BITS>(gp, experts, group, stream);
        case kSkinny32x64: return launch_grouped_cfg<2, 4, 2, 2, BITS>(gp, experts, group, stream);
        case kSkinny64x64: return launch_grouped_cfg<4, 4, BITS == 4 ? 1 : 2, 1, BITS>(gp, experts, group, stream);
        default: return hipErrorInvalidValue;
    }
}

// The strip widths the dispatcher uses for the 8-bit formats (BITS = kFmtInt8 or kFmtFp8).
template <int BITS>
hipError_t launch_skinny_8bit(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    const bool w16 = plan.block > 512;
    switch (plan.variant) {
        case kSkinny16x16: return w16 ? launch_cfg<1, 1, 3, 2, 16, BITS>(p, plan, group, stream) : launch_cfg<1, 1, 4, 4, 8, BITS>(p, plan, group, stream);
        case kSkinny16x32: return w16 ? launch_cfg<1, 2, 2, 2, 16, BITS>(p, plan, group, stream) : launch_cfg<1, 2, 4, 4, 8, BITS>(p, plan, group, stream);
        case kSkinny16x48: return w16 ? launch_cfg<1, 3, 2, 2, 16, BITS>(p, plan, group, stream) : launch_cfg<1, 3, 3, 3, 8, BITS>(p, plan, group, stream);
        case kSkinny16x64: return w16 ? launch_cfg<1, 4, 2, 1, 16, BITS>(p, plan, group, stream) : launch_cfg<1, 4, 2, 2, 8, BITS>(p, plan, group, stream);
        case kSkinny16x96: return w16 ? launch_cfg<1, 6, 1, 1, 16, BITS>(p, plan, group, stream) : launch_cfg<1, 6, 3, 2, 8, BITS>(p, plan, group, stream);
        case kSkinny16x128: return w16 ? launch_cfg<1, 8, 1, 1, 16, BITS>(p, plan, group, stream) : launch_cfg<1, 8, 2, 2, 8, BITS>(p, plan, group, stream);
        case kSkinny32x64: return w16 ? hipErrorInvalidValue : launch_cfg<2, 4, 2, 2, 8, BITS>(p, plan, group, stream);
        case kSkinny64x64: return w16 ? hipErrorInvalidValue : launch_cfg<4, 4, 2, 1, 8, BITS>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

}  // namespace tmw4
