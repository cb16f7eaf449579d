// The prefill CTA tiles multiplied with the 32x32x16 matrix instruction.
//
// Same pipeline as the other CTA-tile kernels (paper Sec. 3.1 steps (i)-(iv), Sec. 4.3: X straight into an XOR-swizzled
// LDS double buffer one stage ahead, packed weights two stages ahead in rotating register sets, the fragments of the next
// MFMA step converted between the MFMAs of the current one, explicit load-counter wait and plain barrier per stage), same
// packed weight format, same wave tile of 128 rows x 64 columns and the same 128 accumulator registers.  What differs is
// the shape of the matrix instruction: a 32x32x16 MFMA does the work of two 16x16x32 ones and keeps the SIMD from issuing
// vector instructions for about as long as one of them, so the conversion's vector instructions fit into the shadow of the
// matrix work where with 16x16x32 they do not (measured on bare loops of MFMAs and independent vector instructions,
// two waves per SIMD: three vector instructions per 16x16x32-equivalent leave the pipe 97 % busy with 32x32x16 and 74 %
// with 16x16x32).  In the full kernel that does not carry over: the same number of cycles per launch as the 16x16x32 form
// and a lower clock under load, 10 % slower in all on every shape tried, so this form is launched on request only
// (tm_set_mfma_shape(32)); it stays built and under test as the record of that measurement.
//
// The packed format gives lane (c, h) of a 16-column tile the eight codes k = 32t + 8h .. 8h + 7 of column c (word t).  A
// 32x32x16 A operand wants lane (r, g) to hold row r of 32 and the contraction slots 8g .. 8g + 7.  Swapping the odd
// 16-lane rows of tile 2j's word with the even rows of tile 2j + 1's (one v_permlane16_swap on the packed words, before
// the conversion) yields two registers whose rows are [tile 2j, tile 2j+1, tile 2j, tile 2j+1]: the first holds the K
// blocks h = 0 and 2, the second h = 1 and 3, each a valid A operand over 32 columns whose slot g is the same K block for
// every row.  The X operand of the first is then X[m][32t + 16g .. + 7], of the second X[m][32t + 8 + 16g .. + 7]: the
// same LDS image, another fragment address.  The scale/zero words are swapped the same way once per group.
#include "tm_w4_tile_impl.h"

namespace tmw4 {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ f32x16 mfma32x32x16(f16x8 a, f16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// rows (16 lanes each) [a0, b0, a2, b2] and [a1, b1, a3, b3] of the two words
__device__ __forceinline__ void swap_rows(uint32_t a, uint32_t b, uint32_t& even, uint32_t& odd)
{
    const auto r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
    even = r[0];
    odd = r[1];
}

// CTA tile = 128 rows x (NW * 64) columns, NW waves of 128 x 64 each; 64-deep stages (KW = 2), weights two stages ahead.
// GPU = K-groups per 128-row unit.  No wave sets and no K split: the launches this kernel takes have neither.
template <int NW, int GPU>
__device__ __forceinline__ void tile32_body(const GemmParams& p, const int tile_m, const int tile_n)
{
    constexpr int KW = 2, PD = 2, TN = 4, NP = 2, MB = 4;
    constexpr int NT_ = NW * 64;
    constexpr int BM = 128, BN = NW * 64;
    constexpr int BKS = 32 * KW;                           // halves of K per stage
    constexpr int CPR = BKS / 8;                           // 16-byte chunks per X row and stage
    constexpr int CH = (BM * CPR) / NT_;                   // chunks per thread and stage
    static_assert((BM * CPR) % NT_ == 0, "whole chunks per thread");
    constexpr int SG = (KW * GPU) / 4 > 0 ? (KW * GPU) / 4 : 1;   // K-groups touched by one stage
    constexpr size_t kXsBytes = (size_t)BM * BKS * sizeof(uint16_t);
    __shared__ __attribute__((aligned(16))) unsigned char smem0[kXsBytes];
    __shared__ __attribute__((aligned(16))) unsigned char smem1[kXsBytes];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mrow = lane & 31, g = lane >> 5;             // operand row (of 32) and contraction half of this lane
    const Magic mg = make_magic();

    const int m0 = tile_m * BM;
    const int nt_end = min(p.NT, (tile_n + 1) * (BN / 16));
    const int nt0 = (tile_n * BN) / 16 + wave * TN;        // first 16-column tile of this wave
    const int nst = (p.KU * 4) / KW;                       // stages (the host checks that K is a whole number of them)
    const int last = nst - 1;

    f32x16 acc[MB][NP];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NP; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // X: global memory -> LDS, chunk position idx = i*NT_ + tid <-> (row idx / CPR, slot idx % CPR); slot s of row r holds
    // chunk s ^ ((r >> 1) & 7).  A fragment read of this kernel covers 32 consecutive rows x 2 chunks; timed on bare loops of
    // such reads, the swizzle by (r & 7) that serves the 16-row fragments of the other tile kernels costs these 50 % more
    // cycles (bank conflicts), the one by ((r >> 1) & 7) none.
    auto swz = [](int row) { return (row >> 1) & 7; };
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.X, (uint32_t)p.M * (uint32_t)p.K * 2u);
    uint32_t x_off[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int idx = i * NT_ + tid;
        const int row = min(m0 + idx / CPR, p.M - 1);                  // rows past M repeat the last row
        const int kc = (idx % CPR) ^ swz(idx / CPR);
        x_off[i] = (uint32_t)row * (uint32_t)p.K * 2u + (uint32_t)kc * 16u;
    }
    auto load_x = [&](int buf, int st) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int first = i * NT_ + wave * 64;         // wave-uniform: the wave's 64 chunks are contiguous in LDS
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                x_rsrc, (__attribute__((address_space(3))) void*)((buf ? smem1 : smem0) + (size_t)first * 16), 16,
                x_off[i], st * (BKS * 2), 0, 0);
#else
            (void)first;
            (void)buf;
            (void)st;
            (void)x_rsrc;
#endif
        }
    };
    // X operand of MFMA step tt, K blocks `half` (0: h = 0 and 2, 1: h = 1 and 3), row block mb: lane (mrow, g) wants
    // chunk 4tt + 2g + half of row 32mb + mrow, which sits in slot chunk ^ swz(mrow) (32mb does not change the swizzle).
    uint32_t xd[KW][2];
#pragma unroll
    for (int tt = 0; tt < KW; ++tt)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
            xd[tt][hf] = (uint32_t)mrow * (BKS * 2) + (((uint32_t)(4 * tt + 2 * g + hf)) ^ (uint32_t)swz(mrow)) * 16u;
    auto x_frag = [&](int buf, int tt, int hf, int mb) -> const f16x8* {
        return (const f16x8*)((buf ? smem1 : smem0) + xd[tt][hf] + mb * (32 * BKS * 2));
    };

    const uint32_t w_lane = (uint32_t)lane * 16u, sz_lane = (uint32_t)(lane & 15) * 4u;
    uint32_t wset[PD + 1][TN][KW];
    uint32_t sset[PD + 1][TN][SG];
    __amdgpu_buffer_rsrc_t w_rsrc[TN], s_rsrc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const bool live = nt0 + j < nt_end;                // wave-uniform
        const int nt = min(nt0 + j, nt_end - 1);
        w_rsrc[j] = make_rsrc((const char*)p.W + (size_t)nt * p.KU * 1024, live ? (uint32_t)p.KU * 1024u : 0u);
        s_rsrc[j] = make_rsrc((const char*)p.SZ + (size_t)nt * p.G * 64, live ? (uint32_t)p.G * 64u : 0u);
    }
    auto load_w = [&](uint32_t (&w)[TN][KW], uint32_t (&s)[TN][SG], int st) {
        const int wbyte = ((st * KW) / 4) * 1024 + ((st * KW) % 4) * 4;
        const int grp0 = (st * KW * GPU) / 4;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int gq = 0; gq < SG; ++gq)
                s[j][gq] = __builtin_amdgcn_raw_buffer_load_b32(s_rsrc[j], sz_lane, (grp0 + gq) * 64, 0);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(w_rsrc[j], w_lane, wbyte, 0);
            w[j][0] = v.x;
            w[j][1] = v.y;
        }
    };

    // The two A operands of column pair np (16-column tiles 2np and 2np + 1) for MFMA step tt.
    auto convert_pair = [&](const uint32_t (&w)[TN][KW], const uint32_t (&s)[TN][SG], int tt, int np, f16x8& fa, f16x8& fb) {
        uint32_t wa, wb, sa, sb;
        swap_rows(w[2 * np][tt], w[2 * np + 1][tt], wa, wb);
        swap_rows(s[2 * np][(tt * GPU) / 4 % SG], s[2 * np + 1][(tt * GPU) / 4 % SG], sa, sb);
        (void)sb;                                          // both results carry [tile 2np, tile 2np+1, ...]: the words are equal along h
        const GroupConst gc = make_group_const(sa);
        fa = dequant8(wa, gc, mg);
        fb = dequant8(wb, gc, mg);
    };

    // One 32-deep MFMA step over the wave's 128 x 64 tile: four row blocks x two column pairs x two K halves, the
    // operands of the next step converted one column pair per two row blocks, X fragments read one row block ahead.
    auto step = [&](int buf, int tt, const f16x8 (&ca)[NP], const f16x8 (&cb)[NP], f16x8 (&na)[NP], f16x8 (&nb)[NP],
                    const uint32_t (&wsrc)[TN][KW], const uint32_t (&ssrc)[TN][SG], int tt_next) {
        f16x8 xa = *x_frag(buf, tt, 0, 0);
        f16x8 xb = *x_frag(buf, tt, 1, 0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            f16x8 ya = xa, yb = xb;
            if (mb + 1 < MB) {
                ya = *x_frag(buf, tt, 0, mb + 1);
                yb = *x_frag(buf, tt, 1, mb + 1);
            }
            if (mb == 0) convert_pair(wsrc, ssrc, tt_next, 0, na[0], nb[0]);
            if (mb == 2) convert_pair(wsrc, ssrc, tt_next, 1, na[1], nb[1]);
#pragma unroll
            for (int np = 0; np < NP; ++np) acc[mb][np] = mfma32x32x16(ca[np], xa, acc[mb][np]);
#pragma unroll
            for (int np = 0; np < NP; ++np) acc[mb][np] = mfma32x32x16(cb[np], xb, acc[mb][np]);
            __builtin_amdgcn_sched_barrier(0);
            xa = ya;
            xb = yb;
        }
    };

    {
        f16x8 fa0[NP], fb0[NP], fa1[NP], fb1[NP];
        constexpr int kWLoads = TN * SG + TN;
        auto stage_barrier = [&](auto NLOADS) {
            constexpr int n = decltype(NLOADS)::value < 63 ? decltype(NLOADS)::value : 63;
            // vmcnt = n (the X loads of the next stage are older than the last n weight loads), lgkmcnt = 0
            __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | (7 << 4) | (0 << 8));
            __builtin_amdgcn_s_barrier();
        };
        load_x(0, 0);
        __builtin_amdgcn_sched_barrier(0);
        load_w(wset[0], sset[0], 0);
        static_for<1, PD>([&](auto R) {
            constexpr int r = decltype(R)::value;
            load_w(wset[r % (PD + 1)], sset[r % (PD + 1)], min(r, last));
        });
#pragma unroll
        for (int np = 0; np < NP; ++np) convert_pair(wset[0], sset[0], 0, np, fa0[np], fb0[np]);
        stage_barrier(std::integral_constant<int, PD * kWLoads>{});
        constexpr int PERIOD = PD * (PD + 1);
        for (int base = 0; base < nst; base += PERIOD) {
            static_for<0, PERIOD>([&](auto PH) {
                constexpr int ph = decltype(PH)::value;
                const int r = base + ph;
                if (r < nst) {
                    constexpr int wi = ph % (PD + 1);              // W(r)
                    constexpr int wn = (ph + 1) % (PD + 1);        // W(r + 1)
                    constexpr int wf = (ph + PD) % (PD + 1);       // set that takes W(r + PD)
                    constexpr int buf = ph & 1;                    // = r & 1: PERIOD is even
                    load_x(buf ^ 1, min(r + 1, last));
                    __builtin_amdgcn_sched_barrier(0);
                    load_w(wset[wf], sset[wf], min(r + PD, last));
                    // the scale/zero words of the next stage stay opaque until the step that first needs them, or the
                    // compiler derives their constants right after the loads that fetch them
                    step(buf, 0, fa0, fb0, fa1, fb1, wset[wi], sset[wi], 1);
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int gq = 0; gq < SG; ++gq) asm volatile("" : "+v"(sset[wn][j][gq]));
                    step(buf, 1, fa1, fb1, fa0, fb0, wset[wn], sset[wn], 0);
                    stage_barrier(std::integral_constant<int, kWLoads>{});
                }
            });
        }
    }

    // Epilogue.  acc[mb][np][4i + r] = Y[m0 + 32mb + mrow][16*(nt0 + 2np + i/2) + 8*(i%2) + 4g + r]: register group i of
    // a 32x32 result holds rows 8i + 4g .. + 3 of the A side, i.e. four consecutive columns of Y.
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m0 + 32 * mb + mrow;
        if (m >= p.M) continue;
#pragma unroll
        for (int np = 0; np < NP; ++np)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int nt = nt0 + 2 * np + (i >> 1);
                if (nt >= nt_end) continue;
                store_quad(p, m, nt * 16 + 8 * (i & 1) + 4 * g, acc[mb][np][4 * i + 0], acc[mb][np][4 * i + 1],
                           acc[mb][np][4 * i + 2], acc[mb][np][4 * i + 3]);
            }
    }
}

template <int NW, int GPU>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void tile32_kernel(GemmParams p)
{
    // XCD-aware numbering, as in the other CTA-tile kernels
    const int tiles = p.tiles_m * p.tiles_n;
    const int chunk = (tiles + 7) / 8;
    const int b = blockIdx.x % (chunk * 8);
    const int logical = (b % 8) * chunk + b / 8;
    if (logical >= tiles || blockIdx.x >= chunk * 8) return;
    const int panel_tiles = kPanelN * p.tiles_m;
    const int panel = logical / panel_tiles;
    const int within = logical % panel_tiles;
    const int pw = min(kPanelN, p.tiles_n - panel * kPanelN);
    const int tile_m = within / pw, tile_n = panel * kPanelN + within % pw;
    tile32_body<NW, GPU>(p, tile_m, tile_n);
}

template <int NW>
hipError_t launch_nw(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    dim3 grid(plan.grid), block(NW * 64);
    // what the kernel assumes: one K range of whole 64-deep stages, one wave set, its own CTA size
    if (plan.block != NW * 64 || plan.split != 1 || plan.kgroups != 1 || plan.stage_steps != 2 || p.split != 1 || (p.KU * 4) % 2)
        return hipErrorInvalidValue;
    switch (group) {
        case 128: hipLaunchKernelGGL((tile32_kernel<NW, 1>), grid, block, 0, stream, p); break;
        case 64: hipLaunchKernelGGL((tile32_kernel<NW, 2>), grid, block, 0, stream, p); break;
        case 32: hipLaunchKernelGGL((tile32_kernel<NW, 4>), grid, block, 0, stream, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_tile32(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    switch (plan.variant) {
        case kTile128x256: return launch_nw<4>(p, plan, group, stream);
        case kTile128x512: return launch_nw<8>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
