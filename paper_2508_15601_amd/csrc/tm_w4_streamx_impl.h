// Decode kernels, one-shot form, for more than 16 rows (16 < M <= 16 * TM, TM = 2 or 4 row tiles).
//
// Same organisation as the one-shot kernels for M <= 16 (tm_w4_stream_impl.h; paper Sec. 3.1 steps (i)-(iv), Sec. 4.3's
// memory pipeline as deep as the K range): one CTA per column strip, the waves split K, a wave issues every weight load
// of its K units at once and multiplies as the bytes arrive, no CTA barrier before the arithmetic.  What changes with
// more rows is X: M x K fp16 values no longer fit into LDS, so every wave keeps a two-slot ring of "pieces" there -
// the 16 * TM rows of X for half a packed unit of K (64 values = one 128-byte line per row) - and refills a slot with
// direct-to-LDS loads as soon as the piece in it has been multiplied.  The two slots are two separate LDS objects, so
// that the compiler can tell a refill of one from the fragment reads of the other.
//
// Conversion is the tile kernels' (I2F by bit manipulation, exact subtract of the zero-point, one rounded multiply by
// the scale): with two or four row tiles per converted fragment the second MFMA that cancels the conversion bias in
// the M <= 16 kernels would double the matrix work, which is no longer free.
//
// LDS image of a piece: [row r < 16 * TM][8 chunks of 16 bytes]; chunk q of row r sits in slot q ^ (r & 7), so that the
// eight lanes a 128-bit LDS read serves together fall into eight different 16-byte bank groups.
#pragma once
#include "tm_w4_stream_impl.h"

namespace tmw4 {

namespace {

template <int TM, int NTW, int GPU, int NI, int WAVES>
__device__ __forceinline__ void rows_body(const GemmParams& p, const int strip, const int sk, const int nt0,
                                          unsigned char* __restrict__ xs0, unsigned char* __restrict__ xs1, uint32_t& s_last)
{
    constexpr int GU = GPU;                        // K-groups per 128-row unit
    constexpr int TG = 4 / GU;                     // MFMA k-steps per K-group
    constexpr int kPiece = 16 * TM * 128;          // bytes of one piece
    constexpr int kPieceLoads = kPiece / 1024;     // load instructions per piece (64 lanes x 16 bytes each)
    constexpr int Q = 2 * NI;                      // pieces per wave
    constexpr int kWLoads = NI * NTW * (GU + 1);   // weight and scale/zero load instructions per wave
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, h = lane >> 4;
    const int ku0 = sk * p.ku_per_split;
    const int kus = min(p.KU, ku0 + p.ku_per_split) - ku0;         // packed units in this K slice
    const Magic mg = make_magic();
    unsigned char* const slot0 = xs0 + (size_t)wave * kPiece;
    unsigned char* const slot1 = xs1 + (size_t)wave * kPiece;

    // ---- piece q of this wave: half (q & 1) of its unit q >> 1.  One load instruction moves eight rows of 128 bytes
    // to 1 KiB of consecutive LDS.  Rows at and past M and units past the K slice get an offset outside the descriptor:
    // zeros are written and no memory is touched.
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.X, (uint32_t)p.M * (uint32_t)p.K * 2u);
    const uint32_t k2 = (uint32_t)p.K * 2u;
    // per-lane byte offset of each of a piece's loads, without the K part (the host admits this kernel only where
    // M * K * 2 < 2^31, so 0x80000000 lies outside the descriptor)
    uint32_t x_off[kPieceLoads];
#pragma unroll
    for (int e = 0; e < kPieceLoads; ++e) {
        const int row = 8 * e + (lane >> 3);
        const int qch = (lane & 7) ^ (row & 7);
        x_off[e] = row < p.M ? (uint32_t)row * k2 + (uint32_t)qch * 16u : 0x80000000u;
    }
    auto load_piece = [&](int q, unsigned char* slot) {
        const int ul = wave + (q >> 1) * WAVES;                    // wave-uniform
        const bool in = ul < kus;
        const uint32_t kbyte = (uint32_t)(ku0 + ul) * 256u + (uint32_t)(q & 1) * 128u;
#pragma unroll
        for (int e = 0; e < kPieceLoads; ++e) {
            const uint32_t off = in ? x_off[e] + kbyte : 0x80000000u;      // rows past M stay outside: kbyte < 2^31
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(x_rsrc, (__attribute__((address_space(3))) void*)(slot + e * 1024), 16, off,
                                                     0, 0, 0);
#else
            (void)off;
            (void)slot;
            (void)x_rsrc;
#endif
        }
    };
    load_piece(0, slot0);
    load_piece(1, slot1);
    __builtin_amdgcn_sched_barrier(0);             // the counts in the waits below are exact only if nothing moves across

    // ---- every weight load of this wave, in the order of use
    StreamRegs<NTW, GU, NI> st;
    {
        const uint32_t w_lane = (uint32_t)lane * 16u, s_lane = (uint32_t)c * 4u;
        const char* wbase = (const char*)p.W + (size_t)nt0 * p.KU * 1024;
        const char* sbase = (const char*)p.SZ + (size_t)nt0 * p.G * 64;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int ul = wave + i * WAVES;
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

    f32x4 acc[TM][NTW];
#pragma unroll
    for (int im = 0; im < TM; ++im)
#pragma unroll
        for (int j = 0; j < NTW; ++j) acc[im][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // fragment of MFMA step t2 (0 or 1) of a piece, row tile im: lane (c, h) reads chunk 4 * t2 + h of row 16 * im + c
    const uint32_t x_rd = (uint32_t)c * 128u;
    const uint32_t x_swz = (uint32_t)(c & 7);

    // ---- piece by piece.  The load counter retires in order, so "at most n loads outstanding" with n = the loads
    // issued after a piece's own means that piece has landed.  Pieces 0 and 1 are older than the weight loads; every
    // later piece is younger than all of them and than everything but the one refill issued after it.
    static_for<0, Q>([&](auto QI) {
        constexpr int q = decltype(QI)::value;
        constexpr int i = q >> 1;
        constexpr int younger = q == 0 ? kPieceLoads + kWLoads : q == 1 ? kWLoads + (Q > 2 ? kPieceLoads : 0)
                                                                        : (q + 1 < Q ? kPieceLoads : 0);
        constexpr int n = younger < 63 ? younger : 63;     // the counter field holds up to 63; less only waits longer
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8));
        __builtin_amdgcn_sched_barrier(0);
        unsigned char* const slot = (q & 1) ? slot1 : slot0;
        const int ul = wave + i * WAVES;
        if (ul < kus) {                                    // wave-uniform
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                constexpr int tbase = 2 * (q & 1);
                const int t = tbase + t2;                  // MFMA step inside the unit (compile-time after unrolling)
                f16x8 xa[TM];
#pragma unroll
                for (int im = 0; im < TM; ++im)
                    xa[im] = *(const f16x8*)(slot + im * 2048 + x_rd + (((uint32_t)(4 * t2 + h)) ^ x_swz) * 16u);
#pragma unroll
                for (int j = 0; j < NTW; ++j) {
                    const GroupConst gc = make_group_const(st.sz[i][j][t / TG]);
                    const f16x8 b = dequant8(st.wq[i][j][t], gc, mg);
#pragma unroll
                    for (int im = 0; im < TM; ++im) acc[im][j] = mfma16x16x32(xa[im], b, acc[im][j]);
                }
            }
        }
        // this piece's fragment reads have all been consumed by issued MFMAs: its slot takes the piece after next
        if constexpr (q + 2 < Q) {
            __builtin_amdgcn_sched_barrier(0);
            load_piece(q + 2, slot);
        }
    });

    // ---- cross-wave sum, one row tile at a time: column tiles 0..3 meet in the first X slot array, 4..7 in the second
    // (each holds WAVES x 4 tiles x 4 registers x 64 lanes floats), a thread owns two neighbouring columns of one
    // accumulator register, every sum runs in wave order.
    const int pl = (tid & 31) * 2;
    constexpr int kPasses = (NTW * 4 + WAVES * 2 - 1) / (WAVES * 2);
#pragma unroll
    for (int im = 0; im < TM; ++im) {
        __syncthreads();                           // every wave is done with its X slots / with the previous row tile
#pragma unroll
        for (int j = 0; j < NTW; ++j) {
            float* red = (float*)(j < 4 ? xs0 : xs1);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (16 * im + r < p.M) red[(((j & 3) * 4 + r) * WAVES + wave) * 64 + lane] = acc[im][j][r];
        }
        __syncthreads();
#pragma unroll
        for (int ps = 0; ps < kPasses; ++ps) {
            const int jr = (tid >> 5) + ps * WAVES * 2;
            const int m = 16 * im + 4 * (pl >> 4) + (jr & 3);
            if (jr < NTW * 4 && m < p.M) {
                const float* src = (const float*)((jr >> 2) < 4 ? xs0 : xs1) + (size_t)(jr & 15) * WAVES * 64 + pl;
                float2 tv[WAVES];
#pragma unroll
                for (int w = 0; w < WAVES; ++w) tv[w] = *(const float2*)(src + w * 64);
                __builtin_amdgcn_sched_barrier(0);
                float v0 = 0.f, v1 = 0.f;
#pragma unroll
                for (int w = 0; w < WAVES; ++w) {
                    v0 += tv[w].x;
                    v1 += tv[w].y;
                }
                const int n = (nt0 + (jr >> 2)) * 16 + (pl & 15);
                if (p.split == 1) store_pair(p, m, n, v0, v1);
                else st_partial2(p.partial + ((size_t)sk * p.strips + strip) * p.slot_floats + (im * NTW * 4 + jr) * 64 + pl, v0, v1);
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
            for (int im = 0; im < TM; ++im) {
#pragma unroll
                for (int ps = 0; ps < kPasses; ++ps) {
                    const int jr = (tid >> 5) + ps * WAVES * 2;
                    const int m = 16 * im + 4 * (pl >> 4) + (jr & 3);
                    if (jr < NTW * 4 && m < p.M) {
                        const int n = (nt0 + (jr >> 2)) * 16 + (pl & 15);
                        float v0, v1;
                        sum_partials2(p.partial + (size_t)strip * p.slot_floats + (im * NTW * 4 + jr) * 64 + pl,
                                      (size_t)p.strips * p.slot_floats, p.split, v0, v1);
                        store_pair(p, m, n, v0, v1);
                    }
                }
            }
            if (tid == 0) __hip_atomic_store(&p.counters[strip], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// NTW = the wider of the two strip widths of the launch, as in stream_kernel.
template <int TM, int NTW, int GPU, int NI, int MAXW>
__global__ __launch_bounds__(MAXW * 64) void rows_kernel(GemmParams p)
{
    __shared__ __attribute__((aligned(16))) unsigned char xs0[MAXW * 16 * TM * 128];
    __shared__ __attribute__((aligned(16))) unsigned char xs1[MAXW * 16 * TM * 128];
    __shared__ uint32_t s_last;
    const int strip = blockIdx.x, sk = blockIdx.y;
    const int nt0 = strip * p.strip_base + min(strip, p.strip_rem);
    if constexpr (NTW > 1) {
        if (strip >= p.strip_rem && p.strip_base < NTW) {          // CTA-uniform
            rows_body<TM, NTW - 1, GPU, NI, MAXW>(p, strip, sk, nt0, xs0, xs1, s_last);
            return;
        }
    }
    rows_body<TM, NTW, GPU, NI, MAXW>(p, strip, sk, nt0, xs0, xs1, s_last);
}

// Which (rows, strip width, K-groups per unit, units per wave, CTA size) combinations exist: the registers a wave needs
// for its weights in flight, its accumulators and one step of fragments must fit 128 per lane in CTAs of 16 waves, 256
// in CTAs of 8 (built only where 16 do not fit), and the reduction needs at most eight column tiles.
constexpr bool rows_built(int tm, int ntw, int gpu, int ni, int maxw)
{
    const int regs = ni * ntw * (4 + gpu) + tm * ntw * 4 + 4 * tm + 3 * ntw + 24;
    // four row tiles: the two slot arrays of 16 waves would need 256 KiB of LDS, so CTAs of 8 waves only
    if (tm == 4) return ntw <= 8 && gpu <= 2 && maxw == 8 && regs <= 250;
    return ntw <= 8 && gpu <= 2 && (maxw == 16 ? regs <= 128 : (regs > 128 && regs <= 250));
}

template <int TM, int NTW, int GPU, int NI, int MAXW>
hipError_t launch_rows_one(const GemmParams& p, const Plan& plan, hipStream_t stream)
{
    if constexpr (rows_built(TM, NTW, GPU, NI, MAXW)) {
        dim3 grid(plan.strips, plan.split), block(plan.block);
        if (plan.block != MAXW * 64 || plan.split > 65535) return hipErrorInvalidValue;
        hipLaunchKernelGGL((rows_kernel<TM, NTW, GPU, NI, MAXW>), grid, block, 0, stream, p);
        return hipGetLastError();
    } else {
        return hipErrorInvalidValue;
    }
}

template <int TM, int NTW, int NI>
hipError_t launch_rows_ni(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    if (plan.block > 512) {
        switch (group) {
            case 128: return launch_rows_one<TM, NTW, 1, NI, 16>(p, plan, stream);
            case 64: return launch_rows_one<TM, NTW, 2, NI, 16>(p, plan, stream);
            default: return hipErrorInvalidValue;
        }
    }
    switch (group) {
        case 128: return launch_rows_one<TM, NTW, 1, NI, 8>(p, plan, stream);
        case 64: return launch_rows_one<TM, NTW, 2, NI, 8>(p, plan, stream);
        default: return hipErrorInvalidValue;
    }
}

template <int TM, int NTW>
hipError_t launch_rows_ntw(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    switch (plan.stream_ni) {
        case 1: return launch_rows_ni<TM, NTW, 1>(p, plan, group, stream);
        case 2: return launch_rows_ni<TM, NTW, 2>(p, plan, group, stream);
        case 3: return launch_rows_ni<TM, NTW, 3>(p, plan, group, stream);
        case 4: return launch_rows_ni<TM, NTW, 4>(p, plan, group, stream);
        case 6: return launch_rows_ni<TM, NTW, 6>(p, plan, group, stream);
        case 8: return launch_rows_ni<TM, NTW, 8>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

template <int TM>
hipError_t launch_rows_tm(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    const int ntw = p.strip_base + (p.strip_rem > 0 ? 1 : 0);
    if ((uint64_t)p.M * (uint64_t)p.K * 2u >= (1ull << 31) || p.M > 16 * TM) return hipErrorInvalidValue;
    switch (ntw) {
        case 1: return launch_rows_ntw<TM, 1>(p, plan, group, stream);
        case 2: return launch_rows_ntw<TM, 2>(p, plan, group, stream);
        case 3: return launch_rows_ntw<TM, 3>(p, plan, group, stream);
        case 4: return launch_rows_ntw<TM, 4>(p, plan, group, stream);
        case 5: return launch_rows_ntw<TM, 5>(p, plan, group, stream);
        case 6: return launch_rows_ntw<TM, 6>(p, plan, group, stream);
        case 7: return launch_rows_ntw<TM, 7>(p, plan, group, stream);
        case 8: return launch_rows_ntw<TM, 8>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

// host-side twin of rows_built for the dispatcher: units per wave a launch would take, 0 if no kernel is built for it
inline int rows_units(int tm, int ntw, int group, int kus, int waves)
{
    if (group != 128 && group != 64) return 0;
    int ni = (kus + waves - 1) / waves;
    const int built[] = {1, 2, 3, 4, 6, 8};
    for (int b : built)
        if (b >= ni) return rows_built(tm, ntw, 128 / group, b, waves) ? b : 0;
    return 0;
}

}  // namespace

}  // namespace tmw4
