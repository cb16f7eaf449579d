// Fused dequantise-and-multiply for M > 32: CTA tiles with the activations staged through LDS.
//
// Online stage of the GEMM pipeline (paper Sec. 3.1 steps (i)-(iv)) with the software-pipelined main loop of
// Sec. 4.3: while the matrix cores work on one 64-deep K slice, the vector ALUs convert the weight fragments of
// that slice (I2F + zero/scale) between the MFMAs, and the memory units fetch the next X slice and the next
// half-unit of packed weights.
//
// Differences from the paper's design: packed weights go from HBM/L2 straight into registers in matrix-core operand
// order (no shared-memory stage, no matrix-load instruction, hence nothing to swizzle); only X passes through LDS,
// in a padded row-major layout (144-byte pitch) that makes the 16-lane 128-bit fragment reads conflict-free.
// CTAs are numbered so that the CTAs resident on one XCD (one L2) cover a compact block of output tiles.
#include "tm_w4_host.h"

namespace tmw4 {

namespace {

constexpr int kHalfK = 64;                 // K depth of one LDS stage (half a packed unit)
constexpr int kPitch = kHalfK + 8;         // LDS row pitch in halves (144 bytes)
constexpr int kPanelN = 8;                 // output tiles per panel row (XCD-local rasterisation)

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int TM, int TN, int WGM, int WGN, int GPU>
__global__ __launch_bounds__(256) void tile_kernel(GemmParams p)
{
    constexpr int BM = WGM * TM * 16, BN = WGN * TN * 16;
    constexpr int CH = (BM * 8 + 255) / 256;   // 16-byte chunks of one X stage per thread (BM rows x 8 chunks)
    constexpr int GH = GPU == 4 ? 2 : 1;       // K-groups touched by one 64-deep half-step
    static_assert(WGM * WGN == 4, "four waves per CTA");
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][BM * kPitch];
    __shared__ uint32_t s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, h = lane >> 4;
    const int wm = wave % WGM, wn = wave / WGM;

    // XCD-aware numbering: consecutive block ids go to different XCDs, so the ids congruent mod 8 (one XCD) are
    // mapped to consecutive logical tiles, and logical tiles walk panels of kPanelN tiles along N.
    const int tiles = p.tiles_m * p.tiles_n;
    const int chunk = (tiles + 7) / 8;
    const int sk = blockIdx.x / (chunk * 8);
    const int b = blockIdx.x % (chunk * 8);
    const int logical = (b % 8) * chunk + b / 8;
    if (logical >= tiles) return;
    const int panel_tiles = kPanelN * p.tiles_m;
    const int panel = logical / panel_tiles;
    const int within = logical % panel_tiles;
    const int pw = min(kPanelN, p.tiles_n - panel * kPanelN);      // width of this panel
    const int tile_m = within / pw, tile_n = panel * kPanelN + within % pw;

    const int m0 = tile_m * BM;
    const int nt0 = (tile_n * BN) / 16 + wn * TN;          // first 16-column tile of this wave
    const int hs0 = 2 * sk * p.ku_per_split;
    const int hs1 = 2 * min(p.KU, (sk + 1) * p.ku_per_split);

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // global -> register staging of one X stage: thread owns chunks idx = i*256 + tid -> (row idx/8, chunk idx%8)
    u32x4 xreg[CH];
    auto load_x = [&](int hs) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int idx = i * 256 + tid;
            if (BM * 8 % 256 == 0 || idx < BM * 8) {
                int row = m0 + (idx >> 3);
                row = row < p.M ? row : p.M - 1;
                xreg[i] = *(const u32x4*)(p.X + (size_t)row * p.K + (size_t)hs * kHalfK + (idx & 7) * 8);
            }
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int idx = i * 256 + tid;
            if (BM * 8 % 256 == 0 || idx < BM * 8)
                *(u32x4*)(&xs[buf][(idx >> 3) * kPitch + (idx & 7) * 8]) = xreg[i];
        }
    };

    // packed weights of one half-step: the lane's words t = 2*half, 2*half+1 of each n-tile's unit
    u32x2 wq[TN], wq_next[TN];
    uint32_t sz[TN][GH], sz_next[TN][GH];
    auto load_w = [&](u32x2 (&w)[TN], uint32_t (&s)[TN][GH], int hs) {
        const int ku = hs >> 1, half = hs & 1;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int nt = nt0 + j;
            if (nt < p.NT) {
                const u32x2* src = (const u32x2*)&p.W[((size_t)nt * p.KU + ku) * 64 + lane];
                w[j] = src[half];
#pragma unroll
                for (int g = 0; g < GH; ++g) {
                    int grp = GPU == 1 ? ku : (GPU == 2 ? 2 * ku + half : 4 * ku + 2 * half + g);
                    s[j][g] = p.SZ[((size_t)nt * p.G + grp) * 16 + c];
                }
            } else {
                w[j] = u32x2{0, 0};
#pragma unroll
                for (int g = 0; g < GH; ++g) s[j][g] = 0;
            }
        }
    };
    auto compute = [&](int buf) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            f16x8 a[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int row = (wm * TM + i) * 16 + c;
                a[i] = *(const f16x8*)(&xs[buf][row * kPitch + 32 * tt + 8 * h]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                GroupConst gc = make_group_const(sz[j][GH == 2 ? tt : 0]);
                f16x8 bfrag = dequant8(wq[j][tt], gc);
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[i][j] = mfma16x16x32(a[i], bfrag, acc[i][j]);
            }
        }
    };

    if (hs0 < hs1) {
        load_x(hs0);
        load_w(wq, sz, hs0);
        store_x(0);
        __syncthreads();
        for (int hs = hs0; hs < hs1; ++hs) {
            const bool more = hs + 1 < hs1;
            const int buf = (hs - hs0) & 1;
            if (more) {
                load_x(hs + 1);
                load_w(wq_next, sz_next, hs + 1);
            }
            compute(buf);
            if (more) {
                store_x(buf ^ 1);
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    wq[j] = wq_next[j];
#pragma unroll
                    for (int g = 0; g < GH; ++g) sz[j][g] = sz_next[j][g];
                }
            }
            __syncthreads();
        }
    }

    // Epilogue.  Lane (c, h) holds Y[m0 + (wm*TM + i)*16 + 4h + r][16*(nt0 + j) + c] in acc[i][j][r].
    if (p.split == 1) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int m = m0 + (wm * TM + i) * 16 + 4 * h + r;
                if (m >= p.M) continue;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    int nt = nt0 + j;
                    if (nt < p.NT) p.Y[(size_t)m * p.N + nt * 16 + c] = f32_to_f16_bits(acc[i][j][r]);
                }
            }
        return;
    }

    const int tile = tile_m + tile_n * p.tiles_m;          // counter index
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int m = m0 + (wm * TM + i) * 16 + 4 * h + r;
            if (m >= p.M) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int nt = nt0 + j;
                if (nt < p.NT) st_partial(p.partial + ((size_t)sk * p.M + m) * p.N + nt * 16 + c, acc[i][j][r]);
            }
        }
    wait_stores_done();
    __syncthreads();
    if (tid == 0) {
        uint32_t prev = atomicAdd(&p.counters[tile], 1u);
        s_last = (prev == (uint32_t)p.split - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int m = m0 + (wm * TM + i) * 16 + 4 * h + r;
            if (m >= p.M) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int nt = nt0 + j;
                if (nt >= p.NT) continue;
                float v = 0.f;
                for (int s = 0; s < p.split; ++s) v += ld_partial(p.partial + ((size_t)s * p.M + m) * p.N + nt * 16 + c);
                p.Y[(size_t)m * p.N + nt * 16 + c] = f32_to_f16_bits(v);
            }
        }
    if (tid == 0) __hip_atomic_store(&p.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int TM, int TN, int WGM, int WGN>
hipError_t launch_shape(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    dim3 grid(plan.grid), block(plan.block);
    switch (group) {
        case 128: hipLaunchKernelGGL((tile_kernel<TM, TN, WGM, WGN, 1>), grid, block, 0, stream, p); break;
        case 64: hipLaunchKernelGGL((tile_kernel<TM, TN, WGM, WGN, 2>), grid, block, 0, stream, p); break;
        case 32: hipLaunchKernelGGL((tile_kernel<TM, TN, WGM, WGN, 4>), grid, block, 0, stream, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_tile(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    switch (plan.variant) {
        case kTile32x256: return launch_shape<2, 4, 1, 4>(p, plan, group, stream);
        case kTile64x256: return launch_shape<4, 4, 1, 4>(p, plan, group, stream);
        case kTile128x128: return launch_shape<4, 4, 2, 2>(p, plan, group, stream);
        case kTile256x256: return launch_shape<8, 8, 2, 2>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
