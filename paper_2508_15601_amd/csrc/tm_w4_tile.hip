// Fused dequantise-and-multiply for M > 64: CTA tiles with the activations staged through LDS.
//
// Online stage of the GEMM pipeline (paper Sec. 3.1 steps (i)-(iv)) with the software-pipelined main loop of
// Sec. 4.3: while the matrix cores work on one 64-deep K slice, the vector ALUs convert the next weight fragments
// (I2F + zero/scale) and the memory units fetch the following X slice and the next unit of packed weights.
//
// Differences from the paper's design: packed weights go from HBM/L2 straight into registers in matrix-core operand
// order (no shared-memory stage, no matrix-load instruction, hence nothing to swizzle); only X passes through LDS,
// in a padded row-major layout (144-byte pitch) that makes the 16-lane 128-bit fragment reads conflict-free.
#include "tm_w4_host.h"

namespace tmw4 {

namespace {

constexpr int kHalfK = 64;                 // K depth of one LDS stage (half a packed unit)
constexpr int kPitch = kHalfK + 8;         // LDS row pitch in halves (144 bytes)

template <int TM, int TN, int WGM, int WGN, int GPU>
__global__ __launch_bounds__(256) void tile_kernel(GemmParams p)
{
    constexpr int BM = WGM * TM * 16, BN = WGN * TN * 16;
    constexpr int CH = BM / 32;            // 16-byte chunks of one X stage per thread (BM rows x 8 chunks / 256)
    static_assert(WGM * WGN == 4, "four waves per CTA");
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][BM * kPitch];
    __shared__ uint32_t s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, h = lane >> 4;
    const int wm = wave % WGM, wn = wave / WGM;

    const int tiles = p.tiles_m * p.tiles_n;
    const int tile = blockIdx.x % tiles;
    const int sk = blockIdx.x / tiles;
    const int tile_m = tile % p.tiles_m, tile_n = tile / p.tiles_m;
    const int m0 = tile_m * BM;
    const int nt0 = (tile_n * BN) / 16 + wn * TN;          // first 16-column tile of this wave
    const int ku0 = sk * p.ku_per_split;
    const int ku1 = min(p.KU, ku0 + p.ku_per_split);

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // global -> register staging of one X stage: thread owns chunks idx = i*256 + tid -> (row idx/8, chunk idx%8)
    u32x4 xreg[CH];
    auto load_x = [&](int ku, int half) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int idx = i * 256 + tid;
            int row = m0 + (idx >> 3);
            row = row < p.M ? row : p.M - 1;
            xreg[i] = *(const u32x4*)(p.X + (size_t)row * p.K + (size_t)ku * kUnitK + half * kHalfK + (idx & 7) * 8);
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            int idx = i * 256 + tid;
            *(u32x4*)(&xs[buf][(idx >> 3) * kPitch + (idx & 7) * 8]) = xreg[i];
        }
    };

    u32x4 wq[TN], wq_next[TN];
    uint32_t sz[TN][GPU], sz_next[TN][GPU];
    auto load_w = [&](u32x4 (&w)[TN], uint32_t (&s)[TN][GPU], int ku) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int nt = nt0 + j;
            if (nt < p.NT) {
                w[j] = p.W[((size_t)nt * p.KU + ku) * 64 + lane];
#pragma unroll
                for (int g = 0; g < GPU; ++g) s[j][g] = p.SZ[((size_t)nt * p.G + ku * GPU + g) * 16 + c];
            } else {
                w[j] = u32x4{0, 0, 0, 0};
#pragma unroll
                for (int g = 0; g < GPU; ++g) s[j][g] = 0;
            }
        }
    };
    auto compute_half = [&](int buf, int half) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const int t = 2 * half + tt;
            f16x8 a[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int row = (wm * TM + i) * 16 + c;
                a[i] = *(const f16x8*)(&xs[buf][row * kPitch + 32 * tt + 8 * h]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                GroupConst gc = make_group_const(sz[j][(t * GPU) / 4]);
                f16x8 b = dequant8(wq[j][t], gc);
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[i][j] = mfma16x16x32(a[i], b, acc[i][j]);
            }
        }
    };

    if (ku0 < ku1) {
        load_x(ku0, 0);
        load_w(wq, sz, ku0);
        store_x(0);
        __syncthreads();
        for (int ku = ku0; ku < ku1; ++ku) {
            const bool more = ku + 1 < ku1;
            load_x(ku, 1);
            if (more) load_w(wq_next, sz_next, ku + 1);
            compute_half(0, 0);
            store_x(1);
            __syncthreads();
            if (more) load_x(ku + 1, 0);
            compute_half(1, 1);
            if (more) {
                store_x(0);
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    wq[j] = wq_next[j];
#pragma unroll
                    for (int g = 0; g < GPU; ++g) sz[j][g] = sz_next[j][g];
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

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            int m = m0 + (wm * TM + i) * 16 + 4 * h + r;
            if (m >= p.M) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int nt = nt0 + j;
                if (nt < p.NT) p.partial[((size_t)sk * p.M + m) * p.N + nt * 16 + c] = acc[i][j][r];
            }
        }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        uint32_t prev = atomicAdd(&p.counters[tile], 1u);
        s_last = (prev == (uint32_t)p.split - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
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
                for (int s = 0; s < p.split; ++s) v += p.partial[((size_t)s * p.M + m) * p.N + nt * 16 + c];
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
        case kTile128: return launch_shape<4, 4, 2, 2>(p, plan, group, stream);
        case kTile256: return launch_shape<8, 8, 2, 2>(p, plan, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
