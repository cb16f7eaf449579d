// Grouped (mixture-of-experts) launch of the CTA-tile kernels, for experts with more rows than the decode kernels
// take in one pass.  Same body as tile_kernel, same build flags as the small tiles; what differs is how a CTA finds
// its tile: the rows per expert are only known on the device, so the grid covers an upper bound of row tiles and
// every CTA locates its (expert, row tile) by a prefix scan over the experts' row-tile counts.
#include "tm_w4_tile_impl.h"

namespace tmw4 {

namespace {

template <int TM, int TN, int NW, int GPU, int KW, int FMT = kFmtInt4, int PD = (TM <= 8 ? 2 : 1)>
__global__ __launch_bounds__(NW * 64) void tile_grouped_kernel(GroupedParams gp)
{
    constexpr int BM = TM * 16;
    // Same XCD-aware numbering as tile_kernel, over gp.mtiles row-tile slots x gp.tiles_n column tiles.
    const int tiles = gp.mtiles * gp.tiles_n;
    const int chunk = (tiles + 7) / 8;
    const int b = blockIdx.x;
    const int logical = (b % 8) * chunk + b / 8;
    if (logical >= tiles) return;
    const int panel_tiles = kPanelN * gp.mtiles;
    const int panel = logical / panel_tiles;
    const int within = logical % panel_tiles;
    const int pw = min(kPanelN, gp.tiles_n - panel * kPanelN);
    const int tile_n = panel * kPanelN + within % pw;
    int want = within / pw;                         // row-tile slot, counted over all experts in order

    // Slot -> (expert, row tile): 64 experts per step, an inclusive scan of their row-tile counts across the wave.
    // Every lane also fetches its candidate's buffer addresses, so the search costs one round trip to memory.
    const int lane = threadIdx.x & 63;
    int r0 = 0, r1 = 0, tile_m = 0;
    uint64_t wptr = 0, szptr = 0;
    bool found = false;
    for (int base = 0; base < gp.experts; base += 64) {
        const int e = base + lane;
        int a = 0, z = 0;
        uint64_t tw = 0, ts = 0;
        if (e < gp.experts) {
            a = gp.offsets[e];
            z = gp.offsets[e + 1];
            tw = gp.table[2 * e];
            ts = gp.table[2 * e + 1];
        }
        a = min(max(a, 0), gp.total_rows);          // rows are clamped to the buffers whatever the offsets hold
        z = max(min(z, gp.total_rows), a);
        const int cnt = (z - a + BM - 1) / BM;
        int incl = cnt;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(incl, d);
            if (lane >= d) incl += t;
        }
        const int total = __builtin_amdgcn_readlane(incl, 63);
        if (want < total) {
            const uint64_t hit = __ballot(cnt > 0 && incl - cnt <= want && want < incl);
            const int src = __builtin_ctzll(hit);   // exactly one lane
            r0 = __builtin_amdgcn_readlane(a, src);
            r1 = __builtin_amdgcn_readlane(z, src);
            tile_m = want - __builtin_amdgcn_readlane(incl - cnt, src);
            wptr = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(tw >> 32), src) << 32) |
                   (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)tw, src);
            szptr = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(ts >> 32), src) << 32) |
                    (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)ts, src);
            found = true;
            break;
        }
        want -= total;
    }
    if (!found) return;                             // the grid's upper bound was not needed

    GemmParams p{};
    p.X = gp.X + (size_t)r0 * gp.K;
    p.ldy = gp.act ? gp.N / 2 : gp.N;
    p.act = gp.act;
    p.epi = gp.act;
    p.Y = gp.Y + (size_t)r0 * p.ldy;
    p.W = (const u32x4*)wptr;
    p.SZ = (const uint32_t*)szptr;
    p.M = r1 - r0;
    p.K = gp.K;
    p.N = gp.N;
    p.KU = gp.KU;
    p.NT = gp.NT;
    p.G = gp.G;
    p.split = 1;
    p.ku_per_split = gp.KU;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = gp.tiles_n;
    tile_body<TM, TN, NW, GPU, KW, PD, 1, FMT>(p, tile_m, tile_n, 0);
}

template <int TM, int TN, int KW, int FMT = kFmtInt4>
hipError_t launch_grouped_shape(GroupedParams gp, int experts, int group, hipStream_t stream)
{
    constexpr int BM = TM * 16, BN = 4 * TN * 16;
    constexpr int SPU = FMT == kFmtInt4 ? 4 : 2;                             // MFMA steps per packed unit
    if ((gp.KU * SPU) % KW) return hipErrorInvalidValue;                     // whole stages
    if ((uint64_t)gp.total_rows * (uint64_t)gp.K >= (1ull << 31)) return hipErrorInvalidValue;   // 32-bit X offsets
    gp.tiles_n = (gp.N + BN - 1) / BN;
    // every expert with rows adds at most one partly filled row tile
    gp.mtiles = gp.total_rows / BM + (gp.total_rows < experts ? gp.total_rows : experts);
    const long tiles = (long)gp.mtiles * gp.tiles_n;
    if (tiles <= 0 || tiles > (1l << 30)) return hipErrorInvalidValue;
    dim3 grid((unsigned)(((tiles + 7) / 8) * 8)), block(256);
    switch (group) {
        case 128: hipLaunchKernelGGL((tile_grouped_kernel<TM, TN, 4, 1, KW, FMT>), grid, block, 0, stream, gp); break;
        case 64: hipLaunchKernelGGL((tile_grouped_kernel<TM, TN, 4, 2, KW, FMT>), grid, block, 0, stream, gp); break;
        case 32: hipLaunchKernelGGL((tile_grouped_kernel<TM, TN, 4, 4, KW, FMT>), grid, block, 0, stream, gp); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_tile_grouped(const GroupedParams& gp, int variant, int experts, int group, hipStream_t stream)
{
    if (experts <= 0) return hipErrorInvalidValue;
    switch (variant) {
        case kTile64x128: return launch_grouped_shape<4, 2, 4>(gp, experts, group, stream);
        case kTile128x256: return launch_grouped_shape<8, 4, 2>(gp, experts, group, stream);
        default: return hipErrorInvalidValue;
    }
}

// The 8-bit formats (integer codes, FP8 E4M3): the same two tile shapes.
hipError_t launch_tile_grouped_8bit(const GroupedParams& gp, int variant, int experts, int group, bool fp8, hipStream_t stream)
{
    if (experts <= 0) return hipErrorInvalidValue;
    switch (variant) {
        case kTile64x128:
            return fp8 ? launch_grouped_shape<4, 2, 4, kFmtFp8>(gp, experts, group, stream)
                       : launch_grouped_shape<4, 2, 4, kFmtInt8>(gp, experts, group, stream);
        case kTile128x256:
            return fp8 ? launch_grouped_shape<8, 4, 2, kFmtFp8>(gp, experts, group, stream)
                       : launch_grouped_shape<8, 4, 2, kFmtInt8>(gp, experts, group, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tmw4
