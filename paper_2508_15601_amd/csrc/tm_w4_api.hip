// C ABI of libtm_w4: argument checking, handle and workspace management, kernel selection.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "tm_attn.h"
#include "tm_w4.h"
#include "tm_w4_host.h"

namespace tmw4 {

namespace {

constexpr uint32_t kMagic = 0x74573461u;              // "tW4a"
constexpr size_t kPartialBudget = 32u << 20;          // bytes of fp32 partial sums a plan may use
constexpr size_t kWorkspaceBytes = kCounterBytes + kPartialBudget;
constexpr size_t kXpermBytes = 32u << 20;             // activations regrouped for activation-order handles
constexpr int kMaxDevices = 16;
// split-K partial sums the allocation-free entry point can hold (tm_gemm_w4a16_static)
constexpr size_t kStaticPartialBytes = 8u << 20;
constexpr size_t kStaticBytes = kCounterBytes + kStaticPartialBytes;

thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

int fail_hip(hipError_t e, const char* what)
{
    return fail(e == hipErrorOutOfMemory ? TM_ENOMEM : TM_EHIP, "%s: %s", what, hipGetErrorString(e));
}

struct DeviceState {
    bool checked = false;
    bool supported = false;
    void* workspace = nullptr;
    void* xperm = nullptr;     // kXpermBytes, allocated with the first activation-order handle
    void* static_ws = nullptr; // this device's copy of the static scratch array, resolved at the first static call
    int num_cu = 256;
};
DeviceState g_dev[kMaxDevices];
std::mutex g_mutex;
int g_force_variant = -1;
int g_force_split = 0;
int g_force_waves = 0;
int g_force_stage = 0;
int g_force_mfma = 0;           // 32 = the prefill tiles on the 32x32x16 matrix instruction; 0 or 16 = 16x16x32 like every other kernel

// Current device must be gfx950; result cached per device.
int check_device(int* dev_out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(TM_EUNSUPPORTED, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState& d = g_dev[dev];
    if (!d.checked) {
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, dev);
        if (e != hipSuccess) return fail_hip(e, "hipGetDeviceProperties");
        d.supported = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
        d.num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        d.checked = true;
    }
    if (!d.supported) return fail(TM_EUNSUPPORTED, "device %d is not gfx950", dev);
    *dev_out = dev;
    return TM_OK;
}

int ensure_workspace(int dev)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState& d = g_dev[dev];
    if (d.workspace) return TM_OK;
    void* ws = nullptr;
    hipError_t e = hipMalloc(&ws, kWorkspaceBytes);
    if (e != hipSuccess) return fail_hip(e, "hipMalloc(workspace)");
    e = hipMemset(ws, 0, kCounterBytes);
    // The clear runs on the null stream, which a caller's non-blocking stream does not wait for: finish it here, once,
    // so that the first GEMM on any stream finds the counters at zero.
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e == hipSuccess) e = stream_setup();       // per-kernel LDS limits of the one-shot decode kernels
    if (e == hipSuccess) e = stream_grouped_setup();
    if (e != hipSuccess) {
        (void)hipFree(ws);
        return fail_hip(e, "workspace set-up");
    }
    d.workspace = ws;
    return TM_OK;
}

}  // namespace

}  // namespace tmw4

// Scratch of the allocation-free entry point: the split-K arrival counters followed by the fp32 partial sums, one copy
// per GPU, held for the life of the process.  In host code this name is only a handle for hipGetSymbolAddress; the
// device address it yields (kept per device in DeviceState::static_ws) is what kernels and fills receive.
static __device__ __align__(256) unsigned char scratch[tmw4::kStaticBytes];

namespace tmw4 {
namespace {
__global__ void clear_words_kernel(uint32_t* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}
}  // namespace
}  // namespace tmw4

struct tm_packed_w4 {
    uint32_t magic;
    int K, N, group, device;
    int bits;          // width of the weight codes: 4, or 8 (tm_pack_w8, tm_pack_w8_fp8)
    bool fp8;          // the 8-bit codes are FP8 E4M3 numbers, not integers
    bool gate_up;      // columns interleaved as (gate j, up j) pairs (tm_pack_w4_gate_up)
    int32_t* perm;     // activation-order handles: packed row i is checkpoint row perm[i] (device, K entries); else null
    uint32_t* w;       // K*N/8 words
    uint32_t* sz;      // (K/group)*N words
    size_t w_bytes, sz_bytes;
};

struct tm_kv_cache {
    uint32_t magic;
    int device;
    tmw4::AttnCache kv;
    size_t code_bytes, pair_bytes;
};

struct tm_expert_group {
    uint32_t magic;
    int experts, K, N, group, device;
    bool gate_up;      // every expert is a gate/up handle with interleaved columns
    int bits;          // 4 or 8 bits per code, the same for every expert
    bool fp8;          // 8-bit codes are FP8 E4M3 values
    uint64_t* table;   // device: per expert, address of the packed weights and of the scale/zero words
};

namespace tmw4 {

namespace {

constexpr uint32_t kGroupMagic = 0x746D4547u;

bool valid(const tm_packed_w4* p) { return p && p->magic == kMagic; }
bool valid(const tm_expert_group* g) { return g && g->magic == kGroupMagic; }
int ceil_div(int a, int b);

// Kernel choice for the grouped launch.  The rows per expert live on the device, so the row-tile height comes from
// the average load (total_rows / experts) and the strip width from how many strips the experts that can be active
// need to cover the chip; wide strips reuse each activation fragment for more weights.
void grouped_plan(const tm_expert_group* g, int total_rows, int num_cu, int* variant, int* strips)
{
    const int NT = g->N / kUnitN;
    // row tiles sized for the busiest expert of a balanced routing: mean load plus three standard deviations
    const int mean = ceil_div(total_rows, g->experts);
    int dev3 = 0;
    while ((dev3 + 1) * (dev3 + 1) <= 9 * mean) ++dev3;
    const int avg = total_rows < mean + dev3 ? total_rows : mean + dev3;
    const int active = total_rows < g->experts ? total_rows : g->experts;
    const int want = ceil_div(2 * num_cu, active > 0 ? active : 1);         // strips per expert for two CTAs per CU
    int per = NT / (want > NT ? NT : want);                                  // tiles per strip, at least one
    int v;
    if (g_force_variant >= 0) v = g_force_variant;
    else if (avg > 192) v = kTile128x256;            // prefill-sized loads: CTA tiles, weights read once per row tile
    else if (avg > 64) v = kTile64x128;
    else if (avg > 32) v = kSkinny64x64;
    else if (avg > 16) v = kSkinny32x64;
    else v = per >= 8 ? kSkinny16x128 : per >= 4 ? kSkinny16x64 : per >= 2 ? kSkinny16x32 : kSkinny16x16;
    const int ntw = is_skinny(v) ? skinny_ntw(v) : 1;
    if (per > ntw) per = ntw;
    int st = ceil_div(NT, per);
    *variant = v;
    *strips = st;
}

int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Kernel and split-K selection.
//  - M <= 32: the skinny kernels.  The strip width (16/32/64 columns per wave) is the widest that still yields at
//    least one CTA per CU, because wider strips reuse each activation fragment for more weights; K is split inside
//    the CTA (8 or 16 waves), and across CTAs only when the strips alone cannot fill the chip.
//  - larger M: CTA tiles; the tile grows with M, and K is split across CTAs while the tiles are too few.
// Split factors are bounded so that every wave keeps at least one unit and the partial sums fit the workspace.
// Floats of split-K partial sums one CTA of a decode kernel hands over: its whole accumulator tile, 16 rows per row
// tile x 16 columns per column tile of the kernel's template width (at least the widest strip of the launch).
int decode_slot_floats(int variant, int NT, int strips)
{
    const int widest = ceil_div(NT, strips > 0 ? strips : 1);
    const int ntw = skinny_ntw(variant) > widest ? skinny_ntw(variant) : widest;
    return ntw * 256 * (skinny_rows(variant) / 16);
}

// Which kernel family and shape a launch takes when nothing is forced (a forced variant is checked against the weight
// format and passed through).
// Deep and narrow layers at 33 ... 64 rows (K of 80 packed units or more, N such that 64 x 64 tiles with K split in four
// make about one CTA per CU): the 64 x 64 CTA tile with its split outruns the decode kernels with an X ring, whose CTAs
// each stream a quarter of a long X (K = 11008, N = 4096: 15.7 against 17.7 us at M = 64, 15.2 against 16.4 us at M = 40;
// K = 14336: 18.5 against 19.6 us; at K = 8192 and below the X ring wins or ties).
static bool deep_narrow_tile64(const tm_packed_w4* h, int M, int num_cu)
{
    const long t = ceil_div(h->N, 64);
    return h->bits == 4 && M > 32 && M <= 64 && h->K / kUnitK >= 80 && t * 4 <= num_cu && t * 8 > num_cu &&
           g_force_variant < 0 && g_force_split == 0 && g_force_waves == 0 && g_force_stage == 0;
}

static int choose_variant(const tm_packed_w4* h, int M, int num_cu, int NT)
{
    const bool w8 = h->bits == 8;
    int variant = g_force_variant;
    // 8-bit formats: the decode kernels up to 64 rows, three CTA-tile shapes above
    if (w8 && variant >= 0 && !(variant == kSkinny16x16 || variant == kSkinny16x32 || variant == kSkinny16x48 ||
                                variant == kSkinny16x64 || variant == kSkinny16x96 || variant == kSkinny16x128 ||
                                variant == kSkinny32x64 || variant == kSkinny64x64 || variant == kTile32x128 ||
                                variant == kTile64x128 || variant == kTile128x256))
        variant = -1;
    if (variant < 0 && w8 && M > 16) {
        auto ctas = [&](int v) { return (long)ceil_div(M, tile_bm(v)) * ceil_div(h->N, tile_bn(v)); };
        // up to 64 rows: narrow outputs (N <= 8192 on 256 CUs) stay with the decode kernels and split K, wide ones take
        // the short tiles (measured at N = 22016: 24.4 vs 32.3 us at M = 32, 28.8 vs 47.6 us at M = 64)
        const bool narrow = ceil_div(NT, 4) * 2 <= num_cu;
        if (M <= 32) variant = narrow ? kSkinny32x64 : kTile32x128;
        else if (M <= 64) variant = narrow ? kSkinny64x64 : kTile64x128;
        else if (ctas(kTile128x256) >= num_cu) variant = kTile128x256;
        else if (ctas(kTile64x128) >= num_cu) variant = kTile64x128;
        else variant = kTile32x128;
    } else if (variant < 0) {
        if (M <= 16) {
            // One CTA per CU: the column tiles are dealt evenly over min(NT, #CU) strips (widths differ by at most
            // one tile), because a CU sustains only ~25 GB/s of weight traffic and the slowest CU sets the time.
            // Outputs wider than eight column tiles per CU (the widest strip) go in two or more whole rounds of CTAs.
            const int rounds = ceil_div(ceil_div(NT, 8), num_cu);
            const int per_cu = ceil_div(NT, rounds * num_cu);
            variant = per_cu <= 1 ? kSkinny16x16 : per_cu <= 2 ? kSkinny16x32 : per_cu <= 3 ? kSkinny16x48
                    : per_cu <= 4 ? kSkinny16x64 : per_cu <= 6 ? kSkinny16x96 : kSkinny16x128;
            // Deep-and-narrow layers with many rows: every strip re-reads all M*K activations, which then outweighs
            // the weights; 64-column strips with K split over four CTAs read a quarter of X each (measured
            // 11.2 vs 14.2 us at K=11008, N=4096, M=16; not a gain at K=4096).
            // (at K = 8192 exactly, split in two: 32-column strips, which make one CTA per CU where 64-column ones make one
            // per two - K = 8192, N = 4096, M = 16: 8.3 against 9.8 us)
            if (per_cu <= 1 && M > 8 && h->K >= 8192 && NT >= num_cu) variant = h->K == 8192 ? kSkinny16x32 : kSkinny16x64;
        } else if (M <= 32 && ceil_div(NT, 4) * 2 <= num_cu) {
            // narrow outputs (N <= 8192 on 256 CUs): 64-column strips with K split across CTAs so that every
            // CU gets one CTA; each CTA then re-reads only its K slice of X
            variant = kSkinny32x64;
        } else {
            // CTA tiles.  ctas(v) tiles of variant v run in ceil(ctas / #CU) rounds, and a round lasts about as
            // long as the tile is wide (a CU streams weights at a fixed rate of its own), so of two widths the one
            // with the smaller rounds x width wins: 96 columns for N = 22016 (230 CTAs instead of 172).
            auto ctas = [&](int v) { return (long)ceil_div(M, tile_bm(v)) * ceil_div(h->N, tile_bn(v)); };
            auto cost = [&](int v) { return (long)ceil_div((int)ctas(v), num_cu) * tile_bn(v); };
            if (M <= 32) {
                variant = cost(kTile32x96) < cost(kTile32x128) ? kTile32x96 : kTile32x128;
            } else if (M <= 64) {
                if (deep_narrow_tile64(h, M, num_cu)) variant = kTile64x64;
                else if (ceil_div(NT, 8) * 4 <= num_cu) variant = kTile32x128;      // narrow: more CTAs, K split on top
                else variant = cost(kTile64x96) < cost(kTile64x128) ? kTile64x96 : kTile64x128;
            } else {
                // The shape with the least estimated time: rounds of CTAs times the time of one round.  A round of
                // 64 x 64 tiles is the unit; the others were measured against it on eight layer shapes (K 4096 ... 11008,
                // N 4096 ... 28672, M 96 ... 512): 32 x 128 1.15, 64 x 128 1.3, 128 x 128 2.37, 128 x 256 3.78.  The short tiles
                // run as one CTA of 8 or 16 waves per CU, so their rounds are whole; two CTAs of the 128-row tiles share
                // a CU, and every round after the first adds 0.6 of one; 128 x 256 tiles that leave more than a tenth of the
                // CUs idle are charged 5 % more.  Over the 48 cases the choice averaged 2 % behind the best forced shape
                // (the same plan timed twice differs by 3-8 %): K = 5120, N = 15360, M = 128: 27.9 us on 240 tiles of
                // 64 x 128 against 36.6 us on 480 of 64 x 64; K = N = 8192, M = 512: 79.1 us on 256 tiles of 128 x 128
                // against 81.6 us on 512 of 64 x 128; M = 1024 there: 131 us on 256 tiles of 128 x 256 against 134 us on
                // 512 of 128 x 128.  Ties go to the larger tile.
                const int shapes[5] = {kTile128x256, kTile128x128, kTile64x128, kTile32x128, kTile64x64};
                const int round_time[5] = {378, 237, 130, 115, 100};
                long best = -1;
                for (int i = 0; i < 5; ++i) {
                    const long rounds = ceil_div((int)ctas(shapes[i]), num_cu);
                    long est = tile_bm(shapes[i]) >= 128 ? round_time[i] * (10 + 6 * (rounds - 1)) : round_time[i] * 10 * rounds;
                    // a single round of 128-row tiles runs with two wave sets per CTA: 12 % (128 x 128) and 5 % (128 x 256) faster
                    if (rounds == 1 && tile_bm(shapes[i]) >= 128) est = shapes[i] == kTile128x128 ? est * 88 / 100 : est * 95 / 100;
                    if (shapes[i] == kTile128x256 && ctas(shapes[i]) * 10 < 9L * num_cu) est += est / 20;
                    if (best < 0 || est < best) {
                        best = est;
                        variant = shapes[i];
                    }
                }
                // Many rounds of 128 x 256 tiles: the same work as CTAs of eight waves on 128 x 512 tiles, one per CU, which
                // load every X stage once for 512 columns instead of once per 256 (half the L2 -> LDS traffic for X:
                // 1-3.5 % faster at K = 4096, N = 22016, M = 2048, at K = N = 8192 and at K = 4096, N = 12288 with M = 4096,
                // and at K = 8192, N = 28672, M = 1024; the same speed at M = 4096 there), where N leaves no half-empty
                // tile and the rounds come out the same.
                if (variant == kTile128x256 && ctas(kTile128x256) >= 3L * num_cu && h->N % 512 == 0 &&
                    ceil_div((int)ctas(kTile128x512), num_cu) <= ceil_div((int)ctas(kTile128x256), 2 * num_cu))
                    variant = kTile128x512;
            }
        }
    }
    return variant;
}

// The plan of the one-shot decode kernels with an X ring, if they take the launch (true, `pl` complete).
// 16 < M <= 64, 4-bit codes: the one-shot decode kernels with a ring of X pieces per wave, about one CTA per CU.  Every
// CTA streams the X rows of its K slice through its CU's load path, so wider strips with K split across CTAs (each
// CTA then reads a part of X only) are weighed against narrow strips that need no merge.
// A forced 16-row decode variant fixes the strip width (and the forced split the split) instead; the forced 32- and
// 64-row variants keep meaning the ring-buffered kernels.
static bool plan_x_ring(const tm_packed_w4* h, int M, int num_cu, int KU, int NT, int max_split_ws, Plan& pl)
{
    if (deep_narrow_tile64(h, M, num_cu)) return false;
    if (h->bits == 4 && M > 16 && M <= 64 && g_force_stage != 1 && (uint64_t)M * h->K * 2u < (1ull << 31) &&
        (g_force_variant < 0 || (is_skinny(g_force_variant) && skinny_rows(g_force_variant) == 16))) {
        auto emit = [&](int strips, int split, int kps, int w, int ni) {
            pl.variant = M <= 32 ? kSkinny32x64 : kSkinny64x64;     // in name only: the strip width is NT / strips
            pl.split = split;
            pl.ku_per_split = kps;
            pl.strips = strips;
            pl.stage_steps = 2;
            pl.kgroups = 1;
            pl.stream_ni = ni;
            pl.tiles_m = 1;
            pl.tiles_n = strips;
            pl.block = (unsigned)w * 64;
            pl.grid = (unsigned)(strips * split);
            pl.ws_bytes = kCounterBytes + (split > 1 ? (size_t)split * strips * decode_slot_floats(pl.variant, NT, strips) * sizeof(float) : 0);
        };
        if (g_force_variant >= 0) {
            const int ntw = skinny_ntw(g_force_variant);
            const int strips = ceil_div(NT, ntw);
            int split = g_force_split > 0 ? g_force_split : 1;
            if (split > KU) split = KU;
            if (split > max_split_ws) split = max_split_ws;
            const int kps = ceil_div(KU, split);
            split = ceil_div(KU, kps);
            const int tries[2] = {g_force_waves >= 8 ? g_force_waves : (M > 32 ? 8 : 16), g_force_waves >= 8 ? g_force_waves : 8};
            for (int w : tries) {
                const int ni = strips <= kMaxCounters ? rows_units_per_wave(M, ceil_div(NT, strips), h->group, kps, w) : 0;
                if (ni > 0) {
                    emit(strips, split, kps, w, ni);
                    return true;
                }
            }
        } else if (NT <= 4 * num_cu) {
            // Strips of one to four column tiles, K split over up to eight CTAs: of the combinations that are built and
            // give at most one CTA per CU, the one with the least estimated time.  The estimate is a fit to 146 timed
            // combinations on fourteen layer shapes (K 1536 ... 28672, N 1024 ... 10240; rms residual 0.6 us at 32 rows,
            // 0.9 us at 64; it ranks the fastest measured combination first on all of them): a constant, the weight
            // units a CTA converts (strip width x units per K slice), the pieces of X it streams (units per K slice),
            // and the merge of the partial sums when K is split, growing with the split.  CTAs of 8 waves at up to 32
            // rows run 1.5 us behind CTAs of 16 with the same work.  Examples at M = 32: K = N = 8192, 13.7 us on
            // 32-column strips unsplit against 16.4 us on 64-column strips split in two; K = 11008, N = 4096, 12.7 us on
            // 64-column strips split in four against 14.5 us on 16-column strips unsplit; K = 13824, N = 5120, 17.3 us
            // on 64-column strips split in three against 28.7 us on the ring-buffered kernel; K = 4096, N = 1024, 6.3 us
            // unsplit on 64 CTAs against 7.1 us split in four.  Wider outputs stay with the CTA tiles (K = 4096,
            // N = 22016: 17.4 against 16.3 us at M = 32, 27.9 against 20.5 us at M = 64).  Up to 32 rows, two rounds of
            // 8-wave CTAs are taken where one round is not built (K = 28672, N = 8192: 43.6 us against 53.5 us).
            const long c0 = M <= 32 ? 3224 : 4222, cw = M <= 32 ? 52 : 87, cx = M <= 32 ? 65 : 47;
            const long cs = M <= 32 ? 2354 : 3375, cm = M <= 32 ? 258 : 243;
            long best = -1;
            int b_strips = 0, b_split = 0, b_kps = 0, b_w = 0, b_ni = 0;
            for (int ntw = 1; ntw <= 4; ++ntw) {
                const int strips = ceil_div(NT, ntw);
                if (strips > kMaxCounters) continue;
                for (int want = 1; want <= 8; ++want) {
                    if (g_force_split > 0 && want != g_force_split) continue;
                    if (want > KU || want > max_split_ws) break;
                    const int kps = ceil_div(KU, want);
                    const int split = ceil_div(KU, kps);
                    if (split != want) continue;
                    const long ctas = (long)strips * split;
                    const int rounds = (int)ceil_div((int)ctas, num_cu);
                    if (rounds > (M <= 32 ? 2 : 1)) continue;
                    for (int w = (M <= 32 && rounds == 1) ? 16 : 8; w >= 8; w -= 8) {
                        if (g_force_waves >= 8 && w != g_force_waves) continue;
                        const int ni = rows_units_per_wave(M, ceil_div(NT, strips), h->group, kps, w);
                        if (ni <= 0) continue;
                        long est = c0 + cw * ntw * kps + cx * kps + (split > 1 ? cs + cm * (split - 1) : 0) + (M <= 32 && w == 8 ? 1500 : 0);
                        est *= rounds;
                        if (best < 0 || est < best) {
                            best = est;
                            b_strips = strips; b_split = split; b_kps = kps; b_w = w; b_ni = ni;
                        }
                        break;
                    }
                }
            }
            if (best >= 0) {
                emit(b_strips, b_split, b_kps, b_w, b_ni);
                return true;
            }
        }
    }
    return false;
}

// Above 64 rows, 4-bit codes, nothing forced: tile shape and K split are weighed together.  The shape
// chosen above (on the unsplit launch) is compared with itself split and with the four shapes up to 128 x 128
// split two to eight ways into at most one CTA per CU; another shape is taken if the estimate puts it 5 % or
// more ahead.  The estimate is a least-squares fit to 1041 timed plans (16 layer shapes, K 2048 ... 28672,
// N 1024 ... 28672, M 96 ... 512, rms error 9 %): a fixed part, the K loop of a CTA (per shape; faster while the
// chip is not full; per round of CTAs), and for a split the hand-over of the partial tiles.  Its picks average
// 1 % behind the fastest measured plan of a case (worst 13 %), where shape first and split second averaged
// 3.6 % (worst 20 %): K = 13824, N = 5120, M = 128 runs 27.6 us on 64 x 128 tiles split in three against
// 38.9 us on 64 x 64 tiles unsplit; K = 11008, N = 4096, M = 256 31.3 against 38.4 us; K = 28672, N = 8192,
// M = 256 124 us on 128 x 128 tiles split in four against 139 us.
static void weigh_tile_shape_and_split(const tm_packed_w4* h, int M, int num_cu, int KU, int& variant, int& split, Plan& pl)
{
    const bool w8 = h->bits == 8;
    const int tiles = pl.tiles_m * pl.tiles_n;
    if (!w8 && M > 64 && g_force_variant < 0 && g_force_split == 0) {
        auto joint = [&](int v, int sp) -> double {
            const double ck = v == kTile32x128 ? 371 : v == kTile64x64 ? 337 : v == kTile64x128 ? 532 : v == kTile128x128 ? 397 : 848;
            const long t = (long)ceil_div(M, tile_bm(v)) * ceil_div(h->N, tile_bn(v));
            const long ctas = t * sp;
            const int rounds = (int)((ctas + num_cu - 1) / num_cu);
            const double occ = ctas < num_cu ? (double)ctas / num_cu : 1.0;
            double r = rounds;
            if (tile_bm(v) >= 128) r = rounds == 1 ? (v == kTile128x128 ? 2.498 : 2.239) : 1.0 + 3.005 * (rounds - 1);
            double est = 5576.0 + ck * ceil_div(KU, sp) * (0.763 + 0.237 * occ) * r;
            if (sp > 1) est += -215.0 + 714.0 * sp + 0.000462 * sp * t * tile_bm(v) * tile_bn(v) * 4;
            return est;
        };
        auto whole = [&](int sp) { const int kps = ceil_div(KU, sp); return sp == 1 || (kps >= 4 && ceil_div(KU, kps) == sp); };
        const bool modelled = variant == kTile32x128 || variant == kTile64x64 || variant == kTile64x128 ||
                              variant == kTile128x128 || variant == kTile128x256;
        if (modelled) {
            const int splits[6] = {1, 2, 3, 4, 6, 8};
            double base = -1;
            int base_split = 1;
            for (int sp : splits) {
                if (!whole(sp) || (sp > 1 && (long)tiles * sp > num_cu)) continue;
                const double e = joint(variant, sp);
                if (base < 0 || e < base) {
                    base = e;
                    base_split = sp;
                }
            }
            int best_v = variant, best_s = base_split;
            double best = base;
            const int others[4] = {kTile64x128, kTile128x128, kTile64x64, kTile32x128};
            for (int v : others) {
                if (v == variant) continue;
                const long t = (long)ceil_div(M, tile_bm(v)) * ceil_div(h->N, tile_bn(v));
                for (int sp : splits) {
                    if (sp == 1 || !whole(sp) || t * sp > num_cu) continue;
                    const double e = joint(v, sp);
                    if (e < 0.95 * base && e < best) {
                        best = e;
                        best_v = v;
                        best_s = sp;
                    }
                }
            }
            variant = pl.variant = best_v;
            split = best_s;
            pl.tiles_m = ceil_div(M, tile_bm(variant));
            pl.tiles_n = ceil_div(h->N, tile_bn(variant));
            pl.block = (unsigned)tile_threads(variant);
        }
    }
}

Plan make_plan(const tm_packed_w4* h, int M, int num_cu)
{
    // packed units along K: 128 rows of 4-bit codes or 64 rows of 8-bit codes (1 KiB per 16 columns either way)
    const int KU = h->bits == 8 ? h->K / 64 : h->K / kUnitK, NT = h->N / kUnitN;
    Plan pl{};
    const bool w8 = h->bits == 8;
    int variant = choose_variant(h, M, num_cu, NT);
    const size_t out_bytes = (size_t)M * h->N * sizeof(float);
    int max_split_ws = (int)(kPartialBudget / (out_bytes ? out_bytes : 1));
    if (max_split_ws < 1) max_split_ws = 1;
    if (plan_x_ring(h, M, num_cu, KU, NT, max_split_ws, pl)) return pl;
    if (is_skinny(variant) && M > skinny_rows(variant))        // a forced skinny variant must still cover M
        variant = M <= 32 ? kSkinny32x64 : (M <= 64 ? kSkinny64x64 : (w8 ? kTile64x128 : kTile64x256));
    pl.variant = variant;
    int split = 1;
    if (is_skinny(variant)) {
        const int ntw = skinny_ntw(variant);
        // fewest strips the variant can take; when chosen automatically for M <= 16 that is one strip per CU
        int strips = ceil_div(NT, ntw);
        if (g_force_variant < 0 && M <= 16 && NT >= num_cu && strips < num_cu && !(variant == kSkinny16x64 && NT / num_cu <= 1))
            strips = num_cu;
        // wider than one round of the widest strips: whole rounds of evenly dealt strips, not one round and a remainder
        // (K = 3584, N = 37888, 2368 column tiles: 512 strips of 4-5 tiles instead of 296 of 8)
        if (g_force_variant < 0 && M <= 16 && NT > 8 * num_cu) strips = num_cu * ceil_div(ceil_div(NT, 8), num_cu);
        int waves = (strips <= num_cu && KU >= 32) ? 16 : 8;
        // many rows on wide strips: 8 waves with a deeper register ring measured 2-3 % faster than 16 waves
        if (M > 8 && ntw >= 3 && skinny_rows(variant) == 16) waves = 8;
        if (g_force_waves >= 8) waves = g_force_waves;
        if (variant == kSkinny32x64 || skinny_rows(variant) == 64) waves = 8;   // register footprint: 8-wave CTAs only
        pl.tiles_m = 1;
        pl.tiles_n = strips;
        pl.strips = strips;
        pl.block = (unsigned)waves * 64;
        if (strips * 2 <= num_cu) {                // too few strips: split K across CTAs as well, up to one CTA per CU
            int want = num_cu / strips;            // (one more would put some CUs through two CTAs in a row)
            int max_by_k = KU / waves > 0 ? KU / waves : 1;
            split = want < max_by_k ? want : max_by_k;
            // Decode shapes: the smallest split with which the one-shot form fits, none if it fits unsplit.  These
            // layers are a few megabytes, so a launch is mostly latency, and the merge of split partial sums (two more
            // dependent trips through memory, about 2 us) costs more than the shorter K slices save: K = 4096,
            // N = 2048, M = 1 runs 3.6-3.9 us on 128 unsplit CTAs against 5.1-5.9 us on 256 split in two; K = 8192,
            // N = 1024 4.8 against 5.3-5.9 us split in four.  Where X is too large for the unsplit form (K = 12800,
            // N = 1536, M = 16: 15.4 us on the ring-buffered kernel) the split that brings it into LDS wins even with
            // more CTAs than CUs (10.0 us split in four, 384 CTAs, against 11.1 us on the ring-buffered kernel split in two).
            if (g_force_variant < 0 && g_force_split == 0 && g_force_stage != 1 && g_force_waves == 0 && h->bits == 4 &&
                M <= 16 && skinny_rows(variant) == 16) {
                const int widest = ceil_div(NT, strips);
                int mp_log = 0;
                while ((1 << mp_log) < M) ++mp_log;
                for (int sp = 1; sp <= 8 && strips * sp <= 2 * num_cu && sp <= KU && sp <= max_split_ws; ++sp) {
                    const int kps = ceil_div(KU, sp);
                    if (ceil_div(KU, kps) != sp) continue;
                    bool fits = false;
                    for (int w : {16, 8}) {
                        const int ni = stream_units_per_wave(widest, h->group, kps, w);
                        int red_off;
                        if (ni > 0 && stream_lds(ni, mp_log, widest, w, &red_off) <= kStreamLdsBudget) fits = true;
                    }
                    if (fits) {
                        split = sp;
                        break;
                    }
                }
            }
        }
    } else {
        pl.tiles_m = ceil_div(M, tile_bm(variant));
        pl.tiles_n = ceil_div(h->N, tile_bn(variant));
        pl.block = (unsigned)tile_threads(variant);
        int tiles = pl.tiles_m * pl.tiles_n;
        // Split K only when fewer than half the CUs would get a tile, at most up to one round of CTAs, and as far as an
        // estimate of the launch says it pays: a fixed part, the K loop of one CTA (per 1024 rows of K: 2.4 us on the
        // 64 x 64 tile, more on the larger ones), and for a split the hand-over of the partial tiles (three dependent
        // trips through memory, about 2.5 us, plus the traffic of the partial sums).  Measured: K = N = 4096, M = 128
        // 12.9 us split in two against 14.5 us unsplit; K = 8192, N = 2048, M = 128 13.9 us split in four against
        // 23.7 us; K = 5120, N = 2560 14.0 us split in three against 18.0 us; K = 16384, N = 1024 16-17 us split in six
        // against 42 us.
        if (tiles * 2 <= num_cu) {
            const int v = variant;
            // ns per 128 rows of K
            const long ck = v == kTile64x64 ? 300 : v == kTile32x128 || v == kTile32x96 ? 315 : v == kTile64x128 || v == kTile64x96 ? 390
                          : v == kTile128x64 ? 410 : v == kTile128x128 ? 630 : 1080;
            const long tile_bytes = (long)tile_bm(v) * tile_bn(v) * 4;
            const int smax = num_cu / tiles < 8 ? num_cu / tiles : 8;
            long best = -1;
            for (int sp = 1; sp <= smax; ++sp) {
                const int kps = ceil_div(KU, sp);
                if (sp > 1 && (kps < 4 || ceil_div(KU, kps) != sp)) continue;
                long est = 5500 + ck * kps / (w8 ? 2 : 1);                                   // 8-bit units are 64 rows
                if (sp > 1) est += 2500 + 300 * sp + sp * tiles * tile_bytes / 4000;         // 4 MB of partial sums per us
                if (best < 0 || est < best) {
                    best = est;
                    split = sp;
                }
            }
        }
        weigh_tile_shape_and_split(h, M, num_cu, KU, variant, split, pl);
    }
    if (g_force_split > 0) split = g_force_split;
    if (pl.tiles_m * pl.tiles_n > kMaxCounters) split = 1;     // one arrival counter per output tile
    if (split > KU) split = KU;
    // bytes of one K slice's partial sums: M x N floats in output order (decode kernels), whole tiles in the CTA-tile
    // kernels' own order
    size_t slice_bytes = out_bytes;
    if (!is_skinny(variant)) {
        slice_bytes = (size_t)pl.tiles_m * pl.tiles_n * tile_bm(variant) * tile_bn(variant) * sizeof(float);
        max_split_ws = (int)(kPartialBudget / slice_bytes);
        if (max_split_ws < 1) max_split_ws = 1;
    }
    if (split > max_split_ws) split = max_split_ws;
    if (split < 1) split = 1;
    pl.ku_per_split = ceil_div(KU, split);
    pl.stage_steps = 2;
    pl.kgroups = 1;
    if (!is_skinny(variant)) {
        // Stage depth: short tiles finish the MFMAs of a 64-deep stage long before the next stage can arrive, so
        // they take stages one or two packed units deep; tall tiles keep 64-deep stages (smaller LDS, two CTAs/CU).
        const int bm = tile_bm(variant);
        int steps = bm <= 64 ? 8 : (variant == kTile128x128 ? 4 : 2);
        if (g_force_stage > 1) steps = g_force_stage;
        if (bm > 128 || variant == kTile128x512) steps = 2;
        if (bm == 128 && steps == 8) steps = 4;
        if (variant == kTile128x256) steps = 2;      // register budget of the 128 x 256 tile
        // Wave sets per CTA (each takes its own slice of every stage): short tiles take four (two for the
        // 96-column tiles, whose sets are two waves wide) unless there are two or more CTAs per CU anyway.
        int kg = 1;
        if (tile_two_waves(variant)) kg = tile_bn(variant) == 96 ? 2 : 4;
        // (64-row tiles: two sets with 128-deep stages measured ahead of four sets with 64-deep ones, 40.2 against
        // 42.0 us at K = N = 8192, M = 256)
        else if (bm <= 64 && (long)pl.tiles_m * pl.tiles_n * split < 2L * num_cu) kg = bm == 64 ? 2 : 4;
        // (128-row tiles with at most one CTA per CU: two sets, 7-14 % faster than one - K = N = 8192, M = 384: 60 against
        // 70 us on 192 tiles of 128 x 128; slower once CTAs run in two rounds, K = 4096, N = 28672, M = 256: 72 against 64 us)
        else if ((variant == kTile128x128 || variant == kTile128x256) && (long)pl.tiles_m * pl.tiles_n * split <= num_cu) kg = 2;
        if (bm <= 64 && kg > 1 && g_force_stage <= 1) steps = 4;
        if (g_force_waves >= 4) kg = g_force_waves * 64 / tile_threads(variant);
        if (!tile_has_kgroups(variant, kg)) kg = tile_has_kgroups(variant, 1) ? 1 : 4;
        if (w8) {
            // the 8-bit tiles are built in one depth each, with one or two wave sets (four on the 32-row tile; one set
            // fewer at group 32, where the kernels with the most sets would spill registers)
            steps = variant == kTile128x256 ? 2 : 4;
            const int most = variant == kTile32x128 ? 4 : 2;
            if (kg > most) kg = most;
            if (h->group == 32 && variant != kTile64x128 && kg == most) kg /= 2;
            if (kg < 1) kg = 1;
        }
        // both X buffers (bm rows x (32*steps*kg + 16) halves each) must fit the 160 KiB of LDS
        while (kg > 1 && 2L * bm * (32 * steps * kg + 16) * 2 > 160 * 1024) {
            if (steps > 2) steps /= 2; else kg /= 2;
        }
        // depths the multi-set kernels are built with (register budget: 128 per lane in CTAs of 16 waves)
        const int waves_total = kg * tile_threads(variant) / 64;
        if (waves_total == 16 && steps > (bm <= 32 ? 4 : 2)) steps = bm <= 32 ? 4 : 2;
        if (kg > 1 && waves_total > 8 && steps == 8) steps = 4;
        if (tile_bn(variant) == 96 && steps == 8) steps = 4;       // three tiles per wave: no registers for 256-deep stages
        if (kg == 2 && bm == 64 && steps == 8 && h->group == 32) steps = 4;
        // the kernels assume whole stages: a stage is steps*kg/4 packed units when that is one or more (steps*kg/2 units
        // of the 8-bit formats, whose depth is fixed)
        // (four two-wave sets with 128-deep stages give up two sets before they give up depth: K = 11008, N = 4096,
        // M = 256 on 64 x 64 tiles runs 35.0 us with two sets of 128-deep stages against 38.2 us with four of 64-deep ones)
        while (!w8 && steps * kg > 4 && KU % (steps * kg / 4)) {
            if (kg == 4 && steps == 4 && tile_two_waves(variant) && g_force_waves < 4) kg = 2;
            else if (steps > 2) steps /= 2;
            else kg /= 2;
        }
        while (w8 && kg > 1 && KU % (steps * kg / 2)) kg /= 2;
        const int ups = steps * kg / (w8 ? 2 : 4);  // packed units per stage
        if (ups > 1 && pl.ku_per_split % ups) pl.ku_per_split += ups - pl.ku_per_split % ups;
        pl.stage_steps = steps;
        pl.kgroups = kg;
        pl.block = (unsigned)tile_threads(variant) * kg;
        // On request (tm_set_mfma_shape(32)) the unsplit, single-set launches of the two prefill tiles run on the 32x32x16
        // matrix instruction: the same cycle count as the 16x16x32 form at a lower clock under load, 10 % slower in all
        // (K = 8192, N = 28672, M = 4096: 1655-1665 against 1505-1513 us), so never by itself.
        if (!w8 && (variant == kTile128x256 || variant == kTile128x512) && kg == 1 && steps == 2 &&
            ceil_div(KU, pl.ku_per_split) == 1 && g_force_mfma == 32)
            pl.mfma32 = 1;
    }
    split = ceil_div(KU, pl.ku_per_split);         // drop empty splits
    pl.split = split;
    pl.stream_ni = 0;
    if (is_skinny(variant) && skinny_rows(variant) == 16 && h->bits == 4 && g_force_stage != 1 && M <= 16) {
        // The one-shot form of the decode kernels, where it is built for the strip width and the K slice and the
        // slice of X fits into LDS: CTAs of 16 waves if a wave's share of the slice fits its registers, else 8.
        const int widest = ceil_div(NT, pl.strips);
        int mp_log = 0;
        while ((1 << mp_log) < M) ++mp_log;
        const int tries[2] = {g_force_waves >= 8 ? g_force_waves : 16, g_force_waves >= 8 ? g_force_waves : 8};
        for (int w : tries) {
            const int ni = stream_units_per_wave(widest, h->group, pl.ku_per_split, w);
            int red_off;
            if (ni > 0 && stream_lds(ni, mp_log, widest, w, &red_off) <= kStreamLdsBudget) {
                pl.stream_ni = ni;
                pl.block = (unsigned)w * 64;
                break;
            }
        }
    }
    // Decode layers whose slice of X does not fit the one-shot form as planned (K beyond 8192 at M = 8 ... 16, or more
    // packed units per wave than a wave can hold): wider strips with K split over two, four or eight CTAs, about one CTA per CU
    // in all, if the one-shot form fits then.  Each CTA streams a half or a quarter of X, and the one-shot kernels
    // outrun the ring-buffered ones by more than the merge costs (K = 11008, N = 4096, M = 8: 8.8 against 10.4 us;
    // K = 14336, N = 4096: 11.1 us at M = 16 this way against 13.1 us at M = 8 without).
    if (is_skinny(variant) && skinny_rows(variant) == 16 && h->bits == 4 && M <= 16 && pl.stream_ni == 0 && split == 1 &&
        g_force_variant < 0 && g_force_split == 0 && g_force_stage != 1 && NT <= 2 * num_cu) {
        int mp_log = 0;
        while ((1 << mp_log) < M) ++mp_log;
        for (int sp = 2; sp <= 8 && pl.stream_ni == 0; sp *= 2) {
            const int ntw = ceil_div(NT * sp, num_cu);
            const int strips = ceil_div(NT, ntw);
            if (ntw > 8 || sp > KU || sp > max_split_ws) break;
            const int kps = ceil_div(KU, sp);
            const int widest = ceil_div(NT, strips);
            for (int w : {16, 8}) {
                const int ni = stream_units_per_wave(widest, h->group, kps, g_force_waves >= 8 ? g_force_waves : w);
                int red_off;
                if (ni > 0 && stream_lds(ni, mp_log, widest, g_force_waves >= 8 ? g_force_waves : w, &red_off) <= kStreamLdsBudget) {
                    pl.variant = widest <= 1 ? kSkinny16x16 : widest <= 2 ? kSkinny16x32 : widest <= 3 ? kSkinny16x48
                               : widest <= 4 ? kSkinny16x64 : widest <= 6 ? kSkinny16x96 : kSkinny16x128;
                    variant = pl.variant;
                    pl.stream_ni = ni;
                    pl.block = (unsigned)(g_force_waves >= 8 ? g_force_waves : w) * 64;
                    pl.strips = strips;
                    pl.tiles_n = strips;
                    pl.ku_per_split = kps;
                    split = ceil_div(KU, kps);
                    pl.split = split;
                    break;
                }
            }
        }
        // Still no one-shot form (K beyond about 24000 on outputs wider than one strip per CU): the ring-buffered
        // kernel on 64-column strips with K split so that every CU gets one CTA, because each CTA streams the rows
        // of X of its own K slice only (K = 28672, N = 8192: 26.4 against 32.9 us at M = 8, 31.1 against 37.1 us at
        // M = 16 on 32-column strips unsplit).
        const int strips4 = ceil_div(NT, 4);
        int sp = num_cu / strips4;
        if (sp > max_split_ws) sp = max_split_ws;
        if (sp > 8) sp = 8;
        if (pl.stream_ni == 0 && M > 4 && (size_t)M * h->K * 2 > 256 * 1024 && sp >= 2 && KU / sp >= 16) {
            pl.variant = variant = kSkinny16x64;
            pl.strips = pl.tiles_n = strips4;
            pl.ku_per_split = ceil_div(KU, sp);
            split = ceil_div(KU, pl.ku_per_split);
            pl.split = split;
            pl.block = (M > 8 ? 8u : 16u) * 64u;
        }
    }
    if (is_skinny(variant)) {
        pl.grid = (unsigned)(pl.tiles_n * split);
    } else {
        int chunk = ceil_div(pl.tiles_m * pl.tiles_n, 8);      // tiles are dealt to the 8 XCDs in equal chunks
        pl.grid = (unsigned)(chunk * 8 * split);
    }
    if (is_skinny(variant)) {
        slice_bytes = (size_t)pl.strips * decode_slot_floats(variant, NT, pl.strips) * sizeof(float);
        if (split > 1 && split * slice_bytes > kPartialBudget) {       // never at the benchmark shapes: the unsplit ring-buffered kernel
            split = pl.split = 1;
            pl.ku_per_split = KU;
            pl.stream_ni = 0;
            pl.grid = (unsigned)pl.tiles_n;
        }
    }
    pl.ws_bytes = kCounterBytes + (split > 1 ? (size_t)split * slice_bytes : 0);
    return pl;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// x_regrouped: X already follows the packed row order of an activation-order handle
int run_gemm(const uint16_t* X, const tm_packed_w4* h, uint16_t* Y, int M, void* ws, size_t ws_bytes, bool own_ws,
             hipStream_t stream, bool x_regrouped = false, const tm_epilogue* epi = nullptr)
{
    if (!valid(h)) return fail(TM_EINVAL, "packed handle is null or invalid");
    if (M < 0 || M >= (1 << 24)) return fail(TM_EINVAL, "M = %d out of range", M);
    if (M == 0) return TM_OK;
    if (!X || !Y) return fail(TM_EINVAL, "X or Y is null");
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 15)) return fail(TM_EINVAL, "X and Y must be 16-byte aligned");
    if ((uint64_t)M * (uint64_t)h->K >= (1ull << 31)) return fail(TM_EINVAL, "M*K must be below 2^31");
    const bool act = epi && epi->act != TM_ACT_NONE;
    if (epi) {
        if (epi->act != TM_ACT_NONE && epi->act != TM_ACT_SILU_MUL) return fail(TM_EINVAL, "unknown activation %d", epi->act);
        if (act && !h->gate_up) return fail(TM_EINVAL, "silu(gate)*up needs a handle made by tm_pack_w4_gate_up");
        if (((uintptr_t)epi->bias & 15) || ((uintptr_t)epi->residual & 15))
            return fail(TM_EINVAL, "bias and residual must be 16-byte aligned");
    }
    if (h->gate_up && !act) return fail(TM_EINVAL, "a gate/up handle holds interleaved columns: call tm_gemm_w4a16_ex with TM_ACT_SILU_MUL");
    const int ldy = act ? h->N / 2 : h->N;
    int dev;
    int rc = check_device(&dev);
    if (rc != TM_OK) return rc;
    if (dev != h->device) return fail(TM_EINVAL, "handle belongs to device %d, current device is %d", h->device, dev);
    if (h->perm && !x_regrouped) {
        // activation-order handle: gather the columns of X into the packed row order, then multiply.  With the
        // library's buffers the rows go through in passes that fit the regroup buffer; a caller workspace carries
        // its own regroup area behind the split-K area of the full-size plan.
        if (own_ws) {
            uint16_t* xb = (uint16_t*)g_dev[dev].xperm;
            if (!xb) return fail(TM_EINVAL, "library regroup buffer missing");
            const int rows_max = (int)(kXpermBytes / ((size_t)h->K * 2)) > 0 ? (int)(kXpermBytes / ((size_t)h->K * 2)) : 0;
            if (rows_max < 1) return fail(TM_EINVAL, "K = %d too large for the regroup buffer", h->K);
            for (int m0 = 0; m0 < M; m0 += rows_max) {
                const int rows = M - m0 < rows_max ? M - m0 : rows_max;
                hipError_t e = launch_permute_x(X + (size_t)m0 * h->K, h->perm, xb, rows, h->K, stream);
                if (e != hipSuccess) return fail_hip(e, "regroup launch");
                tm_epilogue part{};
                if (epi) {
                    part = *epi;
                    if (part.residual) part.residual += (size_t)m0 * ldy;
                }
                rc = run_gemm(xb, h, Y + (size_t)m0 * ldy, rows, ws, ws_bytes, own_ws, stream, true, epi ? &part : nullptr);
                if (rc != TM_OK) return rc;
            }
            return TM_OK;
        }
        if (!ws) return fail(TM_EINVAL, "workspace is null");
        if ((uintptr_t)ws & 255) return fail(TM_EINVAL, "workspace must be 256-byte aligned");
        const size_t plan_bytes = align256(make_plan(h, M, g_dev[dev].num_cu).ws_bytes);
        const size_t need = plan_bytes + (size_t)M * h->K * 2;
        if (ws_bytes < need) return fail(TM_EINVAL, "workspace too small: %zu < %zu", ws_bytes, need);
        uint16_t* xb = (uint16_t*)((char*)ws + plan_bytes);
        hipError_t e = launch_permute_x(X, h->perm, xb, M, h->K, stream);
        if (e != hipSuccess) return fail_hip(e, "regroup launch");
        return run_gemm(xb, h, Y, M, ws, plan_bytes, own_ws, stream, true, epi);
    }
    Plan pl = make_plan(h, M, g_dev[dev].num_cu);
    if (own_ws) {
        ws = g_dev[dev].workspace;
        ws_bytes = kWorkspaceBytes;
        if (!ws) return fail(TM_EINVAL, "library workspace missing");
    } else {
        if (!ws) return fail(TM_EINVAL, "workspace is null");
        if ((uintptr_t)ws & 255) return fail(TM_EINVAL, "workspace must be 256-byte aligned");
    }
    if (ws_bytes < pl.ws_bytes) return fail(TM_EINVAL, "workspace too small: %zu < %zu", ws_bytes, pl.ws_bytes);
    if (pl.split > 1 && pl.tiles_m * pl.tiles_n > kMaxCounters) return fail(TM_EINVAL, "too many output tiles for split-K");

    GemmParams p{};
    p.X = X;
    p.W = (const u32x4*)h->w;
    p.SZ = h->sz;
    p.Y = Y;
    p.counters = (uint32_t*)ws;
    p.partial = (float*)((char*)ws + kCounterBytes);
    p.M = M;
    p.K = h->K;
    p.N = h->N;
    p.KU = h->bits == 8 ? h->K / 64 : h->K / kUnitK;
    p.NT = h->N / kUnitN;
    p.G = h->K / h->group;
    p.split = pl.split;
    p.ku_per_split = pl.ku_per_split;
    p.tiles_m = pl.tiles_m;
    p.tiles_n = pl.tiles_n;
    p.strips = pl.strips;
    p.slot_floats = is_skinny(pl.variant) ? decode_slot_floats(pl.variant, p.NT, pl.strips) : 0;
    if (pl.strips > 0) {
        p.strip_base = p.NT / pl.strips;
        p.strip_rem = p.NT % pl.strips;
    }
    p.ldy = ldy;
    while ((1 << p.mp_log) < M) ++p.mp_log;
    if (epi) {
        p.bias = epi->bias;
        p.residual = epi->residual;
        p.act = act ? 1 : 0;
        p.epi = (p.bias != nullptr) | (p.residual != nullptr) | p.act;
    }
    hipError_t e = h->bits == 8 ? (!is_skinny(pl.variant) ? launch_tile_8bit(p, pl, h->group, h->fp8, stream)
                                   : h->fp8 ? launch_skinny_f8(p, pl, h->group, stream)
                                            : launch_skinny_w8(p, pl, h->group, stream))
                   : pl.stream_ni > 0      ? (M > 16 ? launch_rows(p, pl, h->group, stream) : launch_stream(p, pl, h->group, stream))
                   : is_skinny(pl.variant) ? launch_skinny(p, pl, h->group, stream)
                                           : launch_tile(p, pl, h->group, stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return TM_OK;
}

}  // namespace

}  // namespace tmw4

using namespace tmw4;

extern "C" {

static tm_packed_w4* pack_impl(const void* qweight, const uint16_t* scales, const void* zeros, int K, int N, int group,
                               int layout, int bits, bool fp8, tm_stream stream)
{
    if (layout != TM_LAYOUT_N8 && layout != TM_LAYOUT_N8_INTERLEAVED && layout != TM_LAYOUT_K8) {
        fail(TM_EINVAL, "unknown layout %d", layout);
        return nullptr;
    }
    if (!qweight || !scales) {
        fail(TM_EINVAL, "qweight or scales is null");
        return nullptr;
    }
    if (K <= 0 || N <= 0 || K % kUnitK || N % kUnitN) {
        fail(TM_EINVAL, "need K %% 128 == 0 and N %% 16 == 0 (K = %d, N = %d)", K, N);
        return nullptr;
    }
    if (group != 32 && group != 64 && !(group >= 128 && group % 128 == 0 && K % group == 0)) {
        fail(TM_EINVAL, "group must be 32, 64 or a multiple of 128 that divides K (got %d)", group);
        return nullptr;
    }
    if ((double)K * (double)N >= 1099511627776.0) {
        fail(TM_EINVAL, "K*N too large");
        return nullptr;
    }
    if (((uintptr_t)qweight & 3) || ((uintptr_t)scales & 1) || ((uintptr_t)zeros & (layout == TM_LAYOUT_N8 ? 1 : 3))) {
        fail(TM_EINVAL, "misaligned input");
        return nullptr;
    }
    const int caller_group = group;
    if (group > 128) group = 128;                  // coarser groups are stored replicated at the kernels' 128 rows
    int dev;
    if (check_device(&dev) != TM_OK) return nullptr;
    if (ensure_workspace(dev) != TM_OK) return nullptr;
    tm_packed_w4* h = new (std::nothrow) tm_packed_w4();
    if (!h) {
        fail(TM_ENOMEM, "host allocation failed");
        return nullptr;
    }
    h->magic = kMagic;
    h->K = K;
    h->N = N;
    h->group = group;
    h->device = dev;
    h->bits = bits;
    h->fp8 = fp8;
    h->perm = nullptr;
    h->w_bytes = (size_t)K * N * bits / 8;
    h->sz_bytes = (size_t)(K / group) * N * 4;
    hipError_t e = hipMalloc((void**)&h->w, h->w_bytes);
    if (e == hipSuccess) {
        e = hipMalloc((void**)&h->sz, h->sz_bytes);
        if (e != hipSuccess) (void)hipFree(h->w);
    }
    if (e != hipSuccess) {
        fail_hip(e, "hipMalloc(packed)");
        delete h;
        return nullptr;
    }
    e = bits == 4 ? launch_repack((const uint32_t*)qweight, scales, zeros, h->w, h->sz, K, N, caller_group, layout,
                                  (hipStream_t)stream)
                  : launch_repack8((const uint32_t*)qweight, scales, (const uint16_t*)zeros, h->w, h->sz, K, N,
                                   caller_group, fp8, (hipStream_t)stream);
    if (e != hipSuccess) {
        fail_hip(e, "repack launch");
        (void)hipFree(h->w);
        (void)hipFree(h->sz);
        delete h;
        return nullptr;
    }
    return h;
}

tm_packed_w4* tm_pack_w4_layout(const void* qweight, const uint16_t* scales, const void* zeros, int K, int N,
                                int group, int layout, tm_stream stream)
{
    return pack_impl(qweight, scales, zeros, K, N, group, layout, 4, false, stream);
}

tm_packed_w4* tm_pack_w4_actorder(const void* qweight, const uint16_t* scales, const void* zeros, const int32_t* g_idx,
                                  int K, int N, int group, int layout, tm_stream stream)
{
    if (!g_idx || ((uintptr_t)g_idx & 3)) {
        fail(TM_EINVAL, "g_idx is null or misaligned");
        return nullptr;
    }
    if (!qweight || K <= 0 || N <= 0 || K % kUnitK || N % kUnitN || group <= 0 || K % group ||
        (layout != TM_LAYOUT_N8 && layout != TM_LAYOUT_N8_INTERLEAVED && layout != TM_LAYOUT_K8)) {
        fail(TM_EINVAL, "bad shape, group or layout (K = %d, N = %d, group = %d, layout = %d)", K, N, group, layout);
        return nullptr;
    }
    int dev;
    if (check_device(&dev) != TM_OK) return nullptr;
    hipStream_t st = (hipStream_t)stream;
    // the group indices come to the host once: the row order is fixed here, offline
    std::vector<int32_t> gi((size_t)K), perm((size_t)K);
    hipError_t e = hipStreamSynchronize(st);
    if (e == hipSuccess) e = hipMemcpy(gi.data(), g_idx, (size_t)K * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) {
        fail_hip(e, "reading g_idx");
        return nullptr;
    }
    const int G = K / group;
    std::vector<int> fill((size_t)G, 0);
    for (int k = 0; k < K; ++k) {
        if (gi[k] < 0 || gi[k] >= G || fill[gi[k]] >= group) {
            fail(TM_EINVAL, "g_idx must name each of the %d groups exactly %d times (row %d)", G, group, k);
            return nullptr;
        }
        perm[(size_t)gi[k] * group + fill[gi[k]]++] = k;       // stable: rows of a group keep their order
    }
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        if (!g_dev[dev].xperm) {
            e = hipMalloc(&g_dev[dev].xperm, kXpermBytes);
            if (e != hipSuccess) {
                g_dev[dev].xperm = nullptr;
                fail_hip(e, "hipMalloc(regroup buffer)");
                return nullptr;
            }
        }
    }
    int32_t* dperm = nullptr;
    uint32_t* tmp = nullptr;
    e = hipMalloc((void**)&dperm, (size_t)K * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&tmp, (size_t)K * N / 2);
    if (e == hipSuccess) e = hipMemcpy(dperm, perm.data(), (size_t)K * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = launch_permute_rows((const uint32_t*)qweight, dperm, tmp, K, N, layout == TM_LAYOUT_K8, st);
    tm_packed_w4* h = nullptr;
    if (e == hipSuccess) {
        h = pack_impl(tmp, scales, zeros, K, N, group, layout, 4, false, stream);
        if (h) e = hipStreamSynchronize(st);               // tmp is released below
    } else {
        fail_hip(e, "activation-order regrouping");
    }
    if (tmp) (void)hipFree(tmp);
    if (!h || e != hipSuccess) {
        if (h) {
            fail_hip(e, "activation-order pack");
            tm_free_packed(h);
        }
        if (dperm) (void)hipFree(dperm);
        return nullptr;
    }
    h->perm = dperm;
    return h;
}

tm_packed_w4* tm_pack_w8(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros, int K, int N,
                         int group, tm_stream stream)
{
    return pack_impl(qweight, scales, zeros, K, N, group, TM_LAYOUT_N8, 8, false, stream);
}

tm_packed_w4* tm_pack_w8_fp8(const uint32_t* qweight, const uint16_t* scales, int K, int N, int group, tm_stream stream)
{
    return pack_impl(qweight, scales, nullptr, K, N, group, TM_LAYOUT_N8, 8, true, stream);
}

tm_packed_w4* tm_pack_w4_on(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros, int K, int N,
                            int group, tm_stream stream)
{
    return tm_pack_w4_layout(qweight, scales, zeros, K, N, group, TM_LAYOUT_N8, stream);
}

tm_packed_w4* tm_pack_w4(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros, int K, int N,
                         int group)
{
    return tm_pack_w4_on(qweight, scales, zeros, K, N, group, nullptr);
}

int tm_gemm_w4a16(const uint16_t* X, const tm_packed_w4* packed, uint16_t* Y, int M, tm_stream stream)
{
    return run_gemm(X, packed, Y, M, nullptr, 0, true, (hipStream_t)stream);
}

int tm_gemm_w4a16_ex(const uint16_t* X, const tm_packed_w4* packed, uint16_t* Y, int M, const tm_epilogue* epilogue,
                     tm_stream stream)
{
    return run_gemm(X, packed, Y, M, nullptr, 0, true, (hipStream_t)stream, false, epilogue);
}

tm_packed_w4* tm_pack_w4_gate_up(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros, int K, int N,
                                 int group, tm_stream stream)
{
    if (!qweight || !scales) {
        fail(TM_EINVAL, "qweight or scales is null");
        return nullptr;
    }
    if (K <= 0 || N <= 0 || K % kUnitK || N % 32) {
        fail(TM_EINVAL, "need K %% 128 == 0 and N %% 32 == 0 (two halves of whole 16-column tiles; K = %d, N = %d)", K, N);
        return nullptr;
    }
    if (group != 32 && group != 64 && !(group >= 128 && group % 128 == 0 && K % group == 0)) {
        fail(TM_EINVAL, "group must be 32, 64 or a multiple of 128 that divides K (got %d)", group);
        return nullptr;
    }
    int dev;
    if (check_device(&dev) != TM_OK) return nullptr;
    hipStream_t st = (hipStream_t)stream;
    const int G = K / group;
    uint32_t* q2 = nullptr;
    uint16_t *s2 = nullptr, *z2 = nullptr;
    hipError_t e = hipMalloc((void**)&q2, (size_t)K * N / 2);
    if (e == hipSuccess) e = hipMalloc((void**)&s2, (size_t)G * N * 2);
    if (e == hipSuccess && zeros) e = hipMalloc((void**)&z2, (size_t)G * N * 2);
    if (e == hipSuccess) e = launch_interleave_gate_up(qweight, scales, zeros, q2, s2, z2, K, N, G, st);
    tm_packed_w4* h = nullptr;
    if (e == hipSuccess) {
        h = pack_impl(q2, s2, zeros ? z2 : nullptr, K, N, group, TM_LAYOUT_N8, 4, false, stream);
        if (h) e = hipStreamSynchronize(st);               // the temporaries are released below
    } else {
        fail_hip(e, "gate/up interleave");
    }
    if (q2) (void)hipFree(q2);
    if (s2) (void)hipFree(s2);
    if (z2) (void)hipFree(z2);
    if (h && e != hipSuccess) {
        fail_hip(e, "gate/up pack");
        tm_free_packed(h);
        return nullptr;
    }
    if (h) h->gate_up = true;
    return h;
}

tm_expert_group* tm_group_experts(const tm_packed_w4* const* experts, int num_experts)
{
    if (!experts || num_experts <= 0 || num_experts > 65535) {
        fail(TM_EINVAL, "experts is null or num_experts = %d out of range (1..65535)", num_experts);
        return nullptr;
    }
    for (int e = 0; e < num_experts; ++e) {
        if (!valid(experts[e])) {
            fail(TM_EINVAL, "expert %d: handle is null or invalid", e);
            return nullptr;
        }
        if (experts[e]->perm) {
            fail(TM_EUNSUPPORTED, "expert %d: grouped GEMM takes weights in plain row order only", e);
            return nullptr;
        }
        if (experts[e]->bits != experts[0]->bits || experts[e]->fp8 != experts[0]->fp8) {
            fail(TM_EINVAL, "expert %d differs from expert 0 in weight format", e);
            return nullptr;
        }
        if (experts[e]->gate_up != experts[0]->gate_up) {
            fail(TM_EINVAL, "expert %d: gate/up handles and plain handles cannot share a group", e);
            return nullptr;
        }
        if (experts[e]->K != experts[0]->K || experts[e]->N != experts[0]->N ||
            experts[e]->group != experts[0]->group || experts[e]->device != experts[0]->device) {
            fail(TM_EINVAL, "expert %d differs from expert 0 in K, N, group or device", e);
            return nullptr;
        }
    }
    int dev;
    if (check_device(&dev) != TM_OK) return nullptr;
    if (dev != experts[0]->device) {
        fail(TM_EINVAL, "experts live on device %d, current device is %d", experts[0]->device, dev);
        return nullptr;
    }
    std::vector<uint64_t> host(2 * (size_t)num_experts);
    for (int e = 0; e < num_experts; ++e) {
        host[2 * e] = (uint64_t)(uintptr_t)experts[e]->w;
        host[2 * e + 1] = (uint64_t)(uintptr_t)experts[e]->sz;
    }
    tm_expert_group* g = new (std::nothrow) tm_expert_group();
    if (!g) {
        fail(TM_ENOMEM, "host allocation failed");
        return nullptr;
    }
    hipError_t e = hipMalloc((void**)&g->table, host.size() * sizeof(uint64_t));
    if (e == hipSuccess) {
        e = hipMemcpy(g->table, host.data(), host.size() * sizeof(uint64_t), hipMemcpyHostToDevice);
        if (e != hipSuccess) (void)hipFree(g->table);
    }
    if (e != hipSuccess) {
        fail_hip(e, "expert table");
        delete g;
        return nullptr;
    }
    g->magic = kGroupMagic;
    g->experts = num_experts;
    g->K = experts[0]->K;
    g->gate_up = experts[0]->gate_up;
    g->bits = experts[0]->bits;
    g->fp8 = experts[0]->fp8;
    g->N = experts[0]->N;
    g->group = experts[0]->group;
    g->device = dev;
    return g;
}

void tm_free_expert_group(tm_expert_group* group)
{
    if (!valid(group)) return;
    group->magic = 0;
    (void)hipFree(group->table);
    delete group;
}

// Decode batches of 4-bit experts (at most about sixteen rows per expert): the one-shot kernels, launched as the
// single-GEMM plan of one expert at sixteen rows would launch them, once per expert that has rows (8 experts of
// 4096 x 28672, 2 rows: 27 us against 32 us on the ring-buffered grouped kernel).  False: no such plan.
static bool grouped_one_shot(const tm_expert_group* group, int variant, int strips, int num_cu, Plan* one)
{
    if (group->bits != 4 || !is_skinny(variant) || skinny_rows(variant) != 16 || g_force_variant >= 0 || g_force_stage == 1) return false;
    const int KU = group->K / kUnitK, NT = group->N / kUnitN;
    // large experts: the strips the single-GEMM plan of one expert takes at sixteen rows, as long as a CTA still streams
    // 128 KiB of weights or more (8 experts of 4096 x 28672, 8 rows: 63.9 us on 256 strips per expert against 70.5 us
    // on the 224 strips of the grouped plan); small experts keep the grouped plan's wider strips (128 experts of
    // 4096 x 3072, 32 rows: 44 us on 24 strips per expert against 65 us on 192)
    {
        tm_packed_w4 shape{};
        shape.K = group->K;
        shape.N = group->N;
        shape.group = group->group;
        shape.bits = 4;
        const Plan single = make_plan(&shape, 16, num_cu);
        if (single.stream_ni > 0 && single.split == 1 && is_skinny(single.variant) && skinny_rows(single.variant) == 16 &&
            (size_t)group->K * group->N / 2 / single.strips >= 128 * 1024) {
            *one = single;
            return true;
        }
    }
    const int widest = ceil_div(NT, strips);
    if (widest > 8) return false;
    for (int w : {16, 8}) {
        if (g_force_waves >= 8 && w != g_force_waves) continue;
        const int ni = stream_units_per_wave(widest, group->group, KU, w);
        int red_off;
        if (ni > 0 && stream_lds(ni, 4, widest, w, &red_off) <= kStreamLdsBudget) {
            *one = Plan{};
            one->variant = variant;
            one->strips = strips;
            one->split = 1;
            one->stream_ni = ni;
            one->block = (unsigned)w * 64;
            return true;
        }
    }
    return false;
}

static int run_grouped(const uint16_t* X, const tm_expert_group* group, const int32_t* offsets, uint16_t* Y, int total_rows,
                       int act, tm_stream stream)
{
    if (!valid(group)) return fail(TM_EINVAL, "expert group is null or invalid");
    if (act != TM_ACT_NONE && act != TM_ACT_SILU_MUL) return fail(TM_EINVAL, "unknown activation %d", act);
    if ((act == TM_ACT_SILU_MUL) != group->gate_up)
        return fail(TM_EINVAL, "silu(gate)*up takes experts packed by tm_pack_w4_gate_up, and such experts nothing else");
    if (total_rows == 0) return TM_OK;
    if (!X || !Y || !offsets) return fail(TM_EINVAL, "X, Y or offsets is null");
    if (total_rows < 0 || total_rows >= (1 << 24))
        return fail(TM_EINVAL, "total_rows = %d out of range", total_rows);
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 15) || ((uintptr_t)offsets & 3)) return fail(TM_EINVAL, "misaligned X, Y or offsets");
    int dev;
    int rc = check_device(&dev);
    if (rc != TM_OK) return rc;
    if (dev != group->device) return fail(TM_EINVAL, "experts live on device %d, current device is %d", group->device, dev);
    int variant, strips;
    grouped_plan(group, total_rows, g_dev[dev].num_cu, &variant, &strips);
    GroupedParams gp{};
    gp.X = X;
    gp.Y = Y;
    gp.table = group->table;
    gp.offsets = offsets;
    gp.K = group->K;
    gp.N = group->N;
    gp.KU = group->bits == 8 ? group->K / 64 : group->K / kUnitK;
    gp.NT = group->N / kUnitN;
    gp.G = group->K / group->group;
    gp.strips = strips;
    gp.strip_base = gp.NT / strips;
    gp.strip_rem = gp.NT % strips;
    gp.total_rows = total_rows;
    gp.experts = group->experts;
    gp.act = act == TM_ACT_SILU_MUL ? 1 : 0;
    if (!is_skinny(variant) && (uint64_t)total_rows * (uint64_t)group->K >= (1ull << 31))
        return fail(TM_EINVAL, "total_rows*K must be below 2^31 for prefill-sized expert loads");
    hipError_t e;
    Plan one;
    if (grouped_one_shot(group, variant, strips, g_dev[dev].num_cu, &one)) {
        int red_off;
        gp.strips = one.strips;
        gp.strip_base = gp.NT / one.strips;
        gp.strip_rem = gp.NT % one.strips;
        gp.lds_bytes = (int)stream_lds(one.stream_ni, 4, ceil_div(gp.NT, one.strips), (int)one.block / 64, &red_off);
        e = launch_stream_grouped(gp, group->experts, group->group, one.stream_ni, (int)one.block, (hipStream_t)stream);
        if (e != hipSuccess) return fail_hip(e, "grouped kernel launch");
        return TM_OK;
    }
    if (group->bits == 8) {
        e = !is_skinny(variant) ? launch_tile_grouped_8bit(gp, variant, group->experts, group->group, group->fp8, (hipStream_t)stream)
            : group->fp8       ? launch_skinny_grouped_f8(gp, variant, group->experts, group->group, (hipStream_t)stream)
                               : launch_skinny_grouped_w8(gp, variant, group->experts, group->group, (hipStream_t)stream);
    } else {
        e = is_skinny(variant) ? launch_skinny_grouped(gp, variant, group->experts, group->group, (hipStream_t)stream)
                               : launch_tile_grouped(gp, variant, group->experts, group->group, (hipStream_t)stream);
    }
    if (e != hipSuccess) return fail_hip(e, "grouped kernel launch");
    return TM_OK;
}

int tm_gemm_w4a16_grouped(const uint16_t* X, const tm_expert_group* group, const int32_t* offsets, uint16_t* Y,
                          int total_rows, tm_stream stream)
{
    return run_grouped(X, group, offsets, Y, total_rows, TM_ACT_NONE, stream);
}

int tm_gemm_w4a16_grouped_act(const uint16_t* X, const tm_expert_group* group, const int32_t* offsets, uint16_t* Y,
                              int total_rows, int act, tm_stream stream)
{
    return run_grouped(X, group, offsets, Y, total_rows, act, stream);
}

int tm_get_grouped_plan(const tm_expert_group* group, int total_rows, int* variant, int* strips)
{
    if (!valid(group)) return fail(TM_EINVAL, "expert group is null or invalid");
    if (total_rows <= 0) return fail(TM_EINVAL, "total_rows = %d out of range", total_rows);
    int dev = group->device;
    int cu = (dev >= 0 && dev < kMaxDevices && g_dev[dev].checked) ? g_dev[dev].num_cu : 256;
    int v, st;
    grouped_plan(group, total_rows, cu, &v, &st);
    if (variant) *variant = v;
    if (strips) *strips = st;
    return TM_OK;
}

int tm_gemm_w4a16_ws(const uint16_t* X, const tm_packed_w4* packed, uint16_t* Y, int M, void* workspace,
                     size_t workspace_bytes, tm_stream stream)
{
    return run_gemm(X, packed, Y, M, workspace, workspace_bytes, false, (hipStream_t)stream);
}

int tm_gemm_w4a16_static(const uint16_t* X, const tm_packed_w4* packed, uint16_t* Y, int M, tm_stream stream)
{
    if (!valid(packed)) return fail(TM_EINVAL, "packed handle is null or invalid");
    if (M < 0 || M >= (1 << 24)) return fail(TM_EINVAL, "M = %d out of range", M);
    if (M == 0) return TM_OK;
    int dev;
    int rc = check_device(&dev);
    if (rc != TM_OK) return rc;
    if (dev != packed->device) return fail(TM_EINVAL, "handle belongs to device %d, current device is %d", packed->device, dev);
    size_t need = make_plan(packed, M, g_dev[dev].num_cu).ws_bytes;
    if (packed->perm) need = align256(need) + (size_t)M * packed->K * 2;
    if (need > kStaticBytes)
        return fail(TM_EINVAL, "this call needs %zu bytes of scratch and the static buffer holds %zu: use tm_gemm_w4a16 or "
                    "tm_gemm_w4a16_ws", need, (size_t)kStaticBytes);
    void* ws;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        DeviceState& d = g_dev[dev];
        if (!d.static_ws) {
            // first call on this device: its copy of the array has its own address; the counters must start at zero
            // (a fill kernel on the caller's stream, ordered before the GEMM that follows; no memset node, so the call
            // stays capturable)
            void* ptr = nullptr;
            hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) return fail_hip(e, "hipGetSymbolAddress(scratch)");
            hipLaunchKernelGGL(clear_words_kernel, dim3(kMaxCounters / 256), dim3(256), 0, (hipStream_t)stream,
                               (uint32_t*)ptr, kMaxCounters);
            e = hipGetLastError();
            if (e != hipSuccess) return fail_hip(e, "clearing the static scratch");
            d.static_ws = ptr;
        }
        ws = d.static_ws;
    }
    return run_gemm(X, packed, Y, M, ws, kStaticBytes, false, (hipStream_t)stream);
}

int tm_reset_workspace(void* workspace, tm_stream stream)
{
    int dev;
    int rc = check_device(&dev);
    if (rc != TM_OK) return rc;
    if (workspace && ((uintptr_t)workspace & 255)) return fail(TM_EINVAL, "workspace must be 256-byte aligned");
    void* targets[2] = {workspace, nullptr};
    if (!workspace) {
        std::lock_guard<std::mutex> lock(g_mutex);
        targets[0] = g_dev[dev].workspace;
        targets[1] = g_dev[dev].static_ws;
    }
    for (void* t : targets) {
        if (!t) continue;
        hipLaunchKernelGGL(clear_words_kernel, dim3(kMaxCounters / 256), dim3(256), 0, (hipStream_t)stream, (uint32_t*)t,
                           kMaxCounters);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail_hip(e, "clearing the arrival counters");
    }
    return TM_OK;
}

size_t tm_gemm_workspace_bytes(const tm_packed_w4* packed, int M)
{
    if (!valid(packed) || M <= 0 || M >= (1 << 24)) {
        if (!valid(packed)) fail(TM_EINVAL, "packed handle is null or invalid");
        return 0;
    }
    int dev = packed->device;
    int cu = (dev >= 0 && dev < kMaxDevices && g_dev[dev].checked) ? g_dev[dev].num_cu : 256;
    const size_t plan_bytes = make_plan(packed, M, cu).ws_bytes;
    return packed->perm ? align256(plan_bytes) + (size_t)M * packed->K * 2 : plan_bytes;
}

void tm_free_packed(tm_packed_w4* packed)
{
    if (!valid(packed)) return;
    packed->magic = 0;
    (void)hipFree(packed->w);
    (void)hipFree(packed->sz);
    if (packed->perm) (void)hipFree(packed->perm);
    delete packed;
}

int tm_packed_info(const tm_packed_w4* packed, int* K, int* N, int* group, size_t* bytes)
{
    if (!valid(packed)) return fail(TM_EINVAL, "packed handle is null or invalid");
    if (K) *K = packed->K;
    if (N) *N = packed->N;
    if (group) *group = packed->group;
    if (bytes) *bytes = packed->w_bytes + packed->sz_bytes;
    return TM_OK;
}

int tm_packed_bits(const tm_packed_w4* packed)
{
    if (!valid(packed)) return fail(TM_EINVAL, "packed handle is null or invalid");
    return packed->bits;
}

int tm_unpack_w4(const tm_packed_w4* packed, uint32_t* qweight_out, uint16_t* scales_out, uint16_t* zeros_out,
                 tm_stream stream)
{
    if (!valid(packed)) return fail(TM_EINVAL, "packed handle is null or invalid");
    if (packed->bits != 4) return fail(TM_EUNSUPPORTED, "tm_unpack_w4 handles 4-bit weights only");
    hipError_t e = launch_unpack(packed->w, packed->sz, qweight_out, scales_out, zeros_out, packed->K, packed->N,
                                 packed->group, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "unpack launch");
    return TM_OK;
}

int tm_packed_raw(const tm_packed_w4* packed, const void** weights, size_t* weight_bytes, const void** scale_zero,
                  size_t* scale_zero_bytes)
{
    if (!valid(packed)) return fail(TM_EINVAL, "packed handle is null or invalid");
    if (weights) *weights = packed->w;
    if (weight_bytes) *weight_bytes = packed->w_bytes;
    if (scale_zero) *scale_zero = packed->sz;
    if (scale_zero_bytes) *scale_zero_bytes = packed->sz_bytes;
    return TM_OK;
}

int tm_get_plan(const tm_packed_w4* packed, int M, int* variant, int* split_k, int* grid, int* block)
{
    if (!valid(packed)) return fail(TM_EINVAL, "packed handle is null or invalid");
    if (M <= 0 || M >= (1 << 24)) return fail(TM_EINVAL, "M = %d out of range", M);
    int dev = packed->device;
    int cu = (dev >= 0 && dev < kMaxDevices && g_dev[dev].checked) ? g_dev[dev].num_cu : 256;
    Plan pl = make_plan(packed, M, cu);
    if (variant) *variant = pl.variant;
    if (split_k) *split_k = pl.split;
    if (grid) *grid = (int)pl.grid;
    if (block) *block = (int)pl.block;
    return TM_OK;
}

int tm_get_plan_units_per_wave(const tm_packed_w4* packed, int M)
{
    if (!valid(packed)) return fail(TM_EINVAL, "packed handle is null or invalid");
    if (M <= 0 || M >= (1 << 24)) return fail(TM_EINVAL, "M = %d out of range", M);
    int dev = packed->device;
    int cu = (dev >= 0 && dev < kMaxDevices && g_dev[dev].checked) ? g_dev[dev].num_cu : 256;
    return make_plan(packed, M, cu).stream_ni;
}

int tm_set_variant(int variant, int split_k)
{
    if (variant < -1 || variant >= kNumVariants) return fail(TM_EINVAL, "unknown variant %d", variant);
    if (split_k < 0 || split_k > 256) return fail(TM_EINVAL, "split_k = %d out of range", split_k);
    g_force_variant = variant;
    g_force_split = split_k;
    return TM_OK;
}

int tm_set_mfma_shape(int shape)
{
    if (shape != 0 && shape != 16 && shape != 32) return fail(TM_EINVAL, "shape must be 0 (auto), 16 or 32");
    g_force_mfma = shape;
    return TM_OK;
}

int tm_get_plan_mfma_shape(const tm_packed_w4* packed, int M)
{
    if (!valid(packed)) return fail(TM_EINVAL, "packed handle is null or invalid");
    if (M <= 0 || M >= (1 << 24)) return fail(TM_EINVAL, "M = %d out of range", M);
    int dev = packed->device;
    int cu = (dev >= 0 && dev < kMaxDevices && g_dev[dev].checked) ? g_dev[dev].num_cu : 256;
    return make_plan(packed, M, cu).mfma32 ? 32 : 16;
}

int tm_set_launch(int waves, int stage_steps)
{
    if (waves != 0 && waves != 4 && waves != 8 && waves != 16) return fail(TM_EINVAL, "waves must be 0 (auto), 4, 8 or 16");
    if (stage_steps != 0 && stage_steps != 1 && stage_steps != 2 && stage_steps != 4 && stage_steps != 8)
        return fail(TM_EINVAL, "stage_steps must be 0 (auto), 1, 2, 4 or 8");
    g_force_waves = waves;
    g_force_stage = stage_steps;
    return TM_OK;
}

const char* tm_variant_name(int variant)
{
    switch (variant) {
        case kSkinny16x16: return "skinny16x16";
        case kSkinny16x32: return "skinny16x32";
        case kSkinny16x64: return "skinny16x64";
        case kSkinny32x32: return "skinny32x32";
        case kSkinny32x64: return "skinny32x64";
        case kSkinny16x48: return "skinny16x48";
        case kSkinny16x96: return "skinny16x96";
        case kSkinny16x128: return "skinny16x128";
        case kSkinny64x32: return "skinny64x32";
        case kSkinny64x48: return "skinny64x48";
        case kSkinny64x64: return "skinny64x64";
        case kTile32x256: return "tile32x256";
        case kTile64x256: return "tile64x256";
        case kTile128x256: return "tile128x256";
        case kTile256x256: return "tile256x256";
        case kTile64x128: return "tile64x128";
        case kTile128x128: return "tile128x128";
        case kTile192x256: return "tile192x256";
        case kTile128x512: return "tile128x512";
        case kTile32x128: return "tile32x128";
        case kTile32x96: return "tile32x96";
        case kTile64x96: return "tile64x96";
        case kTile64x64: return "tile64x64";
        case kTile128x64: return "tile128x64";
        default: return "";
    }
}

int tm_bench_copy(void* dst, const void* src, size_t bytes, tm_stream stream)
{
    if (!dst || !src) return fail(TM_EINVAL, "null pointer");
    if ((bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return fail(TM_EINVAL, "need 16-byte multiples");
    hipError_t e = launch_copy(dst, src, bytes, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "copy launch");
    return TM_OK;
}

int tm_bench_read(const void* src, size_t bytes, void* sink, tm_stream stream)
{
    if (!src || !sink) return fail(TM_EINVAL, "null pointer");
    if ((bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)sink & 3)) return fail(TM_EINVAL, "need 16-byte multiples");
    hipError_t e = launch_read(src, bytes, sink, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "read launch");
    return TM_OK;
}

int tm_bench_read_shape(const void* src, size_t bytes, void* sink, int grid, int block, int unroll, int flags, tm_stream stream)
{
    if (!src || !sink) return fail(TM_EINVAL, "null pointer");
    if ((bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)sink & 3)) return fail(TM_EINVAL, "need 16-byte multiples");
    if (grid < 1 || grid > (1 << 20) || block < 64 || block > 1024 || block % 64) return fail(TM_EINVAL, "grid or block out of range");
    if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8 && unroll != 16) return fail(TM_EINVAL, "unroll must be 1, 2, 4, 8 or 16");
    if (flags & ~7) return fail(TM_EINVAL, "unknown flags");
    hipError_t e = launch_read_shape(src, bytes, sink, (unsigned)grid, (unsigned)block, unroll, flags, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "read launch");
    return TM_OK;
}

int tm_bench_mfma(void* out, int grid, int block, int iters, int pattern, tm_stream stream)
{
    if (!out || ((uintptr_t)out & 15)) return fail(TM_EINVAL, "out must be a 16-byte aligned device location");
    if (grid < 1 || grid > (1 << 16) || block < 64 || block > 1024 || block % 64) return fail(TM_EINVAL, "grid or block out of range");
    if (iters < 1 || iters > (1 << 22)) return fail(TM_EINVAL, "iters = %d out of range", iters);
    if (pattern < 0 || pattern > 2) return fail(TM_EINVAL, "pattern must be 0, 1 or 2");
    int dev;
    int rc = check_device(&dev);
    if (rc != TM_OK) return rc;
    hipError_t e = launch_mfma_loop(out, (unsigned)grid, (unsigned)block, iters, pattern, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "mfma loop launch");
    return TM_OK;
}

int tm_bench_clock(void* out, int delay_micros, int micros, tm_stream stream)
{
    if (!out || ((uintptr_t)out & 15)) return fail(TM_EINVAL, "out must be a 16-byte aligned device location");
    if (micros < 1 || micros > 20000) return fail(TM_EINVAL, "micros = %d out of range (1 ... 20000)", micros);
    if (delay_micros < 0 || delay_micros > 100000) return fail(TM_EINVAL, "delay_micros = %d out of range (0 ... 100000)", delay_micros);
    int dev;
    int rc = check_device(&dev);
    if (rc != TM_OK) return rc;
    int khz = 0;
    hipError_t e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
    if (e != hipSuccess || khz <= 0) return fail(TM_EHIP, "no constant-rate counter frequency for device %d", dev);
    const uint32_t delay = (uint32_t)((double)delay_micros * khz / 1000.0);
    const uint32_t ticks = (uint32_t)((double)micros * khz / 1000.0);
    // a round sleeps about a thousand shader clocks (0.3 ... 1 us): eight rounds per microsecond bound the kernel's life
    e = launch_clock_probe(out, delay, ticks, (delay_micros + micros) * 8 + 64, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "clock probe launch");
    return khz;
}

const char* tm_last_error(void) { return g_error; }

const char* tm_version(void) { return "tm_w4 0.1 (gfx950)"; }


// ---------------------------------------------------------------------------------------- attention over a KV cache

static bool valid_kv(const tm_kv_cache* c) { return c && c->magic == 0x746D4B56u; }

tm_kv_cache* tm_kv_create(int batch, int kv_heads, int capacity, int bits)
{
    if (batch <= 0 || kv_heads <= 0 || capacity <= 0 || batch > 65535 || kv_heads > 65535 || (bits != 8 && bits != 4)) {
        fail(TM_EINVAL, "need 1 <= batch, kv_heads <= 65535, capacity > 0, bits 8 or 4 (got %d, %d, %d, %d)", batch, kv_heads,
             capacity, bits);
        return nullptr;
    }
    const long tok = 256 / bits;                          // tokens per 4 KiB block of codes
    const long cap = ((long)capacity + tok - 1) / tok * tok;
    const double codes = (double)batch * kv_heads * (double)cap * 128.0;
    if (cap >= (1L << 24) || codes >= 1.0e12) {
        fail(TM_EINVAL, "cache too large");
        return nullptr;
    }
    int dev;
    if (check_device(&dev) != TM_OK) return nullptr;
    tm_kv_cache* c = new (std::nothrow) tm_kv_cache();
    if (!c) {
        fail(TM_ENOMEM, "host allocation failed");
        return nullptr;
    }
    c->device = dev;
    c->kv.batch = batch;
    c->kv.heads = kv_heads;
    c->kv.cap = (int)cap;
    c->kv.bits = bits;
    // partial results of split contexts: at most 1024 (sequence, head, split) slots of 8.3 KiB, at most 64 splits
    int ms = 1024 / (batch * kv_heads);
    c->kv.max_splits = ms < 1 ? 1 : (ms > 64 ? 64 : ms);
    c->code_bytes = (size_t)batch * kv_heads * cap * 128 * bits / 8;
    c->pair_bytes = (size_t)batch * kv_heads * cap * 8;
    const size_t part_bytes = (size_t)batch * kv_heads * c->kv.max_splits * (32 + 128 * 16) * sizeof(float);
    hipError_t e = hipMalloc((void**)&c->kv.k, c->code_bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&c->kv.v, c->code_bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&c->kv.sz, c->pair_bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&c->kv.partial, part_bytes + (size_t)batch * kv_heads * sizeof(uint32_t));
    if (e == hipSuccess) {
        c->kv.counters = (uint32_t*)((char*)c->kv.partial + part_bytes);
        e = hipMemset(c->kv.counters, 0, (size_t)batch * kv_heads * sizeof(uint32_t));
    }
    if (e != hipSuccess) {
        fail_hip(e, "hipMalloc(kv cache)");
        if (c->kv.k) (void)hipFree(c->kv.k);
        if (c->kv.v) (void)hipFree(c->kv.v);
        if (c->kv.sz) (void)hipFree(c->kv.sz);
        if (c->kv.partial) (void)hipFree(c->kv.partial);
        delete c;
        return nullptr;
    }
    c->magic = 0x746D4B56u;
    return c;
}

void tm_kv_free(tm_kv_cache* cache)
{
    if (!valid_kv(cache)) return;
    cache->magic = 0;
    (void)hipFree(cache->kv.k);
    (void)hipFree(cache->kv.v);
    (void)hipFree(cache->kv.sz);
    (void)hipFree(cache->kv.partial);
    delete cache;
}

int tm_kv_append(tm_kv_cache* cache, const uint16_t* K_new, const uint16_t* V_new, const int32_t* positions, int count,
                 tm_stream stream)
{
    if (!valid_kv(cache)) return fail(TM_EINVAL, "cache handle is null or invalid");
    if (count == 0) return TM_OK;
    if (!K_new || !V_new || !positions) return fail(TM_EINVAL, "K_new, V_new or positions is null");
    if (count < 0 || count > cache->kv.cap) return fail(TM_EINVAL, "count = %d out of range", count);
    if (((uintptr_t)K_new & 1) || ((uintptr_t)V_new & 1) || ((uintptr_t)positions & 3)) return fail(TM_EINVAL, "misaligned input");
    if (cache->kv.bits == 4 && ((((uintptr_t)K_new | (uintptr_t)V_new) & 15)))
        return fail(TM_EINVAL, "a 4-bit cache needs 16-byte aligned K_new and V_new");
    int dev;
    int rc = check_device(&dev);
    if (rc != TM_OK) return rc;
    if (dev != cache->device) return fail(TM_EINVAL, "cache lives on device %d, current device is %d", cache->device, dev);
    hipError_t e = launch_kv_append(cache->kv, K_new, V_new, positions, count, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "kv append launch");
    return TM_OK;
}

int tm_attn_decode(const uint16_t* Q, const tm_kv_cache* cache, const int32_t* lens, uint16_t* O, int q_heads, float scale,
                   int max_len, tm_stream stream)
{
    if (!valid_kv(cache)) return fail(TM_EINVAL, "cache handle is null or invalid");
    if (!Q || !O || !lens) return fail(TM_EINVAL, "Q, O or lens is null");
    if (((uintptr_t)Q & 15) || ((uintptr_t)O & 15) || ((uintptr_t)lens & 3)) return fail(TM_EINVAL, "misaligned Q, O or lens");
    const int hk = cache->kv.heads;
    if (q_heads <= 0 || q_heads % hk || q_heads / hk > 128)
        return fail(TM_EINVAL, "q_heads = %d must be 1..128 times the cache's %d heads", q_heads, hk);
    if (!(scale > 0.0f) || !(scale < 1.0e6f)) return fail(TM_EINVAL, "scale out of range");
    if (max_len <= 0 || max_len > cache->kv.cap) max_len = cache->kv.cap;
    int dev;
    int rc = check_device(&dev);
    if (rc != TM_OK) return rc;
    if (dev != cache->device) return fail(TM_EINVAL, "cache lives on device %d, current device is %d", cache->device, dev);
    hipError_t e = launch_attn_decode(cache->kv, Q, lens, O, q_heads, scale, max_len, g_dev[dev].num_cu, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "attention launch");
    return TM_OK;
}

int tm_attn_prefill(const uint16_t* Q, const tm_kv_cache* cache, const int32_t* positions, const int32_t* counts, int count,
                    uint16_t* O, int q_heads, float scale, tm_stream stream)
{
    if (!valid_kv(cache)) return fail(TM_EINVAL, "cache handle is null or invalid");
    if (!Q || !O || !positions) return fail(TM_EINVAL, "Q, O or positions is null");
    if (((uintptr_t)Q & 15) || ((uintptr_t)O & 15) || ((uintptr_t)positions & 3) || ((uintptr_t)counts & 3))
        return fail(TM_EINVAL, "misaligned Q, O, positions or counts");
    const int hk = cache->kv.heads;
    if (q_heads <= 0 || q_heads % hk || q_heads / hk > 128)
        return fail(TM_EINVAL, "q_heads = %d must be 1..128 times the cache's %d heads", q_heads, hk);
    if (!(scale > 0.0f) || !(scale < 1.0e6f)) return fail(TM_EINVAL, "scale out of range");
    const int tpg = 16 / (q_heads / hk < 16 ? q_heads / hk : 16);     // tokens per CTA in the widest pass
    if (count <= 0 || count > 65535 * tpg) return fail(TM_EINVAL, "count = %d out of range (1..%d)", count, 65535 * tpg);
    if ((uint64_t)cache->kv.batch * (uint64_t)count >= (1ull << 31)) return fail(TM_EINVAL, "batch * count too large");
    int dev;
    int rc = check_device(&dev);
    if (rc != TM_OK) return rc;
    if (dev != cache->device) return fail(TM_EINVAL, "cache lives on device %d, current device is %d", cache->device, dev);
    hipError_t e = launch_attn_prefill(cache->kv, Q, positions, counts, count, O, q_heads, scale, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "attention launch");
    return TM_OK;
}

int tm_kv_raw(const tm_kv_cache* cache, void** k_codes, void** v_codes, void** pairs, size_t* code_bytes, size_t* pair_bytes)
{
    if (!valid_kv(cache)) return fail(TM_EINVAL, "cache handle is null or invalid");
    if (k_codes) *k_codes = cache->kv.k;
    if (v_codes) *v_codes = cache->kv.v;
    if (pairs) *pairs = cache->kv.sz;
    if (code_bytes) *code_bytes = cache->code_bytes;
    if (pair_bytes) *pair_bytes = cache->pair_bytes;
    return TM_OK;
}

}  // extern "C"
