// Offline hardware-aware weight packing (paper Sec. 4.1) and its inverse, plus the two measurement kernels.
//
// On gfx950 the operand layout of the 16x16x32 fp16 matrix-core instruction is a closed-form index map, so the
// paper's four steps (widen, pass through the fp16 fragment-load path, compress, store coalesced) collapse into a
// gather: a 128 x 128 block of the interchange matrix is staged in LDS with coalesced row reads, and every thread
// assembles complete 32-bit words of the fragment-ordered buffer, which are written as contiguous 1 KiB units.
#include "tm_w4_device.h"
#include "tm_w4_host.h"

namespace tmw4 {

// LAYOUT selects how the interchange words are read (values of tm_layout):
//   0  u32 [K][N/8], nibble t = column 8j+t          1  same shape, nibble p = column 8j + (0,2,4,6,1,3,5,7)[p]
//   2  u32 [K/8][N], nibble t = row 8i+t
// Layouts 0 and 1 stage the block as 128 rows x 16 words; layout 2 as 16 row-words x 128 columns, where the eight
// rows one output word needs (32t + 8h + e, e = 0..7) are exactly one staged word.
template <int LAYOUT>
__global__ __launch_bounds__(256) void repack_w4_kernel(const uint32_t* __restrict__ qweight,
                                                        uint32_t* __restrict__ out, int K, int N)
{
    // A CTA covers 128 rows x kTiles 16-column tiles.  The N-major layouts take 16 tiles so that a row segment is
    // 32 words = 128 contiguous bytes (with 64-byte segments the memory system fetched twice the bytes read).
    constexpr int kTiles = LAYOUT == 2 ? 8 : 16;
    constexpr int kRows = LAYOUT == 2 ? 16 : 128, kPitch = LAYOUT == 2 ? 132 : 33;
    __shared__ uint32_t tile[kRows][kPitch];
    const int KU = K / kUnitK, NT = N / kUnitN, NW = N / 8;
    const int ku = blockIdx.y;
    const int nt0 = blockIdx.x * kTiles;
    const int tid = threadIdx.x;
    constexpr int kWords = LAYOUT == 2 ? 16 * 128 : 128 * 32;      // staged words per CTA
    for (int i = 0; i < kWords / 256; ++i) {
        int idx = i * 256 + tid;
        if constexpr (LAYOUT == 2) {
            int row = idx >> 7, col = idx & 127;
            int gc = nt0 * 16 + col;
            tile[row][col] = gc < N ? qweight[(size_t)(ku * 16 + row) * N + gc] : 0u;
        } else {
            int row = idx >> 5, wc = idx & 31;
            int gw = nt0 * 2 + wc;
            uint32_t v = gw < NW ? qweight[(size_t)(ku * kUnitK + row) * NW + gw] : 0u;
            if constexpr (LAYOUT == 1) {
                uint32_t u = 0;                      // nibble p -> nibble o(p) = 2*(p&3) + (p>>2)
#pragma unroll
                for (int p = 0; p < 8; ++p) u |= ((v >> (4 * p)) & 0xFu) << (4 * (2 * (p & 3) + (p >> 2)));
                v = u;
            }
            tile[row][wc] = v;
        }
    }
    __syncthreads();
    const int lane = tid >> 2, t = tid & 3;
    const int c = lane & 15, h = lane >> 4;
    for (int j = 0; j < kTiles; ++j) {
        int nt = nt0 + j;
        if (nt >= NT) break;
        int col = 16 * j + c;
        uint32_t w = 0;
        if constexpr (LAYOUT == 2) {
            uint32_t v = tile[4 * t + h][col];
#pragma unroll
            for (int e = 0; e < 8; ++e) w |= ((v >> (4 * e)) & 0xFu) << (4 * (4 * (e & 1) + (e >> 1)));
        } else {
            int wc = col >> 3, sh = 4 * (col & 7);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint32_t nib = (tile[32 * t + 8 * h + e][wc] >> sh) & 0xFu;
                w |= nib << (4 * (4 * (e & 1) + (e >> 1)));
            }
        }
        out[((size_t)nt * KU + ku) * kUnitWords + tid] = w;
    }
}

// 8-bit codes: interchange words u32 [K][N/4] (byte t = column 4j+t) -> units of 16 columns x 64 rows, word
// 4*lane + 2*tt + hf = rows 64*ks + 32*tt + 8*h + 4*hf + b in byte b (lane = 16*h + c).  A CTA stages 128 rows x 128
// columns (128-byte row segments) and writes the 8 x 2 units they make.
__global__ __launch_bounds__(256) void repack_w8_kernel(const uint32_t* __restrict__ qweight,
                                                        uint32_t* __restrict__ out, int K, int N)
{
    __shared__ uint32_t tile[128][33];
    const int KS = K / 64, NT = N / kUnitN, NW = N / 4;
    const int ku = blockIdx.y;
    const int nt0 = blockIdx.x * 8;
    const int tid = threadIdx.x;
    for (int i = 0; i < 16; ++i) {
        int idx = i * 256 + tid;
        int row = idx >> 5, wc = idx & 31;
        int gw = nt0 * 4 + wc;
        tile[row][wc] = gw < NW ? qweight[(size_t)(ku * 128 + row) * NW + gw] : 0u;
    }
    __syncthreads();
    const int lane = tid >> 2, wi = tid & 3;
    const int c = lane & 15, h = lane >> 4;
    const int r0 = 32 * (wi >> 1) + 8 * h + 4 * (wi & 1);
    for (int j = 0; j < 8; ++j) {
        int nt = nt0 + j;
        if (nt >= NT) break;
        int col = 16 * j + c;
        int wc = col >> 2, sh = 8 * (col & 3);
#pragma unroll
        for (int su = 0; su < 2; ++su) {
            uint32_t w = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) w |= ((tile[64 * su + r0 + b][wc] >> sh) & 0xFFu) << (8 * b);
            out[((size_t)nt * KS + 2 * ku + su) * kUnitWords + tid] = w;
        }
    }
}

// ZFMT: 0 zeros are fp16 [G][N]; 1 u32 [G][N/8], nibble t = column 8j+t; 2 u32 [G][N/8], nibble p = column
// 8j + (0,2,4,6,1,3,5,7)[p].  Packed integers are widened to the fp16 pattern the GEMM kernels expect.
// G counts the stored groups; source row g / rep feeds stored group g (rep > 1 when the caller's groups are coarser
// than the 128 rows the kernels work with).  zeros == nullptr stands for the symmetric zero-point 8.
template <int ZFMT>
__global__ __launch_bounds__(256) void repack_sz_kernel(const uint16_t* __restrict__ scales,
                                                        const void* __restrict__ zeros,
                                                        uint32_t* __restrict__ out, int G, int N, int rep, uint32_t sym_zero)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t total = (size_t)G * N;
    if (idx >= total) return;
    int c = idx & 15;
    size_t r = idx >> 4;
    int g = (int)(r % G) / rep;
    int nt = (int)(r / G);
    int n = 16 * nt + c;
    size_t src = (size_t)g * N + n;
    uint32_t zb;
    if (!zeros) {
        zb = sym_zero;                             // fp16 8.0 (4-bit codes) or 128.0 (8-bit codes)
    } else if constexpr (ZFMT == 0) {
        zb = ((const uint16_t*)zeros)[src];
    } else {
        int t = n & 7;
        int pos = ZFMT == 1 ? t : (t >> 1) + 4 * (t & 1);
        uint32_t zi = (((const uint32_t*)zeros)[(size_t)g * (N / 8) + (n >> 3)] >> (4 * pos)) & 0xFu;
        _Float16 zf = (_Float16)(int)zi;
        zb = __builtin_bit_cast(unsigned short, zf);
    }
    out[idx] = (uint32_t)scales[src] | (zb << 16);
}

// Inverse permutation (test hook): one thread per interchange word (k, j).
__global__ __launch_bounds__(256) void unpack_w4_kernel(const uint32_t* __restrict__ packed,
                                                        uint32_t* __restrict__ qweight, int K, int N)
{
    const int KU = K / kUnitK, NW = N / 8;
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)K * NW) return;
    int k = (int)(idx / NW), j = (int)(idx % NW);
    int ku = k >> 7, kk = k & 127;
    int t = kk >> 5, h = (kk >> 3) & 3, e = kk & 7;
    int p = 4 * (e & 1) + (e >> 1);
    uint32_t w = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int n = 8 * j + i;
        int nt = n >> 4, c = n & 15;
        uint32_t src = packed[((size_t)nt * KU + ku) * kUnitWords + 4 * (16 * h + c) + t];
        w |= ((src >> (4 * p)) & 0xFu) << (4 * i);
    }
    qweight[idx] = w;
}

__global__ __launch_bounds__(256) void unpack_sz_kernel(const uint32_t* __restrict__ sz, uint16_t* __restrict__ scales,
                                                        uint16_t* __restrict__ zeros, int G, int N)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)G * N) return;
    int g = (int)(idx / N), n = (int)(idx % N);
    uint32_t w = sz[((size_t)(n >> 4) * G + g) * 16 + (n & 15)];
    if (scales) scales[idx] = (uint16_t)(w & 0xFFFFu);
    if (zeros) zeros[idx] = (uint16_t)(w >> 16);
}

__global__ __launch_bounds__(256) void copy16_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16)
{
    size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void read16_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* sink)
{
    size_t stride = (size_t)gridDim.x * 256;
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) acc ^= src[i];
    uint32_t v = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (v == 0x9E3779B9u) *sink = v;               // practically never taken; keeps the loads alive
}

// A loop of nothing but matrix instructions: eight independent 16x16x32 fp16 MFMAs per iteration and wave, operands in
// registers.  What the matrix pipes of this chip sustain at the clock it holds under that load; the first wave also
// reports how far the shader clock counter and the constant-rate counter advanced over its loop.  pattern 0: zero
// operands (the pipes switch the least); 1: values in (-1, 1) that differ per lane and element, the same pair of
// operands for every instruction; 2: a different pair for each of the eight instructions of an iteration, so that the
// operand latches switch with every instruction, as they do in a GEMM.
__global__ __launch_bounds__(1024) void mfma_loop_kernel(int iters, int pattern, uint32_t* out)
{
    const uint32_t lane = threadIdx.x & 63;
    f16x8 a[8], b[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t h = ((lane * 8u + (uint32_t)i + 1u) * 2654435761u) ^ (pattern == 2 ? (uint32_t)j * 0x9E3779B9u : 0u);
            const float va = pattern ? (float)((int)(h >> 20 & 255) - 128) * (1.0f / 128.0f) : 0.0f;
            const float vb = pattern ? (float)((int)(h >> 8 & 255) - 128) * (1.0f / 128.0f) : 0.0f;
            a[j][i] = (_Float16)va;
            b[j][i] = (_Float16)vb;
        }
    }
    f32x4 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint64_t c0 = clock64(), r0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = mfma16x16x32(a[j], b[j], acc[j]);
    }
    const uint64_t c1 = clock64(), r1 = wall_clock64();
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) sum += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = (uint32_t)(c1 - c0);
        out[1] = (uint32_t)(r1 - r0);
    }
    if (sum == 12345.6789f) out[2] = 1;            // practically never taken; keeps the loop alive
}

// One wave that does nothing but watch two counters: it sleeps through `delay` ticks of the constant-rate counter, then
// records how far the shader clock counter and the constant-rate counter advance over the next `ticks`.  Launched on a
// second stream *before* other work (it needs a wave slot and a few registers, which a launch that fills the register
// file leaves to nobody), it reports the shader clock the chip holds under that work.  Ends by itself: the loop is
// bounded by its iteration count whatever the counters do.
__global__ __launch_bounds__(64) void clock_probe_kernel(uint32_t delay, uint32_t ticks, int max_rounds, uint32_t* out)
{
    const uint64_t start = wall_clock64();
    uint64_t c0 = clock64(), r0 = start, c1 = c0, r1 = r0;
    bool watching = delay == 0;
    for (int i = 0; i < max_rounds; ++i) {
        __builtin_amdgcn_s_sleep(16);              // about a thousand clocks asleep per round: no issue slots taken
        c1 = clock64();
        r1 = wall_clock64();
        if (!watching) {
            if (r1 - start >= delay) {
                watching = true;
                c0 = c1;
                r0 = r1;
            }
        } else if (r1 - r0 >= ticks) {
            break;
        }
    }
    if (threadIdx.x == 0) {
        out[0] = watching ? (uint32_t)(c1 - c0) : 0u;
        out[1] = watching ? (uint32_t)(r1 - r0) : 0u;
    }
}

// The read-only stream in a chosen launch shape, for finding the best streaming shape of this chip at a given byte
// count: every thread keeps U 128-bit loads in flight per round; CHUNKED gives each CTA one contiguous slice of the
// buffer (as a weight-streaming CTA has) instead of interleaving the CTAs; NT uses the non-temporal load policy.
template <int U, bool NT, bool CHUNKED>
__global__ void read_shape_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* sink)
{
    const size_t threads = blockDim.x;
    size_t begin, end, stride;
    if (CHUNKED) {
        const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
        begin = (size_t)blockIdx.x * per + threadIdx.x;
        end = min(n16, (size_t)(blockIdx.x + 1) * per);
        stride = threads;
    } else {
        begin = (size_t)blockIdx.x * threads + threadIdx.x;
        end = n16;
        stride = (size_t)gridDim.x * threads;
    }
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = begin; i < end; i += stride * U) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t at = i + u * stride;
            v[u] = u32x4{0, 0, 0, 0};
            if (at < end) v[u] = NT ? __builtin_nontemporal_load(src + at) : src[at];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9E3779B9u) *sink = x;               // practically never taken; keeps the loads alive
}

// Every CTA reads the WHOLE buffer (as every CTA of a GEMM reads all of X): with a buffer that stays in the L2 this
// measures how fast a compute unit can be fed from the L2, apart from HBM.  CTA b starts a b-th of the way in and
// wraps, so that the CTAs do not all ask for the same line at the same moment.
template <int U, bool NT>
__global__ void read_shared_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* sink)
{
    const size_t threads = blockDim.x;
    const size_t rot = (n16 / gridDim.x) * blockIdx.x;
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = threadIdx.x; i < n16; i += threads * U) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            size_t at = i + u * threads;
            v[u] = u32x4{0, 0, 0, 0};
            if (at < n16) {
                at += rot;
                if (at >= n16) at -= n16;
                v[u] = NT ? __builtin_nontemporal_load(src + at) : src[at];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9E3779B9u) *sink = x;
}

// Activation-order checkpoints: row i of the matrix that gets packed is row perm[i] of the checkpoint, so that the
// rows of one K-group become consecutive.  N-major words move whole; a K-major word is rebuilt from eight rows.
__global__ __launch_bounds__(256) void permute_rows_kernel(const uint32_t* __restrict__ in, const int32_t* __restrict__ perm,
                                                           uint32_t* __restrict__ out, int K, int N, int k_major)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (k_major) {
        if (idx >= (size_t)(K / 8) * N) return;
        int i = (int)(idx / N), n = (int)(idx % N);
        uint32_t w = 0;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            int src = perm[8 * i + t];
            w |= ((in[(size_t)(src >> 3) * N + n] >> (4 * (src & 7))) & 0xFu) << (4 * t);
        }
        out[idx] = w;
    } else {
        const int NW = N / 8;
        if (idx >= (size_t)K * NW) return;
        int r = (int)(idx / NW), j = (int)(idx % NW);
        out[idx] = in[(size_t)perm[r] * NW + j];
    }
}

// X'[m][i] = X[m][perm[i]]: the activations follow the rows of the packed matrix.  One thread per 16-byte chunk.
__global__ __launch_bounds__(256) void permute_x_kernel(const uint16_t* __restrict__ X, const int32_t* __restrict__ perm,
                                                        uint16_t* __restrict__ out, int M, int K)
{
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int KC = K / 8;
    if (idx >= (size_t)M * KC) return;
    int m = (int)(idx / KC), c = (int)(idx % KC);
    const uint16_t* row = X + (size_t)m * K;
    u32x4 v;
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = row[perm[8 * c + e]];
    v.x = h[0] | (h[1] << 16);
    v.y = h[2] | (h[3] << 16);
    v.z = h[4] | (h[5] << 16);
    v.w = h[6] | (h[7] << 16);
    *(u32x4*)(out + (size_t)m * K + 8 * c) = v;
}

// Column interleave of a fused [gate | up] weight (N = 2*I columns): output column 2j is gate column j, 2j + 1 is up
// column I + j, so that every thread of a GEMM epilogue that holds two neighbouring columns holds a matching pair.
// Codes: output word (k, w) = columns 8w .. 8w+7 takes four nibbles of gate word w/2 and four of up word I/8 + w/2.
__global__ __launch_bounds__(256) void interleave_gate_up_q_kernel(const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
                                                                   int K, int N)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int words = N / 8;
    if (idx >= (size_t)K * words) return;
    const int w = (int)(idx % words);
    const size_t row = idx / words * words;
    const int sh = 16 * (w & 1);                                // nibbles 0..3 or 4..7 of the source words
    const uint32_t g = in[row + (w >> 1)] >> sh, u = in[row + (N / 16) + (w >> 1)] >> sh;
    uint32_t o = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) o |= (((g >> (4 * i)) & 15u) << (8 * i)) | (((u >> (4 * i)) & 15u) << (8 * i + 4));
    out[idx] = o;
}

__global__ __launch_bounds__(256) void interleave_gate_up_f16_kernel(const uint16_t* __restrict__ in, uint16_t* __restrict__ out,
                                                                     int G, int N)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)G * N) return;
    const int c = (int)(idx % N);
    out[idx] = in[idx - c + ((c & 1) ? N / 2 + (c >> 1) : (c >> 1))];
}

// ------------------------------------------------------------------------------------------ host launchers

hipError_t launch_permute_rows(const uint32_t* in, const int32_t* perm, uint32_t* out, int K, int N, int k_major,
                               hipStream_t stream)
{
    size_t total = (size_t)K * N / 8;
    hipLaunchKernelGGL(permute_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, in, perm, out, K,
                       N, k_major);
    return hipGetLastError();
}

hipError_t launch_interleave_gate_up(const uint32_t* q, const uint16_t* s, const uint16_t* z, uint32_t* q_out, uint16_t* s_out,
                                     uint16_t* z_out, int K, int N, int G, hipStream_t stream)
{
    const size_t nq = (size_t)K * N / 8, nf = (size_t)G * N;
    hipLaunchKernelGGL(interleave_gate_up_q_kernel, dim3((unsigned)((nq + 255) / 256)), dim3(256), 0, stream, q, q_out, K, N);
    hipLaunchKernelGGL(interleave_gate_up_f16_kernel, dim3((unsigned)((nf + 255) / 256)), dim3(256), 0, stream, s, s_out, G, N);
    if (z) hipLaunchKernelGGL(interleave_gate_up_f16_kernel, dim3((unsigned)((nf + 255) / 256)), dim3(256), 0, stream, z, z_out, G, N);
    return hipGetLastError();
}

hipError_t launch_permute_x(const uint16_t* X, const int32_t* perm, uint16_t* out, int M, int K, hipStream_t stream)
{
    size_t total = (size_t)M * (K / 8);
    hipLaunchKernelGGL(permute_x_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, X, perm, out, M, K);
    return hipGetLastError();
}


hipError_t launch_repack(const uint32_t* qweight, const uint16_t* scales, const void* zeros, uint32_t* w_out,
                         uint32_t* sz_out, int K, int N, int group, int layout, hipStream_t stream)
{
    // group is what the caller's scales are laid out for; coarser groups than 128 rows are stored as 128
    const int stored = group > 128 ? 128 : group, rep = group / stored;
    const int KU = K / kUnitK, NT = N / kUnitN, G = K / stored;
    const int tiles_per_cta = layout == 2 ? 8 : 16;     // as in repack_w4_kernel
    dim3 grid((NT + tiles_per_cta - 1) / tiles_per_cta, KU);
    size_t total = (size_t)G * N;
    dim3 szgrid((unsigned)((total + 255) / 256));
    switch (layout) {
    case 0:
        hipLaunchKernelGGL(repack_w4_kernel<0>, grid, dim3(256), 0, stream, qweight, w_out, K, N);
        hipLaunchKernelGGL(repack_sz_kernel<0>, szgrid, dim3(256), 0, stream, scales, zeros, sz_out, G, N, rep, 0x4800u);
        break;
    case 1:
        hipLaunchKernelGGL(repack_w4_kernel<1>, grid, dim3(256), 0, stream, qweight, w_out, K, N);
        hipLaunchKernelGGL(repack_sz_kernel<2>, szgrid, dim3(256), 0, stream, scales, zeros, sz_out, G, N, rep, 0x4800u);
        break;
    case 2:
        hipLaunchKernelGGL(repack_w4_kernel<2>, grid, dim3(256), 0, stream, qweight, w_out, K, N);
        hipLaunchKernelGGL(repack_sz_kernel<1>, szgrid, dim3(256), 0, stream, scales, zeros, sz_out, G, N, rep, 0x4800u);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_repack8(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros, uint32_t* w_out,
                          uint32_t* sz_out, int K, int N, int group, bool fp8, hipStream_t stream)
{
    const int stored = group > 128 ? 128 : group, rep = group / stored;
    const int NT = N / kUnitN, G = K / stored;
    dim3 grid((NT + 7) / 8, K / 128);
    hipLaunchKernelGGL(repack_w8_kernel, grid, dim3(256), 0, stream, qweight, w_out, K, N);
    size_t total = (size_t)G * N;
    hipLaunchKernelGGL(repack_sz_kernel<0>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, scales,
                       (const void*)zeros, sz_out, G, N, rep, fp8 ? 0u : 0x5800u);   // FP8 codes carry no zero-point
    return hipGetLastError();
}

hipError_t launch_unpack(const uint32_t* w, const uint32_t* sz, uint32_t* qweight_out, uint16_t* scales_out,
                         uint16_t* zeros_out, int K, int N, int group, hipStream_t stream)
{
    const int G = K / group;
    if (qweight_out) {
        size_t total = (size_t)K * (N / 8);
        hipLaunchKernelGGL(unpack_w4_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, w,
                           qweight_out, K, N);
    }
    if (scales_out || zeros_out) {
        size_t total = (size_t)G * N;
        hipLaunchKernelGGL(unpack_sz_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, sz,
                           scales_out, zeros_out, G, N);
    }
    return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream)
{
    size_t n16 = bytes / 16;
    unsigned blocks = (unsigned)((n16 + 255) / 256 < 8192 ? (n16 + 255) / 256 : 8192);
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(copy16_kernel, dim3(blocks), dim3(256), 0, stream, (u32x4*)dst, (const u32x4*)src, n16);
    return hipGetLastError();
}

hipError_t launch_read(const void* src, size_t bytes, void* sink, hipStream_t stream)
{
    size_t n16 = bytes / 16;
    unsigned blocks = (unsigned)((n16 + 255) / 256 < 8192 ? (n16 + 255) / 256 : 8192);
    if (blocks == 0) return hipSuccess;
    hipLaunchKernelGGL(read16_kernel, dim3(blocks), dim3(256), 0, stream, (const u32x4*)src, n16, (uint32_t*)sink);
    return hipGetLastError();
}

template <int U>
static void launch_read_u(const void* src, size_t n16, void* sink, unsigned grid, unsigned block, int flags, hipStream_t stream)
{
    const u32x4* p = (const u32x4*)src;
    uint32_t* sk = (uint32_t*)sink;
    if (flags & 4) {
        if (flags & 1) hipLaunchKernelGGL((read_shared_kernel<U, true>), dim3(grid), dim3(block), 0, stream, p, n16, sk);
        else hipLaunchKernelGGL((read_shared_kernel<U, false>), dim3(grid), dim3(block), 0, stream, p, n16, sk);
        return;
    }
    switch (flags & 3) {
        case 0: hipLaunchKernelGGL((read_shape_kernel<U, false, false>), dim3(grid), dim3(block), 0, stream, p, n16, sk); break;
        case 1: hipLaunchKernelGGL((read_shape_kernel<U, true, false>), dim3(grid), dim3(block), 0, stream, p, n16, sk); break;
        case 2: hipLaunchKernelGGL((read_shape_kernel<U, false, true>), dim3(grid), dim3(block), 0, stream, p, n16, sk); break;
        default: hipLaunchKernelGGL((read_shape_kernel<U, true, true>), dim3(grid), dim3(block), 0, stream, p, n16, sk); break;
    }
}

hipError_t launch_read_shape(const void* src, size_t bytes, void* sink, unsigned grid, unsigned block, int unroll, int flags,
                             hipStream_t stream)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    switch (unroll) {
        case 1: launch_read_u<1>(src, n16, sink, grid, block, flags, stream); break;
        case 2: launch_read_u<2>(src, n16, sink, grid, block, flags, stream); break;
        case 4: launch_read_u<4>(src, n16, sink, grid, block, flags, stream); break;
        case 8: launch_read_u<8>(src, n16, sink, grid, block, flags, stream); break;
        case 16: launch_read_u<16>(src, n16, sink, grid, block, flags, stream); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_mfma_loop(void* out, unsigned grid, unsigned block, int iters, int pattern, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(grid), dim3(block), 0, stream, iters, pattern, (uint32_t*)out);
    return hipGetLastError();
}

hipError_t launch_clock_probe(void* out, uint32_t delay, uint32_t ticks, int max_rounds, hipStream_t stream)
{
    hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, stream, delay, ticks, max_rounds, (uint32_t*)out);
    return hipGetLastError();
}

}  // namespace tmw4
