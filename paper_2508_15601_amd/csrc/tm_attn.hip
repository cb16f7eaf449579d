// Decode attention over an 8-bit KV cache (paper Sec. 3.3 attention pipeline; Sec. 4.2, 4.3, 4.4), and the kernel that
// quantises new keys / values into the cache.
//
// What differs from the paper's design, which rearranges Q in shared memory so that a 32-lane fragment load of the
// low-bit K tile lines up with it, and stages K/V tiles through shared memory:
//   - The matrix-core operand layout of gfx950 is an explicit index map, and a dot product does not care in which
//     order its 128 dimensions are visited.  Lane (c, h) of a wave therefore simply takes the 32 consecutive key bytes
//     32h .. 32h+31 of "its" token as the k-values of the four MFMA steps, and the query operand is loaded once in that
//     same order.  That is the whole of the head alignment: no LDS, no shuffle, for any code width.
//   - Scores are computed transposed (S^T = K Q^T, tokens as rows).  The MFMA result layout then hands every lane the
//     probabilities of exactly the tokens whose value bytes it needs as the k-values of O^T = V^T P^T, so P never
//     leaves its registers either; the cache stores V in blocks of 32 tokens in that operand order.
//   - Scale and zero-point are per token, i.e. per row of S^T and per k-index of the second product: they are applied
//     to four scores and eight probabilities per lane and block instead of to 2 x 128 code values per token.  The codes
//     enter the matrix cores as 1024 + q (one byte permute per two codes); the bias and the zero-point leave through
//     one fp32 term per query head.
//   - The cache itself is stored in operand order (blocks of 32 tokens x 128 dimensions), the hardware-aware packing of
//     the weights applied to K and V: every load instruction of a wave reads 1 KiB of consecutive bytes (row-major keys
//     had every instruction touch half of sixteen 128-byte rows: 4.1 instead of 5.7 TB/s).
//   - The codes of the next two 32-token blocks are in flight in registers while the current block is multiplied; the
//     blocks' scale/zero words go through a small per-wave LDS ring (direct-to-LDS loads); a CTA's waves take blocks
//     round-robin and meet in LDS at the end; long contexts are split across CTAs and merged by a second, tiny kernel.
#include "tm_w4_host.h"

namespace tmw4 {

namespace {


constexpr int kHeadDim = 128;
constexpr float kNegBig = -1.0e30f;     // "minus infinity" that stays finite under subtraction
constexpr float kMaskFloor = -1.0e20f;  // far below any score, far above kNegBig: exp2(kNegBig - kMaskFloor) is 0
constexpr int kNonTemporal = 2;         // cache-policy bit of a buffer load: streamed once, do not keep

// 2^x by the hardware instruction alone: arguments here are <= 0 and a result below the smallest normal number may
// flush to zero (the library function spends four more instructions per call on that range).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float xor_max(float v, int mask) { return fmaxf(v, __shfl_xor(v, mask)); }
__device__ __forceinline__ float xor_add(float v, int mask) { return v + __shfl_xor(v, mask); }

// ------------------------------------------------------------------------------------------------ quantise + store
// One wave per (sequence, new token, KV head); lane l owns dimensions l and l + 64 of the key and of the value.
__global__ __launch_bounds__(64) void kv_append_kernel(AttnCache kv, const uint16_t* __restrict__ Kn,
                                                       const uint16_t* __restrict__ Vn,
                                                       const int32_t* __restrict__ positions, int count)
{
    const int lane = threadIdx.x;
    const int h = blockIdx.x % kv.heads;
    const int j = (blockIdx.x / kv.heads) % count;
    const int b = blockIdx.x / (kv.heads * count);
    const int t = positions[b] + j;
    if (t < 0 || t >= kv.cap) return;                       // wave-uniform
    const size_t src = (((size_t)b * count + j) * kv.heads + h) * kHeadDim;
    const size_t bh = (size_t)b * kv.heads + h;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const uint16_t* x = (which ? Vn : Kn) + src;
        const float x0 = (float)__builtin_bit_cast(_Float16, x[lane]);
        const float x1 = (float)__builtin_bit_cast(_Float16, x[lane + 64]);
        float mn = fminf(x0, x1), mx = fmaxf(x0, x1);
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            mn = fminf(mn, __shfl_xor(mn, m));
            mx = fmaxf(mx, __shfl_xor(mx, m));
        }
        _Float16 s16 = (_Float16)((mx - mn) / 255.0f);
        float sf = (float)s16;
        if (!(sf > 0.0f) || __builtin_isinf(sf)) {
            sf = 1.0f;
            s16 = (_Float16)1.0f;
        }
        const float zf = fminf(fmaxf(rintf(-mn / sf), 0.0f), 255.0f);
        const uint32_t q0 = (uint32_t)fminf(fmaxf(rintf(x0 / sf) + zf, 0.0f), 255.0f);
        const uint32_t q1 = (uint32_t)fminf(fmaxf(rintf(x1 / sf) + zf, 0.0f), 255.0f);
        const int u = t & 31;
        uint8_t* blk = (which ? kv.v : kv.k) + (bh * (kv.cap / 32) + (t >> 5)) * 4096;
        if (which == 0) {
            // dimension d -> byte ((j*2 + half)*64 + 16*hh + c)*16 + x, j = u/16, c = u%16, hh = d/32, half = (d%32)/16
            const int j = u >> 4, c = u & 15;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int d = lane + 64 * k;
                blk[((j * 2 + ((d & 31) >> 4)) * 64 + 16 * (d >> 5) + c) * 16 + (d & 15)] = (uint8_t)(k ? q1 : q0);
            }
        } else {
            // dimension d = 16*i + c -> byte ((i/2)*64 + 16*hh + c)*16 + (i%2)*8 + e, hh = (u%16)/4, e = u%4 + 4*(u/16)
            const int hh = (u & 15) >> 2, e = (u & 3) + 4 * (u >> 4);
            const int c = lane & 15;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int i = (lane >> 4) + 4 * k;
                blk[((i >> 1) * 64 + 16 * hh + c) * 16 + (i & 1) * 8 + e] = (uint8_t)(k ? q1 : q0);
            }
        }
        if (lane == 0) {
            const _Float16 z16 = (_Float16)zf;
            kv.sz[(bh * kv.cap + t) * 2 + which] =
                (uint32_t)__builtin_bit_cast(unsigned short, s16) | ((uint32_t)__builtin_bit_cast(unsigned short, z16) << 16);
        }
    }
}

// Prompt-sized appends: one CTA of 256 threads per (KV head, 32-token block touched, sequence).  Sixteen lanes share a
// token (eight dimensions = one 16-byte load each), so a wave quantises four tokens at a time; codes are assembled in
// LDS in cache order and leave as 16-byte stores: a fully covered block is written as 2 x 4 KiB of consecutive bytes.
// A partly covered block keeps its other tokens: key chunks belong to one token each (stored or skipped), value chunks
// hold eight tokens and are merged bytewise with what the cache holds (calls on one cache are ordered on one stream).
// Same arithmetic, operation for operation, as kv_append_kernel.
__global__ __launch_bounds__(256) void kv_append_block_kernel(AttnCache kv, const uint16_t* __restrict__ Kn,
                                                              const uint16_t* __restrict__ Vn,
                                                              const int32_t* __restrict__ positions, int count)
{
    __shared__ __align__(16) uint8_t lds[2][4096];
    const int h = blockIdx.x, b = blockIdx.z;
    const int pos = positions[b];
    long first = pos < 0 ? 0 : pos, last = (long)pos + count;         // tokens [first, last) of the cache are new
    if (last > kv.cap) last = kv.cap;
    if (first >= last) return;
    const int tb = (int)(first >> 5) + (int)blockIdx.y;                // this CTA's block of 32 tokens
    const long t0 = first > (long)tb * 32 ? first : (long)tb * 32;
    const long t1 = last < (long)(tb + 1) * 32 ? last : (long)(tb + 1) * 32;
    if (t0 >= t1) return;                                              // CTA-uniform
    const int u0 = (int)(t0 - (long)tb * 32), u1 = (int)(t1 - (long)tb * 32);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15;                                         // dimensions 8*sub .. 8*sub + 7
    const size_t bh = (size_t)b * kv.heads + h;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int which = it >> 1;                                     // 0: keys, 1: values
        const int u = wave * 8 + (it & 1) * 4 + (lane >> 4);           // token of the block
        const bool live = u >= u0 && u < u1;
        const long t = (long)tb * 32 + u;
        float x[8];
        if (live) {
            const size_t src = (((size_t)b * count + (size_t)(t - pos)) * kv.heads + h) * kHeadDim + 8 * sub;
            const u32x4 raw = *reinterpret_cast<const u32x4*>((which ? Vn : Kn) + src);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                x[2 * k] = (float)__builtin_bit_cast(_Float16, (unsigned short)(raw[k] & 0xffffu));
                x[2 * k + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(raw[k] >> 16));
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) x[k] = 0.f;
        }
        float mn = x[0], mx = x[0];
#pragma unroll
        for (int k = 1; k < 8; ++k) {
            mn = fminf(mn, x[k]);
            mx = fmaxf(mx, x[k]);
        }
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) {
            mn = fminf(mn, __shfl_xor(mn, m));
            mx = fmaxf(mx, __shfl_xor(mx, m));
        }
        _Float16 s16 = (_Float16)((mx - mn) / 255.0f);
        float sf = (float)s16;
        if (!(sf > 0.0f) || __builtin_isinf(sf)) {
            sf = 1.0f;
            s16 = (_Float16)1.0f;
        }
        const float zf = fminf(fmaxf(rintf(-mn / sf), 0.0f), 255.0f);
        uint32_t q[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) q[k] = (uint32_t)fminf(fmaxf(rintf(x[k] / sf) + zf, 0.0f), 255.0f);
        if (which == 0) {
            // dimensions 8*sub .. +7 of token u: eight consecutive bytes of chunk (j*2 + half)*64 + 16*hh + c
            const int d = 8 * sub;
            const int chunk = ((u >> 4) * 2 + ((d & 31) >> 4)) * 64 + 16 * (d >> 5) + (u & 15);
            u32x2 w;
            w[0] = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
            w[1] = q[4] | (q[5] << 8) | (q[6] << 16) | (q[7] << 24);
            *reinterpret_cast<u32x2*>(&lds[0][chunk * 16 + (d & 15)]) = w;
        } else {
            const int hh = (u & 15) >> 2, e = (u & 3) + 4 * (u >> 4);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int d = 8 * sub + k, i = d >> 4;
                lds[1][((i >> 1) * 64 + 16 * hh + (d & 15)) * 16 + (i & 1) * 8 + e] = (uint8_t)q[k];
            }
        }
        if (live && sub == 0) {
            const _Float16 z16 = (_Float16)zf;
            kv.sz[(bh * kv.cap + t) * 2 + which] =
                (uint32_t)__builtin_bit_cast(unsigned short, s16) | ((uint32_t)__builtin_bit_cast(unsigned short, z16) << 16);
        }
    }
    __syncthreads();
    const size_t blk = (bh * (kv.cap / 32) + tb) * 4096;
    const int chunk = threadIdx.x;                                     // 256 chunks of 16 bytes per block
    const u32x4 kc = *reinterpret_cast<const u32x4*>(&lds[0][chunk * 16]);
    u32x4 vc = *reinterpret_cast<const u32x4*>(&lds[1][chunk * 16]);
    u32x4* kdst = reinterpret_cast<u32x4*>(kv.k + blk) + chunk;
    u32x4* vdst = reinterpret_cast<u32x4*>(kv.v + blk) + chunk;
    if (u0 == 0 && u1 == 32) {
        *kdst = kc;
        *vdst = vc;
        return;
    }
    const int ku = (chunk >> 7) * 16 + (chunk & 15);                   // the token of this key chunk
    if (ku >= u0 && ku < u1) *kdst = kc;
    // value chunk: byte e of either half belongs to token (e % 4) + 4*hh + 16*(e / 4), hh = (chunk % 64) / 16
    const int hh = (chunk & 63) >> 4;
    uint32_t keep_lo = 0, keep_hi = 0;                                 // byte masks of tokens e = 0..3 and e = 4..7
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int ua = e + 4 * hh, ub = ua + 16;
        if (ua >= u0 && ua < u1) keep_lo |= 0xffu << (8 * e);
        if (ub >= u0 && ub < u1) keep_hi |= 0xffu << (8 * e);
    }
    const u32x4 old = *vdst;
    vc[0] = (vc[0] & keep_lo) | (old[0] & ~keep_lo);
    vc[1] = (vc[1] & keep_hi) | (old[1] & ~keep_hi);
    vc[2] = (vc[2] & keep_lo) | (old[2] & ~keep_lo);
    vc[3] = (vc[3] & keep_hi) | (old[3] & ~keep_hi);
    *vdst = vc;
}

// 4-bit codes: one CTA of 256 threads per (KV head, 32-token half block touched, sequence), for runs of any length (two
// tokens share bytes of the value block, so tokens are never written by independent waves).  Quantisation as above
// with 15 levels; key codes leave a lane as one whole operand word, value codes are staged as bytes in LDS and gathered
// into operand words (eight tokens per word).  A partly covered half block is merged with what the cache holds: key
// chunks belong to one token each, value words are merged nibble by nibble.
__global__ __launch_bounds__(256) void kv4_append_block_kernel(AttnCache kv, const uint16_t* __restrict__ Kn,
                                                               const uint16_t* __restrict__ Vn,
                                                               const int32_t* __restrict__ positions, int count)
{
    __shared__ __align__(16) uint32_t kwords[512];                     // the key half block in cache order
    __shared__ __align__(8) uint8_t vcodes[32][136];                   // value codes [token][dimension], padded rows
    const int h = blockIdx.x, b = blockIdx.z;
    const int pos = positions[b];
    long first = pos < 0 ? 0 : pos, last = (long)pos + count;
    if (last > kv.cap) last = kv.cap;
    if (first >= last) return;
    const int tb = (int)(first >> 5) + (int)blockIdx.y;
    const long t0 = first > (long)tb * 32 ? first : (long)tb * 32;
    const long t1 = last < (long)(tb + 1) * 32 ? last : (long)(tb + 1) * 32;
    if (t0 >= t1) return;                                              // CTA-uniform
    const int u0 = (int)(t0 - (long)tb * 32), u1 = (int)(t1 - (long)tb * 32);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15;                                         // dimensions 8*sub .. 8*sub + 7
    const size_t bh = (size_t)b * kv.heads + h;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int which = it >> 1;
        const int u = wave * 8 + (it & 1) * 4 + (lane >> 4);
        const bool live = u >= u0 && u < u1;
        const long t = (long)tb * 32 + u;
        float x[8];
        if (live) {
            const size_t src = (((size_t)b * count + (size_t)(t - pos)) * kv.heads + h) * kHeadDim + 8 * sub;
            const u32x4 raw = *reinterpret_cast<const u32x4*>((which ? Vn : Kn) + src);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                x[2 * k] = (float)__builtin_bit_cast(_Float16, (unsigned short)(raw[k] & 0xffffu));
                x[2 * k + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(raw[k] >> 16));
            }
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) x[k] = 0.f;
        }
        float mn = x[0], mx = x[0];
#pragma unroll
        for (int k = 1; k < 8; ++k) {
            mn = fminf(mn, x[k]);
            mx = fmaxf(mx, x[k]);
        }
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) {
            mn = fminf(mn, __shfl_xor(mn, m));
            mx = fmaxf(mx, __shfl_xor(mx, m));
        }
        _Float16 s16 = (_Float16)((mx - mn) / 15.0f);
        float sf = (float)s16;
        if (!(sf > 0.0f) || __builtin_isinf(sf)) {
            sf = 1.0f;
            s16 = (_Float16)1.0f;
        }
        const float zf = fminf(fmaxf(rintf(-mn / sf), 0.0f), 15.0f);
        uint32_t q[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) q[k] = (uint32_t)fminf(fmaxf(rintf(x[k] / sf) + zf, 0.0f), 15.0f);
        if (which == 0) {
            // dimensions 32*hh + 8*tt + e, e = 0..7: word tt of chunk (u/16)*64 + 16*hh + u%16; element e at nibble
            // e/2 + 4*(e % 2)
            const int chunk = (u >> 4) * 64 + 16 * (sub >> 2) + (u & 15);
            uint32_t w = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) w |= q[e] << (4 * ((e >> 1) + 4 * (e & 1)));
            kwords[chunk * 4 + (sub & 3)] = w;
        } else {
            u32x2 w;
            w[0] = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
            w[1] = q[4] | (q[5] << 8) | (q[6] << 16) | (q[7] << 24);
            *reinterpret_cast<u32x2*>(&vcodes[u][8 * sub]) = w;
        }
        if (live && sub == 0) {
            const _Float16 z16 = (_Float16)zf;
            kv.sz[(bh * kv.cap + t) * 2 + which] =
                (uint32_t)__builtin_bit_cast(unsigned short, s16) | ((uint32_t)__builtin_bit_cast(unsigned short, z16) << 16);
        }
    }
    __syncthreads();
    const size_t blk = (bh * (kv.cap / 32) + tb) * 2048;
    const bool whole = u0 == 0 && u1 == 32;
    const int chunk = threadIdx.x & 127;                               // 128 chunks of 16 bytes per half block
    if (threadIdx.x < 128) {
        const int ku = (chunk >> 6) * 16 + (chunk & 15);               // the token of this key chunk
        if (whole || (ku >= u0 && ku < u1))
            reinterpret_cast<u32x4*>(kv.k + blk)[chunk] = *reinterpret_cast<const u32x4*>(&kwords[chunk * 4]);
        return;
    }
    // value chunk (i/4)*64 + 16*hh + c: word i % 4 holds dimension 16*i + c of the tokens (e % 4) + 4*hh + 16*(e / 4)
    const int ii = chunk >> 6, hh = (chunk & 63) >> 4, c = chunk & 15;
    u32x4 vc = {0u, 0u, 0u, 0u};
    uint32_t keep = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int u = (e & 3) + 4 * hh + 16 * (e >> 2);
        const int sh = 4 * ((e >> 1) + 4 * (e & 1));
        if (u >= u0 && u < u1) keep |= 0xfu << sh;
#pragma unroll
        for (int w = 0; w < 4; ++w) vc[w] |= (uint32_t)vcodes[u][16 * (4 * ii + w) + c] << sh;
    }
    u32x4* vdst = reinterpret_cast<u32x4*>(kv.v + blk) + chunk;
    if (!whole) {
        const u32x4 old = *vdst;
#pragma unroll
        for (int w = 0; w < 4; ++w) vc[w] = (vc[w] & keep) | (old[w] & ~keep);
    }
    *vdst = vc;
}

// 4-bit codes, one new token per sequence (the append of a decoding step): one wave per (sequence, KV head); lane l owns
// dimensions l and l + 64.  Key codes: the eight lanes of an operand word OR their nibbles together and one of them
// stores the word.  Value codes: every dimension has its own word, shared with seven other tokens, so each lane replaces
// one nibble in each of its two words (no other wave of the launch touches this sequence and head).
__global__ __launch_bounds__(64) void kv4_append_token_kernel(AttnCache kv, const uint16_t* __restrict__ Kn,
                                                              const uint16_t* __restrict__ Vn,
                                                              const int32_t* __restrict__ positions)
{
    const int lane = threadIdx.x;
    const int h = blockIdx.x % kv.heads, b = blockIdx.x / kv.heads;
    const int t = positions[b];
    if (t < 0 || t >= kv.cap) return;                       // wave-uniform
    const size_t bh = (size_t)b * kv.heads + h;
    const size_t src = bh * kHeadDim;
    const int u = t & 31;
    const size_t blk = (bh * (kv.cap / 32) + (t >> 5)) * 512;      // in words
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        const uint16_t* x = (which ? Vn : Kn) + src;
        const float x0 = (float)__builtin_bit_cast(_Float16, x[lane]);
        const float x1 = (float)__builtin_bit_cast(_Float16, x[lane + 64]);
        float mn = fminf(x0, x1), mx = fmaxf(x0, x1);
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            mn = fminf(mn, __shfl_xor(mn, m));
            mx = fmaxf(mx, __shfl_xor(mx, m));
        }
        _Float16 s16 = (_Float16)((mx - mn) / 15.0f);
        float sf = (float)s16;
        if (!(sf > 0.0f) || __builtin_isinf(sf)) {
            sf = 1.0f;
            s16 = (_Float16)1.0f;
        }
        const float zf = fminf(fmaxf(rintf(-mn / sf), 0.0f), 15.0f);
        const uint32_t q0 = (uint32_t)fminf(fmaxf(rintf(x0 / sf) + zf, 0.0f), 15.0f);
        const uint32_t q1 = (uint32_t)fminf(fmaxf(rintf(x1 / sf) + zf, 0.0f), 15.0f);
        if (which == 0) {
            // dimension d = 32*hh + 8*tt + e: word ((u/16)*64 + 16*hh + u%16)*4 + tt, nibble e/2 + 4*(e % 2)
            const int e = lane & 7;
            const int sh = 4 * ((e >> 1) + 4 * (e & 1));
            uint32_t w0 = q0 << sh, w1 = q1 << sh;
#pragma unroll
            for (int m = 1; m < 8; m <<= 1) {
                w0 |= (uint32_t)__shfl_xor((int)w0, m);
                w1 |= (uint32_t)__shfl_xor((int)w1, m);
            }
            if (e == 0) {
                uint32_t* kw = reinterpret_cast<uint32_t*>(kv.k) + blk;
                const int d = lane;                          // and d + 64: two more 32-dimension groups up
                const int word = ((u >> 4) * 64 + 16 * (d >> 5) + (u & 15)) * 4 + ((d & 31) >> 3);
                kw[word] = w0;
                kw[word + 2 * 16 * 4] = w1;
            }
        } else {
            // dimension d = 16*i + c: word ((i/4)*64 + 16*hh + c)*4 + i%4, hh = (u%16)/4; this token is operand element
            // e = u%4 + 4*(u/16) of the word
            const int e = (u & 3) + 4 * (u >> 4), hh = (u & 15) >> 2;
            const int sh = 4 * ((e >> 1) + 4 * (e & 1));
            uint32_t* vw = reinterpret_cast<uint32_t*>(kv.v) + blk;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int d = lane + 64 * k, i = d >> 4;
                uint32_t* wp = vw + ((i >> 2) * 64 + 16 * hh + (d & 15)) * 4 + (i & 3);
                *wp = (*wp & ~(0xfu << sh)) | ((k ? q1 : q0) << sh);
            }
        }
        if (lane == 0) {
            const _Float16 z16 = (_Float16)zf;
            kv.sz[(bh * kv.cap + t) * 2 + which] =
                (uint32_t)__builtin_bit_cast(unsigned short, s16) | ((uint32_t)__builtin_bit_cast(unsigned short, z16) << 16);
        }
    }
}

// ------------------------------------------------------------------------------------------------ decode attention
// The codes of a block travel in registers (they are the in-flight memory of the pipeline: two blocks ahead).  The 64
// scale/zero words of a block would cost as many registers per lane as its 8 KiB of codes, so they go through LDS
// instead: one direct-to-LDS load per block and wave (lane l fetches word l) into a slot private to the wave.
struct BlockRegs {
    u32x4 k[2][2];      // two 16-token tiles: 32 key bytes of the lane's token (dimensions 32h .. 32h+31)
    u32x4 v[4];         // 64 value bytes: eight 16-row tiles x the lane's eight tokens
};

// Descriptors of one (sequence, head): its K blocks, V blocks and scale/zero words, each cut off after the last block
// of the context.  A load past that end returns zeros without touching memory, which lets the pipeline issue its loads
// unconditionally (the surplus ones at the end of a wave's range cost nothing).
struct HeadRsrc {
    __amdgpu_buffer_rsrc_t k, v, sz;
};

// A block is 4096 bytes of key codes and as many of value codes: 32 tokens of 8-bit codes, or 64 tokens of 4-bit codes
// (two 32-token halves of 2048 bytes each, r.k[half][tile], r.v[2*half + i/4]); the load instructions are the same.
template <int BITS>
__device__ __forceinline__ void load_block(BlockRegs& r, uint32_t* sz_slot, const HeadRsrc& rs, int blk, int lane)
{
    // (the host pass of the compiler only needs the kernel's signature; it cannot express the LDS pointer)
#if defined(__HIP_DEVICE_COMPILE__)
    if constexpr (BITS == 8) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs.sz, (__attribute__((address_space(3))) void*)sz_slot, 4,
                                                 lane * 4 + blk * 256, 0, 0, 0);
    } else {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs.sz, (__attribute__((address_space(3))) void*)sz_slot, 4,
                                                 lane * 4 + blk * 512, 0, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs.sz, (__attribute__((address_space(3))) void*)(sz_slot + 64), 4,
                                                 lane * 4 + blk * 512 + 256, 0, 0, 0);
    }
#else
    (void)sz_slot;
#endif
    // every load instruction of the wave reads 1 KiB of consecutive bytes: the blocks are stored in operand order.
    // The block offset sits in the per-lane offset, which the descriptor's range check covers.
    const int off = lane * 16 + blk * 4096;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        r.k[j][0] = __builtin_amdgcn_raw_buffer_load_b128(rs.k, off + (j * 2 + 0) * 1024, 0, kNonTemporal);
        r.k[j][1] = __builtin_amdgcn_raw_buffer_load_b128(rs.k, off + (j * 2 + 1) * 1024, 0, kNonTemporal);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) r.v[i] = __builtin_amdgcn_raw_buffer_load_b128(rs.v, off + i * 1024, 0, kNonTemporal);
}

// Running state of one wave (per query head m = lane % 16; m_run is equal in the four lanes that share an m, l_run and
// corr are per-lane partial sums over the lane's own tokens).
struct SoftmaxState {
    float m_run, l_run, corr;
};

// Thirty-two tokens (a whole 8-bit block, or half `sb` of a 4-bit block) starting at token t0.  qsum = sum of the
// query's 128 values, qbias = sum of the conversion bias of each code position times the query value it meets.
template <int BITS, bool MASKED>
__device__ __forceinline__ void process_tokens(const BlockRegs& r, int sb, const uint32_t* sz_slot, const f16x8 (&qf)[4],
                                               float qsum, const f32x4& neg_qbias, const Magic& mg, int t0, int len, int lane,
                                               SoftmaxState& st, f32x4 (&acc)[8])
{
    const int h = lane >> 4;
    const int rem = len - t0 - 4 * h;          // slot (j, rr) of this lane is a live token iff 16*j + rr < rem
    // S^T for the two 16-token tiles: rows = tokens, columns = query heads
    float s[2][4];
    uint32_t vw[2][4];                         // (scale, zero-point) of the slot's value row; 0 for a dead token
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        // the accumulator starts at minus the bias term: sum_d (bias_d + q_d) Q_d - sum_d bias_d Q_d = sum_d q_d Q_d
        f32x4 d;
        if constexpr (BITS == 8) {
            d = mfma16x16x32(biased8_w8(r.k[j][0].x, r.k[j][0].y), qf[0], neg_qbias);
            d = mfma16x16x32(biased8_w8(r.k[j][0].z, r.k[j][0].w), qf[1], d);
            d = mfma16x16x32(biased8_w8(r.k[j][1].x, r.k[j][1].y), qf[2], d);
            d = mfma16x16x32(biased8_w8(r.k[j][1].z, r.k[j][1].w), qf[3], d);
        } else {
            const u32x4 w = r.k[sb][j];
            d = mfma16x16x32(biased8(w.x, mg), qf[0], neg_qbias);
            d = mfma16x16x32(biased8(w.y, mg), qf[1], d);
            d = mfma16x16x32(biased8(w.z, mg), qf[2], d);
            d = mfma16x16x32(biased8(w.w, mg), qf[3], d);
        }
        // (K pair, V pair) of the lane's four tokens 16j + 4h .. +3: eight consecutive words of the slot
        const u32x4 p0 = *(const u32x4*)(sz_slot + 32 * j + 8 * h);
        const u32x4 p1 = *(const u32x4*)(sz_slot + 32 * j + 8 * h + 4);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const bool live = !MASKED || 16 * j + rr < rem;
            const f16x2 kp = as_f16x2(rr < 2 ? p0[2 * rr] : p1[2 * (rr - 2)]);
            // a dead token contributes nothing, whatever its pair holds: scale 0 and zero-point 0 for its values
            vw[j][rr] = live ? (rr < 2 ? p0[2 * rr + 1] : p1[2 * (rr - 2) + 1]) : 0u;
            // sum_d q_d Q_d  -  z sum_d Q_d  =  sum_d (q_d - z) Q_d ; times the token's scale.  Both steps are written
            // as fused multiply-adds so that the fp16 pair enters the instruction directly (no separate conversion;
            // an addend of +0 keeps the second one from being folded into a plain multiply).
            const float t = __builtin_fmaf(-(float)kp.y, qsum, d[rr]);
            const float sc = __builtin_fmaf((float)kp.x, t, 0.0f);
            s[j][rr] = live ? sc : kNegBig;
        }
    }
    // online softmax in base 2 (the query carries scale * log2(e))
    float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])), fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
    mx = xor_max(xor_max(mx, 16), 32);
    const float m_new = fmaxf(st.m_run, mx);
    const float alpha = fast_exp2(st.m_run - m_new);
    st.m_run = m_new;
    float psum = 0.f;
    f16x8 pb;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const float p = fast_exp2(s[j][rr] - m_new);    // 0 for masked tokens
            psum += p;
            // probability times the value scale of that token
            pb[4 * j + rr] = (_Float16)__builtin_fmaf((float)as_f16x2(vw[j][rr]).x, p, 0.0f);
        }
    // The correction term must be built from the very fp16 values the matrix core multiplies: the bias is about a
    // thousand times the payload, so one fp16 ulp of disagreement on a single probability shifts a whole output row by
    // several per cent.  Left to itself the compiler rounds p * vs once for the operand (fused multiply-and-convert)
    // and once more, through fp32, for the sum below; the two differ when the fp32 product lands on an fp16 tie.
    // Pinning the packed operand makes it the only copy.
    {
        u32x4 bits = __builtin_bit_cast(u32x4, pb);
        asm volatile("" : "+v"(bits.x), "+v"(bits.y), "+v"(bits.z), "+v"(bits.w));
        pb = __builtin_bit_cast(f16x8, bits);
    }
    // sum over the lane's tokens of (bias + z) * p': the value code of slot (j, rr) is the k-value 4j + rr of the
    // second product and carries the bias 1024 - or 64 at positions 2, 3, 6, 7 of a 4-bit word
    float sum_hi = 0.f, sum_lo = 0.f, zsum = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const float pv = (float)pb[4 * j + rr];
            if (BITS == 8 || rr < 2) sum_hi = __builtin_fmaf(pv, 1.0f, sum_hi);
            else sum_lo = __builtin_fmaf(pv, 1.0f, sum_lo);
            zsum = __builtin_fmaf((float)as_f16x2(vw[j][rr]).y, pv, zsum);
        }
    const float csum = __builtin_fmaf(1024.0f, sum_hi, __builtin_fmaf(64.0f, sum_lo, zsum));
    st.l_run = st.l_run * alpha + psum;
    st.corr = st.corr * alpha + csum;
    // the running maximum seldom moves after the first blocks: rescale only when some query head needs it
    if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] *= alpha;
    }
    // O^T += V^T P'^T : rows = dimensions (eight 16-row tiles), k = the 32 tokens of the block
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        f16x8 a;
        if constexpr (BITS == 8) {
            const u32x4 w = r.v[i >> 1];
            a = (i & 1) ? biased8_w8(w.z, w.w) : biased8_w8(w.x, w.y);
        } else {
            a = biased8(r.v[2 * sb + (i >> 2)][i & 3], mg);
        }
        acc[i] = mfma16x16x32(a, pb, acc[i]);
    }
}

// The same 32 tokens when at most eight query heads share the KV head: the query operand then carries every head twice
// (column c and c + 8 both hold head c % 8), so both score tiles come out with all 16 columns live, and a lane keeps
// tile c / 8 only - four scores instead of eight, half the softmax arithmetic.  The probabilities of the other tile's
// tokens reach the lane through one exchange with lane c ^ 8 before the second product; running sums are per lane over
// its own tokens and meet at the end (xor 8, 16, 32).
__device__ __forceinline__ uint32_t swap_half_rows(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128, 0xf, 0xf, true);      // row_ror:8 = lane c <-> c ^ 8
}

template <int BITS, bool MASKED>
__device__ __forceinline__ void process_tokens_packed(const BlockRegs& r, int sb, const uint32_t* sz_slot,
                                                      const f16x8 (&qf)[4], float qsum, const f32x4& neg_qbias,
                                                      const Magic& mg, int t0, int len, int lane, SoftmaxState& st,
                                                      f32x4 (&acc)[8])
{
    const int h = lane >> 4, jl = (lane >> 3) & 1;           // jl: the 16-token tile this lane keeps
    const int rem = len - t0 - 4 * h - 16 * jl;              // slot rr of this lane is a live token iff rr < rem
    f32x4 d[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if constexpr (BITS == 8) {
            d[j] = mfma16x16x32(biased8_w8(r.k[j][0].x, r.k[j][0].y), qf[0], neg_qbias);
            d[j] = mfma16x16x32(biased8_w8(r.k[j][0].z, r.k[j][0].w), qf[1], d[j]);
            d[j] = mfma16x16x32(biased8_w8(r.k[j][1].x, r.k[j][1].y), qf[2], d[j]);
            d[j] = mfma16x16x32(biased8_w8(r.k[j][1].z, r.k[j][1].w), qf[3], d[j]);
        } else {
            const u32x4 w = r.k[sb][j];
            d[j] = mfma16x16x32(biased8(w.x, mg), qf[0], neg_qbias);
            d[j] = mfma16x16x32(biased8(w.y, mg), qf[1], d[j]);
            d[j] = mfma16x16x32(biased8(w.z, mg), qf[2], d[j]);
            d[j] = mfma16x16x32(biased8(w.w, mg), qf[3], d[j]);
        }
    }
    // (K pair, V pair) of the lane's four tokens 16*jl + 4h .. +3
    const u32x4 p0 = *(const u32x4*)(sz_slot + 32 * jl + 8 * h);
    const u32x4 p1 = *(const u32x4*)(sz_slot + 32 * jl + 8 * h + 4);
    float s[4];
    uint32_t vw[4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const bool live = !MASKED || rr < rem;
        const f16x2 kp = as_f16x2(rr < 2 ? p0[2 * rr] : p1[2 * (rr - 2)]);
        vw[rr] = live ? (rr < 2 ? p0[2 * rr + 1] : p1[2 * (rr - 2) + 1]) : 0u;
        const float dm = jl ? d[1][rr] : d[0][rr];
        const float t = __builtin_fmaf(-(float)kp.y, qsum, dm);
        const float sc = __builtin_fmaf((float)kp.x, t, 0.0f);
        s[rr] = live ? sc : kNegBig;
    }
    float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
    mx = fmaxf(mx, __builtin_bit_cast(float, swap_half_rows(__builtin_bit_cast(uint32_t, mx))));
    mx = xor_max(xor_max(mx, 16), 32);
    const float m_new = fmaxf(st.m_run, mx);
    const float alpha = fast_exp2(st.m_run - m_new);
    st.m_run = m_new;
    float psum = 0.f;
    _Float16 own[4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const float p = fast_exp2(s[rr] - m_new);            // 0 for masked tokens
        psum += p;
        own[rr] = (_Float16)__builtin_fmaf((float)as_f16x2(vw[rr]).x, p, 0.0f);
    }
    // the lane's four probabilities as two operand words, pinned (the correction below must see the very bits the
    // matrix core multiplies), then the other tile's four from lane c ^ 8
    uint32_t o0 = (uint32_t)__builtin_bit_cast(uint16_t, own[0]) | ((uint32_t)__builtin_bit_cast(uint16_t, own[1]) << 16);
    uint32_t o1 = (uint32_t)__builtin_bit_cast(uint16_t, own[2]) | ((uint32_t)__builtin_bit_cast(uint16_t, own[3]) << 16);
    asm volatile("" : "+v"(o0), "+v"(o1));
    const uint32_t x0 = swap_half_rows(o0), x1 = swap_half_rows(o1);
    u32x4 pbits;
    pbits.x = jl ? x0 : o0;                                  // k-values 0..3: tile 0, 4..7: tile 1
    pbits.y = jl ? x1 : o1;
    pbits.z = jl ? o0 : x0;
    pbits.w = jl ? o1 : x1;
    const f16x8 pb = __builtin_bit_cast(f16x8, pbits);
    float sum_hi = 0.f, sum_lo = 0.f, zsum = 0.f;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const float pv = (float)(rr < 2 ? (rr == 0 ? as_f16x2(o0).x : as_f16x2(o0).y) : (rr == 2 ? as_f16x2(o1).x : as_f16x2(o1).y));
        if (BITS == 8 || rr < 2) sum_hi = __builtin_fmaf(pv, 1.0f, sum_hi);
        else sum_lo = __builtin_fmaf(pv, 1.0f, sum_lo);
        zsum = __builtin_fmaf((float)as_f16x2(vw[rr]).y, pv, zsum);
    }
    const float csum = __builtin_fmaf(1024.0f, sum_hi, __builtin_fmaf(64.0f, sum_lo, zsum));
    st.l_run = st.l_run * alpha + psum;
    st.corr = st.corr * alpha + csum;
    if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] *= alpha;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        f16x8 a;
        if constexpr (BITS == 8) {
            const u32x4 w = r.v[i >> 1];
            a = (i & 1) ? biased8_w8(w.z, w.w) : biased8_w8(w.x, w.y);
        } else {
            a = biased8(r.v[2 * sb + (i >> 2)][i & 3], mg);
        }
        acc[i] = mfma16x16x32(a, pb, acc[i]);
    }
}

// len: tokens the lane's query column attends over (the same in every lane at a decoding step; at prefill every column
// has its own causal limit); len_all: the largest of them, wave-uniform.
template <int BITS, bool PACK>
__device__ __forceinline__ void process_block(const BlockRegs& r, const uint32_t* sz_slot, const f16x8 (&qf)[4],
                                              float qsum, const f32x4& neg_qbias, const Magic& mg, int blk, int len, int len_all,
                                              int lane, SoftmaxState& st, f32x4 (&acc)[8])
{
    constexpr int TOK = 256 / BITS;
    const int t0 = blk * TOK;
    // the first 32 tokens always hold a live one; the second half of a 4-bit block may lie wholly behind the context
    // (wave-uniform).  (A second, unmasked copy of the code for blocks inside the context costs more registers than the
    // kernel has: it spills.)
    if constexpr (PACK) {
        process_tokens_packed<BITS, true>(r, 0, sz_slot, qf, qsum, neg_qbias, mg, t0, len, lane, st, acc);
        if constexpr (BITS == 4) {
            if (t0 + 32 < len_all)
                process_tokens_packed<4, true>(r, 1, sz_slot + 64, qf, qsum, neg_qbias, mg, t0 + 32, len, lane, st, acc);
        }
    } else {
        process_tokens<BITS, true>(r, 0, sz_slot, qf, qsum, neg_qbias, mg, t0, len, lane, st, acc);
        if constexpr (BITS == 4) {
            if (t0 + 32 < len_all) process_tokens<4, true>(r, 1, sz_slot + 64, qf, qsum, neg_qbias, mg, t0 + 32, len, lane, st, acc);
        }
    }
}

// Four consecutive dimensions d0 .. d0+3 of query head `head` of sequence b, rounded to fp16.
__device__ __forceinline__ void store_out4(uint16_t* O, int b, int q_heads, int head, int d0, const float (&o)[4])
{
    u32x2 out;
    out.x = (uint32_t)f32_to_f16_bits(o[0]) | ((uint32_t)f32_to_f16_bits(o[1]) << 16);
    out.y = (uint32_t)f32_to_f16_bits(o[2]) | ((uint32_t)f32_to_f16_bits(o[3]) << 16);
    *(u32x2*)(O + ((size_t)b * q_heads + head) * kHeadDim + d0) = out;
}

// grid (kv heads, batch, splits); 256 threads.  Partial layout per (b, h, split): m[16], l[16], out[128][16] floats.
constexpr int kPartialFloats = 32 + kHeadDim * 16;
constexpr int kMergeHere = 8;            // splits the last-arriving CTA merges itself (all their loads in flight at once)

// PREFILL: the same kernel over a chunk of prompt tokens (paper Sec. 3.3: one attention pipeline for both phases).  The 16
// query columns of a CTA are then 16 / G consecutive tokens x the G query heads of the KV head (column c = token c / G,
// head c % G), blockIdx.z counts such token groups instead of context splits, `lens` holds the cache position of every
// sequence's first query token, and each column attends causally over the cache up to its own token: the length that
// masks scores becomes a per-lane value, everything else - loading pipeline, head alignment, biased codes - is shared.
template <int BITS, bool PACK, bool PREFILL = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_decode_kernel(AttnCache kv, const uint16_t* __restrict__ Q,
                                                          const int32_t* __restrict__ lens, uint16_t* __restrict__ O,
                                                          int q_heads, float scale_log2e, int blocks_per_split,
                                                          int splits, int merge_here, int head0, int gw,
                                                          const int32_t* __restrict__ counts = nullptr, int count = 1)
{
    static_assert(!(PREFILL && PACK), "prompt chunks use all 16 query columns");
    __shared__ float sm_ml[4][2][16];
    __shared__ float sm_out[4][8][4][64];
    // scale/zero words of the blocks in flight: [wave][64 words]; one array per ring slot so that the compiler can tell
    // which direct-to-LDS load a read depends on
    constexpr int TOK = 256 / BITS;                 // tokens per block
    __shared__ __attribute__((aligned(16))) uint32_t sz_ring0[4][2 * TOK];
    __shared__ __attribute__((aligned(16))) uint32_t sz_ring1[4][2 * TOK];
    __shared__ __attribute__((aligned(16))) uint32_t sz_ring2[4][2 * TOK];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, h = lane >> 4;
    const int hk = blockIdx.x, b = blockIdx.y, split = blockIdx.z;
    // A launch covers query heads head0 .. head0 + gw - 1 (gw <= 16) of every KV head's group of q_heads / kv.heads:
    // larger groups take one launch per sixteen heads.  G is the width the columns are laid out for, hq the first query
    // head of this CTA.
    const int G = gw;
    const int hq = hk * (q_heads / kv.heads) + head0;
    const size_t bh = (size_t)b * kv.heads + hk;
    int len, len_all;                                        // this lane's column; the CTA's longest column
    int tok = 0, head = c;                                   // query token (within the chunk) and head (within G) of column c
    bool real;
    if constexpr (PREFILL) {
        const int tpg = 16 / G;                              // tokens per CTA
        const int tq = c / G;
        head = c - tq * G;
        tok = split * tpg + tq;
        const int cnt = counts ? min(max(counts[b], 0), count) : count;
        const int first = split * tpg;                       // first token of this group
        if (first >= cnt) return;                            // (uniform) nothing to do for this sequence
        const int pos0 = lens[b];
        const int pos = pos0 + tok;
        real = tq < tpg && tok < cnt && pos >= 0 && pos < kv.cap;
        len = real ? pos + 1 : 0;
        len_all = min(max(pos0 + min(cnt, first + tpg), 0), kv.cap);
        if (!real) tok = first;                              // an address that exists
    } else {
        // the splits cover blocks_per_split * splits blocks (the host's max_len): a longer sequence is cut there
        len = min(min(max(lens[b], 0), kv.cap), blocks_per_split * splits * TOK);
        len_all = len;
        real = (PACK ? (c & 7) : c) < G;
    }
    const int nblk = (len_all + TOK - 1) / TOK;
    const int blk0 = PREFILL ? 0 : split * blocks_per_split;
    const int blk1 = PREFILL ? nblk : min(nblk, blk0 + blocks_per_split);

    // Order of the prologue: the query's raw loads, then at once the first two blocks of the KV memory loading pipeline,
    // and only then the arithmetic on the query, which so runs under the blocks' latency (loads return in order, so the
    // query must be requested first).
    const int qc = PREFILL ? head : (PACK ? (c & 7) : c);    // the query head of operand column c
    f16x8 qraw[4];
    {
        const size_t qrow = PREFILL ? (size_t)b * count + tok : (size_t)b;
        const uint16_t* qp = Q + (qrow * q_heads + (size_t)hq + (real ? qc : 0)) * kHeadDim + 32 * h;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) qraw[tt] = *(const f16x8*)(qp + 8 * tt);
    }

    // KV memory loading pipeline: the next two blocks of this wave are in flight while the current one is multiplied
    // (three register sets and three LDS slots, rotated by unrolling; with one block ahead the waves spent half their
    // time waiting for memory).  Loads are unconditional - past the end of the wave's range they point behind the
    // descriptors' ranges and return zeros without memory traffic - so that the loop body is straight-line code with a
    // known number of loads in flight.
    HeadRsrc rs;
    rs.k = make_rsrc(kv.k + bh * (kv.cap / TOK) * 4096, (uint32_t)nblk * 4096u);
    rs.v = make_rsrc(kv.v + bh * (kv.cap / TOK) * 4096, (uint32_t)nblk * 4096u);
    rs.sz = make_rsrc(kv.sz + bh * kv.cap * 2, (uint32_t)nblk * (8u * TOK));
    uint32_t* const z0 = sz_ring0[wave];
    uint32_t* const z1 = sz_ring1[wave];
    uint32_t* const z2 = sz_ring2[wave];
    BlockRegs r0, r1, r2;
    int blk = blk0 + wave;
    load_block<BITS>(r0, z0, rs, blk < blk1 ? blk : nblk, lane);
    load_block<BITS>(r1, z1, rs, blk + 4 < blk1 ? blk + 4 : nblk, lane);

    // Query operand (adaptive head alignment): column m = c, k-values of step tt = dimensions 32h + 8tt .. +7, the
    // order in which the lane's key bytes arrive; scaled once by scale * log2(e).
    f16x8 qf[4];
    float qsum = 0.f, qbias = 0.f;
    const Magic mg = make_magic();
    {
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                qf[tt][e] = real ? (_Float16)((float)qraw[tt][e] * scale_log2e) : (_Float16)0.0f;
            }
            // the sums below must see the very fp16 values the matrix core multiplies (one rounding, one copy)
            u32x4 bits = __builtin_bit_cast(u32x4, qf[tt]);
            asm volatile("" : "+v"(bits.x), "+v"(bits.y), "+v"(bits.z), "+v"(bits.w));
            qf[tt] = __builtin_bit_cast(f16x8, bits);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                qsum += (float)qf[tt][e];
                qbias += ((e & 2) ? 64.0f : 1024.0f) * (float)qf[tt][e];     // bias of a 4-bit code at operand position e
            }
        }
        qsum = xor_add(xor_add(qsum, 16), 32);
        qbias = BITS == 8 ? 1024.0f * qsum : xor_add(xor_add(qbias, 16), 32);   // every 8-bit code carries the bias 1024
    }
    const f32x4 neg_qbias = {-qbias, -qbias, -qbias, -qbias};

    // (at prefill a wave may meet blocks in which some column has no live token yet: the running maximum then starts
    // above the mask value, so that masked scores still turn into zero probabilities)
    SoftmaxState st{PREFILL ? kMaskFloor : kNegBig, 0.f, 0.f};
    f32x4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (blk < blk1) {
        while (true) {
            load_block<BITS>(r2, z2, rs, blk + 8 < blk1 ? blk + 8 : nblk, lane);
            process_block<BITS, PACK>(r0, z0, qf, qsum, neg_qbias, mg, blk, len, len_all, lane, st, acc);
            blk += 4;
            if (blk >= blk1) break;
            load_block<BITS>(r0, z0, rs, blk + 8 < blk1 ? blk + 8 : nblk, lane);
            process_block<BITS, PACK>(r1, z1, qf, qsum, neg_qbias, mg, blk, len, len_all, lane, st, acc);
            blk += 4;
            if (blk >= blk1) break;
            load_block<BITS>(r1, z1, rs, blk + 8 < blk1 ? blk + 8 : nblk, lane);
            process_block<BITS, PACK>(r2, z2, qf, qsum, neg_qbias, mg, blk, len, len_all, lane, st, acc);
            blk += 4;
            if (blk >= blk1) break;
        }
    }

    // the four lanes of a query head add their partial sums; the waves meet in LDS
    float l_w = xor_add(xor_add(st.l_run, 16), 32);
    float corr_w = xor_add(xor_add(st.corr, 16), 32);
    if constexpr (PACK) {                                    // the two tiles' lanes of a query head
        l_w = xor_add(l_w, 8);
        corr_w = xor_add(corr_w, 8);
    }
    if (h == 0) {
        sm_ml[wave][0][c] = st.m_run;
        sm_ml[wave][1][c] = l_w;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) sm_out[wave][i][rr][lane] = acc[i][rr] - corr_w;   // bias and zero-point leave here
    __syncthreads();
    // thread (wave w, lane) finalises row tiles 2w and 2w+1 of its column
    float M = kNegBig;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, sm_ml[w][0][c]);
    float L = 0.f, f[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        f[w] = exp2f(sm_ml[w][0][c] - M);
        L += sm_ml[w][1][c] * f[w];
    }
    if (splits == 1) {
        const float inv = L > 0.f ? 1.0f / L : 0.f;
#pragma unroll
        for (int ii = 0; ii < 2; ++ii) {
            const int i = 2 * wave + ii;
            float o[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                float v = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) v += sm_out[w][i][rr][lane] * f[w];
                o[rr] = v * inv;
            }
            if constexpr (PREFILL) {
                if (real) store_out4(O, b * count + tok, q_heads, hq + head, 16 * i + 4 * h, o);
            } else {
                if (c < G) store_out4(O, b, q_heads, hq + c, 16 * i + 4 * h, o);
            }
        }
        return;
    }
    if constexpr (PREFILL) return;                           // prompt chunks are never split along the context

    // Split context: this CTA's maximum, denominator and unnormalised rows go to the workspace - values of row tile i,
    // register rr at float 32 + (4*i + rr)*64 + lane, so that writer and reader touch whole 256-byte lines - as
    // write-through stores that CTAs on other XCDs can read back without a device-wide fence.
    float* part = kv.partial + (((size_t)bh * splits) + split) * kPartialFloats;
    if (wave == 0 && h == 0) {
        st_partial(part + c, M);
        st_partial(part + 16 + c, L);
    }
#pragma unroll
    for (int ii = 0; ii < 2; ++ii) {
        const int i = 2 * wave + ii;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) v += sm_out[w][i][rr][lane] * f[w];
            st_partial(part + 32 + (4 * i + rr) * 64 + lane, v);
        }
    }
    if (!merge_here) return;                                  // many splits: the merge kernel follows

    // Few splits: the CTA that arrives last at this (sequence, head)'s counter merges them, in split order.
    __shared__ uint32_t s_last;
    wait_stores_done();
    __syncthreads();
    if (tid == 0) {
        const uint32_t prev = atomicAdd(&kv.counters[bh], 1u);
        s_last = (prev == (uint32_t)splits - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    // at most kMergeHere splits come here: all their loads are issued before the first use (the loop is unrolled and a
    // missing split reads split 0 again with a factor of zero)
    const float* base = kv.partial + (size_t)bh * splits * kPartialFloats;
    float ms[kMergeHere], ls[kMergeHere], vals[kMergeHere][2][4];
#pragma unroll
    for (int sp = 0; sp < kMergeHere; ++sp) {
        const float* ps = base + (size_t)(sp < splits ? sp : 0) * kPartialFloats;
        ms[sp] = ld_partial(ps + c);
        ls[sp] = ld_partial(ps + 16 + c);
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) vals[sp][ii][rr] = ld_partial(ps + 32 + (4 * (2 * wave + ii) + rr) * 64 + lane);
    }
    float Mg = kNegBig;
#pragma unroll
    for (int sp = 0; sp < kMergeHere; ++sp) Mg = fmaxf(Mg, sp < splits ? ms[sp] : kNegBig);
    float Lg = 0.f;
    float o[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int sp = 0; sp < kMergeHere; ++sp) {
        const float fs = sp < splits ? exp2f(ms[sp] - Mg) : 0.f;
        Lg += ls[sp] * fs;
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) o[ii][rr] += vals[sp][ii][rr] * fs;
    }
    const float invg = Lg > 0.f ? 1.0f / Lg : 0.f;
#pragma unroll
    for (int ii = 0; ii < 2; ++ii) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) o[ii][rr] *= invg;
        if (c < G) store_out4(O, b, q_heads, hq + c, 16 * (2 * wave + ii) + 4 * h, o[ii]);
    }
    if (tid == 0) __hip_atomic_store(&kv.counters[bh], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Merge of the context splits: grid (kv heads, batch, 8 chunks of 16 dimensions), 256 threads = 16 query heads x 16.
// Phase 1 (every CTA, all threads): running maximum and denominator over the splits, four splits per thread, reduced
// through LDS; the per-split factors exp2(m_s - M) / L stay in LDS.  Phase 2: thread (m, dd) sums dimension
// 16*chunk + dd of query head m over the splits.
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnCache kv, uint16_t* __restrict__ O, int q_heads, int splits,
                                                         int head0, int gw)
{
    __shared__ float red[16][16];
    __shared__ float fac[64][16];                  // splits <= 64
    const int hk = blockIdx.x, b = blockIdx.y, chunk = blockIdx.z;
    const int G = gw;
    const int hq = hk * (q_heads / kv.heads) + head0;
    const size_t bh = (size_t)b * kv.heads + hk;
    const float* base = kv.partial + (size_t)bh * splits * kPartialFloats;
    const int m = threadIdx.x & 15, g = threadIdx.x >> 4;
    float ms[4], ls[4];
    float mx = kNegBig;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int s = g + 16 * i;
        ms[i] = s < splits ? ld_partial(base + (size_t)s * kPartialFloats + m) : kNegBig;
        ls[i] = s < splits ? ld_partial(base + (size_t)s * kPartialFloats + 16 + m) : 0.f;
        mx = fmaxf(mx, ms[i]);
    }
    red[g][m] = mx;
    __syncthreads();
    float M = kNegBig;
#pragma unroll
    for (int i = 0; i < 16; ++i) M = fmaxf(M, red[i][m]);
    __syncthreads();
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float f = exp2f(ms[i] - M);
        part += ls[i] * f;
        if (g + 16 * i < splits) fac[g + 16 * i][m] = f;
    }
    red[g][m] = part;
    __syncthreads();
    float L = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) L += red[i][m];
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    if (m >= G) return;
    const int d = 16 * chunk + g;
    // dimension d = 16*chunk + 4*hh + rr of query head m sits at float 32 + (4*chunk + rr)*64 + 16*hh + m
    const int at = 32 + (4 * chunk + (g & 3)) * 64 + 16 * (g >> 2) + m;
    float v = 0.f;
#pragma unroll 8
    for (int s = 0; s < splits; ++s) v += ld_partial(base + (size_t)s * kPartialFloats + at) * fac[s][m];
    O[((size_t)b * q_heads + (size_t)hq + m) * kHeadDim + d] = f32_to_f16_bits(v * inv);
}

}  // namespace

hipError_t launch_kv_append(const AttnCache& kv, const uint16_t* Kn, const uint16_t* Vn, const int32_t* positions,
                            int count, hipStream_t stream)
{
    const long waves = (long)kv.batch * count * kv.heads;
    if (waves <= 0 || waves > 0x7fffffffL) return hipErrorInvalidValue;
    if (kv.bits == 4) {
        if (kv.heads > 65535 || kv.batch > 65535 || ((((uintptr_t)Kn | (uintptr_t)Vn) & 15))) return hipErrorInvalidValue;
        if (count == 1) {
            hipLaunchKernelGGL(kv4_append_token_kernel, dim3((unsigned)waves), dim3(64), 0, stream, kv, Kn, Vn, positions);
            return hipGetLastError();
        }
        const unsigned blocks = (unsigned)((count + 31) / 32 + 1);
        hipLaunchKernelGGL(kv4_append_block_kernel, dim3(kv.heads, blocks, kv.batch), dim3(256), 0, stream, kv, Kn, Vn,
                           positions, count);
        return hipGetLastError();
    }
    if (count >= 16 && kv.heads <= 65535 && kv.batch <= 65535 && !(((uintptr_t)Kn | (uintptr_t)Vn) & 15)) {
        // blocks a run of `count` tokens can touch: one more than it fills when it starts inside a block
        const unsigned blocks = (unsigned)((count + 31) / 32 + 1);
        hipLaunchKernelGGL(kv_append_block_kernel, dim3(kv.heads, blocks, kv.batch), dim3(256), 0, stream, kv, Kn, Vn,
                           positions, count);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)waves), dim3(64), 0, stream, kv, Kn, Vn, positions, count);
    return hipGetLastError();
}

hipError_t launch_attn_decode(const AttnCache& kv, const uint16_t* Q, const int32_t* lens, uint16_t* O, int q_heads,
                              float scale, int max_len, int num_cu, hipStream_t stream)
{
    const int tok = 256 / kv.bits;                                   // tokens per 4 KiB block
    const int nblk = (max_len + tok - 1) / tok;
    // enough CTAs for two per CU - what is resident at once with two waves per SIMD; a third would run in a second,
    // half-empty round (measured: 28.5 instead of 31.8 us at batch 8 x 8192) - at least four blocks per wave and split,
    // and no more partial results than the cache's workspace holds
    int splits = (2 * num_cu + kv.batch * kv.heads - 1) / (kv.batch * kv.heads);
    // (short contexts: up to eight splits of at least two blocks per wave - a 2048-token context is cut in four or
    // eight instead of two or four pieces, which shortens each CTA's serial chain more than the merge costs)
    const int few = nblk / 8 < 8 ? nblk / 8 : 8;
    const int by_work = nblk / 16 > few ? nblk / 16 : (few > 0 ? few : 1);
    if (splits > by_work) splits = by_work;
    if (splits > kv.max_splits) splits = kv.max_splits;
    // four splits merge without a second launch: worth more than a fuller second half-round as soon as four splits
    // give every CU a CTA (batch 8 x 8192: 26.4 instead of 29.3 us; at batch 1 the GPU would be left mostly empty)
    if (splits > 4 && kv.batch * kv.heads * 4 >= num_cu) splits = 4;
    if (splits < 1) splits = 1;
    const int bps = (nblk + splits - 1) / splits;
    splits = (nblk + bps - 1) / bps > 0 ? (nblk + bps - 1) / bps : 1;
    if (kv.heads > 65535 || kv.batch > 65535) return hipErrorInvalidValue;
    const float scale_log2e = scale * 1.4426950408889634f;
    // up to eight splits are merged by the CTA that finishes last, with all its loads in flight at once (two splits:
    // 27.6 instead of 29.7 us at batch 32 x 2048; a loop over the splits, one load chain after the other, cost 11.5
    // instead of 8.5 us at batch 1 x 2048); more splits go to the merge kernel, which spreads a (sequence, head) over
    // eight CTAs
    const int merge_here = splits > 1 && splits <= kMergeHere;
    const dim3 grid(kv.heads, kv.batch, splits);
    // one pass per sixteen query heads of a KV head's group (the sixteen columns of an MFMA tile); the passes follow
    // each other on the stream and share the cache's split workspace
    const int group = q_heads / kv.heads;
    for (int head0 = 0; head0 < group; head0 += 16) {
        const int gw = group - head0 < 16 ? group - head0 : 16;
        const bool pack = gw <= 8;                           // both score tiles share one softmax pass
        if (kv.bits == 8 && pack)
            hipLaunchKernelGGL((attn_decode_kernel<8, true>), grid, dim3(256), 0, stream, kv, Q, lens, O, q_heads, scale_log2e,
                               bps, splits, merge_here, head0, gw);
        else if (kv.bits == 8)
            hipLaunchKernelGGL((attn_decode_kernel<8, false>), grid, dim3(256), 0, stream, kv, Q, lens, O, q_heads, scale_log2e,
                               bps, splits, merge_here, head0, gw);
        else if (pack)
            hipLaunchKernelGGL((attn_decode_kernel<4, true>), grid, dim3(256), 0, stream, kv, Q, lens, O, q_heads, scale_log2e,
                               bps, splits, merge_here, head0, gw);
        else
            hipLaunchKernelGGL((attn_decode_kernel<4, false>), grid, dim3(256), 0, stream, kv, Q, lens, O, q_heads, scale_log2e,
                               bps, splits, merge_here, head0, gw);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (splits > 1 && !merge_here) {
            hipLaunchKernelGGL(attn_merge_kernel, dim3(kv.heads, kv.batch, 8), dim3(256), 0, stream, kv, O, q_heads, splits, head0, gw);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t launch_attn_prefill(const AttnCache& kv, const uint16_t* Q, const int32_t* positions, const int32_t* counts,
                               int count, uint16_t* O, int q_heads, float scale, hipStream_t stream)
{
    const int group = q_heads / kv.heads;
    const float scale_log2e = scale * 1.4426950408889634f;
    for (int head0 = 0; head0 < group; head0 += 16) {        // one pass per sixteen query heads of a group, as at decode
        const int gw = group - head0 < 16 ? group - head0 : 16;
        const int tpg = 16 / gw;                             // query tokens per CTA
        const int groups = (count + tpg - 1) / tpg;
        if (kv.heads > 65535 || kv.batch > 65535 || groups > 65535 || groups < 1) return hipErrorInvalidValue;
        const dim3 grid(kv.heads, kv.batch, groups);
        if (kv.bits == 8)
            hipLaunchKernelGGL((attn_decode_kernel<8, false, true>), grid, dim3(256), 0, stream, kv, Q, positions, O, q_heads,
                               scale_log2e, 0, 1, 0, head0, gw, counts, count);
        else
            hipLaunchKernelGGL((attn_decode_kernel<4, false, true>), grid, dim3(256), 0, stream, kv, Q, positions, O, q_heads,
                               scale_log2e, 0, 1, 0, head0, gw, counts, count);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace tmw4
