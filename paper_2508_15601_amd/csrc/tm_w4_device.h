// Device-side building blocks shared by the GEMM kernels: vector types, the packed-layout index helpers,
// the int4 -> fp16 conversion and the gfx950 matrix-core wrapper.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace tmw4 {

// compile-time loop: f(std::integral_constant<int, I>{}) for I = B .. E-1
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kUnitK = 128;       // rows of one packed unit
constexpr int kUnitN = 16;        // columns of one packed unit
constexpr int kUnitWords = 256;   // u32 words per unit (64 lanes x 4)
constexpr int kMaxCounters = 16384;                       // split-K arrival counters at the head of a workspace
constexpr size_t kCounterBytes = kMaxCounters * sizeof(uint32_t);

// Problem description handed to every GEMM kernel.
struct GemmParams {
    const uint16_t* X;        // fp16 [M][K]
    const u32x4* W;           // packed weights, one u32x4 per (unit, lane)
    const uint32_t* SZ;       // packed scale|zero<<16 words
    uint16_t* Y;              // fp16 [M][N]
    float* partial;           // split-K partial sums (fp32), in the kernels' accumulator order: [split][strip] slots
                              // of slot_floats in the decode kernels, [split][tile] whole tiles in the CTA-tile kernels
    uint32_t* counters;       // split-K arrival counters, zero between launches
    int M, K, N;
    int KU;                   // K / 128
    int NT;                   // N / 16
    int G;                    // K / group
    int split;                // split-K factor (>= 1)
    int ku_per_split;         // k-units per split (ceil)
    int tiles_m, tiles_n;     // tile kernel only
    int strips;               // skinny kernel only: the NT column tiles are dealt into this many strips
    int strip_base, strip_rem;  // NT / strips and NT % strips: strip s owns strip_base tiles (+1 if s < strip_rem),
                                // starting at tile s * strip_base + min(s, strip_rem)
    // Fused epilogue (all optional; 0 / null = plain Y = X * dequant(W)).
    const uint16_t* bias;     // fp16 [N] in the caller's column order, added to the sums
    const uint16_t* residual; // fp16 [M][ldy], added last
    int act;                  // 1: columns are interleaved (gate, up) pairs and Y[m][n/2] = silu(gate) * up
    int ldy;                  // row stride of Y and residual: N, or N/2 with act
    int epi;                  // 0: none of the three is set (the stores take the plain path on one test)
    int mp_log;               // stream kernels: log2 of M rounded up to a power of two (rows of an X region in LDS)
    int red_off;              // stream kernels: LDS byte offset of the reduction tiles; 0 = they reuse the X regions
    int slot_floats;          // decode kernels: floats of partial sums per (K slice, strip): 64 * M rounded up to 16 * widest strip
};

// Grouped (mixture-of-experts) launch: rows [offsets[e], offsets[e+1]) of X and Y belong to expert e.
struct GroupedParams {
    const uint16_t* X;
    uint16_t* Y;
    const uint64_t* table;      // per expert: address of the packed weights, address of the scale/zero words
    const int32_t* offsets;     // [experts + 1], ascending
    int K, N, KU, NT, G, strips, total_rows, experts;
    int strip_base, strip_rem;  // as in GemmParams
    int tiles_n, mtiles;        // tile kernels: column tiles, and the upper bound of row tiles over all experts
    int act;                    // 1: gate/up experts, Y[r][n/2] = silu(gate) * up, row stride N/2
    int lds_bytes;              // one-shot decode kernels: dynamic LDS of the launch
};

// Quantised KV cache of the attention kernels: 8-bit codes, one scale/zero pair per token and head.
struct AttnCache {
    uint8_t* k;          // [batch*heads][cap/32] blocks of 32 tokens (4096 or 2048 bytes) in K*Q^T operand order
    uint8_t* v;          // [batch*heads][cap/32] blocks of 32 tokens in V^T*P^T operand order
    uint32_t* sz;        // [batch*heads][cap][2] scale | zero << 16: K pair, V pair
    float* partial;      // split workspace: [batch*heads][max_splits] x (m[16], l[16], out[32 registers][64 lanes])
    uint32_t* counters;  // [batch*heads] arrival counters of the split merge, zero between launches
    int batch, heads, cap, max_splits;
    int bits;            // 8 or 4 bits per code; cap is a multiple of 256 / bits
};

// Raw buffer descriptor over `bytes` bytes at p (gfx9 layout: 32-bit data format, no swizzle, no stride).  Loads
// through it take a per-lane 32-bit byte offset plus a scalar one; lanes whose offset falls outside return zero
// without touching memory.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
constexpr int kNonTemporalLoad = 2;      // cache-policy bit of a buffer load: streamed once, do not keep

__device__ __forceinline__ f16x2 as_f16x2(uint32_t u) { return __builtin_bit_cast(f16x2, u); }

// Per-(column, K-group) constants of the conversion: the scale in both halves, and the two exact offsets that
// remove the conversion bias together with the zero-point.
struct GroupConst {
    f16x2 s2;        // (s, s)
    f16x2 off1024;   // (-(1024 + z), -(1024 + z))
    f16x2 off64;     // (-(64 + z), -(64 + z))
};

__device__ __forceinline__ GroupConst make_group_const(uint32_t sz)
{
    f16x2 p = as_f16x2(sz);
    _Float16 s = p.x, z = p.y;
    GroupConst g;
    g.s2 = f16x2{s, s};
    _Float16 a = (_Float16)(-1024.0f) - z;   // exact: 1024 + z is an fp16 integer (z <= 15, or <= 255 for 8-bit codes)
    _Float16 b = (_Float16)(-64.0f) - z;
    g.off1024 = f16x2{a, a};
    g.off64 = f16x2{b, b};
    return g;
}

// The two exponent patterns of the conversion, held in vector registers: gfx950 encodes at most one scalar or
// literal operand per VALU instruction, so "(w & mask) | magic" only fuses into one v_and_or_b32 when the magic
// comes from a VGPR.  Call once per kernel, outside the loops.
struct Magic {
    uint32_t m1024;  // 0x6400 in both halves: fp16 1024
    uint32_t m64;    // 0x5400 in both halves: fp16 64
};
__device__ __forceinline__ Magic make_magic()
{
    Magic m{0x64006400u, 0x54005400u};
    asm("" : "+v"(m.m1024));
    asm("" : "+v"(m.m64));
    return m;
}

// Integer-to-float by bit manipulation (paper Sec. 3.1 step (iii), Sec. 4.3 "I2F conversion and FMA").
// A nibble q OR-ed into the mantissa of 0x6400 is the fp16 number 1024 + q; a nibble sitting four bits higher
// OR-ed into 0x5400 is 64 + q.  Adding the matching offset gives q - z exactly; one multiply applies the scale
// (a single rounding per weight).  The packed word stores weight e at nibble 4*(e&1) + (e>>1), so the four
// masked words below are already the fp16 pairs (e0,e1), (e2,e3), (e4,e5), (e6,e7) of a matrix-core operand.
// 13 vector instructions per 8 weights: 1 shift, 4 and-or, 4 packed adds, 4 packed multiplies.
__device__ __forceinline__ f16x8 dequant8(uint32_t w, const GroupConst& g, const Magic& mg)
{
    uint32_t a0 = (w & 0x000F000Fu) | mg.m1024;
    uint32_t a1 = (w & 0x00F000F0u) | mg.m64;
    uint32_t w8 = w >> 8;
    uint32_t a2 = (w8 & 0x000F000Fu) | mg.m1024;
    uint32_t a3 = (w8 & 0x00F000F0u) | mg.m64;
    f16x2 r0 = (as_f16x2(a0) + g.off1024) * g.s2;
    f16x2 r1 = (as_f16x2(a1) + g.off64) * g.s2;
    f16x2 r2 = (as_f16x2(a2) + g.off1024) * g.s2;
    f16x2 r3 = (as_f16x2(a3) + g.off64) * g.s2;
    return f16x8{r0.x, r0.y, r1.x, r1.y, r2.x, r2.y, r3.x, r3.y};
}

// The bit-manipulation half of the conversion alone: the eight fp16 values (1024 + q) / (64 + q), alternating in
// pairs (e0,e1: +1024; e2,e3: +64; e4,e5: +1024; e6,e7: +64), still carrying their conversion bias.
__device__ __forceinline__ f16x8 biased8(uint32_t w, const Magic& mg)
{
    u32x4 r;
    r.x = (w & 0x000F000Fu) | mg.m1024;
    r.y = (w & 0x00F000F0u) | mg.m64;
    uint32_t w8 = w >> 8;
    r.z = (w8 & 0x000F000Fu) | mg.m1024;
    r.w = (w8 & 0x00F000F0u) | mg.m64;
    return __builtin_bit_cast(f16x8, r);
}

// The operand that cancels that bias together with the zero-point inside the matrix core: multiplying the same
// activations by -(bias + z) and accumulating into the same fp32 tile leaves sum_k x_k * (q_k - z) exactly
// (every product is exact in fp32; only the accumulation order rounds).
__device__ __forceinline__ f16x8 bias_cancel8(_Float16 z)
{
    _Float16 a = (_Float16)(-1024.0f) - z;   // exact: 1024 + z <= 1039 is an fp16 integer
    _Float16 b = (_Float16)(-64.0f) - z;
    return f16x8{a, a, b, b, a, a, b, b};
}

// 8-bit codes.  A byte b placed under the exponent byte 0x64 is the fp16 number 1024 + b (b fills the low eight
// mantissa bits), so one byte permute (v_perm_b32 against the constant 0x64646464) turns two codes into two fp16
// values: four permutes per eight weights.  w0 holds the codes e0..e3 in bytes 0..3, w1 holds e4..e7.
__device__ __forceinline__ f16x8 biased8_w8(uint32_t w0, uint32_t w1)
{
    const uint32_t hi = 0x64646464u;               // selector bytes 4..7 pick from here, 0..3 from the weight word
    u32x4 r;
    r.x = __builtin_amdgcn_perm(hi, w0, 0x04010400u);
    r.y = __builtin_amdgcn_perm(hi, w0, 0x04030402u);
    r.z = __builtin_amdgcn_perm(hi, w1, 0x04010400u);
    r.w = __builtin_amdgcn_perm(hi, w1, 0x04030402u);
    return __builtin_bit_cast(f16x8, r);
}

// -(1024 + z) in all eight places: exact, because 1024 + z <= 1279 is an fp16 integer.
__device__ __forceinline__ f16x8 bias_cancel8_w8(_Float16 z)
{
    _Float16 a = (_Float16)(-1024.0f) - z;
    return f16x8{a, a, a, a, a, a, a, a};
}

// (1024 + q) - (1024 + z) = q - z exactly (|q - z| <= 255), then one rounded multiply by the scale:
// 12 vector instructions per 8 weights.
__device__ __forceinline__ f16x8 dequant8_w8(uint32_t w0, uint32_t w1, const GroupConst& g)
{
    const uint32_t hi = 0x64646464u;
    f16x2 r0 = (as_f16x2(__builtin_amdgcn_perm(hi, w0, 0x04010400u)) + g.off1024) * g.s2;
    f16x2 r1 = (as_f16x2(__builtin_amdgcn_perm(hi, w0, 0x04030402u)) + g.off1024) * g.s2;
    f16x2 r2 = (as_f16x2(__builtin_amdgcn_perm(hi, w1, 0x04010400u)) + g.off1024) * g.s2;
    f16x2 r3 = (as_f16x2(__builtin_amdgcn_perm(hi, w1, 0x04030402u)) + g.off1024) * g.s2;
    return f16x8{r0.x, r0.y, r1.x, r1.y, r2.x, r2.y, r3.x, r3.y};
}

// Weight formats of the decode kernels' BITS parameter: 4-bit and 8-bit integer codes, and FP8 (OCP E4M3) codes,
// which share the 8-bit packed layout and need neither a conversion bias nor a zero-point.
constexpr int kFmtInt4 = 4, kFmtInt8 = 8, kFmtFp8 = 18;

// Eight FP8 E4M3 codes -> eight fp16 values (every E4M3 value is an fp16 value, so the conversion is exact):
// gfx950 converts two codes per instruction (v_cvt_scalef32_pk_f16_fp8 with scale 1).
__device__ __forceinline__ f16x8 cvt8_fp8(uint32_t w0, uint32_t w1)
{
    f16x2 r0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w0, 1.0f, false);
    f16x2 r1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w0, 1.0f, true);
    f16x2 r2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w1, 1.0f, false);
    f16x2 r3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w1, 1.0f, true);
    return f16x8{r0.x, r0.y, r1.x, r1.y, r2.x, r2.y, r3.x, r3.y};
}

// D = A(16x32) * B(32x16) + C on the matrix cores.  Lane l supplies row l%16 of A and column l%16 of B, each
// with the eight k-values 8*(l/16) .. 8*(l/16)+7; it receives D[4*(l/16) + r][l%16] in c[r].
__device__ __forceinline__ f32x4 mfma16x16x32(f16x8 a, f16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Split-K partial sums cross CTAs (and therefore XCDs, whose L2 caches are not coherent with each other).
// They are written and read with device-scope relaxed atomics, which the hardware performs as write-through
// stores and cache-bypassing loads; a device-scope fence would instead write back and invalidate the whole L2 on
// every call, which costs far more than the kernel itself.  Ordering against the arrival counter comes from
// wait_stores_done() (every wave drains its own stores) followed by a CTA barrier before the counter is bumped.
__device__ __forceinline__ void st_partial(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_partial2(float* p, float a, float b)
{
    uint64_t u = (uint64_t)__builtin_bit_cast(uint32_t, a) | ((uint64_t)__builtin_bit_cast(uint32_t, b) << 32);
    __hip_atomic_store((uint64_t*)p, u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_partial(const float* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ld_partial2(const float* p, float& a, float& b)
{
    uint64_t u = __hip_atomic_load((const uint64_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    a = __builtin_bit_cast(float, (uint32_t)u);
    b = __builtin_bit_cast(float, (uint32_t)(u >> 32));
}
// Sum over the K splits of one pair of neighbouring outputs, in split order (a fixed order: the result does not depend
// on which CTA arrives last).  The loads of four splits are issued before the first add: each of them is a round trip
// past the caches, and a loop of load-then-add over a split count known only at run time pays those trips one after the
// other.  first = address of the pair in split 0, stride = floats between consecutive splits.
__device__ __forceinline__ void sum_partials2(const float* first, size_t stride, int split, float& v0, float& v1)
{
    v0 = 0.f;
    v1 = 0.f;
    for (int s0 = 0; s0 < split; s0 += 4) {
        float a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) ld_partial2(first + (size_t)min(s0 + u, split - 1) * stride, a[u], b[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (s0 + u < split) {                  // uniform over the launch
                v0 += a[u];
                v1 += b[u];
            }
        }
    }
}

__device__ __forceinline__ void wait_stores_done()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // this wave's write-through stores have completed
}

__device__ __forceinline__ uint16_t f32_to_f16_bits(float v)
{
    _Float16 h = (_Float16)v;          // v_cvt_f16_f32, round-to-nearest-even
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }

// silu(g) * u in fp32; exp2 of a large positive argument gives +inf and the quotient 0, as it should.
__device__ __forceinline__ float silu_mul(float g, float u)
{
    return g / (1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g)) * u;
}

// The one place where sums become outputs.  v0, v1 are the fp32 sums of columns n, n + 1 (n even) of row m.  All
// branches are uniform over the launch.  With act the packed weight's columns are interleaved - kernel column 2j is
// gate column j, 2j + 1 is up column j of the caller's [gate | up] matrix - so every thread that holds a pair holds a
// matching one, and the pair collapses into output column n / 2.
__device__ __forceinline__ void store_pair(const GemmParams& p, int m, int n, float v0, float v1)
{
    if (p.epi == 0) {
        *(uint32_t*)(p.Y + (size_t)m * p.N + n) = (uint32_t)f32_to_f16_bits(v0) | ((uint32_t)f32_to_f16_bits(v1) << 16);
        return;
    }
    if (p.act) {
        if (p.bias) {
            v0 += f16_bits_to_f32(p.bias[n >> 1]);
            v1 += f16_bits_to_f32(p.bias[(p.N >> 1) + (n >> 1)]);
        }
        float y = silu_mul(v0, v1);
        const size_t at = (size_t)m * p.ldy + (n >> 1);
        if (p.residual) y += f16_bits_to_f32(p.residual[at]);
        p.Y[at] = f32_to_f16_bits(y);
        return;
    }
    const size_t at = (size_t)m * p.ldy + n;
    if (p.bias) {
        const uint32_t b = *(const uint32_t*)(p.bias + n);
        v0 += f16_bits_to_f32((uint16_t)b);
        v1 += f16_bits_to_f32((uint16_t)(b >> 16));
    }
    if (p.residual) {
        const uint32_t r = *(const uint32_t*)(p.residual + at);
        v0 += f16_bits_to_f32((uint16_t)r);
        v1 += f16_bits_to_f32((uint16_t)(r >> 16));
    }
    *(uint32_t*)(p.Y + at) = (uint32_t)f32_to_f16_bits(v0) | ((uint32_t)f32_to_f16_bits(v1) << 16);
}

// Four consecutive columns n .. n + 3 (n a multiple of 4) of row m.
__device__ __forceinline__ void store_quad(const GemmParams& p, int m, int n, float v0, float v1, float v2, float v3)
{
    if (p.epi == 0) {
        u32x2 o;
        o.x = (uint32_t)f32_to_f16_bits(v0) | ((uint32_t)f32_to_f16_bits(v1) << 16);
        o.y = (uint32_t)f32_to_f16_bits(v2) | ((uint32_t)f32_to_f16_bits(v3) << 16);
        *(u32x2*)(p.Y + (size_t)m * p.N + n) = o;
        return;
    }
    if (p.act) {
        if (p.bias) {
            const uint32_t bg = *(const uint32_t*)(p.bias + (n >> 1));
            const uint32_t bu = *(const uint32_t*)(p.bias + (p.N >> 1) + (n >> 1));
            v0 += f16_bits_to_f32((uint16_t)bg);
            v1 += f16_bits_to_f32((uint16_t)bu);
            v2 += f16_bits_to_f32((uint16_t)(bg >> 16));
            v3 += f16_bits_to_f32((uint16_t)(bu >> 16));
        }
        float y0 = silu_mul(v0, v1), y1 = silu_mul(v2, v3);
        const size_t at = (size_t)m * p.ldy + (n >> 1);
        if (p.residual) {
            const uint32_t r = *(const uint32_t*)(p.residual + at);
            y0 += f16_bits_to_f32((uint16_t)r);
            y1 += f16_bits_to_f32((uint16_t)(r >> 16));
        }
        *(uint32_t*)(p.Y + at) = (uint32_t)f32_to_f16_bits(y0) | ((uint32_t)f32_to_f16_bits(y1) << 16);
        return;
    }
    const size_t at = (size_t)m * p.ldy + n;
    if (p.bias) {
        const u32x2 b = *(const u32x2*)(p.bias + n);
        v0 += f16_bits_to_f32((uint16_t)b.x);
        v1 += f16_bits_to_f32((uint16_t)(b.x >> 16));
        v2 += f16_bits_to_f32((uint16_t)b.y);
        v3 += f16_bits_to_f32((uint16_t)(b.y >> 16));
    }
    if (p.residual) {
        const u32x2 r = *(const u32x2*)(p.residual + at);
        v0 += f16_bits_to_f32((uint16_t)r.x);
        v1 += f16_bits_to_f32((uint16_t)(r.x >> 16));
        v2 += f16_bits_to_f32((uint16_t)r.y);
        v3 += f16_bits_to_f32((uint16_t)(r.y >> 16));
    }
    u32x2 o;
    o.x = (uint32_t)f32_to_f16_bits(v0) | ((uint32_t)f32_to_f16_bits(v1) << 16);
    o.y = (uint32_t)f32_to_f16_bits(v2) | ((uint32_t)f32_to_f16_bits(v3) << 16);
    *(u32x2*)(p.Y + at) = o;
}

}  // namespace tmw4
