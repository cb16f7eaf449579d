// Fused dequantise-and-multiply for M > 32: CTA tiles with the activations staged through LDS.
//
// Online stage of the GEMM pipeline (paper Sec. 3.1 steps (i)-(iv)) with the software-pipelined main loop of
// Sec. 4.3: while the matrix cores work on one 32-deep K step, the vector ALUs convert the weight fragments of
// the next step (I2F, then zero-point and scale: one exact subtract and one rounded multiply per weight) between
// the MFMAs, and the memory units fetch the next stage of X and of packed weights.
//
// Differences from the paper's design: packed weights go from HBM/L2 straight into registers in matrix-core operand
// order (no shared-memory stage, no matrix-load instruction, hence nothing to swizzle); only X passes through LDS,
// loaded there directly from global memory, in a row-major layout whose 16-byte chunks are XOR-swizzled within a
// row so that the 128-bit fragment reads are bank-conflict-free.
// The four waves of a CTA split the tile along N only, so every weight fragment is converted exactly once per CTA
// and feeds TM MFMAs.  The weight fragment is the A operand, so a lane ends up with four consecutive columns of
// one output row and stores them as one 8-byte word.  CTAs are numbered so that the CTAs resident on one XCD
// (one L2) cover a compact block of output tiles.
//
// A pipeline stage is KW MFMA steps (32*KW rows of K) deep.  Tall tiles use 64-deep stages (their MFMA time per
// stage already exceeds the memory latency); short tiles use 128- or 256-deep stages, because with few rows the
// MFMAs of a 64-deep stage finish long before the next stage can arrive from L2/HBM.
#pragma once
#include <type_traits>

#include "tm_w4_host.h"

namespace tmw4 {

namespace {

constexpr int kPanelN = 8;                 // output tiles per panel row (XCD-local rasterisation)


// CTA tile = (TM*16) rows x (NW*TN*16) columns; wave w of NW owns columns [w*TN*16, (w+1)*TN*16) and all rows.
// KG > 1 puts KG such sets of NW waves into one CTA: set kg multiplies the kg-th slice (32*KW rows of K) of every
// stage, and the KG partial tiles meet in LDS at the end.  That doubles or quadruples the waves per SIMD, which
// hide each other's LDS and memory latency, without adding CTAs (every CTA re-reads its rows of X) and without
// partial sums in global memory.
// GPU = K-groups per 128-row unit, KW = MFMA steps per pipeline stage (2, 4 or 8).
// An X fragment read from LDS (1 KiB per wave) feeds TN MFMAs.
// PD = prefetch distance of the packed weights in stages (the memory pipeline depth of paper Sec. 4.3): the weight
// loads of stage s+PD are issued while stage s is multiplied.  Register sets rotate by compile-time phase (the loop
// is unrolled PD*(PD+1) times), never by copies, because a copy would wait for the load it renames.  PD = 2 wherever
// the registers allow (tiles up to 128 rows): one stage of MFMAs is shorter than an HBM round trip.  X runs one
// stage ahead, through the second LDS buffer.
//
// tile_body is one CTA's work on output tile (tile_m, tile_n) and K split sk of one GEMM.
// FMT is the weight format (kFmtInt4, kFmtInt8, kFmtFp8): 8-bit codes take two words per MFMA step and their packed
// units hold two steps (64 rows) instead of four.
template <int TM, int TN, int NW, int GPU, int KW, int PD, int KG, int FMT = kFmtInt4>
__device__ __forceinline__ void tile_body(const GemmParams& p, const int tile_m, const int tile_n, const int sk)
{
    constexpr int WPS = FMT == kFmtInt4 ? 1 : 2;           // packed words per lane and MFMA step
    constexpr int SPU = FMT == kFmtInt4 ? 4 : 2;           // MFMA steps per packed unit
    constexpr int NT_ = NW * KG * 64;                      // threads per CTA
    constexpr int BM = TM * 16, BN = NW * TN * 16;
    constexpr int BK = 32 * KW;                            // halves of K per stage and wave set
    constexpr int BKS = BK * KG;                           // halves of K per stage
    constexpr int CPR = BKS / 8;                           // 16-byte chunks per X row and stage
    constexpr int CH = (BM * CPR + NT_ - 1) / NT_;         // chunks per thread and stage
    constexpr int SG = (KW * GPU) / 4 > 0 ? (KW * GPU) / 4 : 1;   // K-groups touched by one stage
    constexpr int UW = KW > SPU ? KW / SPU : 1;            // packed units touched by one stage
    constexpr int WPU = (KW > SPU ? SPU : KW) * WPS;       // words of a unit used by one stage
    // two X buffers, separate objects so that the compiler can tell a write into one from a read of the other;
    // after the K loop the first also carries the wave sets' partial tiles
    constexpr size_t kXsBytes = (size_t)BM * BKS * sizeof(uint16_t);
    // one wave set's partial tile; the sets' tiles meet pairwise (see the end of the K loop), as many at a time as fit
    constexpr size_t kSetTileBytes = (size_t)NW * TM * TN * 64 * sizeof(f32x4);
    // (a tile of more than 64 KiB is handed over in row parts, so that the buffer stays at 64 KiB)
    constexpr size_t kRedCap = 64 * 1024;
    constexpr int kRedParts = kSetTileBytes > kRedCap ? (int)(kSetTileBytes / kRedCap) : 1;
    static_assert(kSetTileBytes <= kRedCap || (kSetTileBytes % kRedCap == 0 && TM % kRedParts == 0), "set tile parts");
    constexpr size_t kRedBytes = KG > 1 ? kSetTileBytes / kRedParts : 0;
    __shared__ __attribute__((aligned(16))) unsigned char smem0[kXsBytes > kRedBytes ? kXsBytes : kRedBytes];
    __shared__ __attribute__((aligned(16))) unsigned char smem1[kXsBytes];
    __shared__ uint32_t s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave = wave_id % NW, kg = wave_id / NW;       // column slot and K slice of this wave
    const int c = lane & 15, h = lane >> 4;
    const Magic mg = make_magic();

    const int m0 = tile_m * BM;
    const int nt_end = min(p.NT, (tile_n + 1) * (BN / 16));    // 16-column tiles of this CTA end here
    const int nt0 = (tile_n * BN) / 16 + wave * TN;        // first 16-column tile of this wave
    // stages of this CTA's K range (the host makes ku_per_split a multiple of UW when KW > 4)
    const int st0 = (sk * p.ku_per_split * SPU) / (KW * KG);
    const int st1 = (min(p.KU, (sk + 1) * p.ku_per_split) * SPU) / (KW * KG);

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // All global loads are buffer loads: a descriptor in scalar registers, a 32-bit per-lane byte offset that
    // never changes, and a scalar offset that advances along K.  That leaves no vector address arithmetic in the
    // K loop and no address register a later load could overwrite; reads past a descriptor's size return zero.
    //
    // X goes from global memory straight into LDS (`buffer_load ... lds`): no staging registers, no LDS store
    // instructions.  Such a load writes the 64 lanes' 16-byte chunks to consecutive LDS addresses, so the LDS image
    // of a stage is simply chunk position idx = i*NT_ + tid <-> (row idx / CPR, slot idx % CPR), unpadded; what
    // varies is which chunk of the row a lane fetches: slot s of row r holds chunk s ^ (r & kSwz), kSwz = 15 (7 for
    // 64-deep stages, whose rows have only eight chunks).  With that XOR the 128-bit fragment reads of rows
    // c = 0..15 fall into different 16-byte bank groups (SQ_LDS_BANK_CONFLICT reads zero), which padding achieved
    // in the register-staged version of this kernel.
    constexpr int kSwz = CPR >= 16 ? 15 : 7;
    const __amdgpu_buffer_rsrc_t x_rsrc = make_rsrc(p.X, (uint32_t)p.M * (uint32_t)p.K * 2u);
    uint32_t x_off[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int idx = i * NT_ + tid;
        const int row = min(m0 + idx / CPR, p.M - 1);                  // rows past M repeat the last row
        const int kc = (idx % CPR) ^ ((idx / CPR) & kSwz);
        x_off[i] = (uint32_t)row * (uint32_t)p.K * 2u + (uint32_t)kc * 16u;
    }
    auto load_x = [&](int buf, int st) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int first = i * NT_ + wave_id * 64;      // wave-uniform: the wave's 64 chunks are contiguous in LDS
            // (the host pass of the compiler only needs the kernel's signature; it cannot express the LDS pointer)
#if defined(__HIP_DEVICE_COMPILE__)
            if ((BM * CPR) % NT_ == 0 || first < BM * CPR)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    x_rsrc, (__attribute__((address_space(3))) void*)((buf ? smem1 : smem0) + (size_t)first * 16),
                    16, x_off[i], st * (BKS * 2), 0, 0);
#else
            (void)first;
            (void)buf;
            (void)st;
            (void)x_rsrc;
#endif
        }
    };
    // Fragment of MFMA step tt, row tile i: lane (c, h) wants chunk 4q + h of row 16i + c, q = kg*KW + tt; it sits
    // at byte (16i + c) * BKS*2 + (q ^ f) * 64 + (h ^ (c & 3)) * 16 with f = the swizzle bits of c above its low
    // two.  (q + 4) ^ f = (q ^ f) + 4, so one lane base per tt mod 4 serves all steps and everything else is an
    // immediate offset.
    constexpr int NXB = KW < 4 ? KW : 4;
    uint32_t xd_base[NXB];
#pragma unroll
    for (int t = 0; t < NXB; ++t) {
        const uint32_t f = ((uint32_t)c & kSwz) >> 2;
        const uint32_t q = (uint32_t)kg * KW + t;
        xd_base[t] = (uint32_t)c * (BKS * 2) + (q ^ f) * 64u + (((uint32_t)h ^ ((uint32_t)c & 3u)) * 16u) - t * 64u;
    }
    auto x_frag = [&](int buf, int tt, int i) -> const f16x8* {
        return (const f16x8*)((buf ? smem1 : smem0) + xd_base[tt % NXB] + tt * 64 + i * (16 * BKS * 2));
    };

    // packed weights of one stage: words [st*KW, st*KW + KW) of the lane's K sequence, for each n-tile
    // packed weights and scale/zero words of stage r live in register set r % (PD + 1)
    const uint32_t w_lane = (uint32_t)lane * 16u, sz_lane = (uint32_t)c * 4u;
    uint32_t wset[PD + 1][TN][KW * WPS];
    uint32_t sset[PD + 1][TN][SG];
    // one descriptor per 16-column tile of this wave: its K/128 packed units, and its K/group scale/zero rows.
    // A tile past the edge of the strip gets empty descriptors: its loads return zero without touching memory
    // (its results are never stored), which keeps the K loop free of branches.
    __amdgpu_buffer_rsrc_t w_rsrc[TN], s_rsrc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const bool live = nt0 + j < nt_end;                // wave-uniform
        const int nt = min(nt0 + j, nt_end - 1);
        w_rsrc[j] = make_rsrc((const char*)p.W + (size_t)nt * p.KU * 1024, live ? (uint32_t)p.KU * 1024u : 0u);
        s_rsrc[j] = make_rsrc((const char*)p.SZ + (size_t)nt * p.G * 64, live ? (uint32_t)p.G * 64u : 0u);
    }
    auto load_w = [&](uint32_t (&w)[TN][KW * WPS], uint32_t (&s)[TN][SG], int stage) {
        const int st = stage * KG + kg;                    // this wave set's slice of the stage
        // packed unit of the slice, and the first of the lane's four words in it (non-zero only for KW == 2)
        const int wbyte = ((st * KW) / SPU) * 1024 + ((st * KW) % SPU) * 4 * WPS;
        const int grp0 = (st * KW * GPU) / 4;              // first K-group of the slice
        // Issue order = order of first use one or two stages later (the load counter retires in order): the
        // scale/zero words, then the weights.  (The X loads of a stage are issued before this call.)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < SG; ++g)
                s[j][g] = __builtin_amdgcn_raw_buffer_load_b32(s_rsrc[j], sz_lane, (grp0 + g) * 64, 0);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int u = 0; u < UW; ++u) {
                if constexpr (WPU == 2) {
                    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(w_rsrc[j], w_lane + u * 1024, wbyte, 0);
                    w[j][0] = v.x;
                    w[j][1] = v.y;
                } else {
                    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc[j], w_lane + u * 1024, wbyte, 0);
                    w[j][4 * u + 0] = v.x;
                    w[j][4 * u + 1] = v.y;
                    w[j][4 * u + 2] = v.z;
                    w[j][4 * u + 3] = v.w;
                }
            }
        }
    };

    // One 32-deep MFMA step over the whole CTA-row tile, software-pipelined as in paper Sec. 4.3: while the
    // matrix cores consume the converted fragments `cur`, the vector ALU converts the fragments of the NEXT step
    // into `nxt`, a few at a time between groups of MFMAs, and LDS reads run one row-pair ahead of their use.
    // The scheduling barriers keep the compiler from hoisting all LDS reads and conversions to the top, which
    // would both starve the matrix cores and blow the register budget.
    // The fp16 operand of MFMA step tt from the stage's packed words (paper Sec. 3.1 step (iii)).
    auto convert = [&](const uint32_t (&wj)[KW * WPS], int tt, uint32_t szw) -> f16x8 {
        const GroupConst gc = make_group_const(szw);
        if constexpr (FMT == kFmtInt4) {
            return dequant8(wj[tt], gc, mg);
        } else if constexpr (FMT == kFmtInt8) {
            return dequant8_w8(wj[2 * tt], wj[2 * tt + 1], gc);
        } else {
            const f16x8 v = cvt8_fp8(wj[2 * tt], wj[2 * tt + 1]);
            const _Float16 sc = gc.s2.x;
            return v * f16x8{sc, sc, sc, sc, sc, sc, sc, sc};
        }
    };
    constexpr int PAIRS = TM / 2;
    auto step = [&](int buf, int tt, const f16x8 (&cur)[TN], f16x8 (&nxt)[TN], const uint32_t (&wsrc)[TN][KW * WPS],
                    const uint32_t (&ssrc)[TN][SG], int tt_next) {
        f16x8 x0 = *x_frag(buf, tt, 0);
        f16x8 x1 = *x_frag(buf, tt, 1);
#pragma unroll
        for (int ip = 0; ip < PAIRS; ++ip) {
            f16x8 n0 = x0, n1 = x1;
            if (ip + 1 < PAIRS) {
                n0 = *x_frag(buf, tt, 2 * ip + 2);
                n1 = *x_frag(buf, tt, 2 * ip + 3);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j)
                if (j * PAIRS / TN == ip)          // spread the TN conversions over the row pairs
                    nxt[j] = convert(wsrc[j], tt_next, ssrc[j][(tt_next * GPU) / 4 % SG]);
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[2 * ip][j] = mfma16x16x32(cur[j], x0, acc[2 * ip][j]);
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[2 * ip + 1][j] = mfma16x16x32(cur[j], x1, acc[2 * ip + 1][j]);
            __builtin_amdgcn_sched_barrier(0);
            x0 = n0;
            x1 = n1;
        }
    };

    // Short tiles (TM <= 4) have registers for a whole step of X fragments: every step first issues the LDS reads
    // of the NEXT step, so that only the first step after a barrier waits for LDS.  With one or two waves per SIMD
    // nothing else would cover that latency (measured: about 300 cycles per step before, of which 130 were the
    // wait for the fragments just requested).
    constexpr bool XAHEAD = TM <= 4;
    constexpr int XF = XAHEAD ? TM : 1;
    f16x8 xfa[XF], xfb[XF];
    auto read_x = [&](f16x8 (&xf)[XF], int buf, int tt) {
#pragma unroll
        for (int i = 0; i < XF; ++i) xf[i] = *x_frag(buf, tt, i);
    };
    auto step_ahead = [&](const f16x8 (&xc)[XF], f16x8 (&xn)[XF], int buf, int tt_x_next, const f16x8 (&cur)[TN],
                          f16x8 (&nxt)[TN], const uint32_t (&wsrc)[TN][KW * WPS], const uint32_t (&ssrc)[TN][SG],
                          int tt_next) {
        if (tt_x_next >= 0) read_x(xn, buf, tt_x_next);
#pragma unroll
        for (int i = 0; i < XF; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
                if (j * XF / TN == i)              // spread the TN conversions over the rows
                    nxt[j] = convert(wsrc[j], tt_next, ssrc[j][(tt_next * GPU) / 4 % SG]);
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = mfma16x16x32(cur[j], xc[i], acc[i][j]);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    if (st0 < st1) {
        f16x8 wfa[TN], wfb[TN];
        const int nst = st1 - st0, last = st1 - 1;
        // prologue: stage 0 of X into LDS buffer 0; stages 0..PD-1 of W into their register sets
        // End of a stage.  The X loads are the first loads of every stage and each load_w call issues exactly
        // kWLoads load instructions after them, so "at most NLOADS loads outstanding" (the load counter retires in
        // order) means the X of the next stage has landed in LDS while the weight prefetch stays in flight across
        // the barrier.  A plain barrier instruction, not __syncthreads(): the fence in the latter waits for every
        // outstanding direct-to-LDS load, i.e. for everything younger in the queue as well.
        constexpr int kWLoads = TN * SG + TN * UW;
        auto stage_barrier = [&](auto NLOADS) {
            // the counter field has 6 bits; a smaller bound only waits for a few weight loads more
            constexpr int n = decltype(NLOADS)::value < 63 ? decltype(NLOADS)::value : 63;
            // vmcnt = n, lgkmcnt = 0 (this wave's LDS reads are done), expcnt untouched
            __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | (7 << 4) | (0 << 8));
            __builtin_amdgcn_s_barrier();
        };
        load_x(0, st0);
        __builtin_amdgcn_sched_barrier(0);                 // nothing may be scheduled across: the count above is exact
        load_w(wset[0], sset[0], st0);
        static_for<1, PD>([&](auto R) {
            constexpr int r = decltype(R)::value;
            load_w(wset[r % (PD + 1)], sset[r % (PD + 1)], min(st0 + r, last));
        });
#pragma unroll
        for (int j = 0; j < TN; ++j) wfa[j] = convert(wset[0][j], 0, sset[0][j][0]);
        stage_barrier(std::integral_constant<int, PD * kWLoads>{});
        constexpr int PERIOD = PD * (PD + 1);
        for (int base = 0; base < nst; base += PERIOD) {
            static_for<0, PERIOD>([&](auto PH) {
                constexpr int ph = decltype(PH)::value;
                const int r = base + ph;               // stage relative to st0 (uniform)
                if (r < nst) {
                    constexpr int wi = ph % (PD + 1);              // W(r)
                    constexpr int wn = (ph + 1) % (PD + 1);        // W(r + 1)
                    constexpr int wf = (ph + PD) % (PD + 1);       // set that takes W(r + PD)
                    constexpr int buf = ph & 1;                    // = r & 1: PERIOD is even
                    if constexpr (XAHEAD) read_x(xfa, buf, 0);
                    // stages past the end re-fetch the last one instead of branching; that data is never used
                    // X of the next stage goes straight into the other LDS buffer, which every wave finished
                    // reading before the barrier that ended the previous stage; these loads come first
                    load_x(buf ^ 1, min(st0 + r + 1, last));
                    __builtin_amdgcn_sched_barrier(0);
                    load_w(wset[wf], sset[wf], min(st0 + r + PD, last));
                    // The group constants derive from the scale/zero words alone, so the compiler would compute
                    // them right after the load that fetches those words, i.e. wait for loads just issued.  The
                    // words of the NEXT stage are therefore made opaque right before the stage's last step, the
                    // first place that needs them; being first in issue order, they have landed long before.
                    auto pin_next_sz = [&]() {
#pragma unroll
                        for (int j = 0; j < TN; ++j)
#pragma unroll
                            for (int g = 0; g < SG; ++g) asm volatile("" : "+v"(sset[wn][j][g]));
                    };
#pragma unroll
                    for (int tt = 0; tt < KW; tt += 2) {
                        if constexpr (XAHEAD) {
                            step_ahead(xfa, xfb, buf, tt + 1, wfa, wfb, wset[wi], sset[wi], tt + 1);
                            if (tt + 2 < KW) {
                                step_ahead(xfb, xfa, buf, tt + 2, wfb, wfa, wset[wi], sset[wi], tt + 2);
                            } else {
                                pin_next_sz();
                                step_ahead(xfb, xfa, buf, -1, wfb, wfa, wset[wn], sset[wn], 0);
                            }
                        } else {
                            step(buf, tt, wfa, wfb, wset[wi], sset[wi], tt + 1);
                            if (tt + 2 < KW) {
                                step(buf, tt + 1, wfb, wfa, wset[wi], sset[wi], tt + 2);
                            } else {
                                pin_next_sz();
                                step(buf, tt + 1, wfb, wfa, wset[wn], sset[wn], 0);
                            }
                        }
                    }
                    stage_barrier(std::integral_constant<int, kWLoads>{});
                }
            });
        }
    }

    // The wave sets' partial tiles meet in LDS (the X buffers are free after the loop's last barrier), pairwise: in
    // each round the upper half of the remaining sets hands its tiles to the lower half (set s takes the tile of set
    // s + half), as many tiles per pass as the first buffer holds.  A fixed tree, so the sum has a fixed order; set 0
    // ends up with the total and alone runs the epilogue.
    bool writer = true;
    if constexpr (KG > 1) {
        f32x4* red = (f32x4*)smem0;
        constexpr int kSetRegs = NW * TM * TN * 64;                    // f32x4 slots of one set's tile
        constexpr int kCapRaw = (int)(sizeof(smem0) / kSetTileBytes);
        static_for<0, 3>([&](auto R) {                                 // up to three halvings: KG = 2, 4 or 8
            constexpr int active = KG >> decltype(R)::value;
            if constexpr (active > 1 && kRedParts > 1) {
                // one pair of sets at a time, TM / kRedParts row tiles per hand-over
                constexpr int half = active / 2;
                constexpr int kRows = TM / kRedParts;
                static_for<0, half * kRedParts>([&](auto P) {
                    constexpr int pair = decltype(P)::value / kRedParts, part = decltype(P)::value % kRedParts;
                    f32x4* slot = red + (size_t)wave * (kRows * TN * 64) + lane;
                    if (kg == half + pair) {
#pragma unroll
                        for (int i = 0; i < kRows; ++i)
#pragma unroll
                            for (int j = 0; j < TN; ++j) slot[(i * TN + j) * 64] = acc[part * kRows + i][j];
                    }
                    __syncthreads();
                    if (kg == pair) {
#pragma unroll
                        for (int i = 0; i < kRows; ++i)
#pragma unroll
                            for (int j = 0; j < TN; ++j) acc[part * kRows + i][j] += slot[(i * TN + j) * 64];
                    }
                    if constexpr (!(active == 2 && decltype(P)::value == half * kRedParts - 1)) __syncthreads();
                });
            } else if constexpr (active > 1) {
                constexpr int half = active / 2;
                constexpr int cap = kCapRaw < half ? kCapRaw : half;
                constexpr int passes = (half + cap - 1) / cap;
                static_for<0, passes>([&](auto P) {
                    constexpr int p0 = decltype(P)::value * cap;
                    constexpr int p1 = p0 + cap < half ? p0 + cap : half;
                    if (kg >= half + p0 && kg < half + p1) {
                        f32x4* dst = red + (size_t)(kg - half - p0) * kSetRegs + (size_t)wave * (TM * TN * 64) + lane;
#pragma unroll
                        for (int i = 0; i < TM; ++i)
#pragma unroll
                            for (int j = 0; j < TN; ++j) dst[(i * TN + j) * 64] = acc[i][j];
                    }
                    __syncthreads();
                    if (kg >= p0 && kg < p1) {
                        const f32x4* src = red + (size_t)(kg - p0) * kSetRegs + (size_t)wave * (TM * TN * 64) + lane;
#pragma unroll
                        for (int i = 0; i < TM; ++i)
#pragma unroll
                            for (int j = 0; j < TN; ++j) acc[i][j] += src[(i * TN + j) * 64];
                    }
                    if constexpr (!(active == 2 && decltype(P)::value == passes - 1)) __syncthreads();
                });
            }
        });
        writer = kg == 0;
    }

    // Epilogue.  acc[i][j][r] = Y[m0 + 16i + c][16*(nt0 + j) + 4h + r]: four consecutive columns per lane.
    if (p.split == 1) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + i * 16 + c;
            if (m >= p.M || !writer) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int nt = nt0 + j;
                if (nt >= nt_end) continue;
                store_quad(p, m, nt * 16 + 4 * h, acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
            }
        }
        return;
    }

    const int tile = tile_m + tile_n * p.tiles_m;          // counter index
    // Partial tiles live in the workspace in accumulator order, [split][tile][wave][row tile][column tile][half][lane]
    // pairs of floats: only CTAs of the same tile exchange them, so the layout is free, and in this one every store and
    // load instruction of a wave covers 512 consecutive bytes (in output order a wave's 8-byte pieces would fall into
    // sixteen different rows).  Rows and columns past the edges of Y are stored and summed like the rest and never
    // written to Y.
    constexpr size_t kTileFloats = (size_t)BM * BN;
    const size_t tile_slot = (size_t)tile * kTileFloats + (size_t)wave * (TM * TN * 256) + (size_t)lane * 2;
    const size_t split_stride = (size_t)p.tiles_m * p.tiles_n * kTileFloats;
    if (writer) {
        float* dst = p.partial + (size_t)sk * split_stride + tile_slot;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                st_partial2(dst + (i * TN + j) * 256, acc[i][j][0], acc[i][j][1]);
                st_partial2(dst + (i * TN + j) * 256 + 128, acc[i][j][2], acc[i][j][3]);
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
    // The last CTA adds the partial tiles in split order.  Every load is a round trip past the caches (1.5-2 us), so the
    // work is spread and batched: wave set kg takes the row tiles kg, kg + KG, ... (any set can - the sums come from
    // global memory, not from its accumulators, and its waves cover the same columns as set 0's), and the loads of RB
    // row tiles x up to UB splits x all column tiles are issued before the first add (the accumulators are dead by now:
    // their registers hold the loaded values).
    constexpr int UB = (TM <= 8 && TN <= 4) ? 4 : 1;       // splits per batch; the largest tiles have no registers to spare
    constexpr int RC = (TM + KG - 1) / KG;                 // row tiles per wave set
    constexpr int RBmax = 64 / (UB * TN * 4) > 0 ? 64 / (UB * TN * 4) : 1;
    constexpr int RB = RBmax < RC ? RBmax : RC;            // row tiles per batch
#pragma unroll
    for (int r0 = 0; r0 < RC; r0 += RB) {
        float v[RB][TN][4];
        int mrow[RB], irow[RB];
        bool live[RB];
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
            const int i = kg + (r0 + rr) * KG;
            const int m = m0 + i * 16 + c;
            live[rr] = r0 + rr < RC && i < TM && m < p.M;
            mrow[rr] = m;
            irow[rr] = i < TM ? i : 0;                     // row tiles past the last re-read the first
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) v[rr][j][r] = 0.f;
        }
        for (int s0 = 0; s0 < p.split; s0 += UB) {
            float a[RB][UB][TN][4];
#pragma unroll
            for (int rr = 0; rr < RB; ++rr)
#pragma unroll
                for (int u = 0; u < UB; ++u) {
                    const float* src = p.partial + (size_t)min(s0 + u, p.split - 1) * split_stride + tile_slot + (size_t)irow[rr] * (TN * 256);
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        ld_partial2(src + j * 256, a[rr][u][j][0], a[rr][u][j][1]);
                        ld_partial2(src + j * 256 + 128, a[rr][u][j][2], a[rr][u][j][3]);
                    }
                }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                if (s0 + u < p.split) {
#pragma unroll
                    for (int rr = 0; rr < RB; ++rr)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
#pragma unroll
                            for (int r = 0; r < 4; ++r) v[rr][j][r] += a[rr][u][j][r];
                }
            }
        }
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
            if (!live[rr]) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int nt = nt0 + j;
                if (nt >= nt_end) continue;
                store_quad(p, mrow[rr], nt * 16 + 4 * h, v[rr][j][0], v[rr][j][1], v[rr][j][2], v[rr][j][3]);
            }
        }
    }
    if (tid == 0) __hip_atomic_store(&p.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int TM, int TN, int NW, int GPU, int KW, int PD = (TM <= 8 ? 2 : 1), int KG = 1, int FMT = kFmtInt4>
__global__ __launch_bounds__(NW * KG * 64) void tile_kernel(GemmParams p)
{
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
    tile_body<TM, TN, NW, GPU, KW, PD, KG, FMT>(p, tile_m, tile_n, sk);
}

// KW8: stages two packed units deep (needs an even number of units per K split, which the host checks);
// otherwise one unit deep for short tiles and half a unit for tall ones.
template <int TM, int TN, int NW, int KW, int KG = 1, int FMT = kFmtInt4>
hipError_t launch_shape(const GemmParams& p, const Plan& plan, int group, hipStream_t stream)
{
    constexpr int PD = TM <= 8 ? 2 : 1;                // the 192- and 256-row tiles have no registers for more
    constexpr int SPU = FMT == kFmtInt4 ? 4 : 2;       // MFMA steps per packed unit
    dim3 grid(plan.grid), block(NW * KG * 64);
    // the kernel assumes whole stages: every K split is a multiple of the stage depth, and so is K
    if (plan.block != NW * KG * 64 || plan.stage_steps != KW || plan.kgroups != KG) return hipErrorInvalidValue;
    if ((plan.ku_per_split * SPU) % (KW * KG) || (p.KU * SPU) % (KW * KG)) return hipErrorInvalidValue;
    switch (group) {
        case 128: hipLaunchKernelGGL((tile_kernel<TM, TN, NW, 1, KW, PD, KG, FMT>), grid, block, 0, stream, p); break;
        case 64: hipLaunchKernelGGL((tile_kernel<TM, TN, NW, 2, KW, PD, KG, FMT>), grid, block, 0, stream, p); break;
        case 32: hipLaunchKernelGGL((tile_kernel<TM, TN, NW, 4, KW, PD, KG, FMT>), grid, block, 0, stream, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

}  // namespace tmw4
