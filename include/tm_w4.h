/*
 * tm_w4 — W4A16 weight-only-quantised GEMM for AMD Instinct MI355X (gfx950).
 *
 *     Y[M,N] (fp16) = X[M,K] (fp16) * dequant(Wq)[K,N],   dequant(Wq)[k][n] = (q[k][n] - z[k/g][n]) * s[k/g][n]
 *
 * Two stages, following the GEMM pipeline of the paper (Sec. 3.3 "GEMM pipeline design"):
 *   offline  tm_pack_w4      — hardware-aware weight packing (Sec. 4.1): the int4 weights are permuted once into the
 *                              order in which the matrix-core fragments consume them, so that the online stage needs
 *                              no run-time layout transformation;
 *   online   tm_gemm_w4a16   — the mixed-precision GEMM (Sec. 3.1 steps (i)-(iv), Sec. 4.3): packed weights are
 *                              loaded with coalesced 128-bit loads, converted int4 -> fp16 by bit manipulation,
 *                              zero-point and scale are applied per K-group, and fp16 matrix-core instructions
 *                              accumulate in fp32; the result is rounded once to fp16.
 *
 * Conventions
 *   - Plain C ABI.  Every pointer is a DEVICE pointer on the current HIP device unless a parameter says "host".
 *     The caller owns all buffers it passes in; the library owns what a tm_packed_w4 handle refers to.
 *   - fp16 values travel as their 16-bit patterns (uint16_t).
 *   - No call synchronises the device or the stream.  Work is enqueued on the given stream (NULL = the null stream)
 *     and the caller keeps argument buffers alive until that work has run.
 *   - Functions returning int return TM_OK (0) or a negative tm_status; functions returning a pointer return NULL on
 *     error.  tm_last_error() then describes the failure (thread-local).  No C++ exception crosses this boundary.
 *   - Shape limits: K % 128 == 0, N % 16 == 0, group in {32, 64, 128}, 0 <= M < 2^24, K*N < 2^40.
 */
#ifndef TM_W4_H
#define TM_W4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TM_API __attribute__((visibility("default")))

typedef enum tm_status {
    TM_OK = 0,
    TM_EINVAL = -1,        /* null pointer, bad shape, misaligned buffer, workspace too small */
    TM_EUNSUPPORTED = -2,  /* current device is not gfx950 */
    TM_EHIP = -3,          /* a HIP runtime call failed; tm_last_error() carries its message */
    TM_ENOMEM = -4         /* device allocation failed */
} tm_status;

typedef struct tm_packed_w4 tm_packed_w4;  /* opaque handle; immutable after creation */
typedef void* tm_stream;                   /* a hipStream_t */

/*
 * Offline hardware-aware weight packing (paper Sec. 4.1, steps (i)-(iv); here a closed-form permutation because the
 * gfx950 matrix-core operand layout is an explicit lane/register index map).
 *
 *   qweight  u32 [K][N/8]       interchange layout "eight INT4 values per 32-bit word" (Sec. 3.2, M2):
 *                               nibble t (bits 4t..4t+3) of word (k, j) is q[k][8j + t], values 0..15
 *   scales   fp16 [K/group][N]  s, finite and positive; group = 32, 64 or a multiple of 128 dividing K
 *   zeros    fp16 [K/group][N]  z, integer-valued in [0, 15] (NULL: z = 8 everywhere, see tm_pack_w4_layout)
 *
 * Allocates the handle's device buffers (K*N/2 bytes of weights, 4*K*N/group bytes of scale/zero pairs), makes sure
 * the device-wide split-K workspace is large enough for this shape, and enqueues the repack kernels on `stream`.
 * The inputs may be released once that stream work has completed.  Returns NULL on error.
 *
 * Packed layout (also what tm_packed_raw exposes):
 *   weights: units of 16 columns x 128 rows; unit (nt, ku) is the 256 u32 words starting at ((nt*(K/128))+ku)*256;
 *            word 4*lane + t (lane = 16*h + c, c in 0..15, h in 0..3, t in 0..3) holds column 16*nt + c, rows
 *            128*ku + 32*t + 8*h + e (e = 0..7), weight e in nibble 4*(e&1) + (e>>1).
 *   scale/zero: u32 word ((nt*(K/group)) + G)*16 + c = scale bits | zero bits << 16 for column 16*nt + c, group G.
 */
TM_API tm_packed_w4* tm_pack_w4(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros,
                                int K, int N, int group);
/* Same, on an explicit stream (tm_pack_w4 uses the null stream). */
TM_API tm_packed_w4* tm_pack_w4_on(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros,
                                   int K, int N, int group, tm_stream stream);

/*
 * The same packing from the other word orders in which 4-bit checkpoints keep (q, s, z) (paper Sec. 4.1: one offline
 * pack step absorbs the format differences, so the online GEMM sees a single layout).  The result is bit-identical to
 * tm_pack_w4 of the same integers; only the reading side differs.
 *
 *   TM_LAYOUT_N8              qweight u32 [K][N/8], nibble t of word (k, j) = q[k][8j + t];  zeros fp16 [K/group][N]
 *                             (exactly tm_pack_w4_on)
 *   TM_LAYOUT_N8_INTERLEAVED  qweight u32 [K][N/8], nibble p of word (k, j) = q[k][8j + o(p)], o = 0,2,4,6,1,3,5,7
 *                             (even columns in the low half-word, odd columns in the high half-word);
 *                             zeros u32 [K/group][N/8], integers 0..15 packed in the same nibble order
 *   TM_LAYOUT_K8              qweight u32 [K/8][N], nibble t of word (i, n) = q[8i + t][n];
 *                             zeros u32 [K/group][N/8], nibble t of word (G, j) = z[G][8j + t]
 *
 * scales is fp16 [K/group][N] in every layout.  Two further conventions are read here (and by tm_pack_w4 / _on):
 *   - group may also be any multiple of 128 that divides K (group == K: one scale per output channel); such weights
 *     are stored with their scale/zero rows repeated at the kernels' group of 128, which is what tm_packed_info then
 *     reports;
 *   - zeros == NULL means symmetric quantisation: every zero-point is 8 (q - 8 in [-8, 7]).
 * The zero integers are used as stored (a checkpoint convention that
 * keeps z - 1 must be undone by the caller).  Shapes, alignment (4 bytes for u32 buffers), ownership and errors are
 * those of tm_pack_w4_on; an unknown layout is TM_EINVAL (NULL return).
 */
typedef enum tm_layout { TM_LAYOUT_N8 = 0, TM_LAYOUT_N8_INTERLEAVED = 1, TM_LAYOUT_K8 = 2 } tm_layout;
TM_API tm_packed_w4* tm_pack_w4_layout(const void* qweight, const uint16_t* scales, const void* zeros, int K, int N,
                                       int group, int layout, tm_stream stream);

/*
 * Activation-order checkpoints: the K-group of row k is g_idx[k] instead of k / group, i.e.
 *     dequant(Wq)[k][n] = (q[k][n] - z[g_idx[k]][n]) * s[g_idx[k]][n].
 * g_idx is a DEVICE array of K int32 in which every group 0 .. K/group-1 occurs exactly `group` times (anything else is
 * TM_EINVAL).  The pack sorts the rows by group once (stable), so the online GEMM sees the ordinary layout; the row order
 * is kept in the handle and tm_gemm_w4a16 gathers the columns of X accordingly before it multiplies (one small extra
 * kernel).  qweight / scales / zeros / layout as for tm_pack_w4_layout.  Unlike the other pack calls this one
 * synchronises `stream` (it reads g_idx on the host and frees a temporary) and allocates, per device, a 32 MiB buffer
 * for the regrouped activations; a GEMM whose M*K*2 bytes exceed it runs in several passes.  With tm_gemm_w4a16_ws the
 * regrouped activations live in the caller's workspace instead (tm_gemm_workspace_bytes includes them).  tm_unpack_w4
 * returns the rows in packed (group-sorted) order; tm_group_experts does not take such handles.
 */
TM_API tm_packed_w4* tm_pack_w4_actorder(const void* qweight, const uint16_t* scales, const void* zeros,
                                         const int32_t* g_idx, int K, int N, int group, int layout, tm_stream stream);

/*
 * 8-bit weight codes (W8A16) through the same two stages; the paper presents packing and the fused GEMM as independent
 * of the weight width (Sec. 3.3, Sec. 4.1).  qweight is u32 [K][N/4], byte t (bits 8t..8t+7) of word (k, j) =
 * q[k][4j + t], codes 0..255; scales fp16 [K/group][N]; zeros fp16 [K/group][N], integer-valued in [0, 255], or NULL for
 * the symmetric zero-point 128.  Shapes, groups, alignment, ownership and errors as for tm_pack_w4_on.  The handle works
 * with tm_gemm_w4a16 / tm_gemm_w4a16_ws, tm_packed_info, tm_packed_raw, tm_get_plan, tm_free_packed and
 * tm_group_experts (all experts of a group in one format); tm_unpack_w4 takes 4-bit handles only (TM_EUNSUPPORTED).
 *
 * Packed layout: units of 16 columns x 64 rows (1 KiB); unit (nt, ks) is the 256 words from ((nt*(K/64))+ks)*256;
 * word 4*lane + 2*tt + hf (lane = 16*h + c, tt, hf in 0..1) holds column 16*nt + c, rows 64*ks + 32*tt + 8*h + 4*hf + b
 * in byte b.  Scale/zero words as for 4-bit weights.
 */
TM_API tm_packed_w4* tm_pack_w8(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros, int K, int N,
                                int group, tm_stream stream);
/*
 * FP8 weights (the paper's evaluation includes an FP8 model, Sec. 5.3): the 8-bit codes are numbers of the OCP FP8 E4M3
 * format (finite-only: bias 7, largest value 448, S.1111.111 = NaN) and
 *     dequant(Wq)[k][n] = fp8(q[k][n]) * s[k/group][n]          (no zero-point).
 * qweight u32 [K][N/4] as for tm_pack_w8, scales fp16 [K/group][N].  Same packed layout and the same
 * supporting calls as tm_pack_w8.  NaN codes propagate.
 */
TM_API tm_packed_w4* tm_pack_w8_fp8(const uint32_t* qweight, const uint16_t* scales, int K, int N, int group,
                                    tm_stream stream);
/* Width of the handle's weight codes: 4 or 8 (negative status on error). */
TM_API int tm_packed_bits(const tm_packed_w4* packed);

/*
 * Online mixed-precision GEMM (paper Sec. 3.1 steps (i)-(iv) and Sec. 4.3): Y = X * dequant(packed).
 *
 *   X  fp16 [M][K] row-major, 16-byte aligned        Y  fp16 [M][N] row-major, 16-byte aligned;  M*K < 2^31
 *
 * Picks a kernel variant and a split-K factor from (M, K, N, group) and enqueues it on `stream`.  Never allocates.
 * Split-K partial sums go through the library's device-wide workspace and are reduced in a fixed order, so results
 * are bit-identical from run to run.  Because that workspace is shared, calls on one device must be ordered on one
 * stream (or serialised by the caller); use tm_gemm_w4a16_ws for concurrent streams.  M == 0 is a successful no-op.
 */
TM_API int tm_gemm_w4a16(const uint16_t* X, const tm_packed_w4* packed, uint16_t* Y, int M, tm_stream stream);

/*
 * The same product with what surrounds it in a transformer block fused into the kernels' final store (not a technique
 * of the paper; it removes the extra pass over Y that an unfused bias / activation / residual costs):
 *
 *     T = X * dequant(packed) + bias                                   bias fp16 [N], or NULL
 *     U = T                        (TM_ACT_NONE)                       [M][N]
 *       = silu(T_gate) * T_up      (TM_ACT_SILU_MUL)                   [M][N/2], silu(x) = x / (1 + exp(-x))
 *     Y = fp16(U + residual)                                           residual fp16 [M][N or N/2], or NULL
 *
 * all in fp32 on the fp32 sums, rounded once.  TM_ACT_SILU_MUL takes the fused gate+up projection of a gated MLP: the
 * weight's columns are [gate (N/2) | up (N/2)] and the handle must come from tm_pack_w4_gate_up, which stores gate
 * column j and up column j side by side so that one thread holds both; such a handle is accepted by this call with
 * TM_ACT_SILU_MUL only.  bias and residual follow the caller's column order and must be 16-byte aligned; Y as above.
 * epilogue == NULL is tm_gemm_w4a16.  Works for every weight format a handle can hold.
 */
typedef enum tm_activation { TM_ACT_NONE = 0, TM_ACT_SILU_MUL = 1 } tm_activation;
typedef struct tm_epilogue {
    const uint16_t* bias;      /* device, fp16 [N], or NULL */
    const uint16_t* residual;  /* device, fp16 [M][N] (TM_ACT_NONE) or [M][N/2] (TM_ACT_SILU_MUL), or NULL */
    int act;                   /* tm_activation */
} tm_epilogue;
TM_API int tm_gemm_w4a16_ex(const uint16_t* X, const tm_packed_w4* packed, uint16_t* Y, int M, const tm_epilogue* epilogue,
                            tm_stream stream);
/*
 * tm_pack_w4 for a fused [gate | up] weight (N = 2 * intermediate size, N % 32 == 0; inputs in the layout of
 * tm_pack_w4, zeros may be NULL): the columns are interleaved as (gate j, up j) pairs before the packing.  Synchronises
 * `stream` once (the interleaved copies are temporaries).  The handle serves tm_gemm_w4a16_ex with TM_ACT_SILU_MUL.
 */
TM_API tm_packed_w4* tm_pack_w4_gate_up(const uint32_t* qweight, const uint16_t* scales, const uint16_t* zeros, int K, int N,
                                        int group, tm_stream stream);

/*
 * Same multiply with a caller-owned workspace of at least tm_gemm_workspace_bytes(packed, M) bytes, 256-byte aligned.
 * The workspace must be zero-filled once before its first use; every call leaves it ready for the next one.
 * Distinct workspaces may be used concurrently on distinct streams.
 */
TM_API int tm_gemm_w4a16_ws(const uint16_t* X, const tm_packed_w4* packed, uint16_t* Y, int M,
                            void* workspace, size_t workspace_bytes, tm_stream stream);

/*
 * tm_gemm_w4a16 for callers that cannot allocate device memory or let a library do so on their behalf: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same plan and bit-identical
 * results; the split-K arrival counters and partial sums live in a fixed array inside the library's device image
 * (64 KiB of counters + 8 MiB of partial sums per GPU, held until the process ends) instead of the workspace that
 * tm_pack_w4 allocates.  The call itself allocates and frees nothing and never synchronises.  A plan whose partial
 * sums (split_k * M * N * 4 bytes; for activation-order handles plus M * K * 2 bytes of regrouped activations) exceed
 * the 8 MiB is refused with TM_EINVAL and a message that names both sizes; nothing is launched then.  All calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two threads) race and must be
 * serialised by the caller.  The first call on a device clears the counters with a small kernel on `stream`; every call
 * returns them to zero, so the array is ready for the next call whatever its shape.  X, Y, M, stream, errors: as
 * tm_gemm_w4a16.
 */
TM_API int tm_gemm_w4a16_static(const uint16_t* X, const tm_packed_w4* packed, uint16_t* Y, int M, tm_stream stream);

/*
 * Returns the split-K arrival counters of a workspace to zero (a small kernel on `stream`): of the caller's workspace, or,
 * with workspace == NULL, of the library's own workspace and of the static scratch of tm_gemm_w4a16_static on the current
 * device.  Every GEMM leaves the counters at zero, so this is needed only after a launch that did not run to completion
 * (a device error, an aborted stream): counters left part-way would make a later call pick the wrong CTA as the last one.
 * Must not overlap with a GEMM that uses the same workspace.
 */
TM_API int tm_reset_workspace(void* workspace, tm_stream stream);

/* Workspace bytes the plan for this (packed, M) needs (0 is never returned for M > 0; 0 on error or M == 0). */
TM_API size_t tm_gemm_workspace_bytes(const tm_packed_w4* packed, int M);

/* Releases the handle and its device buffers.  NULL is ignored.  The caller makes sure no enqueued work still uses it. */
TM_API void tm_free_packed(tm_packed_w4* packed);

/*
 * Grouped GEMM for mixture-of-experts layers.  The paper's evaluation includes MoE models (Sec. 5.1, Sec. 5.3) and
 * describes no separate kernel for them: an expert layer is the same mixed-precision GEMM (Sec. 3.1) once per expert,
 * each on the rows routed to it.  With the rows of X sorted by expert,
 *
 *     Y[r][:] = X[r][:] * dequant(expert e),   offsets[e] <= r < offsets[e+1],   e = 0 .. num_experts-1
 *
 * tm_group_experts (offline, once per layer): `experts` is a HOST array of num_experts handles (1..65535) with equal
 * K, N, group, device and weight format (4-bit, 8-bit integer or FP8 codes; not activation-order handles); it allocates a small device table of their buffer addresses (synchronous copy).  The group
 * borrows the handles: they must outlive it.  Returns NULL on error.  tm_free_expert_group releases the table only.
 *
 * tm_gemm_w4a16_grouped (online): X fp16 [total_rows][K], Y fp16 [total_rows][N], both 16-byte aligned; offsets is a
 * DEVICE array of num_experts + 1 ascending int32 row indices, so routing results never pass through the host.  One
 * launch covers all experts, and only experts with rows occupy CTAs.  Rows outside
 * [offsets[0], offsets[num_experts]) are left untouched; offsets are clamped to [0, total_rows].  Never allocates,
 * uses no workspace (K is not split across CTAs), results are bit-identical from run to run.  The kernel is chosen
 * from total_rows / num_experts (the per-expert counts are not known on the host): decode-sized loads run the decode
 * kernels (an expert with more rows than one pass takes, 16-64, is processed in several passes), prefill-sized
 * loads (about 64 rows per expert and more) run the CTA-tile kernels, which need total_rows * K < 2^31.  The choice
 * assumes a roughly balanced routing (mean load plus three standard deviations); under a heavily skewed one the result
 * is still exact, but an expert with many times the average load is taken in passes that each stream its weights again.
 * total_rows == 0 is a successful no-op; total_rows < 2^24.
 */
typedef struct tm_expert_group tm_expert_group;
TM_API tm_expert_group* tm_group_experts(const tm_packed_w4* const* experts, int num_experts);
TM_API void tm_free_expert_group(tm_expert_group* group);
TM_API int tm_gemm_w4a16_grouped(const uint16_t* X, const tm_expert_group* group, const int32_t* offsets, uint16_t* Y,
                                 int total_rows, tm_stream stream);
/*
 * The grouped call with the gated MLP's activation fused (see tm_gemm_w4a16_ex): every expert of the group is a handle
 * of tm_pack_w4_gate_up and Y is fp16 [total_rows][N/2], Y[r] = silu(T_gate) * T_up of T = X[r] * dequant(expert).
 * act must be TM_ACT_SILU_MUL for such a group and TM_ACT_NONE (= tm_gemm_w4a16_grouped) for any other.
 */
TM_API int tm_gemm_w4a16_grouped_act(const uint16_t* X, const tm_expert_group* group, const int32_t* offsets, uint16_t* Y,
                                     int total_rows, int act, tm_stream stream);
/* Kernel variant and strips per expert the grouped launch would use (host out-pointers, may be NULL). */
TM_API int tm_get_grouped_plan(const tm_expert_group* group, int total_rows, int* variant, int* strips);

/* Shape of a handle; any out-pointer (host) may be NULL.  `bytes` = device bytes held (weights + scale/zero pairs). */
TM_API int tm_packed_info(const tm_packed_w4* packed, int* K, int* N, int* group, size_t* bytes);

/*
 * Test hooks for the bit-exact packing check.
 * tm_unpack_w4 runs the inverse permutation on the device: qweight_out u32 [K][N/8], scales_out / zeros_out
 * fp16 [K/group][N] (any of the three may be NULL).  tm_packed_raw returns the handle's device buffers (host
 * out-pointers; the memory stays owned by the handle) so that an independent unpacker can be run on a copy.
 */
TM_API int tm_unpack_w4(const tm_packed_w4* packed, uint32_t* qweight_out, uint16_t* scales_out,
                        uint16_t* zeros_out, tm_stream stream);
TM_API int tm_packed_raw(const tm_packed_w4* packed, const void** weights, size_t* weight_bytes,
                         const void** scale_zero, size_t* scale_zero_bytes);

/*
 * Kernel selection (the run-time counterpart of the tile configuration the paper's packing is meant to make
 * unnecessary to hand-tune per architecture, Sec. 4.1).  tm_get_plan reports what tm_gemm_w4a16 would launch for M
 * rows (host out-pointers, any may be NULL).  tm_set_variant overrides the choice process-wide for sweeps:
 * variant -1 / split_k 0 restore automatic selection.  tm_variant_name(-1..) returns "" past the last variant.
 */
TM_API int tm_get_plan(const tm_packed_w4* packed, int M, int* variant, int* split_k, int* grid, int* block);
/*
 * The decode shapes (M <= 16, 4-bit codes) have two forms of their kernels: the one-shot form, in which a wave requests
 * its whole share of the weight stream at once and keeps its rows of X in LDS (taken when the share fits the registers
 * and the rows fit LDS), and the ring-buffered form.  Returns the packed units per wave of the one-shot form the plan for
 * M rows uses, 0 if the plan uses the ring-buffered form or another kernel family, a negative status on error.
 */
TM_API int tm_get_plan_units_per_wave(const tm_packed_w4* packed, int M);
TM_API int tm_set_variant(int variant, int split_k);
/*
 * Two more launch parameters for sweeps, 0 = automatic.
 *   waves        waves per CTA: 8 or 16 for the skinny (M <= 16/32/64) kernels, which split K inside the CTA; 4, 8 or
 *                16 for the tile kernels, whose CTAs hold one, two or four sets of waves, each set multiplying its
 *                own slice of every K stage (a value a variant is not built with falls back to its default);
 *   stage_steps  MFMA steps of 32 K-rows per pipeline stage and wave set of the tile kernels: 2, 4 or 8 (a request
 *                the shape or the variant's register budget cannot honour falls back to the nearest valid depth);
 *                1 leaves the tile kernels alone and makes the decode shapes (M <= 16) take the ring-buffered form of
 *                their kernels where they would take the one-shot form.
 */
TM_API int tm_set_launch(int waves, int stage_steps);
/*
 * The matrix instruction of the prefill CTA tiles (128 x 256 and 128 x 512, unsplit, one wave set): 0 = automatic and 16 =
 * the 16x16x32 form every other kernel uses; 32 = the 32x32x16 form (a second build of the same pipeline, measured 10 %
 * slower on this chip and therefore never chosen automatically).  A sweep and test setting like the two above.
 * tm_get_plan_mfma_shape reports which of the two a launch of M rows takes (16 or 32; negative = error).
 */
TM_API int tm_set_mfma_shape(int shape);
TM_API int tm_get_plan_mfma_shape(const tm_packed_w4* packed, int M);
TM_API const char* tm_variant_name(int variant);

/*
 * Measurement helpers (not part of the method): a plain 128-bit copy kernel of known size, used to calibrate the
 * profiler's HBM byte counters, and a read-only streaming kernel that gives the achievable HBM read ceiling.
 * `bytes` must be a multiple of 16; `sink` is a 4-byte device location the read kernel may write.
 */
TM_API int tm_bench_copy(void* dst, const void* src, size_t bytes, tm_stream stream);
TM_API int tm_bench_read(const void* src, size_t bytes, void* sink, tm_stream stream);
/*
 * The same read-only stream in a chosen launch shape, to find the best streaming shape at a given byte count (the
 * ceiling a weight-streaming kernel of that size can be held against): `grid` CTAs of `block` threads (a multiple of 64,
 * at most 1024), `unroll` (1, 2, 4, 8 or 16) 128-bit loads in flight per thread; flags bit 0 = non-temporal loads,
 * bit 1 = every CTA reads one contiguous slice of the buffer instead of interleaving with the others, bit 2 = every CTA
 * reads the whole buffer (the way every CTA of a GEMM reads all of X; `grid` x `bytes` are then moved in total, and a
 * buffer that stays in the L2 measures how fast the compute units can be fed from there; bit 1 is ignored).
 */
#define TM_READ_NONTEMPORAL 1
#define TM_READ_CHUNKED 2
#define TM_READ_SHARED 4
TM_API int tm_bench_read_shape(const void* src, size_t bytes, void* sink, int grid, int block, int unroll, int flags,
                               tm_stream stream);

/*
 * A kernel of matrix instructions only, to find what the matrix pipes sustain at the clock the chip holds under that load
 * (the ceiling an MFMA-bound kernel can be held against, beside the data-sheet peak): `grid` CTAs of `block` threads
 * (a multiple of 64, at most 1024), every wave issuing `iters` x 8 independent 16x16x32 fp16 MFMAs (16 384 flop each) on
 * register operands; pattern 0 = zero operands, 1 = operands that differ per lane, the same for every instruction,
 * 2 = a different operand pair for each of the eight instructions (the operand latches switch as they do in a GEMM).  `out` is a 16-byte aligned device
 * location of four 32-bit words: word 0 receives the shader clock counter's advance over the first wave's loop, word 1
 * the advance of the constant-rate counter (`hipDeviceAttributeWallClockRate`) over the same loop.
 */
TM_API int tm_bench_mfma(void* out, int grid, int block, int iters, int pattern, tm_stream stream);

/*
 * One wave that sleeps through `delay_micros` (0 ... 100000) microseconds of the constant-rate counter, then watches the
 * shader clock counter for `micros` (1 ... 20000) microseconds and writes both counters' advance over that stretch to
 * `out` (16-byte aligned device location: word 0 shader clocks, word 1 constant-rate ticks).  Launched on a second stream
 * *before* other work is queued it gives the clock the chip holds under that work (a launch that fills the register
 * file would keep a later probe waiting until it has drained); it takes no LDS, one wave slot and a few registers, and
 * ends by itself.  Returns the constant-rate counter's frequency in kHz (positive) or a negative error code.
 */
TM_API int tm_bench_clock(void* out, int delay_micros, int micros, tm_stream stream);

TM_API const char* tm_last_error(void);
TM_API const char* tm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TM_W4_H */
