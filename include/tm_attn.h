/*
 * tm_attn — decode attention over a quantised KV cache for AMD Instinct MI355X (gfx950); part of libtm_w4.
 *
 * The attention pipeline of the paper (Sec. 3.3 "attention pipeline design"): at a decoding step each query head
 * attends over the keys and values cached for its sequence,
 *
 *     O[b][h] = softmax(scale * K^[b][h/G] q[b][h]) V^[b][h/G],      K^ = (Kq - zK) * sK,   V^ = (Vq - zV) * sV,
 *
 * with the cache kept as low-bit integer codes (Sec. 3.1: the same workflow with INT4/INT8 KV caches).  The paper does
 * not state the cache's quantisation granularity; here every token and KV head has one asymmetric scale / zero-point
 * pair over the 128 values of the head, for 8-bit or 4-bit codes (x^ = (q - z) * s, s = fp16((max - min)/qmax),
 * z = round(-min/s), qmax = 255 or 15).
 *
 *   Q branch (Sec. 4.2, adaptive head alignment): the query fragments are arranged once per call so that their
 *     per-lane dimension order equals the order in which a lane receives the low-bit key bytes; no key is reshuffled.
 *   KV branch (Sec. 4.4, KV memory loading pipeline; Sec. 4.3): key and value codes are loaded straight into matrix-core
 *     operand order, two blocks ahead of the block being multiplied, converted by bit manipulation; scale and zero-point
 *     are applied to the scores and probabilities (per token), never to the 128 values of a token.
 *
 * Conventions as in tm_w4.h: plain C ABI, DEVICE pointers unless marked host, fp16 as uint16_t bit patterns, nothing
 * synchronises, work is enqueued on the given stream, negative tm_status codes with tm_last_error().
 * Head dimension is 128.  Grouped-query attention: q_heads = G * kv_heads, 1 <= G <= 128 (a KV head's G query heads are
 * taken sixteen at a time - the sixteen columns of a matrix-core tile - in passes that follow each other on the stream;
 * up to G = 16 that is one pass).
 */
#ifndef TM_ATTN_H
#define TM_ATTN_H

#include "tm_w4.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tm_kv_cache tm_kv_cache;   /* opaque; owns its device buffers */

/*
 * A cache for `batch` sequences x `kv_heads` heads x `capacity` tokens of `bits`-bit codes (bits 8 or 4; the capacity is
 * rounded up to a multiple of 256 / bits tokens).  Allocates 2 * batch*kv_heads*capacity*128*bits/8 bytes of codes,
 * 8 bytes of scale/zero pairs per token and head, and the split workspace of tm_attn_decode (a few MiB).  Contents start
 * undefined.  NULL on error.
 *
 * Layout (also what tm_kv_raw exposes); bh = b*kv_heads + h.  The cache is kept in matrix-core operand order (the
 * hardware-aware packing of Sec. 4.1 applied to the cache): codes in blocks of 32 tokens x 128 dimensions (4096 bytes),
 * block bh*(capacity/32) + t/32, token u = t % 32, such that every load instruction of a wave reads 1 KiB of consecutive
 * bytes and each lane receives exactly its operand bytes:
 *   K block   dimension d at byte ((j*2 + half)*64 + 16*hh + c)*16 + x,  j = u / 16, c = u % 16, hh = d / 32,
 *             half = (d % 32) / 16, x = d % 16
 *   V block   dimension d at byte ((i/2)*64 + 16*hh + c)*16 + (i % 2)*8 + e,  c = d % 16, i = d / 16,
 *             hh = (u % 16) / 4, e = u % 4 + 4*(u / 16)
 *   pairs     u32 word (bh*capacity + t)*2 + {0: K, 1: V} = scale bits | zero bits << 16
 * 4-bit codes: blocks of 32 tokens are 2048 bytes of little-endian 32-bit words, eight codes per word; the code of
 * operand element e sits in bits 4p .. 4p+3, p = e/2 + 4*(e % 2) (the order the bit-manipulation conversion emits):
 *   K block   word ((u/16)*64 + 16*(d/32) + u%16)*4 + (d%32)/8, element e = d % 8
 *   V block   word ((i/4)*64 + 16*hh + c)*4 + i%4, i = d / 16, c = d % 16, hh = (u % 16) / 4, element e = u%4 + 4*(u/16)
 */
TM_API tm_kv_cache* tm_kv_create(int batch, int kv_heads, int capacity, int bits);
TM_API void tm_kv_free(tm_kv_cache* cache);

/*
 * Quantise and store `count` new tokens per sequence: K_new, V_new fp16 [batch][count][kv_heads][128]; sequence b's
 * tokens go to positions[b] .. positions[b] + count - 1 (positions: int32 [batch]; tokens that would fall outside
 * [0, capacity) are dropped).  Codes are decided in fp32 with the fp16-rounded scale, round half to even.
 * Runs of 16 or more tokens with 16-byte aligned K_new and V_new take a block-wise kernel that writes whole 4 KiB cache
 * blocks; the stored bytes are the same either way.  A 4-bit cache needs 16-byte aligned K_new and V_new.  Appends to
 * one cache must be ordered on one stream.
 */
TM_API int tm_kv_append(tm_kv_cache* cache, const uint16_t* K_new, const uint16_t* V_new, const int32_t* positions,
                        int count, tm_stream stream);

/*
 * One decoding step.  Q fp16 [batch][q_heads][128], O fp16 [batch][q_heads][128], both 16-byte aligned; lens int32
 * [batch] = tokens cached per sequence (clamped to [0, capacity]; a sequence with 0 tokens gets O = 0).  max_len (host)
 * is an upper bound of lens that steers how the context is split across CTAs; pass the capacity (or 0) if unknown.  A
 * sequence longer than max_len rounded up to whole blocks and splits attends over that many leading tokens only.  Never
 * allocates.
 * Partial results of split contexts go through the cache's own workspace: calls on one cache must be ordered on one
 * stream.  Results are bit-identical from run to run.
 */
TM_API int tm_attn_decode(const uint16_t* Q, const tm_kv_cache* cache, const int32_t* lens, uint16_t* O, int q_heads,
                          float scale, int max_len, tm_stream stream);

/*
 * A chunk of prompt tokens (the prefill side of the attention pipeline, paper Sec. 3.3; Sec. 4.2 and 4.4 apply as at a
 * decoding step).  Q fp16 [batch][count][q_heads][128] and O fp16 of the same shape, both 16-byte aligned: query token i
 * of sequence b sits at cache position positions[b] + i (positions: int32 [batch], device) and attends causally over
 * cache tokens 0 .. positions[b] + i; its own key and value must already be in the cache (tm_kv_append first, on the same
 * stream).  counts (int32 [batch], device, or NULL = every sequence has `count` tokens) gives the query tokens each
 * sequence really has, so that prompts of different lengths share one call: rows i >= counts[b] of O, and rows whose
 * position falls outside [0, capacity), are left untouched.  q_heads and scale as for tm_attn_decode; 1 <= count <= 65535
 * * (16 / min(G, 16)), G = q_heads / kv_heads.  One CTA takes 16 / min(G, 16) consecutive tokens of one KV head and streams
 * the cache up to the last of them; the context is not split, so a short chunk far into a long context is served by few
 * CTAs (use tm_attn_decode per token there).  Never allocates, uses no workspace, results are bit-identical from run to
 * run.
 */
TM_API int tm_attn_prefill(const uint16_t* Q, const tm_kv_cache* cache, const int32_t* positions, const int32_t* counts,
                           int count, uint16_t* O, int q_heads, float scale, tm_stream stream);

/* Test hook: the cache's device buffers and sizes (host out-pointers, any may be NULL); memory stays owned by the cache. */
TM_API int tm_kv_raw(const tm_kv_cache* cache, void** k_codes, void** v_codes, void** pairs, size_t* code_bytes,
                     size_t* pair_bytes);

#ifdef __cplusplus
}
#endif
#endif
