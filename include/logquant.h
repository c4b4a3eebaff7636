/*
 * logquant.h - C ABI of the MI355X (gfx950) LogQuant decode hot path.
 *
 * LogQuant (arXiv 2503.19950) keeps a log-sparse set of past tokens at original
 * precision (Algorithm 1, Sec. 2.5), quantizes every token that leaves that set
 * to 2 bits (Fig. 6 caption, Sec. 2.3; INT2 and group size G in Sec. 3.1, keys
 * per channel in Sec. 2.5; 4 bits as the variant of Sec. 3.2.1), stores both regions one after the other without
 * regard to token positions (Sec. 2.4, Eq. 3) and attends over both with one
 * softmax (Eq. 2, with the 1/sqrt(d) of Eq. 6).
 *
 * Conventions for every entry point
 *   - All buffer pointers are caller-owned DEVICE memory unless marked HOST.
 *     The library never allocates, frees or synchronises; work is enqueued on
 *     the given HIP stream (passed as void*, 0 = default stream).
 *   - lq_config and lq_cache are HOST structs.  Token counts live in the host
 *     struct (lock-step batch: every sequence has the same length; see lq_cache_seq
 *     at the end for per-sequence lengths) and are updated synchronously by the call
 *     that changes them.
 *   - Errors are return codes.  Argument and state errors are detected before
 *     anything is enqueued and leave the cache untouched.
 *   - T is the cache element type (fp16 or bf16); q, out and new tokens are of type T.
 *     Scales and zero-points are values of T (see the quantizer below) but are stored
 *     as fp16 for either T, which is the form the decode kernel's matrix operands need:
 *     for a bf16 cache the conversion is exact for values in fp16's normal range
 *     (6.1e-5 <= |x| <= 65504), rounds to nearest below it and overflows above it.
 *
 * Physical layouts.  Row order inside either region carries no meaning for
 * attention (Eq. 3), so every buffer is stored in the order the decode kernel's
 * 64-lane matrix instructions consume it; a lane then reads its operand with
 * one contiguous 16-byte load.  With
 *     bh    = b * Hkv + h                     (batch row b, kv head h)
 *     NKC   = d / 32,  NNT = d / 16,  NGC = ceil(d / G),  W = fp_budget/2,
 *     CAP   = 3W rounded up to a multiple of 32,  WQ = ceil(W / G) * G
 *     kperm(x) = 8*((x % 16) / 4) + 4*(x / 16) + (x % 4)          for 0 <= x < 32
 * the element (slot t, channel c) of one (b, h) slice lives at:
 *
 *   k_fp[buf]   T     index (((bh*(CAP/16) + t/16)*NKC + c/32)*64 + 16*((c%32)/8) + t%16)*8 + c%8
 *   v_fp[buf]   T     index (((bh*(CAP/32) + t/32)*NNT + c/16)*64 + 16*(k/8) + c%16)*8 + k%8,
 *                     k = kperm(t % 32)
 *   pos_fp[buf] i32   index b*CAP + t                     absolute position of fp slot t
 *
 *   k_codes     u32   word  ((bh*(q_capacity/32) + t/32)*64 + 16*((c%32)/8) + t%16)*NKC + o/2,
 *                     o = ((t%32)/16)*NKC + c/32,
 *                     bits [p, p+2) with p = 8*(o%2) + 2*((c%8)/2) + 16*(c%2)
 *   v_codes     u32   word  ((bh*(q_capacity/32) + t/32)*64 + 16*(k/8) + c%16)*NKC + (c/16)/2,
 *                     k = kperm(t % 32),
 *                     bits [p, p+2) with p = 8*((c/16)%2) + 2*((k%8)/2) + 16*(k%2)
 *   with bits = 4 a lane owns one word per operand instead of half a word:
 *   k_codes     u32   word  ((bh*(q_capacity/32) + t/32)*64 + 16*((c%32)/8) + t%16)*2*NKC + o,
 *                     bits [p, p+4) with p = 4*((c%8)/2) + 16*(c%2)
 *   v_codes     u32   word  ((bh*(q_capacity/32) + t/32)*64 + 16*(k/8) + c%16)*2*NKC + c/16,
 *                     bits [p, p+4) with p = 4*((k%8)/2) + 16*(k%2)
 *   k_scale, k_zero   f16 index (bh*(q_capacity/G) + t/G)*d + c      one per channel per G slots
 *   v_scale, v_zero   f16 index ((bh*(q_capacity/32) + t/32)*NGC + c/G)*32 + kperm(t % 32)
 *   pos_q       i32   index b*q_capacity + t              absolute position of quantized slot t
 *
 * Slots 0..n_fp-1 of the fp region are in the logical order of Algorithm 1's
 * list.  The quantized region is filled in eviction order, WQ slots per filtering
 * event: the i-th row an event removes (0 <= i < W) goes to slot (n_q before the
 * event) + i.  When G divides W (WQ == W) every slot below n_q holds a token.
 * Otherwise (e.g. the paper's W = floor(R/3), R = 128 or 256, with G = 64; Sec. 3.1,
 * appendix D) the last key group of an event is short and the WQ - W slots behind it
 * are padding: zero codes, zero value scales and zero-points, pos_q = -1; attention
 * gives them no weight.  Content of slots beyond the counts is unspecified and
 * never influences a result.
 *
 * Quantizer (one group of values x_i of type T, n = 2^bits - 1 steps; a reading, the
 * paper prints no formula): zero z = min x_i (with -0 stored as +0); scale
 * s = T((f32(max) - f32(min)) / n) with IEEE fp32 subtract and divide and
 * round-to-nearest-even to T; code_i = sum over k = 0..n-1 of [x_i - z >= (k + 1/2) s]
 * with the subtraction exact (fp64), all 0 when s == 0; dequantized value
 * z + code_i * s.  bits = 2 is the paper's main setting (INT2, Sec. 3.1), bits = 4 its
 * higher-precision variant (Sec. 3.2.1, Table 3).  Key groups: one channel, G consecutive
 * quantized slots (G tokens evicted together), the last group of a filtering event
 * shorter (W mod G tokens) when G does not divide W.  Value groups: one slot, G
 * consecutive channels, the last group shorter when G does not divide d.
 */
#ifndef LOGQUANT_H
#define LOGQUANT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LQ_OK = 0,
  LQ_ERR_NULL = 1,        /* a required pointer is null                              */
  LQ_ERR_SHAPE = 2,       /* inconsistent B/Hq/Hkv/d/fp_budget/group/q_capacity       */
  LQ_ERR_UNSUPPORTED = 3, /* valid in the paper but not built: bits not 2 or 4, G not in
                             {32,64,128}, d not in {64,96,128}, B*Hq > 65535           */
  LQ_ERR_CAPACITY = 4,    /* fp region or quantized region would overflow             */
  LQ_ERR_STATE = 5,       /* call not allowed in the cache's current state            */
  LQ_ERR_HIP = 6          /* the HIP runtime reported a launch error                  */
} lq_status;

typedef enum { LQ_F16 = 0, LQ_BF16 = 1 } lq_dtype;

/* Immutable problem description (HOST). */
typedef struct {
  int32_t B;           /* batch rows                                                   */
  int32_t Hq;          /* query heads; query head h reads kv head h / (Hq/Hkv)         */
  int32_t Hkv;         /* kv heads, Hq % Hkv == 0                                      */
  int32_t d;           /* head dimension, one of 64, 96, 128                           */
  int32_t fp_budget;   /* F = 2W: fp tokens left after a compress; fp capacity is 3W   */
  int32_t group;       /* G: quantization group size, 32/64/128                        */
  int32_t bits;        /* 2 or 4                                                       */
  int32_t dtype;       /* lq_dtype                                                     */
  int32_t q_capacity;  /* max quantized slots per sequence; multiple of WQ and of 64   */
} lq_config;

/* Cache state (HOST struct, DEVICE buffers; layouts above). */
typedef struct {
  void     *k_fp[2];     /* two copies: compress reads buffer `cur`, writes the other  */
  void     *v_fp[2];
  int32_t  *pos_fp[2];
  uint32_t *k_codes, *v_codes;
  void     *k_scale, *k_zero, *v_scale, *v_zero;
  int32_t  *pos_q;
  int32_t   cur;         /* which fp buffer is live (0 or 1)                           */
  int32_t   n_fp;        /* tokens in the fp region, 0..3W                             */
  int32_t   n_q;         /* slots in the quantized region, multiple of WQ              */
} lq_cache;

/* Byte sizes of every buffer of lq_cache for a given config (HOST out). */
typedef struct {
  size_t k_fp, v_fp, pos_fp;            /* each of the two copies                      */
  size_t k_codes, v_codes, k_meta, v_meta, pos_q; /* k_meta: k_scale and k_zero each   */
  size_t workspace;                     /* logquant_workspace_bytes                    */
} lq_sizes;

/* Sizes of the buffers the caller has to provide.  Pure host arithmetic.
 * Returns LQ_ERR_NULL / LQ_ERR_SHAPE / LQ_ERR_UNSUPPORTED for a bad config. */
lq_status logquant_sizes(const lq_config *cfg, lq_sizes *out);

/* Bytes of the scratch buffer `workspace` that compress and decode_attn take
 * (ticket counters and partial softmax states of the context splits); 0 for an
 * invalid config. */
size_t logquant_workspace_bytes(const lq_config *cfg);

/* Prepare a freshly allocated workspace: zero the ticket counters at its head.
 * Call once per workspace before its first use by logquant_decode_attn (and again
 * only if a launch that used it was torn down mid-flight); decode_attn leaves the
 * counters at zero.  A workspace serves one stream at a time. */
lq_status logquant_workspace_init(const lq_config *cfg, void *workspace, void *stream);

/* Algorithm 1, the append branch: store n_new new tokens per sequence in fp
 * slots n_fp .. n_fp+n_new-1 and record their absolute positions
 * n_fp + (n_q/WQ)*W .. (every token ever appended is either in the fp region or in
 * the quantized region, so the number of tokens held is the next position).
 *   k_new, v_new : DEVICE [B][Hkv][n_new][d] T, row-major.
 * Requires n_fp + n_new <= 3W (else LQ_ERR_CAPACITY).  On success n_fp += n_new.
 * The caller runs logquant_compress when n_fp reaches 3W. */
lq_status logquant_append(const lq_config *cfg, lq_cache *cache, const void *k_new,
                          const void *v_new, int32_t n_new, void *stream);

/* Algorithm 1, the filtering branch, plus the quantization of what it removes
 * (Fig. 6 caption; Sec. 2.3).  Requires n_fp == 3W (else LQ_ERR_STATE) and
 * n_q + WQ <= q_capacity (else LQ_ERR_CAPACITY).  For every sequence and kv head:
 *   - logical fp rows 1,3,..,2W-1 are quantized with the quantizer above and
 *     appended, in that order, as quantized slots n_q .. n_q+W-1 (codes, scales,
 *     zero-points, positions); slots n_q+W .. n_q+WQ-1 become padding;
 *   - logical rows 0,2,..,2W-2 followed by rows 2W..3W-1 become rows 0..2W-1 of
 *     the other fp buffer, which becomes the live one (cache->cur flips).
 * On success n_fp = 2W, n_q += WQ.  `workspace` is not used at present and may
 * be null.
 * Input contract: the rows being quantized are finite and |x| <= 65504 (always true
 * of an fp16 cache; a bf16 cache may hold larger values, whose scales and zero-points
 * would overflow the fp16 they are stored in - the call does not look at the data and
 * returns LQ_OK, and attention over such a group is then undefined). */
lq_status logquant_compress(const lq_config *cfg, lq_cache *cache, void *workspace,
                            void *stream);

/* Bulk prefill: the state that Algorithm 1 reaches after L calls of
 * logquant_append(.., 1) on an empty cache, with logquant_compress run each time the
 * list becomes full (3W rows), produced from the whole prompt in one launch.  The
 * result is bit-identical to that sequence of calls: the same rows stay at original
 * precision in the same logical order, the evicted rows of each filtering event are
 * quantized in the same groups (Sec. 2.5; Fig. 6 caption) and stored in the same
 * slots.
 *   k, v : DEVICE [B][Hkv][L][d] T, row-major (as for logquant_append with n_new = L).
 * Requires an empty cache (n_fp == n_q == 0, else LQ_ERR_STATE), L >= 1 (else
 * LQ_ERR_SHAPE) and E*WQ <= q_capacity for the E = 0 (L < 3W) or floor((L-3W)/W)+1
 * events (else LQ_ERR_CAPACITY).  On success n_q = E*WQ, n_fp = L - E*W, and the live fp
 * buffer is unchanged (cache->cur).
 * Input contract as for logquant_compress: finite values, |x| <= 65504. */
lq_status logquant_prefill(const lq_config *cfg, lq_cache *cache, const void *k, const void *v,
                           int32_t L, void *stream);

/* Algorithm 1 in closed form (pure host arithmetic, no config needed): the positions
 * that L appends with window W (filtering as soon as the list holds 3W rows) leave
 * in the original-precision list (logical order: pos_fp, *n_fp entries, fewer than
 * 3W) and hand to the quantizer (eviction order: pos_q, *n_q entries).  HOST arrays:
 * pos_fp needs room for min(L, 3W) ints, pos_q for max(0, L - 2W) ints; either may be
 * null to get only the counts.
 * Returns LQ_ERR_SHAPE for W < 1 or L < 0. */
lq_status logquant_prefill_positions(int32_t W, int32_t L, int32_t *pos_fp, int32_t *n_fp,
                                     int32_t *pos_q, int32_t *n_q);

/* Decode attention, Eq. 2 with Eq. 6's scaling, over the whole cache:
 *   out[b][h] = softmax_t( scale * q[b][h] . k_t ) applied to v_t,
 * t running over the n_fp original-precision rows and the dequantized rows of the
 * n_q quantized slots (padding slots excluded)
 * of kv head h / (Hq/Hkv); one softmax over both regions (Sec. 2.4).  The 2-bit
 * rows are dequantized in registers, never in memory.
 *   q   : DEVICE [B][Hq][d] T          out : DEVICE [B][Hq][d] T
 *   softmax_scale <= 0 selects 1/sqrt(d).
 *   workspace : DEVICE, logquant_workspace_bytes(cfg) bytes, prepared once with
 *               logquant_workspace_init; not shared between concurrent calls.
 * Requires n_fp + n_q >= 1 (else LQ_ERR_STATE).  The cache is not modified.
 * Finite inputs only; 8 |q_c s_c| (a query element times a key scale) is assumed to stay
 * below fp16 range (65504). */
lq_status logquant_decode_attn(const lq_config *cfg, const lq_cache *cache, const void *q,
                               float softmax_scale, void *out, void *workspace,
                               void *stream);

/* logquant_decode_attn for callers that cannot allocate device memory or hand over a
 * workspace (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same kernels, with the scratch that `workspace` provides (counters and
 * the partial results of the context splits) taken from a device array inside the
 * library, 12 MiB per GPU the library runs on, held until the process ends.  The call
 * allocates and frees nothing.  Same arguments, requirements and results as
 * logquant_decode_attn otherwise.
 * Limits: B*Hq <= 3640 (4 MiB of counters) and logquant_workspace_bytes(cfg) minus its
 * counter part <= 8 MiB; a larger config returns LQ_ERR_CAPACITY before anything is
 * launched.  All calls on one GPU share the one array: calls that overlap in time on
 * one GPU (two streams, two threads) race and give undefined results, and the first call
 * on a GPU also enqueues the one-off clearing of the counters on `stream`, so later calls
 * on other streams must be ordered after it. */
lq_status logquant_decode_attn_static(const lq_config *cfg, const lq_cache *cache, const void *q,
                                      float softmax_scale, void *out, void *stream);

/* One decode step in one launch: logquant_append of one new token per sequence
 * (Algorithm 1, the append branch) followed by logquant_decode_attn over the cache
 * including that token (Eq. 2; Sec. 2.4), with the same results as the two calls.
 *   k_new, v_new : DEVICE [B][Hkv][1][d] T      q, out, workspace: as for decode_attn.
 * Requires n_fp + 1 < 3W (else LQ_ERR_STATE): at the step that fills the window the
 * caller appends, runs logquant_compress and attends with the separate calls.
 * On success n_fp += 1. */
lq_status logquant_decode_step(const lq_config *cfg, lq_cache *cache, const void *k_new,
                               const void *v_new, const void *q, float softmax_scale, void *out,
                               void *workspace, void *stream);

/* Launch shape logquant_decode_attn would use for these counts (HOST out), so a
 * harness can report bytes per launch; pure host arithmetic.
 * The planner reads four environment variables, once per process, as overrides for
 * experiments and for the tests that force every kernel shape (unset or 0: the planner
 * decides; results do not depend on them beyond the order of the fp32 sums):
 *   LOGQUANT_ATTN_WPB      wavefronts per workgroup: 4, 8 or 12
 *   LOGQUANT_ATTN_SPLITS   context splits per (batch row, kv head, head group)
 *   LOGQUANT_ATTN_CUS      compute units to plan for (default 256)
 *   LOGQUANT_ATTN_DYNAMIC  0: static tile schedule (default 1: tiles drawn from pool
 *                          counters when a wavefront has five or more) */
typedef struct {
  int32_t blocks;           /* workgroups of the attention kernel                    */
  int32_t waves_per_block;
  int32_t splits;           /* context splits per (batch row, kv head)               */
  int32_t fp_waves;         /* of splits*waves_per_block waves, those on the fp rows */
  int64_t bytes_read;       /* cache bytes one call must read (codes, scales,
                               zero-points, fp rows of live slots)                   */
} lq_plan;
lq_status logquant_decode_plan(const lq_config *cfg, int32_t n_fp, int32_t n_q, lq_plan *out);

/* ---- Per-sequence lengths ---------------------------------------------------------
 * Algorithm 1 runs per sequence (Sec. 2.5): in a batch whose sequences have different
 * lengths every sequence fills its window, and runs its filtering events, at its own
 * pace.  The calls below are the ones above with the counts kept per batch row.  The
 * device buffers and their layouts are those of lq_cache (one q_capacity and one fp
 * capacity for all rows); cur, n_fp and n_q are HOST arrays of B entries, owned by the
 * caller and updated by the calls; seq_state is DEVICE scratch of
 * logquant_seq_state_bytes(cfg) bytes through which each call hands the counts to its
 * kernels (written by every call, so it carries nothing between calls; a cache serves
 * one stream at a time).  Errors are detected before anything is launched or changed. */
typedef struct {
  void     *k_fp[2];
  void     *v_fp[2];
  int32_t  *pos_fp[2];
  uint32_t *k_codes, *v_codes;
  void     *k_scale, *k_zero, *v_scale, *v_zero;
  int32_t  *pos_q;
  int32_t  *cur;         /* HOST [B]: which fp buffer of row b is live                  */
  int32_t  *n_fp;        /* HOST [B]: tokens in row b's fp region, 0..3W                */
  int32_t  *n_q;         /* HOST [B]: slots in row b's quantized region, multiple of WQ */
  void     *seq_state;   /* DEVICE scratch, logquant_seq_state_bytes(cfg) bytes         */
} lq_cache_seq;

size_t logquant_seq_state_bytes(const lq_config *cfg);   /* 0 for an invalid config */

/* logquant_prefill with one prompt length per row: L is a HOST array of B lengths,
 * 0 <= L[b] <= L_stride (else LQ_ERR_SHAPE); k, v : DEVICE [B][Hkv][L_stride][d] T, of which
 * row b's first L[b] tokens are read.  Requires every row empty (else LQ_ERR_STATE). */
lq_status logquant_prefill_seq(const lq_config *cfg, lq_cache_seq *cache, const void *k,
                               const void *v, const int32_t *L, int32_t L_stride, void *stream);

/* logquant_append of one token for every row b with active[b] != 0 (HOST array of B
 * entries; null: all rows).  k_new, v_new : DEVICE [B][Hkv][1][d] T (rows that sit out are
 * not read).  Requires n_fp[b] + 1 <= 3W for the active rows (else LQ_ERR_CAPACITY). */
lq_status logquant_append_seq(const lq_config *cfg, lq_cache_seq *cache, const void *k_new,
                              const void *v_new, const int32_t *active, void *stream);

/* logquant_compress for every row whose n_fp == 3W, in one launch (no such row: nothing
 * is launched, LQ_OK).  LQ_ERR_CAPACITY if one of them has no room for the event. */
lq_status logquant_compress_seq(const lq_config *cfg, lq_cache_seq *cache, void *stream);

/* logquant_decode_attn / logquant_decode_step with per-row counts.  Every row needs at
 * least one token (else LQ_ERR_STATE); decode_step requires n_fp[b] + 1 < 3W for every
 * row (else LQ_ERR_STATE: append, compress and attend with the separate calls). */
lq_status logquant_decode_attn_seq(const lq_config *cfg, const lq_cache_seq *cache, const void *q,
                                   float softmax_scale, void *out, void *workspace, void *stream);
lq_status logquant_decode_step_seq(const lq_config *cfg, lq_cache_seq *cache, const void *k_new,
                                   const void *v_new, const void *q, float softmax_scale, void *out,
                                   void *workspace, void *stream);
/* Launch shape for per-row counts (HOST arrays of B entries): planned for the longest row,
 * bytes_read summed over the rows; fp_waves is the longest row's share. */
lq_status logquant_decode_plan_seq(const lq_config *cfg, const int32_t *n_fp, const int32_t *n_q,
                                   lq_plan *out);

/* Measurement helper (not a step of the method): one streaming read of `bytes` bytes of
 * DEVICE memory at `buf` (16-byte aligned, bytes >= 16; a tail of bytes % 16 is not read),
 * enqueued on `stream`.  `sink`: DEVICE, 8192 uint32 words the kernel folds what it read
 * into (so that the reads cannot be optimised away).  The benchmark uses it to report what
 * plain reading reaches for the byte count of one decode-attention launch (the HBM roofline
 * of Sec. 3.2.4's memory-bound decode step, measured rather than nominal). */
lq_status logquant_read_probe(const void *buf, size_t bytes, void *sink, void *stream);

const char *logquant_status_string(lq_status s);

#ifdef __cplusplus
}
#endif
#endif /* LOGQUANT_H */
