/*
 * tokenscale.h -- C ABI of the MI355X mixed paged-attention library.
 *
 * The library implements the GPU work a Convertible Decoder performs in one serving iteration
 * (paper Sec. 3.4, Sec. 4.4): a decode batch (one query token per sequence) runs next to
 * absorbed chunked-prefill requests (many query tokens, causal, attending to their cached
 * prefix), in one attention pass over a paged KV cache that also stores the iteration's new
 * K/V (Sec. 2.1: prefill builds the cache for all input tokens, each decode iteration adds the
 * last token's entry).  Token Velocity -- tokens an instance releases per second (Sec. 3.2) --
 * is kept per context as host-side counters.
 *
 * Conventions
 *   - Pointers marked DEV are device memory of the context's GPU, HOST are host memory.
 *     The caller owns every buffer and the stream; the library owns only its scratch.
 *   - GPU calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and never synchronise the device, except when scratch has to grow (see
 *     ts_reserve).  A context's calls may move from one stream to another: the first call
 *     on the new stream waits (on the device) for the context's previous call; calls that
 *     overlap in time on two streams need two contexts.
 *   - HOST arrays are consumed before the call returns.
 *   - Return value 0 = TS_OK, negative = error; ts_last_error() gives the text.  Everything
 *     that can be checked from host data is checked before any launch: a failing call has no
 *     side effect on device memory.  Page ids inside block_table are device data and are not
 *     validated: ids outside [0,num_pages) are undefined behaviour.
 *
 * Batch description (shared by the GPU calls)
 *   S = num_seqs sequences.  Sequence s brings q_lens[s] >= 0 new tokens and, once they are
 *   appended, holds ctx_lens[s] >= q_lens[s] tokens; prefix_s = ctx_lens[s] - q_lens[s] tokens
 *   are already cached.  New token i of sequence s has position prefix_s + i and sees keys
 *   0 .. prefix_s + i (causal).  q_lens[s] == 1 is a decode row, > 1 a prefill chunk, 0 is
 *   skipped.  Tokens are packed by sequence: row index = sum of q_lens of earlier sequences + i;
 *   T = sum of q_lens.
 *   block_table[s][j] (int32, row stride max_pages_per_seq) is the physical page holding
 *   positions 16j .. 16j+15 of sequence s; entries past ceil(ctx_lens[s]/16) are ignored.
 *   Two sequences must not append into the same physical page in one call.
 *
 * Cache layout (per cache, K and V are separate buffers of ts_cache_bytes() bytes)
 *   tiles ordered [page][kv_head]; with x = 16 bytes / element size (4 f32, 8 bf16, 16 fp8):
 *     K tile: element (slot, dim) at  (dim / x) * 16 * x + slot * x + dim % x
 *     V tile: element (slot, dim) at  dim * 16 + slot
 *   i.e. K keeps 16-byte dim-chunks of the 16 tokens together, V is stored token-fastest.
 *   Both are the operand order of the matrix instructions that consume them, so every load of
 *   the attention kernels is a full, aligned 16-byte (or 8-byte) vector of one tile.
 *   fp8 caches hold OCP e4m3 (bias 7, max 448, no inf) of value / scale[kv_head], the division
 *   in IEEE single precision, rounded to nearest-even, saturating to +-448, NaN kept.
 */
#ifndef TOKENSCALE_H
#define TOKENSCALE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TS_PAGE_SIZE 16

typedef struct ts_ctx ts_ctx;

typedef enum { TS_F32 = 0, TS_BF16 = 1, TS_FP8_E4M3 = 2 } ts_dtype;

enum { TS_MIXED_SEPARATE = 0, TS_MIXED_ONE_KERNEL = 1, TS_MIXED_CORESIDENT = 2 };   /* option "mixed_mode" */

enum {
    TS_OK = 0,
    TS_ERR_INVALID_ARG = -1,  /* null pointer, bad length, bad descriptor                  */
    TS_ERR_UNSUPPORTED = -2,  /* valid but not implemented combination                     */
    TS_ERR_HIP = -3,          /* a HIP runtime call failed (text in ts_last_error)          */
    TS_ERR_NOMEM = -4         /* scratch allocation failed                                  */
};

/* Geometry of one attention layer; fixed for the lifetime of a context.
 * Supported: head_dim 64 or 128; num_q_heads a multiple of num_kv_heads with a group size
 * <= 16; page_size 16; (q_dtype, kv_dtype) in {(F32,F32), (BF16,BF16), (BF16,FP8_E4M3)}. */
typedef struct {
    int32_t num_q_heads, num_kv_heads, head_dim;
    int32_t page_size;
    int32_t q_dtype, kv_dtype;        /* ts_dtype */
    int64_t num_pages;                /* size of the physical page pool */
    int32_t max_pages_per_seq;        /* row stride of block_table */
} ts_attn_desc;

/* Host only.  TS_OK if the descriptor is supported, else the error code. */
int ts_check_desc(const ts_attn_desc *desc);

/* Host only.  Bytes of ONE cache buffer (K or V) for this descriptor, 0 if it is invalid. */
int64_t ts_cache_bytes(const ts_attn_desc *desc);

/* Creates a context on GPU `device` (made current for the calling thread during the call).
 * Allocates an initial scratch and the pinned staging ring (4 x 1 MiB) for the work lists. */
int ts_create(const ts_attn_desc *desc, int device, ts_ctx **out);
int ts_destroy(ts_ctx *ctx);

/* Pre-sizes scratch for batches of up to max_tokens query tokens, max_seqs sequences and
 * max_ctx_pages cache pages in total over the batch (sum over sequences of ceil(ctx/16)), so
 * that later GPU calls with batches inside these limits never allocate.  The sizes follow the
 * options in force at the call ("decode_split_pages", "xcd_count"): set those first, or call
 * ts_reserve again after changing them.  Without it scratch grows on demand, which synchronises
 * the device once per growth. */
int ts_reserve(ts_ctx *ctx, int64_t max_tokens, int64_t max_seqs, int64_t max_ctx_pages);

/* Step a1 -- store the new K/V rows into the paged cache (Sec. 2.1).
 *   k_new, v_new : DEV [T, Hkv, D] of q_dtype, packed by sequence
 *   k_cache, v_cache : DEV, layout above, kv_dtype; written in place
 *   k_scale, v_scale : DEV fp32 [Hkv], FP8 caches only (else may be NULL)
 *   block_table : DEV int32 [S, max_pages_per_seq]
 *   q_lens, ctx_lens : HOST int32 [S]
 * Errors: TS_ERR_INVALID_ARG for null pointers, q_len < 0, ctx_len < q_len,
 * ctx_len > 16 * max_pages_per_seq, num_seqs < 0. */
int ts_kv_append(ts_ctx *ctx, void *stream,
                 const void *k_new, const void *v_new,
                 void *k_cache, void *v_cache,
                 const float *k_scale, const float *v_scale,
                 const int32_t *block_table,
                 const int32_t *q_lens, const int32_t *ctx_lens, int num_seqs);

/* Steps a1..a5 -- one pass of a Convertible Decoder iteration (Sec. 3.4, 4.4): optional
 * append, then softmax attention for every query token of every sequence,
 *   out[row, h, :] = sum_j w_j V_j,  w = softmax_j( sm_scale * <q[row,h,:], K_j> ),
 * over the keys the row sees, K/V taken from the cache through KV head h / (Hq/Hkv); fp8
 * elements are multiplied by their head's scale.
 *   q   : DEV [T, Hq, D] q_dtype        out : DEV [T, Hq, D] q_dtype (nearest-even cast)
 *   k_new, v_new : DEV [T, Hkv, D], or both NULL when the new tokens are already cached
 *   sm_scale : softmax scale, <= 0 selects 1/sqrt(head_dim)
 * Decode rows run as split-K items over the sequence's pages, prefill chunks as causal MFMA
 * tiles; partial results are merged in a fixed order, so results are run-to-run identical.
 * Also adds the batch's token counts to the context's velocity counters. */
int ts_mixed_paged_attention(ts_ctx *ctx, void *stream,
                             const void *q,
                             const void *k_new, const void *v_new,
                             void *k_cache, void *v_cache,
                             const float *k_scale, const float *v_scale,
                             const int32_t *block_table,
                             const int32_t *q_lens, const int32_t *ctx_lens, int num_seqs,
                             float sm_scale,
                             void *out);

/* The same pass for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels, same results as
 * ts_mixed_paged_attention, but all device scratch of the call (work lists, split-K partial results,
 * queue heads of the persistent launch) lives in a static device array of 8 MiB that the library
 * holds on every GPU it runs on until the process ends, and the call makes no device, pinned-host or
 * event allocation and frees nothing (the planner's host-side lists use the ordinary heap).
 * Limits: the batch's work lists must fit 1 MiB - 4 KiB and its split decode rows
 * 7 MiB / (Hq * (D + 2) * 4) partial results (220 for 64 query heads of 128 dims); beyond either the call fails
 * with TS_ERR_UNSUPPORTED before anything is launched, and ts_last_error names the size.  The
 * "kernel_timing" option is ignored, "validate_block_table" is refused (TS_ERR_UNSUPPORTED).
 * The array is shared by every context and call on that GPU and keeps the last call's contents (the
 * call itself puts back to zero what must start at zero): calls that overlap in time on one GPU,
 * from any contexts or streams, race.  Calls on one context are ordered as for the other entry
 * points. */
int ts_mixed_paged_attention_noalloc(ts_ctx *ctx, void *stream,
                                     const void *q,
                                     const void *k_new, const void *v_new,
                                     void *k_cache, void *v_cache,
                                     const float *k_scale, const float *v_scale,
                                     const int32_t *block_table,
                                     const int32_t *q_lens, const int32_t *ctx_lens, int num_seqs,
                                     float sm_scale,
                                     void *out);

/* Step a6 -- Token Velocity of this context (Sec. 3.2): tokens released per second, separately
 * for prefill chunks (rows of sequences with q_len > 1) and decode rows (q_len == 1), over the
 * window that started at the first pass after the last reset. */
typedef struct {
    double prefill_tok_per_s, decode_tok_per_s;
    uint64_t prefill_tokens, decode_tokens;
    uint64_t passes;
    double window_s;
} ts_velocity;

#define TS_VELOCITY_RESET 1   /* start a new window after reporting                         */
#define TS_VELOCITY_SYNC  2   /* wait for the context's last call to finish on the GPU before
                                 reading the clock (otherwise the call touches no GPU state).
                                 It orders nothing but the clock: to read `out` on the host,
                                 synchronise the stream as usual                            */
int ts_token_velocity(ts_ctx *ctx, ts_velocity *out, int flags);

/* Text of the last error of this context ("" if none); valid until the next call on it.
 * With ctx == NULL: the last error of a failed ts_create on this thread. */
const char *ts_last_error(const ts_ctx *ctx);

/* Tuning knobs (all optional).  Names:
 *   "decode_split_pages"  longest page range of one decode item (0 = choose from the batch)
 *   "decode_merge_in_kernel"  0 (default) = a decode row cut into several items is merged by a small launch behind
 *                         the decode items; 1 = by whichever of its items finishes last (arrival counters,
 *                         device-scope release/acquire around the partial results; the merge reads the partials
 *                         in item order, so the result does not depend on which item came last).  The second
 *                         form saves a launch and is slower on this GPU (the release writes the L2 back)
 *   "decode_fused_append"  1 (default) / 0.  A pass that appends, holds decode rows only and is small (at most 64
 *                         decode items and 32 split rows: its work lists travel as kernel arguments) leaves
 *                         the append to the decode items: the workgroup that reads a row's last page takes the
 *                         new token from k_new / v_new, converts it exactly as the append kernels do, and
 *                         writes its cache entry; the pass has no append launch and no upload of work lists.
 *                         Such passes are bound by their launches.  Same results and same cache bytes either
 *                         way.  (Not with validate_block_table.)
 *   "prefill_path"        0 = MFMA tiles where supported, 1 = force the generic row kernel
 *   "decode_prefetch_tiles"  2..4 KV tiles in flight per decode wave
 *   "mixed_mode"          how a batch that holds decode rows and prefill chunks is launched:
 *                         2 (default, TS_MIXED_CORESIDENT) = the prefill tiles run in resident workgroups,
 *                         at most one per CU, that leave room on their CU for one decode workgroup, and the
 *                         decode items run next to them as a grid of their own on an internal side stream
 *                         (forked from and joined to the caller's stream with events).  A batch in which
 *                         either class is short (estimated below 20 us) takes mode 0 by itself: the fork
 *                         and join would cost more than running side by side hides.
 *                         The side stream is an ordinary stream of the process: where the runtime maps it
 *                         to the hardware queue that also serves the caller's stream (a process has 4 by
 *                         default), the two launches run in turn -- same results, no overlap.  The first
 *                         co-resident call of a context therefore sends a probe ahead (two one-thread
 *                         kernels, at most 60 us, never under stream capture and never in the
 *                         allocation-free entry point); a later call reads its answer without waiting and,
 *                         if the streams ran in turn, replaces the side stream and probes again, up to 4
 *                         times (read-only options "side_stream_overlap": 0 = no answer yet, 1 = side by
 *                         side, 2 = in turn; "side_stream_probes": probes answered).  The probe is made
 *                         against the stream of that call;
 *                         1 (TS_MIXED_ONE_KERNEL) = decode items and prefill tiles share the workgroups of one
 *                         persistent launch;  0 (TS_MIXED_SEPARATE) = decode kernel, then prefill kernel
 *   "prefill_resident_workgroups"  co-resident launch: number of resident prefill workgroups.  0 (default) =
 *                         chosen per batch from the estimated times of its tiles and of its decode scan: all
 *                         CUs when the tiles dominate, fewer (in multiples of the die count) when the scan
 *                         outlasts them, so that the remaining CUs hold decode workgroups only.  A value > 0
 *                         fixes the number (capped at the CU count) and keeps mode 2 for every mixed batch
 *   "prefill_split_min_keys"  a batch whose prefill tiles cannot give every CU a workgroup (a short chunk over a
 *                         long prefix) has its tiles cut along the keys, below their first query position, into
 *                         parts of at least this many keys (multiple of 64, default 512; 0 = never); the
 *                         parts' partial results are merged in part order by a small launch
 *   "prefill_widen_pages" fp8 caches: every tile of a prefill chunk reads the chunk's whole prefix, so the pages
 *                         of the chunks' sequences are widened from e4m3 to bf16 once per pass, into scratch of
 *                         8 KiB * num_kv_heads per page, and the tiles read that copy; a batch whose chunk
 *                         sequences hold more pages than this value (default 16384; 0 = never widen) has its
 *                         tiles widen the cache themselves.  Results are identical either way
 *   "xcd_count"           accelerator dies the prefill launch order is laid out for (default 8)
 *   "kernel_timing"       N > 0 = record HIP events around the launches of every N-th call
 *                         (see ts_kernel_times), 0 = off
 *   "validate_block_table"  debug aid, 0 (default) / 1: the GPU calls first check, on the GPU, that
 *                         every page id the batch uses lies in [0, num_pages), wait for the answer
 *                         (the call is then synchronous) and fail with TS_ERR_INVALID_ARG, caches
 *                         untouched, if one does not
 * Unknown names give TS_ERR_INVALID_ARG. */
int ts_set_option(ts_ctx *ctx, const char *name, int64_t value);

/* Reads an option back (same names as ts_set_option), and the read-only counter
 *   "scratch_allocations"  device and pinned-host allocations this context has made so far
 * (creation and ts_reserve included): a serving loop that must not allocate reads it before and
 * after its calls. */
int ts_get_option(const ts_ctx *ctx, const char *name, int64_t *value);

/* Measurement aid, not a step of the pass: optional per-kernel timing with HIP events recorded on the caller's stream around each launch
 * (enable with ts_set_option(ctx, "kernel_timing", N): every N-th call is timed; two event records
 * per timed launch, each of which idles the GPU for a few microseconds).
 * ts_kernel_times waits for the recorded events, then reports, per kernel, the number of timed
 * launches and their mean duration in milliseconds since the last reset. */
enum { TS_K_APPEND = 0, TS_K_DECODE = 1, TS_K_COMBINE = 2, TS_K_PREFILL = 3, TS_K_ROWS = 4, TS_K_MIXED = 5,
       TS_K_COUNT = 6 };
typedef struct {
    uint64_t launches[TS_K_COUNT];
    double mean_ms[TS_K_COUNT];
} ts_kernel_stats;
int ts_kernel_times(ts_ctx *ctx, ts_kernel_stats *out, int reset);

/* Host only -- step a0.  Describes the work the planner makes of a batch, without touching a
 * GPU: how many decode split items, combine rows, prefill tiles and generic rows.
 * split_pages = 0 lets the planner choose. */
typedef struct {
    int64_t total_tokens, decode_tokens, prefill_tokens;
    int32_t n_decode_items;     /* (row, page range) split-K items, each run for every KV head */
    int32_t n_combine_rows;     /* decode rows that were split and need merging                */
    int32_t n_prefill_tiles;    /* causal query tiles, each run for every KV head              */
    int32_t n_generic_rows;     /* rows sent to the generic row kernel                         */
    int32_t split_pages;        /* pages per decode item actually used                         */
    int32_t tile_tokens;        /* query tokens per prefill tile                               */
    int64_t partial_slots;      /* split-K partial results held in scratch                     */
    int64_t ctx_pages;          /* sum over sequences of ceil(ctx_len/16)                      */
    int32_t mixed_mode;         /* TS_MIXED_* the batch is launched with (SEPARATE if one kind only) */
    int32_t prefill_workgroups; /* co-resident launch: resident workgroups that work through the prefill tiles (else 0) */
    int64_t widened_pages;      /* fp8 caches: pages widened to bf16 before the prefill tiles run   */
    int64_t prefill_parts;      /* partial results of prefill tiles cut along the keys (0 = none cut) */
} ts_plan_info;

int ts_plan_describe(const ts_attn_desc *desc, const int32_t *q_lens, const int32_t *ctx_lens,
                     int num_seqs, int32_t split_pages, ts_plan_info *out);

/* Host only.  Copies one of the planner's work lists as flat int32 records into out (capacity in
 * int32 words); returns the number of records, or a negative error.  Lists and record layouts:
 *   TS_LIST_DECODE  (row, seq, n_keys, page_begin, page_end, partial_slot or -1, 0, 0)
 *   TS_LIST_COMBINE (row, partial_begin, n_split, 0)
 *   TS_LIST_PREFILL (seq, row0, q_len, prefix, tok_begin, tok_count, ctx_len, part or -1, kv_begin, kv_end, 0, 0)
 *                   one causal tile, or one part [kv_begin, kv_end) of a tile cut along the keys
 *   TS_LIST_PFCOMBINE (prefill item of the tile, first part, parts, 0)   cut tiles to merge
 *   TS_LIST_PFMAP   (prefill tile or -1, kv_head)       launch order, workgroup i -> die i % 8
 *   TS_LIST_ROWS    (row, seq, n_keys, 0)
 *   TS_LIST_QUEUE   (kind 0 decode / 1 prefill, item, kv_head, 0)   per-die queues, concatenated (mode 1: both
 *                   kinds interleaved; mode 2: the tiles only)
 *   TS_LIST_QOFF    (offset)                                        n_dies + 1 offsets into the queue
 *   TS_LIST_APPEND  (seq, page_index, slot_lo, slot_hi, row_of_slot_0, 0, 0, 0)   page-wise append work
 *   TS_LIST_APPEND_ROWS (row, seq, pos, 0)                          tokens appended one by one
 *   TS_LIST_WIDEN   (seq, page_index)                               fp8 caches: pages widened to bf16 per pass
 * wg_slots = 0 uses the default number of resident decode workgroups; mixed_mode = TS_MIXED_* as for the
 * option of that name, or -1 for the default. */
enum { TS_LIST_DECODE = 0, TS_LIST_COMBINE = 1, TS_LIST_PREFILL = 2, TS_LIST_PFMAP = 3, TS_LIST_ROWS = 4,
       TS_LIST_QUEUE = 5, TS_LIST_QOFF = 6, TS_LIST_APPEND = 7,
       TS_LIST_APPEND_ROWS = 8, TS_LIST_WIDEN = 9, TS_LIST_PFCOMBINE = 10 };
int64_t ts_plan_export(const ts_attn_desc *desc, const int32_t *q_lens, const int32_t *ctx_lens,
                       int num_seqs, int32_t split_pages, int32_t wg_slots, int32_t mixed_mode, int which,
                       int32_t *out, int64_t capacity);

#ifdef __cplusplus
}
#endif
#endif /* TOKENSCALE_H */
