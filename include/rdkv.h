/*
 * rdkv.h -- C ABI of librdkv: decode attention read directly from a
 * rate-distortion-compressed KV cache, and the one-shot post-prefill
 * compression pass that builds that cache, for AMD MI355X (gfx950).
 *
 * Method: "RDKV: Rate-Distortion Bit Allocation for Joint Eviction and
 * Quantization of the KV Cache" (arxiv 2605.08317).  Section / equation /
 * algorithm numbers below refer to that paper.
 *
 * General rules
 *  - Every pointer argument says whether it is HOST or DEVICE memory.  Device
 *    buffers are owned by the caller unless stated otherwise and must stay valid
 *    until the stream has executed the call's work.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue their work on it and return without waiting for it, with these
 *    exceptions, each stated again at its declaration: rdkv_pack and rdkv_compress
 *    wait once (the tier counts size the arena and the split schedule, so they are
 *    read back); rdkv_cache_reserve_tail and rdkv_cache_rebudget_tail (they replace
 *    the schedule), rdkv_calibrate_eps, rdkv_cache_stats and rdkv_cache_export
 *    (host results) wait for the stream.  rdkv_weights, rdkv_allocate,
 *    rdkv_decode_attn, rdkv_decode_attn_bf16 and rdkv_cache_append never wait.
 *  - Every function returns an rdkv_status and never throws or aborts; host-side
 *    arguments are validated before anything is launched (what only the device can
 *    see -- the values inside a device bit map -- is reported after the one wait of
 *    rdkv_pack, before anything is packed); on failure `*out` handles are left NULL
 *    and rdkv_last_error() holds a message (thread local).
 *  - Scratch memory of a call is released when the call returns, while its kernels
 *    may still be queued.  The allocator hooks of rdkv_config must therefore behave
 *    like a stream-ordered caching allocator used on the call's stream (memory
 *    given back may be handed out again only to work enqueued later on that stream,
 *    or after that stream has drained; PyTorch's caching allocator does this).
 *    Without hooks, scratch comes from hipMallocAsync / hipFreeAsync on the call's
 *    stream and what a cache owns from hipMalloc / hipFree.
 *  - Shapes: head_dim must be 128, hq a multiple of hkv with hq/hkv in
 *    {1,2,4,8}, quantization group size 32 or 128.
 *  - Ragged batch layout: K, V (and per-token arrays) hold, per sequence s in
 *    batch order, a block [hkv][T_s][head_dim] (resp. [hkv][T_s]); blocks are
 *    concatenated without padding.  One "item" is one (sequence, KV head), item
 *    index = s*hkv + h.  Query head j reads KV head j / (hq/hkv).
 */
#ifndef RDKV_H
#define RDKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rdkv_cache rdkv_cache; /* opaque; created by rdkv_pack / rdkv_compress */

typedef enum {
  RDKV_OK = 0,
  RDKV_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad enum */
  RDKV_ERR_SHAPE = 2,       /* unsupported or inconsistent shape */
  RDKV_ERR_UNSUPPORTED = 3, /* valid request this build does not implement */
  RDKV_ERR_ALLOC = 4,       /* device or host allocation failed */
  RDKV_ERR_HIP = 5,         /* a HIP runtime call failed */
  RDKV_ERR_INTERNAL = 6
} rdkv_status;

enum { RDKV_K_TOKENWISE = 0, RDKV_K_CHANNELWISE = 1 };
enum { RDKV_MAX_TIERS = 5 };

/* Device allocator hooks (e.g. a framework's caching allocator). */
typedef void* (*rdkv_alloc_fn)(size_t bytes, void* user);
typedef void (*rdkv_free_fn)(void* ptr, void* user);

/*
 * Problem statement of Sec. 3 and the inputs of Alg. 1, as one POD struct.
 * Fill with rdkv_config_default() and override fields.
 */
typedef struct rdkv_config {
  int32_t batch;            /* number of sequences */
  int32_t hq, hkv;          /* query heads, KV heads (GQA group g = hq/hkv) */
  int32_t head_dim;         /* d; must be 128 */
  const int32_t* seq_lens;  /* HOST [batch]: prefill length T_s of each sequence, T_s >= s_obs */
  int32_t s_obs;            /* observation window S_w (App. B: 32) */
  int32_t pool_kernel;      /* AvgPool1d kernel w (App. B: 5); odd; 1 disables pooling */
  int32_t causal;           /* 1: window row i attends keys t <= T - s_obs + i */
  int32_t k_mode;           /* RDKV_K_TOKENWISE: K rows share the token bit map;
                               RDKV_K_CHANNELWISE: Sec. 3.2 Stage 3 (per-channel K on kept tokens) */
  int32_t group_size;       /* channels of a token row that share a scale and offset: 32 (default), or 128 = one per
                               token row, the per-token format of App. B (V rows; K rows too in token-wise mode).  The
                               stored row keeps its four metadata slots, each repeating the row's scale and offset, so
                               both formats take the same bytes and the same decode kernels */
  const float* budget_bits; /* HOST [batch]: average bits per cache element for each sequence */
  float kv_split_rk;        /* r_K: share of the bit budget given to K in channel-wise mode (0.5) */
  int32_t k_scale_per_channel; /* channel-wise mode: 0 (default) = a scale and zero-point per channel and group of 32
                               retained tokens; 1 = one per channel over all retained tokens of the (sequence, KV
                               head), the format of App. B (the scaled query is then formed once per decode step) */
  int32_t n_tiers;          /* number of entries of tiers[] (<= 5) */
  int32_t tiers[RDKV_MAX_TIERS];   /* ascending bit-widths out of {0,2,4,8,16} (Sec. 3: B) */
  float eps_v[RDKV_MAX_TIERS];     /* distortion table eps_V(b) aligned with tiers[] (Eq. 6, Table 9) */
  float eps_k[RDKV_MAX_TIERS];     /* distortion table eps_K(b) */
  float rel_tol;            /* bisection tolerance delta (App. B: 1e-2) */
  int32_t max_iters;        /* bisection steps I (App. B: 64) */
  rdkv_alloc_fn alloc;      /* NULL: hipMalloc */
  rdkv_free_fn free_;       /* NULL: hipFree */
  void* alloc_user;
} rdkv_config;

/* Summary of a packed cache (all HOST values). */
typedef struct rdkv_stats {
  int64_t n_items;          /* batch * hkv */
  int64_t rows[4];          /* kept tokens per tier, order 16, 8, 4, 2, summed over items */
  int64_t evicted;          /* tokens at 0 bits, summed over items */
  int64_t stored_bytes;     /* bytes a decode step must read: codes + scale/offset metadata, unpadded
                               (channel-wise mode: K codes n * sum_c b_c / 8 and 4 bytes per quantized channel
                               and group of 32 retained tokens, V rows as in token-wise mode) */
  int64_t arena_bytes;      /* bytes allocated for the packed arena (with padding and alignment) */
  int64_t index_bytes;      /* what else the cache's block holds: kept-position lists, bit maps, split schedule, the
                               first split workspace */
  int64_t n_chunks;         /* work items of one decode launch */
  int64_t dense_bytes;      /* 2 * sum_s hkv*T_s*head_dim*2: the uncompressed bf16 K+V */
  int64_t alloc_info;       /* 1 if the cache came from rdkv_compress, so that the fields below are known; else 0 */
  int64_t iterations_max;   /* Alg. 2: most bisection steps any item's token-map search took */
  double lambda_min;        /* Alg. 2: smallest and largest multiplier lambda* of the token-map searches that ran */
  double lambda_max;        /*   (NaN if none ran: budget shortcuts, or alloc_info == 0); per item: rdkv_cache_export */
} rdkv_stats;

/* What rdkv_cache_export copies out (all to HOST memory). */
enum {
  RDKV_EXPORT_COUNTS = 0,   /* int32 [items][4]: rows per tier (16, 8, 4, 2) */
  RDKV_EXPORT_TIER_IDX = 1, /* int32 [sum kept]: kept positions, item-major, tier order 16,8,4,2, ascending */
  RDKV_EXPORT_SEG_OFF = 2,  /* int64 [items][4 tiers][4]: arena byte offsets of K data, K meta, V data, V meta */
  RDKV_EXPORT_ARENA = 3,    /* uint8 [arena_bytes]: the physical packed buffers */
  RDKV_EXPORT_BITS_TOK = 4, /* uint8 [sum_s hkv*T_s]: token bit map */
  RDKV_EXPORT_BITS_CH = 5,  /* uint8 [items][head_dim]: K channel bit map (channel-wise mode) */
  RDKV_EXPORT_LAMBDA = 6,   /* double [items], channel-wise mode [2][items] (token maps, then channel maps): the
                               multiplier lambda of the allocation Alg. 2 returned; NaN where no search ran (the
                               all-16 / all-0 shortcuts, no feasible step).  Caches built by rdkv_compress only:
                               size 0 otherwise */
  RDKV_EXPORT_ITERATIONS = 7 /* int32, same shape: bisection steps taken (0 where no search ran) */
};

const char* rdkv_version(void);
const char* rdkv_last_error(void);

/* Defaults of App. B: S_w = 32, w = 5, causal, token-wise K, group 32, r_K = 0.5,
 * tiers {0,2,4,8,16}, the LLaMA-3.1-8B row of Table 9 (eps(0)=1, eps(16)=0),
 * delta = 1e-2, I = 64.  batch/heads/seq_lens/budget_bits are left zero. */
rdkv_status rdkv_config_default(rdkv_config* cfg);

/*
 * Stage 1 of Alg. 1 (Eq. 2, Eq. 4).
 *   K      DEVICE bf16, ragged [hkv][T_s][d] blocks
 *   Q_obs  DEVICE bf16 [batch][hq][s_obs][d]: the last s_obs prefill queries
 *   w_tok  DEVICE fp32 out, ragged [hkv][T_s]: pooled token weights
 *          w_t = AvgPool(sum over window rows and group heads of softmax(q k^T/sqrt d)_t)
 *   w_ch   DEVICE fp32 out [items][d] or NULL: channel weights
 *          w_c = ||Q_obs[:,c]||_2 ||K[:,c]||_2 / sqrt(d)
 */
rdkv_status rdkv_weights(const rdkv_config* cfg, const void* K, const void* Q_obs,
                         float* w_tok, float* w_ch, void* stream);

/*
 * Stages 2-3 of Alg. 1: the multiple-choice knapsack of Eq. 6 solved by the
 * Lagrangian bisection of Alg. 2, once per item.  The result never exceeds the
 * budget: sum_t bits <= floor(avg_bits * T).
 *   w_tok    DEVICE fp32 ragged [hkv][T_s]
 *   w_ch     DEVICE fp32 [items][d]; required in channel-wise mode, else ignored
 *   bits_tok DEVICE uint8 out, ragged [hkv][T_s]
 *   bits_ch  DEVICE uint8 out [items][d]; required in channel-wise mode, else ignored
 * Token-wise mode: every sequence's budget_bits is the average over K and V alike.
 * Channel-wise mode: V tokens get 2(1-r_K)*budget, then K channels get
 * min(16, 2 r_K budget T / n_kept) average bits over kept tokens.
 */
rdkv_status rdkv_allocate(const rdkv_config* cfg, const float* w_tok, const float* w_ch,
                          uint8_t* bits_tok, uint8_t* bits_ch, void* stream);
/* The same, also returning what Alg. 2 found per item: lambda_out DEVICE double [items] (channel-wise mode:
 * [2][items], token maps then channel maps): the multiplier of the returned allocation, NaN where no search ran;
 * iterations_out DEVICE int32, same shape: bisection steps taken.  Either may be NULL. */
rdkv_status rdkv_allocate_info(const rdkv_config* cfg, const float* w_tok, const float* w_ch,
                               uint8_t* bits_tok, uint8_t* bits_ch, double* lambda_out,
                               int32_t* iterations_out, void* stream);

/*
 * Stage 4 of Alg. 1: partition kept tokens by tier, quantize groups of 32 with an
 * fp16 scale and fp16 offset, bit-pack into per-tier segments, and build the
 * decode split schedule.  Bit maps may hold any mix of {0,2,4,8,16}.
 *   K, V     DEVICE bf16 ragged
 *   bits_tok DEVICE uint8 ragged [hkv][T_s]
 *   bits_ch  DEVICE uint8 [items][d] (channel-wise mode) or NULL
 *   out      HOST: receives the cache handle (library-owned; rdkv_cache_free)
 * Token-wise mode: a token's K row and V row are both stored at bits_tok (groups of 32
 * channels of the row).  Channel-wise mode (Sec. 3.2 Stage 3, App. B): bits_tok is the V
 * map and decides which tokens are retained; the K rows of the retained tokens are stored
 * channel by channel at bits_ch, channels sorted by bit-width, one scale and offset per
 * channel and per 32 consecutive retained tokens of a tier segment (per channel over all
 * retained tokens of the item when cfg->k_scale_per_channel is set); a channel at 0 bits is
 * dropped (it contributes nothing to q.k), a channel at 16 bits keeps its bf16 values.
 * Waits for the stream once (tier counts).  A value in bits_tok or bits_ch outside {0,2,4,8,16} gives
 * RDKV_ERR_INVALID_ARG (found on the device, reported after that wait; nothing has been packed then).
 */
rdkv_status rdkv_pack(const rdkv_config* cfg, const void* K, const void* V,
                      const uint8_t* bits_tok, const uint8_t* bits_ch, void* stream,
                      rdkv_cache** out);

/* The whole one-shot pass: rdkv_weights -> rdkv_allocate -> rdkv_pack (Alg. 1), with one wait for the stream (the
 * tier counts); the multipliers and step counts of Alg. 2 stay with the cache (rdkv_cache_stats / rdkv_cache_export). */
rdkv_status rdkv_compress(const rdkv_config* cfg, const void* K, const void* V,
                          const void* Q_obs, void* stream, rdkv_cache** out);

/*
 * A-priori bound, from the budget alone, on the bytes of the packed arena rdkv_pack / rdkv_compress will allocate
 * through cfg->alloc for this batch (Sec. 3.2: the summed bit-widths of an item never exceed floor(avg_bits * units),
 * so it keeps at most that over the lowest stored bit-width tokens): a caller can reserve memory for a cache before
 * the pass has run.  Needs batch, heads, seq_lens, budget_bits, k_mode, kv_split_rk and tiers; 0 on an invalid config.
 * The bound covers the arena (codes, scales, offsets, padding).  rdkv_pack takes one block through cfg->alloc that
 * holds the arena and the cache's tables (kept positions, bit maps, split schedule, the first split workspace);
 * rdkv_cache_max_table_bytes bounds those tables the same way, so the sum of the two bounds what that one allocation
 * can ask for (rdkv_stats: arena_bytes + index_bytes).
 */
size_t rdkv_cache_max_bytes(const rdkv_config* cfg);
size_t rdkv_cache_max_table_bytes(const rdkv_config* cfg);

/*
 * One decode step over the packed cache (Sec. 3.3, Eq. 7): for every sequence
 * and query head, softmax(q K_hat^T / sqrt d) V_hat over the retained tokens, the
 * tokens appended since (rdkv_cache_append) and the appended tokens compressed
 * later (rdkv_cache_rebudget_tail), dequantization fused into the attention kernel
 * (in channel-wise mode the per-channel scales are folded into the query, App. B).
 *   q    DEVICE bf16 [batch][hq][d]
 *   out  DEVICE fp32 [batch][hq][d]
 *   lse  DEVICE fp32 [batch][hq] or NULL: natural-log sum of exp of the logits
 * An item with no retained token gives out = 0, lse = -inf.  One launch (two when a token-wise cache holds 16-bit
 * rows): the workgroup that finishes an item's last chunk merges the item's split partials.  A cache keeps one
 * split workspace per stream it is decoded on, so steps on different streams may overlap (steps on one stream are
 * serialised by the stream).  The workspace of the stream that built the cache (or last rebuilt its schedule:
 * rdkv_cache_reserve_tail, rdkv_cache_rebudget_tail) exists from the start; the first step on any other stream
 * allocates that stream's workspace through the cache's allocator.  A step issued while its stream is under graph
 * capture allocates nothing and uses that first workspace whatever the stream: replays of such a graph must not
 * overlap each other, nor steps on the stream that built the cache.
 */
rdkv_status rdkv_decode_attn(const rdkv_cache* cache, const void* q, float* out, float* lse,
                             void* stream);

/*
 * The same decode step over an uncompressed bf16 cache (the full-cache baseline
 * of Sec. 4.2), for ratio comparisons.
 *   K, V          DEVICE bf16 ragged [hkv][T_s][d] blocks
 *   seq_lens      HOST [batch]
 *   workspace     DEVICE scratch of at least rdkv_decode_bf16_workspace_bytes()
 */
size_t rdkv_decode_bf16_workspace_bytes(const int32_t* seq_lens, int32_t batch, int32_t hq,
                                        int32_t hkv, int32_t head_dim);
rdkv_status rdkv_decode_attn_bf16(const void* K, const void* V, const int32_t* seq_lens,
                                  int32_t batch, int32_t hq, int32_t hkv, int32_t head_dim,
                                  const void* q, float* out, float* lse, void* workspace,
                                  size_t workspace_bytes, void* stream);

/*
 * rdkv_decode_attn_bf16 for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same step with the same kernels and arguments, minus the workspace.
 * The split partials live in a device array built into the library (rdkv_decode_bf16_noalloc_max_bytes() = 8 MiB on
 * every GPU the library runs on, held until the process ends).  The call allocates nothing.  A batch whose
 * rdkv_decode_bf16_workspace_bytes() exceeds that size is rejected with RDKV_ERR_UNSUPPORTED before anything is
 * launched.  All calls on one GPU share the one array: calls that overlap in time on the same GPU (different
 * streams, or threads) race on it -- issue them on one stream or serialise them.  Every partial slot the merge
 * reads is written by the split kernel of the same call, so the array needs no clearing between calls.
 */
size_t rdkv_decode_bf16_noalloc_max_bytes(void);
rdkv_status rdkv_decode_attn_bf16_noalloc(const void* K, const void* V, const int32_t* seq_lens, int32_t batch,
                                          int32_t hq, int32_t hkv, int32_t head_dim, const void* q, float* out,
                                          float* lse, void* stream);

/*
 * Measurement aid (benchmarks).  While enabled, the calls above bracket their
 * kernels with HIP events on the call's own stream: the decode launch of
 * rdkv_decode_attn (merge included), the split-K kernel of rdkv_decode_attn_bf16,
 * every kernel of rdkv_weights, every kernel of rdkv_allocate, and the kernels of
 * rdkv_pack in two brackets (tier counts before the call's one wait; position
 * lists, quantize and pack after it; the arena's clearing is not inside).
 * rdkv_kernel_timing_read waits for the recorded events, returns the number of
 * brackets of one kind and their summed duration in milliseconds, and clears that
 * kind.  Not for use under graph capture.
 */
enum {
  RDKV_TIME_DECODE_TIERED = 0,
  RDKV_TIME_DECODE_BF16 = 1,
  RDKV_TIME_WEIGHTS = 2,
  RDKV_TIME_ALLOCATE = 3,
  RDKV_TIME_PACK = 4,
  RDKV_TIME_CALIBRATE = 5,
  RDKV_TIME_KINDS = 6
};
rdkv_status rdkv_kernel_timing_enable(int32_t enable);
rdkv_status rdkv_kernel_timing_read(int32_t kind, int64_t* launches, double* total_ms);

/* Zone C of Sec. 3.3 (third term of Eq. 7): tokens generated after the compression pass stay uncompressed (the
 * paper keeps them in FP16; here their bf16 rows are kept verbatim) and rdkv_decode_attn attends to them together
 * with the compressed rows.
 *   rdkv_cache_reserve_tail  once per cache, before the first append: room for max_new_tokens rows per (sequence,
 *                            KV head), 512 bytes per row and item (in whole 64-token tiles), owned by the cache;
 *                            synchronises `stream`.
 *                            Error if max_new_tokens <= 0 or the tail is already reserved.
 *   rdkv_cache_append        one new token per sequence: k_new, v_new are DEVICE bf16 [batch][hkv][head_dim]; the
 *                            copy is enqueued on `stream` (decode calls on the same stream see it).  Error if no
 *                            tail is reserved or it is full; the cache is unchanged then.
 *   rdkv_cache_tail_len      tokens appended so far (0 for a null cache). */
rdkv_status rdkv_cache_reserve_tail(rdkv_cache* cache, int32_t max_new_tokens, void* stream);
rdkv_status rdkv_cache_append(rdkv_cache* cache, const void* k_new, const void* v_new, void* stream);
int32_t rdkv_cache_tail_len(const rdkv_cache* cache);
/* The number of appended tokens lives in a device word of the cache: the append kernel writes its row there and
 * advances it, the decode kernels read it.  A HIP graph that captured rdkv_cache_append followed by
 * rdkv_decode_attn can therefore be replayed token after token (new k_new / v_new / q contents in the same
 * buffers); a replay on a full tail appends nothing.  rdkv_cache_tail_len counts the rdkv_cache_append calls made
 * through the library (replays are not calls); rdkv_cache_tail_len_sync waits for `stream`, reads the device's
 * count, makes it the library's own and returns it in *out (may be NULL). */
rdkv_status rdkv_cache_tail_len_sync(rdkv_cache* cache, void* stream, int32_t* out);

/*
 * Streaming re-budgeting (the extension sketched in App. "Limitations and Future Work"): the appended tokens are
 * compressed by the same pass (Alg. 1) as a sequence of their own and join the compressed zones as one more
 * generation; the tail is empty afterwards and keeps its capacity.  Both cache modes; in channel-wise mode the
 * generation gets its own channel bit map and sorted-channel layout per (sequence, KV head).
 *   cfg     the pass's parameters for the tail: batch, hq, hkv, head_dim, k_mode and k_scale_per_channel as the
 *           cache; seq_lens[s] =
 *           rdkv_cache_tail_len(cache) for every s; budget_bits[s] = average bits per element of the tail of
 *           sequence s; s_obs <= tail length; tiers, distortion tables, tolerance as for rdkv_compress
 *   Q_obs   DEVICE bf16 [batch][hq][s_obs][d]: the decode queries of the last s_obs appended tokens (window row i
 *           sits at tail position n - s_obs + i; the probe's softmax runs over the tail's keys only)
 * Synchronises `stream`.  Replaces the decode schedule: HIP graphs that captured rdkv_decode_attn on this cache must
 * be captured again.  On error the cache is unchanged.
 *   rdkv_cache_generations   number of absorbed generations (0 for a null cache)
 *   rdkv_cache_generation    borrowed handle of generation `index` for rdkv_cache_stats / rdkv_cache_export (owned by
 *                            the cache; never free it); NULL if out of range
 * rdkv_cache_stats of the cache sums over its generations; rdkv_cache_export describes the prompt's zones only.
 */
rdkv_status rdkv_cache_rebudget_tail(rdkv_cache* cache, const rdkv_config* cfg, const void* Q_obs, void* stream);
int32_t rdkv_cache_generations(const rdkv_cache* cache);
const rdkv_cache* rdkv_cache_generation(const rdkv_cache* cache, int32_t index);

/*
 * Calibration of the distortion table (App. B "Calibration"; App. "Calibrated Distortion Tables", Table 9) on the
 * library's own quantizer: for every (sequence, KV head) slice and b in {2, 4, 8} the normalized squared error
 *     eps(b) = sum (x - x_hat_b)^2 / sum x^2
 * over all tokens of the slice (every token retained; 0 for a slice that is all zero).  eps(0) = 1 (removal) and
 * eps(16) = 0 (bits kept verbatim) hold by definition and are not returned.  The paper averages the slice values over
 * layers, heads and calibration sequences; that average is left to the caller.
 *   K, V    DEVICE bf16, ragged [hkv][T_s][d] blocks (cfg: batch, hq, hkv, head_dim, seq_lens, k_mode,
 *           k_scale_per_channel; budgets, tiers and the probe fields are not read; T_s >= 1)
 *   eps_v   HOST double out [items][3] (b = 2, 4, 8): V quantized per token, groups of cfg->group_size channels
 *           (128: one scale per token row, the "per-token" quantity of Table 9)
 *   eps_k   HOST double out [items][3]: K at the granularity cfg selects -- token-wise: as V; channel-wise: groups of
 *           32 consecutive tokens of a channel starting at token 0 (last group may be short), or one scale per
 *           channel over all tokens when k_scale_per_channel is set
 * Codes are those rdkv_pack would store; errors and sums are fp64.  Synchronises `stream` (host results).
 */
rdkv_status rdkv_calibrate_eps(const rdkv_config* cfg, const void* K, const void* V, double* eps_k, double* eps_v,
                               void* stream);

/*
 * Shape of a channel-wise K row (Sec. 3.2 Stage 3; App. B: channels sorted into bit-width segments): the number of
 * 32-bit words a retained token's K row takes under the channel bit map bits_ch (HOST uint8 [128], values out of
 * {0,2,4,8,16}) -- every bit-width segment padded to whole words, the 16-bit one to whole word pairs, the row to an
 * even count; a K tile of 64 tokens takes 256 bytes per word.  Host computation, nothing is launched.  Returns -1 for
 * a null pointer or a value that is no tier.  rdkv_k_row_words_max(): the longest row the decode kernel holds (every
 * valid map fits).
 */
int32_t rdkv_k_row_words(const uint8_t* bits_ch);
int32_t rdkv_k_row_words_max(void);

/* Introspection (tests, benchmarks). */
rdkv_status rdkv_cache_stats(const rdkv_cache* cache, rdkv_stats* out);
/* Size in bytes of an export; 0 for an unknown `what`. */
size_t rdkv_cache_export_bytes(const rdkv_cache* cache, int what);
/* Copies the export to HOST memory `dst` of `bytes` >= rdkv_cache_export_bytes(); synchronous. */
rdkv_status rdkv_cache_export(const rdkv_cache* cache, int what, void* dst, size_t bytes);
/* Releases the cache, its generations and workspaces through the allocator it was built with (a null handle is a
 * no-op).  The memory goes back at once: the caller makes sure that no work that reads the cache (a decode step, an
 * append, a graph replay) is still queued on any stream. */
void rdkv_cache_free(rdkv_cache* cache);

#ifdef __cplusplus
}
#endif
#endif /* RDKV_H */
