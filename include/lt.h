/*
 * lt.h -- C ABI of the LightTransfer hot path for one AMD MI355X (gfx950).
 *
 * What the library computes (LightTransfer, arXiv 2410.13846):
 *   - lt_lazy_ratio   the lazy ratio r_i of a layer (Section "LightTransfer-Test", Eq. 1)
 *   - lt_select_lazy  which layers become lazy: the ones a max-priority queue of capacity P
 *                     would pop, i.e. the L - P largest ratios (same section; Figure 3)
 *   - lt_append_kv    KV cache of a hybrid stack: full layers keep every token, lazy layers keep
 *                     only the initial and the most recent tokens (same section, last paragraph)
 *   - lt_decode_attn  one decoding step of attention per layer (Section "Preliminary", decoding
 *                     stage): softmax(q K^T + M) V with M the causal mask in a full layer and the
 *                     sink mask (first w_sink, last w_recent positions) in a lazy layer
 *                     (Appendix "Theoretical Analysis")
 *
 * Conventions for every call
 *   Pointers marked "device" are HIP device addresses on the current device; "host" are ordinary
 *   host addresses.  The caller owns ALL device memory (KV slab, workspaces, inputs, outputs) and
 *   the stream; the library never allocates or frees device memory.  Device work is enqueued on
 *   `stream` (a hipStream_t passed as void*; NULL is the default stream) and the call returns
 *   without waiting for it.  Token counts live on the host, so no call synchronises.
 *   bf16 tensors are raw 16-bit patterns, dense and row-major in the stated shape unless strides
 *   are given; fp32 outputs are dense.  head_dim must be 128.  A layer keeps one token count per
 *   batch while every call adds the same number of tokens to every sequence; lt_append_kv_ragged,
 *   lt_reset_sequence, lt_decode_step_active and paged contexts switch a layer to one count per
 *   sequence (batch <= 128 then).
 *   Errors: every call validates its arguments and the state it needs on the host, before it
 *   enqueues the work it was asked for, and returns a status; on any status other than LT_OK no
 *   token was appended, no token count changed and no cache byte was written.  Two things may
 *   still have happened on an error path and are harmless: the first decode call on a context
 *   enqueues the one-off zeroing of its counters before its launch, and a call that needs
 *   per-sequence counts (see above) switches the layer's bookkeeping to them, which changes no
 *   length.  In an online context (lt_create_online) a layer's first append reserves a full-size
 *   slot; if that append's launch is then refused by the runtime (LT_ERR_HIP) the slot stays with
 *   the layer.  There are no exceptions and no aborts; different lt_ctx objects are independent,
 *   and one lt_ctx must not be used from two threads at once.  The only process-wide state is the
 *   scratch array of lt_lazy_ratio_static.
 */
#ifndef LT_H
#define LT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lt_ctx lt_ctx; /* opaque, host memory owned by the library */

typedef enum {
    LT_OK = 0,
    LT_ERR_INVALID_ARG = 1, /* NULL pointer, negative size, unknown enum value, NaN ratio */
    LT_ERR_SHAPE = 2,       /* sizes that do not fit together (heads, head_dim, w_last > n, ...) */
    LT_ERR_CAPACITY = 3,    /* a full layer would exceed max_tokens, or a buffer is too small */
    LT_ERR_STATE = 4,       /* call out of order (decode on an empty layer, ...) */
    LT_ERR_HIP = 5,         /* the HIP runtime refused a launch or an event call */
    LT_ERR_NOMEM = 6        /* host allocation failed */
} lt_status;

/* Which keys count as X_recent in the lazy ratio.  Eq. 1 together with the per-row kept sets of
 * the appendix gives each query its own window ending at that query (PER_QUERY, the default and
 * exactly the mass streaming attention keeps); Table 1 slices the last w_recent prompt keys once
 * for all queries (FIXED).  Both apply the causal mask. */
typedef enum { LT_RECENT_PER_QUERY = 0, LT_RECENT_FIXED = 1 } lt_ratio_mode;

typedef struct lt_config {
    int32_t n_layers;     /* L */
    int32_t batch;        /* B, sequences decoded together */
    int32_t n_q_heads;    /* Hq */
    int32_t n_kv_heads;   /* Hkv, divides Hq; query head h reads KV head h / (Hq/Hkv); Hq/Hkv <= 8 */
    int32_t head_dim;     /* 128 */
    int32_t w_sink;       /* initial tokens a lazy layer keeps (Appendix A: 4) */
    int32_t w_recent;     /* most recent tokens a lazy layer keeps, current token included (1020) */
    int64_t max_tokens;   /* capacity of a full layer's cache, in tokens per sequence */
    float softmax_scale;  /* multiplies q.k before the softmax; 0 selects 1/sqrt(head_dim) */
} lt_config;

/* ---- KV-cache manager -------------------------------------------------------------------- */

/* Bytes of device memory the KV slab needs for this configuration and lazy mask: per layer one K
 * and one V block of bf16 [B][Hkv][cap][128], cap = max_tokens (full layer) or w_sink + w_recent
 * (lazy layer), each block aligned to 256 bytes.  Returns 0 on invalid arguments.
 * is_lazy: host, L entries, non-zero = lazy. */
size_t lt_kv_bytes(const lt_config *cfg, const uint8_t *is_lazy);

/* Bytes of device workspace lt_decode_attn / lt_decode_step need (fp32 partial results of the
 * split over the key axis, and one counter per (sequence, KV head)).  The first decode call on a
 * context zeroes the counters on its stream; use one stream at a time per context.  Returns 0 on
 * invalid arguments. */
size_t lt_workspace_bytes(const lt_config *cfg);

/* Create the host-side state of a hybrid stack over caller-owned device memory.
 * kv_slab (device, >= lt_kv_bytes, 256-byte aligned) and workspace (device, >= lt_workspace_bytes,
 * 256-byte aligned) stay owned by the caller and must outlive the context.  Nothing is enqueued:
 * cache contents are undefined until appended.  *out receives the context. */
lt_status lt_create(const lt_config *cfg, const uint8_t *is_lazy, void *kv_slab, size_t kv_bytes,
                    void *workspace, size_t ws_bytes, lt_ctx **out);

/* Free the host-side state.  Device memory is untouched.  NULL is allowed. */
void lt_destroy(lt_ctx *ctx);

/* Forget every token of every layer (host counters only).  The next decode call zeroes the split
 * counters in the workspace again, so a context whose launch failed half-way is usable after this. */
lt_status lt_reset(lt_ctx *ctx);

/* Tokens appended to a layer so far (total) and entries its cache holds (stored:
 * total for a full layer, min(total, w_sink + w_recent) for a lazy one).  Either output may be NULL. */
lt_status lt_layer_len(const lt_ctx *ctx, int32_t layer, int64_t *total_tokens, int64_t *stored_tokens);

/* Where a layer's cache lives inside the slab: device addresses of its K and V blocks, strides in
 * bf16 elements between sequences and between KV heads (token stride is 128), capacity in tokens,
 * and whether it is lazy.  Any output may be NULL.  In a lazy layer the token at absolute position
 * p sits in slot p when p < w_sink and in slot w_sink + (p - w_sink) mod w_recent otherwise. */
lt_status lt_layer_view(const lt_ctx *ctx, int32_t layer, void **k_dev, void **v_dev,
                        int64_t *stride_b, int64_t *stride_h, int64_t *capacity, int32_t *is_lazy);

/* ---- lazy-layer identification ------------------------------------------------------------ */

/* Bytes of device workspace lt_lazy_ratio needs for a prompt of n tokens scored over its last
 * w_last queries (partial sums of the key ranges, per-head sums, counters of finished ranges; the
 * call clears the counters itself).  Returns 0 on invalid arguments. */
size_t lt_lazy_ratio_workspace_bytes(const lt_config *cfg, int64_t n, int32_t w_last);

/* Lazy ratio of one layer (Eq. 1): for each of the last w_last prompt positions p = n-w_last..n-1
 * and each query head, the share rho of the causal softmax row of that query (keys 0..p, logits
 * softmax_scale * q.k) that falls on the first w_sink keys and on the recent keys
 * (PER_QUERY: p-w_recent+1..p; FIXED: n-w_recent..n-1, up to p); the union is a set.
 *   q_last        device, bf16 [B][Hq][w_last][128], queries of positions n-w_last..n-1
 *   k             device, bf16, key of (sequence b, KV head g, position j) at element offset
 *                 b*k_stride_b + g*k_stride_h + j*k_stride_t; the 128 dims are contiguous and
 *                 every stride is a multiple of 8 elements (may point into the KV slab)
 *   n, w_last     prompt length and number of scored queries, 1 <= w_last <= min(n, 64)
 *   workspace     device, >= lt_lazy_ratio_workspace_bytes(cfg, n, w_last), 256-byte aligned
 *   rho_dev       device, fp32 [B][Hq][w_last], may be NULL
 *   ratio_seq_dev device, fp32 [B]: mean of rho over heads and queries of each sequence, may be NULL
 *   ratio_mean_dev device, fp32 [1]: mean of ratio_seq over the batch (the layer's r_i)
 * Uses cfg->batch, head counts, head_dim, w_sink, w_recent and softmax_scale. */
lt_status lt_lazy_ratio(const lt_config *cfg, const void *q_last, const void *k, int64_t k_stride_b,
                        int64_t k_stride_h, int64_t k_stride_t, int64_t n, int32_t w_last,
                        lt_ratio_mode mode, void *workspace, size_t ws_bytes, float *rho_dev,
                        float *ratio_seq_dev, float *ratio_mean_dev, void *stream);

/* lt_lazy_ratio for callers that cannot allocate or bring a workspace: code recorded under stream
 * capture into a HIP graph, tight serving loops, harnesses that forbid device allocation.  Same
 * arguments, outputs, results and errors as lt_lazy_ratio, without `workspace` / `ws_bytes`: the
 * partial sums and counters live in an 8 MiB array that is part of the library's code object (one
 * copy per GPU, held until the process ends).  The call allocates nothing on host or device and
 * frees nothing; on its first use on a device it looks the array's address up (do that first call
 * outside a capture).  LT_ERR_CAPACITY, with nothing enqueued, when
 * lt_lazy_ratio_workspace_bytes(cfg, n, w_last) exceeds 8 MiB (about 10 000 (sequence, query head)
 * pairs at w_last = 64; every configuration of the benchmark needs less than 1 MiB).  All calls on
 * one GPU share the array, which keeps the last call's contents: the counters in it are cleared by
 * a small fill launch at the start of every call, nothing else needs to start at zero; two calls
 * whose kernels may overlap on one GPU (different streams, or different threads) race; calls on one
 * stream are safe. */
lt_status lt_lazy_ratio_static(const lt_config *cfg, const void *q_last, const void *k, int64_t k_stride_b,
                               int64_t k_stride_h, int64_t k_stride_t, int64_t n, int32_t w_last,
                               lt_ratio_mode mode, float *rho_dev, float *ratio_seq_dev,
                               float *ratio_mean_dev, void *stream);

/* Bytes of device workspace lt_lazy_ratio_lse needs.  Returns 0 on invalid arguments. */
size_t lt_lazy_ratio_lse_workspace_bytes(const lt_config *cfg, int64_t n, int32_t w_last);

/* Lazy ratio of one layer from the log-sum-exp the prefill attention already produced (Table 1:
 * rho = exp(LSE over the initial and recent keys - LSE of the whole causal row)).  Only the first
 * w_sink keys and the keys from the earliest recent key of a scored query onwards are read, so the
 * cost does not grow with n.  Same result as lt_lazy_ratio when lse_rows holds the rows' true LSE.
 *   lse_rows      device, fp32: natural-log LSE (softmax_scale included) of the causal row of
 *                 (sequence b, head h, position n-w_last+t) at element b*lse_stride_b +
 *                 h*lse_stride_h + t; lt_prefill_attn's lse_out + (n_queries - w_last) with strides
 *                 Hq*n_queries, n_queries
 *   workspace     device, >= lt_lazy_ratio_lse_workspace_bytes(cfg, n, w_last), 256-byte aligned
 * Every other argument, the outputs and the errors are those of lt_lazy_ratio. */
lt_status lt_lazy_ratio_lse(const lt_config *cfg, const void *q_last, const void *k, int64_t k_stride_b,
                            int64_t k_stride_h, int64_t k_stride_t, int64_t n, int32_t w_last,
                            lt_ratio_mode mode, const float *lse_rows, int64_t lse_stride_b,
                            int64_t lse_stride_h, void *workspace, size_t ws_bytes, float *rho_dev,
                            float *ratio_seq_dev, float *ratio_mean_dev, void *stream);

/* Prefill attention of one layer (Section "Preliminary", prefilling: position p attends to
 * positions 0..p; Appendix "Theoretical Analysis": softmax(Q K^T + M) V) for the last n_queries of
 * n positions: n_queries = n is the prefill of a whole prompt, a smaller n_queries one chunk of a
 * chunked prefill whose earlier keys and values are already in place.
 *   mask  LT_MASK_CAUSAL: M is the causal mask.  LT_MASK_STREAMING: the sink mask, position p
 *         attends to the first w_sink and the last w_recent positions of 0..p (p included), as a
 *         layer that runs streaming attention from the start does (LightTransfer-Train).
 *   q         device, bf16 [B][Hq][n_queries][128], the queries of positions n-n_queries .. n-1
 *   k, v      device, bf16, positions 0 .. n-1; (sequence b, KV head g, position j) at element
 *             offset b*kv_stride_b + g*kv_stride_h + j*kv_stride_t of each; 128 dims contiguous,
 *             strides multiples of 8, 128 <= kv_stride_t < 2^24 (may point into the KV slab of a
 *             full layer after lt_append_kv)
 *   out       device, [B][Hq][n_queries][128], bf16 (LT_OUT_BF16) or fp32 (LT_OUT_F32)
 *   lse_out   device, fp32 [B][Hq][n_queries]: natural log of each row's softmax denominator
 *             (softmax_scale included), may be NULL
 * Logits and sums are fp32; the probabilities enter the P V product rounded to bf16 (the values are
 * bf16 already), accumulation is fp32.  Uses cfg->batch, head counts, head_dim, w_sink, w_recent,
 * softmax_scale.  Nothing is allocated; the launch is asynchronous on `stream`.
 * Errors: LT_ERR_INVALID_ARG (NULL or misaligned pointers, bad enums, n or n_queries <= 0),
 * LT_ERR_SHAPE (n_queries > n, unsupported head shape or strides, streaming mask with an empty
 * window). */
typedef enum lt_mask_mode { LT_MASK_CAUSAL = 0, LT_MASK_STREAMING = 1 } lt_mask_mode;
typedef enum lt_out_dtype { LT_OUT_BF16 = 0, LT_OUT_F32 = 1 } lt_out_dtype;
lt_status lt_prefill_attn(const lt_config *cfg, const void *q, const void *k, const void *v,
                          int64_t kv_stride_b, int64_t kv_stride_h, int64_t kv_stride_t, int64_t n, int64_t n_queries,
                          lt_mask_mode mask, lt_out_dtype out_dtype, void *out, float *lse_out, void *stream);

/* Choose the lazy layers (pure host code): the n_lazy layers with the largest ratios, ties going
 * to the lower layer index; this is the set a max-priority queue of capacity L - n_lazy pops when
 * layers are pushed in order.
 *   ratios_host  host, fp32 [L]; a NaN is rejected with LT_ERR_INVALID_ARG
 *   is_lazy_out  host, uint8 [L], 1 = lazy
 *   order_out    host, int32 [L], layers from laziest to least lazy; may be NULL */
lt_status lt_select_lazy(const float *ratios_host, int32_t n_layers, int32_t n_lazy, uint8_t *is_lazy_out,
                         int32_t *order_out);

/* Pre-selection of a fixed lazy set from many samples (Section "LightTransfer-Train"; pure host
 * code): every sample contributes the lazy set it would choose on its own (lt_lazy_ratio +
 * lt_select_lazy on the sample's question + answer); the n_lazy layers chosen most often become
 * the fixed set, equal frequencies going to the lower layer index.
 *   is_lazy_samples  host, uint8 [n_samples][n_layers], non-zero = sample chose the layer
 *   is_lazy_out      host, uint8 [n_layers], 1 = selected
 *   count_out        host, int32 [n_layers], frequency of every layer; may be NULL */
lt_status lt_preselect_lazy(const uint8_t *is_lazy_samples, int32_t n_samples, int32_t n_layers, int32_t n_lazy,
                            uint8_t *is_lazy_out, int32_t *count_out);

/* ---- online identification during prefill (Section "LightTransfer-Test", Figure 3) ---------- */

/* The paper's procedure: after each layer's prefill its (ratio, layer) is pushed into a
 * max-priority queue of capacity P; when the queue overflows, the layer with the highest ratio
 * is popped, becomes lazy, and its cache is reduced at once, which frees memory for the next
 * layer's cache.  Peak memory is P + 1 full caches instead of L. */
typedef struct lt_queue lt_queue; /* opaque, host memory owned by the library */

/* A queue that keeps `capacity` = P entries.  *out receives it. */
lt_status lt_queue_create(int32_t capacity, lt_queue **out);
void lt_queue_destroy(lt_queue *q); /* NULL is allowed */

/* Push one layer's ratio (pure host code).  *popped_layer receives the layer that left the queue
 * -- the highest ratio held, ties to the lower layer index, possibly the one just pushed -- or
 * -1 if the queue did not overflow.  NaN ratios are rejected. */
lt_status lt_select_push(lt_queue *q, float ratio, int32_t layer, int32_t *popped_layer);

/* Bytes of KV slab for the online procedure with n_full = P layers kept full:
 * min(P + 1, L) full-size slots and L - P ring slots.  Returns 0 on invalid arguments. */
size_t lt_kv_bytes_online(const lt_config *cfg, int32_t n_full);

/* Like lt_create, but no lazy mask is known yet: every layer starts as a full layer without
 * storage and takes a free full-size slot at its first lt_append_kv (LT_ERR_CAPACITY if all
 * min(P + 1, L) slots are in use).  lt_reset returns every layer to that state. */
lt_status lt_create_online(const lt_config *cfg, int32_t n_full, void *kv_slab, size_t kv_bytes, void *workspace,
                           size_t ws_bytes, lt_ctx **out);

/* Turn a full layer of an online context into a lazy one: its first w_sink and last w_recent
 * tokens are copied (enqueued on `stream`) into a free ring slot, each to the slot lt_append_kv
 * would have used, and its full-size slot becomes available to appends enqueued afterwards on the
 * same stream.  The token count is unchanged.  LT_ERR_STATE if the context was made by lt_create
 * or the layer is already lazy; LT_ERR_CAPACITY if all L - P ring slots are in use. */
lt_status lt_truncate_layer(lt_ctx *ctx, int32_t layer, void *stream);

/* ---- decoding ----------------------------------------------------------------------------- */

/* Append n_new tokens (the same count for every sequence) to a layer.
 *   k_new, v_new  device, bf16 [B][Hkv][n_new][128]
 * Full layer: tokens go to positions total..total+n_new-1; LT_ERR_CAPACITY if that exceeds
 * max_tokens.  Lazy layer: a token whose absolute position is neither among the first w_sink nor
 * among the last w_recent after this call is dropped, every other token goes to its ring slot
 * (see lt_layer_view), so a bulk append of a whole prompt leaves exactly the reduced cache. */
lt_status lt_append_kv(lt_ctx *ctx, int32_t layer, const void *k_new, const void *v_new, int64_t n_new,
                       void *stream);

/* Ragged batches (serving: prompts of different lengths in one batch).  Like lt_append_kv, but
 * sequence b brings only its first n_per_seq_host[b] tokens of the padded input (0 <= n <= n_max);
 * from then on the layer keeps one token count per sequence: later lt_append_kv / lt_decode_step
 * calls add the same number of tokens to every sequence, lt_decode_attn / lt_decode_step attend,
 * for sequence b, over that sequence's own stored entries (all of its tokens in a full layer, its
 * own first w_sink and last w_recent in a lazy layer), and a sequence without tokens yields out = 0,
 * lse = -inf.  lt_layer_len then reports the longest sequence, lt_seq_len one sequence.
 *   k_new, v_new     device, bf16 [B][Hkv][n_max][128]; rows past a sequence's count are not read
 *   n_per_seq_host   host, int64 [B]
 * The per-sequence counts travel to the kernels as launch arguments: nothing is allocated or copied.
 * LT_ERR_SHAPE if batch > 128; LT_ERR_STATE on a context made by lt_create_online; LT_ERR_CAPACITY
 * if the longest sequence would exceed max_tokens. */
lt_status lt_append_kv_ragged(lt_ctx *ctx, int32_t layer, const void *k_new, const void *v_new, int64_t n_max,
                              const int64_t *n_per_seq_host, void *stream);

/* Tokens appended to / stored for one sequence of a layer (equal for all sequences unless
 * lt_append_kv_ragged was used).  Either output may be NULL. */
lt_status lt_seq_len(const lt_ctx *ctx, int32_t layer, int32_t sequence, int64_t *total_tokens, int64_t *stored_tokens);

/* Forget the tokens of one sequence in every layer (host counters only): the slot is free for a new
 * prompt, brought by lt_append_kv_ragged with a count of 0 for the other sequences.  Turns the
 * context into the per-sequence mode of lt_append_kv_ragged.  LT_ERR_SHAPE if batch > 128;
 * LT_ERR_STATE on a context made by lt_create_online. */
lt_status lt_reset_sequence(lt_ctx *ctx, int32_t sequence);

/* ---- paged storage for the full layers (serving; the paper's Section "LightTransfer-Test" keeps
 * the whole cache of a non-lazy layer, which a server stores page by page so that sequences of
 * different and growing lengths share one pool) -------------------------------------------------
 *
 * A full layer owns a K pool and a V pool of bf16 [n_pages][Hkv][page_tokens][128]; ONE block
 * table, int32 [B][max_pages] with max_pages = ceil(max_tokens / page_tokens), serves all full
 * layers: token p of sequence b lives in page table[b][p / page_tokens] of each full layer's pools,
 * at row p mod page_tokens.  -1 = no page.  The caller assigns pages (two sequences may name the same
 * page only if neither is appended to while they do); the library checks on the host, before every
 * launch, that each token a kernel will read or write has a page inside the pool, so a bad table is
 * an error code and never a stray access.  Lazy layers keep their rings, one per sequence, as in
 * lt_create.  Lengths are per sequence throughout (see lt_append_kv_ragged); every other call works
 * as on a context from lt_create, except lt_truncate_layer (LT_ERR_STATE), and lt_layer_view, whose
 * strides for a full layer are those inside one page (stride_b = the stride between pages).
 *
 * page_tokens: a power of two, 64 <= page_tokens <= 2^20.  batch <= 128.
 * lt_kv_bytes_paged: bytes of the slab (table + pools + rings); 0 on invalid arguments.
 * lt_create_paged: LT_ERR_SHAPE if page_tokens is no such power of two, batch > 128, or max_tokens
 * exceeds what the split decode kernel covers with pages this small (255 pages per workgroup). */
size_t lt_kv_bytes_paged(const lt_config *cfg, const uint8_t *is_lazy, int32_t page_tokens, int32_t n_pages);
lt_status lt_create_paged(const lt_config *cfg, const uint8_t *is_lazy, int32_t page_tokens, int32_t n_pages,
                          void *kv_slab, size_t kv_bytes, void *workspace, size_t ws_bytes, lt_ctx **out);

/* Replace the block table.
 *   table_host  host, int32 [B][max_pages]; every entry -1 or in [0, n_pages)
 * The pages that hold a sequence's tokens so far must stay named (LT_ERR_STATE otherwise); entries
 * beyond may be set ahead of need.  LT_ERR_INVALID_ARG for an entry outside the pool.  The call waits
 * for the work already on `stream` (kernels may be reading the old table), copies, and waits for the
 * copy: tables change when a sequence crosses a page or a slot changes hands, not every step.
 * lt_append_kv(_ragged) and lt_decode_step return LT_ERR_STATE, with nothing enqueued, when a token
 * they would store has no page. */
lt_status lt_set_block_table(lt_ctx *ctx, const int32_t *table_host, void *stream);

/* Element type of `out` in lt_decode_attn / lt_decode_step from now on: LT_OUT_F32 (the default)
 * or LT_OUT_BF16 (rounded to nearest even from the fp32 result; what a bf16 model consumes). */
lt_status lt_set_output_dtype(lt_ctx *ctx, lt_out_dtype dtype);

/* Attention of the newest token of every sequence over the layer's cache, to be called after the
 * token's own K/V were appended (the causal mask keeps the diagonal).
 *   q        device, bf16 [B][Hq][128]
 *   out      device, [B][Hq][128], fp32 unless lt_set_output_dtype chose bf16:
 *            sum_j softmax_j(softmax_scale * q.k_j) v_j over the stored entries
 *   lse_out  device, fp32 [B][Hq]: natural-log of the softmax denominator; may be NULL
 * One launch: workgroups each take a range of the stored entries and the last one to finish
 * merges the ranges by their log-sum-exp.  On long histories (thousands of keys per workgroup) the
 * last part of the entries is shared out at run time, so the fp32 sums can be taken in a
 * different order from launch to launch and outputs may differ in their last bits (a few 1e-7)
 * between two calls on the same inputs; lt_set_shared_tail in lt_measure.h switches that off.
 * LT_ERR_STATE if the layer is empty. */
lt_status lt_decode_attn(lt_ctx *ctx, int32_t layer, const void *q, void *out, float *lse_out, void *stream);

/* One decoding step of a layer in a single launch: lt_append_kv of one token followed by
 * lt_decode_attn, with the same result and the same effect on the cache and the token count.
 *   k_new, v_new  device, bf16 [B][Hkv][128], the K/V of the token being generated
 * The decode kernel takes the new token from k_new / v_new and stores it into its cache slot on
 * the way.  LT_ERR_CAPACITY as for lt_append_kv; on error nothing is enqueued or counted. */
lt_status lt_decode_step(lt_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new, void *out,
                         float *lse_out, void *stream);

/* lt_decode_step for the sequences that are still generating (serving: others have finished or their
 * slot is empty).  active_host: host, uint8 [B], non-zero = takes part.  A sequence that sits the step out
 * gets no token, keeps its length, is not read at all, and its rows of out / lse_out are 0 / -inf.  Turns
 * the context into the per-sequence mode of lt_append_kv_ragged.  LT_ERR_SHAPE if batch > 128; LT_ERR_STATE on
 * a context made by lt_create_online, and when no active sequence has anything to attend over;
 * LT_ERR_CAPACITY / (paged) LT_ERR_STATE look at the active sequences only. */
lt_status lt_decode_step_active(lt_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new,
                                const uint8_t *active_host, void *out, float *lse_out, void *stream);

/* Tuning knobs and measurement aids (split size, event timing, read-rate probe) are declared in
 * lt_measure.h; the product path does not need them. */

const char *lt_status_str(lt_status status);

#ifdef __cplusplus
}
#endif
#endif /* LT_H */
