// Internal launch interface between the C-ABI layer (lt_api.cpp) and the gfx950 kernels.
// Plain pointers and sizes only; every launcher validates nothing (the API layer does) and
// returns the HIP status of its launches.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ltk {

constexpr int kHeadDim = 128;          // bf16 elements per key / value / query vector
constexpr int kMaxGroup = 8;           // query heads per KV head
constexpr int kWideBlockKeys = 2048;    // decode workgroups with at most this many keys run eight wavefronts, else four
constexpr int kKeyGranule = 64;        // keys_per_block is a multiple of this
constexpr int kMaxSplits = 512;        // most key ranges one (sequence, KV head) is split into
constexpr int kTicketStride = 64;      // uint32 slots between tickets: one per 256 bytes, so they spread over memory channels;
                                       // slot 1 after a ticket counts the pieces handed out of the shared tail
constexpr int kTailKeys = 32;          // keys per piece of the shared tail (two tiles)
constexpr int kMaxRaggedBatch = 128;   // sequences a launch can give their own lengths (the lengths travel as kernel arguments: 2 KB of the 4 KB there are)
constexpr int kScoreTileKeys = 128;    // key ranges of the scoring kernel are multiples of this

struct AppendArgs {
    const uint16_t *k_new, *v_new;     // [B][Hkv][n_new][128]
    uint16_t *k_cache, *v_cache;       // layer blocks
    int64_t stride_b, stride_h;        // cache strides in elements
    int64_t n_new, total_before;       // tokens in this call, tokens already in the layer
    int32_t batch, n_kv_heads;
    int32_t is_lazy, w_sink, w_recent;
    // ragged batches: sequence b brings n_new_b[b] <= n_new tokens (rows beyond are padding) and holds total_before_b[b]
    int32_t ragged;
    int64_t n_new_b[kMaxRaggedBatch], total_before_b[kMaxRaggedBatch];
    // paged full layer (block_table != nullptr): k_cache / v_cache are pools [page][Hkv][1 << page_shift][128] and
    // token p of sequence b lives in page block_table[b * max_pages + (p >> page_shift)]
    const int32_t *block_table;
    int32_t max_pages, page_shift;
};
hipError_t append(const AppendArgs &a, hipStream_t stream);

struct TruncateArgs {
    const uint16_t *k_full, *v_full;   // full-layer blocks [B][Hkv][cap_full][128]
    uint16_t *k_ring, *v_ring;         // ring blocks       [B][Hkv][w_sink + w_recent][128]
    int64_t stride_b_full, stride_h_full, stride_b_ring, stride_h_ring;
    int64_t total;                     // tokens the layer holds
    int32_t batch, n_kv_heads, w_sink, w_recent;
};
hipError_t truncate(const TruncateArgs &a, hipStream_t stream);

struct DecodeArgs {
    uint16_t *k_cache, *v_cache;
    const uint16_t *k_new, *v_new;     // [B][Hkv][128] token of this step to append on the fly, or nullptr
    int32_t new_slot;                  // cache entry the new token belongs to (used when k_new != nullptr)
    unsigned int *tickets;             // [B][Hkv] tickets kTicketStride apart, zero between launches
    const uint16_t *q;                 // [B][Hq][128]
    float *part_acc;                   // [B][Hq][S][128]  un-normalised partial outputs
    float *part_ml;                    // [B][Hq][S][2]    running max (log2 units) and sum
    void *out;                         // [B][Hq][128] fp32, or bf16 when out_bf16
    float *lse;                        // [B][Hq] or nullptr
    int64_t stride_b, stride_h;
    int32_t batch, n_q_heads, n_kv_heads;
    int32_t stored;                    // cache entries to attend over
    int32_t keys_per_block, n_splits;
    float scale_log2e;                 // softmax_scale * log2(e)
    int32_t lazy_tag;                  // selects the kernel instantiation (name) only
    int32_t out_bf16;                  // out holds bf16 instead of fp32
    uint32_t spread_tiles;             // window (4 KB tiles, a power of two) the workgroups' start addresses are spread over; 0: pseudo-random starts
    // Keys from tail_begin on (a multiple of kKeyGranule) belong to no workgroup's range: the wavefronts of the
    // (sequence, KV head) take them in pieces of kTailKeys, first come first served, once their own tiles are done.
    // The n_splits ranges of keys_per_block keys then cover [0, tail_begin).  INT32_MAX: no shared tail.
    int32_t tail_begin;
    int32_t matrix_cores;              // 1: the kernel that forms both products on the matrix cores; 0: the vector kernel
};
// ragged batches: per-sequence stored entries (<= stored, which sizes the grid) and new-token slots (-1: dropped);
// a separate argument block, so that launches for equal-length batches do not carry it
struct RaggedArgs {
    int32_t stored_b[kMaxRaggedBatch], new_slot_b[kMaxRaggedBatch];
};
// paged full layer: per-sequence lengths as above, and k_cache / v_cache are pools [page][Hkv][1 << page_shift][128];
// entry (p >> page_shift) of a sequence's row of the block table names the page that holds its token p.  A workgroup's
// key range may touch at most kMaxRangePages pages (the launcher's keys_per_block sees to that).
constexpr int kMaxRangePages = 256;     // four registers of 64 lanes
struct PagedArgs {
    RaggedArgs lengths;
    const int32_t *block_table;        // device, [B][max_pages]
    int32_t max_pages, page_shift;
};
// ragged == nullptr and paged == nullptr: equal lengths, contiguous cache.  At most one of the two is given.
hipError_t decode(const DecodeArgs &a, const RaggedArgs *ragged, const PagedArgs *paged, hipStream_t stream);
hipError_t zero_tickets(unsigned int *tickets, int n, hipStream_t stream);
hipError_t probe_read(const void *buf, int64_t bytes, uint32_t *sink, hipStream_t stream);

struct ScoreArgs {
    const uint16_t *q_last;            // [B][Hq][w][128]
    const uint16_t *k;
    int64_t k_stride_b, k_stride_h, k_stride_t;
    int64_t n;
    int32_t w_last, batch, n_q_heads, n_kv_heads;
    int32_t w_sink, w_recent, fixed_mode;
    int32_t keys_per_block, n_chunks;
    // key ranges the chunks cover: chunks [0, n_chunks_a) tile [0, range_a_end), the others
    // [range_b_begin, n).  The dense form has one range (range_a_end = n, n_chunks_a = n_chunks).
    int64_t range_a_end, range_b_begin;
    int32_t n_chunks_a;
    const float *lse_rows;             // natural-log LSE of the causal rows n-w..n-1, or nullptr: computed here
    int64_t lse_stride_b, lse_stride_h;
    float scale_log2e;
    float *part;                       // [B][Hq][n_chunks][3][w]: max (log2 units), causal sum, kept sum
    float *head_scratch;               // [B][Hq] sum of rho over the queries of a head
    unsigned int *tickets;             // [B * Hkv + 1] counters of finished key ranges / finished (sequence, KV head) pairs
    float *rho, *ratio_seq, *ratio_mean;
};
hipError_t lazy_ratio(const ScoreArgs &a, hipStream_t stream);

// Device address, on the current device, of the library's built-in scratch array of
// kStaticScratchBytes bytes (256-byte aligned; zero when the code object is loaded, afterwards it
// keeps what the last launch left).  Looked up once per device; allocates nothing.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
hipError_t static_scratch(void **ptr);

struct PrefillArgs {
    const uint16_t *q;                 // [B][Hq][n_q][128]: the queries of positions n - n_q .. n - 1
    const uint16_t *k, *v;             // [B][Hkv][n][128] through the strides below (elements)
    int64_t kv_stride_b, kv_stride_h, kv_stride_t;
    void *out;                         // [B][Hq][n_q][128] bf16, or fp32 when out_f32
    float *lse;                        // [B][Hq][n_q] natural-log row denominators, or nullptr
    int64_t n, n_q;
    int32_t batch, n_q_heads, n_kv_heads;
    int32_t streaming, w_sink, w_recent;
    int32_t out_f32;
    float scale_log2e;
    int32_t kv_share;                  // set by prefill_attn: workgroups' head groups per KV head (see there), 1 normally
};
hipError_t prefill_attn(const PrefillArgs &a, hipStream_t stream);

}  // namespace ltk
