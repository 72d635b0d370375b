// Stand-ins for the GPU side of the library, for CPU builds of the host layer (csrc/lt_api.cpp) under the
// address and undefined-behaviour sanitizers.  Every kernel launcher records what it was asked to launch and
// returns success without touching its pointers; the few HIP runtime calls the host layer makes are no-ops.
// Test infrastructure only: nothing in the product links this file.
#include "lt_kernels.h"

#include <cstdlib>
#include <cstring>

namespace {
struct StubLog {
    int append = 0, truncate = 0, decode = 0, zero_tickets = 0, probe = 0, score = 0, prefill = 0, memcpy = 0;
    ltk::DecodeArgs last_decode{};
    ltk::AppendArgs last_append{};
    ltk::ScoreArgs last_score{};
    int last_decode_mode = 0;                       // 0 uniform, 1 per-sequence lengths, 2 paged
    int32_t last_stored_b[ltk::kMaxRaggedBatch] = {};
    int32_t last_new_slot_b[ltk::kMaxRaggedBatch] = {};
};
StubLog g_log;
alignas(256) unsigned char g_scratch[256];          // address only: nothing reads or writes through it
}  // namespace

namespace ltk {

hipError_t append(const AppendArgs &a, hipStream_t)
{
    ++g_log.append;
    g_log.last_append = a;
    return hipSuccess;
}
hipError_t truncate(const TruncateArgs &, hipStream_t)
{
    ++g_log.truncate;
    return hipSuccess;
}
hipError_t decode(const DecodeArgs &a, const RaggedArgs *ragged, const PagedArgs *paged, hipStream_t)
{
    ++g_log.decode;
    g_log.last_decode = a;
    g_log.last_decode_mode = paged != nullptr ? 2 : ragged != nullptr ? 1 : 0;
    const RaggedArgs *lengths = paged != nullptr ? &paged->lengths : ragged;
    if (lengths != nullptr) {
        std::memcpy(g_log.last_stored_b, lengths->stored_b, sizeof(g_log.last_stored_b));
        std::memcpy(g_log.last_new_slot_b, lengths->new_slot_b, sizeof(g_log.last_new_slot_b));
    }
    return hipSuccess;
}
hipError_t zero_tickets(unsigned int *, int, hipStream_t)
{
    ++g_log.zero_tickets;
    return hipSuccess;
}
hipError_t probe_read(const void *, int64_t, uint32_t *, hipStream_t)
{
    ++g_log.probe;
    return hipSuccess;
}
hipError_t lazy_ratio(const ScoreArgs &a, hipStream_t)
{
    ++g_log.score;
    g_log.last_score = a;
    return hipSuccess;
}
hipError_t static_scratch(void **ptr)
{
    *ptr = g_scratch;
    return hipSuccess;
}
hipError_t prefill_attn(const PrefillArgs &, hipStream_t)
{
    ++g_log.prefill;
    return hipSuccess;
}

}  // namespace ltk

extern "C" {

// what the tests read back: launch counts, and the shape of the last decode / append / scoring launch
void lt_stub_reset(void) { g_log = StubLog{}; }
void lt_stub_counts(int32_t *out8)
{
    const int v[8] = {g_log.append, g_log.truncate, g_log.decode, g_log.zero_tickets, g_log.probe, g_log.score, g_log.prefill, g_log.memcpy};
    for (int i = 0; i < 8; ++i) out8[i] = v[i];
}
void lt_stub_last_decode(int64_t *out13)
{
    const ltk::DecodeArgs &a = g_log.last_decode;
    const int64_t v[13] = {a.stored, a.keys_per_block, a.n_splits, a.new_slot, a.spread_tiles, a.k_new != nullptr, a.lazy_tag, a.out_bf16,
                           a.stride_b, a.stride_h, g_log.last_decode_mode,
                           (int64_t)(reinterpret_cast<const unsigned char *>(a.v_cache) - reinterpret_cast<const unsigned char *>(a.k_cache)),
                           a.tail_begin};
    for (int i = 0; i < 13; ++i) out13[i] = v[i];
}
void lt_stub_last_lengths(int32_t *stored_b, int32_t *new_slot_b, int32_t n)
{
    for (int i = 0; i < n && i < ltk::kMaxRaggedBatch; ++i) {
        stored_b[i] = g_log.last_stored_b[i];
        new_slot_b[i] = g_log.last_new_slot_b[i];
    }
}
void lt_stub_last_append(int64_t *out8)
{
    const ltk::AppendArgs &a = g_log.last_append;
    const int64_t v[8] = {a.n_new, a.total_before, a.is_lazy, a.ragged, a.stride_b, a.stride_h, a.block_table != nullptr, a.page_shift};
    for (int i = 0; i < 8; ++i) out8[i] = v[i];
}
void lt_stub_last_score(int64_t *out8)
{
    const ltk::ScoreArgs &a = g_log.last_score;
    const int64_t v[8] = {a.keys_per_block, a.n_chunks, a.n_chunks_a, a.range_a_end, a.range_b_begin, a.fixed_mode, a.lse_rows != nullptr,
                          (int64_t)(reinterpret_cast<const unsigned char *>(a.head_scratch) - reinterpret_cast<const unsigned char *>(a.part))};
    for (int i = 0; i < 8; ++i) out8[i] = v[i];
}

// HIP runtime calls of the host layer
hipError_t hipEventCreate(hipEvent_t *event)
{
    *event = static_cast<hipEvent_t>(std::malloc(1));
    return *event != nullptr ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipEventDestroy(hipEvent_t event)
{
    std::free(event);
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t)
{
    *ms = 1.0f;
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipMemcpyAsync(void *, const void *, size_t, hipMemcpyKind, hipStream_t)
{
    ++g_log.memcpy;                                 // destinations are device addresses: nothing is copied here
    return hipSuccess;
}

}  // extern "C"
