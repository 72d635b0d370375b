// C-ABI layer of the LightTransfer hot path: argument validation, the KV-cache manager (slab
// layout, per-layer token counts, ring geometry), lazy-layer selection on the host, and the
// launch plumbing (split heuristics, optional event timing).  All arithmetic of the method runs
// in the kernels behind lt_kernels.h; this file only decides shapes and addresses.
#include "../../include/lt.h"
#include "../../include/lt_measure.h"
#include "lt_kernels.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <climits>
#include <new>
#include <vector>

namespace {

constexpr size_t kAlign = 256;
constexpr int64_t kMaxTokens = (int64_t)1 << 30;        // per-sequence positions are 32-bit inside the decode kernel
constexpr int kMinKeysFull = 256;                       // smallest split the decode workspace is sized for (full layers)
constexpr int kMinKeysLazy = 64;                        // same, lazy layers
constexpr int kMinKeysSharedTail = 8192;                // key ranges at least this long leave a shared tail
constexpr int kMinSplitsWideTail = 16;                  // ranges half as long do when a (sequence, KV head) has this many
constexpr int kMaxEventPairs = 65536;
constexpr float kLog2e = 1.4426950408889634f;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

bool config_ok(const lt_config *c)
{
    if (c == nullptr) return false;
    if (c->n_layers <= 0 || c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0) return false;
    if (c->w_sink < 0 || c->w_recent < 0) return false;
    if (c->max_tokens <= 0 || c->max_tokens > kMaxTokens) return false;
    if (!(c->softmax_scale >= 0.f) || std::isinf(c->softmax_scale)) return false;
    return true;
}

lt_status config_shape(const lt_config *c)
{
    if (c->head_dim != ltk::kHeadDim) return LT_ERR_SHAPE;
    if (c->n_q_heads % c->n_kv_heads != 0) return LT_ERR_SHAPE;
    if (c->n_q_heads / c->n_kv_heads > ltk::kMaxGroup) return LT_ERR_SHAPE;
    if (c->batch > 65535 || c->n_kv_heads > 65535 || c->n_q_heads > 65535) return LT_ERR_SHAPE;   // grid y/z limits
    return LT_OK;
}

float effective_scale(const lt_config *c)
{
    return c->softmax_scale > 0.f ? c->softmax_scale : 1.0f / std::sqrt((float)c->head_dim);
}

int64_t window_of(const lt_config *c) { return (int64_t)c->w_sink + c->w_recent; }

int64_t layer_capacity(const lt_config *c, bool lazy) { return lazy ? window_of(c) : c->max_tokens; }

size_t block_bytes(const lt_config *c, bool lazy)
{
    return align_up((size_t)c->batch * c->n_kv_heads * (size_t)layer_capacity(c, lazy) * ltk::kHeadDim * sizeof(uint16_t));
}

int64_t max_splits(const lt_config *c);

}  // namespace

struct lt_ctx;
static void bind_workspace(lt_ctx *ctx, void *workspace);

namespace {

int64_t max_splits(const lt_config *c)
{
    const int64_t full = ceil_div(c->max_tokens, kMinKeysFull);
    const int64_t lazy = ceil_div(std::max<int64_t>(window_of(c), 1), kMinKeysLazy);
    return std::min<int64_t>(std::max<int64_t>(std::max(full, lazy), 1), ltk::kMaxSplits);
}

struct Layer {
    uint16_t *k = nullptr, *v = nullptr;
    int64_t capacity = 0;
    int64_t total = 0;                          // tokens appended so far (ragged batches: of the longest sequence)
    std::vector<int64_t> total_b;               // ragged batches: tokens of every sequence; empty while all are equal
    bool lazy = false;
    int32_t slot = -1;                          // online mode: index of the full / ring slot in use, -1 = none yet
    int32_t plan[4] = {0, 0, -1, 0};            // most recent decode launch (lt_decode_plan_read); plan[1] = 0: none yet
};

struct EventPair {
    hipEvent_t start, stop;
    int32_t kernel;
};

}  // namespace

struct lt_ctx {
    lt_config cfg;
    std::vector<Layer> layers;
    float *part_acc = nullptr, *part_ml = nullptr;
    unsigned int *tickets = nullptr;           // one counter per (sequence, KV head), zero between launches
    bool tickets_ready = false;                // zeroed by the first decode call (lt_create enqueues nothing)
    int64_t splits_cap = 0;
    int32_t keys_full = 0, keys_lazy = 0;      // 0 = heuristic
    bool out_bf16 = false;                     // decode outputs are bf16 instead of fp32
    bool shared_tail = true;                   // long key ranges end in a part the wavefronts share (lt_set_shared_tail)
    int32_t decode_path = LT_DECODE_AUTO;      // which decode kernel (lt_set_decode_path)
    bool profiling = false;
    std::vector<EventPair> events;             // pool, created on first enable
    size_t events_used = 0;
    // online mode (lt_create_online): layers take storage on demand from two pools of slots
    bool online = false;
    uint8_t *full_pool = nullptr, *ring_pool = nullptr;
    std::vector<uint8_t> full_used, ring_used;
    // paged mode (lt_create_paged): full layers are pools of pages addressed through one block table
    bool paged = false;
    int32_t page_shift = 0, n_pages = 0, max_pages = 0;
    int32_t *table_dev = nullptr;              // [B][max_pages], inside the slab
    std::vector<int32_t> table_host;           // the copy the host checks lengths against; -1 = no page
};

// Max-priority queue of (ratio, layer) with a fixed capacity; small, so a plain vector.
struct lt_queue {
    int32_t capacity = 0;
    std::vector<std::pair<float, int32_t>> entries;
};

static void bind_workspace(lt_ctx *ctx, void *workspace)
{
    const lt_config *cfg = &ctx->cfg;
    ctx->splits_cap = max_splits(cfg);
    const size_t rows = (size_t)cfg->batch * cfg->n_q_heads * (size_t)ctx->splits_cap;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    ctx->part_acc = static_cast<float *>(workspace);
    ctx->part_ml = reinterpret_cast<float *>(ws + align_up(rows * ltk::kHeadDim * sizeof(float)));
    ctx->tickets = reinterpret_cast<unsigned int *>(ws + align_up(rows * ltk::kHeadDim * sizeof(float)) +
                                                    align_up(rows * 2 * sizeof(float)));
}

namespace {

// Online mode: give a layer without storage a free full-size slot.
lt_status assign_full_slot(lt_ctx *ctx, Layer &l)
{
    for (size_t i = 0; i < ctx->full_used.size(); ++i) {
        if (ctx->full_used[i]) continue;
        ctx->full_used[i] = 1;
        const size_t bytes = block_bytes(&ctx->cfg, false);
        uint8_t *base = ctx->full_pool + i * 2 * bytes;
        l.k = reinterpret_cast<uint16_t *>(base);
        l.v = reinterpret_cast<uint16_t *>(base + bytes);
        l.slot = (int32_t)i;
        return LT_OK;
    }
    return LT_ERR_CAPACITY;
}

// Keys per workgroup.  Measured on MI355X, the decode kernel streams fastest with ONE workgroup
// (four wavefronts, 16 KB of loads in flight each) per compute unit reading one long contiguous
// range: 256 workgroups reach 6.6 TB/s where 512 or 768 reach 6.1-6.2 TB/s.  So each of the
// `streams` = B * Hkv key streams is cut into 256 / streams ranges; more streams than compute
// units means one range per stream.  Short ranges are not cut below `lo` keys.
int choose_keys_per_block(int64_t stored, int64_t streams, bool lazy, int64_t splits_cap, int group)
{
    constexpr int64_t workgroups = 256;                        // one per compute unit
    // a window of 2048 entries at batch 1 (eight streams): 32 ranges of 64 keys are 3-7 % faster than 16 of 128 with
    // up to five heads per group (8.7 / 9.4 / 9.8 / 11.6 against 9.0 / 9.9 / 10.5 / 12.1 us for 1 / 2 / 4 / 5 heads),
    // and slower with eight
    const int64_t lo = lazy ? (group <= 5 ? kMinKeysLazy : 2 * kMinKeysLazy) : kMinKeysFull;
    const int64_t splits = std::max<int64_t>(workgroups / streams, 1);
    int64_t keys = ceil_div(ceil_div(stored, splits), ltk::kKeyGranule) * ltk::kKeyGranule;
    keys = std::max(keys, lo);
    keys = std::max(keys, ceil_div(ceil_div(stored, splits_cap), ltk::kKeyGranule) * ltk::kKeyGranule);
    return (int)keys;
}

struct ScopedEvents {
    lt_ctx *ctx;
    hipStream_t stream;
    EventPair *pair = nullptr;
    ScopedEvents(lt_ctx *c, hipStream_t s, int32_t kernel) : ctx(c), stream(s)
    {
        if (!ctx->profiling) return;
        if (ctx->events_used == ctx->events.size() && ctx->events.size() < (size_t)kMaxEventPairs) {
            // a new pair, made when a launch needs it (room for it was reserved by lt_profile_enable); kept for reuse
            EventPair p{};
            if (hipEventCreate(&p.start) != hipSuccess) return;
            if (hipEventCreate(&p.stop) != hipSuccess) {
                (void)hipEventDestroy(p.start);
                return;
            }
            ctx->events.push_back(p);
        }
        if (ctx->events_used < ctx->events.size()) {
            pair = &ctx->events[ctx->events_used++];
            pair->kernel = kernel;
            (void)hipEventRecord(pair->start, stream);
        }
    }
    ~ScopedEvents()
    {
        if (pair != nullptr) (void)hipEventRecord(pair->stop, stream);
    }
};

}  // namespace

extern "C" {

const char *lt_status_str(lt_status s)
{
    switch (s) {
    case LT_OK: return "ok";
    case LT_ERR_INVALID_ARG: return "invalid argument";
    case LT_ERR_SHAPE: return "shapes do not fit together";
    case LT_ERR_CAPACITY: return "capacity exceeded";
    case LT_ERR_STATE: return "call out of order";
    case LT_ERR_HIP: return "HIP runtime error";
    case LT_ERR_NOMEM: return "host allocation failed";
    }
    return "unknown status";
}

size_t lt_kv_bytes(const lt_config *cfg, const uint8_t *is_lazy)
{
    if (!config_ok(cfg) || config_shape(cfg) != LT_OK || is_lazy == nullptr) return 0;
    size_t total = 0;
    for (int i = 0; i < cfg->n_layers; ++i) total += 2 * block_bytes(cfg, is_lazy[i] != 0);
    return total;
}

size_t lt_workspace_bytes(const lt_config *cfg)
{
    if (!config_ok(cfg) || config_shape(cfg) != LT_OK) return 0;
    const size_t rows = (size_t)cfg->batch * cfg->n_q_heads * (size_t)max_splits(cfg);
    return align_up(rows * ltk::kHeadDim * sizeof(float)) + align_up(rows * 2 * sizeof(float)) +
           align_up((size_t)cfg->batch * cfg->n_kv_heads * ltk::kTicketStride * sizeof(unsigned int));
}

lt_status lt_create(const lt_config *cfg, const uint8_t *is_lazy, void *kv_slab, size_t kv_bytes, void *workspace,
                    size_t ws_bytes, lt_ctx **out)
{
    if (out == nullptr) return LT_ERR_INVALID_ARG;
    *out = nullptr;
    if (!config_ok(cfg) || is_lazy == nullptr || kv_slab == nullptr || workspace == nullptr) return LT_ERR_INVALID_ARG;
    const lt_status shape = config_shape(cfg);
    if (shape != LT_OK) return shape;
    if (((uintptr_t)kv_slab % kAlign) != 0 || ((uintptr_t)workspace % kAlign) != 0) return LT_ERR_INVALID_ARG;
    if (kv_bytes < lt_kv_bytes(cfg, is_lazy) || ws_bytes < lt_workspace_bytes(cfg)) return LT_ERR_CAPACITY;

    lt_ctx *ctx = new (std::nothrow) lt_ctx();
    if (ctx == nullptr) return LT_ERR_NOMEM;
    ctx->cfg = *cfg;
    ctx->cfg.softmax_scale = effective_scale(cfg);
    try {
        ctx->layers.resize(cfg->n_layers);
    } catch (const std::bad_alloc &) {
        delete ctx;
        return LT_ERR_NOMEM;
    }
    uint8_t *cursor = static_cast<uint8_t *>(kv_slab);
    for (int i = 0; i < cfg->n_layers; ++i) {
        Layer &l = ctx->layers[i];
        l.lazy = is_lazy[i] != 0;
        l.capacity = layer_capacity(cfg, l.lazy);
        const size_t bytes = block_bytes(cfg, l.lazy);
        l.k = reinterpret_cast<uint16_t *>(cursor);
        l.v = reinterpret_cast<uint16_t *>(cursor + bytes);
        cursor += 2 * bytes;
    }
    bind_workspace(ctx, workspace);
    *out = ctx;
    return LT_OK;
}

size_t lt_kv_bytes_online(const lt_config *cfg, int32_t n_full)
{
    if (!config_ok(cfg) || config_shape(cfg) != LT_OK || n_full < 0 || n_full > cfg->n_layers) return 0;
    const int32_t full_slots = std::min(n_full + 1, cfg->n_layers);
    return (size_t)full_slots * 2 * block_bytes(cfg, false) + (size_t)(cfg->n_layers - n_full) * 2 * block_bytes(cfg, true);
}

lt_status lt_create_online(const lt_config *cfg, int32_t n_full, void *kv_slab, size_t kv_bytes, void *workspace,
                           size_t ws_bytes, lt_ctx **out)
{
    if (out == nullptr) return LT_ERR_INVALID_ARG;
    *out = nullptr;
    if (!config_ok(cfg) || kv_slab == nullptr || workspace == nullptr || n_full < 0) return LT_ERR_INVALID_ARG;
    const lt_status shape = config_shape(cfg);
    if (shape != LT_OK) return shape;
    if (n_full > cfg->n_layers) return LT_ERR_INVALID_ARG;
    if (((uintptr_t)kv_slab % kAlign) != 0 || ((uintptr_t)workspace % kAlign) != 0) return LT_ERR_INVALID_ARG;
    if (kv_bytes < lt_kv_bytes_online(cfg, n_full) || ws_bytes < lt_workspace_bytes(cfg)) return LT_ERR_CAPACITY;

    lt_ctx *ctx = new (std::nothrow) lt_ctx();
    if (ctx == nullptr) return LT_ERR_NOMEM;
    ctx->cfg = *cfg;
    ctx->cfg.softmax_scale = effective_scale(cfg);
    ctx->online = true;
    const int32_t full_slots = std::min(n_full + 1, cfg->n_layers);
    try {
        ctx->layers.resize(cfg->n_layers);
        ctx->full_used.assign(full_slots, 0);
        ctx->ring_used.assign(cfg->n_layers - n_full, 0);
    } catch (const std::bad_alloc &) {
        delete ctx;
        return LT_ERR_NOMEM;
    }
    ctx->full_pool = static_cast<uint8_t *>(kv_slab);
    ctx->ring_pool = ctx->full_pool + (size_t)full_slots * 2 * block_bytes(cfg, false);
    for (Layer &l : ctx->layers) l.capacity = cfg->max_tokens;          // every layer starts out full, without storage
    bind_workspace(ctx, workspace);
    *out = ctx;
    return LT_OK;
}

// ---- paged storage for the full layers ------------------------------------------------------------

static bool paged_args_ok(const lt_config *cfg, const uint8_t *is_lazy, int32_t page_tokens, int32_t n_pages)
{
    if (!config_ok(cfg) || config_shape(cfg) != LT_OK || is_lazy == nullptr) return false;
    if (page_tokens < 64 || page_tokens > (1 << 20) || (page_tokens & (page_tokens - 1)) != 0 || n_pages <= 0) return false;
    if (cfg->batch > ltk::kMaxRaggedBatch) return false;
    return true;
}

static size_t page_pool_bytes(const lt_config *cfg, int32_t page_tokens, int32_t n_pages)
{
    return align_up((size_t)n_pages * cfg->n_kv_heads * (size_t)page_tokens * ltk::kHeadDim * sizeof(uint16_t));
}

static size_t block_table_bytes(const lt_config *cfg, int32_t page_tokens)
{
    return align_up((size_t)cfg->batch * (size_t)ceil_div(cfg->max_tokens, page_tokens) * sizeof(int32_t));
}

size_t lt_kv_bytes_paged(const lt_config *cfg, const uint8_t *is_lazy, int32_t page_tokens, int32_t n_pages)
{
    if (!paged_args_ok(cfg, is_lazy, page_tokens, n_pages)) return 0;
    size_t total = block_table_bytes(cfg, page_tokens);
    for (int i = 0; i < cfg->n_layers; ++i)
        total += is_lazy[i] != 0 ? 2 * block_bytes(cfg, true) : 2 * page_pool_bytes(cfg, page_tokens, n_pages);
    return total;
}

lt_status lt_create_paged(const lt_config *cfg, const uint8_t *is_lazy, int32_t page_tokens, int32_t n_pages, void *kv_slab,
                          size_t kv_bytes, void *workspace, size_t ws_bytes, lt_ctx **out)
{
    if (out == nullptr) return LT_ERR_INVALID_ARG;
    *out = nullptr;
    if (!config_ok(cfg) || is_lazy == nullptr || kv_slab == nullptr || workspace == nullptr) return LT_ERR_INVALID_ARG;
    const lt_status shape = config_shape(cfg);
    if (shape != LT_OK) return shape;
    if (page_tokens <= 0 || n_pages <= 0) return LT_ERR_INVALID_ARG;
    if (!paged_args_ok(cfg, is_lazy, page_tokens, n_pages)) return LT_ERR_SHAPE;
    // a workgroup's key range may touch kMaxRangePages pages and a sequence is cut into at most max_splits ranges
    if (cfg->max_tokens > max_splits(cfg) * (int64_t)(ltk::kMaxRangePages - 1) * page_tokens) return LT_ERR_SHAPE;
    if (((uintptr_t)kv_slab % kAlign) != 0 || ((uintptr_t)workspace % kAlign) != 0) return LT_ERR_INVALID_ARG;
    if (kv_bytes < lt_kv_bytes_paged(cfg, is_lazy, page_tokens, n_pages) || ws_bytes < lt_workspace_bytes(cfg)) return LT_ERR_CAPACITY;

    lt_ctx *ctx = new (std::nothrow) lt_ctx();
    if (ctx == nullptr) return LT_ERR_NOMEM;
    ctx->cfg = *cfg;
    ctx->cfg.softmax_scale = effective_scale(cfg);
    ctx->paged = true;
    ctx->n_pages = n_pages;
    ctx->max_pages = (int32_t)ceil_div(cfg->max_tokens, page_tokens);
    while ((1 << ctx->page_shift) < page_tokens) ++ctx->page_shift;
    try {
        ctx->layers.resize(cfg->n_layers);
        ctx->table_host.assign((size_t)cfg->batch * ctx->max_pages, -1);
        for (Layer &l : ctx->layers) l.total_b.assign((size_t)cfg->batch, 0);   // lengths are always per sequence here
    } catch (const std::bad_alloc &) {
        delete ctx;
        return LT_ERR_NOMEM;
    }
    uint8_t *cursor = static_cast<uint8_t *>(kv_slab);
    ctx->table_dev = reinterpret_cast<int32_t *>(cursor);
    cursor += block_table_bytes(cfg, page_tokens);
    for (int i = 0; i < cfg->n_layers; ++i) {
        Layer &l = ctx->layers[i];
        l.lazy = is_lazy[i] != 0;
        l.capacity = l.lazy ? window_of(cfg) : (int64_t)ctx->max_pages * page_tokens;
        const size_t bytes = l.lazy ? block_bytes(cfg, true) : page_pool_bytes(cfg, page_tokens, n_pages);
        l.k = reinterpret_cast<uint16_t *>(cursor);
        l.v = reinterpret_cast<uint16_t *>(cursor + bytes);
        cursor += 2 * bytes;
    }
    bind_workspace(ctx, workspace);
    *out = ctx;
    return LT_OK;
}

// The pages that tokens [have, want) of a sequence fall into are present in the host copy of the block table.
// (The pages of tokens below `have` were checked when those tokens arrived, and lt_set_block_table refuses a
// table that drops them.)
static bool pages_cover(const lt_ctx *ctx, int32_t sequence, int64_t have, int64_t want)
{
    if (want <= have) return true;
    const int64_t first = have >> ctx->page_shift, last = (want - 1) >> ctx->page_shift;
    if (last >= ctx->max_pages) return false;
    for (int64_t p = first; p <= last; ++p)
        if (ctx->table_host[(size_t)sequence * ctx->max_pages + p] < 0) return false;
    return true;
}

lt_status lt_set_block_table(lt_ctx *ctx, const int32_t *table_host, void *stream)
{
    if (ctx == nullptr || table_host == nullptr) return LT_ERR_INVALID_ARG;
    if (!ctx->paged) return LT_ERR_STATE;
    const size_t entries = (size_t)ctx->cfg.batch * ctx->max_pages;
    for (size_t i = 0; i < entries; ++i)
        if (table_host[i] < -1 || table_host[i] >= ctx->n_pages) return LT_ERR_INVALID_ARG;
    // a page that holds tokens must stay named: every sequence keeps the pages its longest full layer has filled
    for (int32_t b = 0; b < ctx->cfg.batch; ++b) {
        int64_t longest = 0;
        for (const Layer &l : ctx->layers)
            if (!l.lazy) longest = std::max(longest, l.total_b[b]);
        const int64_t pages = (longest + ((int64_t)1 << ctx->page_shift) - 1) >> ctx->page_shift;
        for (int64_t p = 0; p < pages; ++p)
            if (table_host[(size_t)b * ctx->max_pages + p] < 0) return LT_ERR_STATE;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // kernels enqueued earlier may still read the old table; the host copy must not change under the transfer either
    if (hipStreamSynchronize(s) != hipSuccess) return LT_ERR_HIP;
    std::copy(table_host, table_host + entries, ctx->table_host.begin());
    if (hipMemcpyAsync(ctx->table_dev, ctx->table_host.data(), entries * sizeof(int32_t), hipMemcpyHostToDevice, s) != hipSuccess)
        return LT_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return LT_ERR_HIP;
    return LT_OK;
}

lt_status lt_reset_sequence(lt_ctx *ctx, int32_t sequence)
{
    if (ctx == nullptr || sequence < 0 || sequence >= ctx->cfg.batch) return LT_ERR_INVALID_ARG;
    if (ctx->online) return LT_ERR_STATE;      // online identification works on whole batches of equal length
    if (ctx->cfg.batch > ltk::kMaxRaggedBatch) return LT_ERR_SHAPE;
    try {
        for (Layer &l : ctx->layers)
            if (l.total_b.empty()) l.total_b.assign((size_t)ctx->cfg.batch, l.total);
    } catch (const std::bad_alloc &) {
        return LT_ERR_NOMEM;
    }
    for (Layer &l : ctx->layers) {
        l.total_b[sequence] = 0;
        l.total = *std::max_element(l.total_b.begin(), l.total_b.end());
    }
    return LT_OK;
}

void lt_destroy(lt_ctx *ctx)
{
    if (ctx == nullptr) return;
    for (EventPair &p : ctx->events) {
        (void)hipEventDestroy(p.start);
        (void)hipEventDestroy(p.stop);
    }
    delete ctx;
}

lt_status lt_reset(lt_ctx *ctx)
{
    if (ctx == nullptr) return LT_ERR_INVALID_ARG;
    for (Layer &l : ctx->layers) {
        l.total = 0;
        if (ctx->paged) std::fill(l.total_b.begin(), l.total_b.end(), 0);
        else l.total_b.clear();
        if (ctx->online) {                      // back to "full, no storage yet"
            l.k = l.v = nullptr;
            l.slot = -1;
            l.lazy = false;
            l.capacity = ctx->cfg.max_tokens;
        }
    }
    std::fill(ctx->full_used.begin(), ctx->full_used.end(), 0);
    std::fill(ctx->ring_used.begin(), ctx->ring_used.end(), 0);
    // the next decode call zeroes the split counters again: a launch that failed half-way may have left some taken
    ctx->tickets_ready = false;
    return LT_OK;
}

lt_status lt_layer_len(const lt_ctx *ctx, int32_t layer, int64_t *total_tokens, int64_t *stored_tokens)
{
    if (ctx == nullptr || layer < 0 || layer >= ctx->cfg.n_layers) return LT_ERR_INVALID_ARG;
    const Layer &l = ctx->layers[layer];
    if (total_tokens != nullptr) *total_tokens = l.total;
    if (stored_tokens != nullptr) *stored_tokens = std::min(l.total, l.capacity);
    return LT_OK;
}

lt_status lt_layer_view(const lt_ctx *ctx, int32_t layer, void **k_dev, void **v_dev, int64_t *stride_b, int64_t *stride_h,
                        int64_t *capacity, int32_t *is_lazy)
{
    if (ctx == nullptr || layer < 0 || layer >= ctx->cfg.n_layers) return LT_ERR_INVALID_ARG;
    const Layer &l = ctx->layers[layer];
    if (k_dev != nullptr) *k_dev = l.k;
    if (v_dev != nullptr) *v_dev = l.v;
    const int64_t head_tokens = ctx->paged && !l.lazy ? (int64_t)1 << ctx->page_shift : l.capacity;
    if (stride_h != nullptr) *stride_h = head_tokens * ltk::kHeadDim;
    if (stride_b != nullptr) *stride_b = head_tokens * ltk::kHeadDim * ctx->cfg.n_kv_heads;
    if (capacity != nullptr) *capacity = l.capacity;
    if (is_lazy != nullptr) *is_lazy = l.lazy ? 1 : 0;
    return LT_OK;
}

// ---- lazy-layer identification ---------------------------------------------------------------

// Keys per workgroup of the scoring kernel for `keys` keys per (sequence, KV head) in all.  One workgroup (eight
// wavefronts) fills a compute unit, so the B * Hkv key streams are cut into about 256 ranges of equal length, multiples
// of kScoreTileKeys; more streams than compute units: one range each.
static int score_keys_per_block(const lt_config *cfg, int64_t keys)
{
    const int64_t streams = (int64_t)cfg->batch * cfg->n_kv_heads;
    const int64_t ranges = std::max<int64_t>(256 / streams, 1);
    const int64_t per = ceil_div(ceil_div(keys, ranges), ltk::kScoreTileKeys) * ltk::kScoreTileKeys;
    return (int)std::max<int64_t>(per, ltk::kScoreTileKeys);
}

// Workspace of a scoring call with `chunks` key ranges: partial sums, per-head sums of rho, counters.
struct ScoreWorkspace {
    size_t part_bytes, head_bytes, ticket_bytes;
    size_t total() const { return part_bytes + head_bytes + ticket_bytes; }
};

static ScoreWorkspace score_workspace(const lt_config *cfg, int64_t chunks, int32_t w_last)
{
    ScoreWorkspace w;
    w.part_bytes = align_up((size_t)cfg->batch * cfg->n_q_heads * (size_t)w_last * (size_t)chunks * 3 * sizeof(float));
    w.head_bytes = align_up((size_t)cfg->batch * cfg->n_q_heads * sizeof(float));
    w.ticket_bytes = align_up(((size_t)cfg->batch * cfg->n_kv_heads + 1) * sizeof(unsigned int));
    return w;
}

static void bind_score_workspace(ltk::ScoreArgs &a, const lt_config *cfg, void *workspace)
{
    const ScoreWorkspace w = score_workspace(cfg, a.n_chunks, a.w_last);
    uint8_t *base = static_cast<uint8_t *>(workspace);
    a.part = reinterpret_cast<float *>(base);
    a.head_scratch = reinterpret_cast<float *>(base + w.part_bytes);
    a.tickets = reinterpret_cast<unsigned int *>(base + w.part_bytes + w.head_bytes);
}

size_t lt_lazy_ratio_workspace_bytes(const lt_config *cfg, int64_t n, int32_t w_last)
{
    if (!config_ok(cfg) || config_shape(cfg) != LT_OK || n <= 0 || w_last <= 0 || w_last > 64) return 0;
    return score_workspace(cfg, ceil_div(n, score_keys_per_block(cfg, n)), w_last).total();
}

// The dense form behind lt_lazy_ratio and lt_lazy_ratio_static.  workspace == nullptr selects the library's
// built-in scratch array (and its fixed size) instead of a caller's buffer.
static lt_status lazy_ratio_dense(const lt_config *cfg, const void *q_last, const void *k, int64_t k_stride_b, int64_t k_stride_h,
                                  int64_t k_stride_t, int64_t n, int32_t w_last, lt_ratio_mode mode, void *workspace, size_t ws_bytes,
                                  float *rho_dev, float *ratio_seq_dev, float *ratio_mean_dev, void *stream)
{
    if (!config_ok(cfg) || q_last == nullptr || k == nullptr || ratio_mean_dev == nullptr) return LT_ERR_INVALID_ARG;
    if (mode != LT_RECENT_PER_QUERY && mode != LT_RECENT_FIXED) return LT_ERR_INVALID_ARG;
    if (n <= 0 || w_last <= 0 || k_stride_b < 0 || k_stride_h < 0 || k_stride_t <= 0) return LT_ERR_INVALID_ARG;
    const lt_status shape = config_shape(cfg);
    if (shape != LT_OK) return shape;
    if (w_last > n || w_last > 64 || n > kMaxTokens) return LT_ERR_SHAPE;
    if (k_stride_t < ltk::kHeadDim || (k_stride_b % 8) != 0 || (k_stride_h % 8) != 0 || (k_stride_t % 8) != 0) return LT_ERR_SHAPE;
    if (((uintptr_t)q_last % 16) != 0 || ((uintptr_t)k % 16) != 0 || ((uintptr_t)workspace % kAlign) != 0) return LT_ERR_INVALID_ARG;
    if (ws_bytes < lt_lazy_ratio_workspace_bytes(cfg, n, w_last)) return LT_ERR_CAPACITY;
    if (workspace == nullptr && ltk::static_scratch(&workspace) != hipSuccess) return LT_ERR_HIP;

    ltk::ScoreArgs a{};
    a.q_last = static_cast<const uint16_t *>(q_last);
    a.k = static_cast<const uint16_t *>(k);
    a.k_stride_b = k_stride_b;
    a.k_stride_h = k_stride_h;
    a.k_stride_t = k_stride_t;
    a.n = n;
    a.w_last = w_last;
    a.batch = cfg->batch;
    a.n_q_heads = cfg->n_q_heads;
    a.n_kv_heads = cfg->n_kv_heads;
    a.w_sink = cfg->w_sink;
    a.w_recent = cfg->w_recent;
    a.fixed_mode = mode == LT_RECENT_FIXED ? 1 : 0;
    a.keys_per_block = score_keys_per_block(cfg, n);
    a.n_chunks = (int32_t)ceil_div(n, a.keys_per_block);
    a.range_a_end = n;
    a.range_b_begin = n;
    a.n_chunks_a = a.n_chunks;
    a.scale_log2e = effective_scale(cfg) * kLog2e;
    bind_score_workspace(a, cfg, workspace);
    a.rho = rho_dev;
    a.ratio_seq = ratio_seq_dev;
    a.ratio_mean = ratio_mean_dev;
    return ltk::lazy_ratio(a, static_cast<hipStream_t>(stream)) == hipSuccess ? LT_OK : LT_ERR_HIP;
}

lt_status lt_lazy_ratio(const lt_config *cfg, const void *q_last, const void *k, int64_t k_stride_b, int64_t k_stride_h,
                        int64_t k_stride_t, int64_t n, int32_t w_last, lt_ratio_mode mode, void *workspace, size_t ws_bytes,
                        float *rho_dev, float *ratio_seq_dev, float *ratio_mean_dev, void *stream)
{
    if (workspace == nullptr) return LT_ERR_INVALID_ARG;
    return lazy_ratio_dense(cfg, q_last, k, k_stride_b, k_stride_h, k_stride_t, n, w_last, mode, workspace, ws_bytes, rho_dev,
                            ratio_seq_dev, ratio_mean_dev, stream);
}

lt_status lt_lazy_ratio_static(const lt_config *cfg, const void *q_last, const void *k, int64_t k_stride_b, int64_t k_stride_h,
                               int64_t k_stride_t, int64_t n, int32_t w_last, lt_ratio_mode mode, float *rho_dev,
                               float *ratio_seq_dev, float *ratio_mean_dev, void *stream)
{
    // a problem whose partial results do not fit the built-in array is refused (LT_ERR_CAPACITY) before anything is looked up
    return lazy_ratio_dense(cfg, q_last, k, k_stride_b, k_stride_h, k_stride_t, n, w_last, mode, nullptr, ltk::kStaticScratchBytes,
                            rho_dev, ratio_seq_dev, ratio_mean_dev, stream);
}

// Key ranges the window-only form touches: the tiles holding the first w_sink keys and the tiles from
// the earliest recent key of any scored query to the end of the prompt (disjoint, tile-aligned).
struct WindowPlan {
    int64_t a_end, b_begin;
    int32_t keys_per_block, chunks_a, chunks_b;
};

static WindowPlan window_plan(const lt_config *cfg, int64_t n, int32_t w_last, lt_ratio_mode mode)
{
    const int64_t tile = ltk::kScoreTileKeys;
    WindowPlan p{};
    p.a_end = std::min<int64_t>(n, ceil_div(cfg->w_sink, tile) * tile);
    int64_t first_recent = mode == LT_RECENT_FIXED ? n - cfg->w_recent : n - w_last - (int64_t)cfg->w_recent + 1;
    first_recent = std::min<int64_t>(std::max<int64_t>(first_recent, 0), n);
    p.b_begin = std::max<int64_t>(p.a_end, first_recent / tile * tile);
    p.keys_per_block = score_keys_per_block(cfg, p.a_end + (n - p.b_begin));
    // Each of the two parts is cut on its own, so their ranges can add up to more than one workgroup per compute
    // unit; the surplus would run as a second round after the first, on a call that is all fixed cost.  Longer
    // ranges until the workgroups fit in one round (or each part is a single range).
    const int64_t streams = (int64_t)cfg->batch * cfg->n_kv_heads;
    for (;;) {
        p.chunks_a = (int32_t)ceil_div(p.a_end, p.keys_per_block);
        p.chunks_b = (int32_t)ceil_div(n - p.b_begin, p.keys_per_block);
        if ((p.chunks_a + p.chunks_b) * streams <= 256 || (p.chunks_a <= 1 && p.chunks_b <= 1)) break;
        p.keys_per_block += (int32_t)tile;
    }
    return p;
}

size_t lt_lazy_ratio_lse_workspace_bytes(const lt_config *cfg, int64_t n, int32_t w_last)
{
    if (!config_ok(cfg) || config_shape(cfg) != LT_OK || n <= 0 || w_last <= 0 || w_last > 64 || w_last > n) return 0;
    const WindowPlan p = window_plan(cfg, n, w_last, LT_RECENT_PER_QUERY), f = window_plan(cfg, n, w_last, LT_RECENT_FIXED);
    const int64_t chunks = std::max(p.chunks_a + p.chunks_b, f.chunks_a + f.chunks_b);       // either reading fits
    return score_workspace(cfg, chunks, w_last).total();
}

lt_status lt_lazy_ratio_lse(const lt_config *cfg, const void *q_last, const void *k, int64_t k_stride_b, int64_t k_stride_h,
                            int64_t k_stride_t, int64_t n, int32_t w_last, lt_ratio_mode mode, const float *lse_rows,
                            int64_t lse_stride_b, int64_t lse_stride_h, void *workspace, size_t ws_bytes, float *rho_dev,
                            float *ratio_seq_dev, float *ratio_mean_dev, void *stream)
{
    if (!config_ok(cfg) || q_last == nullptr || k == nullptr || lse_rows == nullptr || workspace == nullptr ||
        ratio_mean_dev == nullptr)
        return LT_ERR_INVALID_ARG;
    if (mode != LT_RECENT_PER_QUERY && mode != LT_RECENT_FIXED) return LT_ERR_INVALID_ARG;
    if (n <= 0 || w_last <= 0 || k_stride_b < 0 || k_stride_h < 0 || k_stride_t <= 0 || lse_stride_b < 0 || lse_stride_h < 0)
        return LT_ERR_INVALID_ARG;
    const lt_status shape = config_shape(cfg);
    if (shape != LT_OK) return shape;
    if (w_last > n || w_last > 64 || n > kMaxTokens) return LT_ERR_SHAPE;
    if (k_stride_t < ltk::kHeadDim || (k_stride_b % 8) != 0 || (k_stride_h % 8) != 0 || (k_stride_t % 8) != 0) return LT_ERR_SHAPE;
    if (((uintptr_t)q_last % 16) != 0 || ((uintptr_t)k % 16) != 0 || ((uintptr_t)lse_rows % 4) != 0 ||
        ((uintptr_t)workspace % kAlign) != 0)
        return LT_ERR_INVALID_ARG;
    if (ws_bytes < lt_lazy_ratio_lse_workspace_bytes(cfg, n, w_last)) return LT_ERR_CAPACITY;

    const WindowPlan p = window_plan(cfg, n, w_last, mode);
    ltk::ScoreArgs a{};
    a.q_last = static_cast<const uint16_t *>(q_last);
    a.k = static_cast<const uint16_t *>(k);
    a.k_stride_b = k_stride_b;
    a.k_stride_h = k_stride_h;
    a.k_stride_t = k_stride_t;
    a.n = n;
    a.w_last = w_last;
    a.batch = cfg->batch;
    a.n_q_heads = cfg->n_q_heads;
    a.n_kv_heads = cfg->n_kv_heads;
    a.w_sink = cfg->w_sink;
    a.w_recent = cfg->w_recent;
    a.fixed_mode = mode == LT_RECENT_FIXED ? 1 : 0;
    a.keys_per_block = p.keys_per_block;
    a.n_chunks = p.chunks_a + p.chunks_b;
    a.range_a_end = p.a_end;
    a.range_b_begin = p.b_begin;
    a.n_chunks_a = p.chunks_a;
    a.lse_rows = lse_rows;
    a.lse_stride_b = lse_stride_b;
    a.lse_stride_h = lse_stride_h;
    a.scale_log2e = effective_scale(cfg) * kLog2e;
    bind_score_workspace(a, cfg, workspace);
    a.rho = rho_dev;
    a.ratio_seq = ratio_seq_dev;
    a.ratio_mean = ratio_mean_dev;
    return ltk::lazy_ratio(a, static_cast<hipStream_t>(stream)) == hipSuccess ? LT_OK : LT_ERR_HIP;
}

// ---- prefill attention -------------------------------------------------------------------------

lt_status lt_prefill_attn(const lt_config *cfg, const void *q, const void *k, const void *v, int64_t kv_stride_b,
                          int64_t kv_stride_h, int64_t kv_stride_t, int64_t n, int64_t n_queries, lt_mask_mode mask,
                          lt_out_dtype out_dtype, void *out, float *lse_out, void *stream)
{
    if (!config_ok(cfg) || q == nullptr || k == nullptr || v == nullptr || out == nullptr) return LT_ERR_INVALID_ARG;
    if (mask != LT_MASK_CAUSAL && mask != LT_MASK_STREAMING) return LT_ERR_INVALID_ARG;
    if (out_dtype != LT_OUT_BF16 && out_dtype != LT_OUT_F32) return LT_ERR_INVALID_ARG;
    if (n <= 0 || n_queries <= 0 || kv_stride_b < 0 || kv_stride_h < 0 || kv_stride_t <= 0) return LT_ERR_INVALID_ARG;
    const lt_status shape = config_shape(cfg);
    if (shape != LT_OK) return shape;
    if (n > kMaxTokens || n_queries > n) return LT_ERR_SHAPE;
    if (mask == LT_MASK_STREAMING && cfg->w_sink + cfg->w_recent < 1) return LT_ERR_SHAPE;
    if (kv_stride_t < ltk::kHeadDim || kv_stride_t >= ((int64_t)1 << 24) || (kv_stride_b % 8) != 0 || (kv_stride_h % 8) != 0 ||
        (kv_stride_t % 8) != 0)
        return LT_ERR_SHAPE;
    if (((uintptr_t)q % 16) != 0 || ((uintptr_t)k % 16) != 0 || ((uintptr_t)v % 16) != 0 || ((uintptr_t)out % 16) != 0 ||
        ((uintptr_t)lse_out % 4) != 0)
        return LT_ERR_INVALID_ARG;
    const int64_t blocks = ceil_div(n_queries, 32) * cfg->n_kv_heads * cfg->batch;     // upper bound of the grid
    if (blocks + 8 > (int64_t)0x7fffffff) return LT_ERR_SHAPE;

    ltk::PrefillArgs a{};
    a.q = static_cast<const uint16_t *>(q);
    a.k = static_cast<const uint16_t *>(k);
    a.v = static_cast<const uint16_t *>(v);
    a.kv_stride_b = kv_stride_b;
    a.kv_stride_h = kv_stride_h;
    a.kv_stride_t = kv_stride_t;
    a.out = out;
    a.lse = lse_out;
    a.n = n;
    a.n_q = n_queries;
    a.batch = cfg->batch;
    a.n_q_heads = cfg->n_q_heads;
    a.n_kv_heads = cfg->n_kv_heads;
    a.streaming = mask == LT_MASK_STREAMING ? 1 : 0;
    a.w_sink = cfg->w_sink;
    a.w_recent = cfg->w_recent;
    a.out_f32 = out_dtype == LT_OUT_F32 ? 1 : 0;
    a.scale_log2e = effective_scale(cfg) * kLog2e;
    return ltk::prefill_attn(a, static_cast<hipStream_t>(stream)) == hipSuccess ? LT_OK : LT_ERR_HIP;
}

lt_status lt_select_lazy(const float *ratios_host, int32_t n_layers, int32_t n_lazy, uint8_t *is_lazy_out, int32_t *order_out)
{
    if (ratios_host == nullptr || is_lazy_out == nullptr || n_layers <= 0 || n_lazy < 0 || n_lazy > n_layers)
        return LT_ERR_INVALID_ARG;
    for (int i = 0; i < n_layers; ++i)
        if (std::isnan(ratios_host[i])) return LT_ERR_INVALID_ARG;
    std::vector<int32_t> order;
    try {
        order.resize(n_layers);
    } catch (const std::bad_alloc &) {
        return LT_ERR_NOMEM;
    }
    for (int i = 0; i < n_layers; ++i) order[i] = i;
    // laziest first; equal ratios keep layer order, so ties go to the lower index
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return ratios_host[x] > ratios_host[y]; });
    std::memset(is_lazy_out, 0, (size_t)n_layers);
    for (int i = 0; i < n_lazy; ++i) is_lazy_out[order[i]] = 1;
    if (order_out != nullptr) std::memcpy(order_out, order.data(), (size_t)n_layers * sizeof(int32_t));
    return LT_OK;
}

lt_status lt_preselect_lazy(const uint8_t *is_lazy_samples, int32_t n_samples, int32_t n_layers, int32_t n_lazy,
                            uint8_t *is_lazy_out, int32_t *count_out)
{
    if (is_lazy_samples == nullptr || is_lazy_out == nullptr || n_samples <= 0 || n_layers <= 0 || n_lazy < 0 || n_lazy > n_layers)
        return LT_ERR_INVALID_ARG;
    std::vector<int32_t> count, order;
    try {
        count.assign(n_layers, 0);
        order.resize(n_layers);
    } catch (const std::bad_alloc &) {
        return LT_ERR_NOMEM;
    }
    for (int64_t s = 0; s < n_samples; ++s)
        for (int l = 0; l < n_layers; ++l) count[l] += is_lazy_samples[s * n_layers + l] != 0;
    for (int l = 0; l < n_layers; ++l) order[l] = l;
    // most frequent first; equal counts keep layer order
    std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return count[x] > count[y]; });
    std::memset(is_lazy_out, 0, (size_t)n_layers);
    for (int i = 0; i < n_lazy; ++i) is_lazy_out[order[i]] = 1;
    if (count_out != nullptr) std::memcpy(count_out, count.data(), (size_t)n_layers * sizeof(int32_t));
    return LT_OK;
}

// ---- decoding ------------------------------------------------------------------------------------

static lt_status append_impl(lt_ctx *ctx, int32_t layer, const void *k_new, const void *v_new, int64_t n_new,
                             const int64_t *n_per_seq, void *stream)
{
    if (ctx == nullptr || k_new == nullptr || v_new == nullptr || layer < 0 || layer >= ctx->cfg.n_layers || n_new <= 0)
        return LT_ERR_INVALID_ARG;
    if (((uintptr_t)k_new % 16) != 0 || ((uintptr_t)v_new % 16) != 0) return LT_ERR_INVALID_ARG;
    Layer &l = ctx->layers[layer];
    const int32_t B = ctx->cfg.batch;
    if (n_per_seq != nullptr) {
        if (ctx->online) return LT_ERR_STATE;   // online identification works on whole batches of equal length
        if (B > ltk::kMaxRaggedBatch) return LT_ERR_SHAPE;
        for (int b = 0; b < B; ++b)
            if (n_per_seq[b] < 0 || n_per_seq[b] > n_new) return LT_ERR_INVALID_ARG;
    }
    const bool ragged = n_per_seq != nullptr || !l.total_b.empty();
    if (ragged && B > ltk::kMaxRaggedBatch) return LT_ERR_SHAPE;
    if (n_new > kMaxTokens || l.total + n_new > kMaxTokens) return LT_ERR_CAPACITY;
    int64_t longest_after = l.total + n_new;
    if (ragged) {
        longest_after = 0;
        for (int b = 0; b < B; ++b) {
            const int64_t before = l.total_b.empty() ? l.total : l.total_b[b];
            longest_after = std::max(longest_after, before + (n_per_seq != nullptr ? n_per_seq[b] : n_new));
        }
    }
    if (!l.lazy && longest_after > l.capacity) return LT_ERR_CAPACITY;
    if (ctx->paged && !l.lazy)
        for (int b = 0; b < B; ++b)
            if (!pages_cover(ctx, b, l.total_b[b], l.total_b[b] + (n_per_seq != nullptr ? n_per_seq[b] : n_new))) return LT_ERR_STATE;
    if (ragged && l.total_b.empty()) {
        try {
            l.total_b.assign((size_t)B, l.total);
        } catch (const std::bad_alloc &) {
            return LT_ERR_NOMEM;
        }
    }
    if (ctx->online && l.slot < 0) {
        const lt_status st = assign_full_slot(ctx, l);
        if (st != LT_OK) return st;             // every full-size slot is taken: truncate a layer first
    }
    if (l.capacity > 0) {                       // a lazy layer with an empty window stores nothing
        ltk::AppendArgs a{};
        a.k_new = static_cast<const uint16_t *>(k_new);
        a.v_new = static_cast<const uint16_t *>(v_new);
        a.k_cache = l.k;
        a.v_cache = l.v;
        a.stride_h = l.capacity * ltk::kHeadDim;
        a.stride_b = a.stride_h * ctx->cfg.n_kv_heads;
        a.n_new = n_new;
        a.total_before = l.total;
        a.batch = B;
        a.n_kv_heads = ctx->cfg.n_kv_heads;
        a.is_lazy = l.lazy ? 1 : 0;
        a.w_sink = ctx->cfg.w_sink;
        a.w_recent = ctx->cfg.w_recent;
        a.ragged = ragged ? 1 : 0;
        if (ctx->paged && !l.lazy) {
            a.block_table = ctx->table_dev;
            a.max_pages = ctx->max_pages;
            a.page_shift = ctx->page_shift;
        }
        if (ragged)
            for (int b = 0; b < B; ++b) {
                a.n_new_b[b] = n_per_seq != nullptr ? n_per_seq[b] : n_new;
                a.total_before_b[b] = l.total_b[b];
            }
        ScopedEvents ev(ctx, static_cast<hipStream_t>(stream), LT_KERNEL_APPEND);
        if (ltk::append(a, static_cast<hipStream_t>(stream)) != hipSuccess) return LT_ERR_HIP;
    }
    if (ragged)
        for (int b = 0; b < B; ++b) l.total_b[b] += n_per_seq != nullptr ? n_per_seq[b] : n_new;
    l.total = longest_after;
    return LT_OK;
}

lt_status lt_append_kv(lt_ctx *ctx, int32_t layer, const void *k_new, const void *v_new, int64_t n_new, void *stream)
{
    return append_impl(ctx, layer, k_new, v_new, n_new, nullptr, stream);
}

lt_status lt_append_kv_ragged(lt_ctx *ctx, int32_t layer, const void *k_new, const void *v_new, int64_t n_max,
                              const int64_t *n_per_seq_host, void *stream)
{
    if (n_per_seq_host == nullptr) return LT_ERR_INVALID_ARG;
    return append_impl(ctx, layer, k_new, v_new, n_max, n_per_seq_host, stream);
}

lt_status lt_seq_len(const lt_ctx *ctx, int32_t layer, int32_t sequence, int64_t *total_tokens, int64_t *stored_tokens)
{
    if (ctx == nullptr || layer < 0 || layer >= ctx->cfg.n_layers || sequence < 0 || sequence >= ctx->cfg.batch)
        return LT_ERR_INVALID_ARG;
    const Layer &l = ctx->layers[layer];
    const int64_t total = l.total_b.empty() ? l.total : l.total_b[sequence];
    if (total_tokens != nullptr) *total_tokens = total;
    if (stored_tokens != nullptr) *stored_tokens = l.lazy ? std::min(total, window_of(&ctx->cfg)) : total;
    return LT_OK;
}

lt_status lt_set_output_dtype(lt_ctx *ctx, lt_out_dtype dtype)
{
    if (ctx == nullptr || (dtype != LT_OUT_BF16 && dtype != LT_OUT_F32)) return LT_ERR_INVALID_ARG;
    ctx->out_bf16 = dtype == LT_OUT_BF16;
    return LT_OK;
}

// Ring / growing-cache slot of the token at absolute position p, or -1 if a lazy layer drops it.
static int64_t slot_of(const lt_config &c, const Layer &l, int64_t p)
{
    if (!l.lazy || p < c.w_sink) return p;
    if (c.w_recent == 0) return -1;
    return c.w_sink + (p - c.w_sink) % c.w_recent;
}

// One launch: optional on-the-fly append of this step's token, split attention, merge.
static lt_status launch_decode(lt_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new, void *out,
                               float *lse_out, const uint8_t *active, void *stream)
{
    if (ctx == nullptr || q == nullptr || out == nullptr || layer < 0 || layer >= ctx->cfg.n_layers) return LT_ERR_INVALID_ARG;
    if (((uintptr_t)q % 16) != 0 || ((uintptr_t)k_new % 16) != 0 || ((uintptr_t)v_new % 16) != 0) return LT_ERR_INVALID_ARG;
    Layer &l = ctx->layers[layer];
    const lt_config &c = ctx->cfg;
    const bool fused = k_new != nullptr;
    if (active != nullptr) {                    // a step that skips some sequences needs a length per sequence
        if (ctx->online) return LT_ERR_STATE;
        if (c.batch > ltk::kMaxRaggedBatch) return LT_ERR_SHAPE;
        if (l.total_b.empty()) {
            try {
                l.total_b.assign((size_t)c.batch, l.total);
            } catch (const std::bad_alloc &) {
                return LT_ERR_NOMEM;
            }
        }
    }
    const bool ragged = !l.total_b.empty();
    if (ragged && c.batch > ltk::kMaxRaggedBatch) return LT_ERR_SHAPE;
    auto takes_part = [&](int b) { return active == nullptr || active[b] != 0; };
    // the longest history any sequence of this launch attends over, after the step's token
    int64_t total = l.total + (fused ? 1 : 0);
    if (ragged) {
        total = 0;
        for (int b = 0; b < c.batch; ++b)
            if (takes_part(b)) total = std::max(total, l.total_b[b] + (fused ? 1 : 0));
    }
    if (fused && (total > kMaxTokens || (!l.lazy && total > l.capacity))) return LT_ERR_CAPACITY;
    const int64_t stored = std::min(total, l.capacity);
    if (stored <= 0) return LT_ERR_STATE;
    const bool paged = ctx->paged && !l.lazy;
    if (paged && fused)
        for (int b = 0; b < c.batch; ++b)
            if (takes_part(b) && !pages_cover(ctx, b, l.total_b[b], l.total_b[b] + 1)) return LT_ERR_STATE;   // the new token has no page yet

    ltk::DecodeArgs a{};
    a.k_cache = l.k;
    a.v_cache = l.v;
    int64_t slot = fused ? slot_of(c, l, l.total) : -1;
    bool any_stored = slot >= 0;
    if (ragged && fused) {
        any_stored = false;
        for (int b = 0; b < c.batch; ++b) any_stored = any_stored || (takes_part(b) && slot_of(c, l, l.total_b[b]) >= 0);
    }
    a.k_new = any_stored ? static_cast<const uint16_t *>(k_new) : nullptr;    // a dropped token is simply not stored
    a.v_new = any_stored ? static_cast<const uint16_t *>(v_new) : nullptr;
    a.new_slot = (int32_t)slot;
    a.tickets = ctx->tickets;
    a.q = static_cast<const uint16_t *>(q);
    a.part_acc = ctx->part_acc;
    a.part_ml = ctx->part_ml;
    a.out = out;
    a.lse = lse_out;
    a.stride_h = l.capacity * ltk::kHeadDim;
    a.stride_b = a.stride_h * c.n_kv_heads;
    a.batch = c.batch;
    a.n_q_heads = c.n_q_heads;
    a.n_kv_heads = c.n_kv_heads;
    a.stored = (int32_t)stored;
    const int32_t forced = l.lazy ? ctx->keys_lazy : ctx->keys_full;
    a.keys_per_block = forced > 0 ? forced : choose_keys_per_block(stored, (int64_t)c.batch * c.n_kv_heads, l.lazy, ctx->splits_cap, c.n_q_heads / c.n_kv_heads);
    if (paged) {                                // a workgroup's range may touch at most kMaxRangePages pages
        const int64_t most = ((int64_t)(ltk::kMaxRangePages - 1) << ctx->page_shift) / ltk::kKeyGranule * ltk::kKeyGranule;
        a.keys_per_block = (int32_t)std::min<int64_t>(a.keys_per_block, most);
    }
    a.n_splits = (int32_t)ceil_div(stored, a.keys_per_block);
    a.tail_begin = INT32_MAX;
    // Which kernel.  The vector kernel's instruction count per key grows with the heads of a group: from six heads
    // on it, not the memory, bounds a long range (eight heads: 4.3 TB/s against 6.4 for the matrix-core kernel,
    // whose cost does not depend on the group), and over short ranges it bounds the end of every launch from four
    // heads on (2048 entries, batch 8: 17.0 / 17.6 / 18.2 / 20.6 us for one to four heads against 18.9-19.7 us for
    // the matrix-core kernel with any group).  The matrix-core kernel works on pairs of tiles, so with four or five
    // heads it needs more than one tile per wavefront to pay; with six or more it pays everywhere (a window of 2048
    // entries at batch 1, ranges of 128 keys, eight heads: 13.1 against 15.2 us).
    {
        const int group = c.n_q_heads / c.n_kv_heads;
        const bool short_ranges = a.keys_per_block > 16 * 8 && a.keys_per_block <= ltk::kWideBlockKeys && group >= 4;
        const bool pays = short_ranges || group >= 6;
        a.matrix_cores = ctx->decode_path == LT_DECODE_MATRIX || (ctx->decode_path == LT_DECODE_AUTO && pays) ? 1 : 0;
    }
    // Long ranges leave their last part to the shared tail (see DecodeArgs::tail_begin), which evens out the
    // workgroups' different speeds: an eighth of the keys when a workgroup's range has kMinKeysSharedTail keys or
    // more; with half of that, a quarter when a (sequence, KV head) is spread over at least kMinSplitsWideTail
    // workgroups (128K x batch 1: the many wavefronts of a pair hold two claimed pieces each at the end, so the tail
    // has to be longer to leave something to hand out), and an eighth when it is spread over half as many and a
    // piece is cheap to work through (the matrix-core kernel, or the vector kernel with at most four heads per
    // group: 32K x batch 4 gains 2-3 % either way, where five heads per group lost 1.6 %, measured).  Shorter
    // ranges, paged layers and forced splits keep every key in a fixed place.
    const bool long_ranges = a.keys_per_block >= kMinKeysSharedTail;
    const bool half_ranges = a.keys_per_block >= kMinKeysSharedTail / 2;
    const bool many_ranges = half_ranges && a.n_splits >= kMinSplitsWideTail;
    const bool cheap_pieces = a.matrix_cores || c.n_q_heads / c.n_kv_heads <= 4;
    const bool some_ranges = half_ranges && a.n_splits >= kMinSplitsWideTail / 2 && cheap_pieces;
    if (ctx->shared_tail && forced <= 0 && !paged && a.n_splits > 1 && (long_ranges || many_ranges || some_ranges)) {
        const int64_t streams = (int64_t)c.batch * c.n_kv_heads;
        const int64_t begin = (stored - stored / (many_ranges && !long_ranges ? 4 : 8)) / ltk::kKeyGranule * ltk::kKeyGranule;
        const int32_t keys = choose_keys_per_block(begin, streams, l.lazy, ctx->splits_cap, c.n_q_heads / c.n_kv_heads);
        if (ceil_div(begin, keys) > 1) {
            a.tail_begin = (int32_t)begin;
            a.keys_per_block = keys;
            a.n_splits = (int32_t)ceil_div(begin, keys);
        }
    }
    if (a.n_splits > ctx->splits_cap) return LT_ERR_CAPACITY;
    a.scale_log2e = c.softmax_scale * kLog2e;
    a.lazy_tag = l.lazy ? 1 : 0;
    a.out_bf16 = ctx->out_bf16 ? 1 : 0;
    // window over which the workgroups' start addresses are spread: the largest power of two of 4 KB tiles that
    // fits a workgroup's key range, at most 4 MB; short ranges start at pseudo-random tiles instead
    a.spread_tiles = 0;
    for (uint32_t w = 1024; w >= 128 && !paged; w >>= 1)                     // pages scatter the addresses by themselves
        if ((int64_t)w * 16 <= a.keys_per_block) { a.spread_tiles = w; break; }
    ltk::PagedArgs paged_args;
    ltk::RaggedArgs &per_seq = paged_args.lengths;
    if (ragged)
        for (int b = 0; b < c.batch; ++b) {
            const int64_t total_b = l.total_b[b] + (fused ? 1 : 0);
            // a sequence that sits this step out looks empty to the kernel: nothing read, nothing stored, out = 0
            per_seq.stored_b[b] = takes_part(b) ? (int32_t)std::min(total_b, l.capacity) : 0;
            per_seq.new_slot_b[b] = fused && takes_part(b) ? (int32_t)slot_of(c, l, l.total_b[b]) : -1;
        }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!ctx->tickets_ready) {
        if (ltk::zero_tickets(ctx->tickets, c.batch * c.n_kv_heads * ltk::kTicketStride, s) != hipSuccess) return LT_ERR_HIP;
        ctx->tickets_ready = true;
    }
    {
        ScopedEvents ev(ctx, s, l.lazy ? LT_KERNEL_DECODE_LAZY : LT_KERNEL_DECODE_FULL);
        if (paged) {
            paged_args.block_table = ctx->table_dev;
            paged_args.max_pages = ctx->max_pages;
            paged_args.page_shift = ctx->page_shift;
            a.stride_b = a.stride_h = 0;
        }
        if (ltk::decode(a, ragged && !paged ? &per_seq : nullptr, paged ? &paged_args : nullptr, s) != hipSuccess) return LT_ERR_HIP;
    }
    l.plan[0] = a.keys_per_block;
    l.plan[1] = a.n_splits;
    l.plan[2] = a.tail_begin == INT32_MAX ? -1 : a.tail_begin;
    l.plan[3] = a.matrix_cores;
    if (ragged) {
        if (fused)
            for (int b = 0; b < c.batch; ++b) l.total_b[b] += takes_part(b) ? 1 : 0;
        l.total = *std::max_element(l.total_b.begin(), l.total_b.end());
    } else {
        l.total = total;
    }
    return LT_OK;
}

lt_status lt_decode_attn(lt_ctx *ctx, int32_t layer, const void *q, void *out, float *lse_out, void *stream)
{
    return launch_decode(ctx, layer, q, nullptr, nullptr, out, lse_out, nullptr, stream);
}

lt_status lt_decode_step(lt_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new, void *out,
                         float *lse_out, void *stream)
{
    if (k_new == nullptr || v_new == nullptr) return LT_ERR_INVALID_ARG;
    return launch_decode(ctx, layer, q, k_new, v_new, out, lse_out, nullptr, stream);
}

lt_status lt_decode_step_active(lt_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new,
                                const uint8_t *active_host, void *out, float *lse_out, void *stream)
{
    if (k_new == nullptr || v_new == nullptr || active_host == nullptr) return LT_ERR_INVALID_ARG;
    return launch_decode(ctx, layer, q, k_new, v_new, out, lse_out, active_host, stream);
}

// ---- online identification during prefill ------------------------------------------------------

lt_status lt_queue_create(int32_t capacity, lt_queue **out)
{
    if (out == nullptr) return LT_ERR_INVALID_ARG;
    *out = nullptr;
    if (capacity < 0) return LT_ERR_INVALID_ARG;
    lt_queue *q = new (std::nothrow) lt_queue();
    if (q == nullptr) return LT_ERR_NOMEM;
    q->capacity = capacity;
    try {
        q->entries.reserve((size_t)capacity + 1);
    } catch (const std::bad_alloc &) {
        delete q;
        return LT_ERR_NOMEM;
    }
    *out = q;
    return LT_OK;
}

void lt_queue_destroy(lt_queue *q) { delete q; }

lt_status lt_select_push(lt_queue *q, float ratio, int32_t layer, int32_t *popped_layer)
{
    if (q == nullptr || popped_layer == nullptr || layer < 0 || std::isnan(ratio)) return LT_ERR_INVALID_ARG;
    *popped_layer = -1;
    q->entries.emplace_back(ratio, layer);      // capacity + 1 was reserved
    if ((int64_t)q->entries.size() <= q->capacity) return LT_OK;
    size_t top = 0;                             // highest ratio, ties to the lower layer index
    for (size_t i = 1; i < q->entries.size(); ++i) {
        const auto &e = q->entries[i], &t = q->entries[top];
        if (e.first > t.first || (e.first == t.first && e.second < t.second)) top = i;
    }
    *popped_layer = q->entries[top].second;
    q->entries[top] = q->entries.back();
    q->entries.pop_back();
    return LT_OK;
}

lt_status lt_truncate_layer(lt_ctx *ctx, int32_t layer, void *stream)
{
    if (ctx == nullptr || layer < 0 || layer >= ctx->cfg.n_layers) return LT_ERR_INVALID_ARG;
    if (!ctx->online) return LT_ERR_STATE;
    Layer &l = ctx->layers[layer];
    if (l.lazy) return LT_ERR_STATE;
    const lt_config &c = ctx->cfg;
    const int64_t window = window_of(&c);
    size_t ring = ctx->ring_used.size();
    for (size_t i = 0; i < ctx->ring_used.size(); ++i)
        if (!ctx->ring_used[i]) { ring = i; break; }
    if (ring == ctx->ring_used.size()) return LT_ERR_CAPACITY;      // more lazy layers than the context was sized for
    const size_t ring_bytes = block_bytes(&c, true);
    uint16_t *k_ring = reinterpret_cast<uint16_t *>(ctx->ring_pool + ring * 2 * ring_bytes);
    uint16_t *v_ring = reinterpret_cast<uint16_t *>(ctx->ring_pool + ring * 2 * ring_bytes + ring_bytes);
    if (l.slot >= 0 && l.total > 0 && window > 0) {
        ltk::TruncateArgs a{};
        a.k_full = l.k;
        a.v_full = l.v;
        a.k_ring = k_ring;
        a.v_ring = v_ring;
        a.stride_h_full = l.capacity * ltk::kHeadDim;
        a.stride_b_full = a.stride_h_full * c.n_kv_heads;
        a.stride_h_ring = window * ltk::kHeadDim;
        a.stride_b_ring = a.stride_h_ring * c.n_kv_heads;
        a.total = l.total;
        a.batch = c.batch;
        a.n_kv_heads = c.n_kv_heads;
        a.w_sink = c.w_sink;
        a.w_recent = c.w_recent;
        ScopedEvents ev(ctx, static_cast<hipStream_t>(stream), LT_KERNEL_APPEND);
        if (ltk::truncate(a, static_cast<hipStream_t>(stream)) != hipSuccess) return LT_ERR_HIP;
    }
    if (l.slot >= 0) ctx->full_used[l.slot] = 0;     // reusable by work enqueued later on the same stream
    ctx->ring_used[ring] = 1;
    l.k = k_ring;
    l.v = v_ring;
    l.slot = (int32_t)ring;
    l.lazy = true;
    l.capacity = window;
    return LT_OK;
}

// ---- tuning and measurement --------------------------------------------------------------------

lt_status lt_set_split(lt_ctx *ctx, int32_t keys_per_block_full, int32_t keys_per_block_lazy)
{
    if (ctx == nullptr || keys_per_block_full < 0 || keys_per_block_lazy < 0) return LT_ERR_INVALID_ARG;
    if (keys_per_block_full % ltk::kKeyGranule != 0 || keys_per_block_lazy % ltk::kKeyGranule != 0) return LT_ERR_INVALID_ARG;
    if (keys_per_block_full > 0 && ceil_div(ctx->cfg.max_tokens, keys_per_block_full) > ctx->splits_cap) return LT_ERR_CAPACITY;
    if (keys_per_block_lazy > 0 && ceil_div(std::max<int64_t>(window_of(&ctx->cfg), 1), keys_per_block_lazy) > ctx->splits_cap)
        return LT_ERR_CAPACITY;
    ctx->keys_full = keys_per_block_full;
    ctx->keys_lazy = keys_per_block_lazy;
    return LT_OK;
}

lt_status lt_set_decode_path(lt_ctx *ctx, int32_t path)
{
    if (ctx == nullptr || (path != LT_DECODE_AUTO && path != LT_DECODE_VECTOR && path != LT_DECODE_MATRIX)) return LT_ERR_INVALID_ARG;
    ctx->decode_path = path;
    return LT_OK;
}

lt_status lt_decode_plan_read(lt_ctx *ctx, int32_t layer, int32_t *plan_host)
{
    if (ctx == nullptr || plan_host == nullptr || layer < 0 || layer >= ctx->cfg.n_layers) return LT_ERR_INVALID_ARG;
    const Layer &l = ctx->layers[layer];
    if (l.plan[1] == 0) return LT_ERR_INVALID_ARG;
    std::copy(l.plan, l.plan + 4, plan_host);
    return LT_OK;
}

lt_status lt_set_shared_tail(lt_ctx *ctx, int32_t on)
{
    if (ctx == nullptr) return LT_ERR_INVALID_ARG;
    ctx->shared_tail = on != 0;
    return LT_OK;
}

lt_status lt_probe_read(const void *buf_dev, size_t bytes, void *sink_dev, void *stream)
{
    if (buf_dev == nullptr || sink_dev == nullptr || bytes < 16 * 1024 || ((uintptr_t)buf_dev % 16) != 0 || ((uintptr_t)sink_dev % 4) != 0)
        return LT_ERR_INVALID_ARG;
    return ltk::probe_read(buf_dev, (int64_t)bytes, static_cast<uint32_t *>(sink_dev), static_cast<hipStream_t>(stream)) == hipSuccess
               ? LT_OK : LT_ERR_HIP;
}

lt_status lt_profile_enable(lt_ctx *ctx, int32_t on)
{
    if (ctx == nullptr) return LT_ERR_INVALID_ARG;
    if (on != 0 && ctx->events.capacity() < (size_t)kMaxEventPairs) {
        try {
            ctx->events.reserve(kMaxEventPairs);       // host memory only; the events themselves are made on demand
        } catch (const std::bad_alloc &) {
            return LT_ERR_NOMEM;
        }
    }
    if (on != 0) ctx->events_used = 0;
    ctx->profiling = on != 0;
    return LT_OK;
}

lt_status lt_profile_read(lt_ctx *ctx, int32_t kernel, int64_t *launches, double *total_ms)
{
    if (ctx == nullptr || kernel < 0 || kernel >= LT_KERNEL_COUNT || launches == nullptr || total_ms == nullptr)
        return LT_ERR_INVALID_ARG;
    int64_t count = 0;
    double sum = 0.0;
    for (size_t i = 0; i < ctx->events_used; ++i) {
        const EventPair &p = ctx->events[i];
        if (p.kernel != kernel) continue;
        if (hipEventSynchronize(p.stop) != hipSuccess) return LT_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p.start, p.stop) != hipSuccess) return LT_ERR_HIP;
        sum += ms;
        ++count;
    }
    *launches = count;
    *total_ms = sum;
    return LT_OK;
}

}  // extern "C"
