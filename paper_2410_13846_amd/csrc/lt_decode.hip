// Decode-side kernels for gfx950: KV append (growing cache / sink+recent ring) and split decode
// attention over the key axis with the log-sum-exp merge of the splits done by the workgroup
// that finishes last, so one decode step of a layer is a single launch.
//
// Attention of one query over a set of keys does not depend on the order of the keys, so a
// lazy layer's ring is read as a plain array of `stored` entries and both layer kinds share
// one kernel.  One workgroup streams a contiguous range of keys of one (sequence, KV head)
// once from HBM and applies it to all G query heads of that KV head.
//
// Two kernels do this: lt_decode_kernel forms q.k and p.v with vector instructions (the fastest over
// long ranges while a group has at most five heads), lt_decode_mfma_kernel with the matrix cores (short
// ranges, where the vector instructions are what ends a launch, and larger groups, where they fall
// behind the memory).  They load tiles the same way and share everything after the loop over the keys
// (finish_workgroup); the C-ABI layer picks one per launch.
#include "lt_kernels.h"

#include <type_traits>

namespace ltk {
namespace {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr float kLn2 = 0.69314718055994530942f;

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;   // 16 bytes as one register quad

// Every pointer the kernels see is device memory: say so, or a pointer chosen at run time
// between two buffers is accessed with the slower generic (flat) instructions.
typedef const __attribute__((address_space(1))) u32x4_t *global_quad_ptr;
typedef __attribute__((address_space(1))) u32x4_t *global_quad_wptr;

__device__ __forceinline__ u32x4_t load16(const uint16_t *p) { return *(global_quad_ptr)p; }

// K and V are read exactly once per decode step: stream them past the caches.
__device__ __forceinline__ u32x4_t load16_stream(const uint16_t *p) { return __builtin_nontemporal_load((global_quad_ptr)p); }

__device__ __forceinline__ void store16(uint16_t *p, u32x4_t v) { *(global_quad_wptr)p = v; }
__device__ __forceinline__ void store16_stream(uint16_t *p, u32x4_t v) { __builtin_nontemporal_store(v, (global_quad_wptr)p); }

// Device-scope relaxed atomic store / load: coherent between workgroups anywhere on the chip
// without flushing or invalidating a cache.
__device__ __forceinline__ void publish(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float observe(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// ---------------------------------------------------------------------------------------------
// append: one thread moves 16 bytes of K and 16 bytes of V.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lt_append_kv_kernel(AppendArgs a)
{
    const int g = blockIdx.y, b = blockIdx.z;
    const int64_t n_new = a.ragged ? a.n_new_b[b] : a.n_new;       // tokens this sequence brings
    const int64_t total_before = a.ragged ? a.total_before_b[b] : a.total_before;
    const int64_t per_stream = n_new * 16;                         // uint4 units per (b, g)
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_stream) return;
    const int64_t j = idx >> 4;
    const int c = (int)(idx & 15);
    const int64_t p = total_before + j;                            // absolute position of the token
    int64_t slot = p;
    if (a.is_lazy) {
        if (p >= a.w_sink) {
            const int64_t total_after = total_before + n_new;
            if (a.w_recent == 0 || p < total_after - a.w_recent) return;   // a later token of this call owns the slot
            slot = a.w_sink + (p - a.w_sink) % a.w_recent;
        }
    }
    const int64_t src = (((int64_t)b * a.n_kv_heads + g) * a.n_new + j) * kHeadDim + c * 8;
    int64_t dst = (int64_t)b * a.stride_b + (int64_t)g * a.stride_h + slot * kHeadDim + c * 8;
    if (a.block_table != nullptr) {
        const int64_t page = a.block_table[(int64_t)b * a.max_pages + (slot >> a.page_shift)];
        dst = (((page * a.n_kv_heads + g) << a.page_shift) + (slot & ((1 << a.page_shift) - 1))) * kHeadDim + c * 8;
    }
    // a prompt's K/V pass through once: streamed in and out
    store16_stream(a.k_cache + dst, load16_stream(a.k_new + src));
    store16_stream(a.v_cache + dst, load16_stream(a.v_new + src));
}

// ---------------------------------------------------------------------------------------------
// truncate: a layer that turns lazy keeps the first w_sink and the last w_recent of its `total`
// tokens; they move from its full-size block into a ring block (disjoint memory), each token to
// the slot the append rule would have given it.  One thread moves 16 bytes of K and of V.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lt_truncate_kernel(TruncateArgs a)
{
    const int64_t n_sink = a.total < a.w_sink ? a.total : a.w_sink;
    const int64_t first_recent = (a.total - a.w_recent) > a.w_sink ? (a.total - a.w_recent) : a.w_sink;
    const int64_t n_recent = a.total > first_recent ? a.total - first_recent : 0;
    const int64_t per_stream = (n_sink + n_recent) * 16;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_stream) return;
    const int g = blockIdx.y, b = blockIdx.z;
    const int64_t j = idx >> 4;
    const int c = (int)(idx & 15);
    const int64_t p = j < n_sink ? j : first_recent + (j - n_sink);          // absolute position
    const int64_t slot = p < a.w_sink ? p : a.w_sink + (p - a.w_sink) % a.w_recent;
    const int64_t src = (int64_t)b * a.stride_b_full + (int64_t)g * a.stride_h_full + p * kHeadDim + c * 8;
    const int64_t dst = (int64_t)b * a.stride_b_ring + (int64_t)g * a.stride_h_ring + slot * kHeadDim + c * 8;
    store16_stream(a.k_ring + dst, load16_stream(a.k_full + src));
    store16_stream(a.v_ring + dst, load16_stream(a.v_full + src));
}

// ---------------------------------------------------------------------------------------------
// split decode attention.
//
// Lane layout inside a wavefront: lane = 16*sub + chunk.  One 16-byte load per lane covers four
// consecutive keys (sub = 0..3) times sixteen 8-element slices of the 128 dims (chunk), i.e. one
// fully coalesced kilobyte.  A tile is 16 keys: four such loads of K and four of V.
// Each 16-lane row keeps its own online-softmax state (running max m, sum l, accumulator) for
// the keys it sees, so the main loop needs cross-lane traffic only for the q.k row sums; rows
// and wavefronts are merged once at the end.
// ---------------------------------------------------------------------------------------------
struct Tile {
    u32x4_t k[4];
    u32x4_t v[4];
};

// new_slot (or -1) is the cache entry of the token generated in this step when the append is
// fused into the decode: its K/V are read from the caller's k_new / v_new instead of the cache.
// Every path issues the same eight loads in the same order, so the wait counts of the software
// pipeline stay exact; only the addresses differ, and only in the one tile that holds new_slot.
//
// key0 < 0 marks a fetch past the wavefront's last tile, issued only to keep the load count of
// the pipeline fixed: it reads `hot` (the query vector, already in cache) so that nothing after
// the loop has to wait a full memory latency for data nobody uses.
__device__ __forceinline__ void load_tile(Tile &t, const uint16_t *kb, const uint16_t *vb, int key0, int sub, int chunk,
                                          int last_key, int new_slot, const uint16_t *k_new, const uint16_t *v_new,
                                          const uint16_t *hot)
{
    const uint16_t *kp[4], *vp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int key = key0 + 4 * i + sub;
        key = key < last_key ? key : last_key;                      // clamp: masked later
        key = key > 0 ? key : 0;
        const int64_t off = (int64_t)key * kHeadDim + chunk * 8;
        kp[i] = kb + off;
        vp[i] = vb + off;
    }
    if (key0 < 0) {                                                 // wave-uniform
#pragma unroll
        for (int i = 0; i < 4; ++i) { kp[i] = hot + chunk * 8; vp[i] = hot + chunk * 8; }
    } else if (new_slot >= key0 && new_slot < key0 + 16) {                 // wave-uniform, true for one tile of one workgroup
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int key = key0 + 4 * i + sub;
            key = key < last_key ? key : last_key;
            if (key == new_slot) { kp[i] = k_new + chunk * 8; vp[i] = v_new + chunk * 8; }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        t.k[i] = load16_stream(kp[i]);
        t.v[i] = load16_stream(vp[i]);
    }
}

// The fused append: the lanes that hold the new token write it into its cache entry.  A clamped
// lane may repeat the store with the same bytes.
__device__ __forceinline__ void store_new_token(const Tile &t, uint16_t *kb, uint16_t *vb, int key0, int sub, int chunk,
                                                int last_key, int new_slot)
{
    if (new_slot < key0 || new_slot >= key0 + 16) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int key = key0 + 4 * i + sub;
        key = key < last_key ? key : last_key;
        if (key == new_slot) {
            const int64_t off = (int64_t)key * kHeadDim + chunk * 8;
            store16(kb + off, t.k[i]);
            store16(vb + off, t.v[i]);
        }
    }
}

// Online-softmax state of one 16-lane row.  m (running max, log2 units) is the same in all 16
// lanes of the row.  After the q.k reduction each quad of the row (lanes 4i..4i+3) holds the
// logits of ONE of the row's four keys of a tile (key 4i + sub), for all G heads; l accumulates in
// that layout, so the row's sum is the sum over one lane of each quad.  acc is the row's
// un-normalised output for the lane's eight dims.
template <int G>
struct RowState {
    float m[G];
    float l[G];
    float acc[G][8];
};

// Sum of x over the lanes {l, 15-l} (row_mirror) or {l, 7-l} (row_half_mirror) of a DPP row.
__device__ __forceinline__ float add_mirror(float keep, float send) { return keep + dpp_move<0x140>(send); }
__device__ __forceinline__ float add_half_mirror(float keep, float send) { return keep + dpp_move<0x141>(send); }

// Cross-row exchange (gfx950): with a' and b' the values after the call,
//   swap_rows16: a' = {a.row0, b.row0, a.row2, b.row2},  b' = {a.row1, b.row1, a.row3, b.row3}
//   swap_rows32: a' = {a.row0, a.row1, b.row0, b.row1},  b' = {a.row2, a.row3, b.row2, b.row3}
// (rows are the four 16-lane groups of the wavefront).
// Written as inline assembly: with this toolchain the corresponding builtins compile to code
// that treats their two results as one value.  Both operands are rewritten in place; the
// s_nop keep the wait states these instructions need around other vector instructions, which
// the compiler does not track inside an asm statement.
__device__ __forceinline__ void swap_rows16(float &a, float &b)
{
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void swap_rows32(float &a, float &b)
{
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}

// Maximum of x over the four rows, in every row.
__device__ __forceinline__ float max_rows(float x)
{
    float a = x, b = x;
    swap_rows16(a, b);                      // a: rows {0,0,2,2}, b: rows {1,1,3,3} of x
    const float m = fmaxf(a, b);
    a = m;
    b = m;
    swap_rows32(a, b);                      // a: rows {0,1,0,1}, b: rows {2,3,2,3} of m
    return fmaxf(a, b);
}

// Sums x0..x3 over the four rows; row r of the result holds the total of x_r.
__device__ __forceinline__ float sum_rows4(float x0, float x1, float x2, float x3)
{
    swap_rows16(x0, x1);                    // x0 + x1: rows 0,2 hold x0 over row pairs, rows 1,3 hold x1
    swap_rows16(x2, x3);
    float a = x0 + x1, b = x2 + x3;
    swap_rows32(a, b);                      // a + b: rows 0,1 come from the first pair, rows 2,3 from the second
    return a + b;
}

template <int LANE>
__device__ __forceinline__ float row_broadcast(float x)      // value of lane LANE of the row, in every lane of the row
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x150 + LANE, 0xf, 0xf, true));
}

template <int G>
__device__ __forceinline__ void process_tile(const Tile &t, const uint32_t (&qf)[G][4], RowState<G> &st, int key0, int sub,
                                             int chunk, int end_key, float scale_log2e)
{
    // Partial dot products: lane (sub, chunk) covers dims 8*chunk..8*chunk+7 of keys key0 + 4*i + sub.
    float part[4][G];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float x = dot2_bf16(t.k[i][0], qf[h][0], 0.f);
            x = dot2_bf16(t.k[i][1], qf[h][1], x);
            x = dot2_bf16(t.k[i][2], qf[h][2], x);
            part[i][h] = dot2_bf16(t.k[i][3], qf[h][3], x);
        }
    // Reduce over the 16 lanes of the row and scatter at the same time: each step pairs every lane
    // with one in the other half (then the other quad), keeps the keys of its own half and hands
    // the others over, so the number of values halves; a last all-reduce inside the quad leaves
    // quad i with the complete logits of key i.  44 instructions instead of 64 for a full
    // all-reduce, and the exponentials that follow are computed 4 times instead of 16.
    const bool upper_half = (chunk & 8) != 0, upper_quad = (chunk & 4) != 0;
    float s[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float a0 = add_mirror(upper_half ? part[2][h] : part[0][h], upper_half ? part[0][h] : part[2][h]);
        const float a1 = add_mirror(upper_half ? part[3][h] : part[1][h], upper_half ? part[1][h] : part[3][h]);
        float x = add_half_mirror(upper_quad ? a1 : a0, upper_quad ? a0 : a1);
        x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
        x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
        s[h] = x * scale_log2e;
    }
    const int my_key = key0 + (chunk & 12) + sub;                   // quad i = chunk / 4 holds key 4*i + sub
    const bool valid = my_key < end_key;
    bool grow = false;
#pragma unroll
    for (int h = 0; h < G; ++h) {
        s[h] = valid ? s[h] : -INFINITY;
        grow |= s[h] > st.m[h];
    }
    if (__any(grow)) {                                              // rare after the first tiles
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float tmax = fmaxf(s[h], dpp_move<0x141>(s[h]));        // max over the row's four keys
            tmax = fmaxf(tmax, dpp_move<0x140>(tmax));
            const float m_new = fmaxf(st.m[h], tmax);
            const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(st.m[h] - m_new);
            st.m[h] = m_new;
            st.l[h] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) st.acc[h][e] *= alpha;
        }
    }
    float p[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float m_safe = (st.m[h] == -INFINITY) ? 0.f : st.m[h];
        p[h] = fast_exp2(s[h] - m_safe);
        st.l[h] += p[h];
    }
    // P.V: the probability of key 4*i + sub sits in quad i; broadcast it over the row for load i.
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float vf[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) { vf[2 * e] = bf16_lo(t.v[i][e]); vf[2 * e + 1] = bf16_hi(t.v[i][e]); }
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float pb = i == 0 ? row_broadcast<0>(p[h]) : i == 1 ? row_broadcast<4>(p[h])
                           : i == 2 ? row_broadcast<8>(p[h]) : row_broadcast<12>(p[h]);
#pragma unroll
            for (int e = 0; e < 8; ++e) st.acc[h][e] = fmaf(pb, vf[e], st.acc[h][e]);
        }
    }
}

// LAZY_TAG only gives full and lazy layers distinct kernel names in profiles.  kWaves wavefronts
// per workgroup: four when a workgroup has a long range to stream (memory-bound: more wavefronts
// per compute unit only lower the bandwidth), eight when the range is short and the launch is
// bound by how fast one wavefront gets through its tiles.
// Final output element: fp32, or bf16 (round to nearest even) when the caller asked for it.
__device__ __forceinline__ void store_out(const DecodeArgs &a, int64_t index, float value)
{
    if (a.out_bf16) reinterpret_cast<__bf16 *>(a.out)[index] = (__bf16)value;
    else reinterpret_cast<float *>(a.out)[index] = value;
}

struct NoRaggedArgs {};
// kMode 0: equal lengths; 1: per-sequence lengths; 2: per-sequence lengths and a paged cache
enum { kUniform = 0, kRaggedMode = 1, kPagedMode = 2 };
template <int kMode> struct ModeArgs { typedef NoRaggedArgs type; };
template <> struct ModeArgs<kRaggedMode> { typedef RaggedArgs type; };
template <> struct ModeArgs<kPagedMode> { typedef PagedArgs type; };
__device__ __forceinline__ const RaggedArgs &lengths_of(const RaggedArgs &r) { return r; }
__device__ __forceinline__ const RaggedArgs &lengths_of(const PagedArgs &r) { return r.lengths; }

// Paged cache: lane i of every wavefront holds the pages of the range's pages i, 64 + i, 128 + i, 192 + i; a 16-key
// tile never straddles pages (their size is a multiple of 16), so a tile costs one cross-lane read of one of those
// registers to find its page and no memory access.  shift() is the element offset that, added to the layer's pool,
// makes "base + key * 128" land on the key inside its page.  For the other modes the struct is empty and shift() is 0.
template <bool kPaged>
struct RangePages {
    static constexpr int kRegs = kPaged ? kMaxRangePages / 64 : 1;
    int32_t pages[kRegs] = {};
    int first_page = 0;

    __device__ __forceinline__ void load(const PagedArgs &r, int b, int lane, int begin_key, int end_key, int n_tiles)
    {
        first_page = begin_key >> r.page_shift;
        const int last_page = max(end_key - 1, begin_key) >> r.page_shift;
#pragma unroll
        for (int i = 0; i < kRegs; ++i)
            if (n_tiles > 0 && first_page + 64 * i <= last_page)          // uniform
                pages[i] = r.block_table[(int64_t)b * r.max_pages + min(first_page + 64 * i + lane, last_page)];
    }
    template <typename Other>
    __device__ __forceinline__ void load(const Other &, int, int, int, int, int) {}

    __device__ __forceinline__ int64_t shift(const PagedArgs &r, int key0, int begin_key, int n_kv_heads, int g) const
    {
        const int key = max(key0, begin_key);                       // key0 < 0: a fetch whose tile is never consumed
        const int idx = (key >> r.page_shift) - first_page;         // uniform, below kMaxRangePages
        int32_t page = __builtin_amdgcn_readlane(pages[0], idx & 63);
#pragma unroll
        for (int i = 1; i < kRegs; ++i)
            if ((idx >> 6) == i) page = __builtin_amdgcn_readlane(pages[i], idx & 63);
        const int64_t in_pool = (((int64_t)page * n_kv_heads + g) << r.page_shift) * kHeadDim;
        return in_pool - (int64_t)((key >> r.page_shift) << r.page_shift) * kHeadDim;
    }
    template <typename Other>
    __device__ __forceinline__ int64_t shift(const Other &, int, int, int, int) const { return 0; }
};

// The tile (0 .. wrap - 1) a workgroup starts at inside its range.  Workgroups run in lockstep, and their ranges
// start at multiples of the same strides, so without care they all hit the same few memory channels at the same
// moment (measured: 185 vs 162 us per launch depending on the cache capacity alone).  The order of keys does not
// matter to the result, so each workgroup starts at a tile of its own and wraps around.  The start tiles are chosen
// by absolute address (the memory channels are picked from the address bits): workgroup i of n starts where its
// address is i * window / n modulo a window of spread_tiles 4 KB tiles, so the n address streams, which advance at
// the same pace, stay evenly spread over that window (measured 5 % faster than pseudo-random starts, which remain
// for ranges shorter than any useful window).  Paged layers: pages scatter the high address bits by themselves;
// what the start tile still decides is the position inside a page -- the workgroups of one KV head (whose pages all
// sit at the same offset inside a pool page) start evenly spread over the tiles of a page, at a pseudo-random page
// of their range.
__device__ __forceinline__ int start_tile(const DecodeArgs &a, const uint16_t *range_begin, int begin_key, int wrap, int page_shift)
{
    const unsigned int linear_block = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    if (page_shift > 0) {
        const unsigned int page_tiles = 1u << (page_shift - 4);
        const unsigned int among = gridDim.x * gridDim.z, mine = blockIdx.z * gridDim.x + blockIdx.x;
        const unsigned int want = (unsigned int)(((uint64_t)mine * page_tiles) / among) & (page_tiles - 1);
        const unsigned int in_page = (want - ((unsigned int)begin_key >> 4)) & (page_tiles - 1);
        const unsigned int pages_here = ((unsigned int)wrap + page_tiles - 1) / page_tiles;
        return (int)((in_page + (((linear_block * 2654435761u) >> 12) % pages_here) * page_tiles) % (unsigned int)wrap);
    }
    const unsigned int n_blocks = gridDim.x * gridDim.y * gridDim.z;
    const unsigned int first_tile_addr = (unsigned int)(((uintptr_t)range_begin) >> 12);
    const unsigned int target = (unsigned int)(((uint64_t)linear_block * a.spread_tiles) / n_blocks);
    return a.spread_tiles ? (int)(((target - first_tile_addr) & (a.spread_tiles - 1)) % (unsigned int)wrap)
                          : (int)(((linear_block * 2654435761u) >> 12) % (unsigned int)wrap);
}
__device__ __forceinline__ int page_shift_of(const PagedArgs &r) { return r.page_shift; }
template <typename Other>
__device__ __forceinline__ int page_shift_of(const Other &) { return 0; }

// What every workgroup does after its wavefronts have put their partial results (running max in log2 units, sum,
// un-normalised accumulator) into LDS and passed a barrier: merge the wavefronts, publish the split's partial result,
// and -- in the workgroup that takes the last ticket of its (sequence, KV head) -- merge the splits.  n_pieces > 0:
// the launch used the shared tail, whose counter goes back to zero here.
template <int G, int kWaves>
__device__ __forceinline__ void finish_workgroup(const DecodeArgs &a, int b, int g, int split, int n_pieces, unsigned int *counter,
                                                 const float (&sh_m)[kWaves][G], const float (&sh_l)[kWaves][G],
                                                 const float *sh_acc, int acc_stride)
{
    // sh_acc: wavefront w's accumulator of head h, dim d at sh_acc[w * acc_stride + h * kHeadDim + d]
    constexpr int kThreads = 64 * kWaves;
    __shared__ int sh_is_last;
    __shared__ float sh_merge_m[G][kMaxSplits];
    __shared__ float sh_merge_l[G][kMaxSplits];
    // Merge the wavefronts.  With a single split this is the final result; otherwise store the
    // split's partial result (un-normalised accumulator, running max in log2 units, sum).
    const bool single = a.n_splits == 1;
    for (int idx = threadIdx.x; idx < G * kHeadDim; idx += kThreads) {
        const int h = idx / kHeadDim, dim = idx % kHeadDim;
        float mx = sh_m[0][h];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, sh_m[w][h]);
        float l = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float wgt = (sh_m[w][h] == -INFINITY) ? 0.f : fast_exp2(sh_m[w][h] - mx);
            l += wgt * sh_l[w][h];
            o += wgt * sh_acc[w * acc_stride + h * kHeadDim + dim];
        }
        const int64_t head = (int64_t)b * a.n_q_heads + g * G + h;
        if (single) {
            store_out(a, head * kHeadDim + dim, l > 0.f ? o / l : 0.f);                  // a sequence without tokens gives 0
            if (a.lse != nullptr && dim == 0) a.lse[head] = (mx + log2f(l)) * kLn2;
        } else {
            const int64_t row = head * a.n_splits + split;
            publish(&a.part_acc[row * kHeadDim + dim], o);
            if (dim == 0) { publish(&a.part_ml[row * 2], mx); publish(&a.part_ml[row * 2 + 1], l); }
        }
    }
    if (single) {
        // all wavefronts have left the shared tail (the barrier above): its counter is ready for the next launch
        if (n_pieces > 0 && threadIdx.x == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }

    // The workgroup that takes the last ticket of its (sequence, KV head) merges all splits:
    // softmax over a union of disjoint key sets is the sum of the per-set results weighted by
    // exp(max_c - max) * l_c.
    //
    // Ordering between workgroups, made explicit step by step:
    //  1. Partial results are written with device-scope atomic stores: they bypass the non-coherent
    //     levels and complete at the point every compute unit of the device reads from.
    //  2. Every thread waits until ALL of its own vector-memory operations have been acknowledged
    //     (vmcnt(0); on this architecture stores count in vmcnt), i.e. its partial results are
    //     visible device-wide.  A fence at workgroup scope would not promise that.
    //  3. The barrier makes step 2 of every thread precede the ticket, which one thread takes
    //     with a device-scope atomic add.
    //  4. The merge loads (device-scope atomic loads, never served from a non-coherent cache
    //     line) are issued only by a workgroup that has seen the last ticket value come back:
    //     they depend on it through LDS and a barrier, and the hardware does not issue loads
    //     past an unresolved branch.  Every other workgroup of the (sequence, KV head) took its
    //     ticket after its own step 2, so all partial results are complete by then.
    // No cache write-back or invalidate is involved (a device-scope release fence here costs a
    // whole-L2 write-back per workgroup and doubled the kernel time).
    __builtin_amdgcn_s_waitcnt(0x0F70);                             // vmcnt(0): this thread's publish() stores are acknowledged
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");          // compiler ordering; the hardware wait is the line above
    __syncthreads();
    unsigned int *ticket = a.tickets + ((int64_t)b * a.n_kv_heads + g) * kTicketStride;
    if (threadIdx.x == 0) {
        const unsigned int t_mine = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sh_is_last = (t_mine == (unsigned int)(a.n_splits - 1)) ? 1 : 0;
    }
    __syncthreads();
    if (!sh_is_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");          // compiler ordering: no merge load moves above the ticket
    // Every (head, split) pair's running max and sum go to LDS.  In the same memory round trip every thread
    // requests the partial accumulators of its output elements for the first kEager splits, eight at a time
    // and only as far as there are splits; launches with more splits than that fetch the rest in further batches.
    constexpr int kRounds = (G * kHeadDim + kThreads - 1) / kThreads;     // output elements per thread
    constexpr int kEager = kRounds <= 1 ? 64 : kRounds == 2 ? 32 : 16;
    float part[kRounds][kEager];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int idx = threadIdx.x + r * kThreads;
        const int h = (idx < G * kHeadDim ? idx : 0) / kHeadDim, dim = idx % kHeadDim;
        const float *acc = a.part_acc + ((int64_t)b * a.n_q_heads + g * G + h) * a.n_splits * kHeadDim + dim;
#pragma unroll
        for (int u0 = 0; u0 < kEager; u0 += 8)
            if (u0 < a.n_splits) {                                  // uniform
#pragma unroll
                for (int u = u0; u < u0 + 8; ++u) part[r][u] = observe(acc + (int64_t)min(u, a.n_splits - 1) * kHeadDim);
            }
    }
    // The rows of maxima and sums are padded to a multiple of eight splits with empty entries (-inf, 0), so that
    // what follows reads them eight at a time without looking at the split count.
    const int padded_splits = (a.n_splits + 7) & ~7;
    for (int idx = threadIdx.x; idx < G * padded_splits; idx += kThreads) {
        const int h = idx / padded_splits, c = idx % padded_splits;
        const float *ml = a.part_ml + (((int64_t)b * a.n_q_heads + g * G + h) * a.n_splits + min(c, a.n_splits - 1)) * 2;
        const float m_c = observe(ml), l_c = observe(ml + 1);
        sh_merge_m[h][c] = c < a.n_splits ? m_c : -INFINITY;
        sh_merge_l[h][c] = c < a.n_splits ? l_c : 0.f;
    }
    __syncthreads();
    // One thread per output element.  Everything it reads from LDS comes in groups of eight splits with constant
    // offsets inside the group, so the reads of a group are issued together; a single wavefront per SIMD is left
    // at this point, and reads waited for one by one would cost their full latency each.
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int idx = threadIdx.x + r * kThreads;
        if (idx >= G * kHeadDim) break;
        const int h = idx / kHeadDim, dim = idx % kHeadDim;
        const int64_t head = (int64_t)b * a.n_q_heads + g * G + h;
        const float *acc = a.part_acc + head * a.n_splits * kHeadDim + dim;
        float mx = -INFINITY;
        for (int c0 = 0; c0 < a.n_splits; c0 += 8) {
#pragma unroll
            for (int u = 0; u < 8; ++u) mx = fmaxf(mx, sh_merge_m[h][c0 + u]);
        }
        const float m_safe = mx == -INFINITY ? 0.f : mx;            // no split saw a key: every weight is 0
        float l = 0.f, o = 0.f;
        auto weigh8 = [&](int c0, const float *v) __attribute__((always_inline)) {   // splits c0 .. c0 + 7; empty ones weigh 0
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float wgt = fast_exp2(sh_merge_m[h][c0 + u] - m_safe);
                l = fmaf(wgt, sh_merge_l[h][c0 + u], l);
                o = fmaf(wgt, v[u], o);
            }
        };
#pragma unroll
        for (int u0 = 0; u0 < kEager; u0 += 8)
            if (u0 < a.n_splits) weigh8(u0, &part[r][u0]);
        for (int c0 = kEager; c0 < a.n_splits; c0 += 32) {         // launches with more than kEager splits: 32 per round trip
            float v[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) v[u] = observe(acc + (int64_t)min(c0 + u, a.n_splits - 1) * kHeadDim);
#pragma unroll
            for (int u0 = 0; u0 < 32; u0 += 8)
                if (c0 + u0 < a.n_splits) weigh8(c0 + u0, &v[u0]);
        }
        store_out(a, head * kHeadDim + dim, l > 0.f ? o / l : 0.f);
        if (a.lse != nullptr && dim == 0) a.lse[head] = (mx + log2f(l)) * kLn2;
    }
    if (threadIdx.x == 0) {                                         // ready for the next launch
        __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(ticket + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int G, int LAZY_TAG, int kWaves, int kMode>
__global__ __launch_bounds__(64 * kWaves) void lt_decode_kernel(DecodeArgs a, typename ModeArgs<kMode>::type r)
{
    constexpr bool kRagged = kMode != kUniform, kPaged = kMode == kPagedMode;
    __shared__ float sh_m[kWaves][G];
    __shared__ float sh_l[kWaves][G];
    __shared__ float sh_acc[kWaves][G][kHeadDim];

    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: tile indices stay in SGPRs
    const int sub = lane >> 4, chunk = lane & 15;

    // in a ragged batch a sequence may end before this workgroup's range: then the range is empty and
    // the workgroup contributes an empty partial result
    int stored = a.stored;
    if constexpr (kRagged) stored = lengths_of(r).stored_b[b];
    const int begin_key = split * a.keys_per_block;
    const int end_key = min(min(stored, a.tail_begin), begin_key + a.keys_per_block);
    const int n_tiles = max((end_key - begin_key + 15) >> 4, 0);
    const int wrap = max(n_tiles, 1);
    uint16_t *kb = a.k_cache + (int64_t)b * a.stride_b + (int64_t)g * a.stride_h;
    uint16_t *vb = a.v_cache + (int64_t)b * a.stride_b + (int64_t)g * a.stride_h;
    // fused append: the one tile that holds new_slot takes the token from k_new / v_new
    int new_slot = a.k_new != nullptr ? a.new_slot : -1;
    if constexpr (kRagged) new_slot = a.k_new != nullptr ? lengths_of(r).new_slot_b[b] : -1;
    const int64_t new_off = new_slot >= 0 ? ((int64_t)b * a.n_kv_heads + g) * kHeadDim : 0;
    const uint16_t *k_new = a.k_new + new_off;
    const uint16_t *v_new = a.v_new + new_off;
    const uint16_t *hot = a.q + ((int64_t)b * a.n_q_heads + g * G) * kHeadDim;
    RangePages<kPaged> range_pages;
    range_pages.load(r, b, lane, begin_key, end_key, n_tiles);
    auto tile_shift = [&](int key0) -> int64_t { return range_pages.shift(r, key0, begin_key, a.n_kv_heads, g); };
    if constexpr (kPaged) { kb = a.k_cache; vb = a.v_cache; }
    // `limit` is the end of the keys a tile may hold: the end of the workgroup's range, or `stored` in the shared tail
    auto fetch = [&](Tile &t, int key0, int limit) __attribute__((always_inline)) {
        if constexpr (kPaged) {
            const int64_t shift = tile_shift(key0);
            load_tile(t, kb + shift, vb + shift, key0, sub, chunk, limit - 1, new_slot, k_new, v_new, hot);
        } else {
            load_tile(t, kb, vb, key0, sub, chunk, limit - 1, new_slot, k_new, v_new, hot);
        }
    };
    auto consume = [&](const Tile &t, int key0, int limit, RowState<G> &st, const uint32_t (&qf)[G][4]) __attribute__((always_inline)) {
        if constexpr (kPaged) {
            if (new_slot >= key0 && new_slot < key0 + 16) {         // wave-uniform, true for one tile of one workgroup
                const int64_t shift = tile_shift(key0);
                store_new_token(t, kb + shift, vb + shift, key0, sub, chunk, limit - 1, new_slot);
            }
        } else {
            store_new_token(t, kb, vb, key0, sub, chunk, limit - 1, new_slot);
        }
        process_tile<G>(t, qf, st, key0, sub, chunk, limit, a.scale_log2e);
    };

    uint32_t qf[G][4];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const u32x4_t u = load16(a.q + ((int64_t)b * a.n_q_heads + g * G + h) * kHeadDim + chunk * 8);
        qf[h][0] = u[0]; qf[h][1] = u[1]; qf[h][2] = u[2]; qf[h][3] = u[3];
    }

    RowState<G> st;
#pragma unroll
    for (int h = 0; h < G; ++h) {
        st.m[h] = -INFINITY;
        st.l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[h][e] = 0.f;
    }

    // Wavefront w takes every kWaves-th tile; two tile buffers alternate so the loads of the next
    // tile are in flight while the current one is consumed.  Every fetch is unconditional (past
    // its last tile a wavefront re-fetches tiles it never consumes): with a fixed number of loads
    // between a fetch and its use the wait counts are exact, and a tile is consumed while the
    // following one is still arriving.
    // each workgroup starts at a tile of its own inside its range and wraps around (start_tile)
    const int phase = start_tile(a, kb + (int64_t)begin_key * kHeadDim, begin_key, wrap, page_shift_of(r));
    const int my_tiles = wave < n_tiles ? (n_tiles - wave + kWaves - 1) / kWaves : 0;
    int next_tile = wave + phase, fetched = 0;
    while (next_tile >= wrap) next_tile -= wrap;
    auto advance = [&]() {                                          // first key of the next tile to fetch, -1 past the last
        const int cur = next_tile;
        next_tile += kWaves;
        while (next_tile >= wrap) next_tile -= wrap;
        return fetched++ < my_tiles ? begin_key + 16 * cur : -1;
    };
    // The shared tail (described below): its first two pieces are claimed while the wavefront's last own tiles
    // are on their way, so that the claims have come back when those tiles are done.
    const int n_pieces = !kPaged && stored > a.tail_begin ? (stored - a.tail_begin + kTailKeys - 1) / kTailKeys : 0;
    unsigned int *counter = a.tickets + ((int64_t)b * a.n_kv_heads + g) * kTicketStride + 1;
    // a claim is one atomic add by lane 0; its result is read (readfirstlane) only when the piece is needed
    auto claim = [&]() __attribute__((always_inline)) {
        unsigned int c = 0;
        if (lane == 0) c = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return c;
    };
    unsigned int claim_first = 0, claim_next = 0;
    if (n_pieces > 0 && my_tiles <= 2) { claim_first = claim(); claim_next = claim(); }

    Tile t0, t1;
    int key0 = advance();
    fetch(t0, key0, end_key);
    for (int k = 0; k < my_tiles; k += 2) {
        if (n_pieces > 0 && k > 0 && k + 2 >= my_tiles) { claim_first = claim(); claim_next = claim(); }   // the last round
        const int key1 = advance();
        fetch(t1, key1, end_key);
        consume(t0, key0, end_key, st, qf);
        key0 = advance();
        fetch(t0, key0, end_key);
        if (k + 1 < my_tiles) consume(t1, key1, end_key, st, qf);
    }

    // The shared tail.  Workgroups do not get through equal ranges in equal times: measured with a timestamp per
    // workgroup, those of some of the device's eight XCDs take 5-10 % longer over the same number of keys (which
    // XCDs differs from device to device), and a launch ends with its slowest workgroup.  So the last part of
    // every (sequence, KV head) belongs to no range: a wavefront that has finished its own tiles takes the next
    // piece of kTailKeys keys from a counter of the (sequence, KV head).  The order in which keys reach a
    // wavefront's running softmax does not matter to the result (up to rounding).  Every claim moves the counter
    // forward, so a wavefront leaves the loop after at most n_pieces claims of all wavefronts together; the
    // workgroup that merges the splits puts the counter back to zero.
    if (n_pieces > 0) {                                             // uniform over the workgroup
        // The (sequence, KV head) pairs hand out their pieces at about the same pace, and their tails sit a fixed
        // stride apart: as with the start tiles above, each pair starts at a piece of its own, chosen by absolute
        // address, and wraps around, so that the pairs' reading positions stay spread over the memory channels.
        unsigned int window = 1;
        while (2 * window <= (unsigned int)n_pieces && window < 512) window *= 2;
        const unsigned int n_pairs = gridDim.y * gridDim.z, pair = blockIdx.z * gridDim.y + blockIdx.y;
        const unsigned int tail_addr = (unsigned int)(((uintptr_t)(kb + (int64_t)a.tail_begin * kHeadDim)) / (kTailKeys * kHeadDim * 2));
        const int turn = (int)(((pair * window / n_pairs - tail_addr) & (window - 1)) % (unsigned int)n_pieces);
        auto first_key = [&](int piece) __attribute__((always_inline)) {
            int at = piece + turn;
            at = at >= n_pieces ? at - n_pieces : at;
            return piece < n_pieces ? a.tail_begin + at * kTailKeys : -1;
        };
        auto second_key = [&](int key_a) __attribute__((always_inline)) { return key_a >= 0 && key_a + 16 < stored ? key_a + 16 : -1; };
        // Pieces are claimed two ahead, so a claim has the time of a whole piece to come back, and the tiles of
        // the next piece are requested as the buffers of the current one are consumed: the loads never pause.
        int key_a = first_key((int)__builtin_amdgcn_readfirstlane(claim_first)), key_b = second_key(key_a);
        fetch(t0, key_a, stored);
        fetch(t1, key_b, stored);
        while (key_a >= 0) {
            const unsigned int claim_after = claim();
            const int next_a = first_key((int)__builtin_amdgcn_readfirstlane(claim_next)), next_b = second_key(next_a);
            consume(t0, key_a, stored, st, qf);
            fetch(t0, next_a, stored);
            if (key_b >= 0) consume(t1, key_b, stored, st, qf);
            fetch(t1, next_b, stored);
            claim_next = claim_after;
            key_a = next_a;
            key_b = next_b;
        }
    }

    // Merge the four rows of the wavefront with the cross-row swap instructions of gfx950 (vector
    // ALU, no LDS round trips).  First the rows agree on a common maximum per head and rescale;
    // then sum_rows4 adds four different values over the four rows at once and leaves the total
    // of value number r in row r, so every lane ends up owning two of its eight dims.
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float mx = max_rows(st.m[h]);
        const float wgt = (st.m[h] == -INFINITY) ? 0.f : fast_exp2(st.m[h] - mx);
        float l = st.l[h];
        l += dpp_move<0x141>(l);                                   // one lane of each quad: the row's sum
        l += dpp_move<0x140>(l);
        st.l[h] = l * wgt;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[h][e] *= wgt;
        st.m[h] = mx;
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float lo = sum_rows4(st.acc[h][0], st.acc[h][1], st.acc[h][2], st.acc[h][3]);   // row r: dim 8*chunk + r
        const float hi = sum_rows4(st.acc[h][4], st.acc[h][5], st.acc[h][6], st.acc[h][7]);   // row r: dim 8*chunk + 4 + r
        sh_acc[wave][h][chunk * 8 + sub] = lo;
        sh_acc[wave][h][chunk * 8 + 4 + sub] = hi;
    }
#pragma unroll
    for (int h0 = 0; h0 < G; h0 += 4) {                            // the sums of heads h0..h0+3 land in rows 0..3
        const float l4 = sum_rows4(st.l[h0], h0 + 1 < G ? st.l[h0 + 1] : 0.f, h0 + 2 < G ? st.l[h0 + 2] : 0.f,
                                   h0 + 3 < G ? st.l[h0 + 3] : 0.f);
        if (chunk == 0 && h0 + sub < G) sh_l[wave][h0 + sub] = l4;
    }
    if (lane == 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) sh_m[wave][h] = st.m[h];
    }
    __syncthreads();

    finish_workgroup<G, kWaves>(a, b, g, split, n_pieces, counter, sh_m, sh_l, &sh_acc[0][0][0], G * kHeadDim);
}

// ---------------------------------------------------------------------------------------------
// The same split decode attention with both products on the matrix cores, for short key ranges.
//
// Over a short range a launch is bound by the vector instructions of process_tile (about 400 per 16-key tile
// for four heads: the time of eight tiles per SIMD, not the bytes, ends a launch over 2048 entries).  Here a
// wavefront still loads its tiles the same way (one coalesced kilobyte per load, two tiles in flight), but hands
// each pair of tiles to v_mfma_f32_16x16x32_bf16 through a stretch of LDS of its own:
//   S^T = K Q^T   rows = 16 keys, columns = 16 head slots (G of them in use), contraction over 32 dims per
//                 instruction: K rows are written to LDS as loaded and read back one row per lane;
//   O^T = V^T P^T rows = 16 dims, columns = head slots, contraction over the 32 keys of the pair: V is
//                 transposed 8 x 4 in registers (four keys of a lane's eight dims) on its way into LDS.
// A lane's logits of a tile are those of keys 4 i + j (i = 0..3, j = lane / 16), the keys whose V entries the
// transposing lane j wrote side by side, so the probabilities a lane computes are, packed to bf16, its own piece of
// the B operand.  They go in as two bf16 terms (p = hi + lo): a single bf16 would put 2^-9 of relative error on
// every probability, which the 2e-3 bound on the output does not leave room for; K, Q and V are bf16 already, so
// their products are exact and everything is accumulated in fp32.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_t;
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2v_t __attribute__((ext_vector_type(2)));

constexpr int kMfmaKRow = 2 * kHeadDim + 16;              // bytes of a K row in LDS: 16 bytes of padding spread the row reads over the banks
constexpr int kMfmaVRow = 64 + 16;                        // bytes of a V^T row: 32 key slots of the pair, padded
constexpr int kMfmaWaveBytes = 16 * kMfmaKRow + kHeadDim * kMfmaVRow;   // one K tile + the pair's V^T: 14592 bytes per wavefront

__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi)
{
    const float2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2v_t));
}

__device__ __forceinline__ float sum_rows(float x)                 // sum of x over the four 16-lane rows, in every row
{
    float a = x, b = x;
    swap_rows16(a, b);
    const float s = a + b;
    a = s;
    b = s;
    swap_rows32(a, b);
    return a + b;
}

template <int G, int LAZY_TAG, int kWaves, int kMode>
__global__ __launch_bounds__(64 * kWaves) void lt_decode_mfma_kernel(DecodeArgs a, typename ModeArgs<kMode>::type r)
{
    constexpr bool kRagged = kMode != kUniform, kPaged = kMode == kPagedMode;
    __shared__ float sh_m[kWaves][G];
    __shared__ float sh_l[kWaves][G];
    __shared__ __attribute__((aligned(16))) char sh_stage[kWaves][kMfmaWaveBytes];   // later: each wavefront's accumulators

    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sub = lane >> 4, chunk = lane & 15;               // as a loader: keys 4 i + sub, dims 8 chunk .. 8 chunk + 7
    const int slot = lane & 15, j = lane >> 4;                  // as a matrix operand: row / column `slot`, k-slice j

    int stored = a.stored;
    if constexpr (kRagged) stored = lengths_of(r).stored_b[b];
    const int begin_key = split * a.keys_per_block;
    // the workgroup's own range ends where the shared tail begins (see lt_decode_kernel); a tile lies inside the range
    // or inside the tail, so `stored` is the only bound a key has to be checked against
    const int end_key = min(min(stored, a.tail_begin), begin_key + a.keys_per_block);
    const int n_tiles = max((end_key - begin_key + 15) >> 4, 0);
    const int wrap = max(n_tiles, 1);
    uint16_t *kb = a.k_cache + (int64_t)b * a.stride_b + (int64_t)g * a.stride_h;
    uint16_t *vb = a.v_cache + (int64_t)b * a.stride_b + (int64_t)g * a.stride_h;
    int new_slot = a.k_new != nullptr ? a.new_slot : -1;
    if constexpr (kRagged) new_slot = a.k_new != nullptr ? lengths_of(r).new_slot_b[b] : -1;
    const int64_t new_off = new_slot >= 0 ? ((int64_t)b * a.n_kv_heads + g) * kHeadDim : 0;
    const uint16_t *k_new = a.k_new + new_off;
    const uint16_t *v_new = a.v_new + new_off;
    const uint16_t *hot = a.q + ((int64_t)b * a.n_q_heads + g * G) * kHeadDim;
    RangePages<kPaged> range_pages;                              // paged cache: see RangePages
    range_pages.load(r, b, lane, begin_key, end_key, n_tiles);
    if constexpr (kPaged) {
        kb = a.k_cache;
        vb = a.v_cache;
    }
    auto tile_shift = [&](int key0) -> int64_t { return range_pages.shift(r, key0, begin_key, a.n_kv_heads, g); };
    auto fetch = [&](Tile &t, int key0) __attribute__((always_inline)) {
        const int64_t shift = tile_shift(key0);
        load_tile(t, kb + shift, vb + shift, key0, sub, chunk, stored - 1, new_slot, k_new, v_new, hot);
    };
    auto put_new_token = [&](const Tile &t, int key0) __attribute__((always_inline)) {
        if (new_slot >= key0 && new_slot < key0 + 16) {             // wave-uniform, true for one tile of one workgroup
            const int64_t shift = tile_shift(key0);
            store_new_token(t, kb + shift, vb + shift, key0, sub, chunk, stored - 1, new_slot);
        }
    };

    // Q^T as the B operand: column `slot` is head g G + slot (zeros beyond the group), k-slice j of k-block kb is
    // dims 32 kb + 8 j .. + 7
    bf16x8_t qb[4];
#pragma unroll
    for (int kq = 0; kq < 4; ++kq) {
        u32x4_t u = {0u, 0u, 0u, 0u};
        if (slot < G) u = load16(a.q + ((int64_t)b * a.n_q_heads + g * G + slot) * kHeadDim + 32 * kq + 8 * j);
        qb[kq] = __builtin_bit_cast(bf16x8_t, u);
    }

    const int phase = start_tile(a, kb + (int64_t)begin_key * kHeadDim, begin_key, wrap, page_shift_of(r));
    const int my_tiles = wave < n_tiles ? (n_tiles - wave + kWaves - 1) / kWaves : 0;
    int next_tile = wave + phase, fetched = 0;
    while (next_tile >= wrap) next_tile -= wrap;
    auto advance = [&]() {                                          // first key of the next tile to fetch, -1 past the last
        const int cur = next_tile;
        next_tile += kWaves;
        while (next_tile >= wrap) next_tile -= wrap;
        return fetched++ < my_tiles ? begin_key + 16 * cur : -1;
    };

    char *stage = sh_stage[wave];
    char *k_rows = stage, *v_rows = stage + 16 * kMfmaKRow;
    // this lane's places: where its loaded pieces go, and where its operand rows are read
    const int k_write = sub * kMfmaKRow + chunk * 16;                       // + 4 i rows for load i
    const int k_read = (4 * (slot & 3) + (slot >> 2)) * kMfmaKRow + 16 * j; // operand row `slot` is key 4 (slot % 4) + slot / 4; + 64 per k-block
    const int v_write = 8 * chunk * kMfmaVRow + 16 * sub;                   // + one row per dim of the chunk; 8 bytes further for the pair's second tile
    const int v_read = slot * kMfmaVRow + 16 * j;                           // + 16 rows per dim tile

    float m_run = -INFINITY, l_run = 0.f;       // of this lane's head slot; m_run is the same in the four lanes of a slot
    floatx4_t acc[8];                           // O^T: acc[dt][i] = dim 16 dt + 4 j + i of head slot `slot`
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] = floatx4_t{0.f, 0.f, 0.f, 0.f};

    // S^T of one tile (in LDS rows 0..15) for this lane: logits of keys key0 + 4 i + j, scaled, -inf where there is no key
    auto logits = [&](const Tile &t, int key0, float (&s4)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4_t *>(k_rows + k_write + 4 * i * kMfmaKRow) = t.k[i];
        floatx4_t c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kq = 0; kq < 4; ++kq) {
            const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t *>(k_rows + k_read + 64 * kq));
            c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qb[kq], c, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) s4[i] = (key0 >= 0 && key0 + 4 * i + j < stored) ? c[i] * a.scale_log2e : -INFINITY;
    };
    // the V entries of one tile, transposed, into the pair's V^T rows (second: the tile is the pair's second)
    auto park_values = [&](const Tile &t, int second) __attribute__((always_inline)) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            // dims 2 w (low halves) and 2 w + 1 (high halves) of the lane's four keys
            const uint32_t e0 = __builtin_amdgcn_perm(t.v[1][w], t.v[0][w], 0x05040100u), e1 = __builtin_amdgcn_perm(t.v[3][w], t.v[2][w], 0x05040100u);
            const uint32_t o0 = __builtin_amdgcn_perm(t.v[1][w], t.v[0][w], 0x07060302u), o1 = __builtin_amdgcn_perm(t.v[3][w], t.v[2][w], 0x07060302u);
            typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2_t;
            *reinterpret_cast<u32x2_t *>(v_rows + v_write + (2 * w) * kMfmaVRow + 8 * second) = u32x2_t{e0, e1};
            *reinterpret_cast<u32x2_t *>(v_rows + v_write + (2 * w + 1) * kMfmaVRow + 8 * second) = u32x2_t{o0, o1};
        }
    };

    // The shared tail (see lt_decode_kernel): pieces of two tiles handed out by a counter of the (sequence, KV head).
    // The first two claims are made right away -- every wavefront is in for two pieces -- and each later one when a
    // piece is taken up, so a claim has come back long before its piece is needed.
    const int n_pieces = stored > a.tail_begin ? (stored - a.tail_begin + kTailKeys - 1) / kTailKeys : 0;
    unsigned int *counter = a.tickets + ((int64_t)b * a.n_kv_heads + g) * kTicketStride + 1;
    auto claim = [&]() __attribute__((always_inline)) {
        unsigned int c = 0;
        if (lane == 0) c = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return c;
    };
    unsigned int claim_a = 0, claim_b = 0;
    int turn = 0;
    if (n_pieces > 0) {
        claim_a = claim();
        claim_b = claim();
        unsigned int window = 1;
        while (2 * window <= (unsigned int)n_pieces && window < 512) window *= 2;
        const unsigned int n_pairs = gridDim.y * gridDim.z, pair = blockIdx.z * gridDim.y + blockIdx.y;
        const unsigned int tail_addr = (unsigned int)(((uintptr_t)(kb + (int64_t)a.tail_begin * kHeadDim)) / (kTailKeys * kHeadDim * 2));
        turn = (int)(((pair * window / n_pairs - tail_addr) & (window - 1)) % (unsigned int)n_pieces);
    }
    // first keys of the two tiles of a piece of the tail (-1: no such piece, or no second tile)
    auto piece_keys = [&](unsigned int claimed, int &key_a, int &key_b) __attribute__((always_inline)) {
        const int piece = (int)__builtin_amdgcn_readfirstlane(claimed);
        int at = piece + turn;
        at = at >= n_pieces ? at - n_pieces : at;
        key_a = piece < n_pieces ? a.tail_begin + at * kTailKeys : -1;
        key_b = key_a >= 0 && key_a + 16 < stored ? key_a + 16 : -1;
    };

    // One pair of tiles: new token into the cache, both tiles to LDS, the registers refilled with the next pair,
    // then the two products.
    auto work = [&](Tile &ta, Tile &tb, int &key_a, int &key_b, int after_a, int after_b) __attribute__((always_inline)) {
        put_new_token(ta, key_a);
        if (key_b >= 0) put_new_token(tb, key_b);
        float s[8];
        logits(ta, key_a, reinterpret_cast<float (&)[4]>(s[0]));
        logits(tb, key_b, reinterpret_cast<float (&)[4]>(s[4]));
        park_values(ta, 0);
        park_values(tb, 1);
        // the registers are free: the next pair travels while this one is worked on (refilling each tile as soon as
        // it was in LDS, half a pair earlier, was slower)
        key_a = after_a;
        key_b = after_b;
        fetch(ta, key_a);
        fetch(tb, key_b);

        // online softmax of the head slot over the pair's 32 keys (8 per lane, the four lanes of a slot together)
        float tmax = s[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) tmax = fmaxf(tmax, s[i]);
        tmax = max_rows(tmax);
        if (__any(tmax > m_run)) {
            const float m_new = fmaxf(m_run, tmax);
            const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(m_run - m_new);   // 0 while m_run = -inf
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[dt][i] *= alpha;
        }
        const float m_safe = (m_run == -INFINITY) ? 0.f : m_run;
        float p[8], p_hi[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            p[i] = fast_exp2(s[i] - m_safe);
            l_run += p[i];
        }
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            hi[i] = pack_bf16_pair(p[2 * i], p[2 * i + 1]);
            p_hi[2 * i] = bf16_lo(hi[i]);
            p_hi[2 * i + 1] = bf16_hi(hi[i]);
            lo[i] = pack_bf16_pair(p[2 * i] - p_hi[2 * i], p[2 * i + 1] - p_hi[2 * i + 1]);
        }
        const bf16x8_t b_hi = __builtin_bit_cast(bf16x8_t, u32x4_t{hi[0], hi[1], hi[2], hi[3]});
        const bf16x8_t b_lo = __builtin_bit_cast(bf16x8_t, u32x4_t{lo[0], lo[1], lo[2], lo[3]});
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t *>(v_rows + v_read + 16 * dt * kMfmaVRow));
            acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, b_hi, acc[dt], 0, 0, 0);
            acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, b_lo, acc[dt], 0, 0, 0);
        }
    };

    // The wavefront's own tiles, pair by pair; the last pair is followed by the wavefront's first piece of the tail
    // (claimed at the start), so that the loads do not pause between the two parts.  No claim is made inside this loop:
    // the wait counts of its loads stay exact.
    Tile t0, t1;
    int key0 = advance(), key1 = advance();
    if (key0 < 0 && n_pieces > 0) piece_keys(claim_a, key0, key1);         // a wavefront without tiles of its own
    fetch(t0, key0);
    fetch(t1, key1);
    for (int k = 0; k < my_tiles; k += 2) {
        int after_a = advance(), after_b = advance();
        if (after_a < 0 && n_pieces > 0) piece_keys(claim_a, after_a, after_b);     // the last round
        work(t0, t1, key0, key1, after_a, after_b);
    }
    // the tail: the piece after the one in hand was claimed a round ago (or at the start)
    while (n_pieces > 0 && key0 >= 0) {
        int after_a, after_b;
        piece_keys(claim_b, after_a, after_b);
        claim_b = claim();
        work(t0, t1, key0, key1, after_a, after_b);
    }

    // this wavefront's partial result into LDS: its accumulators go where its tiles were (nobody else reads there)
    const float l_slot = sum_rows(l_run);
    float *acc_out = reinterpret_cast<float *>(stage);
    if (slot < G) {
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) *reinterpret_cast<floatx4_t *>(acc_out + slot * kHeadDim + 16 * dt + 4 * j) = acc[dt];
        if (j == 0) {
            sh_m[wave][slot] = m_run;
            sh_l[wave][slot] = l_slot;
        }
    }
    __syncthreads();
    finish_workgroup<G, kWaves>(a, b, g, split, n_pieces, counter, sh_m, sh_l,
                                reinterpret_cast<const float *>(&sh_stage[0][0]), kMfmaWaveBytes / 4);
}

__global__ void lt_zero_tickets_kernel(unsigned int *tickets, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) tickets[i] = 0u;
}

template <int G, int LAZY_TAG, int kMode>
hipError_t launch_decode_as(const DecodeArgs &a, const typename ModeArgs<kMode>::type &r, hipStream_t stream)
{
    const dim3 grid(a.n_splits, a.n_kv_heads, a.batch);
    // either kernel: eight wavefronts per workgroup for short ranges, four for long ones
    if (a.matrix_cores) {
        if (a.keys_per_block <= kWideBlockKeys) hipLaunchKernelGGL((lt_decode_mfma_kernel<G, LAZY_TAG, 8, kMode>), grid, dim3(512), 0, stream, a, r);
        else hipLaunchKernelGGL((lt_decode_mfma_kernel<G, LAZY_TAG, 4, kMode>), grid, dim3(256), 0, stream, a, r);
        return hipGetLastError();
    }
    // the vector kernel with groups of eight heads always has four: its state needs more than the 256 registers a
    // wavefront has when two share a SIMD
    if constexpr (G < 8) {
        if (a.keys_per_block <= kWideBlockKeys) {
            hipLaunchKernelGGL((lt_decode_kernel<G, LAZY_TAG, 8, kMode>), grid, dim3(512), 0, stream, a, r);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((lt_decode_kernel<G, LAZY_TAG, 4, kMode>), grid, dim3(256), 0, stream, a, r);
    return hipGetLastError();
}

template <int G>
hipError_t launch_decode(const DecodeArgs &a, const RaggedArgs *ragged, const PagedArgs *paged, hipStream_t stream)
{
    if (paged != nullptr) return launch_decode_as<G, 0, kPagedMode>(a, *paged, stream);   // only full layers are paged
    if (ragged != nullptr)
        return a.lazy_tag ? launch_decode_as<G, 1, kRaggedMode>(a, *ragged, stream) : launch_decode_as<G, 0, kRaggedMode>(a, *ragged, stream);
    return a.lazy_tag ? launch_decode_as<G, 1, kUniform>(a, NoRaggedArgs{}, stream) : launch_decode_as<G, 0, kUniform>(a, NoRaggedArgs{}, stream);
}

}  // namespace

hipError_t append(const AppendArgs &a, hipStream_t stream)
{
    const int64_t per_stream = a.n_new * 16;
    const dim3 grid((unsigned)((per_stream + 255) / 256), a.n_kv_heads, a.batch);
    hipLaunchKernelGGL(lt_append_kv_kernel, grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t truncate(const TruncateArgs &a, hipStream_t stream)
{
    const int64_t kept = (a.total < a.w_sink ? a.total : a.w_sink) + (a.total < a.w_recent ? a.total : a.w_recent);
    const dim3 grid((unsigned)((kept * 16 + 255) / 256), a.n_kv_heads, a.batch);    // an upper bound on the kept tokens
    hipLaunchKernelGGL(lt_truncate_kernel, grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t decode(const DecodeArgs &a, const RaggedArgs *ragged, const PagedArgs *paged, hipStream_t stream)
{
    switch (a.n_q_heads / a.n_kv_heads) {
    case 1: return launch_decode<1>(a, ragged, paged, stream);
    case 2: return launch_decode<2>(a, ragged, paged, stream);
    case 3: return launch_decode<3>(a, ragged, paged, stream);
    case 4: return launch_decode<4>(a, ragged, paged, stream);
    case 5: return launch_decode<5>(a, ragged, paged, stream);
    case 6: return launch_decode<6>(a, ragged, paged, stream);
    case 7: return launch_decode<7>(a, ragged, paged, stream);
    case 8: return launch_decode<8>(a, ragged, paged, stream);
    default: return hipErrorInvalidValue;
    }
}

namespace {
// Plain streaming read of a buffer: every workgroup reads its own contiguous share with 16-byte
// non-temporal loads, eight in flight per lane.  The read rate this device sustains, against which
// the decode kernel's rate can be read.
constexpr int kProbeBlocks = 1024;
__global__ __launch_bounds__(256) void lt_probe_read_kernel(const u32x4_t *buf, int64_t per_block, uint32_t *sink)
{
    const u32x4_t *base = buf + (int64_t)blockIdx.x * per_block;
    uint32_t acc = 0;
    for (int64_t i = threadIdx.x; i < per_block; i += 256 * 8) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            int64_t idx = i + u * 256;
            idx = idx < per_block ? idx : per_block - 1;
            v[u] = __builtin_nontemporal_load(base + idx);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    if (acc == 0x9e3779b9u) sink[threadIdx.x & 63] = acc;          // keeps the loads; practically never taken
}
}  // namespace

hipError_t probe_read(const void *buf, int64_t bytes, uint32_t *sink, hipStream_t stream)
{
    const int64_t per_block = bytes / 16 / kProbeBlocks;            // the API layer asks for at least 16 bytes per workgroup
    hipLaunchKernelGGL(lt_probe_read_kernel, dim3(kProbeBlocks), dim3(256), 0, stream, static_cast<const u32x4_t *>(buf), per_block, sink);
    return hipGetLastError();
}

hipError_t zero_tickets(unsigned int *tickets, int n, hipStream_t stream)
{
    hipLaunchKernelGGL(lt_zero_tickets_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, tickets, n);
    return hipGetLastError();
}

}  // namespace ltk
