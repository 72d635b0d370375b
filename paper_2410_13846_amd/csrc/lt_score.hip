// Lazy-ratio scoring for gfx950 (Eq. 1): the last w prompt queries of every head against all
// prompt keys, as a dense bf16 contraction on the matrix cores with fp32 accumulation, reduced
// on the fly to two sums per query -- the softmax denominator over the causal set and the part
// of it that falls on the initial + recent keys.  No attention matrix and no V are touched.
//
// One launch.  One workgroup of eight wavefronts (two per SIMD, which fill each other's stalls; the
// barrier of every tile keeps them in step, so no wavefront is left to run alone at the end) = one
// (sequence, KV head, range of keys).  K tiles travel from global memory straight into LDS
// (global_load_lds_dwordx4, the next tile(s) under way while one is contracted), laid out with an
// XOR swizzle of the 16-byte pieces of a row so that the matrix-operand reads are free of bank
// conflicts.  S^T = K Q^T is formed with v_mfma_f32_32x32x16_bf16: keys are the rows, queries the
// columns, so each lane keeps 16 key logits of ONE query per instruction and the running max /
// sums stay private to the lane until the final merge.  A wavefront owns one or two 32-query
// tiles: every K fragment read from LDS feeds that many matrix instructions.  The matrix
// instructions of one 32-key sub-tile are issued in the same instruction stream as the
// exponentials of the previous sub-tile (two accumulator sets).  On this hardware a SIMD does
// not run vector and matrix instructions at the same time, so the kernel's floor is the sum of
// the two (about equal here), not the larger.
// The workgroup that finishes last for a (sequence, KV head) merges the key ranges, and the one
// that finishes last overall forms the means: the order of every sum is fixed.
#include "lt_kernels.h"

#include <mutex>

// Scratch for callers that cannot bring a workspace of their own (code under stream capture,
// serving loops and harnesses that must not allocate): a fixed array inside the code object,
// one copy per device, alive until the process ends.  In host code `scratch` is only a handle
// for the symbol; the device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[ltk::kStaticScratchBytes];

namespace ltk {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;   // 16 bytes moved as one register quad

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct LaneState {
    float m, sum_causal, sum_kept;
};

// Uniform description of a 32-key sub-tile relative to the masks.
struct TileClass {
    bool fast;      // every (key, query) pair is causal and the kept/dropped decision is the same for all pairs
    bool kept;      // on the fast path: all pairs are kept
};

// Positions are 32-bit: the API keeps prompts below 2^30 tokens and the kernel clamps the windows to the prompt.
__device__ __forceinline__ TileClass classify(int j0, int n, int w, int w_sink, int w_recent, int fixed_mode)
{
    const int j1 = j0 + 31;
    const int p_min = n - w, p_max = n - 1;
    TileClass c;
    const bool all_causal = j1 <= p_min;
    bool all_kept, none_kept;
    if (fixed_mode) {
        all_kept = (j1 < w_sink) || (j0 >= n - w_recent);
        none_kept = (j0 >= w_sink) && (j1 < n - w_recent);
    } else {
        all_kept = (j1 < w_sink) || (j0 > p_max - w_recent);
        none_kept = (j0 >= w_sink) && (j1 <= p_min - w_recent);
    }
    c.fast = all_causal && (all_kept || none_kept);
    c.kept = all_kept;
    return c;
}

__device__ __forceinline__ void update_fast(const floatx16_t &c, LaneState &st, float scale_log2e, bool kept)
{
    float tmax = c[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, c[i]);
    const float m_new = fmaxf(st.m, tmax * scale_log2e);
    const float alpha = fast_exp2(st.m - m_new);              // 0 on the first tile (m = -inf)
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(c[i], scale_log2e, -m_new));
    st.sum_causal = st.sum_causal * alpha + sum;
    st.sum_kept = st.sum_kept * alpha + (kept ? sum : 0.f);
    st.m = m_new;
}

// The same without looking for the maximum: the exponentials are formed against the lane's current
// reference and the sub-tile is taken only if their sum stays within 2^12 in every lane (16 terms of at most
// 2^8).  A larger sum, or a NaN while there is no reference yet, sends the whole wavefront through
// update_fast, which moves the reference.  Any reference gives the same quotient of the two sums; the two
// half-wavefronts and the key ranges are merged later by their references.
constexpr float kQuickSumLimit = 4096.f;
__device__ __forceinline__ void update_quick(const floatx16_t &c, LaneState &st, float scale_log2e, bool kept)
{
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(c[i], scale_log2e, -st.m));
    if (__all(sum <= kQuickSumLimit)) {
        st.sum_causal += sum;
        st.sum_kept += kept ? sum : 0.f;
    } else {
        update_fast(c, st, scale_log2e, kept);
    }
}

// j_end: keys from j_end on belong to another workgroup's range (or lie past the prompt) and are left out.
__device__ __forceinline__ void update_masked(const floatx16_t &c, LaneState &st, float scale_log2e, int j_base,
                                              int p, int n, int w_sink, int w_recent, int fixed_mode, int j_end)
{
    // key row of accumulator register i in this lane: j_base + 8*(i/4) + (i%4)
    float tmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int j = j_base + 8 * (i >> 2) + (i & 3);
        if (j <= p && j < j_end) tmax = fmaxf(tmax, c[i]);
    }
    const float m_new = fmaxf(st.m, tmax * scale_log2e);
    if (m_new == -INFINITY) return;                           // nothing causal seen so far
    const float alpha = fast_exp2(st.m - m_new);
    float sum = 0.f, kept = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int j = j_base + 8 * (i >> 2) + (i & 3);
        const bool causal = j <= p && j < j_end;
        const bool recent = fixed_mode ? (j >= n - w_recent) : (j > p - w_recent);
        const float e = causal ? fast_exp2(fmaf(c[i], scale_log2e, -m_new)) : 0.f;
        sum += e;
        kept += (j < w_sink || recent) ? e : 0.f;
    }
    st.sum_causal = st.sum_causal * alpha + sum;
    st.sum_kept = st.sum_kept * alpha + kept;
    st.m = m_new;
}


// ---------------------------------------------------------------------------------------------
// Staging: a tile of TK keys is TK rows of 256 bytes.  Piece c (16 bytes) of row r lives at byte
// r * 256 + ((c ^ (r & 15)) << 4) of its stage.  A wavefront's global_load_lds instruction writes
// 1 KB = four whole rows, lane l to byte 16 * l after the (uniform) destination, so lane l
// fetches piece (l & 15) ^ (row & 15) of row (l >> 4): still one coalesced kilobyte of memory.
// ---------------------------------------------------------------------------------------------
constexpr int kScoreThreads = 512;
constexpr int kScoreWaves = kScoreThreads / 64;

// One global -> LDS load of 16 bytes per lane: lane l's bytes land at LDS byte address lds_base + 16 * l (lds_base is
// uniform and travels in M0).  Written as inline assembly on purpose: for the compiler's own form of this load the
// wait-count insertion makes every later LDS read wait for ALL loads of this kind that are still under way, the
// prefetched tiles included, which would serialise the pipeline.  Here the waits are explicit (wait_vmcnt below; these
// loads count in vmcnt like any other).  No other instruction of these kernels uses M0.
__device__ __forceinline__ void load_to_lds(const void *src, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" : : "v"(src), "s"(lds_base) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char *)p;
}

// Workgroup barrier without a fence: the waits that order LDS traffic around it are written out by hand
// (a fence would wait for ALL outstanding global-to-LDS loads, the prefetched tiles included).
__device__ __forceinline__ void barrier_no_fence()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// s_waitcnt vmcnt(N) for gfx9 (bits 3:0 and 15:14), the other counters left at their maxima
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ void publish(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float observe(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Merge (m2, c2, k2) into (m, c, k): two partial softmax sums with their references (log2 units).
__device__ __forceinline__ void merge_state(float &m, float &c, float &k, float m2, float c2, float k2)
{
    if (m2 == -INFINITY) return;
    const float m_new = fmaxf(m, m2);
    const float keep = fast_exp2(m - m_new), add = fast_exp2(m2 - m_new);      // keep = 0 while m = -inf
    c = c * keep + add * c2;
    k = k * keep + add * k2;
    m = m_new;
}

// NT: 32-query tiles per wavefront (1, 2 or 3).  KW: wavefronts that own the same query tiles and share the keys between
// them (1 or 2): the eight wavefronts are 8 / KW tile groups x KW key ways.  An LDS tile holds 64 * KW keys, and every
// wavefront contracts two 32-key sub-tiles of it (sub-tiles kw and kw + KW).
template <int NT, int KW>
__global__ __launch_bounds__(kScoreThreads, 1) void lt_lazy_ratio_kernel(ScoreArgs a)
{
    constexpr int TK = 64 * KW;                                 // keys per tile
    constexpr int kStageBytes = TK * 256;
    constexpr int kScoreStages = 65536 / kStageBytes;           // 2 stages of 32 KB or 4 of 16 KB
    constexpr int kLoads = TK * 16 / kScoreThreads;             // global_load_lds per wavefront and tile
    constexpr int kRowsPerRound = kScoreThreads / 16;           // rows one round of loads of the whole workgroup covers (32)
    constexpr int kGroups = kScoreWaves / KW;
    // The only LDS object of the kernel, so it starts at LDS address 0 and every tile load lands below 64 KB.
    // After the tile loop the same memory carries the lane states, the ratios and a flag.
    __shared__ __attribute__((aligned(1024))) char sh_all[kScoreStages * kStageBytes];
    static_assert(kScoreStages * kStageBytes <= 65536, "tile loads address LDS through a 16-bit offset");
    int *sh_flag = reinterpret_cast<int *>(sh_all + 65536 - 64);            // far past the states, sums and ratios

    const int chunk = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: what depends on it stays in scalar registers
    const int col = lane & 31, half = lane >> 5;
    const int tg = wave % kGroups, kw = wave / kGroups;         // tile group and key way of this wavefront
    const int G = a.n_q_heads / a.n_kv_heads;
    const int QH = (a.w_last + 31) >> 5;                        // 32-query tiles per head
    const int QT = G * QH;                                      // query tiles of this KV head's group

    const int n = (int)a.n;
    const int w_sink = min(a.w_sink, n), w_recent = min(a.w_recent, n);   // a window longer than the prompt is the prompt
    int begin_key, end_key;
    if (chunk < a.n_chunks_a) {
        begin_key = chunk * a.keys_per_block;
        end_key = min((int)a.range_a_end, begin_key + a.keys_per_block);
    } else {
        begin_key = (int)a.range_b_begin + (chunk - a.n_chunks_a) * a.keys_per_block;
        end_key = min(n, begin_key + a.keys_per_block);
    }
    const int n_tiles = (end_key - begin_key + TK - 1) / TK;
    const uint16_t *kb = a.k + (int64_t)b * a.k_stride_b + (int64_t)g * a.k_stride_h;
    const uint16_t *hot = a.q_last + ((int64_t)b * a.n_q_heads + g * G) * a.w_last * kHeadDim;   // a line that is in cache anyway

    // ---- tile loads ---------------------------------------------------------------------------------------
    // this lane's row inside a round of loads (32 rows) and the piece it fetches (see the layout above)
    const int my_row = wave * 4 + (lane >> 4);
    const int my_piece = (lane & 15) ^ (my_row & 15);
    int next_issue = 0;
    const uint32_t lds_base = lds_address(sh_all);              // 0
    // source of this lane's first load of the next tile; the tile's other loads are 32 rows apart each
    const uint16_t *next_src = kb + (int64_t)(begin_key + my_row) * a.k_stride_t + my_piece * 8;
    const int64_t rows_round = kRowsPerRound * a.k_stride_t;
    auto issue = [&]() __attribute__((always_inline)) {        // tile `next_issue` -> its stage; past the last tile: dummy loads
        const int j0 = begin_key + next_issue * TK;
        const uint32_t stage_base = lds_base + (next_issue & (kScoreStages - 1)) * kStageBytes;
        if (next_issue < n_tiles && j0 + TK <= n) {             // the common case: every row exists
#pragma unroll
            for (int i = 0; i < kLoads; ++i) load_to_lds(next_src + i * rows_round, stage_base + (i * kRowsPerRound + wave * 4) * 256);
        } else {
#pragma unroll
            for (int i = 0; i < kLoads; ++i) {
                int j = j0 + i * kRowsPerRound + my_row;
                j = j < n ? j : n - 1;                          // rows past the prompt repeat its last key; they are masked
                const uint16_t *src = next_issue < n_tiles ? kb + (int64_t)j * a.k_stride_t + my_piece * 8 : hot + (lane & 15) * 8;
                load_to_lds(src, stage_base + (i * kRowsPerRound + wave * 4) * 256);
            }
        }
        next_src += TK * a.k_stride_t;
        ++next_issue;
    };

    // the first tile(s) are requested before anything else, so that they travel while the query fragments are fetched
    constexpr int kAhead = kScoreStages - 1;
#pragma unroll
    for (int i = 0; i < kAhead; ++i) issue();

    // ---- Q^T fragments (B operand): lane holds, for its query column, the 8 dims 16*s + 8*half .. +7 ---------
    bf16x8_t qf[NT][8];
    int q_pos[NT];                                              // prompt position of this lane's query column per tile
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int qt = tg * NT + nt;
        const int h = g * G + qt / QH;
        const int t = (qt % QH) * 32 + col;
        const bool live = qt < QT && t < a.w_last;
        q_pos[nt] = n - a.w_last + t;
        // dead columns read the group's first query (in bounds) and are zeroed: no branch around the loads
        const uint16_t *src = a.q_last + (((int64_t)b * a.n_q_heads + (live ? h : g * G)) * a.w_last + (live ? t : 0)) * kHeadDim + 8 * half;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const uint4 u = *reinterpret_cast<const uint4 *>(src + 16 * s);
            qf[nt][s] = __builtin_bit_cast(bf16x8_t, live ? u : make_uint4(0u, 0u, 0u, 0u));
        }
    }
    // the fragments and this wavefront's part of the first tile(s) have arrived
    wait_vmcnt<0>();

    LaneState st[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) { st[nt].m = -INFINITY; st[nt].sum_causal = 0.f; st[nt].sum_kept = 0.f; }

    // LDS byte offset of this lane's K fragment for k-step s of this wavefront's first sub-tile of stage 0: row
    // 32 * kw + col, piece 2s + half, swizzled.  The stage and the second sub-tile add compile-time constants, which
    // travel in the offset field of the LDS read: no address arithmetic in the loop.
    int frag_off[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) frag_off[s] = (32 * kw + col) * 256 + (((half ^ (col & 15)) << 4) ^ (s << 5));
    auto k_fragment = [&](int const_bytes, int s) __attribute__((always_inline)) {
        return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t *>(sh_all + frag_off[s] + const_bytes));
    };

    // Fold one sub-tile's logits (masked form): per-element predicates of Eq. 1, and keys outside this workgroup's range out
    auto fold_masked = [&](const floatx16_t (&c)[NT], int j0) __attribute__((always_inline)) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            update_masked(c[nt], st[nt], a.scale_log2e, j0 + 4 * half, q_pos[nt], n, w_sink, w_recent, a.fixed_mode, end_key);
    };
    // Is the whole sub-tile on the mask-free path?
    auto fast_class = [&](int j0, bool &kept) __attribute__((always_inline)) {
        const TileClass cls = classify(j0, n, a.w_last, w_sink, w_recent, a.fixed_mode);
        kept = cls.kept;
        return cls.fast && j0 + 32 <= end_key;
    };

    // Contract the sub-tile at constant byte offset `stage` (from this wavefront's first sub-tile of stage 0) into `next` while folding `prev` (the logits of the sub-tile that began at key
    // j_prev; j_prev < 0: nothing to fold).  On the mask-free path the exponentials of `prev` are issued between the
    // matrix instructions of `next`, two accumulator registers per tile and k-step, against each lane's current
    // reference; the sums are taken only if they stay within 2^12 in every lane, else `prev` is folded again the
    // long way, which moves the reference (any reference gives the same quotient of the two sums).
    auto step = [&](floatx16_t (&next)[NT], int stage, const floatx16_t (&prev)[NT], int j_prev) __attribute__((always_inline)) {
        bool kept = false;
        const bool quick = j_prev >= 0 && fast_class(j_prev, kept);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) next[nt][i] = 0.f;
        if (quick) {
            float sum[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) sum[nt] = 0.f;
            // The order is pinned: one matrix instruction, then the six vector instructions of two logits, and so on,
            // with the K fragment of the next k-step requested one step ahead.  A matrix instruction leaves part of its
            // issue time open to vector instructions of the same wavefront, but only if they sit right behind it.
            bf16x8_t kf = k_fragment(stage, 0);
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const bf16x8_t kf_next = k_fragment(stage, s < 7 ? s + 1 : 7);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    next[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nt][s], next[nt], 0, 0, 0);
                    sum[nt] += fast_exp2(fmaf(prev[nt][2 * s], a.scale_log2e, -st[nt].m));
                    sum[nt] += fast_exp2(fmaf(prev[nt][2 * s + 1], a.scale_log2e, -st[nt].m));
                    __builtin_amdgcn_sched_barrier(0);
                }
                kf = kf_next;
            }
            bool ok = true;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) ok = ok && sum[nt] <= kQuickSumLimit;
            if (__all(ok)) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    st[nt].sum_causal += sum[nt];
                    st[nt].sum_kept += kept ? sum[nt] : 0.f;
                }
            } else {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) update_fast(prev[nt], st[nt], a.scale_log2e, kept);
            }
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const bf16x8_t kf = k_fragment(stage, s);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) next[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nt][s], next[nt], 0, 0, 0);
            }
            if (j_prev >= 0 && j_prev < end_key) fold_masked(prev, j_prev);
        }
    };

    // ---- main loop: tile t sits in stage t % kScoreStages; the following kScoreStages - 1 tiles are on their way ---------
    floatx16_t acc_a[NT], acc_b[NT];
    barrier_no_fence();                                         // everybody's part of tile 0 has landed (each waited above)
    int j_pending = -1;                                         // first key of the sub-tile whose logits wait (in acc_b) to be folded
    for (int tile0 = 0; tile0 < n_tiles; tile0 += kScoreStages) {
#pragma unroll
        for (int u = 0; u < kScoreStages; ++u) {                // the stage of tile tile0 + u is u: a constant in the unrolled body
            const int tile = tile0 + u;
            if (tile >= n_tiles) break;
            issue();                                            // into the stage tile - 1 was read from (all past the last barrier)
            const int j0 = begin_key + tile * TK;
            step(acc_a, u * kStageBytes, acc_b, j_pending);                        // sub-tile kw, while the previous tile's second one is folded
            step(acc_b, u * kStageBytes + 32 * KW * 256, acc_a, j0 + 32 * kw);     // sub-tile kw + KW, while the first is folded
            j_pending = j0 + 32 * (kw + KW);
            wait_vmcnt<(kAhead - 1) * kLoads>();                // tile + 1 has landed (later ones may still be under way)
            barrier_no_fence();                                 // everybody is done reading tile `tile`, and tile + 1 is complete
        }
    }
    wait_vmcnt<0>();                                            // the dummy loads past the last tile
    if (j_pending >= 0 && j_pending < end_key) {
        bool kept = false;
        if (fast_class(j_pending, kept)) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) update_quick(acc_b[nt], st[nt], a.scale_log2e, kept);
        } else {
            fold_masked(acc_b, j_pending);
        }
    }
    barrier_no_fence();                                         // the stages are free: they carry the lane states next

    // ---- merge the lanes and wavefronts that saw different keys of the same query ----------------------------------------------
    float *sh_state = reinterpret_cast<float *>(sh_all);  // [wave][nt][3][64]
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float *dst = sh_state + ((wave * NT + nt) * 3) * 64 + lane;
        dst[0] = st[nt].m;
        dst[64] = st[nt].sum_causal;
        dst[128] = st[nt].sum_kept;
    }
    __syncthreads();
    // entry e = (query tile qt, column): at most 16 * 32 = 512 of them, one per thread
    constexpr int kRounds = 1;
    float fin_m[kRounds], fin_c[kRounds], fin_k[kRounds];
    const bool single = a.n_chunks == 1;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int e = threadIdx.x + r * kScoreThreads;
        const int qt = e >> 5, c = e & 31;
        fin_m[r] = -INFINITY; fin_c[r] = 0.f; fin_k[r] = 0.f;
        const int t = (qt % QH) * 32 + c;
        if (qt >= QT || t >= a.w_last) continue;
        const int src_tg = qt / NT, src_nt = qt % NT;
#pragma unroll
        for (int way = 0; way < KW; ++way)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const float *src = sh_state + (((way * kGroups + src_tg) * NT + src_nt) * 3) * 64 + hf * 32 + c;
                merge_state(fin_m[r], fin_c[r], fin_k[r], src[0], src[64], src[128]);
            }
        if (!single) {
            const int h = g * G + qt / QH;
            float *dst = a.part + (((int64_t)b * a.n_q_heads + h) * a.n_chunks + chunk) * 3 * a.w_last + t;
            publish(dst, fin_m[r]);
            publish(dst + a.w_last, fin_c[r]);
            publish(dst + 2 * a.w_last, fin_k[r]);
        }
    }

    // ---- the last workgroup of a (sequence, KV head) merges the key ranges ------------------------------------------------
    // Ordering: device-scope stores complete (vmcnt 0) in every thread, barrier, then one thread takes the ticket
    // with a device-scope atomic; the workgroup that sees the last ticket issues its device-scope loads only after.
    if (!single) {
        wait_vmcnt<0>();
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned int mine = __hip_atomic_fetch_add(a.tickets + (int64_t)b * a.n_kv_heads + g, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *sh_flag = mine == (unsigned int)(a.n_chunks - 1);
        }
        __syncthreads();
        if (!*sh_flag) return;
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const int e = threadIdx.x + r * kScoreThreads;
            const int qt = e >> 5, c = e & 31;
            const int t = (qt % QH) * 32 + c;
            fin_m[r] = -INFINITY; fin_c[r] = 0.f; fin_k[r] = 0.f;
            if (qt >= QT || t >= a.w_last) continue;
            const int h = g * G + qt / QH;
            const float *src = a.part + ((int64_t)b * a.n_q_heads + h) * a.n_chunks * 3 * a.w_last + t;
            // up to 16 key ranges per round trip, requested four at a time and only as far as there are ranges (these
            // loads go past the caches: every one costs a memory access), merged in range order
            constexpr int kBatch = 16;
            for (int c0 = 0; c0 < a.n_chunks; c0 += kBatch) {
                float m[kBatch], f[kBatch], k[kBatch];
#pragma unroll
                for (int u0 = 0; u0 < kBatch; u0 += 4)
                    if (c0 + u0 < a.n_chunks) {                     // uniform
#pragma unroll
                        for (int u = u0; u < u0 + 4; ++u) {
                            const float *pc = src + (int64_t)min(c0 + u, a.n_chunks - 1) * 3 * a.w_last;
                            m[u] = observe(pc);
                            f[u] = observe(pc + a.w_last);
                            k[u] = observe(pc + 2 * a.w_last);
                        }
                    }
#pragma unroll
                for (int u = 0; u < kBatch; ++u)
                    if (c0 + u < a.n_chunks) merge_state(fin_m[r], fin_c[r], fin_k[r], m[u], f[u], k[u]);
            }
        }
    }

    // ---- rho of every (head, query) of the group, and the heads' sums -----------------------------------------------------------
    float *sh_rho = sh_state;                                   // [QT * 32]; the states in there have been consumed
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int e = threadIdx.x + r * kScoreThreads;
        const int qt = e >> 5, c = e & 31;
        const int t = (qt % QH) * 32 + c;
        float rho = 0.f;
        if (qt < QT && t < a.w_last) {
            const int h = g * G + qt / QH;
            if (a.lse_rows != nullptr) {
                // Table 1: the key ranges covered only the initial and recent keys; the whole row's denominator
                // comes from the prefill attention's log-sum-exp
                const float lse = a.lse_rows[(int64_t)b * a.lse_stride_b + (int64_t)h * a.lse_stride_h + t];
                rho = fin_m[r] == -INFINITY ? 0.f : fin_k[r] * fast_exp2(fin_m[r] - lse * 1.44269504088896340736f);
            } else {
                rho = fin_k[r] / fin_c[r];
            }
            if (a.rho != nullptr) a.rho[((int64_t)b * a.n_q_heads + h) * a.w_last + t] = rho;
        }
        if (e < 16 * 32) sh_rho[e] = rho;
    }
    __syncthreads();
    // a head's sum of rho: wavefront w takes head w; lane t holds query t, then a butterfly over the 64 lanes
    // (a fixed order of additions)
    for (int hh = wave; hh < G; hh += kScoreWaves) {
        float v = lane < a.w_last ? sh_rho[(hh * QH + (lane >> 5)) * 32 + (lane & 31)] : 0.f;
#pragma unroll
        for (int mask = 32; mask > 0; mask >>= 1) v += __shfl_xor(v, mask, 64);
        if (lane == 0) publish(a.head_scratch + (int64_t)b * a.n_q_heads + g * G + hh, v);
    }

    // ---- the last (sequence, KV head) to get here forms the means -------------------------------------------------------------
    wait_vmcnt<0>();
    __syncthreads();
    const int n_groups_total = a.batch * a.n_kv_heads;
    unsigned int *done = a.tickets + n_groups_total;
    if (threadIdx.x == 0) {
        const unsigned int mine = __hip_atomic_fetch_add(done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *sh_flag = mine == (unsigned int)(n_groups_total - 1);
    }
    __syncthreads();
    if (!*sh_flag) return;
    // A sequence's mean: one wavefront per sequence, lane h takes head h (h + 64, ... when there are more), then a
    // butterfly over the lanes; eight sequences per wavefront share a memory round trip.  Every addition has a
    // fixed place, so the result does not depend on the launch.
    float *sh_sum = sh_state;                                   // [kScoreWaves]
    float wave_sum = 0.f;
    for (int b0 = wave; b0 < a.batch; b0 += 8 * kScoreWaves) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int bb = b0 + u * kScoreWaves;
            v[u] = 0.f;
            if (bb < a.batch)                                       // uniform over the wavefront
                for (int h = lane; h < a.n_q_heads; h += 64) v[u] += observe(a.head_scratch + (int64_t)bb * a.n_q_heads + h);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int bb = b0 + u * kScoreWaves;
            float x = v[u];
#pragma unroll
            for (int mask = 32; mask > 0; mask >>= 1) x += __shfl_xor(x, mask, 64);
            if (bb < a.batch) {
                const float rseq = x / (float)(a.n_q_heads * a.w_last);
                if (lane == 0 && a.ratio_seq != nullptr) a.ratio_seq[bb] = rseq;
                wave_sum += rseq;
            }
        }
    }
    __syncthreads();                                            // sh_state is no longer read as rho
    if (lane == 0) sh_sum[wave] = wave_sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float total = 0.f;
#pragma unroll
        for (int w = 0; w < kScoreWaves; ++w) total += sh_sum[w];
        a.ratio_mean[0] = total / (float)a.batch;
    }
}

__global__ void lt_score_zero_tickets_kernel(unsigned int *tickets, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) tickets[i] = 0u;
}

}  // namespace

namespace {
constexpr int kMaxDevices = 64;
void *scratch_ptr[kMaxDevices];                 // device address of `scratch` on each device, nullptr until asked
std::mutex scratch_mutex;
}  // namespace

hipError_t static_scratch(void **ptr)
{
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[device] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        scratch_ptr[device] = p;
    }
    *ptr = scratch_ptr[device];
    return hipSuccess;
}

hipError_t lazy_ratio(const ScoreArgs &a, hipStream_t stream)
{
    // the counters must start at zero whatever the last launch on this workspace left behind
    const int n_tickets = a.batch * a.n_kv_heads + 1;
    hipLaunchKernelGGL(lt_score_zero_tickets_kernel, dim3((n_tickets + 255) / 256), dim3(256), 0, stream, a.tickets, n_tickets);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // query tiles of a KV head's group, dealt to the eight wavefronts: up to twelve tiles, four tile groups (of one,
    // two or three tiles) x two key ways; more, eight tile groups of two tiles that each see every key.  Ten or twelve
    // tiles (five or six heads of 64 queries) would keep only five or six of those eight busy: 0.31 against 0.25 ms
    // per layer at 32K x batch 8 with five heads per KV head.
    const int QT = (a.n_q_heads / a.n_kv_heads) * ((a.w_last + 31) / 32);
    const dim3 grid(a.n_chunks, a.n_kv_heads, a.batch), block(kScoreThreads);
    if (QT <= 4) hipLaunchKernelGGL((lt_lazy_ratio_kernel<1, 2>), grid, block, 0, stream, a);
    else if (QT <= 8) hipLaunchKernelGGL((lt_lazy_ratio_kernel<2, 2>), grid, block, 0, stream, a);
    else if (QT <= 12) hipLaunchKernelGGL((lt_lazy_ratio_kernel<3, 2>), grid, block, 0, stream, a);
    else if (QT <= 16) hipLaunchKernelGGL((lt_lazy_ratio_kernel<2, 1>), grid, block, 0, stream, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ltk
