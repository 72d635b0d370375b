// Prefill attention for gfx950 (Section "Preliminary", prefilling stage; Appendix "Theoretical
// Analysis": softmax(Q K^T + M) V with the causal mask, or the sink mask of streaming attention):
// every prompt position attends to the positions up to itself, and the kernel also returns the
// log-sum-exp of every row, which the lazy-ratio test of Table 1 reuses.
//
// One workgroup = one (sequence, KV head, block of query positions); its wavefronts are the G
// query heads of the group (times QB consecutive sub-blocks of queries when G is small), each
// with NT 32-query column tiles, and all of them share every K and V tile staged in LDS.  Both products
// run on the matrix cores with v_mfma_f32_32x32x16_bf16 in transposed form:
//   S^T = K Q^T   rows = keys, columns = queries: a lane holds 16 logits of ONE query, so the
//                 running max and sum of a softmax row stay in two lanes (the two halves);
//   O^T = V^T P^T rows = head dims, columns = queries: the probabilities a lane has just
//                 computed are, packed to bf16, exactly the B operand of its own column; the V
//                 tile is transposed in registers on its way into LDS, with the keys of each
//                 group of 16 stored in the order the logits have in the accumulator registers,
//                 so that a lane's eight keys of one dim are one 16-byte read.
// The softmax reference point of a row moves only when the row's maximum has grown by more than
// 2^8 since it was set: any reference gives the same quotient, the probabilities stay below 2^8,
// and the accumulator is rescaled a handful of times per row instead of once per tile.
#include "lt_kernels.h"

namespace ltk {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2_t;
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

constexpr int kTileKeys = 64;                 // keys per LDS tile
constexpr int kKRow = kHeadDim + 8;           // 272-byte K rows: 16-byte reads of 32 rows spread over the banks
constexpr int kVtRow = kTileKeys + 8;         // V^T tile: 128 dim rows of 64 key slots, 144-byte rows (16-byte reads of 16 rows spread over the banks)
constexpr float kRescaleStep = 8.f;           // log2 units the row maximum may exceed the reference before it moves
constexpr float kQuickSumLimit = 4096.f;      // 2^(kRescaleStep + 4): 16 probabilities of at most 2^kRescaleStep

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// v_permlane32_swap exchanges the upper half of its first operand with the lower half of the
// second; the s_nop keep the wait states the instruction needs, which the compiler does not
// track inside an asm statement.
__device__ __forceinline__ void swap_halves(float &a, float &b)
{
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float max_halves(float x)
{
    float a = x, b = x;
    swap_halves(a, b);                        // a = lower half of x in both halves, b = upper half
    return fmaxf(a, b);
}
__device__ __forceinline__ float sum_halves(float x)
{
    float a = x, b = x;
    swap_halves(a, b);
    return a + b;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const float2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

// Who stages what.  The first four wavefronts transpose V (four 16-byte loads each); with eight or more
// wavefronts the others copy K and the first four do not, so that no wavefront holds both sets of
// staging registers: they share the slots of one array.
template <int kWaves>
struct Stage {
    static constexpr bool kSplit = kWaves >= 8;
    static constexpr int kFirst = kSplit ? 256 : 0;                      // first thread that copies K
    static constexpr int kThreads = 64 * kWaves - kFirst;
    static constexpr int kTotal = kTileKeys * 16;                        // 16-byte pieces of one 64 x 128 tile
    static constexpr int kPieces = (kTotal + kThreads - 1) / kThreads;
    static constexpr int kFirstSlot = kSplit ? 0 : 4;                    // K's first slot
    static constexpr int kSlots = kSplit ? (kPieces > 4 ? kPieces : 4) : 4 + kPieces;
};

// The staging loads go through buffer descriptors: a load is (uniform descriptor) + (one per-lane byte
// offset that is the same for every tile and every piece), so moving to the next tile or piece costs
// scalar instructions and no vector ones.  A descriptor covers exactly the rows of the tile that lie
// inside the prompt from its own first row on; the hardware returns zeros for anything past that,
// which is how the ragged last tile is handled (those keys are masked as non-causal anyway).
// Offsets inside a tile are 32-bit: the API keeps the token stride below 2^24.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rows_from(const uint16_t *first_row, int rows_left, int64_t stride_t)
{
    const uint32_t bytes = rows_left > 0 ? ((uint32_t)(rows_left - 1) * (uint32_t)stride_t + kHeadDim) * 2u : 0u;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(first_row), 0, (int)bytes, 0x00020000);   // raw buffer of 32-bit words
}

// K: thread i of the copying threads takes pieces i, i + kThreads, ...; piece x is 16 bytes (x % 16) of row x / 16.
template <int W>
__device__ __forceinline__ void fetch_tile(u32x4_t (&pre)[Stage<W>::kSlots], const uint16_t *base, int64_t stride_t, int j0, int n, uint32_t lane_bytes)
{
    const int me = (int)threadIdx.x - Stage<W>::kFirst;
    if (me < 0) return;
    const uint16_t *tile = base + (int64_t)j0 * stride_t;                // uniform
    const int rows = min(n - j0, kTileKeys);
    constexpr int kPieceRows = Stage<W>::kThreads / 16;
#pragma unroll
    for (int i = 0; i < Stage<W>::kPieces; ++i) {
        const __amdgpu_buffer_rsrc_t src = rows_from(tile + (int64_t)(i * kPieceRows) * stride_t, rows - i * kPieceRows, stride_t);
        if ((i + 1) * Stage<W>::kThreads <= Stage<W>::kTotal || me + i * Stage<W>::kThreads < Stage<W>::kTotal)
            pre[Stage<W>::kFirstSlot + i] = __builtin_amdgcn_raw_buffer_load_b128(src, lane_bytes, 0, 0);
    }
}

template <int W, int kRow>
__device__ __forceinline__ void commit_tile(const u32x4_t (&pre)[Stage<W>::kSlots], uint16_t *sh)
{
    const int me = (int)threadIdx.x - Stage<W>::kFirst;
    if (me < 0) return;
#pragma unroll
    for (int i = 0; i < Stage<W>::kPieces; ++i) {
        const int idx = me + i * Stage<W>::kThreads;
        if (idx < Stage<W>::kTotal) *reinterpret_cast<u32x4_t *>(&sh[(idx >> 4) * kRow + (idx & 15) * 8]) = pre[Stage<W>::kFirstSlot + i];
    }
}

// V staging.  Work item (c, kg) = 8 dims x 4 consecutive keys: four 16-byte loads (one per key), an 8 x 4
// transpose in registers, eight 8-byte LDS writes (one per dim).  The first 256 threads do it.  The rows of
// neighbouring dim chunks start on the same bank (8 rows of 144 bytes are a multiple of 128 bytes), so the four
// lanes that share a key group index take four different groups of four keys, 16 keys apart: any 16 consecutive
// lanes then write 32 different banks (the bank-conflict counter reads 0; it read 23 % of the LDS cycles before).
// Slot of key j (0..63) in a V^T row: 16 (j / 16) + {0, 8, 4, 12}[(j % 16) / 4] + j % 4, i.e. within 16 keys the
// order 0-3, 8-11, 4-7, 12-15: slots 8 h .. 8 h + 7 then hold keys 4 h + {0..3} and 8 + 4 h + {0..3}.
template <int kSlots>
__device__ __forceinline__ void fetch_v(u32x4_t (&pre)[kSlots], const uint16_t *base, int64_t stride_t, int j0, int n, uint32_t lane_bytes)
{
    if (threadIdx.x >= 256) return;
    const uint16_t *tile = base + (int64_t)j0 * stride_t;
    const int rows = min(n - j0, kTileKeys);
#pragma unroll
    for (int r = 0; r < 4; ++r)                  // key r of every group of four: one descriptor, r rows further on
        pre[r] = __builtin_amdgcn_raw_buffer_load_b128(rows_from(tile + (int64_t)r * stride_t, rows - r, stride_t), lane_bytes, 0, 0);
}

template <int kSlots>
__device__ __forceinline__ void commit_v(const u32x4_t (&pre)[kSlots], uint16_t *sh)
{
    if (threadIdx.x >= 256) return;
    const int c = 4 * (threadIdx.x >> 6) + (threadIdx.x & 3), kg = ((threadIdx.x >> 2) & 15) ^ ((threadIdx.x & 3) << 2);
    const int slot = 16 * (kg >> 2) + ((0x0C040800 >> (8 * (kg & 3))) & 0xff);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        // dims 2 w (low halves) and 2 w + 1 (high halves) of the four keys
        const u32x2_t even = {__builtin_amdgcn_perm(pre[1][w], pre[0][w], 0x05040100u), __builtin_amdgcn_perm(pre[3][w], pre[2][w], 0x05040100u)};
        const u32x2_t odd = {__builtin_amdgcn_perm(pre[1][w], pre[0][w], 0x07060302u), __builtin_amdgcn_perm(pre[3][w], pre[2][w], 0x07060302u)};
        *reinterpret_cast<u32x2_t *>(&sh[(8 * c + 2 * w) * kVtRow + slot]) = even;
        *reinterpret_cast<u32x2_t *>(&sh[(8 * c + 2 * w + 1) * kVtRow + slot]) = odd;
    }
}

// G: query heads per KV head.  QB: query sub-blocks per workgroup.  NT: 32-query tiles per wavefront.
template <int G, int QB, int NT>
__global__ __launch_bounds__(64 * G * QB) void lt_prefill_attn_kernel(PrefillArgs a)
{
    constexpr int W = G * QB;                          // wavefronts
    constexpr int kWaveQueries = 32 * NT, kBlockQueries = kWaveQueries * QB;
    __shared__ __attribute__((aligned(16))) uint16_t sh_k[2][kTileKeys * kKRow];
    __shared__ __attribute__((aligned(16))) uint16_t sh_v[2][kHeadDim * kVtRow];
    static_assert(W >= 4, "V staging needs 256 threads");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // in a scalar register: what depends on it branches uniformly
    const int col = lane & 31, half = lane >> 5;

    // Workgroups that run at the same time on one XCD (linear index mod 8) work on neighbouring
    // query blocks of the same (sequence, KV head): they walk the same K/V tiles at the same pace
    // and share them in that XCD's L2.  Within a pair the long (late) query blocks go first.
    // positions are 32-bit (the API keeps prompts below 2^30 tokens); a window longer than the prompt is the prompt
    const int n = (int)a.n;
    const int w_sink = min(a.w_sink, n), w_recent = min(a.w_recent, n);
    const int n_q = (int)a.n_q, q_first = n - n_q;              // the queries are the last n_q of the n positions
    const int n_qb = (n_q + kBlockQueries - 1) / kBlockQueries;
    const int64_t total = (int64_t)n_qb * a.n_kv_heads * a.batch;
    const int64_t per_xcd = (total + 7) / 8;
    const int64_t vid = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (vid >= total) return;
    const int pair = (int)(vid / n_qb), qb = n_qb - 1 - (int)(vid % n_qb);
    const int b = pair / a.n_kv_heads, g = pair % a.n_kv_heads;
    const int h = g * G + wave % G;
    const int q_block = q_first + qb * kBlockQueries;
    const int q0 = q_block + (wave / G) * kWaveQueries;             // first query of this wavefront

    // key tiles the block needs: [0, n_a) and [t_b, t_last]
    const int t_last = (min(q_block + kBlockQueries, n) - 1) / kTileKeys;
    int n_a = 0, t_b = 0;
    if (a.streaming) {
        n_a = min((w_sink + kTileKeys - 1) / kTileKeys, t_last + 1);
        const int first_recent = max(q_block - w_recent + 1, 0);
        t_b = max(n_a, first_recent / kTileKeys);
    }
    const int n_tiles = n_a + (t_last + 1 - t_b);
    auto tile_key = [&](int i) { return (i < n_a ? i : t_b + (i - n_a)) * kTileKeys; };

    // g counts head groups of G query heads; kv_share of them read the same KV head
    const uint16_t *kb = a.k + (int64_t)b * a.kv_stride_b + (int64_t)(g / a.kv_share) * a.kv_stride_h;
    const uint16_t *vb = a.v + (int64_t)b * a.kv_stride_b + (int64_t)(g / a.kv_share) * a.kv_stride_h;

    // Q^T fragments (B operand of S^T = K Q^T): for its query column a lane holds dims 16 s + 8 half .. + 7
    bf16x8_t qf[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int p = q0 + nt * 32 + col;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            u32x4_t u = {0u, 0u, 0u, 0u};
            if (p < n)
                u = *reinterpret_cast<const u32x4_t *>(a.q + (((int64_t)b * a.n_q_heads + h) * n_q + (p - q_first)) * kHeadDim + 16 * s + 8 * half);
            qf[nt][s] = __builtin_bit_cast(bf16x8_t, u);
        }
    }

    floatx16_t acc[4][NT];                     // O^T: [32-dim tile][32-query tile]
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[dt][nt][i] = 0.f;
    float m_ref[NT], l_sum[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) { m_ref[nt] = -INFINITY; l_sum[nt] = 0.f; }

    const int win_sink = a.streaming ? w_sink : 0x7fffffff;       // causal attention: every key counts as "initial"

    // S^T of one 32-key sub-tile for this wavefront's queries, masked (raw dot products; -inf where masked)
    auto scores = [&](floatx16_t (&c)[NT], const uint16_t *tile_k, int kt, int j0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) c[nt][i] = 0.f;
        // the chain runs at raised priority: the SIMD's other wavefronts fill the gaps between the
        // matrix instructions with their exponentials instead of delaying them
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const u32x4_t u = *reinterpret_cast<const u32x4_t *>(&tile_k[(32 * kt + col) * kKRow + 16 * s + 8 * half]);
            const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, u);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) c[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nt][s], c[nt], 0, 0, 0);
        }
        __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int p_min = q0 + nt * 32, p_max = p_min + 31;
            // every (key, query) pair of the sub-tile is attended: causal, and inside the initial tokens or
            // inside every query's recent window
            const bool clear = (j0 + 31 <= p_min) && (!a.streaming || j0 + 31 < w_sink || j0 > p_max - w_recent);
            if (!clear) {
                // positions relative to the sub-tile, clamped so that 32-bit compares decide
                const int p = p_min + col;
                const int p_rel = min(max(p - j0, -1), 32);
                const int sink_rel = min(max(win_sink - j0, 0), 32);
                const int old_rel = min(max(p - w_recent - j0, -1), 32);   // last key before the window
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int j_rel = 8 * (i >> 2) + 4 * half + (i & 3);
                    const bool keep = (j_rel <= p_rel) & ((j_rel < sink_rel) | (j_rel > old_rel));
                    c[nt][i] = keep ? c[nt][i] : -INFINITY;
                }
            }
        }
    };

    // c -> probabilities against the reference `mu` (log2 units), in place; returns each column's sum over the lane's 16 keys
    auto probabilities = [&](floatx16_t &c, float mu) {
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            c[i] = fast_exp2(fmaf(c[i], a.scale_log2e, -mu));
            sum += c[i];
        }
        return sum;
    };

    // O^T += V^T P^T for the probabilities in c
    auto accumulate = [&](const floatx16_t (&c)[NT], const uint16_t *tile_v, int kt) {
        bf16x8_t pf[NT][2];                      // P^T fragments: [query tile][16-key step]
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int sp = 0; sp < 2; ++sp) {
                const u32x4_t u = {pack_bf16(c[nt][8 * sp + 0], c[nt][8 * sp + 1]), pack_bf16(c[nt][8 * sp + 2], c[nt][8 * sp + 3]),
                                   pack_bf16(c[nt][8 * sp + 4], c[nt][8 * sp + 5]), pack_bf16(c[nt][8 * sp + 6], c[nt][8 * sp + 7])};
                pf[nt][sp] = __builtin_bit_cast(bf16x8_t, u);
            }
        // k slots 0..7 of a lane are keys 16 sp + 4 half + {0..3} and 16 sp + 8 + 4 half + {0..3}: the order the
        // logits sit in the accumulator registers 8 sp .. 8 sp + 7, and the order of the V^T slots
        // The lane's offset into the V^T tile is rebuilt from the lane number here rather than kept in a register
        // across the loop: with every register taken the compiler parks such a value in scratch memory, and the
        // reload's wait would also wait for the next tile's global loads.
        int lane_now;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_now));
        const uint16_t *v_rows = tile_v + (lane_now & 31) * kVtRow + 8 * (lane_now >> 5) + 32 * kt;
#pragma unroll
        for (int sp = 0; sp < 2; ++sp)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const u32x4_t u = *reinterpret_cast<const u32x4_t *>(&v_rows[32 * dt * kVtRow + 16 * sp]);
                const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, u);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nt][sp], acc[dt][nt], 0, 0, 0);
            }
    };

    // nothing of the sub-tile is visible to this wavefront's queries: later than all of them, or,
    // for streaming attention, between the initial tokens and every query's window
    auto dead = [&](int j0) {
        return j0 > q0 + kWaveQueries - 1 || (a.streaming && j0 >= w_sink && j0 + 31 <= q0 - w_recent);
    };

    u32x4_t pre[Stage<W>::kSlots];             // staging registers: V in slots 0..3 of the first four wavefronts, K see Stage
    // per-lane byte offsets of the staging loads inside a whole tile (see fetch_tile, fetch_v)
    const uint32_t k_me = threadIdx.x - Stage<W>::kFirst;               // unused by the threads that copy no K
    const uint32_t k_lane_bytes = 2u * ((k_me >> 4) * (uint32_t)a.kv_stride_t + (k_me & 15) * 8);
    const uint32_t v_lane_bytes = 2u * (4 * (((threadIdx.x >> 2) & 15) ^ ((threadIdx.x & 3) << 2)) * (uint32_t)a.kv_stride_t
                                        + (4 * (threadIdx.x >> 6) + (threadIdx.x & 3)) * 8);
    auto prefetch = [&](int t) {
        if (t < n_tiles) {
            fetch_tile<W>(pre, kb, a.kv_stride_t, tile_key(t), n, k_lane_bytes);
            fetch_v(pre, vb, a.kv_stride_t, tile_key(t), n, v_lane_bytes);
        }
    };
    auto park = [&](int t) {                     // registers of tile t -> its LDS buffer, then everyone may read it
        if (t < n_tiles) {
            commit_tile<W, kKRow>(pre, sh_k[t & 1]);
            commit_v(pre, sh_v[t & 1]);
        }
        __syncthreads();
    };

    // One sub-tile with the reference of every row moved first where its maximum has outgrown it.
    auto careful = [&](int t, int kt) {
        const int j0 = tile_key(t) + 32 * kt;
        if (dead(j0)) return;
        floatx16_t c[NT];
        scores(c, sh_k[t & 1], kt, j0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float tmax = c[nt][0];
#pragma unroll
            for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, c[nt][i]);
            tmax = max_halves(tmax) * a.scale_log2e;              // the two lanes of a column share one reference
            const bool grow = tmax > m_ref[nt] + kRescaleStep;
            const float alpha = grow ? fast_exp2(m_ref[nt] - tmax) : 1.f;   // 0 when the reference was -inf
            m_ref[nt] = grow ? tmax : m_ref[nt];
            l_sum[nt] *= alpha;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[dt][nt][i] *= alpha;
            l_sum[nt] += probabilities(c[nt], m_ref[nt] == -INFINITY ? 0.f : m_ref[nt]);
        }
        accumulate(c, sh_v[t & 1], kt);
    };
    // The same without touching the references, and without looking for the maximum: the probabilities are
    // formed against the current reference and the sub-tile is taken only if every lane's sum of its 16
    // stays within 2^(kRescaleStep + 4).  A larger sum (or a NaN: no reference yet) means that some logit is
    // more than kRescaleStep above its reference; then nothing is changed and false is returned.
    auto quick = [&](int t, int kt) {
        const int j0 = tile_key(t) + 32 * kt;
        if (dead(j0)) return true;
        floatx16_t c[NT];
        scores(c, sh_k[t & 1], kt, j0);
        float sum[NT];
        bool fits = true;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            sum[nt] = probabilities(c[nt], m_ref[nt]);
            fits = fits && sum[nt] <= kQuickSumLimit;
        }
        if (!__all(fits)) return false;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) l_sum[nt] += sum[nt];
        accumulate(c, sh_v[t & 1], kt);
        return true;
    };

    prefetch(0);
    // The query fragments must have arrived on every path into the tile loop: otherwise the compiler, which
    // cannot tell how many newer loads may be outstanding, makes the first matrix instruction of EVERY sub-tile
    // wait for all outstanding loads, the next tile's prefetch issued just before it included.  Placed after the
    // first tile's loads were issued, the wait costs nothing: park(0) needs those loads next anyway.
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0); expcnt and lgkmcnt left at their maxima
    park(0);
    // The accumulator is multiplied only in the outer loop; the inner loop, which runs until some
    // row's maximum outgrows its reference, touches it with matrix instructions alone, so it can
    // stay in the accumulation registers for the whole stretch.
    int t = 0, kt = 0;
    while (t < n_tiles) {
        if (kt == 0) {
            prefetch(t + 1);
            careful(t, 0);
        }
        careful(t, 1);
        park(t + 1);
        ++t;
        kt = 0;
        while (t < n_tiles) {
            prefetch(t + 1);
            if (!quick(t, 0)) break;
            if (!quick(t, 1)) {
                kt = 1;
                break;
            }
            park(t + 1);
            ++t;
        }
    }

    // normalise and store: a lane holds, for its query, dims 32 dt + 8 (i / 4) + 4 half + (i % 4)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int p = q0 + nt * 32 + col;
        const float l_tot = sum_halves(l_sum[nt]);
        if (p >= n) continue;
        const float inv = 1.f / l_tot;
        const int64_t row = ((int64_t)b * a.n_q_heads + h) * n_q + (p - q_first);
        if (a.lse != nullptr && half == 0) a.lse[row] = (m_ref[nt] + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int gi = 0; gi < 4; ++gi) {
                const int d0 = 32 * dt + 8 * gi + 4 * half;
                const float o0 = acc[dt][nt][4 * gi + 0] * inv, o1 = acc[dt][nt][4 * gi + 1] * inv;
                const float o2 = acc[dt][nt][4 * gi + 2] * inv, o3 = acc[dt][nt][4 * gi + 3] * inv;
                if (a.out_f32) {
                    const float4 o = make_float4(o0, o1, o2, o3);
                    *reinterpret_cast<float4 *>(reinterpret_cast<float *>(a.out) + row * kHeadDim + d0) = o;
                } else {
                    const u32x2_t o = {pack_bf16(o0, o1), pack_bf16(o2, o3)};
                    *reinterpret_cast<u32x2_t *>(reinterpret_cast<uint16_t *>(a.out) + row * kHeadDim + d0) = o;
                }
            }
    }
}

}  // namespace

template <int G, int QB, int NT>
hipError_t launch_prefill(const PrefillArgs &a, hipStream_t stream)
{
    const int64_t block_queries = 32 * NT * QB;
    const int64_t total = (a.n_q + block_queries - 1) / block_queries * a.n_kv_heads * a.batch;
    const int64_t grid = (total + 7) / 8 * 8;
    hipLaunchKernelGGL((lt_prefill_attn_kernel<G, QB, NT>), dim3((unsigned)grid), dim3(64 * G * QB), 0, stream, a);
    return hipGetLastError();
}

// Up to twelve wavefronts per workgroup (three per SIMD, 168 registers each), so that one's matrix
// instructions overlap the others' exponentials; each takes 32 queries.
hipError_t prefill_attn(const PrefillArgs &args, hipStream_t stream)
{
    PrefillArgs a = args;
    a.kv_share = 1;
    // Eight heads per KV head would be eight wavefronts, two per SIMD; as two groups of four heads with three query
    // sub-blocks each they are twelve, and the two groups' workgroups read the same K/V tiles (from the L2, mostly).
    if (a.n_q_heads / a.n_kv_heads == 8) {
        a.kv_share = 2;
        a.n_kv_heads *= 2;
    }
    switch (a.n_q_heads / a.n_kv_heads) {
    case 1: return launch_prefill<1, 12, 1>(a, stream);
    case 2: return launch_prefill<2, 6, 1>(a, stream);
    case 3: return launch_prefill<3, 4, 1>(a, stream);
    case 4: return launch_prefill<4, 3, 1>(a, stream);
    case 5: return launch_prefill<5, 2, 1>(a, stream);
    case 6: return launch_prefill<6, 2, 1>(a, stream);
    case 7: return launch_prefill<7, 1, 1>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace ltk
