// Lazy-ratio scoring for gfx950 (Eq. 1): the last w prompt queries of every head against all
// prompt keys, as a dense bf16 contraction on the matrix cores with fp32 accumulation, reduced
// on the fly to two sums per query -- the softmax denominator over the causal set and the part
// of it that falls on the initial + recent keys.  No attention matrix and no V are touched.
//
// One workgroup = one (sequence, KV head, range of keys); wavefront i of the workgroup owns
// query head g*G + i, so the G heads that share the KV head read each key tile from LDS once.
// S^T = K Q^T is formed with v_mfma_f32_32x32x16_bf16: keys are the rows, queries the columns,
// so each lane keeps 16 key logits of ONE query per instruction and the running max / sums
// stay private to the lane until the final merge.
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

constexpr int kRowPad = 8;                                  // bf16 elements of padding per key row in LDS
constexpr int kRowElems = kHeadDim + kRowPad;               // 272-byte rows: 16-byte reads of 8 rows hit 8 bank groups

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct LaneState {
    float m, sum_causal, sum_kept;
};

// Uniform description of a 32-key sub-tile relative to the masks.
// s_waitcnt immediate for gfx9: vmcnt = 0 (bits 3:0 and 15:14), expcnt and lgkmcnt left at their maxima
constexpr int kWaitVmcnt0 = 0x0F70;

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

__device__ __forceinline__ void update_masked(const floatx16_t &c, LaneState &st, float scale_log2e, int j_base,
                                              int p, int n, int w_sink, int w_recent, int fixed_mode)
{
    // key row of accumulator register i in this lane: j_base + 8*(i/4) + (i%4)
    float tmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int j = j_base + 8 * (i >> 2) + (i & 3);
        if (j <= p) tmax = fmaxf(tmax, c[i]);
    }
    const float m_new = fmaxf(st.m, tmax * scale_log2e);
    if (m_new == -INFINITY) return;                           // nothing causal seen so far
    const float alpha = fast_exp2(st.m - m_new);
    float sum = 0.f, kept = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int j = j_base + 8 * (i >> 2) + (i & 3);
        const bool causal = j <= p;
        const bool recent = fixed_mode ? (j >= n - w_recent) : (j > p - w_recent);
        const float e = causal ? fast_exp2(fmaf(c[i], scale_log2e, -m_new)) : 0.f;
        sum += e;
        kept += (j < w_sink || recent) ? e : 0.f;
    }
    st.sum_causal = st.sum_causal * alpha + sum;
    st.sum_kept = st.sum_kept * alpha + kept;
    st.m = m_new;
}

// A 64-key tile is 1024 16-byte pieces (coalesced rows of 256 B) spread over the workgroup.
// fetch_tile() starts the global loads into registers, commit_tile() parks them in LDS; the MFMA
// work of the current tile runs between the two so the load latency is covered.
template <int G>
struct Staging {
    static constexpr int kThreads = 64 * G;
    static constexpr int kTotal = kScoreTileKeys * 16;
    static constexpr int kPieces = (kTotal + kThreads - 1) / kThreads;
};

template <int G>
__device__ __forceinline__ void fetch_tile(u32x4_t (&pre)[Staging<G>::kPieces], const uint16_t *kb, int64_t stride_t, int j0, int n)
{
#pragma unroll
    for (int i = 0; i < Staging<G>::kPieces; ++i) {
        int idx = threadIdx.x + i * Staging<G>::kThreads;
        idx = idx < Staging<G>::kTotal ? idx : Staging<G>::kTotal - 1;   // surplus threads re-read the last piece
        int j = j0 + (idx >> 4);
        j = j < n ? j : n - 1;                                          // clamp; such keys are masked as non-causal
        pre[i] = *reinterpret_cast<const u32x4_t *>(kb + (int64_t)j * stride_t + (idx & 15) * 8);
    }
}

template <int G>
__device__ __forceinline__ void commit_tile(const u32x4_t (&pre)[Staging<G>::kPieces], uint16_t *sh)
{
#pragma unroll
    for (int i = 0; i < Staging<G>::kPieces; ++i) {
        const int idx = threadIdx.x + i * Staging<G>::kThreads;
        if (idx < Staging<G>::kTotal) *reinterpret_cast<u32x4_t *>(&sh[(idx >> 4) * kRowElems + (idx & 15) * 8]) = pre[i];
    }
}

// G: query heads per KV head.  QH: wavefronts per head, each with its own 32 * NT queries (G * QH wavefronts
// per workgroup).  NT: 32-query column tiles per wavefront.  w <= 32: <G, 1, 1>; w <= 64: <G, 1, 2> for groups of
// up to four heads (more, lighter wavefronts per SIMD), <G, 2, 1> otherwise.
template <int G, int NT, int QH>
__global__ __launch_bounds__(64 * G * QH, 2) void lt_lazy_ratio_partial_kernel(ScoreArgs a)
{
    constexpr int W = G * QH;
    __shared__ __attribute__((aligned(16))) uint16_t sh_k[2][kScoreTileKeys * kRowElems];

    constexpr int kPieces = Staging<W>::kPieces;
    const int chunk = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: what depends on it stays in scalar registers
    const int col = lane & 31, half = lane >> 5;
    const int h = g * G + wave % G;
    const int q_off = (wave / G) * 32 * NT;                              // first query of this wavefront among the w_last

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
    const int n_tiles = (end_key - begin_key + kScoreTileKeys - 1) / kScoreTileKeys;
    const uint16_t *kb = a.k + (int64_t)b * a.k_stride_b + (int64_t)g * a.k_stride_h;

    // Q^T fragments (B operand): lane holds, for its query column, the 8 dims 16*s + 8*half .. +7
    bf16x8_t qf[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int t = q_off + nt * 32 + col;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            uint4 u = make_uint4(0u, 0u, 0u, 0u);
            if (t < a.w_last)
                u = *reinterpret_cast<const uint4 *>(a.q_last + (((int64_t)b * a.n_q_heads + h) * a.w_last + t) * kHeadDim +
                                                     16 * s + 8 * half);
            qf[nt][s] = __builtin_bit_cast(bf16x8_t, u);
        }
    }

    // The query fragments must have arrived on every path into the tile loop: otherwise the compiler, which
    // cannot tell how many newer loads may be outstanding, makes the first matrix instruction of EVERY tile wait
    // for all outstanding loads, the K prefetch issued just before it included.
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);

    LaneState st[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) { st[nt].m = -INFINITY; st[nt].sum_causal = 0.f; st[nt].sum_kept = 0.f; }

    // S^T for one 32-key sub-tile: 8 k-steps of 16 dims, NT column tiles of 32 queries.
    auto contract = [&](floatx16_t (&c)[NT], const uint16_t *tile, int kt) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) c[nt][i] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const u32x4_t u = *reinterpret_cast<const u32x4_t *>(&tile[(32 * kt + col) * kRowElems + 16 * s + 8 * half]);
            const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, u);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) c[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[nt][s], c[nt], 0, 0, 0);
        }
    };
    // Fold one sub-tile's logits into the running max and the two sums of every query column.
    auto fold = [&](const floatx16_t (&c)[NT], int j0) {
        const TileClass cls = classify(j0, n, a.w_last, w_sink, w_recent, a.fixed_mode);
        if (cls.fast) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) update_quick(c[nt], st[nt], a.scale_log2e, cls.kept);
        } else {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int p = n - a.w_last + q_off + nt * 32 + col;     // query position of this lane's column
                update_masked(c[nt], st[nt], a.scale_log2e, j0 + 4 * half, p, n, w_sink, w_recent, a.fixed_mode);
            }
        }
    };

    // Two wavefronts per SIMD (from two workgroups) overlap one's matrix-core work with the
    // other's exponentials.  The K tiles are prefetched two tiles ahead in two register sets, so
    // a global load has two tiles of compute (about 2.5 us) to arrive before it is parked in LDS.
    auto compute = [&](const uint16_t *tile, int j0) {
#pragma unroll
        for (int kt = 0; kt < kScoreTileKeys / 32; ++kt) {
            if (j0 + 32 * kt >= end_key) break;
            floatx16_t c[NT];
            contract(c, tile, kt);
            fold(c, j0 + 32 * kt);
        }
    };
    auto tile_key = [&](int tile) { return begin_key + tile * kScoreTileKeys; };

    u32x4_t pre_even[kPieces], pre_odd[kPieces];
    if (n_tiles > 0) {
        fetch_tile<W>(pre_even, kb, a.k_stride_t, tile_key(0), n);
        commit_tile<W>(pre_even, sh_k[0]);
    }
    __syncthreads();
    if (n_tiles > 1) fetch_tile<W>(pre_odd, kb, a.k_stride_t, tile_key(1), n);
    for (int tile = 0; tile < n_tiles; tile += 2) {
        if (tile + 2 < n_tiles) fetch_tile<W>(pre_even, kb, a.k_stride_t, tile_key(tile + 2), n);
        compute(sh_k[0], tile_key(tile));
        if (tile + 1 < n_tiles) {
            commit_tile<W>(pre_odd, sh_k[1]);
            __syncthreads();
            if (tile + 3 < n_tiles) fetch_tile<W>(pre_odd, kb, a.k_stride_t, tile_key(tile + 3), n);
            compute(sh_k[1], tile_key(tile + 1));
            if (tile + 2 < n_tiles) {
                commit_tile<W>(pre_even, sh_k[0]);
                __syncthreads();
            }
        }
    }

    // partial layout [B][Hq][chunk][half][field][w]: each store below is contiguous over the query columns
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int t = q_off + nt * 32 + col;
        if (t < a.w_last) {
            float *dst = a.part + ((((int64_t)b * a.n_q_heads + h) * a.n_chunks + chunk) * 2 + half) * 3 * a.w_last + t;
            dst[0] = st[nt].m;
            dst[a.w_last] = st[nt].sum_causal;
            dst[2 * a.w_last] = st[nt].sum_kept;
        }
    }
}

// rho per (sequence, head, query): one workgroup per (sequence, head), one thread per query,
// merging the chunk partials by their running maxima; the head's sum of rho goes to scratch.
// Fixed-order reductions: the result does not depend on scheduling.
__global__ __launch_bounds__(64) void lt_lazy_ratio_finish_kernel(ScoreArgs a)
{
    __shared__ float sh_sum[64];
    const int h = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
    const int n_part = 2 * a.n_chunks;
    float rho = 0.f;
    if (t < a.w_last) {
        const float *src = a.part + ((int64_t)b * a.n_q_heads + h) * n_part * 3 * a.w_last + t;
        float mx = -INFINITY, causal = 0.f, kept = 0.f;
        for (int c0 = 0; c0 < n_part; c0 += 8) {              // eight partials per round trip
            float m[8], f[8], k[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float *pc = src + (int64_t)min(c0 + u, n_part - 1) * 3 * a.w_last;
                m[u] = pc[0];
                f[u] = pc[a.w_last];
                k[u] = pc[2 * a.w_last];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (c0 + u < n_part && m[u] != -INFINITY) {
                    const float m_new = fmaxf(mx, m[u]);
                    const float keep = fast_exp2(mx - m_new), add = fast_exp2(m[u] - m_new);
                    causal = causal * keep + add * f[u];
                    kept = kept * keep + add * k[u];
                    mx = m_new;
                }
            }
        }
        if (a.lse_rows != nullptr) {
            // Table 1: the chunks covered only the initial and recent keys; the whole row's
            // denominator comes from the prefill attention's log-sum-exp
            const float lse = a.lse_rows[(int64_t)b * a.lse_stride_b + (int64_t)h * a.lse_stride_h + t];
            rho = mx == -INFINITY ? 0.f : kept * fast_exp2(mx - lse * 1.44269504088896340736f);
        } else {
            rho = kept / causal;
        }
        if (a.rho != nullptr) a.rho[((int64_t)b * a.n_q_heads + h) * a.w_last + t] = rho;
    }
    sh_sum[t] = rho;
    __syncthreads();
    for (int step = 32; step > 0; step >>= 1) {
        if (t < step) sh_sum[t] += sh_sum[t + step];
        __syncthreads();
    }
    if (t == 0) a.head_scratch[(int64_t)b * a.n_q_heads + h] = sh_sum[0];
}

// Per-sequence mean over heads and queries, then the batch mean (one workgroup, fixed order).
__global__ __launch_bounds__(64) void lt_lazy_ratio_mean_kernel(ScoreArgs a)
{
    __shared__ float sh_seq[64];
    float total = 0.f;
    for (int b0 = 0; b0 < a.batch; b0 += 64) {
        const int b = b0 + threadIdx.x;
        float r = 0.f;
        if (b < a.batch) {
            float sum = 0.f;
            for (int h = 0; h < a.n_q_heads; ++h) sum += a.head_scratch[(int64_t)b * a.n_q_heads + h];
            r = sum / (float)(a.n_q_heads * a.w_last);
            if (a.ratio_seq != nullptr) a.ratio_seq[b] = r;
        }
        sh_seq[threadIdx.x] = r;
        __syncthreads();
        if (threadIdx.x == 0)
            for (int i = 0; i < 64 && b0 + i < a.batch; ++i) total += sh_seq[i];
        __syncthreads();
    }
    if (threadIdx.x == 0) a.ratio_mean[0] = total / (float)a.batch;
}

}  // namespace

template <int G>
hipError_t launch_partial(const ScoreArgs &a, hipStream_t stream)
{
    const dim3 grid(a.n_chunks, a.n_kv_heads, a.batch);
    if (a.w_last <= 32)
        hipLaunchKernelGGL((lt_lazy_ratio_partial_kernel<G, 1, 1>), grid, dim3(64 * G), 0, stream, a);
    else if constexpr (G <= 4)                       // measured 3 % faster than one wavefront of 64 queries per head
        hipLaunchKernelGGL((lt_lazy_ratio_partial_kernel<G, 1, 2>), grid, dim3(128 * G), 0, stream, a);
    else
        hipLaunchKernelGGL((lt_lazy_ratio_partial_kernel<G, 2, 1>), grid, dim3(64 * G), 0, stream, a);
    return hipGetLastError();
}

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
    hipError_t e;
    switch (a.n_q_heads / a.n_kv_heads) {
    case 1: e = launch_partial<1>(a, stream); break;
    case 2: e = launch_partial<2>(a, stream); break;
    case 3: e = launch_partial<3>(a, stream); break;
    case 4: e = launch_partial<4>(a, stream); break;
    case 5: e = launch_partial<5>(a, stream); break;
    case 6: e = launch_partial<6>(a, stream); break;
    case 7: e = launch_partial<7>(a, stream); break;
    case 8: e = launch_partial<8>(a, stream); break;
    default: e = hipErrorInvalidValue; break;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lt_lazy_ratio_finish_kernel, dim3(a.n_q_heads, a.batch), dim3(64), 0, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lt_lazy_ratio_mean_kernel, dim3(1), dim3(64), 0, stream, a);
    return hipGetLastError();
}

}  // namespace ltk
