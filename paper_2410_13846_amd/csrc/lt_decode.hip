// Decode-side kernels for gfx950: KV append (growing cache / sink+recent ring), split decode
// attention over the key axis, and the log-sum-exp merge of the splits.
//
// Attention of one query over a set of keys does not depend on the order of the keys, so a
// lazy layer's ring is read as a plain array of `stored` entries and both layer kinds share
// one kernel.  One workgroup streams a contiguous range of keys of one (sequence, KV head)
// once from HBM and applies it to all G query heads of that KV head.
#include "lt_kernels.h"

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

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Sum over the 16 lanes of a DPP row; every lane of the row receives the total.
__device__ __forceinline__ float row16_allsum(float x)
{
    x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);  // row_half_mirror
    x += dpp_move<0x140>(x);  // row_mirror
    return x;
}

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;   // 16 bytes as one register quad

__device__ __forceinline__ u32x4_t load16(const uint16_t *p) { return *reinterpret_cast<const u32x4_t *>(p); }

// K and V are read exactly once per decode step: stream them past the caches.
__device__ __forceinline__ u32x4_t load16_stream(const uint16_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
}

// ---------------------------------------------------------------------------------------------
// append: one thread moves 16 bytes of K and 16 bytes of V.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lt_append_kv_kernel(AppendArgs a)
{
    const int64_t per_stream = a.n_new * 16;                       // uint4 units per (b, g)
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_stream) return;
    const int g = blockIdx.y, b = blockIdx.z;
    const int64_t j = idx >> 4;
    const int c = (int)(idx & 15);
    const int64_t p = a.total_before + j;                          // absolute position of the token
    int64_t slot = p;
    if (a.is_lazy) {
        if (p >= a.w_sink) {
            const int64_t total_after = a.total_before + a.n_new;
            if (a.w_recent == 0 || p < total_after - a.w_recent) return;   // a later token of this call owns the slot
            slot = a.w_sink + (p - a.w_sink) % a.w_recent;
        }
    }
    const int64_t src = (((int64_t)b * a.n_kv_heads + g) * a.n_new + j) * kHeadDim + c * 8;
    const int64_t dst = (int64_t)b * a.stride_b + (int64_t)g * a.stride_h + slot * kHeadDim + c * 8;
    *reinterpret_cast<u32x4_t *>(a.k_cache + dst) = load16(a.k_new + src);
    *reinterpret_cast<u32x4_t *>(a.v_cache + dst) = load16(a.v_new + src);
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

__device__ __forceinline__ void load_tile(Tile &t, const uint16_t *kb, const uint16_t *vb, int key0, int sub, int chunk,
                                          int last_key)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int key = key0 + 4 * i + sub;
        key = key < last_key ? key : last_key;                      // clamp: masked later
        const int64_t off = (int64_t)key * kHeadDim + chunk * 8;
        t.k[i] = load16_stream(kb + off);
        t.v[i] = load16_stream(vb + off);
    }
}

template <int G>
struct RowState {
    float m[G];
    float l[G];
    float acc[G][8];
};

template <int G>
__device__ __forceinline__ void process_tile(const Tile &t, const uint32_t (&qf)[G][4], RowState<G> &st, int key0, int sub,
                                             int end_key, float scale_log2e)
{
    float s[4][G];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool valid = key0 + 4 * i + sub < end_key;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float x = dot2_bf16(t.k[i][0], qf[h][0], 0.f);
            x = dot2_bf16(t.k[i][1], qf[h][1], x);
            x = dot2_bf16(t.k[i][2], qf[h][2], x);
            x = dot2_bf16(t.k[i][3], qf[h][3], x);
            x = row16_allsum(x) * scale_log2e;
            s[i][h] = valid ? x : -INFINITY;
        }
    }
    bool grow = false;
    float tmax[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        tmax[h] = fmaxf(fmaxf(s[0][h], s[1][h]), fmaxf(s[2][h], s[3][h]));
        grow |= tmax[h] > st.m[h];
    }
    if (__any(grow)) {                                              // rare after the first tiles
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float m_new = fmaxf(st.m[h], tmax[h]);
            const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(st.m[h] - m_new);
            st.m[h] = m_new;
            st.l[h] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) st.acc[h][e] *= alpha;
        }
    }
    float p[4][G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float m_safe = (st.m[h] == -INFINITY) ? 0.f : st.m[h];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p[i][h] = fast_exp2(s[i][h] - m_safe);
            st.l[h] += p[i][h];
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float vf[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) { vf[2 * e] = bf16_lo(t.v[i][e]); vf[2 * e + 1] = bf16_hi(t.v[i][e]); }
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) st.acc[h][e] = fmaf(p[i][h], vf[e], st.acc[h][e]);
    }
}

template <int G, int LAZY_TAG>
__global__ __launch_bounds__(kDecodeThreads) void lt_decode_partial_kernel(DecodeArgs a)
{
    constexpr int kWaves = kDecodeThreads / 64;
    __shared__ float sh_m[kWaves][G];
    __shared__ float sh_l[kWaves][G];
    __shared__ float sh_acc[kWaves][G][kHeadDim];

    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane >> 4, chunk = lane & 15;

    const int begin_key = split * a.keys_per_block;
    const int end_key = min(a.stored, begin_key + a.keys_per_block);
    const int n_tiles = (end_key - begin_key + 15) >> 4;
    const uint16_t *kb = a.k_cache + (int64_t)b * a.stride_b + (int64_t)g * a.stride_h;
    const uint16_t *vb = a.v_cache + (int64_t)b * a.stride_b + (int64_t)g * a.stride_h;

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

    // Wavefront w takes tiles w, w+4, ...; two tile buffers alternate so the loads of the next
    // tile are in flight while the current one is consumed.
    Tile t0, t1;
    int t = wave;
    if (t < n_tiles) load_tile(t0, kb, vb, begin_key + 16 * t, sub, chunk, end_key - 1);
    while (t < n_tiles) {
        if (t + kWaves < n_tiles) load_tile(t1, kb, vb, begin_key + 16 * (t + kWaves), sub, chunk, end_key - 1);
        process_tile<G>(t0, qf, st, begin_key + 16 * t, sub, end_key, a.scale_log2e);
        t += kWaves;
        if (t >= n_tiles) break;
        if (t + kWaves < n_tiles) load_tile(t0, kb, vb, begin_key + 16 * (t + kWaves), sub, chunk, end_key - 1);
        process_tile<G>(t1, qf, st, begin_key + 16 * t, sub, end_key, a.scale_log2e);
        t += kWaves;
    }

    // Merge the four rows of the wavefront.
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float mx = fmaxf(st.m[h], __shfl_xor(st.m[h], 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float wgt = (st.m[h] == -INFINITY) ? 0.f : fast_exp2(st.m[h] - mx);
        float l = st.l[h] * wgt;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = st.acc[h][e] * wgt;
            x += __shfl_xor(x, 16);
            x += __shfl_xor(x, 32);
            st.acc[h][e] = x;
        }
        st.m[h] = mx;
        st.l[h] = l;
    }
    if (sub == 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            if (chunk == 0) { sh_m[wave][h] = st.m[h]; sh_l[wave][h] = st.l[h]; }
#pragma unroll
            for (int e = 0; e < 8; ++e) sh_acc[wave][h][chunk * 8 + e] = st.acc[h][e];
        }
    }
    __syncthreads();

    // Merge the wavefronts and store this split's partial result.
    for (int idx = threadIdx.x; idx < G * kHeadDim; idx += kDecodeThreads) {
        const int h = idx / kHeadDim, dim = idx % kHeadDim;
        float mx = sh_m[0][h];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, sh_m[w][h]);
        float l = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float wgt = (sh_m[w][h] == -INFINITY) ? 0.f : fast_exp2(sh_m[w][h] - mx);
            l += wgt * sh_l[w][h];
            o += wgt * sh_acc[w][h][dim];
        }
        const int64_t row = ((int64_t)b * a.n_q_heads + g * G + h) * a.n_splits + split;
        a.part_acc[row * kHeadDim + dim] = o;
        if (dim == 0) { a.part_ml[row * 2] = mx; a.part_ml[row * 2 + 1] = l; }
    }
}

// ---------------------------------------------------------------------------------------------
// merge of the splits: softmax over a union of disjoint key sets is the weighted sum of the
// per-set results with weights exp(max_c - max) * l_c.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kHeadDim) void lt_decode_merge_kernel(DecodeArgs a)
{
    const int h = blockIdx.x, b = blockIdx.y, dim = threadIdx.x;
    const int64_t row0 = ((int64_t)b * a.n_q_heads + h) * a.n_splits;
    const float *ml = a.part_ml + row0 * 2;
    const float *acc = a.part_acc + row0 * kHeadDim;
    float mx = -INFINITY;
    for (int c = 0; c < a.n_splits; ++c) mx = fmaxf(mx, ml[2 * c]);
    float l = 0.f, o = 0.f;
    for (int c = 0; c < a.n_splits; ++c) {
        const float wgt = fast_exp2(ml[2 * c] - mx);
        l += wgt * ml[2 * c + 1];
        o += wgt * acc[(int64_t)c * kHeadDim + dim];
    }
    a.out[((int64_t)b * a.n_q_heads + h) * kHeadDim + dim] = o / l;
    if (a.lse != nullptr && dim == 0)
        a.lse[(int64_t)b * a.n_q_heads + h] = (mx + log2f(l)) * 0.69314718055994530942f;
}

template <int G>
hipError_t launch_partial(const DecodeArgs &a, hipStream_t stream)
{
    const dim3 grid(a.n_splits, a.n_kv_heads, a.batch);
    if (a.lazy_tag)
        hipLaunchKernelGGL((lt_decode_partial_kernel<G, 1>), grid, dim3(kDecodeThreads), 0, stream, a);
    else
        hipLaunchKernelGGL((lt_decode_partial_kernel<G, 0>), grid, dim3(kDecodeThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t append(const AppendArgs &a, hipStream_t stream)
{
    const int64_t per_stream = a.n_new * 16;
    const dim3 grid((unsigned)((per_stream + 255) / 256), a.n_kv_heads, a.batch);
    hipLaunchKernelGGL(lt_append_kv_kernel, grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t decode_partial(const DecodeArgs &a, hipStream_t stream)
{
    switch (a.n_q_heads / a.n_kv_heads) {
    case 1: return launch_partial<1>(a, stream);
    case 2: return launch_partial<2>(a, stream);
    case 3: return launch_partial<3>(a, stream);
    case 4: return launch_partial<4>(a, stream);
    case 5: return launch_partial<5>(a, stream);
    case 6: return launch_partial<6>(a, stream);
    case 7: return launch_partial<7>(a, stream);
    case 8: return launch_partial<8>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t decode_merge(const DecodeArgs &a, hipStream_t stream)
{
    hipLaunchKernelGGL(lt_decode_merge_kernel, dim3(a.n_q_heads, a.batch), dim3(kHeadDim), 0, stream, a);
    return hipGetLastError();
}

}  // namespace ltk
