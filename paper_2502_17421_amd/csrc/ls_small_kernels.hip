// The small kernels of the path: tree-mask builder, masked tree attention, log-sum-exp
// merge, and the fused tree attention + merge that closes the whole call.  (LongSpec, Section 3.3; the aggregation appendix.)
#include "ls_internal.hpp"

namespace ls {

// --------------------------------------------------------------------------- (a) ----
// Tree mask: one workgroup per sequence; a thread walks the parent chain of its node and sets
// one bit per node met, itself included.  err_flag[b] is written 0 or 1 on every launch.
__global__ void __launch_bounds__(256)
tree_mask_kernel(const int32_t *__restrict__ parents, int32_t n_tree, uint64_t *__restrict__ mask,
                 int32_t *__restrict__ err_flag)
{
    const int b = blockIdx.x;
    const int words = (n_tree + 63) >> 6;
    build_tree_mask_rows(parents + (size_t)b * n_tree, n_tree, mask + (size_t)b * n_tree * words,
                         err_flag ? err_flag + b : nullptr, threadIdx.x, blockDim.x);
}

hipError_t launch_tree_mask(const int32_t *parents, int32_t batch, int32_t n_tree, uint64_t *mask,
                            int32_t *err_flag, hipStream_t stream)
{
    const int threads = n_tree <= 64 ? 64 : (n_tree <= 128 ? 128 : 256);
    hipLaunchKernelGGL(tree_mask_kernel, dim3(batch), dim3(threads), 0, stream, parents, n_tree, mask, err_flag);
    return hipGetLastError();
}

// --------------------------------------------------------------------------- (c) ----
// Masked tree attention: one wavefront per query row (b, h, i).  The head dimension is
// spread over the 64 lanes; the visible keys are the set bits of the row's mask, walked
// in increasing order.  Each logit is a wavefront-wide sum of per-lane products; the
// softmax state (running max, running sum) is wave-uniform.
template <typename T, int D>
__global__ void __launch_bounds__(256)
tree_attn_kernel(Problem p, const uint64_t *__restrict__ mask, Partials out)
{
    constexpr int EPL = D / kWave;  // elements per lane
    const int lane = threadIdx.x & (kWave - 1);
    const int row = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    const int rows_total = p.batch * p.n_q_heads * p.n_tree;
    if (row >= rows_total) return;
    const int i = row % p.n_tree;
    const int h = (row / p.n_tree) % p.n_q_heads;
    const int b = row / (p.n_tree * p.n_q_heads);
    const int g = h / p.group;
    const int words = (p.n_tree + 63) >> 6;

    const T *qrow = (const T *)p.q + b * p.q_stride[0] + h * p.q_stride[1] + i * p.q_stride[2];
    const T *kbase = (const T *)p.k_tree + b * p.kt_stride[0] + g * p.kt_stride[1];
    const T *vbase = (const T *)p.v_tree + b * p.vt_stride[0] + g * p.vt_stride[1];
    const uint64_t *mrow = mask + ((size_t)b * p.n_tree + i) * words;

    float qv[EPL], acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        qv[e] = Elem<T>::load(qrow + lane * EPL + e) * p.scale_log2;
        acc[e] = 0.f;
    }
    float m_run = -INFINITY, l_run = 0.f;
    for (int w = 0; w < words; ++w) {
        uint64_t bits = mrow[w];
        if (w == words - 1 && (p.n_tree & 63)) bits &= ((uint64_t)1 << (p.n_tree & 63)) - 1;
        while (bits) {
            const int j = (w << 6) + __builtin_ctzll(bits);
            bits &= bits - 1;
            const T *krow = kbase + j * p.kt_stride[2];
            const T *vrow = vbase + j * p.vt_stride[2];
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) part += qv[e] * Elem<T>::load(krow + lane * EPL + e);
            const float z = wave_sum(part);  // base-2 logit, identical in every lane
            const float m_new = fmaxf(m_run, z);
            const float alpha = exp2f(m_run - m_new);  // 0 on the first key
            const float pj = exp2f(z - m_new);
            l_run = l_run * alpha + pj;
#pragma unroll
            for (int e = 0; e < EPL; ++e)
                acc[e] = acc[e] * alpha + pj * Elem<T>::load(vrow + lane * EPL + e);
            m_run = m_new;
        }
    }
    const size_t prow = out.row((size_t)b * p.n_q_heads + h, 0, p.n_tree, i);
    float *orow = (float *)out.o + prow * D;
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) orow[lane * EPL + e] = acc[e] * inv;
    if (lane == 0) out.lse[prow] = l_run > 0.f ? (m_run + log2f(l_run)) * kLn2 : -INFINITY;
}

hipError_t launch_tree_attn(const Problem &p, int dtype, const uint64_t *mask, const Partials &out,
                            hipStream_t stream)
{
    const int rows = p.batch * p.n_q_heads * p.n_tree;
    const dim3 block(256), grid((rows + 3) / 4);
#define LS_TREE_CASE(T, DD) \
    hipLaunchKernelGGL((tree_attn_kernel<T, DD>), grid, block, 0, stream, p, mask, out)
    if (dtype == LS_BF16 && p.head_dim == 128) LS_TREE_CASE(uint16_t, 128);
    else if (dtype == LS_BF16 && p.head_dim == 64) LS_TREE_CASE(uint16_t, 64);
    else if (dtype == LS_F16 && p.head_dim == 128) LS_TREE_CASE(half_t, 128);
    else if (dtype == LS_F16 && p.head_dim == 64) LS_TREE_CASE(half_t, 64);
    else if (dtype == LS_F32 && p.head_dim == 128) LS_TREE_CASE(float, 128);
    else if (dtype == LS_F32 && p.head_dim == 64) LS_TREE_CASE(float, 64);
    else return hipErrorInvalidValue;
#undef LS_TREE_CASE
    return hipGetLastError();
}

// --------------------------------------------------------------------------- (d) ----
// Merge: one thread per (query row, 4 consecutive head-dim elements).  First pass finds
// the largest part LSE, second pass accumulates exp(LSE_k - max) weighted outputs and the
// weight sum; the result is out = sum_k w_k O_k / sum_k w_k, lse = max + log(sum_k w_k),
// which is the two-term aggregation rule of Section 3.3 applied to all parts at once.
__device__ __forceinline__ float4 load4(const float *p) { return *(const float4 *)p; }
__device__ __forceinline__ float4 load4(const uint16_t *p)
{
    const uint2 v = *(const uint2 *)p;
    return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                       __uint_as_float(v.y & 0xffff0000u));
}

__device__ __forceinline__ float4 load4(const half_t *p)
{
    const uint2 v = *(const uint2 *)p;
    return make_float4(half_to_float((uint16_t)v.x), half_to_float((uint16_t)(v.x >> 16)),
                       half_to_float((uint16_t)v.y), half_to_float((uint16_t)(v.y >> 16)));
}

template <typename T, typename PT, int D>
__global__ void __launch_bounds__(256)
merge_kernel(int32_t rows_total, int32_t n_q_heads, int32_t n_tree, int32_t n_parts,
             const PT *__restrict__ o_parts, const float *__restrict__ lse_parts, T *__restrict__ out,
             int64_t os0, int64_t os1, int64_t os2, float *__restrict__ lse)
{
    constexpr int TPR = D / 4;  // threads per row
    const int tid = blockIdx.x * blockDim.x + threadIdx.x;
    const int row = tid / TPR;
    const int c = (tid % TPR) * 4;
    if (row >= rows_total) return;
    const int i = row % n_tree;
    const int h = (row / n_tree) % n_q_heads;
    const int b = row / (n_tree * n_q_heads);
    const size_t bh = (size_t)b * n_q_heads + h;
    const float *lp = lse_parts + bh * n_parts * n_tree + i;

    float top = -INFINITY;
    for (int k = 0; k < n_parts; ++k) top = fmaxf(top, lp[(size_t)k * n_tree]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float wsum = 0.f;
    if (top > -INFINITY) {
        for (int k = 0; k < n_parts; ++k) {
            const float l = lp[(size_t)k * n_tree];
            if (l == -INFINITY) continue;
            const float w = exp2f((l - top) * kLog2e);
            const float4 o = load4(o_parts + ((bh * n_parts + k) * n_tree + i) * D + c);
            acc.x += w * o.x;
            acc.y += w * o.y;
            acc.z += w * o.z;
            acc.w += w * o.w;
            wsum += w;
        }
    }
    const float inv = wsum > 0.f ? 1.f / wsum : 0.f;
    T *orow = out + b * os0 + h * os1 + i * os2 + c;
    Elem<T>::store(orow + 0, acc.x * inv);
    Elem<T>::store(orow + 1, acc.y * inv);
    Elem<T>::store(orow + 2, acc.z * inv);
    Elem<T>::store(orow + 3, acc.w * inv);
    if (c == 0) lse[row] = wsum > 0.f ? top + log2f(wsum) * kLn2 : -INFINITY;
}

hipError_t launch_merge(int32_t batch, int32_t n_q_heads, int32_t n_tree, int32_t head_dim, int dtype,
                        int32_t n_parts, const void *o_parts, int parts_are_16bit, const float *lse_parts, void *out,
                        const int64_t o_stride[3], float *lse, hipStream_t stream)
{
    const int rows = batch * n_q_heads * n_tree;
    const int threads = rows * (head_dim / 4);
    const dim3 block(256), grid((threads + 255) / 256);
#define LS_MERGE_CASE(T, PT, DD)                                                                              \
    hipLaunchKernelGGL((merge_kernel<T, PT, DD>), grid, block, 0, stream, rows, n_q_heads, n_tree, n_parts,     \
                       (const PT *)o_parts, lse_parts, (T *)out, o_stride[0], o_stride[1], o_stride[2], lse)
    if (head_dim != 64 && head_dim != 128) return hipErrorInvalidValue;
    // parts are float, or 16-bit parts of a 16-bit problem in the problem's own type
    if (dtype == LS_F32) {
        if (parts_are_16bit) return hipErrorInvalidValue;
        if (head_dim == 128) LS_MERGE_CASE(float, float, 128);
        else LS_MERGE_CASE(float, float, 64);
    } else if (dtype == LS_BF16) {
        if (parts_are_16bit) {
            if (head_dim == 128) LS_MERGE_CASE(uint16_t, uint16_t, 128);
            else LS_MERGE_CASE(uint16_t, uint16_t, 64);
        } else {
            if (head_dim == 128) LS_MERGE_CASE(uint16_t, float, 128);
            else LS_MERGE_CASE(uint16_t, float, 64);
        }
    } else if (dtype == LS_F16) {
        if (parts_are_16bit) {
            if (head_dim == 128) LS_MERGE_CASE(half_t, half_t, 128);
            else LS_MERGE_CASE(half_t, half_t, 64);
        } else {
            if (head_dim == 128) LS_MERGE_CASE(half_t, float, 128);
            else LS_MERGE_CASE(half_t, float, 64);
        }
    } else {
        return hipErrorInvalidValue;
    }
#undef LS_MERGE_CASE
    return hipGetLastError();
}

// --------------------------------------------------------------------- (c) + (d) fused ----
// The tail of the whole path: one wavefront per query row computes the masked tree attention
// of that row (as tree_attn_kernel does, keeping the result in registers) and merges it with
// the row's cached-key partials by the aggregation rule of Section 3.3.  The head dimension
// is spread over the 64 lanes; logits and part weights are wavefront reductions.
template <int EPL> struct Piece;
template <> struct Piece<1> {
    static __device__ __forceinline__ void load(const float *p, float *v) { v[0] = p[0]; }
    static __device__ __forceinline__ void load(const uint16_t *p, float *v) { v[0] = bf16_to_float(p[0]); }
    static __device__ __forceinline__ void store(float *p, const float *v) { p[0] = v[0]; }
    static __device__ __forceinline__ void store(uint16_t *p, const float *v) { p[0] = float_to_bf16(v[0]); }
    static __device__ __forceinline__ void load(const half_t *p, float *v) { v[0] = half_to_float(p[0].bits); }
    static __device__ __forceinline__ void store(half_t *p, const float *v) { p[0].bits = float_to_half(v[0]); }
};
template <> struct Piece<2> {
    static __device__ __forceinline__ void load(const float *p, float *v)
    {
        const float2 t = *(const float2 *)p;
        v[0] = t.x;
        v[1] = t.y;
    }
    static __device__ __forceinline__ void load(const uint16_t *p, float *v)
    {
        const uint32_t t = *(const uint32_t *)p;
        v[0] = __uint_as_float(t << 16);
        v[1] = __uint_as_float(t & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(float *p, const float *v) { *(float2 *)p = make_float2(v[0], v[1]); }
    static __device__ __forceinline__ void store(uint16_t *p, const float *v)
    {
        *(uint32_t *)p = (uint32_t)float_to_bf16(v[0]) | ((uint32_t)float_to_bf16(v[1]) << 16);
    }
    static __device__ __forceinline__ void load(const half_t *p, float *v)
    {
        const uint32_t t = *(const uint32_t *)p;
        v[0] = half_to_float((uint16_t)t);
        v[1] = half_to_float((uint16_t)(t >> 16));
    }
    static __device__ __forceinline__ void store(half_t *p, const float *v)
    {
        *(uint32_t *)p = (uint32_t)float_to_half(v[0]) | ((uint32_t)float_to_half(v[1]) << 16);
    }
};

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// Raw (unconverted) pieces, so that many loads can be in flight before the first is used.
template <typename PT, int EPL> struct Raw;
template <> struct Raw<float, 1> {
    typedef float type;
    static __device__ __forceinline__ type load(const float *p) { return *p; }
    static __device__ __forceinline__ void unpack(type r, float *v) { v[0] = r; }
};
template <> struct Raw<float, 2> {
    typedef float2 type;
    static __device__ __forceinline__ type load(const float *p) { return *(const float2 *)p; }
    static __device__ __forceinline__ void unpack(type r, float *v)
    {
        v[0] = r.x;
        v[1] = r.y;
    }
};
template <> struct Raw<uint16_t, 1> {
    typedef uint16_t type;
    static __device__ __forceinline__ type load(const uint16_t *p) { return *p; }
    static __device__ __forceinline__ void unpack(type r, float *v) { v[0] = bf16_to_float(r); }
};
template <> struct Raw<uint16_t, 2> {
    typedef uint32_t type;
    static __device__ __forceinline__ type load(const uint16_t *p) { return *(const uint32_t *)p; }
    static __device__ __forceinline__ void unpack(type r, float *v)
    {
        v[0] = __uint_as_float(r << 16);
        v[1] = __uint_as_float(r & 0xffff0000u);
    }
};

template <> struct Raw<half_t, 1> {
    typedef uint16_t type;
    static __device__ __forceinline__ type load(const half_t *p) { return p->bits; }
    static __device__ __forceinline__ void unpack(type r, float *v) { v[0] = half_to_float(r); }
};
template <> struct Raw<half_t, 2> {
    typedef uint32_t type;
    static __device__ __forceinline__ type load(const half_t *p) { return *(const uint32_t *)p; }
    static __device__ __forceinline__ void unpack(type r, float *v)
    {
        v[0] = half_to_float((uint16_t)r);
        v[1] = half_to_float((uint16_t)(r >> 16));
    }
};

template <typename T, typename PT, int D, int CHUNK>
__global__ void __launch_bounds__(256)
tree_merge_kernel(Problem p, const uint64_t *__restrict__ mask, Partials parts, int32_t n_cache, T *__restrict__ out,
                  int64_t os0, int64_t os1, int64_t os2, float *__restrict__ lse)
{
    constexpr int EPL = D / kWave;
    // CHUNK: split rows requested before any is used
    constexpr int KB = 8;  // tree keys requested together
    typedef Raw<PT, EPL> RP;
    typedef Raw<T, EPL> RT;
    const int lane = threadIdx.x & (kWave - 1);
    const int row = blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
    const int rows_total = p.batch * p.n_q_heads * p.n_tree;
    if (row >= rows_total) return;
    const int i = row % p.n_tree;
    const int h = (row / p.n_tree) % p.n_q_heads;
    const int b = row / (p.n_tree * p.n_q_heads);
    const int g = h / p.group;
    const int words = (p.n_tree + 63) >> 6;

    const size_t prow0 = parts.row((size_t)b * p.n_q_heads + h, 0, p.n_tree, i);
    const float *lp = parts.lse + prow0;
    const PT *op = (const PT *)parts.o + prow0 * D + lane * EPL;
    const size_t lse_step = parts.row_major ? 1 : (size_t)p.n_tree;  // between consecutive parts of one row
    const size_t part_step = lse_step * D;

    // Order of requests (loads return in the order they were issued): the query row and the
    // mask word first, a short round trip; then the row's first visible tree keys; then the
    // cached-key partials, by far the most bytes.  The partials are merged among themselves as
    // they arrive, then the tree keys (long there by then) are worked through, and a two-term
    // merge of the two results ends the row.
    const T *qrow = (const T *)p.q + b * p.q_stride[0] + h * p.q_stride[1] + i * p.q_stride[2];
    const T *kbase = (const T *)p.k_tree + b * p.kt_stride[0] + g * p.kt_stride[1] + lane * EPL;
    const T *vbase = (const T *)p.v_tree + b * p.vt_stride[0] + g * p.vt_stride[1] + lane * EPL;
    const uint64_t *mrow = mask + ((size_t)b * p.n_tree + i) * words;
    float qv[EPL], acc[EPL];
    RT::unpack(RT::load(qrow + lane * EPL), qv);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        qv[e] *= p.scale_log2;
        acc[e] = 0.f;
    }
    auto mask_word = [&](int w) {
        uint64_t bits = mrow[w];
        if (w == words - 1 && (p.n_tree & 63)) bits &= ((uint64_t)1 << (p.n_tree & 63)) - 1;
        return bits;
    };
    // up to KB visible keys at a time, all their rows requested before the first is used
    int idx[KB];
    typename RT::type kr[KB], vr[KB];
    auto request_keys = [&](uint64_t &bits, int w) {
#pragma unroll
        for (int u = 0; u < KB; ++u) {
            idx[u] = bits ? (w << 6) + __builtin_ctzll(bits) : -1;
            bits &= bits - 1;  // 0 stays 0
            const int j = idx[u] < 0 ? 0 : idx[u];
            kr[u] = RT::load(kbase + j * p.kt_stride[2]);
            vr[u] = RT::load(vbase + j * p.vt_stride[2]);
        }
    };
    float m_run = -INFINITY, l_run = 0.f;
    auto use_keys = [&]() {
#pragma unroll
        for (int u = 0; u < KB; ++u) {
            if (idx[u] < 0) break;  // wave-uniform
            float kv[EPL], vv[EPL];
            RT::unpack(kr[u], kv);
            RT::unpack(vr[u], vv);
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) part += qv[e] * kv[e];
            const float z = wave_sum(part);
            const float m_new = fmaxf(m_run, z);
            const float alpha = exp2f(m_run - m_new);
            const float pj = exp2f(z - m_new);
            l_run = l_run * alpha + pj;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = acc[e] * alpha + pj * vv[e];
            m_run = m_new;
        }
    };
    uint64_t bits0 = 0;
    if (mask != nullptr) {  // no mask: no tree part, merge of the cached-key partials only
        bits0 = mask_word(0);
        request_keys(bits0, 0);
    }
    // the first 64 part LSEs (one per lane) and the first CHUNK split rows
    const float l_first = lane < n_cache ? lp[(size_t)lane * lse_step] : -INFINITY;
    typename RP::type raw[CHUNK];
#pragma unroll
    for (int k = 0; k < CHUNK; ++k) {
        const int part = k < n_cache ? k : (n_cache > 0 ? n_cache - 1 : 0);  // clamped: always a valid row
        if (n_cache > 0) raw[k] = RP::load(op + (size_t)part * part_step);
    }

    // ---- merge of the cached-key partials among themselves -----------------------------------
    float top_c = wave_max(l_first);
    for (int s0 = kWave; s0 < n_cache; s0 += kWave) {
        const int s = s0 + lane;
        const float l = s < n_cache ? lp[(size_t)s * lse_step] : -INFINITY;
        top_c = fmaxf(top_c, wave_max(l));
    }
    float o[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = 0.f;
    float w_lane = 0.f;  // this lane's part weights, summed over the 64-part groups
    if (top_c != -INFINITY) {
        for (int s0 = 0; s0 < n_cache; s0 += kWave) {
            const int s = s0 + lane;
            const float l = s0 == 0 ? l_first : (s < n_cache ? lp[(size_t)s * lse_step] : -INFINITY);
            const float w = l == -INFINITY ? 0.f : exp2f((l - top_c) * kLog2e);
            w_lane += w;
            const int cnt = n_cache - s0 < kWave ? n_cache - s0 : kWave;
            for (int c0 = 0; c0 < cnt; c0 += CHUNK) {
                if (s0 + c0 > 0) {
#pragma unroll
                    for (int k = 0; k < CHUNK; ++k) {
                        const int part = s0 + c0 + k < n_cache ? s0 + c0 + k : n_cache - 1;
                        raw[k] = RP::load(op + (size_t)part * part_step);
                    }
                }
#pragma unroll
                for (int k = 0; k < CHUNK; ++k) {
                    // past the last part the lane weight is 0 (the clamped row was still a valid read);
                    // empty parts may hold anything, so they are selected out rather than multiplied
                    const float wk =
                        __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w), c0 + k));
                    float v[EPL];
                    RP::unpack(raw[k], v);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) o[e] += wk > 0.f ? wk * v[e] : 0.f;
                }
            }
        }
    }
    const float wsum_c = wave_sum(w_lane);  // 0 if no cached key is visible

    // ---- masked attention over the tree keys (unnormalised, base-2 logits) ----------------
    if (mask != nullptr) {
        use_keys();
        for (int w = 0; w < words; ++w) {
            uint64_t bits = w == 0 ? bits0 : mask_word(w);
            while (bits) {
                request_keys(bits, w);
                use_keys();
            }
        }
    }

    // ---- the two results, merged by the aggregation rule ----------------------------------------
    T *orow = out + b * os0 + h * os1 + i * os2 + lane * EPL;
    const float lse_c = wsum_c > 0.f ? top_c + log2f(wsum_c) * kLn2 : -INFINITY;
    const float lse_t = l_run > 0.f ? (m_run + log2f(l_run)) * kLn2 : -INFINITY;
    const float top = fmaxf(lse_c, lse_t);
    if (top == -INFINITY) {  // no visible key at all
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] = 0.f;
        Piece<EPL>::store(orow, o);
        if (lane == 0) lse[row] = -INFINITY;
        return;
    }
    const float wa = wsum_c > 0.f ? exp2f((lse_c - top) * kLog2e) : 0.f;
    const float wb = l_run > 0.f ? exp2f((lse_t - top) * kLog2e) : 0.f;
    const float inv = 1.f / (wa + wb);
    const float sa = wsum_c > 0.f ? wa * inv / wsum_c : 0.f;
    const float sb = l_run > 0.f ? wb * inv / l_run : 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = o[e] * sa + acc[e] * sb;
    Piece<EPL>::store(orow, o);
    if (lane == 0) lse[row] = top + log2f(wa + wb) * kLn2;
}

hipError_t launch_tree_merge(const Problem &p, int dtype, const uint64_t *mask, const Partials &cache_parts,
                             int32_t n_cache_parts, void *out, const int64_t o_stride[3], float *lse,
                             hipStream_t stream)
{
    const int rows = p.batch * p.n_q_heads * p.n_tree;
    const dim3 block(256), grid((rows + 3) / 4);
#define LS_TM_LAUNCH(T, PT, DD, CH)                                                                          \
    hipLaunchKernelGGL((tree_merge_kernel<T, PT, DD, CH>), grid, block, 0, stream, p, mask, cache_parts,      \
                       n_cache_parts, (T *)out, o_stride[0], o_stride[1], o_stride[2], lse)
#define LS_TM_CASE(T, PT, DD)                          \
    do {                                               \
        if (n_cache_parts <= 8) LS_TM_LAUNCH(T, PT, DD, 8); \
        else LS_TM_LAUNCH(T, PT, DD, 32);              \
    } while (0)
    if (p.head_dim != 64 && p.head_dim != 128) return hipErrorInvalidValue;
    if (dtype == LS_BF16) {
        if (cache_parts.o_is_16bit) {
            if (p.head_dim == 128) LS_TM_CASE(uint16_t, uint16_t, 128);
            else LS_TM_CASE(uint16_t, uint16_t, 64);
        } else {
            if (p.head_dim == 128) LS_TM_CASE(uint16_t, float, 128);
            else LS_TM_CASE(uint16_t, float, 64);
        }
    } else if (dtype == LS_F16) {
        if (cache_parts.o_is_16bit) {
            if (p.head_dim == 128) LS_TM_CASE(half_t, half_t, 128);
            else LS_TM_CASE(half_t, half_t, 64);
        } else {
            if (p.head_dim == 128) LS_TM_CASE(half_t, float, 128);
            else LS_TM_CASE(half_t, float, 64);
        }
    } else {
        if (cache_parts.o_is_16bit) return hipErrorInvalidValue;
        if (p.head_dim == 128) LS_TM_CASE(float, float, 128);
        else LS_TM_CASE(float, float, 64);
    }
#undef LS_TM_CASE
#undef LS_TM_LAUNCH
    return hipGetLastError();
}

}  // namespace ls
