// The small kernels of the path: tree-mask builder, masked tree attention, log-sum-exp
// merge, and the fused tree attention + merge that closes the whole call.  (LongSpec, Section 3.3; the aggregation appendix.)
#include "ls_internal.hpp"
#include "ls_tail.hpp"

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

// Zeroes n 32-bit words (the arrival counters of the single-launch call; a kernel rather than a
// memset so that the call may sit in a captured graph).
__global__ void __launch_bounds__(256) clear_words_kernel(uint32_t *__restrict__ words, int32_t n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) words[i] = 0u;
}

hipError_t launch_clear_words(uint32_t *words, int32_t n, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(clear_words_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, words, n);
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
// The kernel that ends the two-launch call: tail_rows (ls_tail.hpp) over all query rows.
// The whole-wavefront-per-row form is taken for more than 16 split rows per query row and at most
// this many rows (eight wavefronts per SIMD).
constexpr int kTailWideMaxRows = 8192;

// Waves per SIMD the compiler must leave room for (every load carries a 64-bit address of its
// own, so the register count is well above that of the data in flight).  The form for many rows
// (16 lanes per row, four 16-bit split rows per request) fits three; calls with tens of thousands of
// rows run in rounds of resident wavefronts, and a third wavefront per SIMD shortens them more
// than the registers it gives up would.
template <int LPR, int CH, int PART_BYTES> constexpr int tail_waves_per_simd()
{
    return (LPR == 16 && CH == 16) || CH * PART_BYTES >= 256 ? 1 : (LPR == 16 && CH * PART_BYTES < 128 ? 3 : 2);
}

template <typename T, typename PT, int D, int LPR, int CH>
__global__ void __launch_bounds__(kWave, (tail_waves_per_simd<LPR, CH, (int)sizeof(PT) * D / LPR>()))
tree_merge_kernel(Problem p, const uint64_t *__restrict__ mask, Partials parts, int32_t n_cache, T *__restrict__ out,
                  int64_t os0, int64_t os1, int64_t os2, float *__restrict__ lse)
{
    // Rows are numbered (sequence, KV head, tree node, query head within the group), so that the
    // rows of one wavefront mostly share their tree node and KV head.
    constexpr int RPW = kWave / LPR;  // query rows per wavefront
    const int lane = threadIdx.x;
    const int rows_total = p.batch * p.n_q_heads * p.n_tree;
    int r = blockIdx.x * RPW + lane / LPR;
    const bool live = r < rows_total;
    r = live ? r : rows_total - 1;  // lanes past the last row repeat it and store nothing
    const int hh = r % p.group;
    int t = r / p.group;
    const int i = t % p.n_tree;
    t /= p.n_tree;
    const int g = t % p.n_kv_heads;
    const int b = t / p.n_kv_heads;
    const uint64_t *mask_b = mask ? mask + (size_t)b * p.n_tree * ((p.n_tree + 63) >> 6) : nullptr;
    tail_rows<T, PT, D, LPR, CH>(p, mask_b, parts, n_cache, out, os0, os1, os2, lse, b, g * p.group + hh, i, live, lane);
}

hipError_t launch_tree_merge(const Problem &p, int dtype, const uint64_t *mask, const Partials &cache_parts,
                             int32_t n_cache_parts, void *out, const int64_t o_stride[3], float *lse,
                             hipStream_t stream)
{
    const int rows = p.batch * p.n_q_heads * p.n_tree;
    // a whole wavefront per row: few rows, each with many split rows (see the kernel's comment)
    const bool wide = n_cache_parts > 16 && rows <= kTailWideMaxRows;
    const int rows_per_wave = wide ? 1 : 4;
    const dim3 block(kWave), grid((rows + rows_per_wave - 1) / rows_per_wave);
#define LS_TM_LAUNCH(T, PT, DD, LPR, CH)                                                                          \
    hipLaunchKernelGGL((tree_merge_kernel<T, PT, DD, LPR, CH>), grid, block, 0, stream, p, mask, cache_parts,     \
                       n_cache_parts, (T *)out, o_stride[0], o_stride[1], o_stride[2], lse)
#define LS_TM_CASE(T, PT, DD)                                        \
    do {                                                             \
        if (wide) LS_TM_LAUNCH(T, PT, DD, 64, 32);                   \
        else if (n_cache_parts <= 8) LS_TM_LAUNCH(T, PT, DD, 16, 4); \
        else LS_TM_LAUNCH(T, PT, DD, 16, 16);                        \
    } while (0)
    if (p.head_dim != 64 && p.head_dim != 128) return hipErrorInvalidValue;
    if (rows <= 0) return hipSuccess;
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
