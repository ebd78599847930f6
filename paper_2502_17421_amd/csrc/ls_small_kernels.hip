// The three small kernels of the path: tree-mask builder, masked tree attention,
// log-sum-exp merge.  (LongSpec, Section 3.3; the aggregation appendix.)
#include "ls_internal.hpp"

namespace ls {

// --------------------------------------------------------------------------- (a) ----
// Tree mask: thread i walks the parent chain of node i and sets one bit per node met,
// itself included.  The chain index strictly decreases, so the walk ends after at most
// i steps whatever the array holds; an entry outside {-1} u [0, j) ends the walk and is
// reported in err_flag[b] (written 0 or 1 on every launch).
template <int WORDS>
__global__ void __launch_bounds__(LS_MAX_TREE)
tree_mask_kernel(const int32_t *__restrict__ parents, int32_t n_tree, uint64_t *__restrict__ mask,
                 int32_t *__restrict__ err_flag)
{
    const int b = blockIdx.x;
    const int i = threadIdx.x;
    const int32_t *par = parents + (size_t)b * n_tree;
    uint64_t bits[WORDS];
#pragma unroll
    for (int w = 0; w < WORDS; ++w) bits[w] = 0;
    int bad = 0;
    int j = i < n_tree ? i : -1;
    while (j >= 0) {
#pragma unroll
        for (int w = 0; w < WORDS; ++w)
            if ((j >> 6) == w) bits[w] |= (uint64_t)1 << (j & 63);
        int p = par[j];
        if (p < -1 || p >= j) {
            bad = 1;
            p = -1;
        }
        j = p;
    }
    if (i < n_tree) {
        const int words = (n_tree + 63) >> 6;
        uint64_t *row = mask + ((size_t)b * n_tree + i) * words;
#pragma unroll
        for (int w = 0; w < WORDS; ++w)
            if (w < words) row[w] = bits[w];
    }
    const int any_bad = __syncthreads_or(bad);
    if (i == 0 && err_flag) err_flag[b] = any_bad ? 1 : 0;
}

hipError_t launch_tree_mask(const int32_t *parents, int32_t batch, int32_t n_tree, uint64_t *mask,
                            int32_t *err_flag, hipStream_t stream)
{
    static_assert(LS_MAX_TREE == 128, "two mask words");
    hipLaunchKernelGGL(tree_mask_kernel<2>, dim3(batch), dim3(LS_MAX_TREE), 0, stream, parents, n_tree,
                       mask, err_flag);
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
    const size_t prow = (((size_t)b * p.n_q_heads + h) * out.parts_stride + out.part_base) * p.n_tree + i;
    float *orow = out.o + prow * D;
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
template <typename T, int D>
__global__ void __launch_bounds__(256)
merge_kernel(int32_t rows_total, int32_t n_q_heads, int32_t n_tree, int32_t n_parts,
             const float *__restrict__ o_parts, const float *__restrict__ lse_parts, T *__restrict__ out,
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
            const float4 o = *(const float4 *)(o_parts + ((bh * n_parts + k) * n_tree + i) * D + c);
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
                        int32_t n_parts, const float *o_parts, const float *lse_parts, void *out,
                        const int64_t o_stride[3], float *lse, hipStream_t stream)
{
    const int rows = batch * n_q_heads * n_tree;
    const int threads = rows * (head_dim / 4);
    const dim3 block(256), grid((threads + 255) / 256);
#define LS_MERGE_CASE(T, DD)                                                                           \
    hipLaunchKernelGGL((merge_kernel<T, DD>), grid, block, 0, stream, rows, n_q_heads, n_tree, n_parts, \
                       o_parts, lse_parts, (T *)out, o_stride[0], o_stride[1], o_stride[2], lse)
    if (dtype == LS_BF16 && head_dim == 128) LS_MERGE_CASE(uint16_t, 128);
    else if (dtype == LS_BF16 && head_dim == 64) LS_MERGE_CASE(uint16_t, 64);
    else if (dtype == LS_F32 && head_dim == 128) LS_MERGE_CASE(float, 128);
    else if (dtype == LS_F32 && head_dim == 64) LS_MERGE_CASE(float, 64);
    else return hipErrorInvalidValue;
#undef LS_MERGE_CASE
    return hipGetLastError();
}

}  // namespace ls
