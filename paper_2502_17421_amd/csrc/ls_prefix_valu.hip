// Split-KV attention over the cached keys on the vector ALUs, with float arithmetic
// throughout.  This is the true-fp32 variant of step (b) (appendix: o_cache, LSE_cache per
// split) and the fallback for shapes the MFMA kernel does not take.
//
// One workgroup = one (sequence, KV head, block of 32 query rows, key split).  The query
// rows of a KV head are the G*T rows (g, t) of its G query heads.  Keys are streamed in
// tiles of 32 through LDS; scores, the online softmax and the P*V product are computed per
// tile.  Thread (r, c) = (tid / 8, tid % 8) owns query row r: it computes the scores of
// keys c, c+8, c+16, c+24 of the tile and accumulates output columns 4(c+8i) .. 4(c+8i)+3.
#include "ls_internal.hpp"

namespace ls {

namespace {
constexpr int TQ = 32;  // query rows per workgroup
constexpr int TK = 32;  // keys per tile

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
}

template <typename T, int D>
__global__ void __launch_bounds__(256)
prefix_valu_kernel(Problem p, SplitPlan plan, Partials out, MaskJob mask_job)
{
    constexpr int KP = D + 4;  // padded row, still 16-byte aligned: the 8 rows a wave reads together hit distinct banks
    __shared__ __attribute__((aligned(16))) float q_s[TQ][KP];
    __shared__ __attribute__((aligned(16))) float k_s[TK][KP];
    __shared__ __attribute__((aligned(16))) float v_s[TK][D];
    __shared__ __attribute__((aligned(16))) float p_s[TQ][TK + 4];

    const int tid = threadIdx.x;
    const int r = tid >> 3, c = tid & 7;
    // One extra z-slice of the grid (present only in the whole-path launch) builds the tree masks,
    // one workgroup per sequence, so that the call needs one launch less.
    if ((int)blockIdx.z == p.batch * p.n_kv_heads) {
        const int mb = blockIdx.y * gridDim.x + blockIdx.x;
        if (mb >= p.batch) return;
        const int words = (p.n_tree + 63) >> 6;
        build_tree_mask_rows(mask_job.parents + (size_t)mb * p.n_tree, p.n_tree,
                             mask_job.mask + (size_t)mb * p.n_tree * words,
                             mask_job.err_flag ? mask_job.err_flag + mb : nullptr, tid, (int)blockDim.x);
        return;
    }
    const int split = blockIdx.x;
    const int qblock = blockIdx.y;
    const int b = blockIdx.z / p.n_kv_heads;
    const int g = blockIdx.z % p.n_kv_heads;
    const int rows_kv = p.group * p.n_tree;  // query rows that share this KV head

    int plen = p.prefix_lens ? p.prefix_lens[b] : p.prefix_len_all;
    plen = plen < 0 ? 0 : (plen > p.max_prefix_len ? p.max_prefix_len : plen);
    const int k_lo = split * plan.split_len;
    int k_hi = k_lo + plan.split_len;
    k_hi = k_hi > plen ? plen : k_hi;

    // my query row
    const int m = qblock * TQ + r;
    const bool row_ok = m < rows_kv;
    const int hq = g * p.group + (row_ok ? m / p.n_tree : 0);
    const int ti = row_ok ? m % p.n_tree : 0;

    // stage the query block, pre-multiplied by scale*log2(e); 4 consecutive elements per thread
    // and step, all loads of a thread issued before the first LDS store
    constexpr int QV = TQ * D / 4 / 256;  // 4-element pieces per thread
    {
        float4 qv[QV];
#pragma unroll
        for (int n = 0; n < QV; ++n) {
            const int e = (tid + n * 256) * 4;
            const int rr = e / D, dd = e % D;
            const int mm = qblock * TQ + rr;
            qv[n] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (mm < rows_kv) {
                const T *qp = (const T *)p.q + b * p.q_stride[0] + (g * p.group + mm / p.n_tree) * p.q_stride[1] +
                              (mm % p.n_tree) * p.q_stride[2];
                qv[n] = load4(qp + dd);
            }
        }
#pragma unroll
        for (int n = 0; n < QV; ++n) {
            const int e = (tid + n * 256) * 4;
            const int rr = e / D, dd = e % D;
            *(float4 *)&q_s[rr][dd] = make_float4(qv[n].x * p.scale_log2, qv[n].y * p.scale_log2,
                                                  qv[n].z * p.scale_log2, qv[n].w * p.scale_log2);
        }
    }

    // thread (r, c) accumulates output columns 4*(c + 8*i) .. +3 of row r, i < D/32
    float4 acc[D / 32];
#pragma unroll
    for (int i = 0; i < D / 32; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    float m_run = -INFINITY, l_run = 0.f;

    const T *kbase = (const T *)p.k_cache + b * p.kc_stride[0] + g * p.kc_stride[1];
    const T *vbase = (const T *)p.v_cache + b * p.vc_stride[0] + g * p.vc_stride[1];

    for (int k0 = k_lo; k0 < k_hi; k0 += TK) {
        __syncthreads();  // previous tile fully consumed (and q_s visible on the first pass)
        {
            constexpr int KV = TK * D / 4 / 256;  // 4-element pieces per thread and tensor
            float4 kr[KV], vr[KV];
#pragma unroll
            for (int n = 0; n < KV; ++n) {
                const int e = (tid + n * 256) * 4;
                const int jj = e / D, dd = e % D;
                const int key = k0 + jj;
                kr[n] = make_float4(0.f, 0.f, 0.f, 0.f);
                vr[n] = kr[n];
                if (key < k_hi) {
                    kr[n] = load4(kbase + key * p.kc_stride[2] + dd);
                    vr[n] = load4(vbase + key * p.vc_stride[2] + dd);
                }
            }
#pragma unroll
            for (int n = 0; n < KV; ++n) {
                const int e = (tid + n * 256) * 4;
                const int jj = e / D, dd = e % D;
                *(float4 *)&k_s[jj][dd] = kr[n];
                *(float4 *)&v_s[jj][dd] = vr[n];
            }
        }
        __syncthreads();

        float s[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) s[a] = 0.f;
        // 16 head-dim elements per step: all 20 LDS reads of a step are issued before the first
        // product, so their latencies overlap instead of adding up
        for (int dd = 0; dd < D; dd += 16) {
            float4 q4[4], k4[4][4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                q4[u] = *(const float4 *)&q_s[r][dd + 4 * u];
#pragma unroll
                for (int a = 0; a < 4; ++a) k4[a][u] = *(const float4 *)&k_s[c + 8 * a][dd + 4 * u];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    s[a] += q4[u].x * k4[a][u].x + q4[u].y * k4[a][u].y + q4[u].z * k4[a][u].z + q4[u].w * k4[a][u].w;
        }
        float tmax = -INFINITY;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            if (k0 + c + 8 * a >= k_hi) s[a] = -INFINITY;
            tmax = fmaxf(tmax, s[a]);
        }
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, off, kWave));
        const float m_new = fmaxf(m_run, tmax);  // finite: every tile holds at least one key
        const float alpha = exp2f(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const float pj = exp2f(s[a] - m_new);
            p_s[r][c + 8 * a] = pj;
            psum += pj;
        }
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) psum += __shfl_xor(psum, off, kWave);
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int i = 0; i < D / 32; ++i) {
            acc[i].x *= alpha;
            acc[i].y *= alpha;
            acc[i].z *= alpha;
            acc[i].w *= alpha;
        }
        __syncthreads();  // p_s row r complete
        for (int jj = 0; jj < TK; jj += 4) {  // likewise: the reads of four keys first, then the products
            const float4 p4 = *(const float4 *)&p_s[r][jj];
            const float pj[4] = {p4.x, p4.y, p4.z, p4.w};
            float4 v4[4][D / 32];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < D / 32; ++i) v4[u][i] = *(const float4 *)&v_s[jj + u][4 * (c + 8 * i)];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < D / 32; ++i) {
                    acc[i].x += pj[u] * v4[u][i].x;
                    acc[i].y += pj[u] * v4[u][i].y;
                    acc[i].z += pj[u] * v4[u][i].z;
                    acc[i].w += pj[u] * v4[u][i].w;
                }
        }
    }

    if (!row_ok) return;
    const size_t prow = out.row((size_t)b * p.n_q_heads + hq, split, p.n_tree, ti);
    if (l_run > 0.f) {
        const float inv = 1.f / l_run;
        float *orow = (float *)out.o + prow * D;
#pragma unroll
        for (int i = 0; i < D / 32; ++i)
            *(float4 *)(orow + 4 * (c + 8 * i)) = make_float4(acc[i].x * inv, acc[i].y * inv, acc[i].z * inv,
                                                              acc[i].w * inv);
        if (c == 0) out.lse[prow] = (m_run + log2f(l_run)) * kLn2;
    } else if (c == 0) {
        out.lse[prow] = -INFINITY;
    }
}

hipError_t launch_prefix_valu(const Problem &p, int dtype, const SplitPlan &plan, const Partials &out,
                              const MaskJob &mask_job, hipStream_t stream)
{
    const int rows_kv = p.group * p.n_tree;
    const int n_qblocks = (rows_kv + TQ - 1) / TQ;
    const bool with_mask = mask_job.parents != nullptr;
    // the mask slice offers n_splits * n_qblocks workgroups: enough for the batch?
    if (with_mask && (int64_t)plan.n_splits * n_qblocks < p.batch) return hipErrorInvalidValue;
    const dim3 block(256), grid(plan.n_splits, n_qblocks, p.batch * p.n_kv_heads + (with_mask ? 1 : 0));
#define LS_PV_CASE(T, DD) \
    hipLaunchKernelGGL((prefix_valu_kernel<T, DD>), grid, block, 0, stream, p, plan, out, mask_job)
    if (dtype == LS_BF16 && p.head_dim == 128) LS_PV_CASE(uint16_t, 128);
    else if (dtype == LS_BF16 && p.head_dim == 64) LS_PV_CASE(uint16_t, 64);
    else if (dtype == LS_F16 && p.head_dim == 128) LS_PV_CASE(half_t, 128);
    else if (dtype == LS_F16 && p.head_dim == 64) LS_PV_CASE(half_t, 64);
    else if (dtype == LS_F32 && p.head_dim == 128) LS_PV_CASE(float, 128);
    else if (dtype == LS_F32 && p.head_dim == 64) LS_PV_CASE(float, 64);
    else return hipErrorInvalidValue;
#undef LS_PV_CASE
    return hipGetLastError();
}

}  // namespace ls
