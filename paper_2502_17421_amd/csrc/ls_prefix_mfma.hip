// Split-KV attention over the cached keys on the bf16 matrix cores (gfx950 MFMA).
// Step (b) of the path: per key split, o_cache and LSE_cache of the aggregation appendix.
//
// Work decomposition.  All G*T query rows that share a KV head (G query heads x T tree
// tokens) form one dense query tile, so every cached K/V row is fetched from HBM once per
// KV head and used by all of them.  A workgroup owns (sequence, KV head, key split, block
// of up to WQ*NT*32 query rows); wave wq of the workgroup owns NT groups of 32 query rows.
// Keys stream through LDS in tiles of 64.
//
// Operand orientation.  Scores are computed transposed, S^T = K Q^T (keys along the MFMA
// M axis, queries along N).  With the 32x32 accumulator layout a lane then holds, for ONE
// query (column = lane % 32), 4-key runs of the tile: exactly the per-lane contraction
// slices that the B operand of the next product O^T = V^T P^T needs.  So the softmax
// numerators go from accumulator registers to the second MFMA with a bf16 pack and no
// cross-lane traffic, and the per-query max / sum are a register reduction plus one
// exchange between lane l and lane l ^ 32.
//
// MFMA layouts used (v_mfma_f32_32x32x16_bf16, A is 32xK, B is Kx32, K = 16):
//   A: lane l holds row l % 32, contraction indices 8*(l/32) .. 8*(l/32)+7
//   B: lane l holds column l % 32, same contraction indices
//   C/D: lane l, register r holds row 8*(r/4) + 4*(l/32) + r%4, column l % 32
// Only the C/D layout and the pairing of contraction slices between A and B matter.
#include "ls_internal.hpp"

namespace ls {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int TK = 64;   // keys per LDS tile
constexpr int KTW = 2;   // 32-key MFMA row tiles per key tile
constexpr int VPAD = 4;  // padding (elements) of a transposed V row in LDS

__device__ __forceinline__ floatx16 mfma32(bf16x8 a, bf16x8 b, floatx16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    floatx2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

}  // namespace

template <int D, int NT, int WQ>
__global__ void __launch_bounds__(WQ * 64)
prefix_mfma_kernel(Problem p, SplitPlan plan, Partials out)
{
    constexpr int NTHREADS = WQ * 64;
    constexpr int KSTEPS = D / 16;  // contraction steps of S^T = K Q^T
    constexpr int MT = D / 32;      // 32-row tiles of O^T along head_dim
    constexpr int CH = D / 8;       // 16-byte chunks per K/V row
    constexpr int VROW = TK + VPAD;
    constexpr int CHUNKS = TK * CH / NTHREADS;  // 16-byte chunks each thread stages per tile and tensor
    static_assert(TK * CH % NTHREADS == 0, "tile must divide over the workgroup");

    __shared__ __attribute__((aligned(16))) uint16_t k_s[TK * D];   // [key][chunk ^ (key % CH)][8]
    __shared__ __attribute__((aligned(16))) uint16_t vt_s[D * VROW];  // [d][key], V transposed

    const int tid = threadIdx.x;
    const int wq = tid >> 6;
    const int lane = tid & 63;
    const int li = lane & 31;
    const int lh = lane >> 5;

    const int split = blockIdx.x;
    const int qblock = blockIdx.y;
    const int b = blockIdx.z / p.n_kv_heads;
    const int g = blockIdx.z % p.n_kv_heads;
    const int rows_kv = p.group * p.n_tree;

    int plen = p.prefix_lens[b];
    plen = plen < 0 ? 0 : (plen > p.max_prefix_len ? p.max_prefix_len : plen);
    const int k_lo = split * plan.split_len;
    int k_hi = k_lo + plan.split_len;
    k_hi = k_hi > plen ? plen : k_hi;

    // The query rows of this lane: one per 32-row group nt.
    int q_row[NT];
    bool q_ok[NT];
    size_t part_row[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int m = (qblock * WQ + wq) * (NT * 32) + nt * 32 + li;
        q_row[nt] = m;
        q_ok[nt] = m < rows_kv;
        const int hq = g * p.group + (q_ok[nt] ? m / p.n_tree : 0);
        const int ti = q_ok[nt] ? m % p.n_tree : 0;
        part_row[nt] = (((size_t)b * p.n_q_heads + hq) * out.parts_stride + out.part_base + split) * p.n_tree + ti;
    }

    if (k_lo >= k_hi) {  // empty split: weight zero in the merge
        if (lh == 0) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (q_ok[nt]) out.lse[part_row[nt]] = -INFINITY;
        }
        return;
    }

    // Q^T as the B operand, kept in registers for the whole split.
    bf16x8 q_reg[NT][KSTEPS];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int m = q_row[nt];
        const uint16_t *qp = (const uint16_t *)p.q + b * p.q_stride[0] +
                             (g * p.group + (q_ok[nt] ? m / p.n_tree : 0)) * p.q_stride[1] +
                             (q_ok[nt] ? m % p.n_tree : 0) * p.q_stride[2];
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (q_ok[nt]) v = *(const uint4 *)(qp + kk * 16 + lh * 8);
            q_reg[nt][kk] = __builtin_bit_cast(bf16x8, v);
        }
    }

    floatx16 o_acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[mt][nt][r] = 0.f;
    float m_run[NT], l_run[NT];  // running max of raw scores; running sum (this lane's keys only)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_run[nt] = -INFINITY;
        l_run[nt] = 0.f;
    }

    const uint16_t *kbase = (const uint16_t *)p.k_cache + b * p.kc_stride[0] + g * p.kc_stride[1];
    const uint16_t *vbase = (const uint16_t *)p.v_cache + b * p.vc_stride[0] + g * p.vc_stride[1];
    const float c = p.scale_log2;

    uint4 k_stage[CHUNKS], v_stage[CHUNKS];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int n = 0; n < CHUNKS; ++n) {
            const int e = tid + n * NTHREADS;
            const int row = e / CH, cpos = e % CH;
            const int key = k0 + row;
            uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
            if (key < k_hi) {
                kv = *(const uint4 *)(kbase + key * p.kc_stride[2] + cpos * 8);
                vv = *(const uint4 *)(vbase + key * p.vc_stride[2] + cpos * 8);
            }
            k_stage[n] = kv;
            v_stage[n] = vv;
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int n = 0; n < CHUNKS; ++n) {
            const int e = tid + n * NTHREADS;
            const int row = e / CH, cpos = e % CH;
            *(uint4 *)(k_s + row * D + ((cpos ^ (row & (CH - 1))) * 8)) = k_stage[n];
            const uint32_t w[4] = {v_stage[n].x, v_stage[n].y, v_stage[n].z, v_stage[n].w};
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                vt_s[(cpos * 8 + 2 * e2) * VROW + row] = (uint16_t)(w[e2] & 0xffffu);
                vt_s[(cpos * 8 + 2 * e2 + 1) * VROW + row] = (uint16_t)(w[e2] >> 16);
            }
        }
    };

    fetch(k_lo);
    for (int k0 = k_lo; k0 < k_hi; k0 += TK) {
        __syncthreads();  // every wave is done reading the previous tile
        stash();
        __syncthreads();
        if (k0 + TK < k_hi) fetch(k0 + TK);  // in flight while this tile is consumed

        // ---- S^T = K Q^T --------------------------------------------------------------
        floatx16 s_acc[KTW][NT];
#pragma unroll
        for (int kt = 0; kt < KTW; ++kt) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) s_acc[kt][nt][r] = 0.f;
            const int row = kt * 32 + li;
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
                const int pos = (2 * kk + lh) ^ (row & (CH - 1));
                const bf16x8 a = __builtin_bit_cast(bf16x8, *(const uint4 *)(k_s + row * D + pos * 8));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) s_acc[kt][nt] = mfma32(a, q_reg[nt][kk], s_acc[kt][nt]);
            }
        }

        // keys past the end of the split weigh nothing (only the last tile can hold any)
        if (k0 + TK > k_hi) {
#pragma unroll
            for (int kt = 0; kt < KTW; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = k0 + kt * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                    if (key >= k_hi) {
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) s_acc[kt][nt][r] = -INFINITY;
                    }
                }
        }

        // ---- online softmax, one query per lane and group ---------------------------------
        uint32_t p_pk[KTW][NT][8];  // bf16 pairs: the B operands of the second product
        bool rescale = false;
        float alpha[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float mx = s_acc[0][nt][0];
#pragma unroll
            for (int kt = 0; kt < KTW; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_acc[kt][nt][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float m_new = fmaxf(m_run[nt], mx);  // finite: the tile holds at least one key
            alpha[nt] = exp2f((m_run[nt] - m_new) * c);
            rescale |= (m_new != m_run[nt]);
            m_run[nt] = m_new;
            const float mc = m_new * c;
            float sum = 0.f;
#pragma unroll
            for (int kt = 0; kt < KTW; ++kt)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float p0 = exp2f(s_acc[kt][nt][r] * c - mc);
                    const float p1 = exp2f(s_acc[kt][nt][r + 1] * c - mc);
                    sum += p0 + p1;
                    p_pk[kt][nt][r >> 1] = pack_bf16(p0, p1);
                }
            l_run[nt] = l_run[nt] * alpha[nt] + sum;
        }
        if (__any(rescale)) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[mt][nt][r] *= alpha[nt];
        }

        // ---- O^T += V^T P^T ------------------------------------------------------------
#pragma unroll
        for (int kt = 0; kt < KTW; ++kt)
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                bf16x8 pb[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const uint4 v = make_uint4(p_pk[kt][nt][4 * a], p_pk[kt][nt][4 * a + 1],
                                               p_pk[kt][nt][4 * a + 2], p_pk[kt][nt][4 * a + 3]);
                    pb[nt] = __builtin_bit_cast(bf16x8, v);
                }
                const int koff = kt * 32 + a * 16 + 4 * lh;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const uint16_t *vp = vt_s + (mt * 32 + li) * VROW + koff;
                    const uint2 lo = *(const uint2 *)vp;
                    const uint2 hi = *(const uint2 *)(vp + 8);
                    const bf16x8 av = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) o_acc[mt][nt] = mfma32(av, pb[nt], o_acc[mt][nt]);
                }
            }
    }

    // ---- epilogue: normalise and store this split's partial result -----------------------
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const float l_tot = l_run[nt] + __shfl_xor(l_run[nt], 32, kWave);
        if (!q_ok[nt]) continue;
        const float inv = 1.f / l_tot;
        float *orow = out.o + part_row[nt] * D;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                float4 v;
                v.x = o_acc[mt][nt][4 * rg + 0] * inv;
                v.y = o_acc[mt][nt][4 * rg + 1] * inv;
                v.z = o_acc[mt][nt][4 * rg + 2] * inv;
                v.w = o_acc[mt][nt][4 * rg + 3] * inv;
                *(float4 *)(orow + mt * 32 + 8 * rg + 4 * lh) = v;
            }
        if (lh == 0) out.lse[part_row[nt]] = (m_run[nt] * c + log2f(l_tot)) * kLn2;
    }
}

bool prefix_mfma_supports(const Problem &p, int dtype)
{
    return dtype == LS_BF16 && (p.head_dim == 128 || p.head_dim == 64);
}

hipError_t launch_prefix_mfma(const Problem &p, const SplitPlan &plan, const Partials &out, hipStream_t stream)
{
    const int rows_kv = p.group * p.n_tree;
    const unsigned gz = p.batch * p.n_kv_heads;
#define LS_PM_CASE(DD, NT, WQ)                                                                  \
    do {                                                                                          \
        const dim3 grid(plan.n_splits, (rows_kv + (WQ) * (NT) * 32 - 1) / ((WQ) * (NT) * 32), gz); \
        hipLaunchKernelGGL((prefix_mfma_kernel<DD, NT, WQ>), grid, dim3((WQ) * 64), 0, stream, p, plan, out); \
    } while (0)
    if (p.head_dim == 128) {
        if (rows_kv > 128) LS_PM_CASE(128, 2, 4);
        else if (rows_kv > 64) LS_PM_CASE(128, 1, 4);
        else if (rows_kv > 32) LS_PM_CASE(128, 1, 2);
        else LS_PM_CASE(128, 1, 1);
    } else if (p.head_dim == 64) {
        if (rows_kv > 128) LS_PM_CASE(64, 2, 4);
        else if (rows_kv > 64) LS_PM_CASE(64, 1, 4);
        else if (rows_kv > 32) LS_PM_CASE(64, 1, 2);
        else LS_PM_CASE(64, 1, 1);
    } else {
        return hipErrorInvalidValue;
    }
#undef LS_PM_CASE
    return hipGetLastError();
}

}  // namespace ls
