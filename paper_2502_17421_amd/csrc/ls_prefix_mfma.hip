// Split-KV attention over the cached keys on the bf16 matrix cores (gfx950 MFMA).
// Step (b) of the path: per key split, o_cache and LSE_cache of the aggregation appendix.
//
// Work decomposition.  All G*T query rows that share a KV head (G query heads x T tree
// tokens) form one dense query tile, so every cached K/V row is fetched from HBM once per
// KV head and used by all of them.  A workgroup owns (sequence, KV head, key split, block
// of up to WQ*NT*32 query rows); wave wq of the workgroup owns NT groups of 32 query rows.
//
// Data movement.  K and V rows go HBM -> LDS directly (global_load_lds_dwordx4, 16 bytes
// per lane, no staging registers) into a ring of NS stages of 64 keys each, so several
// tiles are in flight per compute unit while one is consumed.  The instruction writes LDS
// linearly (lane l -> base + 16*l), so the bank swizzle is applied on the global side:
// the lane that fills LDS slot (row, pos) fetches chunk pos ^ swizzle(row) of that row.
//
// Operand orientation.  Scores are computed transposed, S^T = K Q^T (keys along the MFMA
// M axis, queries along N).  With the 32x32 accumulator layout a lane then holds, for ONE
// query (column = lane % 32), 4-key runs of the tile: exactly the per-lane contraction
// slices that the B operand of the next product O^T = V^T P^T needs.  So the softmax
// numerators go from accumulator registers to the second MFMA with a bf16 pack and no
// cross-lane traffic, and the per-query max / sum are a register reduction plus one
// exchange between the two 32-lane halves.  V^T (the A operand of the second product)
// is read from the row-major V tile with the LDS transpose read ds_read_b64_tr_b16.
//
// MFMA layouts used (v_mfma_f32_32x32x16_bf16, A is 32xK, B is Kx32, K = 16):
//   A: lane l holds row l % 32, contraction indices 8*(l/32) .. 8*(l/32)+7
//   B: lane l holds column l % 32, same contraction indices
//   C/D: lane l, register r holds row 8*(r/4) + 4*(l/32) + r%4, column l % 32
// Only the C/D layout and the pairing of contraction slices between A and B matter.
// ds_read_b64_tr_b16, per block of 16 lanes: lane L receives element L%4 of the four
// 8-byte pieces addressed by lanes L/4, L/4+4, L/4+8, L/4+12 of its block.
#include "ls_internal.hpp"

namespace ls {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int TK = 64;        // keys per LDS stage
constexpr int SUB = 32;       // keys per softmax step (one MFMA row tile)
constexpr float kLazy = 8.f;  // the running max is left alone while scores stay below max + 8 (base 2)

#define LS_LDS(p) ((__attribute__((address_space(3))) void *)(p))
#define LS_GLB(p) ((const __attribute__((address_space(1))) void *)(p))

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

// max / sum across the two 32-lane halves of the wave (lane l with lane l ^ 32)
__device__ __forceinline__ float half_max(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One 64-lane HBM -> LDS copy: lane l moves 16 bytes from its own global address to LDS byte
// lds_base + 16*l (lds_base wave-uniform, passed through M0).  Written as inline assembly so
// that the compiler does not serialise later LDS reads behind all copies still in flight; the
// kernel orders reads after copies itself with wait_vmem + a barrier.
__device__ __forceinline__ void copy_row_group_to_lds(const void *gptr, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_base), "v"(gptr)
                 : "memory");
}

__device__ __forceinline__ uint32_t lds_offset(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

template <int N> __device__ __forceinline__ void wait_vmem()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// V swizzle: row r of a V tile stores its 16-byte chunk c at position c ^ vswz(r).  Rows
// r, r+1, r+2, r+3 then put the 32-byte pieces one transpose read touches on distinct banks.
__device__ __forceinline__ int vswz(int row)
{
    const int k = row & 3;
    return (((k >> 1) << 2) | ((k & 1) << 1) | (k >> 1)) << 1;
}

}  // namespace

template <int D, int NT, int WQ, int NS>
__global__ void __launch_bounds__(WQ * 64)
prefix_mfma_kernel(Problem p, SplitPlan plan, Partials out)
{
    constexpr int KSTEPS = D / 16;            // contraction steps of S^T = K Q^T
    constexpr int MT = D / 32;                // 32-row tiles of O^T along head_dim
    constexpr int CH = D / 8;                 // 16-byte chunks per K/V row
    constexpr int ROWB = D * 2;               // bytes per K/V row
    constexpr int TILEB = TK * ROWB;          // bytes per K (or V) tile
    constexpr int STAGEB = 2 * TILEB;         // K tile then V tile
    constexpr int ROWS_PER_LOAD = 64 / CH;    // rows one 64-lane load instruction covers
    constexpr int LOADS = TK / WQ / ROWS_PER_LOAD;  // load instructions per wave, tile and tensor
    static_assert(TK % (WQ * ROWS_PER_LOAD) == 0, "tile rows must divide over the waves");
    static_assert(NS >= 2 && NS <= 4, "ring depth");
    static_assert((NS - 1) * 2 * LOADS <= 63, "the vmcnt counter holds at most 63 outstanding loads");
    constexpr int INFLIGHT = 2 * LOADS;       // vmem instructions per wave and stage

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

    const int tid = threadIdx.x;
    const int wq = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    bool q_ok[NT];
    size_t part_row[NT];
    const uint16_t *q_ptr[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int m = (qblock * WQ + wq) * (NT * 32) + nt * 32 + li;
        q_ok[nt] = m < rows_kv;
        const int hq = g * p.group + (q_ok[nt] ? m / p.n_tree : 0);
        const int ti = q_ok[nt] ? m % p.n_tree : 0;
        part_row[nt] = (((size_t)b * p.n_q_heads + hq) * out.parts_stride + out.part_base + split) * p.n_tree + ti;
        q_ptr[nt] = (const uint16_t *)p.q + b * p.q_stride[0] + hq * p.q_stride[1] + ti * p.q_stride[2];
    }

    if (k_lo >= k_hi) {  // empty split: weight zero in the merge
        if (lh == 0) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (q_ok[nt]) out.lse[part_row[nt]] = -INFINITY;
        }
        return;
    }

    // Q^T as the B operand, kept in registers for the whole split.  The loads are issued here
    // and collected after the first key tiles have been requested (see collect_q below); they
    // are inline assembly so that no compiler-placed wait for them lands inside the key loop,
    // where it would also wait for every key tile still in flight.
    u32x4 q_raw[NT][KSTEPS];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
            asm volatile("global_load_dwordx4 %0, %1, off"
                         : "=v"(q_raw[nt][kk])
                         : "v"(q_ptr[nt] + kk * 16 + lh * 8)
                         : "memory");

    // ---- HBM -> LDS tile loads ----------------------------------------------------------
    const uint8_t *kbase = (const uint8_t *)p.k_cache + (b * p.kc_stride[0] + g * p.kc_stride[1]) * 2;
    const uint8_t *vbase = (const uint8_t *)p.v_cache + (b * p.vc_stride[0] + g * p.vc_stride[1]) * 2;
    const int64_t k_row_bytes = p.kc_stride[2] * 2, v_row_bytes = p.vc_stride[2] * 2;
    const int ld_row = lane / CH;  // row within one load instruction
    const int ld_pos = lane % CH;  // LDS chunk position this lane fills
    const uint32_t smem_off = lds_offset(smem);
    auto issue_tile = [&](int k0, int stage) {
        const uint32_t ks_off = __builtin_amdgcn_readfirstlane(smem_off + stage * STAGEB);
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const int row0 = (wq * LOADS + j) * ROWS_PER_LOAD;  // wave-uniform
            const int row = row0 + ld_row;
            int key = k0 + row;
            key = key < k_hi ? key : k_hi - 1;  // rows past the end repeat the last row; their scores are masked
            const int kc = ld_pos ^ (row & (CH - 1));
            const int vc = ld_pos ^ (vswz(row) & (CH - 1));
            copy_row_group_to_lds(kbase + key * k_row_bytes + kc * 16, ks_off + row0 * ROWB);
            copy_row_group_to_lds(vbase + key * v_row_bytes + vc * 16, ks_off + TILEB + row0 * ROWB);
        }
    };

    const int n_tiles = (k_hi - k_lo + TK - 1) / TK;
    const int n_prologue = n_tiles < NS - 1 ? n_tiles : NS - 1;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < n_prologue) issue_tile(k_lo + s * TK, s);

    // collect Q: everything older than the prologue tiles has landed
    bool collected = false;
    if constexpr (NS >= 4) {
        if (n_prologue >= 3) {
            wait_vmem<3 * INFLIGHT>();
            collected = true;
        }
    }
    if constexpr (NS >= 3) {
        if (!collected && n_prologue == 2) {
            wait_vmem<2 * INFLIGHT>();
            collected = true;
        }
    }
    if (!collected) wait_vmem<INFLIGHT>();
    bf16x8 q_reg[NT][KSTEPS];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            asm volatile("" : "+v"(q_raw[nt][kk]));  // orders every use below after the wait above
            const u32x4 v = q_ok[nt] ? q_raw[nt][kk] : u32x4{0, 0, 0, 0};
            q_reg[nt][kk] = __builtin_bit_cast(bf16x8, v);
        }

    floatx16 o_acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[mt][nt][r] = 0.f;
    float m_run[NT], l_run[NT];  // reference max of raw scores; running sum over this lane's keys only
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m_run[nt] = -INFINITY;
        l_run[nt] = 0.f;
    }
    const float c = p.scale_log2;

    // per-lane LDS offsets of the operand reads
    const int k_lane_off = li * ROWB;              // + 32*kt rows; chunk (2kk+lh) ^ (li & (CH-1))
    const int k_swz = li & (CH - 1);
    const int tr_s = lane & 15;                    // lane within its 16-lane transpose block
    const int tr_row = 4 * lh + (tr_s >> 2);       // key row (within a 16-key step) this lane addresses
    const int tr_dchunk = 2 * ((lane >> 4) & 1) + ((tr_s & 3) >> 1);  // 16-byte chunk within a 32-wide d tile
    const int tr_sub = (tr_s & 1) * 8;             // byte offset inside the chunk
    const int tr_swz = vswz(tr_row) & (CH - 1);    // rows +8, +16, ... keep row & 3
    int v_lane_off[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
        v_lane_off[mt] = tr_row * ROWB + (((4 * mt + tr_dchunk) ^ tr_swz) * 16) + tr_sub;

    for (int t = 0; t < n_tiles; ++t) {
        // tile t has landed once at most the younger in-flight tiles remain outstanding
        const int younger = n_tiles - 1 - t < NS - 2 ? n_tiles - 1 - t : NS - 2;
        bool waited = false;
        if constexpr (NS >= 4) {
            if (younger >= 2) {
                wait_vmem<2 * INFLIGHT>();
                waited = true;
            }
        }
        if constexpr (NS >= 3) {
            if (!waited && younger == 1) {
                wait_vmem<INFLIGHT>();
                waited = true;
            }
        }
        if (!waited) wait_vmem<0>();
        __syncthreads();  // every wave's part of tile t is in LDS; every wave is done with tile t-1
        if (t + NS - 1 < n_tiles) issue_tile(k_lo + (t + NS - 1) * TK, (t + NS - 1) % NS);

        const uint8_t *ks = smem + (t % NS) * STAGEB;
        const uint8_t *vs = ks + TILEB;
        const int k0 = k_lo + t * TK;

#pragma unroll
        for (int kt = 0; kt < TK / SUB; ++kt) {
            // ---- S^T = K Q^T for 32 keys --------------------------------------------------
            floatx16 s_acc[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) s_acc[nt][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) {
                const int pos = (2 * kk + lh) ^ k_swz;
                const bf16x8 a =
                    __builtin_bit_cast(bf16x8, *(const uint4 *)(ks + kt * SUB * ROWB + k_lane_off + pos * 16));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) s_acc[nt] = mfma32(a, q_reg[nt][kk], s_acc[nt]);
            }
            // keys past the end of the split weigh nothing (only the last tile can hold any)
            if (k0 + (kt + 1) * SUB > k_hi) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = k0 + kt * SUB + 8 * (r >> 2) + 4 * lh + (r & 3);
                    if (key >= k_hi) {
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) s_acc[nt][r] = -INFINITY;
                    }
                }
            }

            // ---- online softmax, one query per lane and group -----------------------------
            float mx[NT];
            bool grow = false;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                float v = s_acc[nt][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) v = fmaxf(v, s_acc[nt][r]);
                mx[nt] = half_max(v);
                grow |= (mx[nt] - m_run[nt]) * c > kLazy;  // also true while m_run is -inf
            }
            if (__any(grow)) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const float m_new = fmaxf(m_run[nt], mx[nt]);
                    // a sub-tile whose keys are all masked leaves m_new = -inf; keep arithmetic finite
                    const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f((m_run[nt] - m_new) * c);
                    m_run[nt] = m_new;
                    l_run[nt] *= alpha;
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o_acc[mt][nt][r] *= alpha;
                }
            }
            uint32_t p_pk[NT][8];  // bf16 pairs: the B operands of the second product
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float mc = m_run[nt] == -INFINITY ? 0.f : m_run[nt] * c;
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(s_acc[nt][r] * c - mc);
                    const float p1 = __builtin_amdgcn_exp2f(s_acc[nt][r + 1] * c - mc);
                    sum += p0 + p1;
                    p_pk[nt][r >> 1] = pack_bf16(p0, p1);
                }
                l_run[nt] += sum;
            }

            // ---- O^T += V^T P^T ---------------------------------------------------------
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                bf16x8 pb[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const uint4 v = make_uint4(p_pk[nt][4 * a], p_pk[nt][4 * a + 1], p_pk[nt][4 * a + 2],
                                               p_pk[nt][4 * a + 3]);
                    pb[nt] = __builtin_bit_cast(bf16x8, v);
                }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const uint8_t *vp = vs + (kt * SUB + a * 16) * ROWB + v_lane_off[mt];
                    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) shortx4 *)LS_LDS(vp));
                    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) shortx4 *)LS_LDS(vp + 8 * ROWB));
                    const uint2 lo2 = __builtin_bit_cast(uint2, lo), hi2 = __builtin_bit_cast(uint2, hi);
                    const bf16x8 av = __builtin_bit_cast(bf16x8, make_uint4(lo2.x, lo2.y, hi2.x, hi2.y));
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) o_acc[mt][nt] = mfma32(av, pb[nt], o_acc[mt][nt]);
                }
            }
        }
    }

    // ---- epilogue: normalise and store this split's partial result -----------------------
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const float l_tot = half_sum(l_run[nt]);
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

namespace {

template <int D, int NT, int WQ, int NS>
hipError_t launch_one(const Problem &p, const SplitPlan &plan, const Partials &out, hipStream_t stream)
{
    constexpr int lds_bytes = NS * 2 * TK * D * 2;
    static_assert(lds_bytes <= 160 * 1024, "LDS ring exceeds the 160 KB of a compute unit");
    auto kernel = prefix_mfma_kernel<D, NT, WQ, NS>;
    static hipError_t attr = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 lds_bytes);
    if (attr != hipSuccess) return attr;
    const int rows_kv = p.group * p.n_tree;
    const int rows_wg = WQ * NT * 32;
    const dim3 grid(plan.n_splits, (rows_kv + rows_wg - 1) / rows_wg, p.batch * p.n_kv_heads);
    hipLaunchKernelGGL(kernel, grid, dim3(WQ * 64), lds_bytes, stream, p, plan, out);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_prefix_mfma(const Problem &p, const SplitPlan &plan, const Partials &out, hipStream_t stream)
{
    const int rows_kv = p.group * p.n_tree;
    if (p.head_dim == 128) {
        if (rows_kv > 128) return launch_one<128, 2, 4, 4>(p, plan, out, stream);
        if (rows_kv > 64) return launch_one<128, 1, 4, 4>(p, plan, out, stream);
        if (rows_kv > 32) return launch_one<128, 1, 2, 4>(p, plan, out, stream);
        return launch_one<128, 1, 1, 2>(p, plan, out, stream);
    }
    if (p.head_dim == 64) {
        if (rows_kv > 128) return launch_one<64, 2, 4, 4>(p, plan, out, stream);
        if (rows_kv > 64) return launch_one<64, 1, 4, 4>(p, plan, out, stream);
        if (rows_kv > 32) return launch_one<64, 1, 2, 4>(p, plan, out, stream);
        return launch_one<64, 1, 1, 4>(p, plan, out, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace ls
