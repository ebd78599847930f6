// Split-KV attention over the cached keys on the 16-bit matrix cores (gfx950 MFMA; bf16 or
// IEEE half inputs, selected by the template flag F16, fp32 accumulation either way).
// Step (b) of the path: per key split, o_cache and LSE_cache of the aggregation appendix.
//
// Work decomposition.  All G*T query rows that share a KV head (G query heads x T tree
// tokens) form one dense query tile, so every cached K/V row is fetched from HBM once per
// KV head and used by all of them.  A workgroup owns (sequence, KV head, key split, block
// of up to NW*32 query rows); each of its NW waves owns 32 query rows and all keys.  With
// NW = 8 two waves share a SIMD.  Each wave runs a software pipeline over 32-key steps whose
// blocks pair the matrix work of the neighbouring steps (output product of step j-1, score
// product of step j+1) with the softmax arithmetic of step j.
//
// Data movement.  K and V rows go HBM -> LDS directly (global_load_lds_dwordx4, 16 bytes
// per lane, no staging registers) into a ring of NS stages of 64 keys each, so several
// tiles are in flight per compute unit while two are being consumed.  The instruction writes LDS
// linearly (lane l -> base + 16*l), so the bank swizzle is applied on the global side:
// the lane that fills LDS slot (row, pos) fetches chunk pos ^ swizzle(row) of that row.
//
// Each split walks its tiles starting at tile (split index mod tile count) and wraps around:
// all workgroups start together, and without this their addresses would differ only by
// multiples of the split size and crowd a few memory channels.
//
// Paged caches: a load instruction covers 4 or 8 consecutive rows, which a page of 16 rows
// or more never splits, so each instruction takes the base of its own page; the page ids of
// the split sit in registers (one lane per page) and are picked with v_readlane.
//
// The partial outputs leave through LDS (free by then) as whole 16-byte-per-lane rows with
// streaming stores; stored straight from the accumulator layout every store would touch 32
// rows with 16 bytes each.
//
// Operand orientation.  Scores are computed transposed, S^T = K Q^T (keys along the MFMA
// M axis, queries along N).  With the 32x32 accumulator layout a lane then holds, for ONE
// query (column = lane % 32), 4-key runs of the tile: exactly the per-lane contraction
// slices that the B operand of the next product O^T = V^T P^T needs.  So the softmax
// numerators go from accumulator registers to the second MFMA with a 16-bit pack and no
// cross-lane traffic, and the per-query max / sum are a register reduction plus one
// exchange between the two 32-lane halves.  V^T (the A operand of the second product)
// is read from the row-major V tile with the LDS transpose read ds_read_b64_tr_b16.
//
// Softmax state.  Per query the kernel keeps a reference exponent m (raw-score units) and
// the sum l of exp2((s - m) * c) over the keys seen, c = scale * log2(e).  m need not be
// the running maximum: any m gives the same O = sum p v / l and LSE = m*c + log2 l as long
// as nothing overflows.  After the first 32 keys have set m, the common path therefore
// skips the max search and only checks that the row sums stay below 2^40 (2^15 for halves,
// whose largest finite value is 65504); a wave that sees
// a larger sum (scores far above everything before) redoes that step on the general path,
// which raises m and rescales O and l.
//
// MFMA layouts used (v_mfma_f32_32x32x16_bf16 / _f16, A is 32xK, B is Kx32, K = 16):
//   A: lane l holds row l % 32, contraction indices 8*(l/32) .. 8*(l/32)+7
//   B: lane l holds column l % 32, same contraction indices
//   C/D: lane l, register r holds row 8*(r/4) + 4*(l/32) + r%4, column l % 32
// Only the C/D layout and the pairing of contraction slices between A and B matter.
// ds_read_b64_tr_b16, per block of 16 lanes: lane L receives element L%4 of the four
// 8-byte pieces addressed by lanes L/4, L/4+4, L/4+8, L/4+12 of its block.
#include <type_traits>

#include "ls_internal.hpp"

namespace ls {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));  // also carries eight IEEE halves as bit patterns
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int TK = 64;              // keys per LDS stage
constexpr int SUB = 32;             // keys per softmax step (one MFMA row tile)
constexpr float kLazy = 8.f;        // general path: m is raised only when a score exceeds it by 2^8
// common path: largest row-sum increment taken without raising m; the numerators are stored in
// the operand type, and a half holds nothing above 65504
template <bool F16> constexpr float kSumCap = F16 ? 0x1p15f : 0x1p40f;

#define LS_LDS(p) ((__attribute__((address_space(3))) void *)(p))

template <bool F16> __device__ __forceinline__ floatx16 mfma32(bf16x8 a, bf16x8 b, floatx16 c)
{
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, a), __builtin_bit_cast(halfx8, b), c,
                                                      0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// two floats to one register of the operand type, round to nearest even
template <bool F16> __device__ __forceinline__ uint32_t pack16(float lo, float hi)
{
    floatx2 f = {lo, hi};
    if constexpr (F16) {
        typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, halfx2));
    } else {
        bf16x2 b = __builtin_convertvector(f, bf16x2);
        return __builtin_bit_cast(uint32_t, b);
    }
}
// the softmax numerators: one instruction per pair in either type (halves round toward zero,
// a bias of 2^-12 of the value that the fp32 row sums do not share; far below the output's
// own rounding)
template <bool F16> __device__ __forceinline__ uint32_t pack_numerators(float lo, float hi)
{
    if constexpr (F16) return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
    else return pack16<false>(lo, hi);
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

// One 64-lane HBM -> LDS copy: lane l moves 16 bytes from base + voff[l] to LDS byte
// lds_base + 16*l (base and lds_base wave-uniform; lds_base goes through M0).  Written as
// inline assembly so that the compiler does not serialise later LDS reads behind all copies
// still in flight; the kernel orders reads after copies itself with wait_vmem + a barrier.
__device__ __forceinline__ void copy_to_lds(const uint8_t *base, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voff), "s"(base)
                 : "memory");
}

__device__ __forceinline__ const uint8_t *uniform_ptr(const uint8_t *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const uint8_t *)(((uint64_t)hi << 32) | lo);
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

template <int D, int NW, int NS, bool F16>
__global__ void __launch_bounds__(NW * 64)
prefix_mfma_kernel(Problem p, SplitPlan plan, Partials out, MaskJob mask_job, int32_t n_qblocks)
{
    constexpr int KSTEPS = D / 16;            // contraction steps of S^T = K Q^T
    constexpr int MT = D / 32;                // 32-row tiles of O^T along head_dim
    constexpr int CH = D / 8;                 // 16-byte chunks per K/V row
    constexpr int ROWB = D * 2;               // bytes per K/V row
    constexpr int TILEB = TK * ROWB;          // bytes per K (or V) tile
    constexpr int STAGEB = 2 * TILEB;         // K tile then V tile
    constexpr int ROWS_PER_LOAD = 64 / CH;    // rows one 64-lane load instruction covers
    constexpr int LOADS = TK / NW / ROWS_PER_LOAD;  // load instructions per wave, tile and tensor
    static_assert(LOADS >= 1 && TK % (NW * ROWS_PER_LOAD) == 0, "tile rows must divide over the waves");
    static_assert(NS >= 2 && NS <= 4, "ring depth");
    constexpr int INFLIGHT = 2 * LOADS;       // vmem instructions per wave and stage
    static_assert((NS - 1) * INFLIGHT <= 63, "the vmcnt counter holds at most 63 outstanding loads");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int tid = threadIdx.x;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int li = lane & 31;
    const int lh = lane >> 5;

    // Linear workgroup index: key split fastest, then query block, then (sequence, KV head).
    // Workgroups past that range (one per sequence, present only in the whole-path launch)
    // build the tree mask, which the kernel that follows this one consumes.
    // Per (sequence, KV head): the full query blocks, n_splits workgroups each, then (if it is cut
    // differently) the last, light query block with rem_splits workgroups.
    const int n_qb_even = plan.rem_splits ? n_qblocks - 1 : n_qblocks;
    const int per_unit = n_qb_even * plan.n_splits + plan.rem_splits;
    const int n_main = per_unit * p.batch * p.n_kv_heads;
    if ((int)blockIdx.x >= n_main) {
        const int mb = blockIdx.x - n_main;
        const int words = (p.n_tree + 63) >> 6;
        build_tree_mask_rows(mask_job.parents + (size_t)mb * p.n_tree, p.n_tree,
                             mask_job.mask + (size_t)mb * p.n_tree * words,
                             mask_job.err_flag ? mask_job.err_flag + mb : nullptr, tid, (int)blockDim.x);
        return;
    }
    const int bz = blockIdx.x / per_unit;
    const int in_unit = blockIdx.x % per_unit;
    const bool light = in_unit >= n_qb_even * plan.n_splits;
    const int split = light ? in_unit - n_qb_even * plan.n_splits : in_unit % plan.n_splits;
    const int qblock = light ? n_qb_even : in_unit / plan.n_splits;
    const int split_len = light ? plan.rem_split_len : plan.split_len;
    const int b = bz / p.n_kv_heads;
    const int g = bz % p.n_kv_heads;
    const int rows_kv = p.group * p.n_tree;

    int plen = p.prefix_lens ? p.prefix_lens[b] : p.prefix_len_all;
    plen = plen < 0 ? 0 : (plen > p.max_prefix_len ? p.max_prefix_len : plen);
    const int k_lo = split * split_len;
    int k_hi = k_lo + split_len;
    k_hi = k_hi > plen ? plen : k_hi;

    // The query row of this lane.
    const int m_row = (qblock * NW + wave) * 32 + li;
    const bool q_ok = m_row < rows_kv;
    const int hq = g * p.group + (q_ok ? m_row / p.n_tree : 0);
    const int ti = q_ok ? m_row % p.n_tree : 0;
    const size_t part_row = out.row((size_t)b * p.n_q_heads + hq, split, p.n_tree, ti);

    if (light && split == 0 && lh == 0 && q_ok) {  // the parts this query block does not produce
        for (int s = plan.rem_splits; s < plan.n_splits; ++s)
            out.lse[out.row((size_t)b * p.n_q_heads + hq, s, p.n_tree, ti)] = -INFINITY;
    }
    if (k_lo >= k_hi) {  // empty split: weight zero in the merge
        if (lh == 0 && q_ok) out.lse[part_row] = -INFINITY;
        return;
    }

    // Q^T as the B operand, kept in registers for the whole split.  The loads are issued here
    // and collected after the first key tiles have been requested; they are inline assembly so
    // that no compiler-placed wait for them lands inside the key loop, where it would also
    // wait for every key tile still in flight.
    const uint16_t *q_ptr = (const uint16_t *)p.q + b * p.q_stride[0] + hq * p.q_stride[1] + ti * p.q_stride[2];
    u32x4 q_raw[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk)
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(q_raw[kk]) : "v"(q_ptr + kk * 16 + lh * 8) : "memory");

    // ---- HBM -> LDS tile loads ----------------------------------------------------------
    const uint8_t *kbase = uniform_ptr((const uint8_t *)p.k_cache + (b * p.kc_stride[0] + g * p.kc_stride[1]) * 2);
    const uint8_t *vbase = uniform_ptr((const uint8_t *)p.v_cache + (b * p.vc_stride[0] + g * p.vc_stride[1]) * 2);
    const int64_t k_row_bytes = p.kc_stride[2] * 2, v_row_bytes = p.vc_stride[2] * 2;
    const int ld_row = lane / CH;  // row within one load instruction
    const int ld_pos = lane % CH;  // LDS chunk position this lane fills
    const uint32_t smem_off = lds_offset(smem);
    // byte offsets of this lane's pieces relative to the first row of a tile (whole tiles)
    uint32_t k_voff[LOADS], v_voff[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int row = (wave * LOADS + j) * ROWS_PER_LOAD + ld_row;
        k_voff[j] = (uint32_t)(row * k_row_bytes) + (ld_pos ^ (row & (CH - 1))) * 16;
        v_voff[j] = (uint32_t)(row * v_row_bytes) + (ld_pos ^ (vswz(row) & (CH - 1))) * 16;
    }
    // Paged cache: the ids of the pages this split touches, page (first_page + 64 j + l) in lane
    // l of register j; a tile request then finds its pages with register reads only.
    const bool paged = p.block_table != nullptr;
    const int page_rows_mask = (1 << p.page_shift) - 1;
    const int first_page = k_lo >> p.page_shift;
    uint32_t page_tab[kMaxSplitPages / 64] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (paged) {
        const int32_t *tab = p.block_table + (size_t)b * p.bt_stride;
#pragma unroll
        for (int j = 0; j < kMaxSplitPages / 64; ++j) {
            const int idx = first_page + 64 * j + lane;
            page_tab[j] = idx < p.bt_stride ? (uint32_t)tab[idx] : 0u;
        }
    }
    auto page_of = [&](int row) -> int64_t {  // row: wave-uniform cache row of this sequence
        const int pidx = (row >> p.page_shift) - first_page;
        const int sel = pidx & 63;
        uint32_t id = __builtin_amdgcn_readlane(page_tab[0], sel);
#pragma unroll
        for (int j = 1; j < kMaxSplitPages / 64; ++j)
            if ((pidx >> 6) == j) id = __builtin_amdgcn_readlane(page_tab[j], sel);
        return (int64_t)id;
    };
    // One load instruction covers ROWS_PER_LOAD consecutive rows, which never straddle a page
    // (page sizes are powers of two >= 16): its base is that of its own page.
    auto issue_tile_paged = [&](int k0, int stage) {
        const uint32_t ks_off = __builtin_amdgcn_readfirstlane(smem_off + stage * STAGEB);
        const int last = k_hi - 1 - k0;  // last valid row of the tile (>= TK - 1 for whole tiles)
#pragma unroll
        for (int j = 0; j < LOADS; ++j) {
            const int row0 = (wave * LOADS + j) * ROWS_PER_LOAD;  // wave-uniform
            // rows past the end of the split repeat its last row, fetched through that row's own group
            const int last_group = last & ~(ROWS_PER_LOAD - 1);
            const int src0 = row0 < last_group ? row0 : last_group;
            const int row = row0 + ld_row;
            int src = src0 + ld_row;
            src = src < last ? src : last;
            const int abs0 = k0 + src0;
            const int64_t page = page_of(abs0);
            const int in_page = abs0 & page_rows_mask;
            const uint8_t *kb = uniform_ptr((const uint8_t *)p.k_cache +
                                            (page * p.kc_stride[0] + g * p.kc_stride[1] + in_page * p.kc_stride[2]) * 2);
            const uint8_t *vb = uniform_ptr((const uint8_t *)p.v_cache +
                                            (page * p.vc_stride[0] + g * p.vc_stride[1] + in_page * p.vc_stride[2]) * 2);
            const uint32_t ko = (uint32_t)((src - src0) * k_row_bytes) + (ld_pos ^ (row & (CH - 1))) * 16;
            const uint32_t vo = (uint32_t)((src - src0) * v_row_bytes) + (ld_pos ^ (vswz(row) & (CH - 1))) * 16;
            copy_to_lds(kb, ko, ks_off + row0 * ROWB);
            copy_to_lds(vb, vo, ks_off + TILEB + row0 * ROWB);
        }
    };
    auto issue_tile = [&](int k0, int stage) {
        if (paged) {
            issue_tile_paged(k0, stage);
            return;
        }
        const uint32_t ks_off = __builtin_amdgcn_readfirstlane(smem_off + stage * STAGEB);
        const uint8_t *kt_base = uniform_ptr(kbase + k0 * k_row_bytes);
        const uint8_t *vt_base = uniform_ptr(vbase + k0 * v_row_bytes);
        if (k0 + TK <= k_hi) {
#pragma unroll
            for (int j = 0; j < LOADS; ++j) {
                const int row0 = (wave * LOADS + j) * ROWS_PER_LOAD;  // wave-uniform
                copy_to_lds(kt_base, k_voff[j], ks_off + row0 * ROWB);
                copy_to_lds(vt_base, v_voff[j], ks_off + TILEB + row0 * ROWB);
            }
        } else {
            // ragged last tile: rows past the end repeat the last valid row; their scores are masked
#pragma unroll
            for (int j = 0; j < LOADS; ++j) {
                const int row0 = (wave * LOADS + j) * ROWS_PER_LOAD;
                const int row = row0 + ld_row;
                const int last = k_hi - 1 - k0;
                const int src = row < last ? row : last;
                const uint32_t ko = (uint32_t)(src * k_row_bytes) + (ld_pos ^ (row & (CH - 1))) * 16;
                const uint32_t vo = (uint32_t)(src * v_row_bytes) + (ld_pos ^ (vswz(row) & (CH - 1))) * 16;
                copy_to_lds(kt_base, ko, ks_off + row0 * ROWB);
                copy_to_lds(vt_base, vo, ks_off + TILEB + row0 * ROWB);
            }
        }
    };

    // Tiles requested ahead of the one being consumed: the V half of a tile is still read one
    // step after its keys were scored (see the pipeline below), so of the NS stages one holds
    // that tile, one the current tile and PD = NS - 2 are in flight.
    constexpr int PD = NS - 2;
    static_assert(PD >= 1 && PD <= 2, "prefetch distance");
    const int n_tiles = (k_hi - k_lo + TK - 1) / TK;
    const int n_prologue = n_tiles < PD ? n_tiles : PD;
    // Tile order: the softmax does not care in which order keys arrive, so split s starts at
    // its tile (s mod n_tiles) and wraps around.  All workgroups start together; with every
    // split reading from its first row their addresses would differ by multiples of the split
    // size only and crowd a few memory channels.
    const int rot = split % n_tiles;
    auto tile_k0 = [&](int t) {
        int tt = t + rot;
        tt = tt >= n_tiles ? tt - n_tiles : tt;
        return k_lo + tt * TK;
    };
#pragma unroll
    for (int s = 0; s < PD; ++s)
        if (s < n_prologue) issue_tile(tile_k0(s), s);

    // collect Q: everything older than the prologue tiles has landed
    if (PD >= 2 && n_prologue == 2) wait_vmem<(PD >= 2 ? 2 : 1) * INFLIGHT>();
    else wait_vmem<INFLIGHT>();
    bf16x8 q_reg[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        asm volatile("" : "+v"(q_raw[kk]));  // orders every use below after the wait above
        const u32x4 v = q_ok ? q_raw[kk] : u32x4{0, 0, 0, 0};
        q_reg[kk] = __builtin_bit_cast(bf16x8, v);
    }

    floatx16 o_acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[mt][r] = 0.f;
    float m_run = -INFINITY;  // reference exponent in raw-score units (see the header comment)
    float l_run = 0.f;        // sum of the numerators over this lane's keys only
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

    // ---- building blocks of the pipeline -----------------------------------------------------
    auto wait_tile = [&](int t) {  // this wave's copies of tile t have landed
        const int younger = n_tiles - 1 - t < PD - 1 ? n_tiles - 1 - t : PD - 1;
        if (PD >= 2 && younger >= 1) wait_vmem<(PD >= 2 ? 1 : 0) * INFLIGHT>();
        else wait_vmem<0>();
    };
    auto fetch_k = [&](const uint8_t *ktile, int kt, bf16x8 (&kf)[KSTEPS]) {
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int pos = (2 * kk + lh) ^ k_swz;
            kf[kk] = __builtin_bit_cast(bf16x8, *(const uint4 *)(ktile + kt * SUB * ROWB + k_lane_off + pos * 16));
        }
    };
    auto fetch_v = [&](const uint8_t *vtile, int kt, bf16x8 (&vf)[2][MT]) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const uint8_t *vp = vtile + (kt * SUB + a * 16) * ROWB + v_lane_off[mt];
                const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) shortx4 *)LS_LDS(vp));
                const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) shortx4 *)LS_LDS(vp + 8 * ROWB));
                const uint2 lo2 = __builtin_bit_cast(uint2, lo), hi2 = __builtin_bit_cast(uint2, hi);
                vf[a][mt] = __builtin_bit_cast(bf16x8, make_uint4(lo2.x, lo2.y, hi2.x, hi2.y));
            }
    };
    auto score = [&](const bf16x8 (&kf)[KSTEPS]) {  // S^T = K Q^T for 32 keys
        floatx16 s_acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) s_acc = mfma32<F16>(kf[kk], q_reg[kk], s_acc);
        return s_acc;
    };
    auto second_product = [&](const bf16x8 (&vf)[2][MT], const uint32_t (&pp)[8]) {  // O^T += V^T P^T
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const bf16x8 pb =
                __builtin_bit_cast(bf16x8, make_uint4(pp[4 * a], pp[4 * a + 1], pp[4 * a + 2], pp[4 * a + 3]));
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) o_acc[mt] = mfma32<F16>(vf[a][mt], pb, o_acc[mt]);
        }
    };
    auto mask_tail = [&](floatx16 &s_acc, int key0) {  // keys past the end of the split weigh nothing
        if (key0 + SUB > k_hi) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (key >= k_hi) s_acc[r] = -INFINITY;
            }
        }
    };
    auto numerators = [&](const floatx16 &s_acc, uint32_t (&pp)[8]) {  // with the current m_run
        const float mc = m_run == -INFINITY ? 0.f : m_run * c;
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = __builtin_amdgcn_exp2f(s_acc[r] * c - mc);
            const float p1 = __builtin_amdgcn_exp2f(s_acc[r + 1] * c - mc);
            pp[r >> 1] = pack_numerators<F16>(p0, p1);
            sum += p0 + p1;
        }
        return sum;
    };
    auto raise_reference = [&](const floatx16 &s_acc) {  // general path: lift m_run, rescale O and l
        float mx = s_acc[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s_acc[r]);
        mx = half_max(mx);
        const bool grow = (mx - m_run) * c > kLazy;  // also true while m_run is -inf
        if (__any(grow)) {
            const float m_new = fmaxf(m_run, mx);
            // a step whose keys are all masked leaves m_new = -inf; keep arithmetic finite
            const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f((m_run - m_new) * c);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[mt][r] *= alpha;
        }
    };

    // ---- software pipeline over 32-key steps --------------------------------------------------
    // Step j scores keys, turns scores into numerators and adds their weighted values to O.
    // One pipeline block handles three independent pieces of neighbouring steps: the output
    // product of step j-1 (matrix core), the softmax arithmetic of step j (vector ALU) and the
    // score product of step j+1 (matrix core).  Every block thus carries 16 matrix instructions
    // next to its vector work, for this wave and for the one sharing its SIMD alike.
    bf16x8 k_frag[KSTEPS];
    bf16x8 v_frag[2][MT];
    uint32_t p_prev[8];
    floatx16 s_cur;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) v_frag[a][mt] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < 8; ++r) p_prev[r] = 0;  // the first block's output product adds zero

    wait_tile(0);
    __syncthreads();
    if (PD < n_tiles) issue_tile(tile_k0(PD), PD % NS);
    // A wave whose 32 rows all lie past the last query row of the KV head (the last query block
    // of a head whose row count is not a multiple of the block) only keeps feeding the ring:
    // its share of every tile, and every barrier of the loop below.
    if ((qblock * NW + wave) * 32 >= rows_kv) {
        for (int t = 0; t + 1 < n_tiles; ++t) {
            wait_tile(t + 1);
            __syncthreads();
            if (t + 1 + PD < n_tiles) issue_tile(tile_k0(t + 1 + PD), (t + 1 + PD) % NS);
        }
        return;
    }
    fetch_k(smem, 0, k_frag);
    s_cur = score(k_frag);
    mask_tail(s_cur, tile_k0(0));
    raise_reference(s_cur);  // sets m_run from the first 32 keys (at least one of them is valid)

    // one block: consumes s_cur / p_prev / v_frag, leaves the next step's in their place
    auto block = [&](auto has_next_tag, const uint8_t *k_next, int kt_next, const uint8_t *v_cur, int kt_cur,
                     int key0_next) {
        constexpr bool has_next = decltype(has_next_tag)::value;
        if constexpr (has_next) fetch_k(k_next, kt_next, k_frag);
        uint32_t p_cur[8];
        floatx16 s_next = s_cur;
        if constexpr (has_next) {
            // output-product and score MFMAs alternate, so that no matrix instruction depends on
            // the one issued just before it
            bf16x8 pb[2];
#pragma unroll
            for (int a = 0; a < 2; ++a)
                pb[a] = __builtin_bit_cast(bf16x8, make_uint4(p_prev[4 * a], p_prev[4 * a + 1], p_prev[4 * a + 2],
                                                              p_prev[4 * a + 3]));
#pragma unroll
            for (int r = 0; r < 16; ++r) s_next[r] = 0.f;
#pragma unroll
            for (int i = 0; i < KSTEPS; ++i) {
                o_acc[i % MT] = mfma32<F16>(v_frag[i / MT][i % MT], pb[i / MT], o_acc[i % MT]);
                s_next = mfma32<F16>(k_frag[i], q_reg[i], s_next);
            }
        } else {
            second_product(v_frag, p_prev);
        }
        float sum = numerators(s_cur, p_cur);
        fetch_v(v_cur, kt_cur, v_frag);
        if (__any(!(sum < kSumCap<F16>))) {  // also catches inf and nan: redo this step on the general path
            raise_reference(s_cur);
            sum = numerators(s_cur, p_cur);
        }
        l_run += sum;
#pragma unroll
        for (int r = 0; r < 8; ++r) p_prev[r] = p_cur[r];
        if constexpr (has_next) mask_tail(s_next, key0_next);
        s_cur = s_next;
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;

    for (int t = 0; t + 1 < n_tiles; ++t) {
        const uint8_t *ks = smem + (t % NS) * STAGEB;
        const uint8_t *vs = ks + TILEB;
        const int k0 = tile_k0(t);
        // first half of tile t: the next step is the second half of the same tile
        block(yes{}, ks, 1, vs, 0, k0 + SUB);
        // second half: the next step opens tile t+1, which needs the barrier
        wait_tile(t + 1);
        __syncthreads();  // tile t+1 is complete in LDS; nobody reads tile t-1 any more
        if (t + 1 + PD < n_tiles) issue_tile(tile_k0(t + 1 + PD), (t + 1 + PD) % NS);
        block(yes{}, smem + ((t + 1) % NS) * STAGEB, 0, vs, 1, tile_k0(t + 1));
    }
    {  // the last tile: its second half has no successor
        const int t = n_tiles - 1;
        const uint8_t *ks = smem + (t % NS) * STAGEB;
        const uint8_t *vs = ks + TILEB;
        block(yes{}, ks, 1, vs, 0, tile_k0(t) + SUB);
        block(no{}, ks, 0, vs, 1, 0);
    }
    second_product(v_frag, p_prev);  // the output product of the last step

    // ---- epilogue: normalise and store this split's partial result -----------------------
    const float l_tot = half_sum(l_run);
    const float inv = 1.f / l_tot;
    if (out.o_is_16bit) {
        // A lane holds 4-element runs of one query row, 256 bytes apart from its neighbours':
        // stored as they are, every store instruction would touch 32 rows with 16 bytes each.
        // The rows go through LDS instead and leave as whole rows, 16 bytes per lane.  The
        // two ring stages after the last tile's are free: no tile was requested into them any
        // more, and every wave has passed the barrier after which their old tiles were dead.
        // Each wave owns a quarter of a stage, so no barrier is needed.
        const int t_last = n_tiles - 1;
        uint8_t *mine = smem + ((t_last + 1 + wave / 4) % NS) * STAGEB + (wave % 4) * (32 * ROWB);
        static_assert(STAGEB == 4 * 32 * ROWB && NW <= 8 && NS >= 4, "four waves stage their rows in one ring stage");
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                uint2 v;
                v.x = pack16<F16>(o_acc[mt][4 * rg + 0] * inv, o_acc[mt][4 * rg + 1] * inv);
                v.y = pack16<F16>(o_acc[mt][4 * rg + 2] * inv, o_acc[mt][4 * rg + 3] * inv);
                const int chunk = (4 * mt + rg) ^ (li & (CH - 1));
                *(uint2 *)(mine + li * ROWB + chunk * 16 + lh * 8) = v;
            }
        // the row index and validity of query row r live in lane r
        const uint32_t my_row = (uint32_t)part_row;
        constexpr int ROWS_PER_STORE = 64 / CH;
#pragma unroll
        for (int j = 0; j < 32 / ROWS_PER_STORE; ++j) {
            const int r = j * ROWS_PER_STORE + lane / CH;
            const int cpos = lane % CH;
            const uint4 v = *(const uint4 *)(mine + r * ROWB + ((cpos ^ (r & (CH - 1))) * 16));
            const uint32_t prow = __shfl(my_row, r);
            const int ok = __shfl((int)q_ok, r);
            // streaming stores: whole rows that nobody on this compute unit reads again; they leave
            // the L2 as they are written instead of in one burst when the kernel ends
            if (ok)
                __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w},
                                            (u32x4 *)((uint16_t *)out.o + (size_t)prow * D + cpos * 8));
        }
        if (!q_ok) return;
    } else {
        if (!q_ok) return;
        float *orow = (float *)out.o + part_row * D;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                float4 v;
                v.x = o_acc[mt][4 * rg + 0] * inv;
                v.y = o_acc[mt][4 * rg + 1] * inv;
                v.z = o_acc[mt][4 * rg + 2] * inv;
                v.w = o_acc[mt][4 * rg + 3] * inv;
                *(float4 *)(orow + mt * 32 + 8 * rg + 4 * lh) = v;
            }
    }
    if (lh == 0) out.lse[part_row] = (m_run * c + log2f(l_tot)) * kLn2;
}

bool prefix_mfma_supports(const Problem &p, int dtype)
{
    // the tile loads address rows of one tile with 32-bit byte offsets
    const int64_t max_row_bytes = 2 * (p.kc_stride[2] > p.vc_stride[2] ? p.kc_stride[2] : p.vc_stride[2]);
    return is_16bit(dtype) && (p.head_dim == 128 || p.head_dim == 64) && max_row_bytes * TK < (1ll << 31);
}

namespace {

template <int D, int NW, int NS, bool F16>
hipError_t launch_one(const Problem &p, const SplitPlan &plan, const Partials &out, const MaskJob &mask_job,
                      hipStream_t stream)
{
    constexpr int lds_bytes = NS * 2 * TK * D * 2;
    static_assert(lds_bytes <= 160 * 1024, "LDS ring exceeds the 160 KB of a compute unit");
    auto kernel = prefix_mfma_kernel<D, NW, NS, F16>;
    static hipError_t attr = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 lds_bytes);
    if (attr != hipSuccess) return attr;
    const int rows_kv = p.group * p.n_tree;
    const int rows_wg = NW * 32;
    const int n_qblocks = (rows_kv + rows_wg - 1) / rows_wg;
    if (plan.rem_splits < 0 || plan.rem_splits > plan.n_splits || (plan.rem_splits && n_qblocks < 2))
        return hipErrorInvalidValue;
    const int64_t per_unit = (int64_t)plan.n_splits * (plan.rem_splits ? n_qblocks - 1 : n_qblocks) + plan.rem_splits;
    const int64_t n_main = per_unit * p.batch * p.n_kv_heads;
    const int64_t n_blocks = n_main + (mask_job.parents ? p.batch : 0);
    if (n_blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kernel, dim3((unsigned)n_blocks), dim3(NW * 64), lds_bytes, stream, p, plan, out, mask_job,
                       n_qblocks);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_prefix_mfma(const Problem &p, int dtype, const SplitPlan &plan, const Partials &out,
                              const MaskJob &mask_job, hipStream_t stream)
{
    const int rows_kv = p.group * p.n_tree;
    const bool f16 = dtype == LS_F16;
#define LS_MFMA_CASE(DD, WW)                                                              \
    (f16 ? launch_one<DD, WW, 4, true>(p, plan, out, mask_job, stream)                   \
         : launch_one<DD, WW, 4, false>(p, plan, out, mask_job, stream))
    if (p.head_dim == 128) return rows_kv > 128 ? LS_MFMA_CASE(128, 8) : LS_MFMA_CASE(128, 4);
    if (p.head_dim == 64) return rows_kv > 128 ? LS_MFMA_CASE(64, 8) : LS_MFMA_CASE(64, 4);
#undef LS_MFMA_CASE
    return hipErrorInvalidValue;
}

}  // namespace ls
