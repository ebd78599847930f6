// Split-KV attention over the cached keys on the 16-bit matrix cores (gfx950 MFMA; bf16 or
// IEEE half inputs, selected by the template flag F16, fp32 accumulation either way).
// Step (b) of the path: per key split, o_cache and LSE_cache of the aggregation appendix.
//
// Work decomposition.  All G*T query rows that share a KV head (G query heads x T tree
// tokens) form one dense query tile, so every cached K/V row is fetched from HBM once per
// KV head.  A workgroup owns (sequence, KV head, key split, block of up to NW*32 query rows);
// each of its NW waves owns 32 query rows and all keys of the split.  With NW = 8 two waves
// share a SIMD (256 registers per lane each), so that one wave's matrix instructions overlap
// the other's vector work; one workgroup per compute unit, so that all of the LDS is one deep
// ring of key tiles.
//
// Data movement.  K and V rows go HBM -> LDS directly (global_load_lds_dwordx4, 16 bytes
// per lane, no staging registers) in tiles of 32 keys.  K tiles and V tiles have rings of
// their own, because a tile's V rows are read two pipeline steps after its K rows: they are
// requested one step later than its K rows, and still arrive a step earlier than needed.  With
// PD requests in flight, issued two at a time (one workgroup barrier per two tiles), the K ring
// has PD + 3 stages and the V ring PD + 4 (PD = 6: 152 KB at head_dim 128; PD = 3: 104 KB): what a
// compute unit has in flight is what hides the HBM latency.  The instruction writes LDS
// linearly (lane l -> base + 16*l), so the bank swizzle is applied on the global side:
// the lane that fills LDS slot (row, pos) fetches chunk pos ^ swizzle(row) of that row.
//
// Each split walks its tiles starting at tile (split index mod tile count) and wraps around:
// all workgroups start together, and without this their addresses would differ only by
// multiples of the split size and crowd a few memory channels.
//
// Paged caches: a load instruction covers 4 or 8 consecutive rows, which a page of 16 rows
// or more never splits, so each instruction takes the base of its own page; the page ids of
// the split are read once into LDS behind the rings, and a tile request picks its pages from
// there.
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
#include "ls_tail.hpp"


namespace ls {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));  // also carries eight IEEE halves as bit patterns
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int TK = 32;              // keys per tile = keys per pipeline step (one MFMA row tile)
// PD, a template parameter of the kernel: requests (a K tile and a V tile each) in flight.  The K
// ring has PD + 3 stages, the V ring PD + 4.  Short splits take PD = 6: nearly all their tiles are
// requested at once and arrive while the first ones are worked on.  Long splits take PD = 3: a
// compute unit's share of the HBM stream fills a window of 13 tiles in about 6 us, during which
// nothing is computed, and three requests in flight are as many as the memory pipeline of a
// compute unit holds anyway.
constexpr int kDeepRequests = 6, kShallowRequests = 3;
constexpr int kDeepMaxTiles = 16;   // splits of at most this many tiles take the deep window
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
// M0 cannot be named as clobbered (the compiler ignores reserved registers in a clobber list and
// warns); it writes M0 itself only for instructions this file does not contain, which the test
// suite checks on the generated assembly (every M0 access belongs to one of these copies).
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

template <int D, int NW, bool F16, bool PAGED, int PD>
__global__ void __launch_bounds__(NW * 64, 2048 / (NW * 64) / 4)  // at most 256 registers per lane: no AGPR copies
prefix_mfma_kernel(Problem p, SplitPlan plan, Partials out, MaskJob mask_job, FusedTail tail, int32_t n_qblocks)
{
    constexpr int KS = PD + 3;                // stages of the K ring
    constexpr int VS = PD + 4;                // stages of the V ring
    constexpr int KSTEPS = D / 16;            // contraction steps of S^T = K Q^T
    constexpr int MT = D / 32;                // 32-row tiles of O^T along head_dim
    constexpr int CH = D / 8;                 // 16-byte chunks per K/V row
    constexpr int ROWB = D * 2;               // bytes per K/V row
    constexpr int TILEB = TK * ROWB;          // bytes per K (or V) tile
    constexpr int ROWS_PER_LOAD = 64 / CH;    // rows one 64-lane load instruction covers
    constexpr int TPT = TK / ROWS_PER_LOAD;   // load instructions per tile and tensor
    // The first NL waves do all the copying.  With two waves per SIMD these are the older ones,
    // which the hardware serves first: they reach every barrier early and have the time.
    constexpr int NL = 4;
    constexpr int LOADS = TPT / NL;           // load instructions per loader wave, tile and tensor
    constexpr int INFLIGHT = 2 * LOADS;       // vmem instructions per loader wave and whole request
    constexpr uint32_t V_RING = KS * TILEB;   // LDS byte offset of the V ring
    static_assert(LOADS >= 1 && TPT % NL == 0 && NL <= NW, "tile rows must divide over the loader waves");
    static_assert((PD + 1) * INFLIGHT <= 63, "the vmcnt counter holds at most 63 outstanding loads");
    static_assert(NW * 32 * ROWB <= (KS + VS) * TILEB, "the partial rows are staged in the rings at the end");

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    const int tid = threadIdx.x;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int li = lane & 31;
    const int lh = lane >> 5;

    // Linear workgroup index: key split fastest, then query block, then (sequence, KV head).
    // Workgroups past that range (one per sequence, present only in the whole-path launch)
    // build the tree mask, which the kernel that follows this one consumes.
    const int per_unit = n_qblocks * plan.n_splits;
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
    const int split = in_unit % plan.n_splits;
    const int qblock = in_unit / plan.n_splits;
    const int b = bz / p.n_kv_heads;
    const int g = bz % p.n_kv_heads;
    const int rows_kv = p.group * p.n_tree;

    // The split's own work (a `return` below leaves this block only; in the single-launch call
    // every wave goes on to the arrival count after it).
    [&]() __attribute__((always_inline)) {
    int plen = p.prefix_lens ? p.prefix_lens[b] : p.prefix_len_all;
    plen = plen < 0 ? 0 : (plen > p.max_prefix_len ? p.max_prefix_len : plen);
    int split_len = plan.split_len;
    if (plan.per_sequence) split_len = ((plen + plan.n_splits - 1) / plan.n_splits + TK - 1) / TK * TK;
    const int k_lo = split * split_len;
    int k_hi = k_lo + split_len;
    k_hi = k_hi > plen ? plen : k_hi;

    // The query row of this lane.
    const int wave_row0 = (qblock * NW + wave) * 32;
    const int m_row = wave_row0 + li;
    const bool q_ok = m_row < rows_kv;
    const int hq = g * p.group + (q_ok ? m_row / p.n_tree : 0);
    const int ti = q_ok ? m_row % p.n_tree : 0;
    const size_t part_row = out.row((size_t)b * p.n_q_heads + hq, split, p.n_tree, ti);

    if (k_lo >= k_hi) {  // empty split: weight zero in the merge
        if (lh == 0 && q_ok) {
            if (tail.counters == nullptr) out.lse[part_row] = -INFINITY;
            else __hip_atomic_store(out.lse + part_row, -INFINITY, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
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
    // The rows a loader wave copies: LOADS groups of ROWS_PER_LOAD rows per tensor, group j starting
    // at tile row load_row0(j).
    const bool loader = wave < NL;
    // With eight waves, the first window of tiles (requests -PD .. -1) is copied by the other four:
    // a wave that issues a whole window sits in the issue stall while the window fills, and the
    // loader waves should be through tile 0 by then.  Wave NL + i copies the rows loader i would.
    const bool starter = NW >= 2 * NL ? (wave >= NL && wave < 2 * NL) : loader;
    auto load_row0 = [&](int j) __attribute__((always_inline)) { return ((wave % NL) * LOADS + j) * ROWS_PER_LOAD; };
    // byte offsets of this lane's pieces relative to the first row of a tile (whole tiles)
    uint32_t k_voff[LOADS], v_voff[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int row = load_row0(j) + ld_row;
        k_voff[j] = (uint32_t)(row * k_row_bytes) + (ld_pos ^ (row & (CH - 1))) * 16;
        v_voff[j] = (uint32_t)(row * v_row_bytes) + (ld_pos ^ (vswz(row) & (CH - 1))) * 16;
    }
    // Paged cache: the ids of the pages this split touches sit in LDS behind the rings (page
    // first_page + i at word i); a tile request reads the ones it needs from there.
    constexpr uint32_t PAGE_TAB = (KS + VS) * TILEB;
    const int page_rows_mask = (1 << p.page_shift) - 1;
    const int first_page = k_lo >> p.page_shift;
    if constexpr (PAGED) {
        const int32_t *tab = p.block_table + (size_t)b * p.bt_stride;
        for (int i = tid; i < kMaxSplitPages; i += NW * 64) {
            const int idx = first_page + i;
            ((uint32_t *)(smem + PAGE_TAB))[i] = idx < p.bt_stride ? (uint32_t)tab[idx] : 0u;
        }
        __syncthreads();
    }
    auto page_of = [&](int row) __attribute__((always_inline)) -> int64_t {  // row: wave-uniform cache row of this sequence
        const int pidx = (row >> p.page_shift) - first_page;
        return (int64_t)__builtin_amdgcn_readfirstlane(((const uint32_t *)(smem + PAGE_TAB))[pidx]);
    };
    // Requests.  issue_rows<IS_V>(k0, tile_base, dst): this wave's LOADS copies of the K (or V) rows
    // of the tile that starts at cache row k0, to the ring stage at LDS byte offset dst.  Rows past
    // the end of the split repeat its last row; their scores are masked.
    // Paged: one load instruction covers ROWS_PER_LOAD consecutive rows, which never straddle a
    // page (page sizes are powers of two >= 16): its base is that of its own page.
    auto issue_rows = [&](auto is_v_tag, int k0, const uint8_t *tile_base, uint32_t dst, bool mine) __attribute__((always_inline)) {
        constexpr bool IS_V = decltype(is_v_tag)::value;
        if (!mine) return;  // wave-uniform
        const uint32_t d0 = __builtin_amdgcn_readfirstlane(smem_off + dst);
        const int last = k_hi - 1 - k0;  // last valid row of the tile (>= TK - 1 for whole tiles)
        const int64_t row_bytes = IS_V ? v_row_bytes : k_row_bytes;
        const int64_t *stride = IS_V ? p.vc_stride : p.kc_stride;
        const uint8_t *tensor = (const uint8_t *)(IS_V ? p.v_cache : p.k_cache);
        auto swz = [&](int row) __attribute__((always_inline)) { return (IS_V ? vswz(row) : row) & (CH - 1); };
        if constexpr (PAGED) {
#pragma unroll
            for (int j = 0; j < LOADS; ++j) {
                const int row0 = load_row0(j);  // wave-uniform
                // rows past the end repeat the last row, fetched through that row's own group
                const int last_group = last & ~(ROWS_PER_LOAD - 1);
                const int src0 = row0 < last_group ? row0 : last_group;
                const int row = row0 + ld_row;
                int src = src0 + ld_row;
                src = src < last ? src : last;
                const int abs0 = k0 + src0;
                const int64_t page = page_of(abs0);
                const int in_page = abs0 & page_rows_mask;
                const uint8_t *base = uniform_ptr(tensor + (page * stride[0] + g * stride[1] + in_page * stride[2]) * 2);
                copy_to_lds(base, (uint32_t)((src - src0) * row_bytes) + (ld_pos ^ swz(row)) * 16, d0 + row0 * ROWB);
            }
        } else {
            const uint8_t *base = tile_base;  // address of the tile's first row (contiguous caches only)
            if (last >= TK - 1) {
#pragma unroll
                for (int j = 0; j < LOADS; ++j)
                    copy_to_lds(base, IS_V ? v_voff[j] : k_voff[j], d0 + load_row0(j) * ROWB);
            } else {
#pragma unroll
                for (int j = 0; j < LOADS; ++j) {
                    const int row0 = load_row0(j);
                    const int row = row0 + ld_row;
                    const int src = row < last ? row : last;
                    copy_to_lds(base, (uint32_t)(src * row_bytes) + (ld_pos ^ swz(row)) * 16, d0 + row0 * ROWB);
                }
            }
        }
    };

    const int n_tiles = (k_hi - k_lo + TK - 1) / TK;
    // Tile order: the softmax does not care in which order keys arrive, so split s starts at
    // its tile (s mod n_tiles) and wraps around.  All workgroups start together; with every
    // split reading from its first row their addresses would differ by multiples of the split
    // size only and crowd a few memory channels.
    const int key_first = k_lo + (split % n_tiles) * TK;  // first key of tile 0
    const int key_wrap = k_lo + n_tiles * TK;
    auto next_key0 = [&](int k0) __attribute__((always_inline)) { return k0 + TK == key_wrap ? k_lo : k0 + TK; };
    auto next_k = [&](uint32_t off) __attribute__((always_inline)) { return off + TILEB == KS * TILEB ? 0u : off + TILEB; };
    auto next_v = [&](uint32_t off) __attribute__((always_inline)) {
        return off + TILEB == V_RING + VS * TILEB ? V_RING : off + TILEB;
    };
    using is_k = std::integral_constant<bool, false>;
    using is_v = std::integral_constant<bool, true>;
    // Requests, in tile order: request r (r >= -(PD+1)) is the K rows of tile r+PD+1 and the V rows
    // of tile r+PD, as far as these tiles exist; a request with both parts is INFLIGHT load
    // instructions per wave.  The state below is that of the next request.
    // (Tile addresses advance by a fixed step and start over where the tile order wraps around.)
    const uint8_t *const k_ptr_lo = uniform_ptr(kbase + k_lo * k_row_bytes), *const v_ptr_lo = uniform_ptr(vbase + k_lo * v_row_bytes);
    int rq_kt = 0, rq_k0 = key_first, rq_vt = 0, rq_v0 = key_first;
    const uint8_t *rq_kptr = uniform_ptr(kbase + key_first * k_row_bytes), *rq_vptr = uniform_ptr(vbase + key_first * v_row_bytes);
    uint32_t rq_koff = 0, rq_voff = V_RING;
    // (mine: this wave is among those that copy this request; every wave keeps the state)
    auto request_k = [&](bool mine) __attribute__((always_inline)) {
        if (rq_kt < n_tiles) issue_rows(is_k{}, rq_k0, rq_kptr, rq_koff, mine);
        ++rq_kt;
        rq_k0 = next_key0(rq_k0);
        rq_kptr = rq_k0 == k_lo ? k_ptr_lo : rq_kptr + TK * k_row_bytes;
        rq_koff = next_k(rq_koff);
    };
    auto request_v = [&](bool mine) __attribute__((always_inline)) {
        if (rq_vt < n_tiles) issue_rows(is_v{}, rq_v0, rq_vptr, rq_voff, mine);
        ++rq_vt;
        rq_v0 = next_key0(rq_v0);
        rq_vptr = rq_v0 == k_lo ? v_ptr_lo : rq_vptr + TK * v_row_bytes;
        rq_voff = next_v(rq_voff);
    };
    request_k(loader);  // request -(PD+1)
#pragma unroll
    for (int r = -PD; r < 0; ++r) {
        request_k(starter);
        request_v(starter);
    }

    // Collect Q and the K rows of tile 0: everything older than requests -PD .. -1 has landed.
    // (A wave that copies nothing has only its Q loads outstanding.)
    // (With eight waves a loader has only Q and tile 0 outstanding and waits for all of it; a
    // starter has its Q loads in front of its PD requests.)
    if (starter && n_tiles > PD) wait_vmem<PD * INFLIGHT>();
    else wait_vmem<0>();  // short split: its requests are not all whole; wait for everything
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
        for (int e = 0; e < 16; ++e) o_acc[mt][e] = 0.f;
    float m_run = -INFINITY;  // reference exponent in raw-score units (see the header comment)
    float l_run = 0.f;        // sum of the numerators over this lane's keys only
    const float c = p.scale_log2;

    // Per-lane LDS addresses of the operand reads for a tile at ring offset 0 (the base of the
    // dynamic LDS is a multiple of 256 and is included).
    // K fragment kk: row li, chunk (2 kk + lh) under the row's swizzle, i.e. at chunk position
    // (2 kk + lh) ^ (li & (CH-1)); the chunk field of the offset is therefore k_off0 ^ (kk << 5).
    // V fragments alike: d tile mt moves the chunk position by mt << 2, i.e. v_off0 ^ (mt << 6).
    const uint32_t k_off0 = smem_off + li * ROWB + ((lh ^ (li & (CH - 1))) * 16);
    const int tr_s = lane & 15;                    // lane within its 16-lane transpose block
    const int tr_row = 4 * lh + (tr_s >> 2);       // key row (within a 16-key step) this lane addresses
    const int tr_dchunk = 2 * ((lane >> 4) & 1) + ((tr_s & 3) >> 1);  // 16-byte chunk within a 32-wide d tile
    const int tr_sub = (tr_s & 1) * 8;             // byte offset inside the chunk
    const int tr_swz = vswz(tr_row) & (CH - 1);    // rows +8, +16, ... keep row & 3
    const uint32_t v_off0 = smem_off + tr_row * ROWB + ((tr_dchunk ^ tr_swz) * 16) + tr_sub;

    // ---- building blocks of the pipeline -----------------------------------------------------
    // Workgroup barrier of the key loop, without the compiler's wait for outstanding LDS reads:
    // the stages that are written after it were last read at least a half-step before it, by
    // matrix instructions that have been issued, so those reads are complete; the reads still
    // outstanding are fragment prefetches from other stages.
    auto ring_barrier = [&]() __attribute__((always_inline)) { asm volatile("s_barrier" ::: "memory"); };
    auto mask_tail = [&](floatx16 &s_acc, int key0) __attribute__((always_inline)) {  // keys past the end of the split weigh nothing
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int key = key0 + 8 * (e >> 2) + 4 * lh + (e & 3);
            if (key >= k_hi) s_acc[e] = -INFINITY;
        }
    };
    auto numerators = [&](const floatx16 &s_acc, uint32_t (&pp)[8]) __attribute__((always_inline)) {  // with the current m_run
        const float mc = m_run == -INFINITY ? 0.f : m_run * c;
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
            const float p0 = __builtin_amdgcn_exp2f(s_acc[e] * c - mc);
            const float p1 = __builtin_amdgcn_exp2f(s_acc[e + 1] * c - mc);
            pp[e >> 1] = pack_numerators<F16>(p0, p1);
            sum += p0 + p1;
        }
        return sum;
    };
    auto raise_reference = [&](const floatx16 &s_acc) __attribute__((always_inline)) {  // general path: lift m_run, rescale O and l
        float mx = s_acc[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s_acc[e]);
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
                for (int e = 0; e < 16; ++e) o_acc[mt][e] *= alpha;
        }
    };

    // ---- software pipeline ---------------------------------------------------------------------
    // A step is one tile: 32 keys against the wave's 32 queries: a score product (KSTEPS matrix
    // instructions), the softmax arithmetic (16 scores per lane) and an output product (KSTEPS
    // matrix instructions).  Three steps are in flight, in two register slots that alternate
    // (even steps slot 0, odd steps slot 1): half-step h issues the score product of step h into
    // its slot X and the output product of step h-2 from the same slot, one matrix instruction
    // at a time, and between them the softmax arithmetic of step h-1 in the other slot.  So
    // every matrix instruction is followed by independent vector work.
    // K and V fragments rotate through FS register slots each: fragment i sits in slot i % FS and
    // is replaced, right after the matrix instruction that reads it, by fragment i + FS (of the
    // same tile, or of the next half-step's tile), FS matrix-instruction pairs before its use.
    // Scheduling barriers pin this order: left to itself the compiler hoists the LDS reads and
    // runs out of registers.
    constexpr int FS = KSTEPS / 2;
    bf16x8 k_frag[FS];
    bf16x8 v_frag[FS];
    floatx16 s_sl[2];
    uint32_t p_sl[2][8];
    float mc = 0.f;
#pragma unroll
    for (int f = 0; f < FS; ++f) v_frag[f] = k_frag[f] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int e = 0; e < 8; ++e) p_sl[x][e] = 0;  // an output product of zeros adds nothing

    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    constexpr int PPG = 8 / KSTEPS;  // score pairs of the softmax per pair of matrix instructions

    // fragment f (0 .. KSTEPS-1) of the K tile / V tile whose per-lane base is k_base / v_base
    // k_base / v_base: LDS ADDRESS (ring base included) of the lane's piece of fragment 0; fragment f
    // differs in the chunk field only, which one XOR reaches (all other terms are multiples of 256).
    typedef __attribute__((address_space(3))) const uint4 *lds_u4;
    typedef __attribute__((address_space(3))) shortx4 *lds_s4;
    auto read_k = [&](uint32_t k_base, int f) __attribute__((always_inline)) {
        return __builtin_bit_cast(bf16x8, *(lds_u4)(uintptr_t)(k_base ^ (uint32_t)(f << 5)));
    };
    auto read_v = [&](uint32_t v_base, int f) __attribute__((always_inline)) {  // f = 16-key half * MT + d tile
        const uint32_t a = (v_base ^ (uint32_t)((f % MT) << 6)) + ((f / MT) * 16) * ROWB;
        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)a);
        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(uintptr_t)(a + 8 * ROWB));
        const uint2 lo2 = __builtin_bit_cast(uint2, lo), hi2 = __builtin_bit_cast(uint2, hi);
        return __builtin_bit_cast(bf16x8, make_uint4(lo2.x, lo2.y, hi2.x, hi2.y));
    };

    // Half-step of slot X.  QK: score product of the tile at LDS offset k_cur into s_sl[X].
    // SM: softmax of s_sl[1-X] into p_sl[1-X].  The output product of p_sl[X] with the V tile at
    // v_cur always runs.  KN / VN: the next half-step has a score product (of the tile at k_next) /
    // an output product (with the tile at v_next), whose first fragments are requested here.
    auto half_step = [&](auto x_tag, auto qk_tag, auto sm_tag, auto kn_tag, auto vn_tag, uint32_t k_cur,
                         uint32_t k_next, uint32_t v_cur, uint32_t v_next) __attribute__((always_inline)) {
        constexpr int X = decltype(x_tag)::value, Y = 1 - X;
        constexpr bool QK = decltype(qk_tag)::value, SM = decltype(sm_tag)::value;
        constexpr bool KN = decltype(kn_tag)::value, VN = decltype(vn_tag)::value;
        bf16x8 pb[2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
            pb[a] = __builtin_bit_cast(bf16x8, make_uint4(p_sl[X][4 * a], p_sl[X][4 * a + 1], p_sl[X][4 * a + 2],
                                                          p_sl[X][4 * a + 3]));
        const float neg_mc = -mc;
        // tile offsets are multiples of 256, so adding them leaves the chunk field alone
        const uint32_t kc = k_cur + k_off0, kn = k_next + k_off0, vc = v_cur + v_off0, vn = v_next + v_off0;
        float sum = 0.f;
        floatx16 s_new;
#pragma unroll
        for (int e = 0; e < 16; ++e) s_new[e] = 0.f;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < KSTEPS; ++i) {
            float pe[PPG][2];
            o_acc[i % MT] = mfma32<F16>(v_frag[i % FS], pb[i / MT], o_acc[i % MT]);
            __builtin_amdgcn_sched_barrier(0);  // the V fragment is dead from here on: replace it
            if constexpr (SM) {
#pragma unroll
                for (int u = 0; u < PPG; ++u) {
                    const int e = 2 * (i * PPG + u);
                    pe[u][0] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_sl[Y][e], c, neg_mc));
                    pe[u][1] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_sl[Y][e + 1], c, neg_mc));
                }
            }
            if (i < FS) v_frag[i % FS] = read_v(vc, i + FS);
            else if constexpr (VN) v_frag[i % FS] = read_v(vn, i - FS);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (QK) s_new = mfma32<F16>(k_frag[i % FS], q_reg[i], s_new);
            __builtin_amdgcn_sched_barrier(0);  // the K fragment is dead from here on: replace it
            if constexpr (SM) {
#pragma unroll
                for (int u = 0; u < PPG; ++u) {
                    p_sl[Y][i * PPG + u] = pack_numerators<F16>(pe[u][0], pe[u][1]);
                    sum += pe[u][0] + pe[u][1];
                    // keeps the pack and the adds here (they would be sunk below the loop, and the
                    // numerators would stay live in fp32 until then)
                    asm volatile("" : "+v"(p_sl[Y][i * PPG + u]), "+v"(sum));
                }
            }
            if (i < FS) {
                if constexpr (QK) k_frag[i % FS] = read_k(kc, i + FS);
            } else if constexpr (KN) {
                k_frag[i % FS] = read_k(kn, i - FS);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (QK) s_sl[X] = s_new;
        if constexpr (SM) {
            if (__any(!(sum < kSumCap<F16>))) {  // also catches inf and nan: redo this step on the general path
                raise_reference(s_sl[Y]);
                sum = numerators(s_sl[Y], p_sl[Y]);
                mc = m_run * c;
            }
            l_run += sum;
        }
    };
    using X0 = std::integral_constant<int, 0>;
    using X1 = std::integral_constant<int, 1>;

    __syncthreads();  // the K rows of tile 0 are complete in LDS
    // Before half-step 1 (which reads K rows of tile 1): request -PD has landed, for this wave and
    // then for everybody; request 0 follows.
    auto advance0 = [&]() __attribute__((always_inline)) {
        if (n_tiles > 1) {
            if (n_tiles > PD) wait_vmem<(PD - 1) * INFLIGHT>();
            else wait_vmem<0>();
            ring_barrier();
            request_k(loader);
            request_v(loader);
        }
    };
    // Before half-steps h and h+1 (h odd), which read K rows up to tile h+2: requests up to h+1-PD
    // have landed; requests h and h+1 follow, into stages last read in half-step h-1 or earlier.
    // Near the end of the split the outstanding requests are not whole any more, and the wave
    // waits for everything.
    // A starter that is not a loader has nothing but the first window outstanding: before pair 1
    // its requests up to 2 - PD have landed, from pair 3 on all of them.
    auto advance_pair = [&](int h) __attribute__((always_inline)) {
        if (starter && !loader) {
            if (h == 1 && 1 + PD < n_tiles) wait_vmem<(PD > 3 ? PD - 3 : 0) * INFLIGHT>();
            else wait_vmem<0>();
        } else if (h + PD < n_tiles) {
            wait_vmem<(PD - 2) * INFLIGHT>();
        } else {
            wait_vmem<0>();
        }
        ring_barrier();
        if (!loader) return;  // wave-uniform: the other waves keep no request state
        // The four requests touch three consecutive tiles (V of t0, K and V of t1, K of t2).  When
        // all three exist, are whole and lie side by side in the cache (no wrap of the tile order),
        // the copies need no checks: one straight run of eight copy instructions per tensor pair.
        bool fast = false;
        if constexpr (!PAGED) fast = rq_kt + 1 < n_tiles && rq_v0 + 3 * TK <= k_hi;
        if (fast) {
            // K of t1, V of t0, K of t2, V of t1: the order of the general path
            auto run = [&](const uint8_t *base, const uint32_t (&voff)[LOADS], uint32_t dst) __attribute__((always_inline)) {
                const uint32_t d0 = __builtin_amdgcn_readfirstlane(smem_off + dst);
#pragma unroll
                for (int j = 0; j < LOADS; ++j) copy_to_lds(base, voff[j], d0 + load_row0(j) * ROWB);
            };
            run(rq_kptr, k_voff, rq_koff);
            rq_koff = next_k(rq_koff);
            run(rq_vptr, v_voff, rq_voff);
            rq_voff = next_v(rq_voff);
            rq_kptr += TK * k_row_bytes;
            rq_vptr += TK * v_row_bytes;
            run(rq_kptr, k_voff, rq_koff);
            rq_koff = next_k(rq_koff);
            run(rq_vptr, v_voff, rq_voff);
            rq_voff = next_v(rq_voff);
            rq_kt += 2;
            rq_vt += 2;
            rq_v0 += 2 * TK;                  // = the old t2: still inside the split
            rq_vptr += TK * v_row_bytes;
            rq_k0 = next_key0(rq_v0);         // the tile after t2 may be where the order wraps
            rq_kptr = rq_k0 == k_lo ? k_ptr_lo : rq_kptr + TK * k_row_bytes;
        } else {
            request_k(true);
            request_v(true);
            request_k(true);
            request_v(true);
        }
    };
    // A wave whose rows all lie past the last query row of the KV head (the last query block of a
    // head whose row count is not a multiple of the block) only keeps feeding the rings: its
    // share of every tile, and every barrier of the code below.
    if (wave_row0 >= rows_kv) {
        advance0();
        for (int h = 1; h + 1 < n_tiles; h += 2) advance_pair(h);
        __syncthreads();
        return;
    }

    // scores of step 0 and the reference exponent
    {
        bf16x8 k0f[KSTEPS];
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) k0f[kk] = read_k(k_off0, kk);
#pragma unroll
        for (int e = 0; e < 16; ++e) s_sl[0][e] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) s_sl[0] = mfma32<F16>(k0f[kk], q_reg[kk], s_sl[0]);
    }
    if (key_first + TK > k_hi) mask_tail(s_sl[0], key_first);
    {  // the reference exponent: the largest of the first 32 scores (at least one key is valid)
        float mx = s_sl[0][0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, s_sl[0][e]);
        m_run = half_max(mx);
    }
    mc = m_run * c;
    advance0();
    if (n_tiles > 1) {
#pragma unroll
        for (int f = 0; f < FS; ++f) k_frag[f] = read_k(TILEB + k_off0, f);
    }

    // Half-step h: scores of step h; output of step h-2; softmax of step h-1.  Steps -1 and -2 do
    // not exist: their numerators are zeros, and the "V tile" they are multiplied with is the K
    // tile in ring stage 0 (any finite data gives zero; rows past the end of a split repeat valid
    // rows).  After the last step there is no next K tile: the reads requested for it return
    // whatever the stage holds, and nothing uses them.  A split with an odd number of tiles ends
    // on a step that does not exist either: all its scores are masked.
    // LDS offsets of K(h), K(h+1), V(h-2), V(h-1), and the first key of tile h:
    uint32_t k_cur = TILEB, k_nxt = 2 * TILEB, v_cur = 0, v_nxt = V_RING;
    int key_h = next_key0(key_first);
    auto step_on = [&]() __attribute__((always_inline)) {
        k_cur = k_nxt;
        k_nxt = next_k(k_nxt);
        v_cur = v_nxt;
        v_nxt = next_v(v_nxt);
        key_h = next_key0(key_h);
    };
    int h = 1;
    for (; h + 1 < n_tiles; h += 2) {
        advance_pair(h);
        half_step(X1{}, yes{}, yes{}, yes{}, yes{}, k_cur, k_nxt, v_cur, v_nxt);
        if (key_h + TK > k_hi) mask_tail(s_sl[1], key_h);
        step_on();
        half_step(X0{}, yes{}, yes{}, yes{}, yes{}, k_cur, k_nxt, v_cur, v_nxt);
        if (key_h + TK > k_hi) mask_tail(s_sl[0], key_h);
        step_on();
    }
    // h = n_tiles - 1 (one step left to score) or h = n_tiles (none: the step scored here is void)
    if (h >= n_tiles) key_h = k_hi;
    half_step(X1{}, yes{}, yes{}, no{}, yes{}, h < n_tiles ? k_cur : 0u, 0, v_cur, v_nxt);
    if (key_h + TK > k_hi) mask_tail(s_sl[1], key_h);
    step_on();
    if (h >= n_tiles) v_nxt = 0;  // V of the void step: any finite data
    half_step(X0{}, no{}, yes{}, no{}, yes{}, 0, 0, v_cur, v_nxt);  // output h-1; softmax h
    step_on();
    half_step(X1{}, no{}, no{}, no{}, no{}, 0, 0, v_cur, 0);       // output h

    // ---- epilogue: normalise and store this split's partial result -----------------------
    __syncthreads();  // every wave is done reading tiles: the rings are free
    const float l_tot = half_sum(l_run);
    const float inv = 1.f / l_tot;
    if (out.o_is_16bit) {
        // A lane holds 4-element runs of one query row, 256 bytes apart from its neighbours':
        // stored as they are, every store instruction would touch 32 rows with 16 bytes each.
        // The rows go through LDS instead (each wave its own 32 rows, so no further barrier)
        // and leave as whole rows, 16 bytes per lane.
        uint8_t *mine = smem + wave * (32 * ROWB);
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
        // the row index and validity of query row j live in lane j
        const uint32_t my_row = (uint32_t)part_row;
        constexpr int ROWS_PER_STORE = 64 / CH;
#pragma unroll
        for (int j = 0; j < 32 / ROWS_PER_STORE; ++j) {
            const int row = j * ROWS_PER_STORE + lane / CH;
            const int cpos = lane % CH;
            const uint4 v = *(const uint4 *)(mine + row * ROWB + ((cpos ^ (row & (CH - 1))) * 16));
            const uint32_t prow = __shfl(my_row, row);
            const int ok = __shfl((int)q_ok, row);
            // streaming stores: whole rows that nobody on this compute unit reads again; they leave
            // the L2 as they are written instead of in one burst when the kernel ends
            uint16_t *dst = (uint16_t *)out.o + (size_t)prow * D + cpos * 8;
            if (ok && tail.counters == nullptr) {
                __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, (u32x4 *)dst);
            } else if (ok) {
                // single-launch call: device-scope stores, complete in the memory all XCDs share when
                // the wave's store counter says so (the rows are read by other workgroups of this launch)
                __hip_atomic_store((uint64_t *)dst, (uint64_t)v.x | ((uint64_t)v.y << 32), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store((uint64_t *)dst + 1, (uint64_t)v.z | ((uint64_t)v.w << 32), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
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
    if (lh == 0) {
        const float lse_part = (m_run * c + log2f(l_tot)) * kLn2;
        if (tail.counters == nullptr) out.lse[part_row] = lse_part;
        else __hip_atomic_store(out.lse + part_row, lse_part, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    }();

    if (tail.counters == nullptr) return;
    // ---- single-launch call (protocol: see FusedTail).  Memory order: the partial rows and LSEs
    // were written with device-scope stores; once a wave's store counter is at zero they are in the
    // memory all XCDs share, so after the barrier a relaxed count says that this workgroup's rows
    // are there.  (A release fence instead starts a write-back of the XCD's whole L2 in every
    // workgroup: counting in then took 7.5 us on average and 13.8 us for the last of 256
    // workgroups, against 1.5 and 2.8.)  The thread that sees the count complete invalidates this
    // compute unit's view (acquire fence) before the barrier that lets the other waves read.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // every wave's rows are out (and nobody uses the staging rows in LDS any more)
    // LDS from here on: the tree-mask rows of this sequence (at most LS_MAX_TREE rows of 8 words),
    // its parent array, a few words that carry the counting thread's findings to the others
    uint64_t *mask_rows = (uint64_t *)smem;
    int32_t *par_lds = (int32_t *)(smem + LS_MAX_TREE * 8 * sizeof(uint64_t));
    volatile uint32_t *word = (volatile uint32_t *)(par_lds + LS_MAX_TREE);
    const int unit = bz * n_qblocks + qblock;
    const uint32_t n_splits = (uint32_t)plan.n_splits;
    uint64_t *arrival = tail.counters + (size_t)unit * kCounterWords;
    // The last wave counts and waits (its first lane); the others build the tree mask meanwhile.
    const bool counting = tid == (NW - 1) * 64;
    uint64_t before = 0;
    if (counting) before = __hip_atomic_fetch_add(arrival, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // the parent array goes to LDS (an entry outside {-1} u [0, i) counts as -1)
    for (int i = tid; i < p.n_tree; i += NW * 64) {
        const int32_t pa = tail.parents[(size_t)b * p.n_tree + i];
        par_lds[i] = pa < -1 || pa >= i ? -1 : pa;
    }
    __syncthreads();
    if (counting) {
        const uint32_t call = (uint32_t)(before >> 32);
        const bool last = (uint32_t)before == n_splits - 1u;
        uint64_t *claims = arrival + 1 + (call & 1u);
        bool go = last;
        if (last) {
            __hip_atomic_store(arrival + 1 + ((call + 1u) & 1u), 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_fetch_add(arrival, (1ull << 32) - n_splits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            for (int poll = 0; poll < tail.spin_limit && !go; ++poll) {
                __builtin_amdgcn_s_sleep(4);
                go = (uint32_t)(__hip_atomic_load(arrival, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32) != call;
            }
        }
        uint32_t mine = 0;
        if (go) {
            const uint64_t bit = 1ull << split;
            mine = (__hip_atomic_fetch_or(claims, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & bit) ? 0u : 1u;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        word[0] = mine;
        word[1] = last ? 1u : 0u;
        word[2] = call & 1u;
    } else if (wave < NW - 1) {
        // the tree-mask rows, walked in LDS: row i gets bit j iff j is i or an ancestor of i
        const int words = (p.n_tree + 63) >> 6;
        for (int node = tid; node < p.n_tree; node += (NW - 1) * 64) {
            int j = node;
            for (int w = words - 1; w >= 0; --w) {
                uint64_t bits = 0;
                while (j >= 0 && (j >> 6) == w) {
                    bits |= (uint64_t)1 << (j & 63);
                    j = par_lds[j];
                }
                mask_rows[(size_t)node * words + w] = bits;
            }
        }
    }
    __syncthreads();
    const bool mine = __builtin_amdgcn_readfirstlane(word[0]) != 0;
    const bool last = __builtin_amdgcn_readfirstlane(word[1]) != 0;
    uint64_t *claims = arrival + 1 + __builtin_amdgcn_readfirstlane(word[2]);
    if (!mine && !last) return;
    // A slice is the block's rows cut into n_splits runs; a wave takes one row at a time.
    typedef std::conditional_t<F16, half_t, uint16_t> T16;
    const int row_base = qblock * NW * 32;
    const int rows_here = rows_kv - row_base < NW * 32 ? rows_kv - row_base : NW * 32;
    const int per_slice = (rows_here + (int)n_splits - 1) / (int)n_splits;
    auto do_slice = [&](int k) {
        const int hi = (k + 1) * per_slice < rows_here ? (k + 1) * per_slice : rows_here;
        for (int r = k * per_slice + wave; r < hi; r += NW) {
            const int m = row_base + r;
            tail_rows<T16, T16, D, 64, 32>(p, mask_rows, out, plan.n_splits, (T16 *)tail.out, tail.o_stride[0],
                                           tail.o_stride[1], tail.o_stride[2], tail.lse, b, g * p.group + m / p.n_tree,
                                           m % p.n_tree, true, lane);
        }
    };
    if (mine) do_slice(split);
    if (!last) return;
    // the slices nobody has taken by now
    __syncthreads();  // everybody has read the words above
    if (counting) {
        const uint64_t all = n_splits >= 64u ? ~0ull : (1ull << n_splits) - 1ull;
        const uint64_t taken = __hip_atomic_fetch_or(claims, all, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint64_t rest = all & ~taken;
        word[0] = (uint32_t)rest;
        word[1] = (uint32_t)(rest >> 32);
    }
    __syncthreads();
    uint64_t rest = (uint64_t)__builtin_amdgcn_readfirstlane(word[0]) |
                    ((uint64_t)__builtin_amdgcn_readfirstlane(word[1]) << 32);
    while (rest) {
        do_slice(__builtin_ctzll(rest));
        rest &= rest - 1;
    }
}

bool prefix_mfma_supports(const Problem &p, int dtype)
{
    // the tile loads address rows of one tile with 32-bit byte offsets
    const int64_t max_row_bytes = 2 * (p.kc_stride[2] > p.vc_stride[2] ? p.kc_stride[2] : p.vc_stride[2]);
    return is_16bit(dtype) && (p.head_dim == 128 || p.head_dim == 64) && max_row_bytes * 64 < (1ll << 31);
}

namespace {

template <int D, int NW, bool F16, bool PAGED, int PD>
hipError_t launch_one(const Problem &p, const SplitPlan &plan, const Partials &out, const MaskJob &mask_job,
                      const FusedTail &tail, hipStream_t stream)
{
    constexpr int lds_bytes = (2 * PD + 7) * TK * D * 2 + (PAGED ? kMaxSplitPages * 4 : 0);
    static_assert(lds_bytes <= 160 * 1024, "the rings exceed the 160 KB of a compute unit");
    auto kernel = prefix_mfma_kernel<D, NW, F16, PAGED, PD>;
    static hipError_t attr = hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 lds_bytes);
    if (attr != hipSuccess) return attr;
    const int rows_kv = p.group * p.n_tree;
    const int n_qblocks = (rows_kv + NW * 32 - 1) / (NW * 32);
    const int64_t n_main = (int64_t)plan.n_splits * n_qblocks * p.batch * p.n_kv_heads;
    const int64_t n_blocks = n_main + (mask_job.parents ? p.batch : 0);
    if (n_blocks > 0x7fffffff) return hipErrorInvalidValue;
    if (tail.counters && (!out.o_is_16bit || plan.n_splits > 64 ||
                          (int64_t)n_qblocks * p.batch * p.n_kv_heads > kMaxArrivalCounters))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(kernel, dim3((unsigned)n_blocks), dim3(NW * 64), lds_bytes, stream, p, plan, out, mask_job,
                       tail, n_qblocks);
    return hipGetLastError();
}

}  // namespace

int prefix_mfma_query_blocks(const Problem &p)
{
    const int rows_kv = p.group * p.n_tree;
    const int per_block = rows_kv > 128 ? 256 : 128;
    return (rows_kv + per_block - 1) / per_block;
}

hipError_t launch_prefix_mfma(const Problem &p, int dtype, const SplitPlan &plan, const Partials &out,
                              const MaskJob &mask_job, const FusedTail &tail, hipStream_t stream)
{
    const int rows_kv = p.group * p.n_tree;
    const bool f16 = dtype == LS_F16;
    const bool paged = p.block_table != nullptr;
    // Above 128 query rows per KV head: 8 waves, two per SIMD, 256 rows per workgroup (the split
    // planner counts on kPrefixRowsPerWorkgroup = 256); else 4 waves.
    const bool deep = plan.split_len <= kDeepMaxTiles * TK;  // few tiles per split: request them all at once
#define LS_MFMA_CASE3(DD, WW, PP)                                                                      \
    (paged ? (f16 ? launch_one<DD, WW, true, true, PP>(p, plan, out, mask_job, tail, stream)           \
                  : launch_one<DD, WW, false, true, PP>(p, plan, out, mask_job, tail, stream))         \
           : (f16 ? launch_one<DD, WW, true, false, PP>(p, plan, out, mask_job, tail, stream)          \
                  : launch_one<DD, WW, false, false, PP>(p, plan, out, mask_job, tail, stream)))
#define LS_MFMA_CASE2(DD, WW) (deep ? LS_MFMA_CASE3(DD, WW, kDeepRequests) : LS_MFMA_CASE3(DD, WW, kShallowRequests))
#define LS_MFMA_CASE(DD) (rows_kv > 128 ? LS_MFMA_CASE2(DD, 8) : LS_MFMA_CASE2(DD, 4))
    if (p.head_dim == 128) return LS_MFMA_CASE(128);
    if (p.head_dim == 64) return LS_MFMA_CASE(64);
#undef LS_MFMA_CASE
#undef LS_MFMA_CASE2
#undef LS_MFMA_CASE3
    return hipErrorInvalidValue;
}

}  // namespace ls
