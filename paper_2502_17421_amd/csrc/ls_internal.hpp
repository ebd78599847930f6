// Internal declarations shared by the host API and the kernel translation units.
// Nothing here is part of the C ABI (see include/ls_attn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ls_attn.h"

namespace ls {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kMaxSplitPages = 512;  // pages one key split of the MFMA kernel may touch (their ids sit in 2 KB of LDS)
constexpr int kPrefixRowsPerWorkgroup = 256;  // query rows per workgroup of the MFMA kernel (8 waves x 32 rows)
constexpr int kPrefixWorkgroupsPerCU = 1;     // workgroups resident per compute unit
constexpr int kMaxSplitLen = 8192;    // cache rows per split on the MFMA path: 512 pages of the smallest page size, 16

// Everything a kernel needs to find its operands; passed by value.
struct Problem {
    const void *q;
    const void *k_cache;
    const void *v_cache;
    const void *k_tree;
    const void *v_tree;
    const int32_t *prefix_lens;  // device, one per sequence; nullptr: every sequence has prefix_len_all rows
    int32_t prefix_len_all;
    // Paged cache (block_table != nullptr): cache row r of sequence b lives in page
    // block_table[b * bt_stride + (r >> page_shift)] at row r & (page_size - 1); kc_stride /
    // vc_stride then mean {between pages, between KV heads inside a page, between rows}.
    const int32_t *block_table;
    int32_t bt_stride, page_shift;
    int32_t batch, n_q_heads, n_kv_heads, group, head_dim, n_tree, max_prefix_len;
    float scale_log2;  // softmax scale times log2(e): logits are kept in base 2 inside kernels
    int64_t q_stride[3], kc_stride[3], vc_stride[3], kt_stride[3], vt_stride[3];
};

// Where partial results go: o [batch, n_q_heads, parts_stride, n_tree, head_dim] in float or
// in the problem's 16-bit type (o_is_16bit), lse [batch, n_q_heads, parts_stride, n_tree]
// float.  A producer writes parts [part_base, part_base + its own count).
struct Partials {
    void *o;
    float *lse;
    int32_t parts_stride;
    int32_t part_base;
    int32_t o_is_16bit;
    // 0: [.., part, tree row, ..] (the layout of the public subsystem entry points);
    // 1: [.., tree row, part, ..]: the parts of one query row lie side by side, which is what
    //    the kernel that merges them reads (the whole-path calls use this inside the workspace)
    int32_t row_major;
    // index of (b, h, part, tree row i) into lse, and times head_dim into o
    __host__ __device__ size_t row(size_t bh, int part, int n_tree, int i) const
    {
        return row_major ? (bh * n_tree + i) * parts_stride + part_base + part
                         : (bh * parts_stride + part_base + part) * n_tree + i;
    }
};

// Work appended to the cached-key launch so that the whole call needs one launch less:
// extra workgroups (one per sequence) that build the tree mask.  parents == nullptr: none.
struct MaskJob {
    const int32_t *parents;
    uint64_t *mask;
    int32_t *err_flag;
};

// Single-launch form of the whole call.  The workgroups of one (sequence, KV head, query block),
// one per key split, share three 64-bit words: an arrival word (call number << 32 | workgroups
// counted in this call) and two claim words used by alternate calls (bit k: the rows of slice k
// are taken).  A workgroup counts itself in after its partial rows are written and fenced.  The
// one that completes the count zeroes the other claim word for the next call and adds
// 2^32 - n_splits to the arrival word: the count is back at zero and the call number has moved,
// which is what the others poll for, at most spin_limit times.  Whoever sees the move claims
// slice (its split index) of the block's rows with a fetch-or and does the tree attention and
// the merge for them; the workgroup that completed the count then claims every slice still free
// (workgroups that gave up, or all of them when spin_limit is 0) and does those too.  So every
// row is written exactly once, by the same code whoever writes it, and no wait is unbounded.
// counters == nullptr: the kernel only writes its partial rows.
struct FusedTail {
    uint64_t *counters;  // three words per (sequence, KV head, query block); zero before the first call
    const int32_t *parents;
    void *out;
    int64_t o_stride[3];
    float *lse;
    int32_t spin_limit;  // polls (about half a microsecond apart) before a workgroup leaves its slice to the last one
};
constexpr int kMaxArrivalCounters = 4096;  // (sequence, KV head, query block) triples one single-launch call may have
constexpr int kCounterWords = 3;           // 64-bit words per triple

struct SplitPlan {
    int32_t n_splits;   // parts the cached-key kernel writes
    int32_t split_len;  // cache rows per split
    // MFMA path, whole-path calls only (their parts are nobody else's business): every sequence
    // cuts ITS cached rows into n_splits equal pieces (a multiple of 32 rows, at most split_len)
    // instead of pieces of split_len rows sized for the longest sequence the cache can hold, so
    // that a short sequence keeps as many workgroups busy as a long one.
    int32_t per_sequence;
    int32_t reserved;
};

// bf16 <-> float on raw 16-bit patterns (round to nearest even, NaN kept quiet).
__device__ __forceinline__ float bf16_to_float(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t float_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Element type tags: float, uint16_t (a bf16 bit pattern) and half_t (an IEEE half bit pattern).
struct half_t {
    uint16_t bits;
};
__device__ __forceinline__ float half_to_float(uint16_t v) { return (float)__builtin_bit_cast(_Float16, v); }
__device__ __forceinline__ uint16_t float_to_half(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }
inline bool is_16bit(int dtype) { return dtype == LS_BF16 || dtype == LS_F16; }

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t *p) { return bf16_to_float(*p); }
    static __device__ __forceinline__ void store(uint16_t *p, float v) { *p = float_to_bf16(v); }
};

template <> struct Elem<half_t> {
    static __device__ __forceinline__ float load(const half_t *p) { return half_to_float(p->bits); }
    static __device__ __forceinline__ void store(half_t *p, float v) { p->bits = float_to_half(v); }
};

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// The tree-mask rows of one sequence, computed by the n_threads threads of a workgroup, node
// tid, tid + n_threads, ... each (all threads of the workgroup must call it; it synchronises
// them once).  A row is built one 64-bit word at a time from the highest word down: the chain
// index strictly decreases, so the walk visits the words in that order and ends after at most
// `node` steps whatever the array holds; an entry outside {-1} u [0, j) ends the walk and is
// reported.
__device__ __forceinline__ void build_tree_mask_rows(const int32_t *__restrict__ par, int32_t n_tree,
                                                     uint64_t *__restrict__ mask_rows,
                                                     int32_t *__restrict__ err_word, int tid, int n_threads)
{
    const int words = (n_tree + 63) >> 6;
    int bad = 0;
    for (int node = tid; node < n_tree; node += n_threads) {
        int j = node;
        for (int w = words - 1; w >= 0; --w) {
            uint64_t bits = 0;
            while (j >= 0 && (j >> 6) == w) {
                bits |= (uint64_t)1 << (j & 63);
                int p = par[j];
                if (p < -1 || p >= j) {
                    bad = 1;
                    p = -1;
                }
                j = p;
            }
            mask_rows[(size_t)node * words + w] = bits;
        }
    }
    const int any_bad = __syncthreads_or(bad);
    if (tid == 0 && err_word) *err_word = any_bad ? 1 : 0;
}

// Host launchers, one per kernel family.  Each returns a hipError_t from the launch.
hipError_t launch_tree_mask(const int32_t *parents, int32_t batch, int32_t n_tree, uint64_t *mask,
                            int32_t *err_flag, hipStream_t stream);
hipError_t launch_tree_attn(const Problem &p, int dtype, const uint64_t *mask, const Partials &out,
                            hipStream_t stream);
hipError_t launch_prefix_valu(const Problem &p, int dtype, const SplitPlan &plan, const Partials &out,
                              const MaskJob &mask_job, hipStream_t stream);
hipError_t launch_prefix_mfma(const Problem &p, int dtype, const SplitPlan &plan, const Partials &out,
                              const MaskJob &mask_job, const FusedTail &tail, hipStream_t stream);
// query blocks per KV head of the MFMA kernel (the arrival counters of a single-launch call are
// batch * n_kv_heads * this many)
int prefix_mfma_query_blocks(const Problem &p);
hipError_t launch_clear_words(uint32_t *words, int32_t n, hipStream_t stream);
bool prefix_mfma_supports(const Problem &p, int dtype);
SplitPlan plan_splits(const ls_desc &d, int32_t n_splits_request);
hipError_t launch_merge(int32_t batch, int32_t n_q_heads, int32_t n_tree, int32_t head_dim, int dtype,
                        int32_t n_parts, const void *o_parts, int parts_are_16bit, const float *lse_parts, void *out,
                        const int64_t o_stride[3], float *lse, hipStream_t stream);
// Masked tree attention and the merge with n_cache_parts cached-key partials in one kernel.
hipError_t launch_tree_merge(const Problem &p, int dtype, const uint64_t *mask, const Partials &cache_parts,
                             int32_t n_cache_parts, void *out, const int64_t o_stride[3], float *lse,
                             hipStream_t stream);

hipError_t launch_tree_accept(const int32_t *parents, const int32_t *draft_tokens, const int32_t *target_tokens,
                              int32_t batch, int32_t n_tree, int32_t *accept_path, int32_t *accept_len,
                              int32_t *next_token, int32_t *err_flag, hipStream_t stream);
hipError_t launch_kv_commit(const Problem &p, int dtype, const int32_t *accept_path, const int32_t *accept_len,
                            void *k_cache, void *v_cache, int32_t *new_prefix_lens, int32_t *err_flag,
                            hipStream_t stream);


}  // namespace ls
