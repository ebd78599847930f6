/*
 * ls_attn.h -- C ABI of the MI355X (gfx950) hybrid tree attention library.
 *
 * The operation is the verification-time attention of LongSpec (arXiv 2502.17421,
 * Section 3.3 "Hybrid Tree Attention"; correctness in the appendix "Correctness for
 * Attention Aggregation"):
 *
 *   Every token of the speculation tree attends to
 *     - all cached key/value rows of the main sequence, with no mask, and
 *     - the tree tokens on its own root path (itself included), i.e. under the
 *       tree mask,
 *   the two parts are computed separately, each returning a normalised output O and the
 *   log-sum-exp LSE of its scaled logits, and are then combined by
 *       LSE_merge = log(exp(LSE_a) + exp(LSE_b))
 *       O_merge   = O_a exp(LSE_a - LSE_merge) + O_b exp(LSE_b - LSE_merge),
 *   which equals one softmax attention over the concatenated keys.
 *
 * The cached part is itself split along the key axis (the "Flash Attention" the paper
 * calls is the split-KV decoding kernel, see the footnote in Section 1); the same merge
 * rule, applied to n_splits + 1 partial results, joins everything.
 *
 * Conventions for every entry point
 *   - Returns LS_OK (0) or a negative ls_status.  No exceptions, no abort.
 *   - Pointers marked DEVICE are device memory owned by the caller; the library
 *     neither allocates nor frees device memory and keeps no device state (the one
 *     exception, a fixed scratch array, is described at ls_hybrid_tree_attn_static).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the null
 *     stream) and the call returns without synchronising.
 *   - Argument errors are found on the host before anything is launched.  A launch
 *     failure reported by HIP maps to LS_ERR_HIP.
 *   - The same inputs give bit-identical outputs (fixed split schedule, no float
 *     atomics).
 *   - Calls are re-entrant; concurrency is by streams.  Calls sharing a workspace or
 *     output buffer must be ordered by the caller.
 *
 * Tensor layouts.  The last (head_dim) axis is contiguous.  Other axes are addressed
 * through element strides in ls_desc, so both [B,H,L,D] and [B,L,H,D] storage work.
 * Every row start must be 16-byte aligned (base pointers and strides*sizeof(elem)
 * multiples of 16).
 *   q        [batch, n_q_heads,  n_tree,      head_dim]   dtype
 *   k_cache  [batch, n_kv_heads, >=prefix_len, head_dim]  dtype   (v_cache alike)
 *   k_tree   [batch, n_kv_heads, n_tree,      head_dim]   dtype   (v_tree alike)
 *   out      [batch, n_q_heads,  n_tree,      head_dim]   dtype
 *   lse      [batch, n_q_heads,  n_tree]                  float, contiguous
 * Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *
 * Supported: dtype bf16, f16 (the precision of the paper's experiments, appendix
 * "Experiments Details") or f32; head_dim 64 or 128; 1 <= n_tree <= 512;
 * n_q_heads a multiple of n_kv_heads; 0 <= prefix length <= max_prefix_len.
 * Anything else returns LS_ERR_UNSUPPORTED.
 */
#ifndef LS_ATTN_H
#define LS_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LS_OK = 0,
    LS_ERR_NULL = -1,        /* a required pointer is NULL */
    LS_ERR_SHAPE = -2,       /* a size is non-positive or inconsistent */
    LS_ERR_DTYPE = -3,       /* dtype is not LS_BF16 / LS_F16 / LS_F32 */
    LS_ERR_STRIDE = -4,      /* a stride or pointer breaks the 16-byte row alignment */
    LS_ERR_TREE = -5,        /* parents is not a topologically ordered forest */
    LS_ERR_WORKSPACE = -6,   /* workspace missing, misaligned or too small */
    LS_ERR_HIP = -7,         /* HIP reported a launch error */
    LS_ERR_UNSUPPORTED = -8  /* valid request outside the supported set */
} ls_status;

typedef enum { LS_BF16 = 0, LS_F32 = 1, LS_F16 = 2 } ls_dtype;

#define LS_MAX_TREE 512

/* Problem descriptor (host memory, read during the call only). */
typedef struct {
    int32_t batch;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t n_tree;           /* tree tokens per sequence (the appendix's M) */
    int32_t max_prefix_len;   /* host-known upper bound of every prefix length; sizes the grid */
    int32_t dtype;            /* ls_dtype of q, k, v and out; lse is always float */
    float   softmax_scale;    /* 0 selects 1/sqrt(head_dim) (the appendix's 1/sqrt(d_qk)) */
    /* element strides of the (batch, head, row) axes; the head_dim axis has stride 1 */
    int64_t q_stride[3];
    int64_t o_stride[3];
    int64_t kc_stride[3];
    int64_t vc_stride[3];
    int64_t kt_stride[3];
    int64_t vt_stride[3];
} ls_desc;

/* Library version, major*10000 + minor*100 + patch. */
int ls_version(void);

/* Static description of a status code; never NULL. */
const char *ls_status_string(int status);

/* Host-only check of the descriptor (shapes, dtype, strides, supported set). */
int ls_validate_desc(const ls_desc *desc);

/*
 * Host-only check of a HOST copy of the parent arrays, [batch, n_tree] int32:
 * parents[b][i] is -1 (a root; several roots are allowed) or in [0, i).
 * Returns LS_OK or LS_ERR_TREE.
 */
int ls_validate_parents_host(const int32_t *parents, int32_t batch, int32_t n_tree);

/*
 * Number of key-axis splits the library would pick for the cached part of this
 * problem (>= 1): what ls_prefix_attn_splitkv uses for n_splits = 0, and what the whole-path
 * calls use.  It depends on the descriptor AND on the number of compute units of the current
 * HIP device (the splits are sized to fill the GPU once); without a device it is computed
 * for 256 compute units (MI355X).  It is stable across calls on one device.  Ask for it, and
 * for ls_workspace_bytes, with the device current on which the call will run.
 */
int ls_prefix_num_splits(const ls_desc *desc, int32_t *n_splits_out);

/*
 * Bytes of DEVICE workspace ls_hybrid_tree_attn needs for this descriptor:
 * the tree mask, one error word per sequence, and the partial outputs (stored in the
 * problem's dtype) and LSEs of the cached part, one per key split (ls_prefix_num_splits, so
 * the size depends on the current device's compute-unit count in the same way).
 * The workspace must be 256-byte aligned.
 */
int ls_workspace_bytes(const ls_desc *desc, size_t *bytes_out);

/*
 * The whole path (Section 3.3): tree mask from `parents`, split-KV attention over the
 * cache, masked attention over the tree tokens, log-sum-exp merge into out / lse.  It runs
 * as two launches: the cached-key kernel (some extra workgroups of which build the mask),
 * then one kernel that does the tree attention and the merge per query row.
 *
 *   prefix_lens  DEVICE int32[batch]; values are clamped into [0, max_prefix_len].
 *                A sequence with prefix length 0 attends to its tree tokens only.
 *   parents      DEVICE int32[batch, n_tree].  An entry outside {-1} u [0, i) is treated
 *                as -1 and sets the sequence's error word in the workspace (see
 *                ls_workspace_error); it never causes an out-of-bounds access.
 *   out, lse     DEVICE, written in full.
 *   workspace    DEVICE, >= ls_workspace_bytes(); contents are scratch.
 */
int ls_hybrid_tree_attn(const ls_desc *desc, const void *q,
                        const void *k_cache, const void *v_cache, const int32_t *prefix_lens,
                        const void *k_tree, const void *v_tree, const int32_t *parents,
                        void *out, float *lse,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same for one sequence whose prefix length the host knows (the form in which Section 3.3
 * states the problem: one main sequence, one set of speculative tokens).  desc->batch must be
 * 1 and 0 <= prefix_len <= desc->max_prefix_len (LS_ERR_SHAPE otherwise); the length travels
 * as a kernel argument, no device array is read.  Workspace as for ls_hybrid_tree_attn with
 * the same descriptor; results are bit-identical to that call with prefix_lens[0] = prefix_len.
 */
int ls_hybrid_tree_attn_single(const ls_desc *desc, const void *q,
                               const void *k_cache, const void *v_cache, int32_t prefix_len,
                               const void *k_tree, const void *v_tree, const int32_t *parents,
                               void *out, float *lse,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * ls_hybrid_tree_attn for callers that cannot allocate device memory or carry a workspace
 * around: code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation.  It takes no workspace: the split partials, the tree mask and the error words
 * go to an array of LS_STATIC_SCRATCH_BYTES that is part of the library's code object (every
 * GPU the library runs on holds one copy from the first use until the process ends).  The
 * call allocates and frees nothing.  Same kernels, same schedule and bit-identical results
 * as ls_hybrid_tree_attn.
 *   - A descriptor whose ls_workspace_bytes() exceeds LS_STATIC_SCRATCH_BYTES is refused with
 *     LS_ERR_WORKSPACE before anything is launched.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 *     (two streams, two threads) race; the caller must order them.  Nothing in the array has
 *     to start at zero: every word a call reads was written by that call.
 *   - The array's address is looked up on the first call on each device (with that device
 *     current); a HIP error there returns LS_ERR_HIP.
 *   - The error words of the last call are not reachable through this entry point; validate
 *     parents on the host (ls_validate_parents_host) or use ls_hybrid_tree_attn.
 */
#define LS_STATIC_SCRATCH_BYTES (64u << 20)
int ls_hybrid_tree_attn_static(const ls_desc *desc, const void *q,
                               const void *k_cache, const void *v_cache, const int32_t *prefix_lens,
                               const void *k_tree, const void *v_tree, const int32_t *parents,
                               void *out, float *lse, void *stream);

/*
 * The whole call as ONE kernel launch (Section 3.3: the two attention results are aggregated;
 * here the aggregation runs inside the kernel that computes the cached-key part).  The
 * workgroups of one (sequence, KV head, query block), one per key split, count themselves in
 * once their partial rows are written and fenced.  When every workgroup of the launch has a
 * compute unit to itself from the start (their number is at most the device's compute units),
 * each then waits, a bounded number of polls, for the count of its block to complete, and
 * does the tree mask, the masked tree attention and the merge, in fixed part order, for its
 * share of the block's rows; the workgroup that completed the count also takes the rows of any
 * workgroup that gave up waiting.  In larger launches nobody waits and the workgroup that
 * completes a block's count does all of that block's rows.  Every row is written once, by the
 * same code whoever writes it: the same inputs give bit-identical outputs.  The results agree
 * with ls_hybrid_tree_attn to rounding (the row sums are taken in another lane order), not bit
 * for bit.
 *
 *   - Arguments, workspace size and error words as for ls_hybrid_tree_attn.
 *   - The counters are the first LS_WORKSPACE_COUNTER_BYTES of the workspace, whatever the
 *     descriptor.  They must be zero before the first call on a workspace and are left in a
 *     state the next call accepts: call ls_workspace_init once on a fresh workspace (and again
 *     after anything else wrote there).  ls_workspace_init enqueues a small kernel, never a
 *     memset, so both calls may sit in a captured HIP graph.  No other entry point reads or
 *     writes the counters.  Calls that share a workspace must not overlap in time.
 *   - Problems outside the matrix-core kernel (float inputs, row strides beyond its reach),
 *     with more than 64 key splits or with more than 4096 (sequence, KV head, query block)
 *     triples run as ls_hybrid_tree_attn does, in two launches.
 *   - ls_set_single_launch_polls(n) sets the number of polls (about half a microsecond
 *     apart) for later calls of this process: 0 makes every launch the nobody-waits form,
 *     a negative n restores the default (about 20 ms); n above 2^24 is LS_ERR_SHAPE.  A wait
 *     that runs out costs time, never correctness.
 *   - On MI355X this form was slower than the two launches of ls_hybrid_tree_attn on every
 *     shape measured (1.07x to 1.3x where the workgroups share the merge, 2x and more where
 *     the last one of a block works alone): it is for callers that must have a single launch.
 */
#define LS_WORKSPACE_COUNTER_BYTES (4096u * 24u)
int ls_workspace_init(void *workspace /* DEVICE, 256-byte aligned */, size_t workspace_bytes, void *stream);
int ls_hybrid_tree_attn_fused(const ls_desc *desc, const void *q,
                              const void *k_cache, const void *v_cache, const int32_t *prefix_lens,
                              const void *k_tree, const void *v_tree, const int32_t *parents,
                              void *out, float *lse,
                              void *workspace, size_t workspace_bytes, void *stream);
int ls_set_single_launch_polls(int32_t polls);

/*
 * Unmasked attention of the query rows over the cached keys only, merged over the key
 * splits: out = o_cache, lse = LSE_cache of the appendix.  This is the cross-attention over
 * the target model's KV cache that the draft model of Section 3.1 runs at every drafting
 * step (its n_tree is the number of tokens drafted in that step), and the cached half of
 * ls_hybrid_tree_attn on its own.  desc->kt_stride / vt_stride are checked like the other
 * strides but address nothing.  Arguments,
 * workspace size and layout rules as for ls_hybrid_tree_attn; a sequence with prefix
 * length 0 gets zeros and lse = -inf.
 */
int ls_cache_attn(const ls_desc *desc, const void *q,
                  const void *k_cache, const void *v_cache, const int32_t *prefix_lens,
                  void *out, float *lse,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * DEVICE address, inside a workspace laid out for `desc`, of the int32[batch] error words
 * that ls_hybrid_tree_attn writes: word b is 1 when sequence b had an invalid parents
 * entry, else 0.  The caller may copy them back after synchronising.  Host-only pointer
 * arithmetic.
 */
int ls_workspace_error(const ls_desc *desc, void *workspace, int32_t **err_word_out);

/* ---- the four subsystems, callable on their own ------------------------------------ */

/*
 * (a) Tree mask (Section 3.3: masks derived from the prefix tree).  Row i gets bit j set
 * iff j == i or j is an ancestor of i.
 *   parents   DEVICE int32[batch, n_tree]
 *   mask      DEVICE uint64[batch, n_tree, ceil(n_tree/64)]; bit j in word j/64, bit j%64
 *   err_flag  DEVICE int32[batch], may be NULL; err_flag[b] is written on every call:
 *             1 if sequence b had an entry outside {-1} u [0, i) (treated as -1), else 0
 */
int ls_build_tree_mask(const int32_t *parents, int32_t batch, int32_t n_tree,
                       uint64_t *mask, int32_t *err_flag, void *stream);

/*
 * (b) Unmasked attention of every tree query over the cached keys, split along the key
 * axis (appendix: o_cache and LSE_cache, per split).  Split s of a sequence covers cache
 * rows [s*L, min((s+1)*L, prefix_len)), L = split length derived from max_prefix_len and
 * n_splits (ls_prefix_split_len).  An empty split writes lse = -inf and leaves its output
 * rows untouched.
 *   n_splits    >= 1, or 0 for the library's choice (ls_prefix_num_splits)
 *   part_dtype  storage type of o_part: LS_F32, or desc->dtype itself when that is LS_BF16 or
 *               LS_F16 (what ls_hybrid_tree_attn uses internally for 16-bit problems)
 *   o_part      DEVICE part_dtype[batch, n_q_heads, n_splits, n_tree, head_dim], normalised
 *   lse_part    DEVICE float[batch, n_q_heads, n_splits, n_tree], natural log
 */
int ls_prefix_attn_splitkv(const ls_desc *desc, const void *q,
                           const void *k_cache, const void *v_cache, const int32_t *prefix_lens,
                           int32_t n_splits, int32_t part_dtype, void *o_part, float *lse_part, void *stream);

/* Split length L (in cache rows) used for a given n_splits (0 = the library's choice). */
int ls_prefix_split_len(const ls_desc *desc, int32_t n_splits, int32_t *split_len_out);

/*
 * (c) Masked attention of every tree query over the tree keys (appendix: o_specs and
 * LSE_specs).  Key j is visible to row i iff bit j of mask row i is set; a row with an
 * empty mask gets lse = -inf and zero output.
 *   mask      DEVICE uint64[batch, n_tree, ceil(n_tree/64)]
 *   o_tree    DEVICE float[batch, n_q_heads, n_tree, head_dim]
 *   lse_tree  DEVICE float[batch, n_q_heads, n_tree]
 */
int ls_tree_attn_masked(const ls_desc *desc, const void *q,
                        const void *k_tree, const void *v_tree, const uint64_t *mask,
                        float *o_tree, float *lse_tree, void *stream);

/*
 * (d) Log-sum-exp merge of n_parts partial results per query row (Section 3.3
 * "Aggregation", applied associatively).  Parts with lse = -inf are skipped, whatever
 * their output rows hold; if every part is empty the row gets lse = -inf and zeros.
 *   part_dtype storage type of o_parts: LS_F32, or desc->dtype when that is LS_BF16 / LS_F16
 *   o_parts    DEVICE part_dtype[batch, n_q_heads, n_parts, n_tree, head_dim]
 *   lse_parts  DEVICE float[batch, n_q_heads, n_parts, n_tree]
 *   out        DEVICE dtype, strided by desc->o_stride;  lse DEVICE float[batch,n_q_heads,n_tree]
 */
int ls_lse_merge(const ls_desc *desc, int32_t n_parts, int32_t part_dtype,
                 const void *o_parts, const float *lse_parts,
                 void *out, float *lse, void *stream);

/* ---- after the attention: the rest of a verification round -------------------------- */

/*
 * Greedy (temperature 0) acceptance of the speculation tree, once the target model has run
 * over it (Section 3.3 "Fast Tree Attention": all candidate sequences are verified in one
 * pass without altering the final result; Section 4.1 evaluates at T = 0).  Node 0 holds
 * the last token already sampled and is always accepted.  From node cur the path continues
 * with the child whose token equals target_tokens[cur] (the lowest node index if several
 * siblings carry it) and ends where no child does; the output is then identical to plain
 * greedy decoding of the target model.
 *   parents        DEVICE int32[batch, n_tree], as for ls_build_tree_mask (an invalid entry
 *                  makes the node a root and sets err_flag)
 *   draft_tokens   DEVICE int32[batch, n_tree]  token at each node
 *   target_tokens  DEVICE int32[batch, n_tree]  the target model's most likely next token
 *                  after the sequence that ends at the node
 *   accept_path    DEVICE int32[batch, n_tree]  out: node indices root first, then -1
 *   accept_len     DEVICE int32[batch]          out: nodes on the path, >= 1
 *   next_token     DEVICE int32[batch]          out: target_tokens at the last accepted node
 *   err_flag       DEVICE int32[batch] or NULL  out: 1 if a parents entry was invalid, else 0
 * n_tree <= LS_MAX_TREE, batch <= 65535.
 */
int ls_tree_accept_greedy(const int32_t *parents, const int32_t *draft_tokens,
                          const int32_t *target_tokens, int32_t batch, int32_t n_tree,
                          int32_t *accept_path, int32_t *accept_len, int32_t *next_token,
                          int32_t *err_flag, void *stream);

/*
 * Moves the accepted tokens' key and value rows from the tree buffers into the cache (the
 * target's cache is updated only when verification is complete, Section 3.2; the "KV cache
 * movement" of the appendix "Experiments Details"):
 *   cache[b, g, prefix_lens[b] + j, :] = tree[b, g, accept_path[b, j], :],  j < accept_len[b]
 * for K and V, bit for bit.  desc gives dtype, shapes and the strides of all four buffers
 * (q_stride / o_stride are checked but address nothing); desc->max_prefix_len is the number
 * of rows the cache holds per sequence.  Rows that would fall outside it, and everything
 * from the first path entry that is not a node, are not written.
 *   k_tree, v_tree    DEVICE, read      k_cache, v_cache  DEVICE, rows written in place
 *   accept_path, accept_len, prefix_lens  DEVICE int32, as above (read only)
 *   new_prefix_lens   DEVICE int32[batch] or NULL, out: prefix_lens[b] + rows moved; must
 *                     not alias prefix_lens (other workgroups still read it)
 *   err_flag          DEVICE int32[batch] or NULL, out: 1 if fewer than accept_len[b] rows
 *                     were moved, else 0
 */
int ls_kv_commit(const ls_desc *desc, const void *k_tree, const void *v_tree,
                 const int32_t *accept_path, const int32_t *accept_len, const int32_t *prefix_lens,
                 void *k_cache, void *v_cache, int32_t *new_prefix_lens, int32_t *err_flag,
                 void *stream);

/* ---- paged caches ---------------------------------------------------------------------- */

/*
 * ls_hybrid_tree_attn over a cache kept in fixed-size pages, the layout serving systems use
 * when sequences grow and shrink (an extension beyond the paper, which keeps one contiguous
 * cache per sequence): cache row r of sequence b is row r % page_size of page
 * block_table[b * bt_stride + r / page_size].
 *   k_pages, v_pages  DEVICE dtype; desc->kc_stride / vc_stride = {between pages, between KV
 *                     heads inside a page, between rows inside a page}, rows 16-byte aligned
 *   block_table       DEVICE int32[batch, bt_stride]; the entries that cover rows below
 *                     prefix_lens[b] must be page indices of k_pages / v_pages (they are not
 *                     checked); other entries are read but never used as addresses
 *   page_size         a power of two >= 16;  bt_stride * page_size >= desc->max_prefix_len
 * dtype LS_BF16 or LS_F16.  Everything else, the workspace size included, as for
 * ls_hybrid_tree_attn.
 */
int ls_hybrid_tree_attn_paged(const ls_desc *desc, const void *q,
                              const void *k_pages, const void *v_pages,
                              const int32_t *block_table, int32_t bt_stride, int32_t page_size,
                              const int32_t *prefix_lens,
                              const void *k_tree, const void *v_tree, const int32_t *parents,
                              void *out, float *lse,
                              void *workspace, size_t workspace_bytes, void *stream);

/* ls_cache_attn over a paged cache; paging arguments as for ls_hybrid_tree_attn_paged. */
int ls_cache_attn_paged(const ls_desc *desc, const void *q,
                        const void *k_pages, const void *v_pages,
                        const int32_t *block_table, int32_t bt_stride, int32_t page_size,
                        const int32_t *prefix_lens, void *out, float *lse,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * ls_kv_commit into a paged cache: row prefix_lens[b] + j of sequence b is looked up in
 * block_table as above; the pages that receive rows must already be in the table.  page_size
 * any power of two; any dtype.
 */
int ls_kv_commit_paged(const ls_desc *desc, const void *k_tree, const void *v_tree,
                       const int32_t *accept_path, const int32_t *accept_len, const int32_t *prefix_lens,
                       void *k_pages, void *v_pages,
                       const int32_t *block_table, int32_t bt_stride, int32_t page_size,
                       int32_t *new_prefix_lens, int32_t *err_flag, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LS_ATTN_H */
