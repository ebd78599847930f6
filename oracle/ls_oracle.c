/*
 * CPU oracle for LongSpec's hybrid tree attention (arXiv 2502.17421).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  Nothing in the product path may call it;
 * only the tests, the smoke check and the benchmark's cpu_baseline leg do.
 * It shares no code, header, table or helper with the HIP kernels.
 *
 * What it computes (Section 3.3 and the appendix "Correctness for Attention
 * Aggregation"):
 *
 *   For one query row q of one speculative-tree token i, the keys it may see
 *   are every cached row of the main sequence (no mask) and those tree rows j
 *   that lie on the path from i up to its root, i itself included (the tree
 *   mask of Section 3.3 "Fast Tree Attention": tokens off that path are wrong
 *   combinations and are removed).  Over that visible set V(i):
 *
 *       z_j  = scale * <q, k_j>                  (appendix: q K^T / sqrt(d_qk))
 *       lse  = log sum_{j in V} exp(z_j)         (appendix eq. (1), natural log)
 *       out  = sum_{j in V} exp(z_j - lse) v_j   (appendix eq. (2)/(3))
 *
 *   This is the monolithic definition: one softmax over [cache || specs].
 *   The oracle never splits the key set and never merges partial results, so
 *   the proposition "split + log-sum-exp merge == monolithic attention" is
 *   something the tests can check against it rather than something built in.
 *
 *   Partial attention over a sub-range of the cache, or over the tree keys
 *   alone, is the same formula with a smaller visible set (the appendix's
 *   o_cache / LSE_cache and o_specs / LSE_specs); the visible set is selected
 *   by the arguments prefix_lo, prefix_hi and use_tree.
 *
 *   ls_oracle_lse_merge evaluates the two aggregation formulas of Section 3.3
 *   ("Aggregation") left to right over a list of partial results; it exists so
 *   that step (d) of the GPU path can be checked alone.  The raw formula
 *   exp(LSE) overflows for large LSE, so both exponentials are taken relative
 *   to the larger of the two operands, which does not change the value.
 *
 * Arithmetic: every product, sum, exp and log is IEEE double.  Inputs arrive
 * as float because the values under test are fp32 or bf16 numbers, both of
 * which a float holds exactly; they are widened to double before first use.
 *
 * Parallelism: an OpenMP "parallel for" over independent output rows only.
 * No blocking, no fusion, no reordering inside a row.
 *
 * Readings taken where the paper is silent (each also listed in the design
 * notes): a tree token sees itself; parents[i] == -1 marks a root and more
 * than one root is allowed; natural-log LSE of the scaled logits; query head h
 * uses KV head h / (Hq / Hkv); an empty visible set gives lse = -inf, out = 0.
 *
 * Two integer steps that follow the attention in a verification round are
 * defined at the end of the file, each with its own comment: the greedy
 * acceptance walk over the tree and the move of the accepted tokens' K/V rows
 * into the cache (pins: tests/test_oracle_accept_pins.py -- a hand-worked
 * case, equality with plain greedy decoding of a toy deterministic model,
 * an all-paths brute force, and indexing written with numpy).
 *
 * Pins: tests/test_oracle_pins.py (brute force, hand-computed case, closed
 * forms, split/merge invariant, chain == causal and other textbook special
 * cases against torch's CPU scaled_dot_product_attention).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int ls_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Returns 0 if parents describes a forest in topological order:
 * parents[i] == -1 (root) or 0 <= parents[i] < i.  Otherwise the index of the
 * first offending entry plus one. */
int ls_oracle_check_parents(const int32_t *parents, int32_t n_tree)
{
    for (int32_t i = 0; i < n_tree; ++i) {
        int32_t p = parents[i];
        if (p < -1 || p >= i)
            return i + 1;
    }
    return 0;
}

/*
 * Tree mask, one row per tree token, as a bit set over tree tokens:
 * bit j of row i is 1 iff j == i or j is an ancestor of i.
 * mask is [n_tree][n_words] uint64, n_words = ceil(n_tree / 64),
 * bit j lives in word j / 64 at position j % 64.
 * Built by walking each row's parent chain upward.
 */
int ls_oracle_tree_mask(const int32_t *parents, int32_t n_tree, uint64_t *mask)
{
    if (ls_oracle_check_parents(parents, n_tree) != 0)
        return -1;
    int32_t n_words = (n_tree + 63) / 64;
    memset(mask, 0, (size_t)n_tree * (size_t)n_words * sizeof(uint64_t));
    for (int32_t i = 0; i < n_tree; ++i) {
        int32_t j = i;
        while (j >= 0) {
            mask[(size_t)i * n_words + j / 64] |= (uint64_t)1 << (j % 64);
            j = parents[j];
        }
    }
    return 0;
}

/*
 * Attention of selected query rows of ONE sequence.
 *
 *   q        [n_q_heads ][n_tree    ][head_dim]   row-major float
 *   k_cache  [n_kv_heads][prefix_len][head_dim]
 *   v_cache  [n_kv_heads][prefix_len][head_dim]
 *   k_tree   [n_kv_heads][n_tree    ][head_dim]
 *   v_tree   [n_kv_heads][n_tree    ][head_dim]
 *   parents  [n_tree]
 *   rows     [n_rows][2] = (query head h, tree row i) of each wanted output
 *   out      [n_rows][head_dim] double,  lse [n_rows] double
 *
 * Visible set of row (h, i): cache rows prefix_lo <= j < prefix_hi, plus, when
 * use_tree != 0, the tree rows on the path i -> root.
 * Returns 0, or -1 on a bad argument.
 */
int ls_oracle_attn_rows(int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                        int32_t n_tree, int64_t prefix_len,
                        const float *q,
                        const float *k_cache, const float *v_cache,
                        const float *k_tree, const float *v_tree,
                        const int32_t *parents, double scale,
                        int64_t prefix_lo, int64_t prefix_hi, int32_t use_tree,
                        const int32_t *rows, int64_t n_rows,
                        double *out, double *lse)
{
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0)
        return -1;
    if (head_dim <= 0 || n_tree <= 0 || prefix_len < 0)
        return -1;
    if (prefix_lo < 0 || prefix_hi > prefix_len || prefix_lo > prefix_hi)
        return -1;
    if (use_tree && ls_oracle_check_parents(parents, n_tree) != 0)
        return -1;
    for (int64_t r = 0; r < n_rows; ++r) {
        if (rows[2 * r] < 0 || rows[2 * r] >= n_q_heads)
            return -1;
        if (rows[2 * r + 1] < 0 || rows[2 * r + 1] >= n_tree)
            return -1;
    }

    const int32_t group = n_q_heads / n_kv_heads;
    const int64_t n_cache = prefix_hi - prefix_lo;
    int failed = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; ++r) {
        const int32_t h = rows[2 * r];
        const int32_t i = rows[2 * r + 1];
        const int32_t g = h / group;
        const float *qrow = q + ((size_t)h * n_tree + i) * head_dim;
        const float *kc = k_cache + (size_t)g * prefix_len * head_dim;
        const float *vc = v_cache + (size_t)g * prefix_len * head_dim;
        const float *kt = k_tree + (size_t)g * n_tree * head_dim;
        const float *vt = v_tree + (size_t)g * n_tree * head_dim;

        /* the visible tree rows: the path from i up to its root */
        int32_t *path = (int32_t *)malloc((size_t)n_tree * sizeof(int32_t));
        int32_t n_path = 0;
        if (use_tree && path) {
            for (int32_t j = i; j >= 0; j = parents[j])
                path[n_path++] = j;
        }
        const int64_t n_vis = n_cache + n_path;
        double *z = (double *)malloc((size_t)(n_vis > 0 ? n_vis : 1) * sizeof(double));
        double *o = out + (size_t)r * head_dim;
        if (!path || !z) {
#pragma omp atomic write
            failed = 1;
            free(path);
            free(z);
            continue;
        }

        /* logits */
        for (int64_t j = 0; j < n_cache; ++j) {
            const float *krow = kc + (size_t)(prefix_lo + j) * head_dim;
            double acc = 0.0;
            for (int32_t d = 0; d < head_dim; ++d)
                acc += (double)qrow[d] * (double)krow[d];
            z[j] = scale * acc;
        }
        for (int32_t a = 0; a < n_path; ++a) {
            const float *krow = kt + (size_t)path[a] * head_dim;
            double acc = 0.0;
            for (int32_t d = 0; d < head_dim; ++d)
                acc += (double)qrow[d] * (double)krow[d];
            z[n_cache + a] = scale * acc;
        }

        for (int32_t d = 0; d < head_dim; ++d)
            o[d] = 0.0;
        if (n_vis == 0) {
            lse[r] = -INFINITY;
            free(path);
            free(z);
            continue;
        }

        /* log-sum-exp, shifted by the largest logit */
        double zmax = z[0];
        for (int64_t j = 1; j < n_vis; ++j)
            if (z[j] > zmax)
                zmax = z[j];
        double denom = 0.0;
        for (int64_t j = 0; j < n_vis; ++j)
            denom += exp(z[j] - zmax);
        lse[r] = zmax + log(denom);

        /* weighted sum of the value rows */
        for (int64_t j = 0; j < n_cache; ++j) {
            const double w = exp(z[j] - zmax) / denom;
            const float *vrow = vc + (size_t)(prefix_lo + j) * head_dim;
            for (int32_t d = 0; d < head_dim; ++d)
                o[d] += w * (double)vrow[d];
        }
        for (int32_t a = 0; a < n_path; ++a) {
            const double w = exp(z[n_cache + a] - zmax) / denom;
            const float *vrow = vt + (size_t)path[a] * head_dim;
            for (int32_t d = 0; d < head_dim; ++d)
                o[d] += w * (double)vrow[d];
        }
        free(path);
        free(z);
    }
    return failed ? -2 : 0;
}

/*
 * Aggregation of partial results (Section 3.3 "Aggregation"), for n_rows
 * independent query rows:
 *
 *   o_parts   [n_rows][n_parts][head_dim] double   (already normalised)
 *   lse_parts [n_rows][n_parts]           double   (-inf = empty part)
 *
 * Starting from part 0, each further part is folded in with the two-term rule
 *     LSE_m = log(exp(LSE_a) + exp(LSE_b))
 *     O_m   = O_a exp(LSE_a - LSE_m) + O_b exp(LSE_b - LSE_m).
 * An empty part has weight zero and is skipped, whatever its o_parts hold.
 */
int ls_oracle_lse_merge(int64_t n_rows, int32_t n_parts, int32_t head_dim,
                        const double *o_parts, const double *lse_parts,
                        double *out, double *lse)
{
    if (n_rows < 0 || n_parts <= 0 || head_dim <= 0)
        return -1;
    for (int64_t r = 0; r < n_rows; ++r) {
        double *o = out + (size_t)r * head_dim;
        double acc_lse = -INFINITY;
        for (int32_t d = 0; d < head_dim; ++d)
            o[d] = 0.0;
        for (int32_t p = 0; p < n_parts; ++p) {
            const double b = lse_parts[(size_t)r * n_parts + p];
            const double *ob = o_parts + ((size_t)r * n_parts + p) * head_dim;
            if (b == -INFINITY)
                continue;
            if (acc_lse == -INFINITY) {
                acc_lse = b;
                for (int32_t d = 0; d < head_dim; ++d)
                    o[d] = ob[d];
                continue;
            }
            const double top = acc_lse > b ? acc_lse : b;
            const double merged = top + log(exp(acc_lse - top) + exp(b - top));
            const double wa = exp(acc_lse - merged);
            const double wb = exp(b - merged);
            for (int32_t d = 0; d < head_dim; ++d)
                o[d] = o[d] * wa + ob[d] * wb;
            acc_lse = merged;
        }
        lse[r] = acc_lse;
    }
    return 0;
}

/*
 * Greedy (temperature 0) acceptance of a speculation tree -- the verification
 * step that follows the target model's pass over the tree (Section 3.3 "Fast
 * Tree Attention": the target verifies all candidate sequences at once without
 * altering the final result; Section 4.1 evaluates at T = 0).
 *
 * The paper does not print the rule; the reading taken is the one that makes
 * the output identical to plain greedy decoding.  Node 0 holds the last token
 * already sampled and is always on the path.  draft_tokens[i] is the token at
 * node i, target_tokens[i] the target model's most likely next token after
 * the sequence that ends at node i.  Walk down from node 0: at node cur, the
 * child whose token equals target_tokens[cur] continues the path (the lowest
 * node index if several siblings carry that token); if there is none the walk
 * stops.  next_token is target_tokens at the last node of the path, the token
 * the target contributes itself.
 *
 *   path     [n_tree] out: node indices root first, the rest filled with -1
 *   returns the number of nodes on the path (>= 1), or -1 on bad arguments.
 */
int32_t ls_oracle_tree_accept_greedy(const int32_t *parents, const int32_t *draft_tokens,
                                     const int32_t *target_tokens, int32_t n_tree,
                                     int32_t *path, int32_t *next_token)
{
    if (!parents || !draft_tokens || !target_tokens || !path || !next_token || n_tree <= 0)
        return -1;
    if (ls_oracle_check_parents(parents, n_tree) != 0)
        return -1;
    for (int32_t i = 0; i < n_tree; ++i)
        path[i] = -1;
    int32_t cur = 0, len = 1;
    path[0] = 0;
    for (;;) {
        int32_t next = -1;
        for (int32_t j = cur + 1; j < n_tree; ++j) {
            if (parents[j] == cur && draft_tokens[j] == target_tokens[cur]) {
                next = j;
                break;
            }
        }
        if (next < 0)
            break;
        path[len++] = next;
        cur = next;
    }
    *next_token = target_tokens[cur];
    return len;
}

/*
 * Moving the accepted tokens' keys and values into the cache (the "KV cache
 * movement" after verification of the appendix "Experiments Details"; the
 * target model updates its cache only once verification is complete, Section
 * 3.2 "Flash Noisy Training").  For one sequence and one tensor (K or V):
 *
 *   cache [n_kv_heads][capacity][head_dim], tree [n_kv_heads][n_tree][head_dim]
 *   cache[g][prefix_len + j][:] = tree[g][path[j]][:]   for j < path_len.
 *
 * Values are copied bit for bit (float holds bf16 and fp32 exactly).  Returns
 * the new prefix length, or -1 if a row would fall outside the cache or a
 * path entry is not a node.
 */
int64_t ls_oracle_kv_commit(int32_t n_kv_heads, int32_t head_dim, int32_t n_tree, int64_t capacity,
                            int64_t prefix_len, const int32_t *path, int32_t path_len,
                            const float *tree, float *cache)
{
    if (!path || !tree || !cache || n_kv_heads <= 0 || head_dim <= 0 || n_tree <= 0)
        return -1;
    if (path_len < 0 || prefix_len < 0 || prefix_len + path_len > capacity)
        return -1;
    for (int32_t j = 0; j < path_len; ++j)
        if (path[j] < 0 || path[j] >= n_tree)
            return -1;
    for (int32_t g = 0; g < n_kv_heads; ++g)
        for (int32_t j = 0; j < path_len; ++j) {
            const float *src = tree + ((size_t)g * n_tree + path[j]) * head_dim;
            float *dst = cache + ((size_t)g * capacity + prefix_len + j) * head_dim;
            memcpy(dst, src, (size_t)head_dim * sizeof(float));
        }
    return prefix_len + path_len;
}
