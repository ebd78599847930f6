// The two integer steps that follow the attention in a verification round: greedy acceptance
// of the speculation tree (Section 3.3 "Fast Tree Attention", evaluated at T = 0 in Section
// 4.1) and the move of the accepted tokens' key/value rows into the cache (the cache is
// updated only once verification is complete, Section 3.2; "KV cache movement" in the
// appendix "Experiments Details").  Both are latency-bound: a tree has at most LS_MAX_TREE nodes.
#include "ls_internal.hpp"

namespace ls {

namespace {

// One workgroup per sequence; a thread takes nodes tid, tid + blockDim.x, ...
//   match[i]   node i carries the token the target predicts after its parent
//   chosen[i]  match[i] and no earlier sibling matches (lowest index wins among equal tokens)
//   node i is on the accepted path iff every node from i up to, not including, node 0 is
//   chosen and that walk ends at node 0.  At most one child of a node is chosen, so the
//   accepted nodes form one root path and a node's position on it is its depth.
__global__ void __launch_bounds__(256)
tree_accept_kernel(const int32_t *__restrict__ parents, const int32_t *__restrict__ draft,
                   const int32_t *__restrict__ target, int32_t n_tree, int32_t *__restrict__ path,
                   int32_t *__restrict__ accept_len, int32_t *__restrict__ next_token,
                   int32_t *__restrict__ err_flag)
{
    __shared__ int32_t par[LS_MAX_TREE];
    __shared__ int32_t tgt[LS_MAX_TREE];
    __shared__ uint8_t match[LS_MAX_TREE];
    __shared__ uint8_t chosen[LS_MAX_TREE];
    __shared__ int32_t len_sh;
    __shared__ int32_t last_sh;
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int step = blockDim.x;
    parents += (size_t)b * n_tree;
    draft += (size_t)b * n_tree;
    target += (size_t)b * n_tree;
    path += (size_t)b * n_tree;

    int bad = 0;
    for (int i = tid; i < n_tree; i += step) {
        int32_t p = parents[i];
        if (p < -1 || p >= i) {  // not a forest in topological order: treat the node as a root
            bad = 1;
            p = -1;
        }
        par[i] = p;
        tgt[i] = target[i];
        path[i] = -1;
    }
    if (tid == 0) {
        len_sh = 0;
        last_sh = 0;
    }
    __syncthreads();
    for (int i = tid; i < n_tree; i += step) match[i] = i > 0 && par[i] >= 0 && draft[i] == tgt[par[i]];
    __syncthreads();
    for (int i = tid; i < n_tree; i += step) {
        bool first = match[i];
        for (int j = 1; j < i && first; ++j)
            if (par[j] == par[i] && match[j]) first = false;
        chosen[i] = first;
    }
    __syncthreads();
    for (int i = tid; i < n_tree; i += step) {
        int cur = i, depth = 0;
        bool on_path = true;
        while (cur > 0) {  // par[cur] < cur, so this ends after at most i steps
            if (!chosen[cur]) {
                on_path = false;
                break;
            }
            cur = par[cur];
            ++depth;
        }
        on_path = on_path && cur == 0;  // a walk that ends at another root is off the path
        if (on_path) {
            path[depth] = i;
            // depth in the high bits, node in the low ones: the maximum names the deepest accepted node
            atomicMax(&last_sh, (depth << 16) | i);
            atomicMax(&len_sh, depth + 1);
        }
    }
    const int any_bad = __syncthreads_or(bad);
    if (tid == 0) {
        // the deepest accepted node reports the token the target adds itself
        next_token[b] = tgt[last_sh & 0xffff];
        accept_len[b] = len_sh;
        if (err_flag) err_flag[b] = any_bad ? 1 : 0;
    }
}

// One workgroup per (sequence, KV head): 16-byte pieces of the accepted rows of K and V are
// copied from the tree buffers to cache rows prefix_len, prefix_len + 1, ...  The number of
// rows moved is the longest prefix of the path whose entries are nodes and whose target rows
// exist; anything shorter than accept_len is reported in err_flag.
__global__ void __launch_bounds__(256)
kv_commit_kernel(Problem p, int elem_bytes, const int32_t *__restrict__ accept_path,
                 const int32_t *__restrict__ accept_len, uint8_t *__restrict__ k_cache,
                 uint8_t *__restrict__ v_cache, int32_t *__restrict__ new_prefix_lens,
                 int32_t *__restrict__ err_flag)
{
    __shared__ int32_t path[LS_MAX_TREE];
    __shared__ int32_t n_sh;
    const int b = blockIdx.x / p.n_kv_heads;
    const int g = blockIdx.x % p.n_kv_heads;
    const int tid = threadIdx.x;

    int plen = p.prefix_lens[b];
    plen = plen < 0 ? 0 : (plen > p.max_prefix_len ? p.max_prefix_len : plen);
    int want = accept_len[b];
    want = want < 0 ? 0 : (want > p.n_tree ? p.n_tree : want);
    int room = p.max_prefix_len - plen;
    int n = want < room ? want : room;
    if (tid == 0) n_sh = n;
    __syncthreads();
    for (int t = tid; t < n; t += blockDim.x) {
        const int32_t node = accept_path[(size_t)b * p.n_tree + t];
        path[t] = node;
        if (node < 0 || node >= p.n_tree) atomicMin(&n_sh, t);  // stop before the first bad entry
    }
    __syncthreads();
    n = n_sh;

    const int chunks = p.head_dim * elem_bytes / 16;  // 16-byte pieces per row
    const uint8_t *kt = (const uint8_t *)p.k_tree + (b * p.kt_stride[0] + g * p.kt_stride[1]) * elem_bytes;
    const uint8_t *vt = (const uint8_t *)p.v_tree + (b * p.vt_stride[0] + g * p.vt_stride[1]) * elem_bytes;
    // contiguous cache: first index = sequence; paged cache: first index = page, found per row
    const int32_t *tab = p.block_table ? p.block_table + (size_t)b * p.bt_stride : nullptr;
    const int page_rows_mask = (1 << p.page_shift) - 1;
    for (int e = tid; e < n * chunks; e += blockDim.x) {
        const int j = e / chunks, c = e % chunks;
        const int64_t node = path[j];
        const int row = plen + j;  // < max_prefix_len <= bt_stride * page size
        const int64_t first = tab ? (int64_t)tab[row >> p.page_shift] : (int64_t)b;
        const int64_t in_row = tab ? (row & page_rows_mask) : row;
        const uint4 kv = *(const uint4 *)(kt + node * p.kt_stride[2] * elem_bytes + c * 16);
        const uint4 vv = *(const uint4 *)(vt + node * p.vt_stride[2] * elem_bytes + c * 16);
        *(uint4 *)(k_cache + (first * p.kc_stride[0] + g * p.kc_stride[1] + in_row * p.kc_stride[2]) * elem_bytes +
                   c * 16) = kv;
        *(uint4 *)(v_cache + (first * p.vc_stride[0] + g * p.vc_stride[1] + in_row * p.vc_stride[2]) * elem_bytes +
                   c * 16) = vv;
    }
    if (g == 0 && tid == 0) {
        if (new_prefix_lens) new_prefix_lens[b] = plen + n;
        if (err_flag) err_flag[b] = n < accept_len[b] ? 1 : 0;
    }
}

}  // namespace

hipError_t launch_tree_accept(const int32_t *parents, const int32_t *draft_tokens, const int32_t *target_tokens,
                              int32_t batch, int32_t n_tree, int32_t *accept_path, int32_t *accept_len,
                              int32_t *next_token, int32_t *err_flag, hipStream_t stream)
{
    const int threads = n_tree <= 64 ? 64 : (n_tree <= 128 ? 128 : 256);
    hipLaunchKernelGGL(tree_accept_kernel, dim3(batch), dim3(threads), 0, stream, parents, draft_tokens,
                       target_tokens, n_tree, accept_path, accept_len, next_token, err_flag);
    return hipGetLastError();
}

hipError_t launch_kv_commit(const Problem &p, int dtype, const int32_t *accept_path, const int32_t *accept_len,
                            void *k_cache, void *v_cache, int32_t *new_prefix_lens, int32_t *err_flag,
                            hipStream_t stream)
{
    const int elem_bytes = is_16bit(dtype) ? 2 : 4;
    hipLaunchKernelGGL(kv_commit_kernel, dim3(p.batch * p.n_kv_heads), dim3(256), 0, stream, p, elem_bytes,
                       accept_path, accept_len, (uint8_t *)k_cache, (uint8_t *)v_cache, new_prefix_lens, err_flag);
    return hipGetLastError();
}

}  // namespace ls
