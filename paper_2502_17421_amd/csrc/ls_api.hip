// Host side of the C ABI declared in include/ls_attn.h: argument checks, split planning,
// workspace layout and kernel dispatch.  No device memory is allocated here.
#include <cmath>
#include <cstring>
#include <mutex>

#include "ls_internal.hpp"

// Workspace of ls_hybrid_tree_attn_static: one array per GPU, part of the loaded code object and
// held until the process ends.  In host code the array's name only identifies the symbol; the
// memory is reached through the per-device address that hipGetSymbolAddress returns.
static __device__ __align__(256) unsigned char scratch[LS_STATIC_SCRATCH_BYTES];

namespace ls {

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

inline size_t elem_size(int dtype) { return is_16bit(dtype) ? 2 : 4; }

int check_stride(const int64_t s[3], int head_dim, size_t esz, bool is_output)
{
    for (int a = 0; a < 3; ++a) {
        if (s[a] < 0) return LS_ERR_STRIDE;
        if ((size_t)s[a] * esz % 16 != 0) return LS_ERR_STRIDE;
    }
    if (s[2] < head_dim) return LS_ERR_STRIDE;
    if (is_output && (s[0] <= 0 || s[1] <= 0)) return LS_ERR_STRIDE;
    return LS_OK;
}

int validate(const ls_desc *d)
{
    if (!d) return LS_ERR_NULL;
    if (d->batch <= 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0 || d->n_tree <= 0 ||
        d->max_prefix_len < 0)
        return LS_ERR_SHAPE;
    if (d->n_q_heads % d->n_kv_heads != 0) return LS_ERR_SHAPE;
    if (d->dtype != LS_BF16 && d->dtype != LS_F32 && d->dtype != LS_F16) return LS_ERR_DTYPE;
    if (!(d->softmax_scale >= 0.f) || std::isinf(d->softmax_scale)) return LS_ERR_SHAPE;
    if (d->head_dim != 64 && d->head_dim != 128) return LS_ERR_UNSUPPORTED;
    if (d->n_tree > LS_MAX_TREE) return LS_ERR_UNSUPPORTED;
    if ((int64_t)d->batch * d->n_kv_heads > 65535) return LS_ERR_UNSUPPORTED;
    if ((int64_t)d->batch * d->n_q_heads * d->n_tree > (1 << 24)) return LS_ERR_UNSUPPORTED;
    const size_t esz = elem_size(d->dtype);
    int rc;
    if ((rc = check_stride(d->q_stride, d->head_dim, esz, false))) return rc;
    if ((rc = check_stride(d->o_stride, d->head_dim, esz, true))) return rc;
    if ((rc = check_stride(d->kc_stride, d->head_dim, esz, false))) return rc;
    if ((rc = check_stride(d->vc_stride, d->head_dim, esz, false))) return rc;
    if ((rc = check_stride(d->kt_stride, d->head_dim, esz, false))) return rc;
    if ((rc = check_stride(d->vt_stride, d->head_dim, esz, false))) return rc;
    return LS_OK;
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

Problem make_problem(const ls_desc &d, const void *q, const void *kc, const void *vc, const int32_t *plens,
                     const void *kt, const void *vt)
{
    Problem p;
    std::memset(&p, 0, sizeof(p));
    p.q = q;
    p.k_cache = kc;
    p.v_cache = vc;
    p.k_tree = kt;
    p.v_tree = vt;
    p.prefix_lens = plens;
    p.prefix_len_all = d.max_prefix_len;
    p.batch = d.batch;
    p.n_q_heads = d.n_q_heads;
    p.n_kv_heads = d.n_kv_heads;
    p.group = d.n_q_heads / d.n_kv_heads;
    p.head_dim = d.head_dim;
    p.n_tree = d.n_tree;
    p.max_prefix_len = d.max_prefix_len;
    const float scale = d.softmax_scale > 0.f ? d.softmax_scale : 1.0f / std::sqrt((float)d.head_dim);
    p.scale_log2 = scale * kLog2e;
    for (int a = 0; a < 3; ++a) {
        p.q_stride[a] = d.q_stride[a];
        p.kc_stride[a] = d.kc_stride[a];
        p.vc_stride[a] = d.vc_stride[a];
        p.kt_stride[a] = d.kt_stride[a];
        p.vt_stride[a] = d.vt_stride[a];
    }
    return p;
}

int compute_units()
{
    static int cached = 0;
    if (cached) return cached;
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
        cached = n;
    else {
        (void)hipGetLastError();
        return 256;  // MI355X; not cached so a later call with a device present asks again
    }
    return cached;
}

// The first bytes of every workspace are the arrival counters of the single-launch call, at a
// place that does not depend on the problem: one ls_workspace_init serves every later call.
constexpr size_t kArrivalBytes = (size_t)kMaxArrivalCounters * kCounterWords * sizeof(uint64_t);
static_assert(kArrivalBytes == LS_WORKSPACE_COUNTER_BYTES, "the header states the size");

// Polls a workgroup of the single-launch call spends waiting for the rest of its (sequence, KV
// head, query block) before it leaves its rows to the last one: about 20 ms.  Waiting makes sense
// only when every workgroup of the launch has a compute unit of its own from the start.
constexpr int32_t kDefaultSpinPolls = 40000;
int32_t g_spin_polls = -1;  // < 0: the default

struct Workspace {
    size_t off_mask, off_err, off_lse, off_o, total;
    int32_t n_parts;
};

Workspace layout(const ls_desc &d, const SplitPlan &plan)
{
    Workspace w;
    const size_t words = (d.n_tree + 63) / 64;
    w.n_parts = plan.n_splits;
    const size_t rows = (size_t)d.batch * d.n_q_heads * w.n_parts * d.n_tree;
    w.off_mask = align_up(kArrivalBytes);
    w.off_err = align_up(w.off_mask + (size_t)d.batch * d.n_tree * words * sizeof(uint64_t));
    w.off_lse = align_up(w.off_err + (size_t)d.batch * sizeof(int32_t));
    w.off_o = align_up(w.off_lse + rows * sizeof(float));
    w.total = align_up(w.off_o + rows * d.head_dim * elem_size(d.dtype));
    return w;
}

}  // namespace

namespace {

constexpr int kMaxDevices = 64;

// Device address of `scratch` on the current device; looked up once per device, with that
// device current.  Returns nullptr (and leaves *dev_out unset) when HIP reports an error.
void *static_scratch_of_current_device()
{
    static std::mutex lock;
    static void *ptr_of[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    std::lock_guard<std::mutex> guard(lock);
    if (!ptr_of[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(::scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptr_of[dev] = ptr;
    }
    return ptr_of[dev];
}

}  // namespace

// Split schedule.  The cached keys of every sequence are cut into pieces of split_len rows
// (a multiple of 64); the grid is sized for max_prefix_len.  Left to the library, the count S
// minimises a modelled time.  Float path: units*S workgroups run in ceil(units*S / slots)
// rounds of max_prefix_len / S keys each, plus a small charge per split.  MFMA path: the
// time of the whole call, cached-key kernel plus the kernel that merges the S parts of every
// row, from figures measured on MI355X (microseconds; f = share of the compute units the
// launch occupies, tiles of 32 keys):
//   kernel = start-up + (rounds - 1) * 5 + rounds * tiles per workgroup * time per tile
//     query blocks of 256 rows: start-up 10.5 up to f = 1/2 and 13 at f = 1, a tile 0.60 and 0.84
//       (the matrix cores are power-limited: half the compute units get through a tile in 0.7
//       of the time that all of them take, so the second half of the chip buys 1.4x, not 2x)
//     query blocks of 128 rows: start-up 6.7 + 1.8 f, a tile 0.50 up to f = 1/2, 0.66 at f = 1
//       (the HBM rate)
//   merge  = 7 + bytes of the partial rows / 3.5 TB/s
// With it a 2048-row call over 8 KV heads takes 16 splits up to about 12k cached keys and 32
// beyond 20k (measured: 8k keys 28.9 against 32.2 us, 12k 32.9 against 39.1, 24k 47.9 against
// 45.7), because every split adds a partial row per query row to write and to merge.
SplitPlan plan_splits(const ls_desc &d, int32_t request)
{
    constexpr int kTile = 64;
    SplitPlan plan;
    const int64_t max_p = d.max_prefix_len;
    int64_t s = request;
    if (s <= 0) {
        const int group = d.n_q_heads / d.n_kv_heads;
        const int rows_kv = group * d.n_tree;
        const int rows_wg = is_16bit(d.dtype) ? kPrefixRowsPerWorkgroup : 32;
        const int64_t units = (int64_t)d.batch * d.n_kv_heads * ((rows_kv + rows_wg - 1) / rows_wg);
        const int64_t slots = (int64_t)compute_units() * (is_16bit(d.dtype) ? kPrefixWorkgroupsPerCU : 1);
        // a split is at least 64 keys (a 512-key window measured 12.8 us in two splits, 10.1 in
        // four and 8.75 in eight: the start-up of a workgroup costs more than its few tiles)
        int64_t s_max = max_p / kTile;
        if (s_max > 64) s_max = 64;
        if (s_max < 1) s_max = 1;
        double best = 0.0;
        bool have = false;
        s = 1;
        const bool mfma = is_16bit(d.dtype);
        const bool heavy = rows_kv > kPrefixRowsPerWorkgroup / 2;
        const double rows_total = (double)d.batch * d.n_q_heads * d.n_tree;
        for (int64_t cand = 1; cand <= s_max; ++cand) {
            int64_t len_c = ((max_p + cand - 1) / cand + kTile - 1) / kTile * kTile;
            if (len_c < kTile) len_c = kTile;
            int64_t n_c = (max_p + len_c - 1) / len_c;  // the count this candidate ends up with
            if (n_c < 1) n_c = 1;
            const int64_t rounds = (units * n_c + slots - 1) / slots;
            double cost;
            if (!mfma) {
                cost = (double)rounds / (double)cand + 0.0005 * (double)cand;
            } else {
                const double f = rounds > 1 ? 1.0 : (double)(units * n_c) / (double)slots;
                const double over = f > 0.5 ? f - 0.5 : 0.0;
                const double tile = heavy ? 0.60 + 0.48 * over : 0.50 + 0.32 * over;
                const double start = heavy ? 10.5 + 5.0 * over : 6.7 + 1.8 * f;
                const double kernel = start + 5.0 * (double)(rounds - 1) + (double)rounds * (double)(len_c / 32) * tile;
                const double merge = 7.0 + rows_total * (double)n_c * d.head_dim * 2.0 / 3.5e6;
                cost = kernel + merge;
            }
            if (mfma && len_c > kMaxSplitLen && cand < s_max) continue;  // longer than a split may be (below)
            // more splits only for a modelled gain that is more than noise (0.05 us; the float path's
            // cost is a ratio, of order 1/S)
            if (!have || cost < best - (mfma ? 0.05 : 1e-9)) {
                have = true;
                best = cost;
                s = cand;
            }
        }
    }
    // the MFMA kernel keeps the page ids of a split in registers, which bounds a split's length;
    // the bound is applied to contiguous caches too, so that one plan serves both layouts
    if (request <= 0 && is_16bit(d.dtype) && (max_p + s - 1) / s > kMaxSplitLen) s = (max_p + kMaxSplitLen - 1) / kMaxSplitLen;
    int64_t len = (max_p + s - 1) / s;
    len = (len + kTile - 1) / kTile * kTile;
    if (len < kTile) len = kTile;
    if (request <= 0) {
        s = (max_p + len - 1) / len;
        if (s < 1) s = 1;
    }
    plan.n_splits = (int32_t)s;
    plan.split_len = (int32_t)len;
    plan.per_sequence = 0;
    plan.reserved = 0;
    return plan;
}

// Schedule of the whole-path calls: as many pieces as the stand-alone cached-key call would cut,
// but on the MFMA path every sequence cuts its own length into that many (SplitPlan::per_sequence).
SplitPlan plan_call(const ls_desc &d)
{
    SplitPlan plan = plan_splits(d, 0);
    plan.per_sequence = is_16bit(d.dtype) ? 1 : 0;
    return plan;
}

}  // namespace ls

using namespace ls;

extern "C" {

int ls_version(void) { return 100; }

const char *ls_status_string(int status)
{
    switch (status) {
    case LS_OK: return "ok";
    case LS_ERR_NULL: return "a required pointer is NULL";
    case LS_ERR_SHAPE: return "a size is non-positive or inconsistent";
    case LS_ERR_DTYPE: return "unknown dtype";
    case LS_ERR_STRIDE: return "stride or pointer breaks the 16-byte row alignment";
    case LS_ERR_TREE: return "parents is not a topologically ordered forest";
    case LS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case LS_ERR_HIP: return "HIP reported a launch error";
    case LS_ERR_UNSUPPORTED: return "request outside the supported set";
    default: return "unknown status";
    }
}

int ls_validate_desc(const ls_desc *desc) { return validate(desc); }

int ls_validate_parents_host(const int32_t *parents, int32_t batch, int32_t n_tree)
{
    if (!parents) return LS_ERR_NULL;
    if (batch <= 0 || n_tree <= 0) return LS_ERR_SHAPE;
    for (int32_t b = 0; b < batch; ++b)
        for (int32_t i = 0; i < n_tree; ++i) {
            const int32_t p = parents[(size_t)b * n_tree + i];
            if (p < -1 || p >= i) return LS_ERR_TREE;
        }
    return LS_OK;
}

int ls_prefix_num_splits(const ls_desc *desc, int32_t *n_splits_out)
{
    if (!n_splits_out) return LS_ERR_NULL;
    const int rc = validate(desc);
    if (rc) return rc;
    *n_splits_out = plan_splits(*desc, 0).n_splits;
    return LS_OK;
}

int ls_prefix_split_len(const ls_desc *desc, int32_t n_splits, int32_t *split_len_out)
{
    if (!split_len_out) return LS_ERR_NULL;
    const int rc = validate(desc);
    if (rc) return rc;
    if (n_splits < 0) return LS_ERR_SHAPE;
    *split_len_out = plan_splits(*desc, n_splits).split_len;
    return LS_OK;
}

int ls_workspace_bytes(const ls_desc *desc, size_t *bytes_out)
{
    if (!bytes_out) return LS_ERR_NULL;
    const int rc = validate(desc);
    if (rc) return rc;
    *bytes_out = layout(*desc, plan_call(*desc)).total;
    return LS_OK;
}

int ls_workspace_error(const ls_desc *desc, void *workspace, int32_t **err_out)
{
    if (!workspace || !err_out) return LS_ERR_NULL;
    const int rc = validate(desc);
    if (rc) return rc;
    *err_out = (int32_t *)((char *)workspace + layout(*desc, plan_call(*desc)).off_err);
    return LS_OK;
}

int ls_build_tree_mask(const int32_t *parents, int32_t batch, int32_t n_tree, uint64_t *mask,
                       int32_t *err_flag, void *stream)
{
    if (!parents || !mask) return LS_ERR_NULL;
    if (batch <= 0 || n_tree <= 0) return LS_ERR_SHAPE;
    if (n_tree > LS_MAX_TREE || batch > 65535) return LS_ERR_UNSUPPORTED;
    return launch_tree_mask(parents, batch, n_tree, mask, err_flag, (hipStream_t)stream) == hipSuccess
               ? LS_OK
               : LS_ERR_HIP;
}

int ls_prefix_attn_splitkv(const ls_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *prefix_lens, int32_t n_splits, int32_t part_dtype, void *o_part,
                           float *lse_part, void *stream)
{
    const int rc = validate(desc);
    if (rc) return rc;
    if (!q || !prefix_lens || !o_part || !lse_part) return LS_ERR_NULL;
    if (desc->max_prefix_len > 0 && (!k_cache || !v_cache)) return LS_ERR_NULL;
    if (n_splits < 0 || n_splits > 65535) return LS_ERR_SHAPE;
    if (part_dtype != LS_F32 && !(is_16bit(part_dtype) && part_dtype == desc->dtype)) return LS_ERR_DTYPE;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(o_part)) return LS_ERR_STRIDE;
    const SplitPlan plan = plan_splits(*desc, n_splits);
    const Problem p = make_problem(*desc, q, k_cache, v_cache, prefix_lens, nullptr, nullptr);
    const Partials out{o_part, lse_part, plan.n_splits, 0, is_16bit(part_dtype)};
    hipError_t e;
    if (prefix_mfma_supports(p, desc->dtype)) {
        e = launch_prefix_mfma(p, desc->dtype, plan, out, MaskJob{nullptr, nullptr, nullptr}, FusedTail{}, (hipStream_t)stream);
    } else {
        if (part_dtype != LS_F32) return LS_ERR_UNSUPPORTED;
        e = launch_prefix_valu(p, desc->dtype, plan, out, MaskJob{nullptr, nullptr, nullptr}, (hipStream_t)stream);
    }
    return e == hipSuccess ? LS_OK : LS_ERR_HIP;
}

int ls_tree_attn_masked(const ls_desc *desc, const void *q, const void *k_tree, const void *v_tree,
                        const uint64_t *mask, float *o_tree, float *lse_tree, void *stream)
{
    const int rc = validate(desc);
    if (rc) return rc;
    if (!q || !k_tree || !v_tree || !mask || !o_tree || !lse_tree) return LS_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_tree) || !aligned16(v_tree) || !aligned16(o_tree)) return LS_ERR_STRIDE;
    const Problem p = make_problem(*desc, q, nullptr, nullptr, nullptr, k_tree, v_tree);
    const Partials out{o_tree, lse_tree, 1, 0, 0};
    return launch_tree_attn(p, desc->dtype, mask, out, (hipStream_t)stream) == hipSuccess ? LS_OK : LS_ERR_HIP;
}

int ls_lse_merge(const ls_desc *desc, int32_t n_parts, int32_t part_dtype, const void *o_parts,
                 const float *lse_parts, void *out, float *lse, void *stream)
{
    const int rc = validate(desc);
    if (rc) return rc;
    if (!o_parts || !lse_parts || !out || !lse) return LS_ERR_NULL;
    if (n_parts <= 0) return LS_ERR_SHAPE;
    if (part_dtype != LS_F32 && !(is_16bit(part_dtype) && part_dtype == desc->dtype)) return LS_ERR_DTYPE;
    if (!aligned16(o_parts) || !aligned16(out)) return LS_ERR_STRIDE;
    return launch_merge(desc->batch, desc->n_q_heads, desc->n_tree, desc->head_dim, desc->dtype, n_parts, o_parts,
                        is_16bit(part_dtype), lse_parts, out, desc->o_stride, lse, (hipStream_t)stream) == hipSuccess
               ? LS_OK
               : LS_ERR_HIP;
}

}  // extern "C"

namespace {
// The whole path for a contiguous cache.  prefix_lens: device array, or nullptr with every
// sequence holding prefix_len_all cached rows.
int hybrid_contiguous(const ls_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                      const int32_t *prefix_lens, int32_t prefix_len_all, const void *k_tree, const void *v_tree,
                      const int32_t *parents, void *out, float *lse, void *workspace, size_t workspace_bytes,
                      void *stream, bool single_launch = false)
{
    const int rc = validate(desc);
    if (rc) return rc;
    if (!q || !k_tree || !v_tree || !parents || !out || !lse) return LS_ERR_NULL;
    if (desc->max_prefix_len > 0 && (!k_cache || !v_cache)) return LS_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_tree) || !aligned16(v_tree) ||
        !aligned16(out))
        return LS_ERR_STRIDE;
    const SplitPlan plan = plan_call(*desc);
    const Workspace w = layout(*desc, plan);
    if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < w.total) return LS_ERR_WORKSPACE;

    char *base = (char *)workspace;
    uint64_t *mask = (uint64_t *)(base + w.off_mask);
    int32_t *err = (int32_t *)(base + w.off_err);
    float *lse_parts = (float *)(base + w.off_lse);
    void *o_parts = base + w.off_o;
    hipStream_t s = (hipStream_t)stream;
    Problem p = make_problem(*desc, q, k_cache, v_cache, prefix_lens, k_tree, v_tree);
    p.prefix_len_all = prefix_len_all;

    // (b) cached keys -> parts [0, n_splits), stored in the problem's dtype; on the MFMA path
    // the same launch carries the workgroups of (a), the tree mask
    const Partials cache_out{o_parts, lse_parts, w.n_parts, 0, is_16bit(desc->dtype), 1};
    if (prefix_mfma_supports(p, desc->dtype)) {
        // Single launch: the last workgroup of each (sequence, KV head, query block) does (c) and (d)
        // for that block's rows; the mask workgroups still fill the workspace's mask and error words.
        const bool fused =
            single_launch && plan.n_splits <= 64 &&
            (int64_t)desc->batch * desc->n_kv_heads * prefix_mfma_query_blocks(p) <= kMaxArrivalCounters;
        FusedTail tail{};
        if (fused) {
            tail.counters = (uint64_t *)base;
            const int64_t n_workgroups =
                (int64_t)desc->batch * desc->n_kv_heads * prefix_mfma_query_blocks(p) * plan.n_splits;
            tail.spin_limit = n_workgroups <= compute_units() ? (g_spin_polls < 0 ? kDefaultSpinPolls : g_spin_polls) : 0;
            tail.parents = parents;
            tail.out = out;
            for (int i = 0; i < 3; ++i) tail.o_stride[i] = desc->o_stride[i];
            tail.lse = lse;
        }
        if (launch_prefix_mfma(p, desc->dtype, plan, cache_out, MaskJob{parents, mask, err}, tail, s) != hipSuccess)
            return LS_ERR_HIP;
        if (fused) return LS_OK;
    } else {
        const Partials f32_out{o_parts, lse_parts, w.n_parts, 0, 0, 1};
        if (is_16bit(desc->dtype)) return LS_ERR_UNSUPPORTED;  // 16-bit row strides beyond the MFMA kernel's range
        // the mask rides on the same launch when its grid slice has a workgroup per sequence
        const int n_qblocks = (p.group * p.n_tree + 31) / 32;
        const bool ride = (int64_t)plan.n_splits * n_qblocks >= desc->batch;
        if (launch_prefix_valu(p, desc->dtype, plan, f32_out, ride ? MaskJob{parents, mask, err} : MaskJob{nullptr, nullptr, nullptr}, s) != hipSuccess)
            return LS_ERR_HIP;
        if (!ride && launch_tree_mask(parents, desc->batch, desc->n_tree, mask, err, s) != hipSuccess) return LS_ERR_HIP;
    }
    // (c) tree keys and (d) merge, one wavefront per query row
    if (launch_tree_merge(p, desc->dtype, mask, cache_out, plan.n_splits, out, desc->o_stride, lse, s) != hipSuccess)
        return LS_ERR_HIP;
    return LS_OK;
}
}  // namespace

extern "C" {

int ls_hybrid_tree_attn(const ls_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                        const int32_t *prefix_lens, const void *k_tree, const void *v_tree,
                        const int32_t *parents, void *out, float *lse, void *workspace, size_t workspace_bytes,
                        void *stream)
{
    if (!prefix_lens) return LS_ERR_NULL;
    return hybrid_contiguous(desc, q, k_cache, v_cache, prefix_lens, 0, k_tree, v_tree, parents, out, lse, workspace,
                             workspace_bytes, stream);
}

int ls_hybrid_tree_attn_single(const ls_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                               int32_t prefix_len, const void *k_tree, const void *v_tree, const int32_t *parents,
                               void *out, float *lse, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!desc) return LS_ERR_NULL;
    if (desc->batch != 1 || prefix_len < 0 || prefix_len > desc->max_prefix_len) return LS_ERR_SHAPE;
    return hybrid_contiguous(desc, q, k_cache, v_cache, nullptr, prefix_len, k_tree, v_tree, parents, out, lse,
                             workspace, workspace_bytes, stream);
}

int ls_hybrid_tree_attn_static(const ls_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                               const int32_t *prefix_lens, const void *k_tree, const void *v_tree,
                               const int32_t *parents, void *out, float *lse, void *stream)
{
    if (!prefix_lens) return LS_ERR_NULL;
    const int rc = validate(desc);
    if (rc) return rc;
    // the size check comes first: a problem that does not fit is refused whatever the device says
    if (layout(*desc, plan_call(*desc)).total > (size_t)LS_STATIC_SCRATCH_BYTES) return LS_ERR_WORKSPACE;
    void *ws = static_scratch_of_current_device();
    if (!ws) return LS_ERR_HIP;
    return hybrid_contiguous(desc, q, k_cache, v_cache, prefix_lens, 0, k_tree, v_tree, parents, out, lse, ws,
                             (size_t)LS_STATIC_SCRATCH_BYTES, stream);
}

int ls_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < kArrivalBytes) return LS_ERR_WORKSPACE;
    return launch_clear_words((uint32_t *)workspace, (int32_t)(kArrivalBytes / sizeof(uint32_t)), (hipStream_t)stream) ==
                   hipSuccess
               ? LS_OK
               : LS_ERR_HIP;
}

int ls_set_single_launch_polls(int32_t polls)
{
    if (polls > (1 << 24)) return LS_ERR_SHAPE;
    g_spin_polls = polls;
    return LS_OK;
}

int ls_hybrid_tree_attn_fused(const ls_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                              const int32_t *prefix_lens, const void *k_tree, const void *v_tree,
                              const int32_t *parents, void *out, float *lse, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    if (!prefix_lens) return LS_ERR_NULL;
    return hybrid_contiguous(desc, q, k_cache, v_cache, prefix_lens, 0, k_tree, v_tree, parents, out, lse, workspace,
                             workspace_bytes, stream, true);
}

int ls_cache_attn(const ls_desc *desc, const void *q, const void *k_cache, const void *v_cache,
                  const int32_t *prefix_lens, void *out, float *lse, void *workspace, size_t workspace_bytes,
                  void *stream)
{
    const int rc = validate(desc);
    if (rc) return rc;
    if (!q || !prefix_lens || !out || !lse) return LS_ERR_NULL;
    if (desc->max_prefix_len > 0 && (!k_cache || !v_cache)) return LS_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return LS_ERR_STRIDE;
    const SplitPlan plan = plan_call(*desc);
    const Workspace w = layout(*desc, plan);
    if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < w.total) return LS_ERR_WORKSPACE;
    char *base = (char *)workspace;
    float *lse_parts = (float *)(base + w.off_lse);
    void *o_parts = base + w.off_o;
    hipStream_t s = (hipStream_t)stream;
    const Problem p = make_problem(*desc, q, k_cache, v_cache, prefix_lens, nullptr, nullptr);
    const bool mfma = prefix_mfma_supports(p, desc->dtype);
    if (!mfma && is_16bit(desc->dtype)) return LS_ERR_UNSUPPORTED;
    const Partials parts{o_parts, lse_parts, w.n_parts, 0, is_16bit(desc->dtype), 1};
    const hipError_t e = mfma ? launch_prefix_mfma(p, desc->dtype, plan, parts, MaskJob{nullptr, nullptr, nullptr}, FusedTail{}, s)
                              : launch_prefix_valu(p, desc->dtype, plan, parts, MaskJob{nullptr, nullptr, nullptr}, s);
    if (e != hipSuccess) return LS_ERR_HIP;
    // the tail kernel without a mask: merge of the split partials only
    if (launch_tree_merge(p, desc->dtype, nullptr, parts, plan.n_splits, out, desc->o_stride, lse, s) != hipSuccess)
        return LS_ERR_HIP;
    return LS_OK;
}

int ls_tree_accept_greedy(const int32_t *parents, const int32_t *draft_tokens, const int32_t *target_tokens,
                          int32_t batch, int32_t n_tree, int32_t *accept_path, int32_t *accept_len,
                          int32_t *next_token, int32_t *err_flag, void *stream)
{
    if (!parents || !draft_tokens || !target_tokens || !accept_path || !accept_len || !next_token) return LS_ERR_NULL;
    if (batch <= 0 || n_tree <= 0) return LS_ERR_SHAPE;
    if (n_tree > LS_MAX_TREE || batch > 65535) return LS_ERR_UNSUPPORTED;
    return launch_tree_accept(parents, draft_tokens, target_tokens, batch, n_tree, accept_path, accept_len, next_token,
                              err_flag, (hipStream_t)stream) == hipSuccess
               ? LS_OK
               : LS_ERR_HIP;
}

int ls_kv_commit(const ls_desc *desc, const void *k_tree, const void *v_tree, const int32_t *accept_path,
                 const int32_t *accept_len, const int32_t *prefix_lens, void *k_cache, void *v_cache,
                 int32_t *new_prefix_lens, int32_t *err_flag, void *stream)
{
    const int rc = validate(desc);
    if (rc) return rc;
    if (!k_tree || !v_tree || !accept_path || !accept_len || !prefix_lens || !k_cache || !v_cache) return LS_ERR_NULL;
    if (new_prefix_lens == prefix_lens) return LS_ERR_NULL;
    if (!aligned16(k_tree) || !aligned16(v_tree) || !aligned16(k_cache) || !aligned16(v_cache)) return LS_ERR_STRIDE;
    if ((int64_t)desc->batch * desc->n_kv_heads > 0x7fffffff) return LS_ERR_UNSUPPORTED;
    const Problem p = make_problem(*desc, nullptr, k_cache, v_cache, prefix_lens, k_tree, v_tree);
    return launch_kv_commit(p, desc->dtype, accept_path, accept_len, k_cache, v_cache, new_prefix_lens, err_flag,
                            (hipStream_t)stream) == hipSuccess
               ? LS_OK
               : LS_ERR_HIP;
}

namespace {

// page_size: a power of two >= 16; the table must cover max_prefix_len rows
int check_paging(const ls_desc *desc, const int32_t *block_table, int32_t bt_stride, int32_t page_size)
{
    if (!block_table) return LS_ERR_NULL;
    if (page_size <= 0 || bt_stride <= 0) return LS_ERR_SHAPE;
    if (page_size < 16 || (page_size & (page_size - 1)) != 0) return LS_ERR_UNSUPPORTED;
    if ((int64_t)bt_stride * page_size < desc->max_prefix_len) return LS_ERR_SHAPE;
    if (!is_16bit(desc->dtype)) return LS_ERR_UNSUPPORTED;  // the float kernel reads contiguous caches only
    return LS_OK;
}

int page_shift_of(int32_t page_size)
{
    int s = 0;
    while ((1 << s) < page_size) ++s;
    return s;
}

}  // namespace

int ls_hybrid_tree_attn_paged(const ls_desc *desc, const void *q, const void *k_pages, const void *v_pages,
                              const int32_t *block_table, int32_t bt_stride, int32_t page_size,
                              const int32_t *prefix_lens, const void *k_tree, const void *v_tree,
                              const int32_t *parents, void *out, float *lse, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    int rc = validate(desc);
    if (rc) return rc;
    if (!q || !prefix_lens || !k_tree || !v_tree || !parents || !out || !lse) return LS_ERR_NULL;
    if (desc->max_prefix_len > 0 && (!k_pages || !v_pages)) return LS_ERR_NULL;
    if ((rc = check_paging(desc, block_table, bt_stride, page_size))) return rc;
    if (!aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages) || !aligned16(k_tree) || !aligned16(v_tree) ||
        !aligned16(out))
        return LS_ERR_STRIDE;
    const SplitPlan plan = plan_call(*desc);
    const Workspace w = layout(*desc, plan);
    if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < w.total) return LS_ERR_WORKSPACE;
    if (plan.split_len > kMaxSplitLen) return LS_ERR_UNSUPPORTED;
    char *base = (char *)workspace;
    uint64_t *mask = (uint64_t *)(base + w.off_mask);
    int32_t *err = (int32_t *)(base + w.off_err);
    Problem p = make_problem(*desc, q, k_pages, v_pages, prefix_lens, k_tree, v_tree);
    p.block_table = block_table;
    p.bt_stride = bt_stride;
    p.page_shift = page_shift_of(page_size);
    if (!prefix_mfma_supports(p, desc->dtype)) return LS_ERR_UNSUPPORTED;
    const Partials parts{base + w.off_o, (float *)(base + w.off_lse), w.n_parts, 0, 1, 1};
    hipStream_t s = (hipStream_t)stream;
    if (launch_prefix_mfma(p, desc->dtype, plan, parts, MaskJob{parents, mask, err}, FusedTail{}, s) != hipSuccess) return LS_ERR_HIP;
    if (launch_tree_merge(p, desc->dtype, mask, parts, plan.n_splits, out, desc->o_stride, lse, s) != hipSuccess)
        return LS_ERR_HIP;
    return LS_OK;
}

int ls_cache_attn_paged(const ls_desc *desc, const void *q, const void *k_pages, const void *v_pages,
                        const int32_t *block_table, int32_t bt_stride, int32_t page_size, const int32_t *prefix_lens,
                        void *out, float *lse, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = validate(desc);
    if (rc) return rc;
    if (!q || !prefix_lens || !out || !lse) return LS_ERR_NULL;
    if (desc->max_prefix_len > 0 && (!k_pages || !v_pages)) return LS_ERR_NULL;
    if ((rc = check_paging(desc, block_table, bt_stride, page_size))) return rc;
    if (!aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages) || !aligned16(out)) return LS_ERR_STRIDE;
    const SplitPlan plan = plan_call(*desc);
    const Workspace w = layout(*desc, plan);
    if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < w.total) return LS_ERR_WORKSPACE;
    if (plan.split_len > kMaxSplitLen) return LS_ERR_UNSUPPORTED;
    char *base = (char *)workspace;
    Problem p = make_problem(*desc, q, k_pages, v_pages, prefix_lens, nullptr, nullptr);
    p.block_table = block_table;
    p.bt_stride = bt_stride;
    p.page_shift = page_shift_of(page_size);
    if (!prefix_mfma_supports(p, desc->dtype)) return LS_ERR_UNSUPPORTED;
    const Partials parts{base + w.off_o, (float *)(base + w.off_lse), w.n_parts, 0, 1, 1};
    hipStream_t s = (hipStream_t)stream;
    if (launch_prefix_mfma(p, desc->dtype, plan, parts, MaskJob{nullptr, nullptr, nullptr}, FusedTail{}, s) != hipSuccess)
        return LS_ERR_HIP;
    if (launch_tree_merge(p, desc->dtype, nullptr, parts, plan.n_splits, out, desc->o_stride, lse, s) != hipSuccess)
        return LS_ERR_HIP;
    return LS_OK;
}

int ls_kv_commit_paged(const ls_desc *desc, const void *k_tree, const void *v_tree, const int32_t *accept_path,
                       const int32_t *accept_len, const int32_t *prefix_lens, void *k_pages, void *v_pages,
                       const int32_t *block_table, int32_t bt_stride, int32_t page_size, int32_t *new_prefix_lens,
                       int32_t *err_flag, void *stream)
{
    int rc = validate(desc);
    if (rc) return rc;
    if (!k_tree || !v_tree || !accept_path || !accept_len || !prefix_lens || !k_pages || !v_pages) return LS_ERR_NULL;
    if (new_prefix_lens == prefix_lens) return LS_ERR_NULL;
    if (!block_table) return LS_ERR_NULL;
    if (page_size <= 0 || bt_stride <= 0) return LS_ERR_SHAPE;
    if ((page_size & (page_size - 1)) != 0) return LS_ERR_UNSUPPORTED;
    if ((int64_t)bt_stride * page_size < desc->max_prefix_len) return LS_ERR_SHAPE;
    if (!aligned16(k_tree) || !aligned16(v_tree) || !aligned16(k_pages) || !aligned16(v_pages)) return LS_ERR_STRIDE;
    Problem p = make_problem(*desc, nullptr, k_pages, v_pages, prefix_lens, k_tree, v_tree);
    p.block_table = block_table;
    p.bt_stride = bt_stride;
    p.page_shift = page_shift_of(page_size);
    return launch_kv_commit(p, desc->dtype, accept_path, accept_len, k_pages, v_pages, new_prefix_lens, err_flag,
                            (hipStream_t)stream) == hipSuccess
               ? LS_OK
               : LS_ERR_HIP;
}

}  // extern "C"
