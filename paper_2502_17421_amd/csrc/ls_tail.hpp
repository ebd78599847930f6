// The tail of the whole path as a device function: masked tree attention of a query row merged
// with the row's cached-key partials by the aggregation rule of Section 3.3.  Used by the kernel
// that ends the two-launch call and by the last workgroup to arrive in the single-launch call.
//
// LPR lanes own one query row (head_dim / LPR consecutive elements each), so a wavefront carries
// 64 / LPR rows that run in lock step.  LPR = 16 (whole 8-, 16- or 32-byte pieces per lane, four
// rows per wavefront) costs the fewest instructions per row and is the form for calls with many
// rows; LPR = 64 spreads a row over a whole wavefront, four times as many wavefronts with a
// quarter of the serial work each, which is faster when the rows are too few to fill the chip
// and each has many split rows to add up.  When the rows of a wavefront share their tree node
// and KV head they share their visible keys, and the K/V rows they fetch are the same addresses,
// which one load instruction fetches once.  A logit is a sum over the LPR lanes (DPP additions
// inside a 16-lane row, then exchanges between rows); a row with fewer visible keys than its
// neighbours idles.
#pragma once

#include "ls_internal.hpp"

namespace ls {

template <int BYTES> struct RawVec {
    uint32_t w[(BYTES + 3) / 4];
};
template <int BYTES> __device__ __forceinline__ RawVec<BYTES> load_raw(const void *p)
{
    RawVec<BYTES> r;
    if constexpr (BYTES == 2) {
        r.w[0] = *(const uint16_t *)p;
    } else if constexpr (BYTES == 4) {
        r.w[0] = *(const uint32_t *)p;
    } else if constexpr (BYTES == 8) {
        const uint2 t = *(const uint2 *)p;
        r.w[0] = t.x;
        r.w[1] = t.y;
    } else {
        static_assert(BYTES % 16 == 0, "larger pieces are whole 16-byte units");
#pragma unroll
        for (int q = 0; q < BYTES / 16; ++q) {
            const uint4 t = ((const uint4 *)p)[q];
            r.w[4 * q + 0] = t.x;
            r.w[4 * q + 1] = t.y;
            r.w[4 * q + 2] = t.z;
            r.w[4 * q + 3] = t.w;
        }
    }
    return r;
}
template <int BYTES> __device__ __forceinline__ void store_raw(void *p, const RawVec<BYTES> &r)
{
    if constexpr (BYTES == 2) {
        *(uint16_t *)p = (uint16_t)r.w[0];
    } else if constexpr (BYTES == 4) {
        *(uint32_t *)p = r.w[0];
    } else if constexpr (BYTES == 8) {
        *(uint2 *)p = make_uint2(r.w[0], r.w[1]);
    } else {
#pragma unroll
        for (int q = 0; q < BYTES / 16; ++q)
            ((uint4 *)p)[q] = make_uint4(r.w[4 * q + 0], r.w[4 * q + 1], r.w[4 * q + 2], r.w[4 * q + 3]);
    }
}
// EPL elements of type T <-> floats
template <typename T, int EPL> struct Lanes;
template <int EPL> struct Lanes<float, EPL> {
    static constexpr int BYTES = 4 * EPL;
    static __device__ __forceinline__ void unpack(const RawVec<BYTES> &r, float *v)
    {
#pragma unroll
        for (int e = 0; e < EPL; ++e) v[e] = __uint_as_float(r.w[e]);
    }
    static __device__ __forceinline__ RawVec<BYTES> pack(const float *v)
    {
        RawVec<BYTES> r;
#pragma unroll
        for (int e = 0; e < EPL; ++e) r.w[e] = __float_as_uint(v[e]);
        return r;
    }
};
template <int EPL> struct Lanes<uint16_t, EPL> {
    static constexpr int BYTES = 2 * EPL;
    static __device__ __forceinline__ void unpack(const RawVec<BYTES> &r, float *v)
    {
        if constexpr (EPL == 1) {
            v[0] = __uint_as_float(r.w[0] << 16);
        } else {
#pragma unroll
            for (int q = 0; q < EPL / 2; ++q) {
                v[2 * q] = __uint_as_float(r.w[q] << 16);
                v[2 * q + 1] = __uint_as_float(r.w[q] & 0xffff0000u);
            }
        }
    }
    static __device__ __forceinline__ RawVec<BYTES> pack(const float *v)
    {
        RawVec<BYTES> r;
        if constexpr (EPL == 1) {
            r.w[0] = float_to_bf16(v[0]);
        } else {
#pragma unroll
            for (int q = 0; q < EPL / 2; ++q)
                r.w[q] = (uint32_t)float_to_bf16(v[2 * q]) | ((uint32_t)float_to_bf16(v[2 * q + 1]) << 16);
        }
        return r;
    }
};
template <int EPL> struct Lanes<half_t, EPL> {
    static constexpr int BYTES = 2 * EPL;
    static __device__ __forceinline__ void unpack(const RawVec<BYTES> &r, float *v)
    {
        if constexpr (EPL == 1) {
            v[0] = half_to_float((uint16_t)r.w[0]);
        } else {
#pragma unroll
            for (int q = 0; q < EPL / 2; ++q) {
                v[2 * q] = half_to_float((uint16_t)r.w[q]);
                v[2 * q + 1] = half_to_float((uint16_t)(r.w[q] >> 16));
            }
        }
    }
    static __device__ __forceinline__ RawVec<BYTES> pack(const float *v)
    {
        RawVec<BYTES> r;
        if constexpr (EPL == 1) {
            r.w[0] = float_to_half(v[0]);
        } else {
#pragma unroll
            for (int q = 0; q < EPL / 2; ++q)
                r.w[q] = (uint32_t)float_to_half(v[2 * q]) | ((uint32_t)float_to_half(v[2 * q + 1]) << 16);
        }
        return r;
    }
};

// Sum / max over the LPR (16 or 64) lanes that own a query row, the result in each of them:
// rotations by 8 and 4 inside a 16-lane DPP row, exchanges inside each group of four lanes, and
// for 64 lanes two exchanges between the DPP rows.
template <int CTRL> __device__ __forceinline__ float dpp_row(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
constexpr int kRowRor8 = 0x128, kRowRor4 = 0x124, kQuadSwap2 = 0x4e /* [2,3,0,1] */, kQuadSwap1 = 0xb1 /* [1,0,3,2] */;
template <int LPR> __device__ __forceinline__ float lanes_sum(float x)
{
    x += dpp_row<kRowRor8>(x);
    x += dpp_row<kRowRor4>(x);
    x += dpp_row<kQuadSwap2>(x);
    x += dpp_row<kQuadSwap1>(x);
    if constexpr (LPR == 64) {
        x += __shfl_xor(x, 16, kWave);
        x += __shfl_xor(x, 32, kWave);
    }
    return x;
}
template <int LPR> __device__ __forceinline__ float lanes_max(float x)
{
    x = fmaxf(x, dpp_row<kRowRor8>(x));
    x = fmaxf(x, dpp_row<kRowRor4>(x));
    x = fmaxf(x, dpp_row<kQuadSwap2>(x));
    x = fmaxf(x, dpp_row<kQuadSwap1>(x));
    if constexpr (LPR == 64) {
        x = fmaxf(x, __shfl_xor(x, 16, kWave));
        x = fmaxf(x, __shfl_xor(x, 32, kWave));
    }
    return x;
}

// One step of a wavefront: the 64 / LPR query rows (b, h, i) its lanes hold (identical within the
// LPR lanes of a row; !live: the lanes repeat a valid row and store nothing).  All 64 lanes must
// be active.  mask: the tree-mask rows of the lane's sequence (any address space); nullptr, in
// every lane, for no tree part.
template <typename T, typename PT, int D, int LPR, int CH>
__device__ __forceinline__ void tail_rows(const Problem &p, const uint64_t *mask, const Partials &parts,
                                          int32_t n_cache, T *__restrict__ out, int64_t os0, int64_t os1, int64_t os2,
                                          float *__restrict__ lse, int b, int h, int i, bool live, int lane)
{
    constexpr int EPL = D / LPR;
    typedef Lanes<T, EPL> LT;
    typedef Lanes<PT, EPL> LP;
    constexpr int QB = LT::BYTES, PB = LP::BYTES;
    // Tree keys per request (K and V rows); two requests are in flight.  With 16 lanes per row a
    // key costs eight registers, and two keys per request keep the wavefront small enough for
    // three or four of them per SIMD, which hides more latency than longer requests do.
    constexpr int KB = LPR == 16 || QB > 16 ? 2 : 4;
    // CH: split rows requested together, at most LPR (their weights come from the lanes of the
    // row).  LPR = 16, CH = 16 keeps two such requests in flight (32 split rows); CH = 4 serves
    // rows of at most 8 parts (one or two requests, one after the other); LPR = 64 has CH = 32.
    static_assert(CH <= LPR && (LPR == 16 || LPR == 64), "");
    constexpr bool TWO_SETS = LPR == 16 && CH == 16 && 2 * CH * PB <= 512;
    const int sl = lane & (LPR - 1);
    const int slot0 = lane & ~(LPR - 1);  // first lane of this row
    const int g = h / p.group;
    const int row = (b * p.n_q_heads + h) * p.n_tree + i;  // index of the row in lse
    const int words = (p.n_tree + 63) >> 6;

    const size_t prow0 = parts.row((size_t)b * p.n_q_heads + h, 0, p.n_tree, i);
    const float *lp = parts.lse + prow0;
    const PT *op = (const PT *)parts.o + prow0 * D + sl * EPL;
    const size_t lse_step = parts.row_major ? 1 : (size_t)p.n_tree;  // between consecutive parts of one row
    const size_t part_step = lse_step * D;

    // Order of requests (loads return in the order they were issued): the query row and the
    // mask word first, a short round trip; then the row's first visible tree keys; then the
    // cached-key partials, by far the most bytes.  The partials are merged among themselves as
    // they arrive, then the tree keys (long there by then) are worked through, further ones being
    // requested a batch ahead, and a two-term merge of the two results ends the row.
    const T *qrow = (const T *)p.q + b * p.q_stride[0] + h * p.q_stride[1] + i * p.q_stride[2] + sl * EPL;
    const T *kbase = (const T *)p.k_tree + b * p.kt_stride[0] + g * p.kt_stride[1] + sl * EPL;
    const T *vbase = (const T *)p.v_tree + b * p.vt_stride[0] + g * p.vt_stride[1] + sl * EPL;
    const uint64_t *mrow = mask + (size_t)i * words;
    float qv[EPL], acc[EPL];
    LT::unpack(load_raw<QB>(qrow), qv);
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        qv[e] *= p.scale_log2;
        acc[e] = 0.f;
    }
    // The visible keys of the row are the set bits of its mask words, taken 128 tree nodes (two
    // words) at a time: lo / hi is what is left of the current pair.
    auto mask_word = [&](int w) -> uint64_t {
        if (mask == nullptr || w >= words) return 0;  // wave-uniform; no mask: no tree part
        uint64_t m = mrow[w];
        if (w == words - 1 && (p.n_tree & 63)) m &= ((uint64_t)1 << (p.n_tree & 63)) - 1;
        return m;
    };
    const int n_pairs = mask == nullptr ? 0 : (words + 1) >> 1;
    int pair = 0;
    uint64_t lo = mask_word(0), hi = mask_word(1);
    // KB visible keys of each row per request, all their K/V rows requested before the first is
    // used; two requests are in flight.
    struct KeyBatch {
        int idx[KB];
        bool any_row[KB];  // wave-uniform: some row of the wavefront has a u-th key in this batch
        RawVec<QB> k[KB], v[KB];
    };
    auto request_keys = [&](KeyBatch &kb) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < KB; ++u) {
            // the lowest set bit of lo, else of hi (selects on values: no branch, nothing addressed)
            const bool in_lo = lo != 0;
            const uint64_t cur = in_lo ? lo : hi;
            const int j_next = cur ? (pair << 7) + (in_lo ? 0 : 64) + __builtin_ctzll(cur) : -1;
            const uint64_t rest = cur & (cur - 1);  // 0 stays 0
            lo = in_lo ? rest : lo;
            hi = in_lo ? hi : rest;
            kb.idx[u] = j_next;
            kb.any_row[u] = __any(kb.idx[u] >= 0);
            if (kb.any_row[u]) {
                const int j = kb.idx[u] < 0 ? 0 : kb.idx[u];
                kb.k[u] = load_raw<QB>(kbase + j * p.kt_stride[2]);
                kb.v[u] = load_raw<QB>(vbase + j * p.vt_stride[2]);
            }
        }
    };
    float m_run = -INFINITY, l_run = 0.f;  // base-2 logits; identical in the lanes of a row
    auto use_keys = [&](const KeyBatch &kb) __attribute__((always_inline)) {
        float z[KB];
        float mx = -INFINITY;
#pragma unroll
        for (int u = 0; u < KB; ++u) {
            z[u] = -INFINITY;
            if (!kb.any_row[u]) continue;
            float kv[EPL];
            LT::unpack(kb.k[u], kv);
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) part += qv[e] * kv[e];
            const float s = lanes_sum<LPR>(part);
            z[u] = kb.idx[u] < 0 ? -INFINITY : s;
            mx = fmaxf(mx, z[u]);
        }
        const float m_new = fmaxf(m_run, mx);
        const float m_ref = m_new == -INFINITY ? 0.f : m_new;  // a row with no key yet keeps zeros
        const float alpha = exp2f(m_run - m_ref);
        l_run *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < KB; ++u) {
            if (!kb.any_row[u]) continue;
            const float pj = exp2f(z[u] - m_ref);  // 0 for a key this row does not see
            float vv[EPL];
            LT::unpack(kb.v[u], vv);
            l_run += pj;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += pj * vv[e];
        }
        m_run = m_new;
    };
    KeyBatch keys_a, keys_b;
    request_keys(keys_a);
    request_keys(keys_b);
    // the LSEs of parts 0 .. 2 LPR - 1 (two per lane of the row) and the first split rows
    const float l_first = sl < n_cache ? lp[(size_t)sl * lse_step] : -INFINITY;
    const float l_second = LPR + sl < n_cache ? lp[(size_t)(LPR + sl) * lse_step] : -INFINITY;
    const int n_batches = (n_cache + CH - 1) / CH;
    RawVec<PB> raw_a[CH];
    auto request_parts = [&](RawVec<PB> (&raw)[CH], int batch) {
#pragma unroll
        for (int k = 0; k < CH; ++k) {
            const int part = batch * CH + k < n_cache ? batch * CH + k : n_cache - 1;  // clamped: always a valid row
            raw[k] = load_raw<PB>(op + (size_t)part * part_step);
        }
    };
    if (n_batches > 0) request_parts(raw_a, 0);

    // ---- merge of the cached-key partials among themselves -----------------------------------
    float o[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = 0.f;
    float w_lane = 0.f;  // this lane's part weights
    float top_c = -INFINITY;
    auto merge_parts = [&](const RawVec<PB> (&raw)[CH], int batch) {
        // lane sl < CH holds the weight of part batch * CH + sl
        const int s = batch * CH + sl;
        float l = -INFINITY;
        if (sl < CH && s < n_cache)
            l = batch == 0 ? l_first : (CH == LPR && batch == 1 ? l_second : lp[(size_t)s * lse_step]);
        const float w = l == -INFINITY ? 0.f : exp2f((l - top_c) * kLog2e);
        w_lane += w;
#pragma unroll
        for (int k = 0; k < CH; ++k) {
            // past the last part the weight is 0 (the clamped row was still a valid read); empty
            // parts may hold anything, so they are selected out rather than multiplied
            const float wk = __shfl(w, slot0 + k, kWave);
            float v[EPL];
            LP::unpack(raw[k], v);
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[e] += wk > 0.f ? wk * v[e] : 0.f;
        }
    };
    auto top_of_all_parts = [&]() {
        float top = fmaxf(l_first, l_second);
        for (int s0 = 2 * LPR; s0 < n_cache; s0 += LPR) {
            const int s = s0 + sl;
            top = fmaxf(top, s < n_cache ? lp[(size_t)s * lse_step] : -INFINITY);
        }
        return lanes_max<LPR>(top);
    };
    if constexpr (TWO_SETS) {
        // two register sets, both requested before the first is used
        RawVec<PB> raw_b[CH];
        if (n_batches > 1) request_parts(raw_b, 1);
        top_c = top_of_all_parts();
        for (int bt = 0; bt < n_batches; bt += 2) {
            merge_parts(raw_a, bt);
            if (bt + 2 < n_batches) request_parts(raw_a, bt + 2);
            if (bt + 1 < n_batches) {
                merge_parts(raw_b, bt + 1);
                if (bt + 3 < n_batches) request_parts(raw_b, bt + 3);
            }
        }
    } else {
        top_c = top_of_all_parts();
        for (int bt = 0; bt < n_batches; ++bt) {
            merge_parts(raw_a, bt);
            if (bt + 1 < n_batches) request_parts(raw_a, bt + 1);
        }
    }
    const float wsum_c = lanes_sum<LPR>(w_lane);  // 0 if no cached key is visible

    // ---- masked attention over the tree keys (unnormalised, base-2 logits) ----------------
    // Keys are handed out in order, so a request whose first slot is empty for every row of the
    // wavefront ends the pair of mask words: whatever was requested after it is empty too.
    while (true) {
        const uint64_t lo_next = mask_word(2 * pair + 2), hi_next = mask_word(2 * pair + 3);  // fetched ahead
        while (true) {
            if (!keys_a.any_row[0]) break;
            use_keys(keys_a);
            request_keys(keys_a);
            if (!keys_b.any_row[0]) break;
            use_keys(keys_b);
            request_keys(keys_b);
        }
        if (++pair >= n_pairs) break;
        lo = lo_next;
        hi = hi_next;
        request_keys(keys_a);
        request_keys(keys_b);
    }

    // ---- the two results, merged by the aggregation rule ----------------------------------------
    T *orow = out + b * os0 + h * os1 + i * os2 + sl * EPL;
    const float lse_c = wsum_c > 0.f ? top_c + log2f(wsum_c) * kLn2 : -INFINITY;
    const float lse_t = l_run > 0.f ? (m_run + log2f(l_run)) * kLn2 : -INFINITY;
    const float top = fmaxf(lse_c, lse_t);
    float lse_row = -INFINITY;
    if (top == -INFINITY) {  // no visible key at all
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] = 0.f;
    } else {
        const float wa = wsum_c > 0.f ? exp2f((lse_c - top) * kLog2e) : 0.f;
        const float wb = l_run > 0.f ? exp2f((lse_t - top) * kLog2e) : 0.f;
        const float inv = 1.f / (wa + wb);
        const float sa = wsum_c > 0.f ? wa * inv / wsum_c : 0.f;
        const float sb = l_run > 0.f ? wb * inv / l_run : 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] = o[e] * sa + acc[e] * sb;
        lse_row = top + log2f(wa + wb) * kLn2;
    }
    if (live) {
        store_raw<QB>(orow, LT::pack(o));
        if (sl == 0) lse[row] = lse_row;
    }
}

}  // namespace ls
