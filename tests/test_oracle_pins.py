"""Pins for the CPU oracle: things fixed by the paper's definition and by mathematics,
none of which come from the oracle itself or from the GPU path.

The paper prints no numeric worked example of attention, so the pins are: a case worked
out by hand from the definition (tests/golden/hand_case.json), brute force by an
independently structured dense-mask implementation, closed forms, the split + LSE-merge
proposition of the appendix, invariances, and special cases that reduce to torch's CPU
scaled_dot_product_attention (chain tree == causal attention, boolean-mask attention,
single-token decode).
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2502_17421_amd import synth


# ------------------------------------------------------------------ helpers ----

def dense_mask_by_closure(parents):
    """Ancestor-or-self relation as a dense boolean matrix, built differently from the
    oracle (boolean matrix closure instead of a parent walk)."""
    t = len(parents)
    adj = np.eye(t, dtype=bool)
    for i, p in enumerate(parents):
        if p >= 0:
            adj[i, p] = True
    reach = adj.copy()
    for _ in range(t):
        nxt = (reach.astype(np.int64) @ adj.astype(np.int64)) > 0
        if np.array_equal(nxt, reach):
            break
        reach = nxt
    return reach


def brute_force(q, kc, vc, kt, vt, parents, scale):
    """Dense masked softmax over the concatenation [cache || tree], python loops, fp64."""
    hq, t, d = q.shape
    hkv, p, _ = kc.shape
    g = hq // hkv
    vis_tree = dense_mask_by_closure(parents)
    out = np.zeros((hq, t, d))
    lse = np.zeros((hq, t))
    for h in range(hq):
        kk = np.concatenate([kc[h // g], kt[h // g]], axis=0).astype(np.float64)
        vv = np.concatenate([vc[h // g], vt[h // g]], axis=0).astype(np.float64)
        for i in range(t):
            allowed = np.concatenate([np.ones(p, dtype=bool), vis_tree[i]])
            num = np.zeros(d)
            den = 0.0
            for j in range(p + t):
                if not allowed[j]:
                    continue
                zj = 0.0
                for c in range(d):
                    zj += float(q[h, i, c]) * kk[j, c]
                e = math.exp(scale * zj)
                den += e
                num += e * vv[j]
            out[h, i] = num / den
            lse[h, i] = math.log(den)
    return out, lse


def small_problem(seed, hq=4, hkv=2, d=3, p=5, t=6, parents=None):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((hq, t, d)).astype(np.float32)
    kc = rng.standard_normal((hkv, p, d)).astype(np.float32)
    vc = rng.standard_normal((hkv, p, d)).astype(np.float32)
    kt = rng.standard_normal((hkv, t, d)).astype(np.float32)
    vt = rng.standard_normal((hkv, t, d)).astype(np.float32)
    if parents is None:
        parents = synth.tree_uniform(rng, t)
    return q, kc, vc, kt, vt, np.asarray(parents, dtype=np.int32)


# ---------------------------------------------------------------- hand case ----

def test_hand_computed_case(golden_dir):
    with open(os.path.join(golden_dir, "hand_case.json")) as f:
        g = json.load(f)
    q = np.asarray(g["q"], dtype=np.float32)
    kc = np.log(np.asarray(g["k_cache_exp"], dtype=np.float64)).astype(np.float32)
    kt = np.log(np.asarray(g["k_tree_exp"], dtype=np.float64)).astype(np.float32)
    vc = np.asarray(g["v_cache"], dtype=np.float32)
    vt = np.asarray(g["v_tree"], dtype=np.float32)
    out, lse = oracle.attn_all(q, kc, vc, kt, vt, g["parents"], scale=g["scale"])
    # float32 storage of ln(n) perturbs each exp-logit by < 1e-7 relative
    np.testing.assert_allclose(out[0, :, 0], g["expect_out"], rtol=0, atol=2e-6)
    np.testing.assert_allclose(np.exp(lse[0]), g["expect_lse_exp"], rtol=1e-6)


# -------------------------------------------------------------- brute force ----

@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_brute_force_tiny(seed):
    q, kc, vc, kt, vt, parents = small_problem(seed)
    scale = 0.7
    out, lse = oracle.attn_all(q, kc, vc, kt, vt, parents, scale=scale)
    bo, bl = brute_force(q, kc, vc, kt, vt, parents, scale)
    np.testing.assert_allclose(out, bo, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, bl, rtol=0, atol=1e-13)


def test_brute_force_forest_and_wide_group():
    # two roots (a forest), one KV head shared by 3 query heads, default scale 1/sqrt(D)
    parents = np.asarray([-1, 0, -1, 2, 1, 2, 3], dtype=np.int32)
    q, kc, vc, kt, vt, _ = small_problem(11, hq=3, hkv=1, d=4, p=3, t=7, parents=parents)
    out, lse = oracle.attn_all(q, kc, vc, kt, vt, parents)
    bo, bl = brute_force(q, kc, vc, kt, vt, parents, 1.0 / math.sqrt(4))
    np.testing.assert_allclose(out, bo, atol=1e-13)
    np.testing.assert_allclose(lse, bl, atol=1e-13)


def test_selected_rows_match_full():
    q, kc, vc, kt, vt, parents = small_problem(5, t=9)
    out, lse = oracle.attn_all(q, kc, vc, kt, vt, parents)
    rows = np.asarray([[3, 8], [0, 0], [2, 5]], dtype=np.int32)
    o2, l2 = oracle.attn_rows(q, kc, vc, kt, vt, parents, rows=rows)
    for n, (h, i) in enumerate(rows):
        np.testing.assert_array_equal(o2[n], out[h, i])
        assert l2[n] == lse[h, i]


# ------------------------------------------------------------- closed forms ----

def test_zero_query_gives_mean_of_visible_values():
    """q = 0: uniform weights, so lse = ln |visible set| = ln(P + depth + 1) and the output
    is the mean of the visible value rows.  Checks the size of the visible set exactly."""
    rng = np.random.default_rng(21)
    t, p, d = 12, 7, 5
    parents = synth.tree_constrained(rng, t, 4, 3)
    depth = synth.tree_depths(parents)
    q, kc, vc, kt, vt, _ = small_problem(22, hq=2, hkv=1, d=d, p=p, t=t, parents=parents)
    q[:] = 0
    out, lse = oracle.attn_all(q, kc, vc, kt, vt, parents)
    for i in range(t):
        path = []
        j = i
        while j >= 0:
            path.append(j)
            j = parents[j]
        assert len(path) == depth[i] + 1
        mean = (vc[0].astype(np.float64).sum(0) + vt[0, path].astype(np.float64).sum(0)) / (p + len(path))
        for h in range(2):
            assert abs(lse[h, i] - math.log(p + depth[i] + 1)) < 1e-14
            np.testing.assert_allclose(out[h, i], mean, atol=1e-14)


def test_equal_keys_also_uniform():
    q, kc, vc, kt, vt, parents = small_problem(31, hq=2, hkv=2, d=4, p=6, t=5)
    kc[:] = kc[:, :1]
    kt[:] = kc[:, :1]
    out, lse = oracle.attn_all(q, kc, vc, kt, vt, parents)
    depth = synth.tree_depths(parents)
    z = 0.5 * np.einsum("htd,hd->ht", q.astype(np.float64), kc[:, 0].astype(np.float64))
    np.testing.assert_allclose(lse, z + np.log(6 + depth + 1)[None, :], atol=1e-13)


def test_constant_values_pass_through_and_weights_sum_to_one():
    q, kc, vc, kt, vt, parents = small_problem(41, p=9, t=8)
    c = np.asarray([1.0, -2.5, 0.125], dtype=np.float32)
    vc[:] = c
    vt[:] = c
    out, _ = oracle.attn_all(q, kc, vc, kt, vt, parents)
    np.testing.assert_allclose(out, np.broadcast_to(c, out.shape), atol=1e-14)


def test_dominant_key_selects_its_value_row():
    q, kc, vc, kt, vt, parents = small_problem(51, hq=1, hkv=1, d=4, p=8, t=3,
                                               parents=[-1, 0, 1])
    lam = 200.0
    kc[0, 5] = lam * q[0, 2]            # cached row 5 dominates for query row 2
    out, lse = oracle.attn_all(q, kc, vc, kt, vt, parents)
    zmax = 0.5 * lam * float(np.dot(q[0, 2].astype(np.float64), q[0, 2].astype(np.float64)))
    np.testing.assert_allclose(out[0, 2], vc[0, 5], atol=1e-12)
    assert abs(lse[0, 2] - zmax) < 1e-6 * zmax


def test_far_away_key_changes_nothing():
    q, kc, vc, kt, vt, parents = small_problem(61, hq=1, hkv=1, d=2, p=4, t=3)
    q[:] = np.abs(q) + 0.5
    base_o, base_l = oracle.attn_all(q, kc, vc, kt, vt, parents)
    kc2 = np.concatenate([kc, np.full((1, 1, 2), -1e4, dtype=np.float32)], axis=1)
    vc2 = np.concatenate([vc, np.full((1, 1, 2), 777.0, dtype=np.float32)], axis=1)
    o2, l2 = oracle.attn_all(q, kc2, vc2, kt, vt, parents)
    np.testing.assert_allclose(o2, base_o, atol=1e-14)
    np.testing.assert_allclose(l2, base_l, atol=1e-14)


# ------------------------------------------- split + merge (the proposition) ----

def np_merge(o_parts, lse_parts):
    """Many-term form of the aggregation formulas, written directly with numpy."""
    lse = np.logaddexp.reduce(lse_parts, axis=1)
    w = np.exp(lse_parts - lse[:, None])
    return np.einsum("np,npd->nd", w, o_parts), lse


@pytest.mark.parametrize("cuts", [[0, 4, 11], [0, 1, 2, 11], [0, 11], [0, 0, 7, 11]])
def test_split_then_merge_equals_monolithic(cuts):
    q, kc, vc, kt, vt, parents = small_problem(71, hq=4, hkv=2, d=6, p=11, t=7)
    full_o, full_l = oracle.attn_rows(q, kc, vc, kt, vt, parents)
    po, pl = [], []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        o, l = oracle.attn_rows(q, kc, vc, kt, vt, parents, prefix_lo=lo, prefix_hi=hi, use_tree=False)
        po.append(o)
        pl.append(l)
    o, l = oracle.attn_rows(q, kc, vc, kt, vt, parents, prefix_lo=0, prefix_hi=0, use_tree=True)
    po.append(o)
    pl.append(l)
    po = np.stack(po, axis=1)
    pl = np.stack(pl, axis=1)
    # an empty range has lse = -inf and zero output
    for k, (lo, hi) in enumerate(zip(cuts[:-1], cuts[1:])):
        if lo == hi:
            assert np.all(np.isneginf(pl[:, k])) and np.all(po[:, k] == 0)
    mo, ml = np_merge(po, pl)
    np.testing.assert_allclose(mo, full_o, atol=1e-13)
    np.testing.assert_allclose(ml, full_l, atol=1e-13)
    # and the oracle's own sequential two-term merge says the same
    oo, ol = oracle.lse_merge(po, pl)
    np.testing.assert_allclose(oo, full_o, atol=1e-13)
    np.testing.assert_allclose(ol, full_l, atol=1e-13)


def test_merge_two_terms_literal_formula():
    """Section 3.3's formulas typed out with raw exp/log on moderate values."""
    rng = np.random.default_rng(81)
    oa, ob = rng.standard_normal((5, 3)), rng.standard_normal((5, 3))
    la, lb = rng.standard_normal(5) * 3, rng.standard_normal(5) * 3
    lm = np.log(np.exp(la) + np.exp(lb))
    om = oa * np.exp(la - lm)[:, None] + ob * np.exp(lb - lm)[:, None]
    o, l = oracle.lse_merge(np.stack([oa, ob], axis=1), np.stack([la, lb], axis=1))
    np.testing.assert_allclose(l, lm, atol=1e-14)
    np.testing.assert_allclose(o, om, atol=1e-14)


def test_merge_large_lse_and_empty_parts():
    o = np.asarray([[[1.0, 2.0], [np.nan, np.nan], [3.0, 6.0]]])
    l = np.asarray([[1000.0, -np.inf, 1000.0 + math.log(3.0)]])
    out, lse = oracle.lse_merge(o, l)
    np.testing.assert_allclose(out[0], [0.25 * 1 + 0.75 * 3, 0.25 * 2 + 0.75 * 6], atol=1e-13)
    assert abs(lse[0] - (1000.0 + math.log(4.0))) < 1e-12
    out, lse = oracle.lse_merge(np.zeros((1, 2, 2)), np.full((1, 2), -np.inf))
    assert np.isneginf(lse[0]) and np.all(out == 0)


# -------------------------------------------------------------- invariances ----

def test_permuting_cached_rows_changes_nothing():
    q, kc, vc, kt, vt, parents = small_problem(91, p=13, t=6)
    o1, l1 = oracle.attn_all(q, kc, vc, kt, vt, parents)
    perm = np.random.default_rng(92).permutation(13)
    o2, l2 = oracle.attn_all(q, kc[:, perm], vc[:, perm], kt, vt, parents)
    np.testing.assert_allclose(o2, o1, atol=1e-13)
    np.testing.assert_allclose(l2, l1, atol=1e-13)


def test_relabelling_tree_nodes_consistently():
    # swap the labels of nodes 2 and 3 (both children of 0, so the order stays topological)
    parents = np.asarray([-1, 0, 0, 0, 2, 3, 4], dtype=np.int32)
    q, kc, vc, kt, vt, _ = small_problem(93, hq=2, hkv=1, d=4, p=4, t=7, parents=parents)
    perm = np.asarray([0, 1, 3, 2, 4, 5, 6])          # new label -> old label
    inv = np.argsort(perm)
    parents2 = np.asarray([-1 if parents[perm[i]] < 0 else inv[parents[perm[i]]] for i in range(7)],
                          dtype=np.int32)
    o1, l1 = oracle.attn_all(q, kc, vc, kt, vt, parents)
    o2, l2 = oracle.attn_all(q[:, perm], kc, vc, kt[:, perm], vt[:, perm], parents2)
    np.testing.assert_allclose(o2, o1[:, perm], atol=1e-13)
    np.testing.assert_allclose(l2, l1[:, perm], atol=1e-13)


# ------------------------------------- special cases vs torch's CPU attention ----

def torch_sdpa(q, k, v, mask=None, causal=False, scale=None):
    tq = torch.from_numpy(np.asarray(q, dtype=np.float64))[None]
    tk = torch.from_numpy(np.asarray(k, dtype=np.float64))[None]
    tv = torch.from_numpy(np.asarray(v, dtype=np.float64))[None]
    tm = None if mask is None else torch.from_numpy(mask)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=tm, is_causal=causal,
                                                         scale=scale)
    return o[0].numpy()


def test_chain_tree_is_causal_attention():
    """A chain-shaped tree makes [cache || tree] an ordinary causal sequence: the tree rows
    are its last T positions."""
    hq, hkv, d, p, t = 4, 2, 8, 10, 6
    q, kc, vc, kt, vt, _ = small_problem(101, hq=hq, hkv=hkv, d=d, p=p, t=t, parents=synth.tree_chain(t))
    out, _ = oracle.attn_all(q, kc, vc, kt, vt, synth.tree_chain(t))
    g = hq // hkv
    k_full = np.repeat(np.concatenate([kc, kt], axis=1), g, axis=0)      # [Hq, P+T, D]
    v_full = np.repeat(np.concatenate([vc, vt], axis=1), g, axis=0)
    q_full = np.concatenate([np.zeros((hq, p, d), dtype=np.float32), q], axis=1)
    ref = torch_sdpa(q_full, k_full, v_full, causal=True)[:, p:]
    np.testing.assert_allclose(out, ref, atol=1e-12)


@pytest.mark.parametrize("kind", ["random", "star", "forest"])
def test_boolean_mask_attention(kind):
    hq, hkv, d, p, t = 6, 2, 16, 33, 20
    rng = np.random.default_rng(111)
    if kind == "random":
        parents = synth.tree_constrained(rng, t, 5, 3)
    elif kind == "star":
        parents = synth.tree_star(t)
    else:
        parents = synth.tree_uniform(rng, t)
        parents[[4, 9]] = -1
    q, kc, vc, kt, vt, _ = small_problem(112, hq=hq, hkv=hkv, d=d, p=p, t=t, parents=parents)
    out, lse = oracle.attn_all(q, kc, vc, kt, vt, parents, scale=0.3)
    g = hq // hkv
    k_full = np.repeat(np.concatenate([kc, kt], axis=1), g, axis=0)
    v_full = np.repeat(np.concatenate([vc, vt], axis=1), g, axis=0)
    mask = np.concatenate([np.ones((t, p), dtype=bool), dense_mask_by_closure(parents)], axis=1)
    ref = torch_sdpa(q, k_full, v_full, mask=mask, scale=0.3)
    np.testing.assert_allclose(out, ref, atol=1e-12)
    # lse against torch.logsumexp of the masked, scaled logits
    logits = 0.3 * torch.einsum("htd,hjd->htj", torch.from_numpy(q.astype(np.float64)),
                                torch.from_numpy(k_full.astype(np.float64)))
    logits = logits.masked_fill(~torch.from_numpy(mask)[None], float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(logits, dim=-1).numpy(), atol=1e-12)


def test_single_token_is_plain_decode_attention():
    q, kc, vc, kt, vt, parents = small_problem(121, hq=2, hkv=2, d=8, p=17, t=1, parents=[-1])
    out, _ = oracle.attn_all(q, kc, vc, kt, vt, parents)
    ref = torch_sdpa(q, np.concatenate([kc, kt], axis=1), np.concatenate([vc, vt], axis=1))
    np.testing.assert_allclose(out, ref, atol=1e-12)


def test_partial_views_vs_torch():
    """Cache-only over a sub-range and tree-only partials are plain / masked attention too."""
    hq, hkv, d, p, t = 2, 1, 8, 12, 5
    q, kc, vc, kt, vt, parents = small_problem(131, hq=hq, hkv=hkv, d=d, p=p, t=t)
    o, _ = oracle.attn_all(q, kc, vc, kt, vt, parents, prefix_lo=3, prefix_hi=10, use_tree=False)
    ref = torch_sdpa(q, np.repeat(kc[:, 3:10], 2, 0), np.repeat(vc[:, 3:10], 2, 0))
    np.testing.assert_allclose(o, ref, atol=1e-12)
    o, _ = oracle.attn_all(q, kc, vc, kt, vt, parents, prefix_lo=0, prefix_hi=0, use_tree=True)
    ref = torch_sdpa(q, np.repeat(kt, 2, 0), np.repeat(vt, 2, 0), mask=dense_mask_by_closure(parents))
    np.testing.assert_allclose(o, ref, atol=1e-12)


# --------------------------------------------------------------------- mask ----

def bits_of(row):
    return [j for w, word in enumerate(row) for j in range(64 * w, 64 * w + 64) if (int(word) >> (j % 64)) & 1]


@pytest.mark.parametrize("t", [1, 5, 64, 65, 100, 128, 129, 300, 512])
def test_mask_properties(t):
    rng = np.random.default_rng(200 + t)
    parents = synth.tree_uniform(rng, t)
    m = oracle.tree_mask(parents)
    assert m.shape == (t, (t + 63) // 64) and m.dtype == np.uint64
    depth = synth.tree_depths(parents)
    closure = dense_mask_by_closure(parents)
    for i in range(t):
        bits = bits_of(m[i])
        assert len(bits) == depth[i] + 1
        assert i in bits and max(bits) == i
        assert bits == list(np.nonzero(closure[i])[0])
        if parents[i] >= 0:
            assert set(bits_of(m[parents[i]])) | {i} == set(bits)


def test_mask_chain_star_forest():
    m = oracle.tree_mask(synth.tree_chain(64))
    assert [int(x) for x in m[:, 0]] == [(1 << (i + 1)) - 1 for i in range(64)]
    m = oracle.tree_mask(synth.tree_star(70))
    assert int(m[0, 0]) == 1 and int(m[69, 0]) == 1 and int(m[69, 1]) == 1 << 5
    assert int(m[3, 0]) == 0b1001
    m = oracle.tree_mask([-1, -1, 1])
    assert [int(x) for x in m[:, 0]] == [1, 2, 6]


@pytest.mark.parametrize("bad", [[0], [-1, 1], [-1, 2, 0], [-1, -2], [-1, 0, 5]])
def test_bad_parents_rejected(bad):
    with pytest.raises(ValueError):
        oracle.tree_mask(bad)
    t = len(bad)
    x = np.zeros((1, t, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.attn_all(x, np.zeros((1, 1, 2), np.float32), np.zeros((1, 1, 2), np.float32), x, x, bad)


# ---------------------------------------------------------- input generator ----

def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(301).standard_normal(20000).astype(np.float32) * 37.0
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-40]   # ties and a denormal
    r = synth.round_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, ref)
    bits = synth.bf16_bits(r)
    back = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(back, r)


def test_workload_trees_respect_limits():
    for name in ("C2", "C4", "C5"):
        w = synth.WORKLOADS[name]
        rng = np.random.default_rng(w.seed)
        parents = synth.tree_constrained(rng, w.n_tree, w.max_depth, w.max_children)
        assert parents[0] == -1 and all(0 <= parents[i] < i for i in range(1, w.n_tree))
        assert synth.tree_depths(parents).max() <= w.max_depth
        if w.max_children is not None:
            assert np.bincount(parents[1:], minlength=w.n_tree).max() <= w.max_children
    assert len(synth.tree_beam(np.random.default_rng(0))) == 69
