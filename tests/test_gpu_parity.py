"""Parity of the HIP path against the CPU oracle, through the C ABI, on a real MI355X.

Small cases are compared element by element (sizes the oracle finishes in seconds that still
span several key tiles, several splits and ragged tails).  The five benchmark shapes are
run at full size in the configuration the benchmark times (library-chosen splits) and
compared on sampled query rows, which the oracle computes one by one.
"""
import dataclasses
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2502_17421_amd import binding as ls
from paper_2502_17421_amd import synth
from util import DeviceBatch, gates, oracle_full, to_dev, torch_dtype

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def device():
    assert torch.cuda.is_available(), "these tests need a GPU"
    ls.lib()
    return torch.device("cuda")


def small(name, prefix, variant="iid", **over):
    w = dataclasses.replace(synth.WORKLOADS[name], **over) if over else synth.WORKLOADS[name]
    return synth.make_batch(w, variant, prefix_override=prefix)


# ------------------------------------------------------------------------- (a) mask ----

@pytest.mark.parametrize("n_tree", [1, 2, 5, 63, 64, 65, 100, 128, 129, 192, 256, 257, 300, 511, 512])
def test_mask_bit_exact(n_tree):
    rng = np.random.default_rng(500 + n_tree)
    trees = [synth.tree_uniform(rng, n_tree), synth.tree_chain(n_tree), synth.tree_star(n_tree),
             synth.tree_constrained(rng, n_tree, 10, 4)]
    forest = synth.tree_uniform(rng, n_tree)
    forest[rng.integers(0, n_tree, size=3)] = -1
    trees.append(forest)
    parents = torch.from_numpy(np.stack(trees)).cuda()
    words = (n_tree + 63) // 64
    mask = torch.full((len(trees), n_tree, words), -1, dtype=torch.int64, device="cuda")
    err = torch.full((len(trees),), 7, dtype=torch.int32, device="cuda")
    ls.ls_build_tree_mask(parents, mask, err)
    torch.cuda.synchronize()
    got = mask.cpu().numpy().view(np.uint64)
    for b, tr in enumerate(trees):
        np.testing.assert_array_equal(got[b], oracle.tree_mask(tr))
    assert err.cpu().tolist() == [0] * len(trees)


def test_mask_invalid_entries_are_flagged_and_cut():
    good = np.asarray([-1, 0, 1, 1, 3, 4], dtype=np.int32)
    bad1 = np.asarray([-1, 0, 5, 1, 3, 2], dtype=np.int32)   # entry 2 points forward
    bad2 = np.asarray([-1, 0, 1, -9, 3, 4], dtype=np.int32)  # entry 3 below -1
    parents = torch.from_numpy(np.stack([good, bad1, bad2])).cuda()
    mask = torch.zeros((3, 6, 1), dtype=torch.int64, device="cuda")
    err = torch.zeros((3,), dtype=torch.int32, device="cuda")
    ls.ls_build_tree_mask(parents, mask, err)
    torch.cuda.synchronize()
    assert err.cpu().tolist() == [0, 1, 1]
    got = mask.cpu().numpy().view(np.uint64)
    cut1, cut2 = bad1.copy(), bad2.copy()
    cut1[2] = -1
    cut2[3] = -1
    np.testing.assert_array_equal(got[0], oracle.tree_mask(good))
    np.testing.assert_array_equal(got[1], oracle.tree_mask(cut1))
    np.testing.assert_array_equal(got[2], oracle.tree_mask(cut2))


# ------------------------------------------------------------------ (c) tree attention ----

@pytest.mark.parametrize("dtype,d,t,hq,hkv", [("f32", 64, 16, 4, 1), ("f32", 128, 37, 6, 2),
                                              ("bf16", 128, 64, 32, 8), ("bf16", 64, 128, 10, 2),
                                              ("bf16", 128, 1, 4, 4)])
def test_tree_attention_alone(dtype, d, t, hq, hkv):
    rng = np.random.default_rng(600 + t)
    seqs = []
    for b in range(2):
        parents = synth.tree_constrained(rng, t, 10, 4) if b == 0 else synth.tree_uniform(rng, t)
        seqs.append(synth.make_sequence(rng, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_tree=t,
                                        prefix_len=1, parents=parents, variant="peaked"))
    dt = torch_dtype(dtype)
    q = torch.stack([to_dev(s.q, dt) for s in seqs])
    kt = torch.stack([to_dev(s.k_tree, dt) for s in seqs])
    vt = torch.stack([to_dev(s.v_tree, dt) for s in seqs])
    mask = torch.from_numpy(np.stack([oracle.tree_mask(s.parents) for s in seqs]).view(np.int64)).cuda()
    o = torch.full((2, hq, t, d), float("nan"), dtype=torch.float32, device="cuda")
    l = torch.full((2, hq, t), float("nan"), dtype=torch.float32, device="cuda")
    desc = ls.make_desc(q, None, None, kt, vt, None, 0)
    ls.ls_tree_attn_masked(desc, q, kt, vt, mask, o, l)
    torch.cuda.synchronize()
    for b, s in enumerate(seqs):
        ro, rl = oracle.attn_all(s.q, s.k_cache, s.v_cache, s.k_tree, s.v_tree, s.parents,
                                 prefix_lo=0, prefix_hi=0, use_tree=True)
        # partial results are float on both dtypes: only the inputs are rounded
        say(gates(o[b].cpu().numpy(), l[b].cpu().numpy(), ro, rl, "f32" if dtype == "f32" else "bf16",
                  f"tree-only {dtype} b={b}", stress=True))
        assert np.abs(o[b].cpu().numpy() - ro).max() < 2e-5


# --------------------------------------------------------------------------- (d) merge ----

@pytest.mark.parametrize("dtype,d,parts_bf16", [("f32", 64, False), ("bf16", 128, False), ("f32", 128, False),
                                                ("bf16", 64, False), ("bf16", 128, True), ("bf16", 64, True)])
def test_merge_alone(dtype, d, parts_bf16):
    rng = np.random.default_rng(700 + d)
    b, hq, t, parts = 2, 3, 9, 5
    o_parts = rng.standard_normal((b, hq, parts, t, d)).astype(np.float32)
    if parts_bf16:
        o_parts = synth.round_to_bf16(o_parts)      # the stored parts are the merge's inputs
    lse_parts = (rng.standard_normal((b, hq, parts, t)) * 4).astype(np.float32)
    lse_parts[0, 0, 1, :] = -np.inf          # an empty part whose output rows hold NaN
    o_parts[0, 0, 1] = np.nan
    lse_parts[1, 2, :, 4] = -np.inf          # a row with every part empty
    dt = torch_dtype(dtype)
    out = torch.full((b, hq, t, d), float("nan"), dtype=dt, device="cuda")
    lse = torch.full((b, hq, t), float("nan"), dtype=torch.float32, device="cuda")
    desc = ls.make_desc(out, None, None, None, None, out, 0)
    desc.n_kv_heads = hq
    dev_parts = torch.from_numpy(o_parts).cuda()
    if parts_bf16:
        dev_parts = dev_parts.to(torch.bfloat16)
    ls.ls_lse_merge(desc, parts, dev_parts, torch.from_numpy(lse_parts).cuda(), out, lse)
    torch.cuda.synchronize()
    ro, rl = oracle.lse_merge(np.moveaxis(o_parts, 2, 3).reshape(-1, parts, d).astype(np.float64),
                              np.moveaxis(lse_parts, 2, 3).reshape(-1, parts).astype(np.float64))
    got_o = out.float().cpu().numpy().reshape(-1, d)
    got_l = lse.cpu().numpy().reshape(-1)
    dead = np.isneginf(rl)
    assert dead.sum() == 1 and np.all(np.isneginf(got_l[dead])) and np.all(got_o[dead] == 0)
    tol = 1e-5 if dtype == "f32" else 2e-2
    assert np.abs(got_o[~dead] - ro[~dead]).max() <= tol
    assert np.abs(got_l[~dead] - rl[~dead]).max() <= 1e-5


# ------------------------------------------------------------- (b) cached keys, by split ----

PREFIX_CASES = [
    # dtype, hq, hkv, d, t, prefix lengths, n_splits
    ("f32", 4, 1, 64, 16, [1024], 0),
    ("f32", 6, 2, 128, 11, [333, 70], 3),
    ("bf16", 32, 8, 128, 64, [1500], 0),       # 256-row query tile, ragged last key tile
    ("bf16", 32, 8, 128, 64, [64 * 7], 7),     # whole tiles only
    ("bf16", 8, 8, 128, 32, [1000, 129], 4),   # MHA: 32-row tile; second sequence leaves splits empty
    ("bf16", 10, 2, 128, 19, [777], 2),        # 95 rows: partly filled row groups
    ("bf16", 40, 8, 128, 128, [900, 2100], 5),  # 640 rows: three query blocks
    ("bf16", 12, 4, 64, 40, [1111], 3),        # head_dim 64
    ("bf16", 4, 4, 128, 5, [1], 1),            # a single cached row
]


@pytest.mark.parametrize("parts_bf16", [False, True])
@pytest.mark.parametrize("dtype,hq,hkv,d,t,plens,n_splits", PREFIX_CASES)
def test_prefix_splits_alone(dtype, hq, hkv, d, t, plens, n_splits, parts_bf16):
    if parts_bf16 and dtype != "bf16":
        pytest.skip("bf16 partials go with bf16 problems")
    rng = np.random.default_rng(800 + hq + t)
    seqs = [synth.make_sequence(rng, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_tree=t,
                                prefix_len=p, parents=synth.tree_chain(t), variant="peaked") for p in plens]
    w = synth.Workload("case", dtype, len(seqs), hq, hkv, d, t, min(plens), max(plens), None, None, 0)
    db = DeviceBatch(synth.Batch(w, "peaked", seqs))
    s = n_splits or ls.ls_prefix_num_splits(db.desc)
    length = ls.ls_prefix_split_len(db.desc, n_splits)
    o = torch.full((len(seqs), hq, s, t, d), float("nan"), dtype=torch.bfloat16 if parts_bf16 else torch.float32,
                   device="cuda")
    l = torch.full((len(seqs), hq, s, t), float("nan"), dtype=torch.float32, device="cuda")
    say(f"prefix-only parts_bf16={parts_bf16} {dtype} hq={hq} hkv={hkv} d={d} t={t} plens={plens} splits={s} len={length}")
    ls.ls_prefix_attn_splitkv(db.desc, db.q, db.k_cache, db.v_cache, db.prefix_lens, n_splits, o, l)
    torch.cuda.synchronize()
    o, l = o.float().cpu().numpy(), l.cpu().numpy()
    for b, sq in enumerate(seqs):
        for k in range(s):
            lo, hi = min(k * length, sq.prefix_len), min((k + 1) * length, sq.prefix_len)
            if lo == hi:
                assert np.all(np.isneginf(l[b, :, k])), f"empty split {k} of sequence {b}"
                continue
            ro, rl = oracle.attn_all(sq.q, sq.k_cache, sq.v_cache, sq.k_tree, sq.v_tree, sq.parents,
                                     prefix_lo=lo, prefix_hi=hi, use_tree=False)
            say(gates(o[b, :, k], l[b, :, k], ro, rl, dtype, f"  b={b} split={k} [{lo},{hi})", stress=True))


# ----------------------------------------------------------------- the whole path, small ----

@pytest.mark.parametrize("variant", ["iid", "peaked", "tree"])
def test_full_path_c1(variant):
    batch = synth.make_batch(synth.WORKLOADS["C1"], variant)
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, "f32", f"C1 {variant}", stress=variant != "iid"))


@pytest.mark.parametrize("name,prefix,variant", [
    ("C2", 2000, "iid"), ("C2", 2000, "peaked"), ("C2", 2000, "tree"),
    ("C3", 3100, "peaked"),
    ("C4", 1777, "iid"), ("C4", 1777, "peaked"), ("C4", 1777, "tree"),
])
def test_full_path_reduced_prefix(name, prefix, variant):
    batch = small(name, prefix, variant)
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, "bf16", f"{name} P={prefix} {variant}",
              stress=variant != "iid"))


@pytest.mark.parametrize("variant", ["iid", "peaked", "tree"])
def test_full_path_ragged_batch(variant):
    """The batched shape with per-sequence prefix lengths (and per-sequence trees)."""
    w = dataclasses.replace(synth.WORKLOADS["C5"], prefix_lo=150, prefix_hi=1900)
    batch = synth.make_batch(w, variant)
    assert len(set(batch.prefix_lens.tolist())) == 4
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, "bf16", f"C5 ragged {variant}",
              stress=variant != "iid"))
    err = ls.ls_workspace_error(db.desc, db.workspace)
    assert err >= db.workspace.data_ptr()


@pytest.mark.parametrize("dtype,hq,hkv,d,t,plens", [
    ("bf16", 8, 2, 64, 24, [1300]),          # head_dim 64 through the whole path
    ("f32", 6, 2, 128, 9, [700, 333]),       # float problem with head_dim 128, two sequences
    ("bf16", 4, 4, 128, 1, [900]),           # a single tree token: plain decode attention
    ("bf16", 14, 2, 128, 100, [2000]),       # 700 rows per KV head, two mask words
    ("bf16", 2, 1, 128, 128, [64, 4100, 1]),  # largest tree, very different lengths
    ("f32", 2, 2, 64, 128, [100]),
])
def test_full_path_other_shapes(dtype, hq, hkv, d, t, plens):
    rng = np.random.default_rng(900 + hq + t)
    seqs = []
    for pl in plens:
        parents = synth.tree_constrained(rng, t, 10, 4) if t > 1 else np.asarray([-1], dtype=np.int32)
        seqs.append(synth.make_sequence(rng, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_tree=t,
                                        prefix_len=pl, parents=parents, variant="peaked"))
    w = synth.Workload("case", dtype, len(seqs), hq, hkv, d, t, min(plens), max(plens), None, None, 0)
    batch = synth.Batch(w, "peaked", seqs)
    db = DeviceBatch(batch)
    say(f"whole path {dtype} hq={hq} hkv={hkv} d={d} t={t} plens={plens} splits={ls.ls_prefix_num_splits(db.desc)}")
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, dtype, "  result", stress=True))


@pytest.mark.parametrize("dtype,hq,hkv,d,t,depth,plens", [
    ("bf16", 2, 1, 128, 8, 4, [30000]),       # one KV head, few rows: > 32 parts, a wavefront per row, several batches
    ("bf16", 4, 1, 64, 8, 4, [20000]),        # the same with head_dim 64: 2-byte pieces per lane
    ("f16", 8, 2, 128, 16, 6, [3000]),        # 17 .. 32 parts, a wavefront per row
    ("bf16", 3, 3, 128, 7, 3, [5000]),        # 21 rows: the last wavefront is part empty; no query grouping
    ("bf16", 10, 2, 128, 300, 40, [1500]),    # five mask words, up to 41 visible keys per row, group of five
    ("bf16", 40, 8, 128, 33, 8, [900, 40]),   # at most four parts, 16 lanes per row
    ("bf16", 40, 8, 128, 33, 8, [2000, 700]), # five to eight parts: two requests of four, one after the other
    ("f16", 20, 4, 64, 130, 9, [1800]),       # the same with head_dim 64 and three mask words
    ("f32", 4, 2, 128, 70, 12, [3000]),       # float rows of 512 bytes, two mask words
])
def test_tail_kernel_forms(dtype, hq, hkv, d, t, depth, plens):
    """Whole-path calls whose shapes select each form of the kernel that ends the call (lanes per
    query row, split rows per request, one or two register sets), checked against the oracle."""
    rng = np.random.default_rng(7100 + hq * t)
    seqs = []
    for pl in plens:
        parents = synth.tree_constrained(rng, t, depth, 4)
        seqs.append(synth.make_sequence(rng, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_tree=t,
                                        prefix_len=pl, parents=parents, variant="peaked"))
    w = synth.Workload("case", dtype, len(seqs), hq, hkv, d, t, min(plens), max(plens), None, None, 0)
    batch = synth.Batch(w, "peaked", seqs)
    db = DeviceBatch(batch)
    say(f"tail forms {dtype} hq={hq} hkv={hkv} d={d} t={t} plens={plens} splits={ls.ls_prefix_num_splits(db.desc)}")
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, dtype, "  result", stress=True))


def test_full_path_token_major_layout():
    batch = small("C2", 1300, "peaked")
    db = DeviceBatch(batch, token_major=True)
    assert db.k_cache.stride(1) == 128 and db.k_cache.stride(2) == 8 * 128
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, "bf16", "C2 token-major", stress=True))


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_empty_prefix_is_tree_only(name):
    w = synth.WORKLOADS[name]
    batch = small(name, 0, "peaked")
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, w.dtype, f"{name} P=0", stress=True))
    # the same through a descriptor that allows a prefix, with device-side length 0
    batch2 = small(name, 200, "peaked")
    db2 = DeviceBatch(batch2)
    db2.prefix_lens.zero_()
    out2, lse2 = db2.run_full()
    torch.cuda.synchronize()
    for s in batch2.seqs:
        s.k_cache, s.v_cache, s.prefix_len = s.k_cache[:, :0], s.v_cache[:, :0], 0
    ro2, rl2 = oracle_full(batch2)
    say(gates(out2.float().cpu().numpy(), lse2.cpu().numpy(), ro2, rl2, w.dtype, f"{name} len=0 on device",
              stress=True))


def test_chain_tree_equals_causal_attention_on_device():
    """Chain-shaped tree: the device result must equal causal attention over [cache || tree]."""
    w = dataclasses.replace(synth.WORKLOADS["C2"], max_depth=None, max_children=None)
    batch = synth.make_batch(w, "peaked", prefix_override=700)
    for s in batch.seqs:
        s.parents = synth.tree_chain(w.n_tree)
    db = DeviceBatch(batch)
    out, _ = db.run_full()
    torch.cuda.synchronize()
    s = batch.seqs[0]
    g = w.group
    k = torch.from_numpy(np.repeat(np.concatenate([s.k_cache, s.k_tree], axis=1), g, axis=0)).double()[None]
    v = torch.from_numpy(np.repeat(np.concatenate([s.v_cache, s.v_tree], axis=1), g, axis=0)).double()[None]
    q = torch.cat([torch.zeros(w.n_q_heads, 700, w.head_dim), torch.from_numpy(s.q)], dim=1).double()[None]
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)[0, :, 700:].numpy()
    err = np.abs(out[0].float().cpu().numpy() - ref).max()
    say(f"chain == causal: max_abs={err:.3e}")
    assert err <= 2e-2 * np.abs(ref).max()


@pytest.mark.parametrize("name,prefix,used", [("C2", 2000, 2000), ("C2", 2000, 1337), ("C2", 2000, 0), ("C1", 1024, 700),
                                              ("C4", 1500, 64)])
def test_single_sequence_form_equals_the_batched_call(name, prefix, used):
    """ls_hybrid_tree_attn_single takes the prefix length by value; same bits as the device-array form."""
    batch = small(name, prefix, "peaked")
    db = DeviceBatch(batch)
    db.prefix_lens.fill_(used)
    out_a, lse_a = db.run_full()
    out_a, lse_a = out_a.clone(), lse_a.clone()
    out_b, lse_b = torch.full_like(db.out, float("nan")), torch.full_like(db.lse, float("nan"))
    ls.ls_hybrid_tree_attn_single(db.desc, db.q, db.k_cache, db.v_cache, used, db.k_tree, db.v_tree, db.parents,
                                  out_b, lse_b, db.workspace)
    torch.cuda.synchronize()
    assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b)
    s = batch.seqs[0]
    ro, rl = oracle.attn_all(s.q, s.k_cache[:, :used], s.v_cache[:, :used], s.k_tree, s.v_tree, s.parents)
    say(gates(out_b.float().cpu().numpy()[0], lse_b.cpu().numpy()[0], ro, rl, batch.workload.dtype,
              f"  single-sequence form {name} prefix {used} of {prefix}", stress=True))


def test_repeat_calls_are_bit_identical():
    batch = small("C2", 2500, "peaked")
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    first_o, first_l = out.clone(), lse.clone()
    for _ in range(10):
        out.fill_(float("nan"))
        db.run_full()
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), first_o.view(torch.int16))
    assert torch.equal(lse.view(torch.int32), first_l.view(torch.int32))


def test_bad_parents_on_device_set_the_error_word():
    batch = small("C2", 300, "iid")
    db = DeviceBatch(batch)
    db.parents[0, 5] = 9
    db.run_full()
    torch.cuda.synchronize()
    addr = ls.ls_workspace_error(db.desc, db.workspace)
    off = addr - db.workspace.data_ptr()
    word = db.workspace[off:off + 4].view(torch.int32).cpu().item()
    assert word == 1
    assert torch.isfinite(db.out.float()).all()


# ------------------------------------- cached keys only (draft-side cross-attention) ----

@pytest.mark.parametrize("dtype,hq,hkv,d,t,plens", [
    ("bf16", 32, 8, 128, 16, [3000]),        # one drafting step of beam width 16, GQA 4:1
    ("bf16", 32, 8, 128, 4, [2100]),         # beam width 4
    ("bf16", 8, 8, 64, 16, [1500, 70, 0]),   # MHA, head_dim 64, a sequence with an empty cache
    ("f32", 4, 1, 64, 16, [1024]),
])
def test_cache_only_attention(dtype, hq, hkv, d, t, plens):
    rng = np.random.default_rng(950 + hq + t)
    seqs = [synth.make_sequence(rng, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_tree=t,
                                prefix_len=pl, parents=synth.tree_chain(t), variant="peaked") for pl in plens]
    w = synth.Workload("case", dtype, len(seqs), hq, hkv, d, t, min(plens), max(plens), None, None, 0, "cross")
    batch = synth.Batch(w, "peaked", seqs)
    db = DeviceBatch(batch)
    out, lse = db.run_cache_only()
    torch.cuda.synchronize()
    out, lse = out.float().cpu().numpy(), lse.cpu().numpy()
    for b, sq in enumerate(seqs):
        if sq.prefix_len == 0:
            assert np.all(out[b] == 0) and np.all(np.isneginf(lse[b]))
            continue
        ro, rl = oracle.attn_all(sq.q, sq.k_cache, sq.v_cache, sq.k_tree, sq.v_tree, sq.parents, use_tree=False)
        say(gates(out[b], lse[b], ro, rl, dtype, f"cache only {dtype} hq={hq} t={t} P={sq.prefix_len}", stress=True))


def test_cache_only_full_size_d1():
    w = synth.WORKLOADS["D1"]
    batch = synth.make_batch(w, "iid")
    db = DeviceBatch(batch)
    out, lse = db.run_cache_only()
    torch.cuda.synchronize()
    sq = batch.seqs[0]
    ro, rl = oracle.attn_all(sq.q, sq.k_cache, sq.v_cache, sq.k_tree, sq.v_tree, sq.parents, use_tree=False)
    say(gates(out[0].float().cpu().numpy(), lse[0].cpu().numpy(), ro, rl, "bf16", "D1 full size, all rows"))


# ------------------------------------------------ properties that hold at any size ----

def _prefix_then_merge(db, n_splits, part_dtype):
    """ls_prefix_attn_splitkv with a chosen split count + ls_tree_attn_masked + ls_lse_merge: the
    path assembled from its stand-alone subsystems (three more launches than the fused call)."""
    w = db.batch.workload
    b, hq, t, d = db.q.shape
    o = torch.zeros((b, hq, n_splits + 1, t, d), dtype=torch.float32, device="cuda")
    l = torch.full((b, hq, n_splits + 1, t), float("-inf"), dtype=torch.float32, device="cuda")
    op = torch.empty((b, hq, n_splits, t, d), dtype=part_dtype, device="cuda")
    lp = torch.empty((b, hq, n_splits, t), dtype=torch.float32, device="cuda")
    ls.ls_prefix_attn_splitkv(db.desc, db.q, db.k_cache, db.v_cache, db.prefix_lens, n_splits, op, lp)
    words = (t + 63) // 64
    mask = torch.zeros((b, t, words), dtype=torch.int64, device="cuda")
    ls.ls_build_tree_mask(db.parents, mask)
    ot = torch.empty((b, hq, t, d), dtype=torch.float32, device="cuda")
    lt = torch.empty((b, hq, t), dtype=torch.float32, device="cuda")
    ls.ls_tree_attn_masked(db.desc, db.q, db.k_tree, db.v_tree, mask, ot, lt)
    o[:, :, :n_splits] = torch.nan_to_num(op.float(), nan=0.0)      # empty splits hold whatever was there
    l[:, :, :n_splits] = lp
    o[:, :, n_splits] = ot
    l[:, :, n_splits] = lt
    out = torch.empty_like(db.out)
    lse = torch.empty_like(db.lse)
    ls.ls_lse_merge(db.desc, n_splits + 1, o, l, out, lse)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), lse.cpu().numpy()


@pytest.mark.parametrize("name,prefix", [("C2", 2300), ("C4", 1500), ("C1", 1024)])
def test_split_count_does_not_matter(name, prefix):
    """The appendix proposition on the device: any number of key splits, assembled from the
    stand-alone subsystems, gives the same result as the fused call (and as the oracle)."""
    batch = small(name, prefix, "peaked")
    w = batch.workload
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    base_o, base_l = out.float().cpu().numpy(), lse.cpu().numpy()
    ro, rl = oracle_full(batch)
    tol = 2e-2 if w.dtype == "bf16" else 1e-5
    for n_splits in (1, 3, 7):
        o, l = _prefix_then_merge(db, n_splits, torch.float32)
        say(gates(o, l, ro, rl, w.dtype, f"{name} assembled, {n_splits} splits, float parts", stress=True))
        assert np.abs(o - base_o).max() <= tol * max(1.0, np.abs(ro).max())
        assert np.abs(l - base_l).max() <= (2e-3 if w.dtype == "bf16" else 2e-5)
    if w.dtype == "bf16":
        o, l = _prefix_then_merge(db, 5, torch.bfloat16)
        say(gates(o, l, ro, rl, w.dtype, f"{name} assembled, 5 splits, bf16 parts", stress=True))


def test_permuting_cached_rows_on_device():
    """Reordering the cached rows (K and V together) changes tile and split membership of every
    key but not the result beyond rounding."""
    batch = small("C2", 1900, "peaked")
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    o1, l1 = out.float().cpu().numpy().copy(), lse.cpu().numpy().copy()
    perm = torch.randperm(1900, device="cuda", generator=torch.Generator(device="cuda").manual_seed(5))
    db.k_cache.copy_(db.k_cache[:, :, perm].clone())
    db.v_cache.copy_(db.v_cache[:, :, perm].clone())
    out, lse = db.run_full()
    torch.cuda.synchronize()
    o2, l2 = out.float().cpu().numpy(), lse.cpu().numpy()
    assert np.abs(l2 - l1).max() < 1e-4
    assert np.abs(o2 - o1).max() <= 2e-2 * np.abs(o1).max()
    assert np.sqrt(((o2 - o1) ** 2).mean()) <= 5e-3 * np.sqrt((o1 ** 2).mean())


def test_scale_override_and_group_mapping():
    """softmax_scale from the descriptor is honoured, and query head h reads KV head h // G:
    with distinct KV heads, shuffling KV heads changes the result unless the query heads move too."""
    batch = small("C2", 800, "peaked")
    db = DeviceBatch(batch)
    db.desc.softmax_scale = 0.05
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch, scale=0.05)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, "bf16", "C2 scale 0.05", stress=True))
    g = batch.workload.group
    hkv = batch.workload.n_kv_heads
    perm = torch.tensor([3, 0, 1, 2, 5, 4, 7, 6], device="cuda")
    qperm = (perm[:, None] * g + torch.arange(g, device="cuda")[None, :]).reshape(-1)
    db2 = DeviceBatch(batch)
    db2.desc.softmax_scale = 0.05
    for name in ("k_cache", "v_cache", "k_tree", "v_tree"):
        getattr(db2, name).copy_(getattr(db2, name)[:, perm].clone())
    db2.q.copy_(db2.q[:, qperm].clone())
    out2, lse2 = db2.run_full()
    torch.cuda.synchronize()
    assert torch.equal(out2.view(torch.int16), out[:, qperm].view(torch.int16)), "head grouping"
    assert hkv == 8


# ------------------------------------------------ the benchmark shapes at full size ----

# rows per sequence that the oracle computes at full size: every row where that takes a second or
# two on the GPU machine's host cores, else a sample of 512 (rows are independent of each other)
FULL_SIZE_ROWS = {"C2": None, "C3": None, "C4": None, "H3": None, "C5": 512, "B3": 512, "L3": 512}


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "C5", "B3", "L3", "H3"])
def test_full_size_rows(name):
    """The benchmark shapes at full size, in the launch configuration the benchmark times, under
    the stated (unscaled) tolerance: max-abs 2e-2 on out for bf16."""
    w = synth.WORKLOADS[name]
    say(f"{name}: drawing inputs")
    batch = synth.make_batch(w, "iid")
    db = DeviceBatch(batch)
    say(f"{name}: prefix lens {batch.prefix_lens.tolist()}, splits {ls.ls_prefix_num_splits(db.desc)}")
    out, lse = db.run_full()
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()
    lse = lse.cpu().numpy()
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))
    n_rows = FULL_SIZE_ROWS[name]
    if n_rows is None:
        ro, rl = oracle_full(batch)
        say(gates(out, lse, ro, rl, w.dtype, f"{name} full size, all {w.n_q_heads * w.n_tree} rows per sequence"))
    else:
        rng = np.random.default_rng(w.seed + 99)
        rows, ro, rl = oracle_full(batch, rows_per_seq=n_rows, rng=rng)
        got_o = np.stack([out[b, rows[b, :, 0], rows[b, :, 1]] for b in range(w.batch)])
        got_l = np.stack([lse[b, rows[b, :, 0], rows[b, :, 1]] for b in range(w.batch)])
        say(gates(got_o, got_l, ro, rl, w.dtype, f"{name} full size, {rows.shape[1]} sampled rows per sequence"))
    # a property that holds for every row at any size: with i.i.d. N(0,1) logits the
    # log-sum-exp sits close to ln(number of visible keys) + 1/2
    expect = np.log(batch.prefix_lens.astype(np.float64))[:, None, None] + 0.5
    assert np.abs(lse - expect).max() < 0.5


@pytest.mark.parametrize("name,prefix", [("C2", None), ("C3", None), ("C2", 1500)])
def test_error_budget_of_the_16_bit_partials(name, prefix):
    """Peaked inputs (outputs of magnitude 4 to 6): how much of the error against the oracle is the
    output format itself, how much the rounding of the split partials to bf16.  The whole path is
    run three ways: the fused call (bf16 partials), the stand-alone subsystems with bf16 partials,
    and the stand-alone subsystems with float partials; the floor is the oracle's own result
    rounded to bf16."""
    w = synth.WORKLOADS[name]
    batch = synth.make_batch(w, "peaked", prefix_override=prefix)
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    fused = out.float().cpu().numpy()
    ro, rl = oracle_full(batch)
    floor = np.abs(synth.round_to_bf16(ro.astype(np.float32)).astype(np.float64) - ro).max()
    n_splits = ls.ls_prefix_num_splits(db.desc)
    o32, l32 = _prefix_then_merge(db, n_splits, torch.float32)
    o16, l16 = _prefix_then_merge(db, n_splits, torch.bfloat16)
    scale = np.abs(ro).max()
    e = {"fused": np.abs(fused - ro).max(), "float partials": np.abs(o32 - ro).max(),
         "bf16 partials": np.abs(o16 - ro).max()}
    rms = {"fused": np.sqrt(((fused - ro) ** 2).mean()), "float partials": np.sqrt(((o32 - ro) ** 2).mean()),
           "bf16 partials": np.sqrt(((o16 - ro) ** 2).mean()),
           "floor": np.sqrt(((synth.round_to_bf16(ro.astype(np.float32)) - ro) ** 2).mean())}
    say(f"{name} peaked prefix {batch.prefix_lens.tolist()} splits {n_splits}: max|ref| {scale:.2f}; max-abs error: "
        f"output format alone {floor:.3e}; float partials {e['float partials']:.3e}; bf16 partials "
        f"{e['bf16 partials']:.3e}; fused call {e['fused']:.3e} | rms: floor {rms['floor']:.3e}, float partials "
        f"{rms['float partials']:.3e}, bf16 partials {rms['bf16 partials']:.3e}, fused {rms['fused']:.3e}")
    # the fused call computes what the assembled path with bf16 partials computes
    assert np.abs(fused - o16).max() <= 2.0 ** -7 * scale
    # with float partials what remains is the output rounding plus the bf16 numerators: a row's
    # result is sum p_i v_i / sum p_i with every p_i in the numerator rounded to bf16 (relative
    # 2^-9) and the denominator not, so it moves by at most 2^-9 max|v| before it is rounded
    vmax = max(max(float(np.abs(sq.v_cache).max()) if sq.prefix_len else 0.0, float(np.abs(sq.v_tree).max()))
               for sq in batch.seqs)
    assert e["float partials"] <= floor + 2.0 ** -9 * vmax * 1.02
    assert e["bf16 partials"] <= 2e-2 * max(1.0, scale) and e["fused"] <= 2e-2 * max(1.0, scale)
    assert rms["float partials"] <= rms["bf16 partials"] * 1.05 + 1e-6


def test_full_size_peaked_c3():
    w = synth.WORKLOADS["C3"]
    batch = synth.make_batch(w, "peaked")
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    rng = np.random.default_rng(4242)
    rows, ro, rl = oracle_full(batch, rows_per_seq=96, rng=rng)
    got_o = out.float().cpu().numpy()[0, rows[0, :, 0], rows[0, :, 1]][None]
    got_l = lse.cpu().numpy()[0, rows[0, :, 0], rows[0, :, 1]][None]
    say(gates(got_o, got_l, ro, rl, "bf16", "C3 full size peaked", stress=True))


def test_two_streams_with_their_own_workspaces_do_not_disturb_each_other():
    """The library keeps no device state of its own: calls on different streams with different
    workspaces may overlap, and each gives the result it gives alone."""
    a, b = DeviceBatch(small("C2", 3000, "peaked")), DeviceBatch(small("C4", 2500, "tree"))
    ref = []
    for db in (a, b):
        o, l = db.run_full()
        torch.cuda.synchronize()
        ref.append((o.clone(), l.clone()))
        db.out.fill_(float("nan"))
        db.lse.fill_(float("nan"))
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(20):
        a.run_full(stream=s1)
        b.run_full(stream=s2)
    torch.cuda.synchronize()
    for db, (o, l) in zip((a, b), ref):
        assert torch.equal(db.out, o) and torch.equal(db.lse, l)


def test_the_call_neither_allocates_nor_waits():
    """Device memory in use is the same before and after many calls, and the host is back from a
    call long before the GPU has finished it (nothing in the call synchronises)."""
    import time
    db = DeviceBatch(synth.make_batch(synth.WORKLOADS["C3"], "iid"))
    db.run_full()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    n = 200
    t0 = time.perf_counter()
    for _ in range(n):
        db.run_full()
    host = time.perf_counter() - t0
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, "device memory in use changed across calls"
    say(f"200 calls: host returned after {host * 1e3:.2f} ms, GPU done after {total * 1e3:.2f} ms")
    assert host < 0.6 * total


def test_whole_call_under_hip_graph_capture():
    """The call allocates nothing and records no memset, so it can be captured; every replay
    (with eager calls and synchronisations in between) must reproduce the eager result bit for
    bit."""
    batch = small("C2", 3000, "peaked")
    db = DeviceBatch(batch)
    db.run_full()
    torch.cuda.synchronize()
    ref_o, ref_l = db.out.clone(), db.lse.clone()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        db.run_full(stream=side)
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            db.run_full(stream=side)
    torch.cuda.synchronize()
    for rep in range(4):
        db.out.zero_()
        db.lse.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(db.out, ref_o) and torch.equal(db.lse, ref_l), f"replay {rep}"
        other = DeviceBatch(small("C2", 500 + 100 * rep, "iid"))   # eager work between replays
        other.run_full()
        torch.cuda.synchronize()


def test_draft_window_self_attention_shape():
    """The draft model's sliding-window self-attention (Section 3.1): at most 512 cached rows
    plus the drafted tree; the same call at a short prefix."""
    batch = synth.make_batch(synth.WORKLOADS["W1"], "peaked")
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, "bf16", "W1 window 512 + 68-node tree", stress=True))
