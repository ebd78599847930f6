"""The same path with IEEE half inputs (the precision of the paper's experiments, appendix
"Experiments Details"): parity against the CPU oracle through the C ABI.  The gates for this
type are derived in tests/util.py."""
import dataclasses
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2502_17421_amd import binding as ls
from paper_2502_17421_amd import synth
from util import DeviceBatch, gates, oracle_full, to_dev

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def batch_of(hq, hkv, d, t, plens, variant, seed, trees="constrained"):
    rng = np.random.default_rng(seed)
    seqs = []
    for pl in plens:
        par = synth.tree_constrained(rng, t, 8, 4) if trees == "constrained" and t > 1 else synth.tree_chain(t)
        seqs.append(synth.make_sequence(rng, dtype="f16", n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_tree=t,
                                        prefix_len=pl, parents=par, variant=variant))
    w = synth.Workload("case", "f16", len(seqs), hq, hkv, d, t, min(plens), max(plens), None, None, 0)
    return synth.Batch(w, variant, seqs)


@pytest.mark.parametrize("hq,hkv,d,t,plens,variant,token_major", [
    (32, 8, 128, 64, [1500], "iid", False),          # 256-row query tile, ragged last key tile
    (32, 8, 128, 64, [1500], "peaked", False),
    (32, 8, 128, 64, [2048], "tree", False),
    (8, 8, 128, 32, [1000, 129, 0], "peaked", False),  # MHA, 32-row tile, ragged batch with an empty cache
    (12, 4, 64, 40, [1111], "peaked", False),          # head_dim 64
    (40, 8, 128, 128, [900, 2100], "iid", False),      # 640 rows: three query blocks, two mask words
    (32, 8, 128, 64, [1300], "peaked", True),          # token-major storage
])
def test_whole_path_half(hq, hkv, d, t, plens, variant, token_major):
    batch = batch_of(hq, hkv, d, t, plens, variant, 9100 + hq + t)
    db = DeviceBatch(batch, token_major=token_major)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, "f16",
              f"f16 hq={hq} hkv={hkv} d={d} t={t} plens={plens} {variant} tm={token_major}", stress=variant != "iid"))


@pytest.mark.parametrize("parts_half", [False, True])
@pytest.mark.parametrize("hq,hkv,d,t,plens,n_splits", [(32, 8, 128, 64, [1500], 0), (10, 2, 128, 19, [777, 64], 3),
                                                        (12, 4, 64, 40, [1111], 5)])
def test_prefix_splits_alone_half(hq, hkv, d, t, plens, n_splits, parts_half):
    batch = batch_of(hq, hkv, d, t, plens, "peaked", 9200 + hq)
    db = DeviceBatch(batch)
    s = n_splits or ls.ls_prefix_num_splits(db.desc)
    length = ls.ls_prefix_split_len(db.desc, n_splits)
    o = torch.full((len(plens), hq, s, t, d), float("nan"), dtype=torch.float16 if parts_half else torch.float32,
                   device="cuda")
    l = torch.full((len(plens), hq, s, t), float("nan"), dtype=torch.float32, device="cuda")
    ls.ls_prefix_attn_splitkv(db.desc, db.q, db.k_cache, db.v_cache, db.prefix_lens, n_splits, o, l)
    torch.cuda.synchronize()
    o, l = o.float().cpu().numpy(), l.cpu().numpy()
    for b, sq in enumerate(batch.seqs):
        for k in range(s):
            lo, hi = k * length, min((k + 1) * length, sq.prefix_len)
            if lo >= hi:
                assert np.all(np.isneginf(l[b, :, k]))
                continue
            ro, rl = oracle.attn_all(sq.q, sq.k_cache, sq.v_cache, sq.k_tree, sq.v_tree, sq.parents, prefix_lo=lo,
                                     prefix_hi=hi, use_tree=False)
            gates(o[b, :, k], l[b, :, k], ro, rl, "f16", f"f16 split {k} of seq {b}", stress=True)
    say(f"f16 prefix-only parts_half={parts_half} hq={hq} d={d} t={t} plens={plens} splits={s}: ok")


def test_merge_alone_half_parts():
    rng = np.random.default_rng(9300)
    b, hq, t, d, parts = 2, 4, 9, 128, 7
    o_parts = synth.round_to_f16(rng.standard_normal((b, hq, parts, t, d)).astype(np.float32))
    lse_parts = rng.normal(0.0, 4.0, size=(b, hq, parts, t)).astype(np.float32)
    lse_parts[0, 1, 2] = -np.inf
    lse_parts[1, :, :, 3] = -np.inf            # a row with no visible key at all
    q = torch.zeros((b, hq, t, d), dtype=torch.float16, device="cuda")
    kv = torch.zeros((b, hq, 1, d), dtype=torch.float16, device="cuda")
    desc = ls.make_desc(q, kv, kv, q, q, q, 0)
    out = torch.full_like(q, float("nan"))
    lse = torch.full((b, hq, t), float("nan"), dtype=torch.float32, device="cuda")
    ls.ls_lse_merge(desc, parts, to_dev(o_parts, torch.float16), torch.from_numpy(lse_parts).cuda(), out, lse)
    torch.cuda.synchronize()
    ro, rl = oracle.lse_merge(o_parts.transpose(0, 1, 3, 2, 4).reshape(-1, parts, d).astype(np.float64),
                              lse_parts.transpose(0, 1, 3, 2).reshape(-1, parts).astype(np.float64))
    got_o = out.float().cpu().numpy().reshape(-1, d)
    got_l = lse.cpu().numpy().reshape(-1)
    dead = np.isneginf(rl)
    assert np.all(np.isneginf(got_l[dead])) and np.all(got_o[dead] == 0)
    assert np.abs(got_o[~dead] - ro[~dead]).max() <= 2e-3 * max(1.0, np.abs(ro[~dead]).max())
    assert np.abs(got_l[~dead] - rl[~dead]).max() <= 1e-5 * max(1.0, np.abs(rl[~dead]).max())


def test_cache_only_half():
    batch = batch_of(32, 8, 128, 16, [3000, 70], "peaked", 9400, trees="chain")
    db = DeviceBatch(batch)
    out, lse = db.run_cache_only()
    torch.cuda.synchronize()
    for b, sq in enumerate(batch.seqs):
        ro, rl = oracle.attn_all(sq.q, sq.k_cache, sq.v_cache, sq.k_tree, sq.v_tree, sq.parents, use_tree=False)
        say(gates(out[b].float().cpu().numpy(), lse[b].cpu().numpy(), ro, rl, "f16", f"f16 cache only P={sq.prefix_len}",
                  stress=True))


def test_full_size_c3_shape_half_sampled_rows():
    w = dataclasses.replace(synth.WORKLOADS["C3"], dtype="f16", name="C3h")
    batch = synth.make_batch(w, "iid")
    db = DeviceBatch(batch)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    rng = np.random.default_rng(9500)
    rows, ro, rl = oracle_full(batch, rows_per_seq=96, rng=rng)
    o = out.float().cpu().numpy()
    l = lse.cpu().numpy()
    got_o = np.stack([o[b][rows[b][:, 0], rows[b][:, 1]] for b in range(w.batch)])
    got_l = np.stack([l[b][rows[b][:, 0], rows[b][:, 1]] for b in range(w.batch)])
    say(gates(got_o, got_l, ro, rl, "f16", "C3 shape in f16, full size, 96 sampled rows"))


def test_part_dtype_must_match_the_problem():
    batch = batch_of(8, 2, 128, 8, [300], "iid", 9600)
    db = DeviceBatch(batch)
    s = ls.ls_prefix_num_splits(db.desc)
    o = torch.empty((1, 8, s, 8, 128), dtype=torch.bfloat16, device="cuda")
    l = torch.empty((1, 8, s, 8), dtype=torch.float32, device="cuda")
    rc = ls.ls_prefix_attn_splitkv(db.desc, db.q, db.k_cache, db.v_cache, db.prefix_lens, 0, o, l, check=False)
    assert rc == ls.LS_ERR_DTYPE
