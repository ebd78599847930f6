"""Shapes whose last query block of a KV head is light (at most 128 of 256 rows): some of its waves
hold no query row at all and only keep copying key tiles.  The paper's own tree (a root and 68
drafted nodes) under 4:1 grouping, 276 rows = 256 + 20, is such a shape."""
import sys

import numpy as np
import pytest
import torch

from paper_2502_17421_amd import binding as ls
from paper_2502_17421_amd import synth
from util import DeviceBatch, gates, oracle_full

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def make(dtype, hq, hkv, d, t, plens, variant, seed, beam=False):
    rng = np.random.default_rng(seed)
    seqs = []
    for pl in plens:
        parents = synth.tree_beam(rng) if beam else synth.tree_constrained(rng, t, 10, 4)
        seqs.append(synth.make_sequence(rng, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_tree=t,
                                        prefix_len=pl, parents=parents, variant=variant))
    w = synth.Workload("case", dtype, len(seqs), hq, hkv, d, t, min(plens), max(plens), None, None, 0)
    return synth.Batch(w, variant, seqs)


def uniform_workspace_bytes(db, w):
    """Workspace size if every query block were cut into ls_prefix_num_splits pieces."""
    up = lambda n: (n + 255) // 256 * 256
    s = ls.ls_prefix_num_splits(db.desc)
    rows = w.batch * w.n_q_heads * s * w.n_tree
    words = (w.n_tree + 63) // 64
    e = 4 if w.dtype == "f32" else 2
    return (ls.LS_WORKSPACE_COUNTER_BYTES + up(w.batch * w.n_tree * words * 8) + up(w.batch * 4) + up(rows * 4) +
            up(rows * w.head_dim * e))


CASES = [
    ("bf16", 32, 8, 128, 69, [3000], "peaked", True),           # 276 rows: one full block + 20 rows
    ("bf16", 32, 8, 128, 69, [2113], "iid", True),              # ragged last tiles
    ("bf16", 8, 1, 128, 69, [5000, 1200, 0], "peaked", True),   # 552 rows: two full blocks + 40; ragged batch
    ("f16", 12, 2, 64, 60, [2500], "iid", False),               # 360 rows: 256 + 104 (four waves, the last ragged)
    ("bf16", 20, 4, 128, 77, [4000, 3100], "tree", False),      # 385 rows: 256 + 129 -> five waves with rows
]


@pytest.mark.parametrize("dtype,hq,hkv,d,t,plens,variant,beam", CASES)
def test_whole_path_with_light_last_block(dtype, hq, hkv, d, t, plens, variant, beam):
    batch = make(dtype, hq, hkv, d, t, plens, variant, 13000 + hq + t, beam)
    db = DeviceBatch(batch)
    # every query block of the whole-path call is cut like the stand-alone cached-key call
    assert ls.ls_workspace_bytes(db.desc) == uniform_workspace_bytes(db, batch.workload)
    say(f"light last block {dtype} hq={hq} hkv={hkv} d={d} t={t} plens={plens} {variant}: "
        f"{ls.ls_prefix_num_splits(db.desc)} pieces")
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, dtype, "  result", stress=True))
    first = (out.clone(), lse.clone())
    db.workspace.fill_(0xFF)     # whatever the workspace held, the result is the same
    out, lse = db.run_full()
    torch.cuda.synchronize()
    assert torch.equal(out, first[0]) and torch.equal(lse, first[1])


def test_cache_only_with_light_last_block():
    batch = make("bf16", 32, 8, 128, 69, [2800], "peaked", 13300, True)
    db = DeviceBatch(batch)
    out, lse = db.run_cache_only()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch, use_tree=False)
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, "bf16", "  cached keys only, 276 rows", stress=True))


def test_paged_with_light_last_block_equals_contiguous():
    batch = make("bf16", 32, 8, 128, 69, [3072], "iid", 13400, True)
    db = DeviceBatch(batch)
    out_c, lse_c = db.run_full()
    out_c, lse_c = out_c.clone(), lse_c.clone()
    ps, per_seq = 32, 3072 // 32
    perm = torch.randperm(per_seq, generator=torch.Generator().manual_seed(9)) + 1    # page 0 stays poison
    table = perm.view(1, per_seq).to(torch.int32).cuda()

    def to_pages(x):
        pages = torch.full((per_seq + 1, x.shape[1], ps, x.shape[3]), float("nan"), dtype=x.dtype, device="cuda")
        pages[perm.cuda()] = x[0].view(x.shape[1], per_seq, ps, x.shape[3]).transpose(0, 1)
        return pages

    kp, vp = to_pages(db.k_cache), to_pages(db.v_cache)
    desc = ls.make_desc(db.q, kp, vp, db.k_tree, db.v_tree, db.out, 3072)
    ws = torch.empty(ls.ls_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    out_p, lse_p = torch.full_like(db.out, float("nan")), torch.full_like(db.lse, float("nan"))
    ls.ls_hybrid_tree_attn_paged(desc, db.q, kp, vp, table, ps, db.prefix_lens, db.k_tree, db.v_tree, db.parents,
                                 out_p, lse_p, ws)
    torch.cuda.synchronize()
    assert torch.equal(out_p, out_c) and torch.equal(lse_p, lse_c)
    ro, rl = oracle_full(batch)
    say(gates(out_p.float().cpu().numpy(), lse_p.cpu().numpy(), ro, rl, "bf16", "  paged, 276 rows", stress=True))
