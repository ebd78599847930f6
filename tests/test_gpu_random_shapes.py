"""Seeded random shapes through the whole path (contiguous and paged) against the oracle: every
draw picks dtype, head_dim, head grouping, tree size and shape (forests included), batch, prefix
lengths (empty, exact tile multiples, ragged) and storage order."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2502_17421_amd import binding as ls
from paper_2502_17421_amd import synth
from util import DeviceBatch, gates, oracle_full

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def draw_tree(rng, t):
    kind = rng.integers(0, 5)
    if kind == 0 or t == 1:
        return synth.tree_chain(t)
    if kind == 1:
        return synth.tree_star(t)
    if kind == 2:
        return synth.tree_constrained(rng, t, int(rng.integers(4, 12)), int(rng.integers(3, 6))) if t < 30 else \
            synth.tree_constrained(rng, t, 10, 4)
    par = synth.tree_uniform(rng, t)
    if kind == 4:                        # a forest: some nodes become roots of their own
        for i in range(1, t):
            if rng.random() < 0.15:
                par[i] = -1
    return par


def draw_case(seed):
    rng = np.random.default_rng(12000 + seed)
    dtype = ["bf16", "bf16", "f16", "f32"][int(rng.integers(0, 4))]
    d = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3, 4, 8]))
    g = int(rng.choice([1, 2, 4, 5, 8]))
    t = int(rng.choice([1, 2, 7, 16, 33, 64, 65, 100, 128]))
    if dtype == "f32":                   # the float kernel is slow: keep it small
        t, g = min(t, 33), min(g, 4)
    b = int(rng.integers(1, 4))
    plens = []
    for _ in range(b):
        kind = rng.integers(0, 4)
        plens.append(0 if kind == 0 else int(rng.integers(1, 5)) * 64 * int(rng.integers(1, 9)) if kind == 1 else
                     int(rng.integers(1, 2500)))
    if max(plens) == 0 and rng.random() < 0.5:
        plens[0] = int(rng.integers(1, 700))
    variant = ["iid", "peaked", "tree"][int(rng.integers(0, 3))]
    seqs = [synth.make_sequence(rng, dtype=dtype, n_q_heads=hkv * g, n_kv_heads=hkv, head_dim=d, n_tree=t, prefix_len=pl,
                                parents=draw_tree(rng, t), variant=variant) for pl in plens]
    w = synth.Workload(f"seed{seed}", dtype, b, hkv * g, hkv, d, t, min(plens), max(plens), None, None, 0)
    return synth.Batch(w, variant, seqs), bool(rng.integers(0, 2)), rng


@pytest.mark.parametrize("seed", range(36))
def test_random_shape_whole_path(seed):
    batch, token_major, rng = draw_case(seed)
    w = batch.workload
    db = DeviceBatch(batch, token_major=token_major)
    out, lse = db.run_full()
    torch.cuda.synchronize()
    ro, rl = oracle_full(batch)
    what = (f"seed {seed}: {w.dtype} B={w.batch} Hq={w.n_q_heads} Hkv={w.n_kv_heads} D={w.head_dim} T={w.n_tree} "
            f"P={batch.prefix_lens.tolist()} {batch.variant} tm={token_major}")
    say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ro, rl, w.dtype, what, stress=True))
    off = ls.ls_workspace_error(db.desc, db.workspace) - db.workspace.data_ptr()
    assert db.workspace[off:off + 4 * w.batch].view(torch.int32).cpu().tolist() == [0] * w.batch


@pytest.mark.parametrize("seed", range(36, 48))
def test_random_shape_paged(seed):
    from test_gpu_paged import PagedBatch
    batch, token_major, rng = draw_case(seed)
    w = batch.workload
    if w.dtype == "f32":
        pytest.skip("paged caches are for the 16-bit types")
    page_size = int(rng.choice([16, 32, 64, 128, 512]))
    pb = PagedBatch(batch, page_size, rng, token_major=token_major)
    out, lse = pb.run()
    ro, rl = oracle_full(batch)
    what = (f"seed {seed} paged {page_size}: {w.dtype} B={w.batch} Hq={w.n_q_heads} Hkv={w.n_kv_heads} D={w.head_dim} "
            f"T={w.n_tree} P={batch.prefix_lens.tolist()} {batch.variant} tm={token_major}")
    say(gates(out, lse, ro, rl, w.dtype, what, stress=True))
