"""The single-launch form of the whole call (ls_hybrid_tree_attn_fused: the workgroups of a
query block count themselves in and merge the block's rows between them, or leave them to the
one that completes the count) through the C ABI: against the CPU oracle, against the two-launch
call, against itself on repeated calls (the arrival order changes from call to call, the bits
must not), and with the bounded wait cut to nothing or next to nothing from the host (every
row is then still written, by the same code, so the bits must not change either).
"""
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


def bits(t):
    return t.contiguous().view(torch.uint8).cpu().numpy().tobytes()


def custom(dtype, hq, hkv, d, t, depth, plens, seed, variant="peaked"):
    rng = np.random.default_rng(seed)
    seqs = []
    for pl in plens:
        parents = synth.tree_constrained(rng, t, depth, 4) if t > 1 else np.asarray([-1], dtype=np.int32)
        seqs.append(synth.make_sequence(rng, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_tree=t,
                                        prefix_len=pl, parents=parents, variant=variant))
    w = synth.Workload("case", dtype, len(seqs), hq, hkv, d, t, min(plens), max(plens), None, None, 0)
    return synth.Batch(w, variant, seqs)


CASES = {
    "C2 shape, 3000 keys": lambda: synth.make_batch(synth.WORKLOADS["C2"], "iid", prefix_override=3000),
    "C3 shape, 9000 keys, peaked": lambda: synth.make_batch(synth.WORKLOADS["C3"], "peaked", prefix_override=9000),
    "ragged batch of four, 640 rows per KV head": lambda: custom("bf16", 40, 8, 128, 128, 10, [700, 64, 2100, 1], 81),
    "276 rows per KV head (two query blocks, one nearly empty)": lambda: custom("bf16", 8, 2, 128, 69, 5, [2500], 82),
    "head_dim 64, f16": lambda: custom("f16", 8, 2, 64, 24, 6, [1300], 83),
    "five mask words": lambda: custom("bf16", 4, 2, 128, 300, 30, [900], 84),
    "no cached keys at all": lambda: custom("bf16", 8, 2, 128, 16, 4, [0, 0], 85),
    "one tree token": lambda: custom("bf16", 4, 4, 128, 1, 1, [900], 86),
    "21 rows, no grouping": lambda: custom("bf16", 3, 3, 128, 7, 3, [5000], 87),
}


@pytest.mark.parametrize("name", list(CASES))
def test_single_launch_call(name):
    batch = CASES[name]()
    w = batch.workload
    db = DeviceBatch(batch)
    say(f"single launch: {name}; splits={ls.ls_prefix_num_splits(db.desc)} prefix={batch.prefix_lens.tolist()}")
    out2, lse2 = db.run_full()          # two launches; creates no counters
    torch.cuda.synchronize()
    out2, lse2 = out2.float().cpu().numpy(), lse2.cpu().numpy()
    db.workspace = None                  # a fresh workspace, filled with 0xFF, counters zeroed by ls_workspace_init
    runs = []
    for rep in range(3):
        db.out.fill_(float("nan"))
        db.lse.fill_(float("nan"))
        out, lse = db.run_fused()
        torch.cuda.synchronize()
        runs.append((bits(out), bits(lse)))
        if rep == 0:
            ref_out, ref_lse = oracle_full(batch)
            say(gates(out.float().cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, w.dtype, "  vs oracle",
                      stress=batch.variant != "iid"))
            tol = 2e-2 * max(1.0, float(np.abs(ref_out).max()))
            assert np.abs(out.float().cpu().numpy() - out2).max() <= tol
            fin = np.isfinite(lse2)
            assert np.array_equal(fin, np.isfinite(lse.cpu().numpy()))
            assert np.abs(lse.cpu().numpy()[fin] - lse2[fin]).max() <= 1e-4
    assert runs[0] == runs[1] == runs[2], "repeated single-launch calls differ"
    # nobody waits (the workgroup that completes a block's count does all its rows), and a wait
    # of one poll (most workgroups give up and leave their rows to that one): the same bits
    try:
        for polls in (0, 1):
            ls.ls_set_single_launch_polls(polls)
            db.out.fill_(float("nan"))
            db.lse.fill_(float("nan"))
            out, lse = db.run_fused()
            torch.cuda.synchronize()
            assert (bits(out), bits(lse)) == runs[0], f"polls={polls} changes the result"
    finally:
        ls.ls_set_single_launch_polls(-1)
    # the arrival words: count back at zero, call number = calls made, for the blocks the call has
    words = db.workspace[:ls.LS_WORKSPACE_COUNTER_BYTES].cpu().numpy().view(np.uint64).reshape(-1, 3)
    assert not (words[:, 0] & np.uint64(0xffffffff)).any()
    calls = (words[:, 0] >> np.uint64(32)).astype(np.int64)
    used = int((calls != 0).sum())
    assert used == 0 or (calls[:used] == 5).all() and not calls[used:].any()
    err = ls.ls_workspace_error(db.desc, db.workspace)
    assert err >= db.workspace.data_ptr()


def test_many_calls_in_a_row_agree_bit_for_bit():
    """The rows one workgroup writes are read by others of the same launch; a row read too early
    would show up as a changed result (or as the NaN the outputs are filled with) on some call."""
    batch = synth.make_batch(synth.WORKLOADS["C3"], "peaked", prefix_override=9000)
    db = DeviceBatch(batch)
    db.workspace = None
    out, lse = db.run_fused()
    torch.cuda.synchronize()
    ref_out, ref_lse = out.clone(), lse.clone()
    bad = 0
    for _ in range(400):
        db.out.fill_(float("nan"))
        db.lse.fill_(float("nan"))
        out, lse = db.run_fused()
        bad += int(not (torch.equal(out.view(torch.int16), ref_out.view(torch.int16)) and
                        torch.equal(lse.view(torch.int32), ref_lse.view(torch.int32))))
    torch.cuda.synchronize()
    say(f"single launch: 400 calls, {bad} differ from the first")
    assert bad == 0


def test_float_problems_take_two_launches_and_match_bit_for_bit():
    batch = synth.make_batch(synth.WORKLOADS["C1"], "peaked")
    db = DeviceBatch(batch)
    out2, lse2 = db.run_full()
    torch.cuda.synchronize()
    b2 = (bits(out2), bits(lse2))
    db.workspace = None
    out, lse = db.run_fused()
    torch.cuda.synchronize()
    assert (bits(out), bits(lse)) == b2


def test_poll_count_is_bounded():
    assert ls.ls_set_single_launch_polls((1 << 24) + 1, check=False) == ls.LS_ERR_SHAPE
    assert ls.ls_set_single_launch_polls(-1, check=False) == ls.LS_OK


def test_workspace_init_rejects_a_short_or_missing_workspace():
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    assert ls.ls_workspace_init(small, check=False) == ls.LS_ERR_WORKSPACE
    assert ls.ls_workspace_init(None, check=False) == ls.LS_ERR_WORKSPACE
