"""The entry point that takes no workspace (ls_hybrid_tree_attn_static: the split partials go to a
fixed array inside the library) against the entry point it is a variant of, through the C ABI.

Same kernels and schedule, so the results must be bit-identical; on top of that the first result
is held against the CPU oracle.  Two calls in a row, the second on a smaller problem, so that
whatever the first call left in the shared array is still there when the second one runs.
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


def run_both(db):
    """(out, lse) of the workspace call and of the static-scratch call on the same device batch."""
    out_ws, lse_ws = db.run_full()
    torch.cuda.synchronize()
    out_ws, lse_ws = out_ws.clone(), lse_ws.clone()
    db.out.fill_(float("nan"))
    db.lse.fill_(float("nan"))
    ls.ls_hybrid_tree_attn_static(db.desc, db.q, db.k_cache, db.v_cache, db.prefix_lens, db.k_tree, db.v_tree,
                                  db.parents, db.out, db.lse)
    torch.cuda.synchronize()
    return (out_ws, lse_ws), (db.out.clone(), db.lse.clone())


def same_bits(a, b):
    return a.contiguous().view(torch.uint8).cpu().numpy().tobytes() == b.contiguous().view(torch.uint8).cpu().numpy().tobytes()


def test_static_scratch_call_matches_the_workspace_call_twice_in_a_row():
    assert torch.cuda.is_available(), "needs a GPU"
    ls.lib()
    # first: 8 KV heads x 256 query rows, 6000 cached keys (many splits, ragged last tile);
    # second: a smaller problem in every respect (fewer heads, shorter tree, shorter prefix)
    first = synth.make_batch(synth.WORKLOADS["C2"], "iid", prefix_override=6000)
    import dataclasses
    small_w = dataclasses.replace(synth.WORKLOADS["C2"], n_q_heads=8, n_kv_heads=2, n_tree=23, seed=4242)
    second = synth.make_batch(small_w, "peaked", prefix_override=777)
    for step, (batch, stress) in enumerate([(first, False), (second, True)]):
        say(f"static scratch: call {step}, workload {batch.workload.name}, prefix {batch.prefix_lens.tolist()}")
        db = DeviceBatch(batch)
        assert ls.ls_workspace_bytes(db.desc) <= ls.LS_STATIC_SCRATCH_BYTES
        (out_ws, lse_ws), (out_st, lse_st) = run_both(db)
        assert same_bits(out_ws, out_st), "out differs between the workspace call and the static-scratch call"
        assert same_bits(lse_ws, lse_st), "lse differs between the workspace call and the static-scratch call"
        ref_out, ref_lse = oracle_full(batch)
        say(gates(out_st.float().cpu().numpy(), lse_st.cpu().numpy(), ref_out, ref_lse, batch.workload.dtype,
                  f"static call {step}", stress=stress))


def test_static_scratch_call_refuses_what_does_not_fit():
    # a descriptor whose workspace exceeds the fixed array: refused on the host, nothing launched
    ls.lib()
    d = ls.ls_desc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim, d.n_tree, d.max_prefix_len = 16, 64, 8, 128, 512, 65536
    d.dtype = ls.LS_BF16
    for name, h, l in (("q_stride", 64, 512), ("o_stride", 64, 512), ("kc_stride", 8, 65536), ("vc_stride", 8, 65536),
                       ("kt_stride", 8, 512), ("vt_stride", 8, 512)):
        f = getattr(d, name)
        f[0], f[1], f[2] = h * l * 128, l * 128, 128
    assert ls.ls_workspace_bytes(d) > ls.LS_STATIC_SCRATCH_BYTES
    one = torch.zeros(64, dtype=torch.int32, device="cuda")
    st = ls.ls_hybrid_tree_attn_static(d, one, one, one, one, one, one, one, one, one, check=False)
    assert st == ls.LS_ERR_WORKSPACE
