"""Parity of the two steps after the attention -- greedy tree acceptance and the move of the
accepted K/V rows into the cache -- against the CPU oracle, through the C ABI, bit for bit."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2502_17421_amd import binding as ls
from paper_2502_17421_amd import synth
from util import to_dev, torch_dtype

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def run_accept(parents, draft, target):
    b, t = parents.shape
    path = torch.full((b, t), -77, dtype=torch.int32, device="cuda")
    n = torch.full((b,), -77, dtype=torch.int32, device="cuda")
    nxt = torch.full((b,), -77, dtype=torch.int32, device="cuda")
    err = torch.full((b,), -77, dtype=torch.int32, device="cuda")
    ls.ls_tree_accept_greedy(dev_i32(parents), dev_i32(draft), dev_i32(target), path, n, nxt, err)
    torch.cuda.synchronize()
    return path.cpu().numpy(), n.cpu().numpy(), nxt.cpu().numpy(), err.cpu().numpy()


@pytest.mark.parametrize("t,vocab,p_follow", [(1, 5, 0.5), (7, 3, 0.5), (64, 4, 0.8), (69, 32000, 0.7),
                                              (128, 2, 0.9), (128, 32000, 0.95), (129, 3, 0.9), (300, 32000, 0.97),
                                              (512, 2, 0.95), (512, 32000, 0.99)])
def test_acceptance_matches_oracle(t, vocab, p_follow):
    rng = np.random.default_rng(8100 + t + vocab)
    b = 9
    parents, draft, target = [], [], []
    for s in range(b):
        if s % 3 == 0:
            par = synth.tree_uniform(rng, t)
        elif s % 3 == 1 and t == 69:
            par = synth.tree_beam(rng)
        elif s % 3 == 1:
            par = synth.tree_chain(t)
        else:
            par = synth.tree_constrained(rng, t, 10, 4) if t > 1 else synth.tree_chain(t)
        d, g = synth.make_tokens(rng, par, vocab, p_follow)
        parents.append(par), draft.append(d), target.append(g)
    parents, draft, target = np.stack(parents), np.stack(draft), np.stack(target)
    path, n, nxt, err = run_accept(parents, draft, target)
    lens = []
    for s in range(b):
        rp, rn, rnext = oracle.tree_accept_greedy(parents[s], draft[s], target[s])
        assert n[s] == rn and nxt[s] == rnext, (s, n[s], rn)
        assert path[s].tolist() == rp.tolist(), s
        lens.append(rn)
    assert np.all(err == 0)
    say(f"acceptance T={t} vocab={vocab}: path lengths {lens}")


def test_acceptance_flags_invalid_parents_and_stays_in_bounds():
    parents = np.array([[-1, 0, 1, 2], [-1, 2, 0, 1], [-1, 0, -5, 2]], dtype=np.int32)
    draft = np.array([[1, 2, 3, 4]] * 3, dtype=np.int32)
    target = np.array([[2, 3, 4, 5]] * 3, dtype=np.int32)
    path, n, nxt, err = run_accept(parents, draft, target)
    assert err.tolist() == [0, 1, 1]
    assert path[0].tolist() == [0, 1, 2, 3] and n[0] == 4 and nxt[0] == 5
    # sequence 1: node 1's entry (2) is not before it -> root; nodes 2 (parent 0, token 3 != 2) stop the path
    assert n[1] == 1 and path[1].tolist() == [0, -1, -1, -1] and nxt[1] == 2
    # sequence 2: node 2 is treated as a root, so the path is 0 -> 1 and ends there
    assert n[2] == 2 and path[2].tolist() == [0, 1, -1, -1] and nxt[2] == 3


def make_case(rng, dtype, b, hkv, d, t, cap, token_major):
    dt = torch_dtype(dtype)

    def draw(shape):
        x = rng.standard_normal(shape, dtype=np.float32)
        return synth.round_to_bf16(x) if dtype == "bf16" else x

    host = {"kc": draw((b, hkv, cap, d)), "vc": draw((b, hkv, cap, d)), "kt": draw((b, hkv, t, d)),
            "vt": draw((b, hkv, t, d))}

    def dev(x):
        y = to_dev(x, dt)
        return y.transpose(1, 2).contiguous().transpose(1, 2) if token_major else y

    devs = {k: dev(v) for k, v in host.items()}
    q = torch.zeros((b, hkv, t, d), dtype=dt, device="cuda")
    desc = ls.make_desc(q, devs["kc"], devs["vc"], devs["kt"], devs["vt"], q, cap)
    return host, devs, desc


@pytest.mark.parametrize("dtype,d,token_major", [("bf16", 128, False), ("bf16", 128, True), ("bf16", 64, False),
                                                 ("f32", 64, False)])
def test_kv_commit_matches_oracle(dtype, d, token_major):
    rng = np.random.default_rng(8200 + d + token_major)
    b, hkv, t, cap = 4, 3, 24, 300
    host, devs, desc = make_case(rng, dtype, b, hkv, d, t, cap, token_major)
    plens = np.array([0, 17, 200, cap - 5], dtype=np.int32)
    lens = np.array([1, 9, 24, 5], dtype=np.int32)
    path = np.full((b, t), -1, dtype=np.int32)
    for s in range(b):
        path[s, :lens[s]] = rng.choice(t, size=lens[s], replace=False)
    new_lens = torch.full((b,), -77, dtype=torch.int32, device="cuda")
    err = torch.full((b,), -77, dtype=torch.int32, device="cuda")
    ls.ls_kv_commit(desc, devs["kt"], devs["vt"], dev_i32(path), dev_i32(lens), dev_i32(plens), devs["kc"],
                    devs["vc"], new_lens, err)
    torch.cuda.synchronize()
    assert err.cpu().tolist() == [0] * b
    for s in range(b):
        for name_c, name_t in (("kc", "kt"), ("vc", "vt")):
            ref, ref_len = oracle.kv_commit(host[name_c][s], host[name_t][s], plens[s], path[s], lens[s])
            got = devs[name_c][s].float().cpu().numpy()
            assert got.tobytes() == ref.tobytes(), (s, name_c)
        assert int(new_lens[s]) == ref_len


def test_kv_commit_clips_at_the_capacity_and_at_bad_entries():
    rng = np.random.default_rng(8300)
    b, hkv, d, t, cap = 3, 2, 128, 8, 40
    host, devs, desc = make_case(rng, "bf16", b, hkv, d, t, cap, False)
    plens = np.array([38, 10, 45], dtype=np.int32)           # the last one lies beyond the capacity: clamped to it
    lens = np.array([4, 5, 2], dtype=np.int32)
    path = np.array([[0, 1, 2, 3, -1, -1, -1, -1], [4, 5, 99, 6, 7, -1, -1, -1], [1, 2, -1, -1, -1, -1, -1, -1]],
                    dtype=np.int32)
    new_lens = torch.zeros((b,), dtype=torch.int32, device="cuda")
    err = torch.zeros((b,), dtype=torch.int32, device="cuda")
    ls.ls_kv_commit(desc, devs["kt"], devs["vt"], dev_i32(path), dev_i32(lens), dev_i32(plens), devs["kc"],
                    devs["vc"], new_lens, err)
    torch.cuda.synchronize()
    assert err.cpu().tolist() == [1, 1, 1]
    assert new_lens.cpu().tolist() == [40, 12, 40]
    for s, (p0, n_ok) in enumerate([(38, 2), (10, 2), (40, 0)]):
        for name_c, name_t in (("kc", "kt"), ("vc", "vt")):
            expect = host[name_c][s].copy()
            expect[:, p0:p0 + n_ok] = host[name_t][s][:, path[s, :n_ok]]
            assert devs[name_c][s].float().cpu().numpy().tobytes() == expect.tobytes(), (s, name_c)


def test_round_of_verification_end_to_end():
    """Attention over cache + tree, acceptance, commit, then attention over the longer cache
    alone: the committed rows must be seen exactly like the tree rows were."""
    rng = np.random.default_rng(8400)
    w = synth.Workload("case", "bf16", 2, 8, 2, 128, 16, 0, 0, None, None, 0)
    cap = 700
    seqs = [synth.make_sequence(rng, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, n_tree=16, prefix_len=pl,
                                parents=synth.tree_chain(16), variant="peaked") for pl in (600, 333)]
    dt = torch.bfloat16
    kc = torch.full((2, 2, cap, 128), float("nan"), dtype=dt, device="cuda")
    vc = torch.full((2, 2, cap, 128), float("nan"), dtype=dt, device="cuda")
    for b, s in enumerate(seqs):
        kc[b, :, :s.prefix_len] = to_dev(s.k_cache, dt)
        vc[b, :, :s.prefix_len] = to_dev(s.v_cache, dt)
    q = torch.stack([to_dev(s.q, dt) for s in seqs])
    kt = torch.stack([to_dev(s.k_tree, dt) for s in seqs])
    vt = torch.stack([to_dev(s.v_tree, dt) for s in seqs])
    parents = dev_i32(np.stack([s.parents for s in seqs]))
    plens = dev_i32([s.prefix_len for s in seqs])
    desc = ls.make_desc(q, kc, vc, kt, vt, q, cap)
    draft = np.tile(np.arange(100, 116, dtype=np.int32), (2, 1))
    target = draft + 1
    target[0, 6] = 5          # sequence 0 accepts nodes 0..6, sequence 1 the whole chain
    path = torch.empty((2, 16), dtype=torch.int32, device="cuda")
    n = torch.empty((2,), dtype=torch.int32, device="cuda")
    nxt = torch.empty((2,), dtype=torch.int32, device="cuda")
    new_lens = torch.empty((2,), dtype=torch.int32, device="cuda")
    err = torch.empty((2,), dtype=torch.int32, device="cuda")
    ls.ls_tree_accept_greedy(parents, dev_i32(draft), dev_i32(target), path, n, nxt, err)
    ls.ls_kv_commit(desc, kt, vt, path, n, plens, kc, vc, new_lens, err)
    torch.cuda.synchronize()
    assert n.cpu().tolist() == [7, 16] and nxt.cpu().tolist() == [5, 116]
    assert new_lens.cpu().tolist() == [607, 349] and err.cpu().tolist() == [0, 0]
    # the last accepted token's query over the new cache alone == its row of hybrid attention over cache + chain
    out = torch.empty_like(q)
    lse = torch.empty(q.shape[:3], dtype=torch.float32, device="cuda")
    ws = torch.empty(ls.ls_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
    ls.ls_cache_attn(desc, q, kc, vc, new_lens, out, lse, ws)
    torch.cuda.synchronize()
    for b, s in enumerate(seqs):
        last = int(n[b]) - 1
        ro, rl = oracle.attn_all(s.q, s.k_cache, s.v_cache, s.k_tree, s.v_tree, s.parents)
        got_o = out[b, :, last].float().cpu().numpy()
        got_l = lse[b, :, last].cpu().numpy()
        assert np.abs(got_o - ro[:, last]).max() <= 2e-2 * max(1.0, np.abs(ro[:, last]).max())
        assert np.abs(got_l - rl[:, last]).max() <= 2e-3
