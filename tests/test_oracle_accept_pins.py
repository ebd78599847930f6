"""Pins for the two integer steps of the oracle that follow the attention: greedy tree
acceptance and the move of accepted K/V rows into the cache (no GPU).

The paper prints no worked example for either, so the pins are: a hand-worked case
(tests/golden/accept_case.json), equality with plain greedy decoding of a toy deterministic
"model" (the property speculative decoding promises: the output is unchanged), a brute
force over all root paths, and the same indexing written with numpy."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2502_17421_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "accept_case.json")


def test_hand_worked_cases():
    g = json.load(open(GOLDEN))
    parents = g["parents"]
    for name, c in g["cases"].items():
        path, n, nxt = oracle.tree_accept_greedy(parents, c["draft"], c["target"])
        assert n == len(c["path"]), name
        assert path[:n].tolist() == c["path"] and np.all(path[n:] == -1), name
        assert nxt == c["next_token"], name


def toy_next_token(seq, vocab):
    """A deterministic stand-in for a language model: next token as a function of the whole sequence."""
    h = 1469598103934665603
    for t in seq:
        h = ((h ^ (int(t) + 1)) * 1099511628211) % (1 << 64)
    return int(h % vocab)


def path_tokens(parents, draft, i):
    toks = []
    while i >= 0:
        toks.append(int(draft[i]))
        i = int(parents[i])
    return toks[::-1]


@pytest.mark.parametrize("seed", range(12))
def test_acceptance_reproduces_plain_greedy_decoding(seed):
    rng = np.random.default_rng(7000 + seed)
    vocab = int(rng.integers(2, 5))          # small, so that branches often match
    t = int(rng.integers(1, 40))
    parents = synth.tree_uniform(rng, t) if seed % 2 else synth.tree_constrained(rng, t, 6, 3)
    context = [int(x) for x in rng.integers(0, vocab, size=5)]
    draft = rng.integers(0, vocab, size=t).astype(np.int32)
    # plant the true continuation along a random root path so that long acceptances occur
    node, seq = 0, context + [int(draft[0])]
    while True:
        kids = [j for j in range(t) if parents[j] == node]
        if not kids or rng.random() < 0.15:
            break
        node = int(rng.choice(kids))
        draft[node] = toy_next_token(seq, vocab)
        seq.append(int(draft[node]))
    target = np.array([toy_next_token(context + path_tokens(parents, draft, i), vocab) for i in range(t)],
                      dtype=np.int32)
    path, n, nxt = oracle.tree_accept_greedy(parents, draft, target)
    # plain greedy decoding from the same state
    seq = context + [int(draft[0])]
    greedy = []
    for _ in range(n):
        greedy.append(toy_next_token(seq, vocab))
        seq.append(greedy[-1])
    accepted = [int(draft[i]) for i in path[1:n]] + [nxt]
    assert accepted == greedy
    # the path is a root path of the tree and cannot be extended
    assert path[0] == 0 and all(parents[path[k]] == path[k - 1] for k in range(1, n))
    last = int(path[n - 1])
    assert not any(parents[j] == last and draft[j] == nxt for j in range(t))


@pytest.mark.parametrize("seed", range(8))
def test_acceptance_against_all_paths_brute_force(seed):
    """With distinct tokens among siblings the accepted nodes are exactly those whose every
    edge up to the root matches the target's prediction at the edge's upper end."""
    rng = np.random.default_rng(7100 + seed)
    t = int(rng.integers(2, 30))
    parents = synth.tree_uniform(rng, t)
    draft = np.zeros(t, dtype=np.int32)
    for i in range(t):                     # sibling-distinct tokens: rank among the siblings
        draft[i] = sum(1 for j in range(i) if parents[j] == parents[i])
    target = rng.integers(0, 3, size=t).astype(np.int32)
    ok = np.zeros(t, dtype=bool)
    ok[0] = True
    for i in range(1, t):
        ok[i] = ok[parents[i]] and draft[i] == target[parents[i]]
    depth = synth.tree_depths(parents)
    expect = sorted(np.nonzero(ok)[0].tolist(), key=lambda i: depth[i])
    path, n, nxt = oracle.tree_accept_greedy(parents, draft, target)
    assert path[:n].tolist() == expect
    assert nxt == target[expect[-1]]


def test_acceptance_special_trees():
    t = 17
    chain = synth.tree_chain(t)
    draft = np.arange(100, 100 + t, dtype=np.int32)
    target = np.arange(101, 101 + t, dtype=np.int32)
    path, n, nxt = oracle.tree_accept_greedy(chain, draft, target)
    assert n == t and path.tolist() == list(range(t)) and nxt == 100 + t
    target[5] = -7                                  # the chain breaks after node 5
    path, n, nxt = oracle.tree_accept_greedy(chain, draft, target)
    assert n == 6 and nxt == -7
    star = synth.tree_star(t)
    draft = np.full(t, 3, dtype=np.int32)
    target = np.full(t, 3, dtype=np.int32)
    path, n, nxt = oracle.tree_accept_greedy(star, draft, target)   # all siblings match: lowest index
    assert n == 2 and path[:2].tolist() == [0, 1]
    path, n, nxt = oracle.tree_accept_greedy([-1], [4], [9])
    assert n == 1 and nxt == 9
    with pytest.raises(ValueError):
        oracle.tree_accept_greedy([-1, 1], [1, 2], [1, 2])          # parent not before child


@pytest.mark.parametrize("seed", range(4))
def test_kv_commit_against_numpy_indexing(seed):
    rng = np.random.default_rng(7200 + seed)
    hkv, cap, d, t = 3, 40, 8, 12
    cache = rng.standard_normal((hkv, cap, d)).astype(np.float32)
    tree = rng.standard_normal((hkv, t, d)).astype(np.float32)
    plen = int(rng.integers(0, 20))
    n = int(rng.integers(0, 9))
    path = np.full(t, -1, dtype=np.int32)
    path[:n] = rng.choice(t, size=n, replace=False)
    new, new_len = oracle.kv_commit(cache, tree, plen, path, n)
    expect = cache.copy()
    expect[:, plen:plen + n, :] = tree[:, path[:n], :]
    assert new_len == plen + n
    assert new.tobytes() == expect.tobytes()


def test_kv_commit_rejects_overflow_and_bad_nodes():
    cache = np.zeros((1, 8, 4), dtype=np.float32)
    tree = np.ones((1, 4, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.kv_commit(cache, tree, 6, [0, 1, 2, -1], 3)
    with pytest.raises(ValueError):
        oracle.kv_commit(cache, tree, 0, [0, 4, -1, -1], 2)
    new, n = oracle.kv_commit(cache, tree, 6, [0, 1, -1, -1], 2)    # exactly fills the cache
    assert n == 8 and np.all(new[0, 6:8] == 1) and np.all(new[0, :6] == 0)
