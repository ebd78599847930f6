"""Paged caches: the whole path and the KV commit over page tables must give what the same
rows give in one contiguous cache.  Reference: the CPU oracle on the contiguous rows (paging
is pure indexing, done here with numpy)."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2502_17421_amd import binding as ls
from paper_2502_17421_amd import synth
from util import gates, oracle_full, to_dev, torch_dtype

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


class PagedBatch:
    """Device tensors of a synth.Batch with the cached rows scattered over shuffled pages.
    Table entries beyond a sequence's rows point at a poison page full of NaN: harmless to read,
    visible if used."""

    def __init__(self, batch, page_size, rng, token_major=False, extra_rows=0):
        w = batch.workload
        dt = torch_dtype(w.dtype)
        seqs = batch.seqs
        b = len(seqs)
        hkv, d = seqs[0].k_tree.shape[0], seqs[0].q.shape[2]
        self.cap = batch.max_prefix_len + extra_rows
        per_seq = [-(-(s.prefix_len + extra_rows) // page_size) for s in seqs]
        n_pages = sum(per_seq) + 1
        ids = rng.permutation(n_pages - 1) + 1                     # page 0 is the poison page
        self.bt_stride = max(1, -(-self.cap // page_size))
        table = np.zeros((b, self.bt_stride), dtype=np.int32)
        k_host = np.full((n_pages, hkv, page_size, d), np.nan, dtype=np.float32)
        v_host = np.full((n_pages, hkv, page_size, d), np.nan, dtype=np.float32)
        at = 0
        for s_i, sq in enumerate(seqs):
            for j in range(per_seq[s_i]):
                pid = int(ids[at]); at += 1
                table[s_i, j] = pid
                lo, hi = j * page_size, min((j + 1) * page_size, sq.prefix_len)
                if hi > lo:
                    k_host[pid, :, :hi - lo] = sq.k_cache[:, lo:hi]
                    v_host[pid, :, :hi - lo] = sq.v_cache[:, lo:hi]
        self.k_host, self.v_host, self.table_host = k_host, v_host, table

        def maybe_tm(x):
            return x.transpose(1, 2).contiguous().transpose(1, 2) if token_major else x

        self.k_pages = maybe_tm(to_dev(k_host, dt))
        self.v_pages = maybe_tm(to_dev(v_host, dt))
        self.table = torch.from_numpy(table).cuda()
        self.q = torch.stack([to_dev(s.q, dt) for s in seqs])
        self.k_tree = torch.stack([to_dev(s.k_tree, dt) for s in seqs])
        self.v_tree = torch.stack([to_dev(s.v_tree, dt) for s in seqs])
        self.parents = torch.from_numpy(np.stack([s.parents for s in seqs])).cuda()
        self.prefix_lens = torch.from_numpy(batch.prefix_lens).cuda()
        self.out = torch.full_like(self.q, float("nan"))
        self.lse = torch.full(self.q.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
        self.page_size = page_size
        self.desc = ls.make_desc(self.q, self.k_pages, self.v_pages, self.k_tree, self.v_tree, self.out, self.cap)
        self.ws = torch.empty(ls.ls_workspace_bytes(self.desc), dtype=torch.uint8, device="cuda")

    def run(self):
        ls.ls_hybrid_tree_attn_paged(self.desc, self.q, self.k_pages, self.v_pages, self.table, self.page_size,
                                     self.prefix_lens, self.k_tree, self.v_tree, self.parents, self.out, self.lse, self.ws)
        torch.cuda.synchronize()
        return self.out.float().cpu().numpy(), self.lse.cpu().numpy()


def batch_of(dtype, hq, hkv, d, t, plens, variant, seed):
    rng = np.random.default_rng(seed)
    seqs = [synth.make_sequence(rng, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n_tree=t, prefix_len=pl,
                                parents=synth.tree_constrained(rng, t, 8, 4) if t > 1 else synth.tree_chain(t),
                                variant=variant) for pl in plens]
    w = synth.Workload("case", dtype, len(seqs), hq, hkv, d, t, min(plens), max(plens), None, None, 0)
    return synth.Batch(w, variant, seqs)


@pytest.mark.parametrize("dtype,hq,hkv,d,t,plens,page_size,token_major", [
    ("bf16", 32, 8, 128, 64, [1500], 16, False),            # smallest pages: four per key tile
    ("bf16", 32, 8, 128, 64, [1500], 64, False),            # one page per key tile
    ("bf16", 32, 8, 128, 64, [1500], 256, False),           # four key tiles per page
    ("bf16", 8, 8, 128, 32, [1000, 129, 0, 65], 32, False),  # ragged batch, an empty cache, tiles ending mid-page
    ("bf16", 12, 4, 64, 40, [1111], 16, False),             # head_dim 64: eight rows per load instruction
    ("f16", 32, 8, 128, 64, [2100], 128, False),
    ("bf16", 32, 8, 128, 64, [1300], 64, True),             # pages stored token-major [page, row, head, D]
    ("bf16", 40, 8, 128, 128, [900, 2100], 16, False),      # three query blocks share the pages
])
def test_whole_path_paged(dtype, hq, hkv, d, t, plens, page_size, token_major):
    batch = batch_of(dtype, hq, hkv, d, t, plens, "peaked", 9700 + hq + page_size)
    pb = PagedBatch(batch, page_size, np.random.default_rng(1), token_major=token_major)
    out, lse = pb.run()
    ro, rl = oracle_full(batch)
    say(gates(out, lse, ro, rl, dtype, f"paged {dtype} hq={hq} d={d} t={t} plens={plens} page={page_size} "
              f"tm={token_major}", stress=True))


def test_paged_longest_split_uses_every_page_register():
    """64 KV heads at 32k rows: 4 splits of 8192 rows, 512 pages of 16 rows per split."""
    batch = batch_of("bf16", 64, 64, 64, 4, [32768], "iid", 9800)
    pb = PagedBatch(batch, 16, np.random.default_rng(2))
    assert ls.ls_prefix_split_len(pb.desc, 0) == 8192
    out, lse = pb.run()
    rng = np.random.default_rng(3)
    rows, ro, rl = oracle_full(batch, rows_per_seq=24, rng=rng)
    got_o = np.stack([out[0][rows[0][:, 0], rows[0][:, 1]]])
    got_l = np.stack([lse[0][rows[0][:, 0], rows[0][:, 1]]])
    say(gates(got_o, got_l, ro, rl, "bf16", "paged, 512 pages per split, 24 sampled rows"))


def test_paged_equals_contiguous_bit_for_bit():
    from util import DeviceBatch
    batch = batch_of("bf16", 32, 8, 128, 64, [3000], "iid", 9900)
    pb = PagedBatch(batch, 64, np.random.default_rng(4))
    out_p, lse_p = pb.run()
    db = DeviceBatch(batch)
    out_c, lse_c = db.run_full()
    torch.cuda.synchronize()
    assert np.array_equal(out_p, out_c.float().cpu().numpy()) and np.array_equal(lse_p, lse_c.cpu().numpy())


def test_cache_only_paged():
    batch = batch_of("bf16", 32, 8, 128, 16, [3000, 70], "peaked", 9990)
    pb = PagedBatch(batch, 16, np.random.default_rng(6))
    ls.ls_cache_attn_paged(pb.desc, pb.q, pb.k_pages, pb.v_pages, pb.table, 16, pb.prefix_lens, pb.out, pb.lse, pb.ws)
    torch.cuda.synchronize()
    for b, sq in enumerate(batch.seqs):
        ro, rl = oracle.attn_all(sq.q, sq.k_cache, sq.v_cache, sq.k_tree, sq.v_tree, sq.parents, use_tree=False)
        say(gates(pb.out[b].float().cpu().numpy(), pb.lse[b].cpu().numpy(), ro, rl, "bf16",
                  f"paged cache only P={sq.prefix_len}", stress=True))


def test_paged_argument_errors():
    batch = batch_of("bf16", 8, 2, 128, 8, [300], "iid", 9950)
    pb = PagedBatch(batch, 64, np.random.default_rng(5))
    args = (pb.desc, pb.q, pb.k_pages, pb.v_pages, pb.table)
    rest = (pb.prefix_lens, pb.k_tree, pb.v_tree, pb.parents, pb.out, pb.lse, pb.ws)
    assert ls.ls_hybrid_tree_attn_paged(*args, 48, *rest, check=False) == ls.LS_ERR_UNSUPPORTED   # not a power of two
    assert ls.ls_hybrid_tree_attn_paged(*args, 8, *rest, check=False) == ls.LS_ERR_UNSUPPORTED    # below 16
    assert ls.ls_hybrid_tree_attn_paged(*args, 32, *rest, check=False) == ls.LS_ERR_SHAPE         # table too short


@pytest.mark.parametrize("dtype,page_size", [("bf16", 16), ("f32", 4), ("f16", 64)])
def test_kv_commit_paged_matches_oracle(dtype, page_size):
    rng = np.random.default_rng(9960 + page_size)
    d = 64 if dtype == "f32" else 128
    batch = batch_of(dtype, 6, 3, d, 24, [0, 17, 200, 295], "iid", 9970)
    pb = PagedBatch(batch, page_size, rng, extra_rows=24)
    lens = np.array([1, 9, 24, 5], dtype=np.int32)
    path = np.full((4, 24), -1, dtype=np.int32)
    for s in range(4):
        path[s, :lens[s]] = rng.choice(24, size=lens[s], replace=False)
    new_lens = torch.full((4,), -77, dtype=torch.int32, device="cuda")
    err = torch.full((4,), -77, dtype=torch.int32, device="cuda")
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    ls.ls_kv_commit_paged(pb.desc, pb.k_tree, pb.v_tree, dev(path), dev(lens), pb.prefix_lens, pb.k_pages, pb.v_pages,
                          pb.table, page_size, new_lens, err)
    torch.cuda.synchronize()
    assert err.cpu().tolist() == [0, 0, 0, 0]
    k_dev = pb.k_pages.float().cpu().numpy()
    v_dev = pb.v_pages.float().cpu().numpy()
    touched = np.zeros(k_dev.shape[0], dtype=bool)
    for s, sq in enumerate(batch.seqs):
        cap = pb.bt_stride * page_size
        for host_pages, tree, dev_pages in ((pb.k_host, sq.k_tree, k_dev), (pb.v_host, sq.v_tree, v_dev)):
            contiguous = np.concatenate([host_pages[pid] for pid in pb.table_host[s]], axis=1)[:, :cap]
            ref, ref_len = oracle.kv_commit(np.nan_to_num(contiguous, nan=-5.0), tree, sq.prefix_len, path[s], lens[s])
            got = np.concatenate([dev_pages[pid] for pid in pb.table_host[s]], axis=1)[:, :cap]
            assert np.nan_to_num(got, nan=-5.0).tobytes() == ref.tobytes(), (s,)
        assert int(new_lens[s]) == ref_len
        touched[pb.table_host[s]] = True
    assert np.all(np.isnan(k_dev[0])) and np.all(np.isnan(v_dev[0]))      # the poison page is untouched
