"""Device-side harness shared by the tests, the smoke check and the benchmark: a synthetic batch
moved to the GPU in the layout the C ABI takes, and the two whole-path calls on it.  Argument
marshalling only; it imports neither the CPU oracle nor anything that does."""
import numpy as np
import torch

from . import binding as ls


def torch_dtype(name):
    return {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[name]


def to_dev(x, dtype, device="cuda"):
    """float32 numpy (values exact in dtype) -> device tensor of dtype."""
    return torch.from_numpy(np.ascontiguousarray(x)).to(device=device, dtype=dtype)


class DeviceBatch:
    """Device tensors of a synth.Batch, [B,H,L,D] layout; ragged prefixes are padded to the
    longest one with NaN rows that a correct kernel never uses."""

    def __init__(self, batch, device="cuda", token_major=False):
        w = batch.workload
        dt = torch_dtype(w.dtype)
        self.batch = batch
        self.dtype_name = w.dtype
        seqs = batch.seqs
        pmax = max(1, batch.max_prefix_len)
        hkv, d = seqs[0].k_tree.shape[0], seqs[0].q.shape[2]

        def stack_cache(attr):
            out = torch.full((len(seqs), hkv, pmax, d), float("nan"), dtype=dt, device=device)
            for b, s in enumerate(seqs):
                if s.prefix_len:
                    out[b, :, :s.prefix_len] = to_dev(getattr(s, attr), dt, device)
            return out

        def maybe_tm(x):
            # token-major storage [B,L,H,D] viewed as [B,H,L,D]
            return x.transpose(1, 2).contiguous().transpose(1, 2) if token_major else x

        self.q = maybe_tm(torch.stack([to_dev(s.q, dt, device) for s in seqs]))
        self.k_cache = maybe_tm(stack_cache("k_cache"))
        self.v_cache = maybe_tm(stack_cache("v_cache"))
        self.k_tree = maybe_tm(torch.stack([to_dev(s.k_tree, dt, device) for s in seqs]))
        self.v_tree = maybe_tm(torch.stack([to_dev(s.v_tree, dt, device) for s in seqs]))
        self.parents = torch.from_numpy(np.stack([s.parents for s in seqs])).to(device)
        self.prefix_lens = torch.from_numpy(batch.prefix_lens).to(device)
        self.max_prefix_len = batch.max_prefix_len
        self.out = maybe_tm(torch.full_like(self.q, float("nan")))
        self.lse = torch.full(self.q.shape[:3], float("nan"), dtype=torch.float32, device=device)
        self.desc = ls.make_desc(self.q, self.k_cache, self.v_cache, self.k_tree, self.v_tree, self.out,
                                 self.max_prefix_len)
        self.workspace = None

    def run_cache_only(self, stream=None):
        if self.workspace is None:
            n = ls.ls_workspace_bytes(self.desc)
            self.workspace = torch.empty(n, dtype=torch.uint8, device=self.q.device)
        ls.ls_cache_attn(self.desc, self.q, self.k_cache, self.v_cache, self.prefix_lens, self.out, self.lse,
                         self.workspace, stream=stream)
        return self.out, self.lse

    def run_full(self, stream=None):
        if self.workspace is None:
            n = ls.ls_workspace_bytes(self.desc)
            self.workspace = torch.empty(n, dtype=torch.uint8, device=self.q.device)
        ls.ls_hybrid_tree_attn(self.desc, self.q, self.k_cache, self.v_cache, self.prefix_lens, self.k_tree,
                               self.v_tree, self.parents, self.out, self.lse, self.workspace, stream=stream)
        return self.out, self.lse

    def run_fused(self, stream=None):
        """The single-launch form; the workspace's arrival counters are zeroed when it is created."""
        if self.workspace is None:
            n = ls.ls_workspace_bytes(self.desc)
            self.workspace = torch.full((n,), 0xFF, dtype=torch.uint8, device=self.q.device)
            ls.ls_workspace_init(self.workspace, stream=stream)
        ls.ls_hybrid_tree_attn_fused(self.desc, self.q, self.k_cache, self.v_cache, self.prefix_lens, self.k_tree,
                                     self.v_tree, self.parents, self.out, self.lse, self.workspace, stream=stream)
        return self.out, self.lse
