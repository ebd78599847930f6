"""ctypes binding of the C ABI in include/ls_attn.h -- argument marshalling only.

Every function here has the name of the C entry point it calls and does nothing but turn
torch tensors into device pointers, sizes and strides.  All arithmetic runs in the HIP
kernels of libls_attn.so.  If the library has not been built the import of the library
raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# LS_ATTN_LIB: load this build of the library instead of the in-tree one (the sanitizer test points it
# at a build whose host code is instrumented)
LIB_PATH = os.environ.get("LS_ATTN_LIB") or os.path.join(_HERE, "libls_attn.so")

LS_OK = 0
LS_ERR_NULL, LS_ERR_SHAPE, LS_ERR_DTYPE, LS_ERR_STRIDE = -1, -2, -3, -4
LS_ERR_TREE, LS_ERR_WORKSPACE, LS_ERR_HIP, LS_ERR_UNSUPPORTED = -5, -6, -7, -8
LS_BF16, LS_F32, LS_F16 = 0, 1, 2
LS_MAX_TREE = 512
LS_STATIC_SCRATCH_BYTES = 64 << 20

_i32, _i64, _f32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_float
_vp, _sz = ctypes.c_void_p, ctypes.c_size_t


class ls_desc(ctypes.Structure):
    _fields_ = [
        ("batch", _i32), ("n_q_heads", _i32), ("n_kv_heads", _i32), ("head_dim", _i32),
        ("n_tree", _i32), ("max_prefix_len", _i32), ("dtype", _i32), ("softmax_scale", _f32),
        ("q_stride", _i64 * 3), ("o_stride", _i64 * 3),
        ("kc_stride", _i64 * 3), ("vc_stride", _i64 * 3),
        ("kt_stride", _i64 * 3), ("vt_stride", _i64 * 3),
    ]


class LsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({ls_status_string(status)})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (python -m paper_2502_17421_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with paper_2502_17421_amd.build.build_library(); "
                           "there is no fallback implementation")
    L = ctypes.CDLL(LIB_PATH)
    dp = ctypes.POINTER(ls_desc)
    L.ls_version.restype = ctypes.c_int
    L.ls_status_string.argtypes = [ctypes.c_int]
    L.ls_status_string.restype = ctypes.c_char_p
    L.ls_validate_desc.argtypes = [dp]
    L.ls_validate_parents_host.argtypes = [_vp, _i32, _i32]
    L.ls_prefix_num_splits.argtypes = [dp, ctypes.POINTER(_i32)]
    L.ls_prefix_split_len.argtypes = [dp, _i32, ctypes.POINTER(_i32)]
    L.ls_workspace_bytes.argtypes = [dp, ctypes.POINTER(_sz)]
    L.ls_workspace_error.argtypes = [dp, _vp, ctypes.POINTER(_vp)]
    L.ls_hybrid_tree_attn.argtypes = [dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    L.ls_hybrid_tree_attn_single.argtypes = [dp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    L.ls_hybrid_tree_attn_static.argtypes = [dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
    L.ls_hybrid_tree_attn_fused.argtypes = [dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    L.ls_workspace_init.argtypes = [_vp, _sz, _vp]
    L.ls_set_single_launch_polls.argtypes = [ctypes.c_int32]
    L.ls_cache_attn.argtypes = [dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    L.ls_build_tree_mask.argtypes = [_vp, _i32, _i32, _vp, _vp, _vp]
    L.ls_prefix_attn_splitkv.argtypes = [dp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp]
    L.ls_tree_attn_masked.argtypes = [dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
    L.ls_lse_merge.argtypes = [dp, _i32, _i32, _vp, _vp, _vp, _vp, _vp]
    L.ls_tree_accept_greedy.argtypes = [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp]
    L.ls_kv_commit.argtypes = [dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
    L.ls_hybrid_tree_attn_paged.argtypes = [dp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                                            _vp]
    L.ls_cache_attn_paged.argtypes = [dp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _sz, _vp]
    L.ls_kv_commit_paged.argtypes = [dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp]
    for name in ("ls_validate_desc", "ls_validate_parents_host", "ls_prefix_num_splits", "ls_prefix_split_len",
                 "ls_workspace_bytes", "ls_workspace_error", "ls_hybrid_tree_attn", "ls_hybrid_tree_attn_single",
                 "ls_hybrid_tree_attn_static",
                 "ls_cache_attn", "ls_build_tree_mask",
                 "ls_prefix_attn_splitkv", "ls_tree_attn_masked", "ls_lse_merge", "ls_tree_accept_greedy",
                 "ls_kv_commit", "ls_hybrid_tree_attn_paged", "ls_cache_attn_paged",
                 "ls_kv_commit_paged"):
        getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    """A torch stream (None = torch's current stream) or a raw integer handle as a hipStream_t."""
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status: int, where: str):
    if status != LS_OK:
        raise LsError(status, where)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return LS_BF16
    if t.dtype == torch.float32:
        return LS_F32
    if t.dtype == torch.float16:
        return LS_F16
    return -1


def make_desc(q, k_cache, v_cache, k_tree, v_tree, out, max_prefix_len: int, softmax_scale: float = 0.0) -> ls_desc:
    """Descriptor for [B,H,L,D]-indexed tensors (any strides on the first three axes).
    k_cache / v_cache may be None when max_prefix_len == 0; k_tree / v_tree / out may be None
    for entry points that do not touch them (their strides are then taken from q)."""
    d = ls_desc()
    b, hq, t, hd = q.shape
    ref_kv = k_cache if k_cache is not None else k_tree
    d.batch, d.n_q_heads, d.head_dim, d.n_tree = b, hq, hd, t
    d.n_kv_heads = ref_kv.shape[1] if ref_kv is not None else hq
    d.max_prefix_len = int(max_prefix_len)
    d.dtype = _dtype_code(q)
    d.softmax_scale = float(softmax_scale)

    def put(field, ten, fallback):
        src = ten if ten is not None else fallback
        assert src.stride(3) == 1, "head_dim axis must be contiguous"
        for a in range(3):
            field[a] = src.stride(a)

    put(d.q_stride, q, q)
    put(d.o_stride, out, q)
    kv_fallback = k_tree if k_tree is not None else (k_cache if k_cache is not None else q)
    put(d.kc_stride, k_cache, kv_fallback)
    put(d.vc_stride, v_cache, kv_fallback)
    put(d.kt_stride, k_tree, kv_fallback)
    put(d.vt_stride, v_tree, kv_fallback)
    return d


# ------------------------------------------------------------------ host-only calls ----

def ls_version() -> int:
    return int(lib().ls_version())


def ls_status_string(status: int) -> str:
    return lib().ls_status_string(int(status)).decode()


def ls_validate_desc(desc: ls_desc) -> int:
    return int(lib().ls_validate_desc(ctypes.byref(desc)))


def ls_validate_parents_host(parents: torch.Tensor) -> int:
    """parents: CPU int32 [batch, n_tree]."""
    assert parents.device.type == "cpu" and parents.dtype == torch.int32 and parents.is_contiguous()
    return int(lib().ls_validate_parents_host(_ptr(parents), parents.shape[0], parents.shape[1]))


def ls_prefix_num_splits(desc: ls_desc) -> int:
    n = _i32(0)
    _check(lib().ls_prefix_num_splits(ctypes.byref(desc), ctypes.byref(n)), "ls_prefix_num_splits")
    return int(n.value)


def ls_prefix_split_len(desc: ls_desc, n_splits: int = 0) -> int:
    n = _i32(0)
    _check(lib().ls_prefix_split_len(ctypes.byref(desc), int(n_splits), ctypes.byref(n)), "ls_prefix_split_len")
    return int(n.value)


def ls_workspace_bytes(desc: ls_desc) -> int:
    n = _sz(0)
    _check(lib().ls_workspace_bytes(ctypes.byref(desc), ctypes.byref(n)), "ls_workspace_bytes")
    return int(n.value)


def ls_workspace_error(desc: ls_desc, workspace: torch.Tensor) -> int:
    """Device address of the per-sequence error words inside `workspace`."""
    p = _vp(0)
    _check(lib().ls_workspace_error(ctypes.byref(desc), _ptr(workspace), ctypes.byref(p)), "ls_workspace_error")
    return int(p.value)


# ----------------------------------------------------------------------- device calls ----

def ls_hybrid_tree_attn(desc, q, k_cache, v_cache, prefix_lens, k_tree, v_tree, parents, out, lse, workspace,
                        stream=None, check: bool = True) -> int:
    st = lib().ls_hybrid_tree_attn(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(prefix_lens),
                                   _ptr(k_tree), _ptr(v_tree), _ptr(parents), _ptr(out), _ptr(lse),
                                   _ptr(workspace), _sz(0 if workspace is None else workspace.numel() *
                                                        workspace.element_size()), _stream(stream))
    if check:
        _check(st, "ls_hybrid_tree_attn")
    return int(st)


def ls_hybrid_tree_attn_single(desc, q, k_cache, v_cache, prefix_len, k_tree, v_tree, parents, out, lse, workspace,
                               stream=None, check: bool = True) -> int:
    """One sequence (desc.batch == 1), prefix length as a host integer."""
    st = lib().ls_hybrid_tree_attn_single(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), int(prefix_len),
                                          _ptr(k_tree), _ptr(v_tree), _ptr(parents), _ptr(out), _ptr(lse),
                                          _ptr(workspace), _sz(0 if workspace is None else workspace.numel() *
                                                               workspace.element_size()), _stream(stream))
    if check:
        _check(st, "ls_hybrid_tree_attn_single")
    return int(st)


def ls_hybrid_tree_attn_static(desc, q, k_cache, v_cache, prefix_lens, k_tree, v_tree, parents, out, lse,
                               stream=None, check: bool = True) -> int:
    """The whole path without a workspace argument (the library's own fixed scratch array)."""
    st = lib().ls_hybrid_tree_attn_static(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                          _ptr(prefix_lens), _ptr(k_tree), _ptr(v_tree), _ptr(parents), _ptr(out),
                                          _ptr(lse), _stream(stream))
    if check:
        _check(st, "ls_hybrid_tree_attn_static")
    return int(st)


LS_WORKSPACE_COUNTER_BYTES = 4096 * 24


def ls_workspace_init(workspace, stream=None, check: bool = True) -> int:
    """Zero the arrival counters at the start of a workspace (needed once before ls_hybrid_tree_attn_fused)."""
    st = lib().ls_workspace_init(_ptr(workspace), _sz(0 if workspace is None else workspace.numel() *
                                                      workspace.element_size()), _stream(stream))
    if check:
        _check(st, "ls_workspace_init")
    return int(st)


def ls_hybrid_tree_attn_fused(desc, q, k_cache, v_cache, prefix_lens, k_tree, v_tree, parents, out, lse, workspace,
                              stream=None, check: bool = True) -> int:
    """The whole path in one launch: the workgroups of a query block merge its rows between them once all
    have written their parts (counters at the workspace start; ls_workspace_init before the first call)."""
    st = lib().ls_hybrid_tree_attn_fused(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(prefix_lens),
                                         _ptr(k_tree), _ptr(v_tree), _ptr(parents), _ptr(out), _ptr(lse),
                                         _ptr(workspace), _sz(0 if workspace is None else workspace.numel() *
                                                              workspace.element_size()), _stream(stream))
    if check:
        _check(st, "ls_hybrid_tree_attn_fused")
    return int(st)


def ls_set_single_launch_polls(polls: int, check: bool = True) -> int:
    """Polls a workgroup of later single-launch calls waits for its query block (0: nobody waits; < 0: default)."""
    st = lib().ls_set_single_launch_polls(ctypes.c_int32(polls))
    if check:
        _check(st, "ls_set_single_launch_polls")
    return int(st)


def ls_cache_attn(desc, q, k_cache, v_cache, prefix_lens, out, lse, workspace, stream=None, check: bool = True) -> int:
    st = lib().ls_cache_attn(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(prefix_lens), _ptr(out),
                             _ptr(lse), _ptr(workspace), _sz(0 if workspace is None else workspace.numel() *
                                                             workspace.element_size()), _stream(stream))
    if check:
        _check(st, "ls_cache_attn")
    return int(st)


def ls_build_tree_mask(parents, mask, err_flag=None, stream=None, check: bool = True) -> int:
    """parents: device int32 [batch, n_tree]; mask: device int64/uint64 storage [batch, n_tree, words]."""
    st = lib().ls_build_tree_mask(_ptr(parents), parents.shape[0], parents.shape[1], _ptr(mask), _ptr(err_flag),
                                  _stream(stream))
    if check:
        _check(st, "ls_build_tree_mask")
    return int(st)


def ls_prefix_attn_splitkv(desc, q, k_cache, v_cache, prefix_lens, n_splits, o_part, lse_part, stream=None,
                           check: bool = True) -> int:
    """o_part: float32 tensor, or a tensor of the problem's own 16-bit type, [B,Hq,n_splits,T,D]; its dtype selects
    part_dtype."""
    st = lib().ls_prefix_attn_splitkv(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(prefix_lens),
                                      int(n_splits), _dtype_code(o_part), _ptr(o_part), _ptr(lse_part),
                                      _stream(stream))
    if check:
        _check(st, "ls_prefix_attn_splitkv")
    return int(st)


def ls_tree_attn_masked(desc, q, k_tree, v_tree, mask, o_tree, lse_tree, stream=None, check: bool = True) -> int:
    st = lib().ls_tree_attn_masked(ctypes.byref(desc), _ptr(q), _ptr(k_tree), _ptr(v_tree), _ptr(mask),
                                   _ptr(o_tree), _ptr(lse_tree), _stream(stream))
    if check:
        _check(st, "ls_tree_attn_masked")
    return int(st)


def ls_lse_merge(desc, n_parts, o_parts, lse_parts, out, lse, stream=None, check: bool = True) -> int:
    st = lib().ls_lse_merge(ctypes.byref(desc), int(n_parts), _dtype_code(o_parts), _ptr(o_parts), _ptr(lse_parts),
                            _ptr(out), _ptr(lse), _stream(stream))
    if check:
        _check(st, "ls_lse_merge")
    return int(st)


def ls_tree_accept_greedy(parents, draft_tokens, target_tokens, accept_path, accept_len, next_token, err_flag=None,
                          stream=None, check: bool = True) -> int:
    """All tensors device int32: parents/draft_tokens/target_tokens/accept_path [batch, n_tree];
    accept_len/next_token/err_flag [batch]."""
    st = lib().ls_tree_accept_greedy(_ptr(parents), _ptr(draft_tokens), _ptr(target_tokens), parents.shape[0],
                                     parents.shape[1], _ptr(accept_path), _ptr(accept_len), _ptr(next_token),
                                     _ptr(err_flag), _stream(stream))
    if check:
        _check(st, "ls_tree_accept_greedy")
    return int(st)


def ls_kv_commit(desc, k_tree, v_tree, accept_path, accept_len, prefix_lens, k_cache, v_cache, new_prefix_lens=None,
                 err_flag=None, stream=None, check: bool = True) -> int:
    st = lib().ls_kv_commit(ctypes.byref(desc), _ptr(k_tree), _ptr(v_tree), _ptr(accept_path), _ptr(accept_len),
                            _ptr(prefix_lens), _ptr(k_cache), _ptr(v_cache), _ptr(new_prefix_lens), _ptr(err_flag),
                            _stream(stream))
    if check:
        _check(st, "ls_kv_commit")
    return int(st)


def ls_hybrid_tree_attn_paged(desc, q, k_pages, v_pages, block_table, page_size, prefix_lens, k_tree, v_tree, parents,
                              out, lse, workspace, stream=None, check: bool = True) -> int:
    """block_table: device int32 [batch, bt_stride]; desc.kc_stride / vc_stride describe one page
    (see make_desc_paged)."""
    st = lib().ls_hybrid_tree_attn_paged(ctypes.byref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                         block_table.shape[1], int(page_size), _ptr(prefix_lens), _ptr(k_tree),
                                         _ptr(v_tree), _ptr(parents), _ptr(out), _ptr(lse), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream))
    if check:
        _check(st, "ls_hybrid_tree_attn_paged")
    return int(st)


def ls_kv_commit_paged(desc, k_tree, v_tree, accept_path, accept_len, prefix_lens, k_pages, v_pages, block_table,
                       page_size, new_prefix_lens=None, err_flag=None, stream=None, check: bool = True) -> int:
    st = lib().ls_kv_commit_paged(ctypes.byref(desc), _ptr(k_tree), _ptr(v_tree), _ptr(accept_path), _ptr(accept_len),
                                  _ptr(prefix_lens), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                  block_table.shape[1], int(page_size), _ptr(new_prefix_lens), _ptr(err_flag),
                                  _stream(stream))
    if check:
        _check(st, "ls_kv_commit_paged")
    return int(st)


def ls_cache_attn_paged(desc, q, k_pages, v_pages, block_table, page_size, prefix_lens, out, lse, workspace,
                        stream=None, check: bool = True) -> int:
    st = lib().ls_cache_attn_paged(ctypes.byref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                   block_table.shape[1], int(page_size), _ptr(prefix_lens), _ptr(out), _ptr(lse),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if check:
        _check(st, "ls_cache_attn_paged")
    return int(st)
