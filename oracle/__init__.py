"""CPU fp64 oracle for hybrid tree attention -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``ls_oracle.c`` (the arithmetic lives there, with the
citations).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the GPU library
and its Python binding never do, and this package never imports them.

Array conventions (numpy, C order, one sequence per call):
    q [Hq,T,D]  k_cache,v_cache [Hkv,P,D]  k_tree,v_tree [Hkv,T,D]  float32
    parents [T] int32;  outputs are float64.
float32 storage is exact for the fp32 and bf16 values under test; all
arithmetic is double (see the C file).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ls_oracle.c")
_LIB = os.path.join(_HERE, "libls_oracle.so")
_lib = None
# LS_ORACLE_LIB: load this build of ls_oracle.c instead (the sanitizer test points it at an
# -fsanitize=address,undefined build)
_OVERRIDE = os.environ.get("LS_ORACLE_LIB")


def build(force: bool = False) -> str:
    """Compile ls_oracle.c with gcc into libls_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not _OVERRIDE:
        build()
    lib = ctypes.CDLL(_OVERRIDE or _LIB)
    i32, i64, f64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_double
    vp = ctypes.c_void_p
    lib.ls_oracle_num_threads.restype = ctypes.c_int
    lib.ls_oracle_check_parents.argtypes = [vp, i32]
    lib.ls_oracle_check_parents.restype = ctypes.c_int
    lib.ls_oracle_tree_mask.argtypes = [vp, i32, vp]
    lib.ls_oracle_tree_mask.restype = ctypes.c_int
    lib.ls_oracle_attn_rows.argtypes = [i32, i32, i32, i32, i64, vp, vp, vp, vp, vp, vp, f64,
                                        i64, i64, i32, vp, i64, vp, vp]
    lib.ls_oracle_attn_rows.restype = ctypes.c_int
    lib.ls_oracle_lse_merge.argtypes = [i64, i32, i32, vp, vp, vp, vp]
    lib.ls_oracle_lse_merge.restype = ctypes.c_int
    lib.ls_oracle_tree_accept_greedy.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.ls_oracle_tree_accept_greedy.restype = i32
    lib.ls_oracle_kv_commit.argtypes = [i32, i32, i32, i64, i64, vp, i32, vp, vp]
    lib.ls_oracle_kv_commit.restype = i64
    _lib = lib
    return lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().ls_oracle_num_threads())


def tree_mask(parents) -> np.ndarray:
    """[T] parents -> [T, ceil(T/64)] uint64 ancestor-or-self bit sets."""
    parents = np.ascontiguousarray(parents, dtype=np.int32)
    assert parents.ndim == 1
    t = parents.shape[0]
    mask = np.zeros((t, (t + 63) // 64), dtype=np.uint64)
    rc = _load().ls_oracle_tree_mask(_ptr(parents), t, _ptr(mask))
    if rc != 0:
        raise ValueError("parents is not a topologically ordered forest")
    return mask


def attn_rows(q, k_cache, v_cache, k_tree, v_tree, parents, rows=None, scale=None,
              prefix_lo=0, prefix_hi=None, use_tree=True):
    """Attention of the query rows listed in ``rows`` ([n,2] of (head, tree row));
    all rows when None.  Returns (out [n,D] float64, lse [n] float64)."""
    q, k_cache, v_cache = _f32(q), _f32(k_cache), _f32(v_cache)
    k_tree, v_tree = _f32(k_tree), _f32(v_tree)
    parents = np.ascontiguousarray(parents, dtype=np.int32)
    hq, t, d = q.shape
    hkv, p, d2 = k_cache.shape
    assert d2 == d and v_cache.shape == k_cache.shape
    assert k_tree.shape == (hkv, t, d) and v_tree.shape == (hkv, t, d)
    assert parents.shape == (t,)
    if rows is None:
        hh, tt = np.meshgrid(np.arange(hq), np.arange(t), indexing="ij")
        rows = np.stack([hh.ravel(), tt.ravel()], axis=1)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    assert rows.ndim == 2 and rows.shape[1] == 2
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    if prefix_hi is None:
        prefix_hi = p
    n = rows.shape[0]
    out = np.empty((n, d), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = _load().ls_oracle_attn_rows(hq, hkv, d, t, p, _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                     _ptr(k_tree), _ptr(v_tree), _ptr(parents), float(scale),
                                     int(prefix_lo), int(prefix_hi), int(bool(use_tree)),
                                     _ptr(rows), n, _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError(f"ls_oracle_attn_rows failed with {rc}")
    return out, lse


def attn_all(q, k_cache, v_cache, k_tree, v_tree, parents, **kw):
    """All rows, reshaped: (out [Hq,T,D], lse [Hq,T])."""
    hq, t, d = np.shape(q)
    out, lse = attn_rows(q, k_cache, v_cache, k_tree, v_tree, parents, rows=None, **kw)
    return out.reshape(hq, t, d), lse.reshape(hq, t)


def lse_merge(o_parts, lse_parts):
    """o_parts [n,parts,D], lse_parts [n,parts] (float64) -> (out [n,D], lse [n])."""
    o_parts = np.ascontiguousarray(o_parts, dtype=np.float64)
    lse_parts = np.ascontiguousarray(lse_parts, dtype=np.float64)
    n, parts, d = o_parts.shape
    assert lse_parts.shape == (n, parts)
    out = np.empty((n, d), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = _load().ls_oracle_lse_merge(n, parts, d, _ptr(o_parts), _ptr(lse_parts), _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError(f"ls_oracle_lse_merge failed with {rc}")
    return out, lse


def tree_accept_greedy(parents, draft_tokens, target_tokens):
    """One sequence: returns (path [T] int32 root first, padded with -1; length; next_token)."""
    parents = np.ascontiguousarray(parents, dtype=np.int32)
    draft = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    target = np.ascontiguousarray(target_tokens, dtype=np.int32)
    t = parents.shape[0]
    assert draft.shape == (t,) and target.shape == (t,)
    path = np.empty(t, dtype=np.int32)
    nxt = np.zeros(1, dtype=np.int32)
    n = _load().ls_oracle_tree_accept_greedy(_ptr(parents), _ptr(draft), _ptr(target), t, _ptr(path), _ptr(nxt))
    if n < 0:
        raise ValueError("ls_oracle_tree_accept_greedy: bad arguments")
    return path, int(n), int(nxt[0])


def kv_commit(cache, tree, prefix_len, path, path_len):
    """cache [Hkv,capacity,D], tree [Hkv,T,D] float32: returns (new cache, new prefix length)."""
    cache = np.array(cache, dtype=np.float32, order="C", copy=True)
    tree = _f32(tree)
    path = np.ascontiguousarray(path, dtype=np.int32)
    hkv, cap, d = cache.shape
    assert tree.shape[0] == hkv and tree.shape[2] == d
    n = _load().ls_oracle_kv_commit(hkv, d, tree.shape[1], cap, int(prefix_len), _ptr(path), int(path_len),
                                    _ptr(tree), _ptr(cache))
    if n < 0:
        raise ValueError("ls_oracle_kv_commit: row outside the cache or bad path")
    return cache, int(n)
