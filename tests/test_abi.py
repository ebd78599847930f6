"""CPU-side tests of the C-ABI library: it loads, exports every function the header
declares, the descriptor struct matches between C and the binding, and argument errors
come back as status codes before anything is launched (no GPU needed)."""
import ctypes
import os
import re
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ls_attn.h")

from paper_2502_17421_amd import binding as ls
from paper_2502_17421_amd import build as ls_build


@pytest.fixture(scope="module", autouse=True)
def built_library():
    if not os.path.exists(ls.LIB_PATH):
        ls_build.build_library()
    return ls.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ls_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(built_library):
    names = declared_functions()
    assert "ls_hybrid_tree_attn" in names and len(names) >= 12
    for n in names:
        assert hasattr(built_library, n), f"{n} declared in ls_attn.h but not exported"
    # and the binding offers a function of the same name for each
    for n in names:
        assert callable(getattr(ls, n)), f"binding lacks {n}"


def test_descriptor_layout_matches_c(tmp_path):
    src = tmp_path / "layout.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "ls_attn.h"\n'
        "int main(void){printf(\"%zu %zu %zu %zu %zu %zu\\n\", sizeof(ls_desc), offsetof(ls_desc, softmax_scale),"
        " offsetof(ls_desc, q_stride), offsetof(ls_desc, o_stride), offsetof(ls_desc, kc_stride),"
        " offsetof(ls_desc, vt_stride)); return 0;}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o",
                    str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    d = ls.ls_desc
    assert got == [ctypes.sizeof(d), d.softmax_scale.offset, d.q_stride.offset, d.o_stride.offset,
                   d.kc_stride.offset, d.vt_stride.offset]


C_CALLER = r"""
#include <stdio.h>
#include <string.h>
#include "ls_attn.h"
/* a plain C caller: fills a descriptor for [B,H,L,D] tensors and asks the host-only entry points */
int main(void)
{
    ls_desc d;
    memset(&d, 0, sizeof d);
    d.batch = 1; d.n_q_heads = 32; d.n_kv_heads = 8; d.head_dim = 128; d.n_tree = 64; d.max_prefix_len = 32768;
    d.dtype = LS_BF16;
    const int64_t hq = 32, hkv = 8, t = 64, p = 32768, dd = 128;
    int64_t *s[6] = {d.q_stride, d.o_stride, d.kc_stride, d.vc_stride, d.kt_stride, d.vt_stride};
    const int64_t heads[6] = {hq, hq, hkv, hkv, hkv, hkv}, rows[6] = {t, t, p, p, t, t};
    for (int i = 0; i < 6; ++i) { s[i][0] = heads[i] * rows[i] * dd; s[i][1] = rows[i] * dd; s[i][2] = dd; }
    int32_t n_splits = 0, split_len = 0;
    size_t bytes = 0;
    int rc = ls_validate_desc(&d);
    if (rc == LS_OK) rc = ls_prefix_num_splits(&d, &n_splits);
    if (rc == LS_OK) rc = ls_prefix_split_len(&d, 0, &split_len);
    if (rc == LS_OK) rc = ls_workspace_bytes(&d, &bytes);
    d.head_dim = 80;
    printf("%d %d %d %zu %d %s\n", rc, n_splits, split_len, bytes, ls_validate_desc(&d), ls_status_string(LS_ERR_UNSUPPORTED));
    return ls_version() >= 100 ? 0 : 1;
}
"""


def test_a_plain_c_program_links_and_calls_the_library(tmp_path):
    """The boundary is a C ABI: a C99 translation unit that includes only the header links
    against the shared library and gets the same answers as the Python binding."""
    src = tmp_path / "caller.c"
    src.write_text(C_CALLER)
    exe = tmp_path / "caller"
    libdir = os.path.dirname(ls.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-lls_attn", "-Wl,--allow-shlib-undefined", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(maxsplit=5)
    d = good_desc(hq=32, hkv=8, t=64, p=32768)
    assert [int(x) for x in out[:5]] == [ls.LS_OK, ls.ls_prefix_num_splits(d), ls.ls_prefix_split_len(d, 0),
                                         ls.ls_workspace_bytes(d), ls.LS_ERR_UNSUPPORTED]
    assert out[5].strip() == ls.ls_status_string(ls.LS_ERR_UNSUPPORTED)


def test_version_and_status_strings():
    assert ls.ls_version() >= 100
    seen = set()
    for code in range(0, -9, -1):
        s = ls.ls_status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 9
    assert ls.ls_status_string(-99) == "unknown status"


def good_desc(dtype=ls.LS_BF16, b=1, hq=8, hkv=2, d=128, t=16, p=1000):
    x = ls.ls_desc()
    x.batch, x.n_q_heads, x.n_kv_heads, x.head_dim, x.n_tree, x.max_prefix_len = b, hq, hkv, d, t, p
    x.dtype = dtype
    x.softmax_scale = 0.0
    for name, h, l in (("q_stride", hq, t), ("o_stride", hq, t), ("kc_stride", hkv, max(p, 1)),
                       ("vc_stride", hkv, max(p, 1)), ("kt_stride", hkv, t), ("vt_stride", hkv, t)):
        f = getattr(x, name)
        f[0], f[1], f[2] = h * l * d, l * d, d
    return x


def test_validate_desc_codes():
    assert ls.ls_validate_desc(good_desc()) == ls.LS_OK
    assert ls.ls_validate_desc(good_desc(dtype=ls.LS_F32, d=64)) == ls.LS_OK
    assert ls.ls_validate_desc(good_desc(dtype=ls.LS_F16)) == ls.LS_OK
    x = good_desc(); x.batch = 0
    assert ls.ls_validate_desc(x) == ls.LS_ERR_SHAPE
    x = good_desc(); x.n_kv_heads = 3
    assert ls.ls_validate_desc(x) == ls.LS_ERR_SHAPE
    x = good_desc(); x.max_prefix_len = -1
    assert ls.ls_validate_desc(x) == ls.LS_ERR_SHAPE
    x = good_desc(); x.softmax_scale = float("nan")
    assert ls.ls_validate_desc(x) == ls.LS_ERR_SHAPE
    x = good_desc(); x.dtype = 7
    assert ls.ls_validate_desc(x) == ls.LS_ERR_DTYPE
    x = good_desc(); x.head_dim = 96
    assert ls.ls_validate_desc(x) == ls.LS_ERR_UNSUPPORTED
    x = good_desc(); x.n_tree = 513
    assert ls.ls_validate_desc(x) == ls.LS_ERR_UNSUPPORTED
    x = good_desc(); x.kc_stride[2] = 132          # 264-byte rows: not 16-byte aligned
    assert ls.ls_validate_desc(x) == ls.LS_ERR_STRIDE
    x = good_desc(); x.q_stride[2] = 64            # rows overlap
    assert ls.ls_validate_desc(x) == ls.LS_ERR_STRIDE
    x = good_desc(); x.o_stride[1] = 0
    assert ls.ls_validate_desc(x) == ls.LS_ERR_STRIDE
    x = good_desc(); x.vt_stride[0] = -128
    assert ls.ls_validate_desc(x) == ls.LS_ERR_STRIDE
    assert ls.lib().ls_validate_desc(None) == ls.LS_ERR_NULL


def test_validate_parents_host():
    ok = torch.tensor([[-1, 0, 0, 2], [-1, -1, 1, 2]], dtype=torch.int32)
    assert ls.ls_validate_parents_host(ok) == ls.LS_OK
    for bad in ([[0, 0]], [[-1, 1]], [[-1, -2]], [[-1, 0, 2]]):
        assert ls.ls_validate_parents_host(torch.tensor(bad, dtype=torch.int32)) == ls.LS_ERR_TREE
    assert ls.lib().ls_validate_parents_host(None, 1, 1) == ls.LS_ERR_NULL


def even_cut_bytes(d, e=2):
    """Workspace size when every query block is cut into ls_prefix_num_splits pieces (the arrival
    counters of the single-launch call come first, at a size that no descriptor changes)."""
    up = lambda n: (n + 255) // 256 * 256
    rows = d.batch * d.n_q_heads * ls.ls_prefix_num_splits(d) * d.n_tree
    words = (d.n_tree + 63) // 64
    return (ls.LS_WORKSPACE_COUNTER_BYTES + up(d.batch * d.n_tree * words * 8) + up(d.batch * 4) + up(rows * 4) +
            up(rows * d.head_dim * e))


def test_workspace_follows_the_schedule_of_the_whole_call():
    """The whole-path calls cut the keys exactly like the stand-alone cached-key call, whatever the
    number of query rows per KV head.  (Without a device the library plans for 256 compute units.)"""
    for d in (good_desc(hq=32, hkv=8, t=64, p=32768),            # 256 rows: one full block
              good_desc(hq=32, hkv=8, t=16, p=32768),            # 64 rows: one block
              good_desc(hq=40, hkv=8, t=128, p=65536, b=4),      # 640 rows: a light third block
              good_desc(hq=20, hkv=4, t=77, p=4000, b=2),        # 385 rows
              good_desc(hq=32, hkv=8, t=69, p=3000),             # 276 rows: 256 + 20
              good_desc(dtype=ls.LS_F16, hq=12, hkv=2, t=60, p=2500, d=64)):
        assert ls.ls_workspace_bytes(d) == even_cut_bytes(d)
    d = good_desc(dtype=ls.LS_F32, hq=32, hkv=8, t=68, p=32768, d=64)
    assert ls.ls_workspace_bytes(d) == even_cut_bytes(d, 4)


def test_split_plan_and_workspace_are_stable_and_sane():
    d = good_desc(hq=32, hkv=8, t=64, p=32768)
    s = ls.ls_prefix_num_splits(d)
    assert s == ls.ls_prefix_num_splits(d) and 1 <= s <= 32768 // 64
    length = ls.ls_prefix_split_len(d, 0)
    assert length % 64 == 0 and (s - 1) * length < 32768 <= s * length
    assert ls.ls_prefix_split_len(d, 5) % 64 == 0 and ls.ls_prefix_split_len(d, 5) * 5 >= 32768
    n = ls.ls_workspace_bytes(d)
    parts = s * 32 * 64
    assert n >= parts * 128 * 2 + parts * 4 + 64 * 8 and n % 256 == 0
    z = good_desc(p=0)
    assert ls.ls_prefix_num_splits(z) >= 1 and ls.ls_workspace_bytes(z) > 0
    # every cache size, both kernels' paths, light and heavy query blocks: the pieces cover the cache
    # exactly once, none is empty, and none is longer than the matrix-core kernel takes
    for dtype, dim in ((ls.LS_BF16, 128), (ls.LS_F32, 64)):
        for hq, hkv, t in ((32, 8, 64), (32, 32, 32), (8, 2, 16)):
            for p_max in list(range(0, 260)) + [511, 512, 1000, 4096, 8191, 8192, 8193, 12288, 65536, 131072, 1 << 20]:
                x = good_desc(dtype=dtype, hq=hq, hkv=hkv, d=dim, t=t, p=p_max)
                n, ln = ls.ls_prefix_num_splits(x), ls.ls_prefix_split_len(x, 0)
                assert n >= 1 and ln >= 64 and ln % 64 == 0, (dtype, hq, p_max, n, ln)
                assert (n - 1) * ln < max(p_max, 1) <= n * ln, (dtype, hq, p_max, n, ln)
                if dtype != ls.LS_F32:
                    assert ln <= 8192
    bad = good_desc(); bad.head_dim = 80
    with pytest.raises(ls.LsError):
        ls.ls_workspace_bytes(bad)


def test_split_counts_of_the_benchmark_shapes():
    """The planner's choices for the named workloads on a 256-unit device (what the figures in the
    design notes were measured with): a change of the model shows up here first."""
    from paper_2502_17421_amd import synth
    code = {"bf16": ls.LS_BF16, "f16": ls.LS_F16, "f32": ls.LS_F32}
    want = {"C2": 16, "C3": 32, "C4": 8, "C5": 8, "D1": 32, "D2": 32, "W1": 8, "H3": 32, "B3": 16, "L3": 8}
    for name, n in want.items():
        w = synth.WORKLOADS[name]
        x = good_desc(dtype=code[w.dtype], b=w.batch, hq=w.n_q_heads, hkv=w.n_kv_heads, d=w.head_dim, t=w.n_tree,
                      p=w.prefix_hi)
        assert ls.ls_prefix_num_splits(x) == n, (name, ls.ls_prefix_num_splits(x), n)


def test_device_entry_points_reject_bad_arguments_on_the_host():
    """Null pointers, bad descriptors and a short workspace come back as codes; nothing is
    launched, so this runs without a GPU (stream handle 0)."""
    d = good_desc()
    L = ls.lib()
    one = ctypes.c_void_p(256)     # a non-null, aligned stand-in that is never dereferenced
    odd = ctypes.c_void_p(260)
    dp = ctypes.byref(d)
    assert L.ls_hybrid_tree_attn(dp, None, one, one, one, one, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_NULL
    assert L.ls_hybrid_tree_attn(dp, one, None, one, one, one, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_NULL
    assert L.ls_hybrid_tree_attn(dp, odd, one, one, one, one, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_STRIDE
    assert L.ls_hybrid_tree_attn(dp, one, one, one, one, one, one, one, one, one, None, 0, None) == ls.LS_ERR_WORKSPACE
    assert L.ls_hybrid_tree_attn(dp, one, one, one, one, one, one, one, one, one, one, 16, None) == ls.LS_ERR_WORKSPACE
    assert L.ls_hybrid_tree_attn(dp, one, one, one, one, one, one, one, one, one, odd, 1 << 40, None) == ls.LS_ERR_WORKSPACE
    bad = good_desc(); bad.n_tree = 0
    assert L.ls_hybrid_tree_attn(ctypes.byref(bad), one, one, one, one, one, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_SHAPE
    single = L.ls_hybrid_tree_attn_single
    assert single(dp, None, one, one, 10, one, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_NULL
    assert single(dp, one, one, one, -1, one, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_SHAPE
    assert single(dp, one, one, one, 1001, one, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_SHAPE   # > max_prefix_len
    assert single(dp, one, one, one, 10, one, one, one, one, one, one, 16, None) == ls.LS_ERR_WORKSPACE
    two = good_desc(b=2)
    assert single(ctypes.byref(two), one, one, one, 10, one, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_SHAPE
    assert single(None, one, one, one, 10, one, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_NULL
    assert L.ls_cache_attn(dp, one, one, None, one, one, one, one, 1 << 40, None) == ls.LS_ERR_NULL
    assert L.ls_cache_attn(dp, one, one, one, one, one, one, one, 16, None) == ls.LS_ERR_WORKSPACE
    assert L.ls_cache_attn(dp, one, odd, one, one, one, one, one, 1 << 40, None) == ls.LS_ERR_STRIDE
    assert L.ls_build_tree_mask(None, 1, 4, one, None, None) == ls.LS_ERR_NULL
    assert L.ls_build_tree_mask(one, 1, 0, one, None, None) == ls.LS_ERR_SHAPE
    assert L.ls_build_tree_mask(one, 1, 513, one, None, None) == ls.LS_ERR_UNSUPPORTED
    assert L.ls_prefix_attn_splitkv(dp, one, one, one, None, 0, ls.LS_F32, one, one, None) == ls.LS_ERR_NULL
    assert L.ls_prefix_attn_splitkv(dp, one, one, one, one, -1, ls.LS_F32, one, one, None) == ls.LS_ERR_SHAPE
    assert L.ls_prefix_attn_splitkv(dp, one, one, one, one, 2, 5, one, one, None) == ls.LS_ERR_DTYPE
    assert L.ls_prefix_attn_splitkv(dp, one, one, one, one, 2, ls.LS_F16, one, one, None) == ls.LS_ERR_DTYPE  # bf16 problem
    assert L.ls_tree_attn_masked(dp, one, one, one, None, one, one, None) == ls.LS_ERR_NULL
    assert L.ls_lse_merge(dp, 0, ls.LS_F32, one, one, one, one, None) == ls.LS_ERR_SHAPE
    assert L.ls_lse_merge(dp, 2, ls.LS_F32, one, one, None, one, None) == ls.LS_ERR_NULL
    assert L.ls_lse_merge(dp, 2, 9, one, one, one, one, None) == ls.LS_ERR_DTYPE
    assert L.ls_tree_accept_greedy(one, one, None, 1, 4, one, one, one, None, None) == ls.LS_ERR_NULL
    assert L.ls_tree_accept_greedy(one, one, one, 0, 4, one, one, one, None, None) == ls.LS_ERR_SHAPE
    assert L.ls_tree_accept_greedy(one, one, one, 1, 513, one, one, one, None, None) == ls.LS_ERR_UNSUPPORTED
    assert L.ls_kv_commit(dp, one, one, one, one, one, None, one, None, None, None) == ls.LS_ERR_NULL
    assert L.ls_kv_commit(dp, one, one, one, one, one, one, one, one, None, None) == ls.LS_ERR_NULL   # aliasing lengths
    assert L.ls_kv_commit(dp, one, odd, one, one, one, one, one, None, None, None) == ls.LS_ERR_STRIDE
    big = 1 << 40
    assert L.ls_hybrid_tree_attn_paged(dp, one, one, one, None, 64, 16, one, one, one, one, one, one, one, big, None) == ls.LS_ERR_NULL
    assert L.ls_hybrid_tree_attn_paged(dp, one, one, one, one, 64, 24, one, one, one, one, one, one, one, big, None) == ls.LS_ERR_UNSUPPORTED
    assert L.ls_hybrid_tree_attn_paged(dp, one, one, one, one, 2, 16, one, one, one, one, one, one, one, big, None) == ls.LS_ERR_SHAPE
    f32 = good_desc(dtype=ls.LS_F32, d=64)
    assert L.ls_hybrid_tree_attn_paged(ctypes.byref(f32), one, one, one, one, 64, 16, one, one, one, one, one, one, one, big, None) == ls.LS_ERR_UNSUPPORTED
    assert L.ls_kv_commit_paged(dp, one, one, one, one, one, one, one, None, 64, 16, None, None, None) == ls.LS_ERR_NULL
    assert L.ls_kv_commit_paged(dp, one, one, one, one, one, one, one, one, 64, 24, None, None, None) == ls.LS_ERR_UNSUPPORTED
    fused = L.ls_hybrid_tree_attn_fused
    assert fused(dp, one, one, one, None, one, one, one, one, one, one, big, None) == ls.LS_ERR_NULL   # no host-side length
    assert fused(dp, None, one, one, one, one, one, one, one, one, one, big, None) == ls.LS_ERR_NULL
    assert fused(dp, one, one, one, one, one, one, one, one, one, one, 16, None) == ls.LS_ERR_WORKSPACE
    assert L.ls_workspace_init(one, 16, None) == ls.LS_ERR_WORKSPACE
    assert L.ls_workspace_init(odd, big, None) == ls.LS_ERR_WORKSPACE
    assert L.ls_set_single_launch_polls((1 << 24) + 1) == ls.LS_ERR_SHAPE
    assert L.ls_set_single_launch_polls(0) == ls.LS_OK
    assert L.ls_set_single_launch_polls(-1) == ls.LS_OK


def test_binding_raises_when_library_is_missing(tmp_path, monkeypatch):
    """No silent fallback: without the built library the binding refuses to work."""
    monkeypatch.setattr(ls, "_lib", None)
    monkeypatch.setattr(ls, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        ls.lib()


def test_product_code_does_not_touch_the_oracle():
    """The package and its sources never import or mention the oracle package."""
    pkg = os.path.join(ROOT, "paper_2502_17421_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), f
                assert "ls_oracle" not in text, f
    for f in ("ls_oracle.c", "__init__.py"):
        text = open(os.path.join(ROOT, "oracle", f)).read()
        assert "paper_2502_17421_amd" not in text and "ls_attn.h" not in text


def test_cached_key_kernels_use_no_scratch_memory():
    """The MFMA kernel orders its LDS reads behind its HBM->LDS copies by counting outstanding
    vector-memory instructions (s_waitcnt vmcnt(N)).  A register spill would add scratch loads
    and stores to that count behind the compiler's back, so no instantiation may spill."""
    if not os.path.exists(ls_build.RESOURCE_REPORT) or ls_build.is_stale():
        ls_build.build_library()
    res = ls_build.kernel_resources()
    kernels = {k: v for k, v in res.items() if "prefix_mfma_kernel" in k}
    assert len(kernels) >= 16, sorted(res)
    for name, r in kernels.items():
        assert r.get("ScratchSize", 0) == 0 and r.get("VGPRs Spill", 0) == 0, (name, r)
        assert r.get("VGPRs", 0) + r.get("AGPRs", 0) <= 256, (name, r)   # two waves per SIMD


def test_only_the_tile_copies_touch_m0(tmp_path):
    """The HBM->LDS copies of the MFMA kernel set M0 inside inline assembly, which cannot declare
    it clobbered.  That is sound as long as the compiler itself never uses M0 in that file: in
    the generated assembly every line that names M0 is the scalar move in front of one copy."""
    asm = tmp_path / "prefix_mfma.s"
    src = os.path.join(ls_build.CSRC, "ls_prefix_mfma.hip")
    flags = [f for f in ls_build.FLAGS if f not in ("-shared", "-fPIC")]
    subprocess.run([ls_build.HIPCC, *flags, "-S", "--cuda-device-only", "-o", str(asm), src], check=True,
                   stderr=subprocess.DEVNULL)
    lines = asm.read_text().splitlines()
    copies = sum("global_load_lds_dwordx4" in ln for ln in lines)
    m0 = [ln.strip() for ln in lines if re.search(r"\bm0\b", ln.split(";")[0])]
    assert copies > 0 and len(m0) == copies
    # the source operand is any scalar register the allocator picked (vcc halves included)
    form = r"s_mov_b32 m0, (s\d+|vcc_lo|vcc_hi)"
    assert all(re.fullmatch(form, ln) for ln in m0), [ln for ln in m0 if not re.fullmatch(form, ln)][:5]
