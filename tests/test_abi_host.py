"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and rejects
bad arguments before anything is launched (no GPU needed, no compute call is made)."""
import ctypes as C
import os
import re

import pytest

from paper_2510_27641_amd import binding as sa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "specattn.h")).read()
    declared = set(re.findall(r"\b(specattn_[a-z_]+)\s*\(", header))
    assert declared == set(sa.EXPORTS)
    lib = sa.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.specattn_version() >= 1000
    assert sa.last_error() == "" or isinstance(sa.last_error(), str)


def _sel(**kw):
    a = sa.SelectArgs()
    a.probs, a.counts, a.indices = 0x1000, 0x2000, 0x3000      # never dereferenced on the host
    a.B, a.H_kv, a.n_max = 2, 4, 1024
    a.probs_stride_b, a.probs_stride_h = 4096, 1024
    a.top_p = 0.9
    a.idx_stride_row, a.idx_capacity = 1024, 1024
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def _attn(**kw):
    a = sa.AttnArgs()
    a.q, a.k, a.v, a.out = 0x1000, 0x2000, 0x3000, 0x4000
    a.indices, a.counts = 0x5000, 0x6000
    a.dtype = sa.BF16
    a.B, a.H_q, a.H_kv, a.T, a.d, a.n_max = 2, 32, 8, 5, 128, 4096
    a.q_stride_b, a.q_stride_h, a.q_stride_t = 32 * 5 * 128, 5 * 128, 128
    a.kv_stride_b, a.kv_stride_h, a.kv_stride_n = 8 * 4096 * 128, 4096 * 128, 128
    a.idx_stride_row, a.idx_capacity = 4096, 4096
    for k, v in kw.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("kw,status", [
    (dict(probs=None), sa.EINVAL), (dict(counts=None), sa.EINVAL), (dict(indices=None), sa.EINVAL),
    (dict(chunk_size=12), sa.ESHAPE), (dict(chunk_size=-1), sa.ESHAPE), (dict(chunk_size=16), sa.EWORKSPACE),
    (dict(chunk_size=16, block_counts=0x7000), sa.EUNSUPPORTED),
    (dict(bisect_iters=65), sa.ESHAPE), (dict(bisect_iters=10), sa.EWORKSPACE),
    (dict(bisect_iters=10, chunk_size=16), sa.EUNSUPPORTED), (dict(bisect_iters=10, block_counts=0x7000), sa.EUNSUPPORTED),
    (dict(top_p=0.0), sa.EINVAL), (dict(top_p=1.5), sa.EINVAL), (dict(top_p=float("nan")), sa.EINVAL),
    (dict(B=0), sa.EINVAL), (dict(n_max=(1 << 20) + 1, probs_stride_h=1 << 21, probs_stride_b=1 << 23), sa.ESHAPE),
    (dict(idx_capacity=0), sa.ESHAPE), (dict(idx_stride_row=8), sa.ESHAPE), (dict(probs_stride_h=512), sa.ESHAPE),
    (dict(emit_physical=1), sa.EINVAL),
    (dict(emit_physical=1, page_table=0x9000, page_size=12, max_pages_per_seq=999), sa.ESHAPE),
    (dict(emit_physical=1, page_table=0x9000, page_size=16, max_pages_per_seq=8), sa.ESHAPE),
])
def test_select_argument_errors(kw, status):
    lib = sa.load()
    a = _sel(**kw)
    assert lib.specattn_topp_select(C.byref(a), None, 0, None) == status
    assert sa.last_error() != ""


@pytest.mark.parametrize("kw,status", [
    (dict(q=None), sa.EINVAL), (dict(out=None), sa.EINVAL), (dict(indices=None), sa.EINVAL),
    (dict(H_q=30), sa.ESHAPE), (dict(T=9), sa.ESHAPE), (dict(d=96), sa.ESHAPE), (dict(dtype=7), sa.EUNSUPPORTED),
    (dict(H_q=128, T=8, dtype=sa.F32, kv_stride_n=128), sa.ESHAPE), (dict(k=0x2004), sa.EALIGN), (dict(kv_stride_n=132), sa.EALIGN),
    (dict(kv_stride_n=64), sa.ESHAPE), (dict(idx_capacity=0), sa.ESHAPE),
    (dict(page_table=0x9000, page_size=10, max_pages_per_seq=1000, kv_stride_page=8 * 16 * 128), sa.ESHAPE),
    (dict(page_table=0x9000, page_size=16, max_pages_per_seq=1000, kv_stride_page=0), sa.ESHAPE),
    (dict(), sa.EWORKSPACE),                                      # valid arguments but no workspace
    (dict(counts=None), sa.EINVAL),                               # a list without counts
    (dict(k_new=0x7000), sa.EINVAL),                              # new keys without new values
    (dict(chunk_size=24), sa.ESHAPE), (dict(chunk_size=16, indices_are_physical=1, page_size=16, kv_stride_page=8 * 16 * 128), sa.EUNSUPPORTED),
    (dict(chunk_size=16, indices=None, counts=None), sa.EUNSUPPORTED),
    (dict(k_new=0x7000, v_new=0x8004), sa.EALIGN),
    (dict(indices=None, counts=None), sa.EWORKSPACE),             # dense call: valid, but no workspace
    (dict(indices=None, counts=None, indices_are_physical=1, page_size=16, kv_stride_page=8 * 16 * 128), sa.EINVAL),
    (dict(workspace=0x10040, workspace_bytes=1 << 30), sa.EWORKSPACE),   # misaligned workspace
    (dict(workspace=0x10000, workspace_bytes=16), sa.EWORKSPACE),        # too small
])
def test_attention_argument_errors(kw, status):
    lib = sa.load()
    a = _attn(**kw)
    assert lib.specattn_sparse_decode_attn(C.byref(a), None) == status
    assert sa.last_error() != ""


def test_workspace_size_is_monotone_and_zero_for_selection():
    assert sa.specattn_workspace_size(_sel(), None) == 0
    small = sa.specattn_workspace_size(None, _attn())
    big = sa.specattn_workspace_size(None, _attn(B=4))
    assert 0 < small <= big
    assert small % 256 == 0
    assert sa.specattn_workspace_size(None, _attn(H_q=30)) == 0


@pytest.mark.parametrize("H_q", [8, 16, 32, 64, 128])
@pytest.mark.parametrize("B,cap", [(1, 4096), (2, 3000), (8, 32768), (64, 512)])
def test_attention_workspace_holds_every_partial_of_the_matrix_core_route(H_q, B, cap):
    """The bf16 / fp16, d = 128 route leaves one partial per (workgroup, row) in slot workgroup + row, at most
    32 query rows wide (larger groups of query heads run as several launches over the same slots), behind a
    256-byte aligned table of rows + 1 ints.  The size query must cover that for any number of query heads per
    kv head (with 8 heads per kv head and T = 5 it once did not: 40 query rows took the portable route's size)."""
    H_kv, T, d = 8, 5, 128
    a = _attn(B=B, H_q=H_q, idx_capacity=cap, idx_stride_row=cap, n_max=max(cap, 4096),
              q_stride_b=H_q * T * d, kv_stride_b=H_kv * max(cap, 4096) * d, kv_stride_h=max(cap, 4096) * d)
    rows = B * H_kv
    n_wg = 256                                                   # no device here: the library assumes 256 compute units
    qtp = 16 if (H_q // H_kv) * T <= 16 else 32
    need = ((rows + 1) * 4 + 255) // 256 * 256 + (n_wg + rows) * qtp * (d + 2) * 4
    assert sa.specattn_workspace_size(None, a) >= need


def test_chunk_selection_workspace_size():
    assert sa.specattn_workspace_size(_sel(chunk_size=16), None) == 2 * 4 * 64 * 4
    assert sa.specattn_workspace_size(_sel(chunk_size=16, n_max=1000, probs_stride_h=1024), None) == ((2 * 4 * 63 * 4 + 255) // 256) * 256


def test_stream_read_rejects_bad_arguments():
    lib = sa.load()
    assert lib.specattn_stream_read(None, 1024, None, None) == sa.EINVAL
    assert lib.specattn_stream_read(0x1000, 0, None, None) == sa.EINVAL
    assert lib.specattn_stream_read(0x1008, 1024, None, None) == sa.EALIGN
    assert lib.specattn_stream_read(0x1000, 1000, None, None) == sa.EALIGN
    assert "16" in sa.last_error()


def _union(**kw):
    a = sa.UnionArgs()
    a.probs, a.counts, a.indices = 0x1000, 0x2000, 0x3000
    a.B, a.H_draft, a.S, a.H_kv, a.n_max = 2, 8, 4, 4, 1024
    a.probs_stride_b, a.probs_stride_row = 8 * 4 * 1024, 1024
    a.top_p = 0.9
    a.idx_stride_row, a.idx_capacity = 1024, 1024
    for k, v in kw.items():
        setattr(a, k, v)
    return a


@pytest.mark.parametrize("kw,status", [
    (dict(probs=None), sa.EINVAL), (dict(indices=None), sa.EINVAL), (dict(counts=None), sa.EINVAL),
    (dict(top_p=0.0), sa.EINVAL), (dict(top_p=float("nan")), sa.EINVAL), (dict(S=0), sa.EINVAL),
    (dict(H_kv=3), sa.ESHAPE), (dict(n_max=(1 << 19) + 1, probs_stride_row=1 << 20), sa.ESHAPE),
    (dict(probs_stride_row=1000), sa.ESHAPE), (dict(idx_capacity=0), sa.ESHAPE),
    (dict(emit_physical=1), sa.EINVAL), (dict(page_table=0x9000, page_size=12, max_pages_per_seq=100), sa.ESHAPE),
    (dict(), sa.EWORKSPACE),
])
def test_union_argument_errors(kw, status):
    lib = sa.load()
    a = _union(**kw)
    assert lib.specattn_topp_select_union(C.byref(a), None, 0, None) == status
    assert sa.last_error() != ""


def test_union_workspace_size():
    small = sa.specattn_union_workspace_size(_union())
    assert small > 0 and small % 256 == 0
    assert sa.specattn_union_workspace_size(_union(S=8)) > small
    assert sa.specattn_union_workspace_size(_union(H_kv=3)) == 0


def test_header_is_plain_c(tmp_path):
    """The public header must compile as C (no C++ constructs), and a C caller must link against the library."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = tmp_path / "caller.c"
    src.write_text(
        '#include "specattn.h"\n'
        "#include <stdio.h>\n"
        "int main(void) {\n"
        "    specattn_select_args s = {0};\n"
        "    specattn_attn_args a = {0};\n"
        "    specattn_union_args u = {0};\n"
        "    /* NULL arguments are rejected on the host: nothing is launched */\n"
        "    int r1 = specattn_topp_select(&s, NULL, 0, NULL);\n"
        "    int r2 = specattn_sparse_decode_attn(&a, NULL);\n"
        "    int r3 = specattn_topp_select_union(&u, NULL, 0, NULL);\n"
        '    printf("%d %d %d %d %s\\n", r1, r2, r3, specattn_version(), specattn_last_error());\n'
        "    return (r1 == SPECATTN_EINVAL && r2 == SPECATTN_EINVAL && r3 == SPECATTN_EINVAL) ? 0 : 1;\n"
        "}\n")
    exe = tmp_path / "caller"
    libdir = os.path.dirname(sa.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
                           "-L", libdir, "-lspecattn", "-Wl,-rpath," + libdir, "-o", str(exe)])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr


def test_check_lists_argument_errors():
    lib = sa.load()
    lib.specattn_check_lists.argtypes = [C.POINTER(sa.AttnArgs), C.c_int64, C.c_void_p, C.c_void_p]
    assert lib.specattn_check_lists(C.byref(_attn(indices=None, counts=None)), 0, 0x7000, None) == sa.EINVAL
    assert lib.specattn_check_lists(C.byref(_attn()), 0, None, None) == sa.EINVAL
    assert lib.specattn_check_lists(C.byref(_attn()), -1, 0x7000, None) == sa.EINVAL
    assert lib.specattn_check_lists(C.byref(_attn(H_q=30)), 0, 0x7000, None) == sa.ESHAPE


def test_layer_mapping_argument_errors_and_sizes():
    lib = sa.load()
    assert lib.specattn_layer_similarity_workspace_size(22, 32, 64, 2048) % 256 == 0
    assert lib.specattn_layer_similarity_workspace_size(22, 32, 64, 2048) >= 22 * 32 * 8
    assert lib.specattn_layer_similarity_workspace_size(0, 32, 64, 2048) == 0
    assert lib.specattn_layer_similarity_workspace_size(300, 300, 64, 2048) == 0          # more than 65535 pairs
    assert lib.specattn_layer_map_workspace_size(22, 32) == ((22 * 32 * 4 + 255) // 256) * 256
    assert lib.specattn_layer_map_workspace_size(1025, 32) == 0
    assert lib.specattn_layer_similarity(None, 0x2000, 2, 2, 2, 8, 0x3000, 0x10000, 1 << 20, None) == sa.EINVAL
    assert lib.specattn_layer_similarity(0x1000, 0x2000, 0, 2, 2, 8, 0x3000, 0x10000, 1 << 20, None) == sa.EINVAL
    assert lib.specattn_layer_similarity(0x1000, 0x2000, 300, 300, 2, 8, 0x3000, 0x10000, 1 << 20, None) == sa.ESHAPE
    assert lib.specattn_layer_similarity(0x1000, 0x2000, 2, 2, 2, 8, 0x3000, None, 0, None) == sa.EWORKSPACE
    assert lib.specattn_layer_similarity(0x1000, 0x2000, 2, 2, 2, 8, 0x3000, 0x10040, 1 << 20, None) == sa.EWORKSPACE
    assert lib.specattn_layer_similarity(0x1000, 0x2000, 2, 2, 2, 8, 0x3000, 0x10000, 8, None) == sa.EWORKSPACE
    assert lib.specattn_layer_map(None, 2, 2, 0x2000, 0x3000, 0x10000, 1 << 20, None) == sa.EINVAL
    assert lib.specattn_layer_map(0x1000, 2, 0, 0x2000, 0x3000, 0x10000, 1 << 20, None) == sa.EINVAL
    assert lib.specattn_layer_map(0x1000, 2000, 2, 0x2000, 0x3000, 0x10000, 1 << 20, None) == sa.ESHAPE
    assert lib.specattn_layer_map(0x1000, 2, 2, 0x2000, 0x3000, None, 0, None) == sa.EWORKSPACE
    assert lib.specattn_layer_map(0x1000, 2, 2, 0x2000, 0x3000, 0x10000, 8, None) == sa.EWORKSPACE
    assert sa.last_error() != ""


def test_large_query_groups_need_the_matrix_core_route():
    """More than 64 query rows per kv head only fit the matrix-core kernel, which also bounds H_kv (512 rows per
    launch): anything else must be refused on the host, not run on the portable kernel whose tables hold 64 rows."""
    lib = sa.load()
    H_kv, T, d = 1024, 5, 128
    a = _attn(B=1, H_q=16 * H_kv, H_kv=H_kv, q_stride_b=16 * H_kv * T * d, q_stride_h=T * d,
              kv_stride_b=H_kv * 4096 * d, workspace=0x10000, workspace_bytes=1 << 40)
    assert lib.specattn_sparse_decode_attn(C.byref(a), None) == sa.ESHAPE
    assert "query rows" in sa.last_error()


def test_csr_argument_errors_and_static_entry_checks():
    lib = sa.load()
    assert lib.specattn_lists_to_csr(0x1000, 64, 64, None, 4, 0x2000, None, None) == sa.EINVAL       # no counts
    assert lib.specattn_lists_to_csr(None, 64, 64, 0x1000, 4, 0x2000, 0x3000, None) == sa.EINVAL     # packed without lists
    assert lib.specattn_lists_to_csr(0x1000, 8, 64, 0x1000, 4, 0x2000, 0x3000, None) == sa.ESHAPE    # stride < capacity
    assert lib.specattn_lists_to_csr(0x1000, 64, 64, 0x1000, 0, 0x2000, None, None) == sa.EINVAL     # no rows
    # the entry point without a workspace validates like the one with, before it touches the device
    assert lib.specattn_sparse_decode_attn_static(C.byref(_attn(q=None)), None) == sa.EINVAL
    assert lib.specattn_sparse_decode_attn_static(C.byref(_attn(d=96)), None) == sa.ESHAPE


def test_fused_entry_refuses_what_has_no_meaning_without_a_list():
    lib = sa.load()
    ws = dict(workspace=0x10000, workspace_bytes=1 << 40)
    s = _sel(B=2, H_kv=8, n_max=4096, probs_stride_b=8 * 4096, probs_stride_h=4096, indices=None)
    assert lib.specattn_fused(C.byref(s), C.byref(_attn(indices_are_physical=1, page_size=16, kv_stride_page=8 * 16 * 128, **ws)), None) == sa.EUNSUPPORTED
    s2 = _sel(B=2, H_kv=8, n_max=4096, probs_stride_b=8 * 4096, probs_stride_h=4096, indices=None, reuse_selection=1)
    assert lib.specattn_fused(C.byref(s2), C.byref(_attn(**ws)), None) == sa.EINVAL                  # nothing to reuse
    s3 = _sel(B=2, H_kv=8, n_max=4096, probs_stride_b=8 * 4096, probs_stride_h=4096, indices=None, chunk_size=16, block_counts=0x7000)
    assert lib.specattn_fused(C.byref(s3), C.byref(_attn(**ws)), None) == sa.EUNSUPPORTED
    # sizes: the on-chip route adds block counts + mask, the list route adds the list
    on_chip = sa.specattn_workspace_size(s, _attn())
    assert on_chip >= sa.specattn_workspace_size(None, _attn()) + 2 * 8 * 4 * 4 + 2 * 8 * 4 * 32 * 4
    s4 = _sel(B=2, H_kv=8, n_max=4096, probs_stride_b=8 * 4096, probs_stride_h=4096, indices=None, chunk_size=16)
    assert sa.specattn_workspace_size(s4, _attn()) >= sa.specattn_workspace_size(None, _attn()) + 2 * 8 * 256 * 4
