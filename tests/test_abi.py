"""Host-side checks of the C ABI (no GPU needed): the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib(hgnn):
    return hgnn.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "hgnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hgnn_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib, hgnn):
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(hgnn.EXPORTS) == names  # the Python binding covers exactly the declared entry points


def test_status_strings(lib):
    for code in range(5):
        assert lib.hgnn_status_str(code).decode().startswith("HGNN_")
    assert b"unknown" in lib.hgnn_status_str(99)


def make_csr(hgnn, nrows=4, ncols=4, nnz=8, rowptr=0x1000, col=0x2000):
    from paper_2411_01109_amd.binding import _CsrStruct
    return _CsrStruct(nrows, ncols, nnz, rowptr, col, None, None)


def test_argument_errors_are_caught_on_the_host(lib, hgnn):
    """Fake non-NULL device addresses: every call below must return before touching the GPU."""
    g = make_csr(hgnn)
    X, Y = 0x10000, 0x20000
    EINVAL, EUNSUP = hgnn.HGNN_EINVAL, hgnn.HGNN_EUNSUPPORTED
    call = lambda *a: lib.hgnn_spmm(ctypes.byref(g), None, 1, *a)
    assert call(X, 8, Y, 8, 7, 0, None, None, 0, None) == EINVAL          # odd F: pad to even (section 4.1)
    assert b"odd" in lib.hgnn_last_error()
    assert call(X, 8, Y, 8, 0, 0, None, None, 0, None) == EINVAL          # F <= 0
    assert call(X, 4, Y, 8, 8, 0, None, None, 0, None) == EINVAL          # ldx < F
    assert call(X, 8, Y, 8, 8, 5, None, None, 0, None) == EINVAL          # unknown reduce op
    assert call(None, 8, Y, 8, 8, 0, None, None, 0, None) == EINVAL       # X NULL with nnz > 0
    assert call(X, 8, None, 8, 8, 0, None, None, 0, None) == EINVAL       # Y NULL
    assert lib.hgnn_plan_create(ctypes.byref(g), 256, 64, 1, -1, ctypes.byref(ctypes.c_void_p()), None) == EINVAL
    assert lib.hgnn_spmm(ctypes.byref(g), None, 3, X, 8, Y, 8, 8, 0, None, None, 0, None) == EINVAL  # H does not divide F
    assert lib.hgnn_spmm(None, None, 1, X, 8, Y, 8, 8, 0, None, None, 0, None) == EINVAL             # graph NULL
    bad = make_csr(hgnn, rowptr=None)
    assert lib.hgnn_spmm(ctypes.byref(bad), None, 1, X, 8, Y, 8, 8, 0, None, None, 0, None) == EINVAL
    big = make_csr(hgnn, nnz=1 << 31)
    assert lib.hgnn_spmm(ctypes.byref(big), None, 1, X, 8, Y, 8, 8, 0, None, None, 0, None) == EINVAL
    # discretized: plan required
    assert lib.hgnn_spmm_discretized(None, ctypes.byref(g), None, 1, X, 8, Y, 8, 8, 0, None, None) == EINVAL
    # sddmm / softmax
    sd = lambda *a: lib.hgnn_sddmm(ctypes.byref(g), None, *a)
    assert sd(0, 1, 7, X, 8, X, 8, None, None, 0.2, Y, None) == EINVAL      # odd F
    assert sd(7, 1, 8, X, 8, X, 8, None, None, 0.2, Y, None) == EINVAL      # unknown op
    assert sd(0, 1, 8, None, 8, X, 8, None, None, 0.2, Y, None) == EINVAL   # U NULL
    assert sd(1, 1, 8, X, 8, X, 8, None, None, 0.2, Y, None) == EINVAL      # GAT score without a_l / a_r
    assert lib.hgnn_edge_softmax(ctypes.byref(g), None, 0, X, Y, None) == EINVAL
    assert lib.hgnn_edge_softmax(ctypes.byref(g), None, 1, None, Y, None) == EINVAL
    assert lib.hgnn_edge_softmax_bwd(ctypes.byref(g), None, 1, X, None, None, 0.2, Y, None) == EINVAL
    assert lib.hgnn_edge_rowsum(ctypes.byref(g), None, 0, X, Y, None) == EINVAL
    eidg = make_csr(hgnn)
    eidg.eid = 0x3000
    assert lib.hgnn_edge_softmax(ctypes.byref(eidg), None, 1, X, Y, None) == EUNSUP
    # plan_create argument checks come before any device work
    out = ctypes.c_void_p()
    assert lib.hgnn_plan_create(ctypes.byref(g), 0, 64, 1, 1, ctypes.byref(out), None) == EINVAL
    assert lib.hgnn_plan_create(ctypes.byref(g), 4096, 64, 1, 1, ctypes.byref(out), None) == EINVAL
    assert lib.hgnn_plan_create(ctypes.byref(g), 256, 12, 1, 1, ctypes.byref(out), None) == EINVAL
    assert lib.hgnn_plan_create(ctypes.byref(g), 256, 64, 1, 65, ctypes.byref(out), None) == EINVAL
    assert lib.hgnn_plan_create(ctypes.byref(g), 256, 64, 1, 1, None, None) == EINVAL
    assert out.value is None
    lib.hgnn_plan_destroy(None)  # no-op
    assert lib.hgnn_plan_num_segments(None) == 0


def test_extension_entry_points_check_arguments_on_the_host(lib, hgnn):
    """The variant, group, fused-GAT and table helpers refuse a missing plan or a bad scalar before any launch."""
    g = make_csr(hgnn)
    gp = ctypes.byref(g)
    X, Y, A = 0x10000, 0x20000, 0x30000
    EINVAL = hgnn.HGNN_EINVAL
    assert lib.hgnn_spmm_discretized_variant(None, gp, None, 1, X, 8, Y, 8, 8, 0, None, 0, None) == EINVAL
    assert lib.hgnn_plan_add_groups(None, gp, 32, None) == EINVAL
    assert lib.hgnn_plan_num_groups(None) == 0
    assert lib.hgnn_plan_group_edges(None) == 0
    assert lib.hgnn_plan_groups_export(None, gp, X, Y) == EINVAL
    assert lib.hgnn_gat_forward_fused(gp, None, 1, 8, X, 8, X, 8, A, A, 0.2, Y, 8, A, None) == EINVAL
    assert lib.hgnn_gat_alpha(gp, None, 1, 8, X, 8, X, 8, A, A, 0.2, A, Y, None) == EINVAL
    assert lib.hgnn_gat_backward_fused(gp, None, gp, None, 1, 8, X, 8, X, 8, A, A, 0.2, Y, 8, A, X, 8,
                                       Y, 8, A, A, None) == EINVAL
    assert lib.hgnn_gat_forward_fused_save(gp, None, 1, 8, X, 8, X, 8, A, A, 0.2, Y, 8, A, Y, 8, A, None) == EINVAL
    assert lib.hgnn_gat_forward_fused_save(gp, None, 1, 8, X, 8, X, 8, A, A, 0.2, Y, 8, A, None, 8, A, None) == EINVAL
    assert b"required" in lib.hgnn_last_error()
    assert lib.hgnn_gat_backward_fused_saved(gp, None, gp, None, 1, 8, X, 8, X, 8, A, A, 0.2, Y, 8, A, None, 8, None, X, 8,
                                             Y, 8, A, A, None) == EINVAL
    assert lib.hgnn_edge_to_transposed(None, 1, X, Y, None) == EINVAL
    assert lib.hgnn_edge_to_transposed(gp, 1, X, Y, None) == EINVAL           # a transposed graph carries eid
    assert lib.hgnn_scale_rows(4, 0, X, 8, A, Y, 8, None) == EINVAL            # F <= 0
    assert lib.hgnn_scale_rows(4, 8, X, 12, A, Y, 8, None) == hgnn.HGNN_EUNSUPPORTED  # pitch not a multiple of 8
    assert lib.hgnn_scale_rows(4, 8, X, 4, A, Y, 8, None) == EINVAL            # pitch < F
    assert lib.hgnn_scale_rows(4, 8, X, 8, None, Y, 8, None) == EINVAL         # scale NULL
    assert lib.hgnn_scale_rows(-1, 8, X, 8, A, Y, 8, None) == EINVAL
    # column slices and the column sums over them; the static-scratch SpMM: argument checks come before any launch
    assert lib.hgnn_plan_add_slices(None, gp, 0, None) == EINVAL
    assert lib.hgnn_plan_num_slices(None) == 0
    assert lib.hgnn_edge_colsum(gp, None, 1, X, Y, None) == EINVAL
    assert lib.hgnn_edge_colsum(None, None, 1, X, Y, None) == EINVAL
    assert lib.hgnn_spmm_static_limit() == 32 << 20
    assert lib.hgnn_spmm_static(None, None, 1, X, 8, Y, 8, 8, 0, None, None) == EINVAL
    assert lib.hgnn_spmm_static(gp, None, 1, X, 8, Y, 8, 7, 0, None, None) == EINVAL   # odd F
    huge = make_csr(hgnn, nrows=1000, ncols=1000, nnz=40_000_000)
    assert lib.hgnn_spmm_static(ctypes.byref(huge), None, 1, X, 128, Y, 128, 128, 0, None, None) == hgnn.HGNN_EUNSUPPORTED
    assert b"static" in lib.hgnn_last_error()
    l2, llc = ctypes.c_int64(-1), ctypes.c_int64(-1)
    lib.hgnn_plan_cache_bytes(None, ctypes.byref(l2), ctypes.byref(llc))
    assert l2.value == 0 and llc.value == 0
    assert lib.hgnn_plan_set_vector_halves(None, 8) == EINVAL
    assert lib.hgnn_plan_vector_halves(None) == 0
    # workspace of the plan-free SpMM: a bound from the sizes alone; nothing when no row can be long
    assert lib.hgnn_spmm_workspace(4, 4, 8, 64) == 0
    assert lib.hgnn_spmm_workspace(0, 0, 0, 64) == 0
    small, big = lib.hgnn_spmm_workspace(1000, 1000, 100000, 64), lib.hgnn_spmm_workspace(1000, 1000, 100000, 128)
    assert 0 < small < big and small % 256 == 0
    # long rows over a table beyond the L2s (30 MB, rows of 490): room for the fp32 partial rows of the column passes
    # on top of the long rows' scratch, which ncols = 0 gives alone; a short-row graph of the same size gets none
    V, E, F = 233000, 114000000, 64
    hubs_only, full = lib.hgnn_spmm_workspace(V, 0, E, F), lib.hgnn_spmm_workspace(V, V, E, F)
    assert hubs_only > 0 and full >= hubs_only + 2 * V * F * 4 and (full - hubs_only) % 256 == 0
    assert lib.hgnn_spmm_workspace(V, V, 20 * V, F) == lib.hgnn_spmm_workspace(V, 0, 20 * V, F)
    assert lib.hgnn_plan_col_blocks(None) == 0 and lib.hgnn_plan_col_blocks_fine(None) == 0


def test_header_is_plain_c_and_links(lib):
    """include/hgnn.h compiles as strict C99 (and as C++), and a C program that calls the library through it links
    against libhgnn.so and runs the host-only calls (no GPU needed for status strings and argument errors)."""
    src = r"""
#include <stdio.h>
#include <string.h>
#include "hgnn.h"
int main(void) {
  hgnn_csr g;
  memset(&g, 0, sizeof g);
  if (strncmp(hgnn_status_str(HGNN_EINVAL), "HGNN_", 5) != 0) return 1;
  if (hgnn_spmm(NULL, NULL, 1, NULL, 8, NULL, 8, 8, HGNN_SUM, NULL, NULL, 0, NULL) != HGNN_EINVAL) return 2;
  if (hgnn_last_error()[0] == 0) return 3;
  if (hgnn_linear_wgrad_workspace(64, 64) == 0) return 4;
  if (hgnn_plan_num_segments(NULL) != 0) return 5;
  puts("ok");
  return 0;
}
"""
    inc = os.path.join(ROOT, "include")
    libdir = os.path.join(ROOT, "paper_2411_01109_amd")
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "t.c")
        open(c, "w").write(src)
        subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-c", c, "-o", os.path.join(d, "t.o")])
        subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Werror", "-I", inc, "-x", "c++", "-c", c, "-o", os.path.join(d, "t2.o")])
        exe = os.path.join(d, "t")
        subprocess.check_call(["gcc", os.path.join(d, "t.o"), "-o", exe, "-L", libdir, "-lhgnn", "-Wl,-rpath," + libdir])
        out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        assert out.returncode == 0 and out.stdout.strip() == "ok", (out.returncode, out.stdout, out.stderr)


def test_binding_refuses_cpu_tensors(hgnn):
    import torch
    with pytest.raises(TypeError):
        hgnn.Csr(torch.zeros(3, dtype=torch.int32), torch.zeros(2, dtype=torch.int32))


def test_product_path_has_no_oracle_or_fallback():
    """Neither the package nor bench's product leg may import the oracle; the oracle must not import the package."""
    pkg = os.path.join(ROOT, "paper_2411_01109_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2411_01109_amd" not in text and "libhgnn" not in text and "hgnn.h" not in text, f


def test_coo_to_csr_argument_errors_are_caught_on_the_host(lib, hgnn):
    """Fake non-NULL device addresses: each call must return before anything is launched."""
    R, C, P, O = 0x1000, 0x2000, 0x3000, 0x4000
    EINVAL = hgnn.HGNN_EINVAL
    assert lib.hgnn_coo_to_csr(4, 4, 8, R, C, None, O, None, None) == EINVAL      # rowptr NULL
    assert lib.hgnn_coo_to_csr(4, 4, 8, None, C, P, O, None, None) == EINVAL      # row NULL with edges
    assert lib.hgnn_coo_to_csr(4, 4, 8, R, C, P, None, None, None) == EINVAL      # col_out NULL with edges
    assert lib.hgnn_coo_to_csr(-1, 4, 0, R, C, P, O, None, None) == EINVAL        # negative size
    assert lib.hgnn_coo_to_csr(0, 4, 8, R, C, P, O, None, None) == EINVAL         # edges without rows
    assert lib.hgnn_coo_to_csr(4, 4, 1 << 31, R, C, P, O, None, None) == EINVAL   # nnz beyond int32
    assert b"int32" in lib.hgnn_last_error()
