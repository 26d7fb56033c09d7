"""Host-side logic of libsdnn and the shape of its C ABI.  No GPU compute."""
import ctypes as C
import os
import re

import numpy as np
import pytest
import scipy.sparse as sp

from paper_2104_11805_amd import sdnn, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sdnn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(sdnn_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 15
    assert declared == set(sdnn.SIGNATURES), declared ^ set(sdnn.SIGNATURES)
    l = sdnn.lib()
    for name in declared:
        assert hasattr(l, name), name
    assert b"gfx950" in l.sdnn_version()


def _csr(layer):
    return layer.n_out, layer.n_in, layer.row_ptr, layer.col_idx


def test_check_csr_accepts_generated_layers_and_rejects_malformed():
    lay = wl.random_layer(3, 9, 7, 0.4)
    assert sdnn.sdnn_check_csr(*_csr(lay)) == 0
    bad = lay.col_idx.copy(); bad[1] = 7
    assert sdnn.sdnn_check_csr(lay.n_out, lay.n_in, lay.row_ptr, bad) == sdnn.SDNN_EINVAL
    assert "out of range" in sdnn.last_error()
    r0 = next(j for j in range(lay.n_out) if lay.row_ptr[j + 1] - lay.row_ptr[j] >= 2)
    dup = lay.col_idx.copy(); dup[lay.row_ptr[r0] + 1] = dup[lay.row_ptr[r0]]
    assert sdnn.sdnn_check_csr(lay.n_out, lay.n_in, lay.row_ptr, dup) == sdnn.SDNN_EINVAL
    assert "ascending" in sdnn.last_error()
    rp = lay.row_ptr.copy(); rp[0] = 1
    assert sdnn.sdnn_check_csr(lay.n_out, lay.n_in, rp, lay.col_idx) == sdnn.SDNN_EINVAL
    rp = lay.row_ptr.copy(); rp[3] = rp[2] - 1
    assert sdnn.sdnn_check_csr(lay.n_out, lay.n_in, rp, lay.col_idx) == sdnn.SDNN_EINVAL
    assert sdnn.sdnn_check_csr(-1, 3, lay.row_ptr, lay.col_idx) == sdnn.SDNN_EINVAL
    # empty matrix is fine
    assert sdnn.sdnn_check_csr(0, 5, np.zeros(1, np.int32), np.zeros(0, np.int32)) == 0


@pytest.mark.parametrize("shape", [(13, 9), (9, 13), (64, 64), (1, 5), (5, 1)])
def test_transpose_pattern_against_scipy_and_involution(shape):
    lay = wl.random_layer(17, shape[0], shape[1], 0.35)
    t_rp, t_ri, t_pm = sdnn.sdnn_transpose_pattern(*_csr(lay))
    nnz = lay.nnz
    assert sorted(t_pm.tolist()) == list(range(nnz)), "perm is not a bijection"
    tags = np.arange(1, nnz + 1, dtype=np.float64)
    csc = sp.csr_matrix((tags, lay.col_idx, lay.row_ptr), shape=shape).tocsc()
    csc.sort_indices()
    np.testing.assert_array_equal(t_rp, csc.indptr)
    np.testing.assert_array_equal(t_ri, csc.indices)
    np.testing.assert_array_equal(t_pm, csc.data.astype(np.int64) - 1)
    for i in range(shape[1]):
        seg = t_ri[t_rp[i]:t_rp[i + 1]]
        assert (np.diff(seg) > 0).all()
        assert (lay.col_idx[t_pm[t_rp[i]:t_rp[i + 1]]] == i).all()
    # transpose(transpose(W)) == W
    b_rp, b_ri, b_pm = sdnn.sdnn_transpose_pattern(shape[1], shape[0], t_rp, t_ri)
    np.testing.assert_array_equal(b_rp, lay.row_ptr)
    np.testing.assert_array_equal(b_ri, lay.col_idx)
    np.testing.assert_array_equal(t_pm[b_pm], np.arange(nnz))


def test_transpose_of_benchmark_layer_counts_column_links():
    lay = wl.regular_layer(1001, 1024, 32, 0.0625, -0.3)
    t_rp, t_ri, t_pm = sdnn.sdnn_transpose_pattern(*_csr(lay))
    np.testing.assert_array_equal(np.diff(t_rp), np.bincount(lay.col_idx, minlength=1024))
    assert t_rp[-1] == lay.nnz == 32 * 1024


def test_row_schedule_is_stable_longest_first():
    lay = wl.irregular_layer(5, 256)
    order = sdnn.sdnn_row_schedule(lay.n_out, lay.row_ptr)
    lens = np.diff(lay.row_ptr)
    assert sorted(order.tolist()) == list(range(256))
    assert (np.diff(lens[order]) <= 0).all()
    ties = lens[order][1:] == lens[order][:-1]
    assert (np.diff(order)[ties] > 0).all()


def _layer_array(layers):
    keep, arr = [], (sdnn.sdnn_layer * len(layers))()
    for k, l in enumerate(layers):
        a = [np.ascontiguousarray(l.row_ptr, np.int32), np.ascontiguousarray(l.col_idx, np.int32),
             np.ascontiguousarray(l.values, np.float32), np.ascontiguousarray(l.bias, np.float32)]
        keep += a
        arr[k] = sdnn.sdnn_layer(l.n_out, l.n_in, *[x.ctypes.data for x in a])
    return arr, keep


def test_workspace_bytes_and_argument_errors_without_gpu():
    net = wl.tiny_net(1, sizes=(7, 9, 6, 8))
    arr, keep = _layer_array(net.layers)
    l = sdnn.lib()
    n = C.c_size_t(0)
    cfg = sdnn.sdnn_config(float("inf"), 16, 1, 1, 0)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(cfg), C.byref(n)) == 0
    train_bytes = n.value
    nnz = sum(x.nnz for x in net.layers)
    # CSR + transposed index (5 x 4 bytes per entry) + activations and deltas
    assert train_bytes >= 20 * nnz + 4 * 16 * (2 * (9 + 6 + 8) + 7)
    cfg_inf = sdnn.sdnn_config(float("inf"), 16, 0, 1, 0, 0, 0, 0, sdnn.SDNN_LDS_OFF)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(cfg_inf), C.byref(n)) == 0
    assert 0 < n.value < train_bytes
    # an inference net of narrow layers also holds the lane-major copy for the LDS-resident forward:
    # 8 bytes per entry of the 64-row blocks, each as deep as its longest row
    plain_inf = n.value
    cfg_lds = sdnn.sdnn_config(float("inf"), 16, 0, 1, 0)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(cfg_lds), C.byref(n)) == 0
    padded = sum(64 * int(np.diff(x.row_ptr).max()) for x in net.layers)       # one block per layer here
    assert n.value >= plain_inf + 8 * padded
    bad = sdnn.sdnn_config(32.0, 4, 0, 1, 0, 0, 0, 0, 5)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(bad), C.byref(n)) == sdnn.SDNN_EINVAL
    bad = sdnn.sdnn_config(32.0, 4, 0, 1, 0, 0, -2)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(bad), C.byref(n)) == sdnn.SDNN_EINVAL
    bad = sdnn.sdnn_config(32.0, 4, 0, 1, 0, 0, 0, 2)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(bad), C.byref(n)) == sdnn.SDNN_EINVAL
    # argument errors are reported before any GPU work
    bad = sdnn.sdnn_config(float("inf"), 0, 1, 1, 0)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(bad), C.byref(n)) == sdnn.SDNN_EINVAL
    bad = sdnn.sdnn_config(0.0, 4, 1, 1, 0)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(bad), C.byref(n)) == sdnn.SDNN_EINVAL
    assert l.sdnn_workspace_bytes(arr, 0, C.byref(cfg), C.byref(n)) == sdnn.SDNN_EINVAL
    bad = sdnn.sdnn_config(32.0, 4, 1, 1, 7)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(bad), C.byref(n)) == sdnn.SDNN_EINVAL
    assert "activation" in sdnn.last_error()
    bad = sdnn.sdnn_config(32.0, 4, 1, 1, 0, 2)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(bad), C.byref(n)) == sdnn.SDNN_EINVAL
    assert "fuse_gradient" in sdnn.last_error()
    # the fused gradient keeps, per stored entry, two partial gradients, the value in transposed order and the four
    # arrays of the way back to CSR order (4 + 4 + 4 + 2 + 4 + 2 + 4 bytes; each array 256-byte aligned per layer)
    fused = sdnn.sdnn_config(float("inf"), 16, 1, 1, 0, sdnn.SDNN_FUSE_ON)
    nf = C.c_size_t(0)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(fused), C.byref(nf)) == 0
    assert train_bytes + 24 * nnz <= nf.value <= train_bytes + 24 * nnz + 3 * 7 * 256
    off = sdnn.sdnn_config(float("inf"), 16, 1, 1, 0, sdnn.SDNN_FUSE_OFF)
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(off), C.byref(nf)) == 0 and nf.value == train_bytes
    sig = sdnn.sdnn_config(0.0, 4, 1, 1, sdnn.SDNN_ACT_SIGMOID)      # the cap is ignored for the sigmoid
    assert l.sdnn_workspace_bytes(arr, 3, C.byref(sig), C.byref(n)) == 0
    h = C.c_void_p(1)
    assert l.sdnn_create(arr, 3, C.byref(cfg), None, train_bytes, None, C.byref(h)) == sdnn.SDNN_EINVAL
    assert h.value is None
    assert l.sdnn_create(arr, 3, C.byref(cfg), C.c_void_p(4096 + 8), train_bytes, None, C.byref(h)) == sdnn.SDNN_EINVAL
    assert "aligned" in sdnn.last_error()
    assert l.sdnn_create(arr, 3, C.byref(cfg), C.c_void_p(4096), train_bytes - 1, None, C.byref(h)) == sdnn.SDNN_ENOMEM
    # consecutive layers must chain
    arr2, keep2 = _layer_array([net.layers[0], net.layers[2]])
    assert l.sdnn_workspace_bytes(arr2, 2, C.byref(cfg), C.byref(n)) == sdnn.SDNN_EINVAL
    # calls on a NULL net
    assert l.sdnn_forward(None, None, 1, None, None) == sdnn.SDNN_EINVAL
    assert l.sdnn_backward(None, None, None) == sdnn.SDNN_EINVAL
    assert l.sdnn_sgd_step(None, 0.1, None) == sdnn.SDNN_EINVAL
    l.sdnn_destroy(None)
    # the measurement aid checks its arguments before it touches the GPU
    assert l.sdnn_gather_probe(None, 16, 1, None, 4, 8, None, None) == sdnn.SDNN_EINVAL
    assert l.sdnn_gather_probe(C.c_void_p(4096), 16, 3, C.c_void_p(4096), 4, 8, C.c_void_p(4096), None) == sdnn.SDNN_EINVAL
    assert l.sdnn_gather_probe(C.c_void_p(4096), 16, 1, C.c_void_p(4096), 6, 8, C.c_void_p(4096), None) == sdnn.SDNN_EINVAL
    assert l.sdnn_gather_probe(C.c_void_p(4096), 16, 1, C.c_void_p(4096), 4, 12, C.c_void_p(4096), None) == sdnn.SDNN_EINVAL
    assert l.sdnn_gather_probe(C.c_void_p(4096), 1 << 24, 4, C.c_void_p(4096), 4, 8, C.c_void_p(4096), None) == sdnn.SDNN_EINVAL
    assert l.sdnn_forward_noalloc(None, None, 1, None, None) == sdnn.SDNN_EINVAL


def test_malformed_layer_is_rejected_by_create_without_gpu():
    net = wl.tiny_net(2, sizes=(7, 9, 6))
    net.layers[1].col_idx = net.layers[1].col_idx.copy()
    net.layers[1].col_idx[0] = 99
    arr, keep = _layer_array(net.layers)
    cfg = sdnn.sdnn_config(32.0, 4, 1, 1, 0)
    h = C.c_void_p()
    assert sdnn.lib().sdnn_create(arr, 2, C.byref(cfg), C.c_void_p(4096), 1 << 30, None, C.byref(h)) == sdnn.SDNN_EINVAL
    assert "layer 2" in sdnn.last_error()


def test_host_setup_routines_under_sanitizers(tmp_path):
    """sdnn_setup.cpp (CSR check, transposed index, row schedule, row clustering and dealing) with ASan + UBSan on the host."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = tmp_path / "host_setup_sanitize"
    # the HIP vector-type header is only needed for device descriptors: give the host build a stand-in
    stub = tmp_path / "hip"
    stub.mkdir()
    (stub / "hip_vector_types.h").write_text("struct int4 { int x, y, z, w; };\nstruct int2 { int x, y; };\n")
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", str(tmp_path), os.path.join(ROOT, "tests", "host_setup_sanitize.cpp"),
           os.path.join(ROOT, "paper_2104_11805_amd", "csrc", "sdnn_setup.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)
    out = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "host setup: ok" in out.stdout


def test_header_is_plain_c_and_host_entry_points_link(tmp_path):
    """include/sdnn.h compiled as C99 (-pedantic -Werror) into a program that links libsdnn.so and calls
    the host-only entry points."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sdnn.lib()                                      # makes sure the library is built
    exe = str(tmp_path / "c_abi_check")
    libdir = os.path.dirname(sdnn.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(root, "include"),
                    os.path.join(root, "tests", "c_abi_check.c"), "-o", exe, "-L", libdir, "-lsdnn",
                    "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    assert "c abi ok" in out


def test_row_clustering_finds_planted_clusters_and_deals_them_to_one_xcd():
    """Structured pattern (rows j, j + n/32, ... share their 32 columns): the greedy clustering recovers exactly
    those groups; the dealing puts each on one XCD's schedule places; random patterns stay in length order."""
    n = 2048
    lay = wl.strided_layer(3, n)
    order, cl = sdnn.sdnn_cluster_rows(n, n, lay.row_ptr, lay.col_idx)
    assert sorted(order.tolist()) == list(range(n))
    assert cl.max() + 1 == n // 32 and (np.bincount(cl) == 32).all()
    stride = n // 32
    for c in range(cl.max() + 1):
        assert len(set((np.nonzero(cl == c)[0] % stride).tolist())) == 1
    assert (np.diff(cl[order]) >= 0).all()                       # cluster by cluster
    dealt = sdnn.sdnn_deal_rows_to_xcds(n, lay.row_ptr, order)
    assert sorted(dealt.tolist()) == list(range(n))
    xcd_of_row = np.empty(n, int)
    xcd_of_row[dealt] = (np.arange(n) // 4) % 8
    assert all(len(set(xcd_of_row[cl == c].tolist())) == 1 for c in range(cl.max() + 1))
    # capped clusters
    order2, cl2 = sdnn.sdnn_cluster_rows(n, n, lay.row_ptr, lay.col_idx, 8)
    assert np.bincount(cl2).max() <= 8 and sorted(order2.tolist()) == list(range(n))
    # nothing shared: every row its own cluster, the order is the longest-first schedule
    rnd = wl.regular_layer(2001, 1024, 32, 0.0625, -0.3)
    order3, cl3 = sdnn.sdnn_cluster_rows(1024, 1024, rnd.row_ptr, rnd.col_idx)
    assert cl3.max() + 1 == 1024 and np.array_equal(order3, sdnn.sdnn_row_schedule(1024, rnd.row_ptr))
    irr = wl.irregular_layer(5, 512)
    order4, _ = sdnn.sdnn_cluster_rows(512, 512, irr.row_ptr, irr.col_idx)
    dealt4 = sdnn.sdnn_deal_rows_to_xcds(512, irr.row_ptr, order4)
    assert sorted(order4.tolist()) == list(range(512)) and sorted(dealt4.tolist()) == list(range(512))
    # degenerate sizes and errors
    e_order, _ = sdnn.sdnn_cluster_rows(0, 5, np.zeros(1, np.int32), np.zeros(0, np.int32))
    assert e_order.size == 0
    assert sdnn.lib().sdnn_cluster_rows(4, 4, None, None, 8, None, None) == sdnn.SDNN_EINVAL
    assert sdnn.lib().sdnn_deal_rows_to_xcds(4, None, None, None) == sdnn.SDNN_EINVAL
