"""The C-ABI library loads without a GPU and exports every function include/tma.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2305_09887_amd", "libtma.so")


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "tma.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tma_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2305_09887_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(LIB)


def test_header_declares_the_north_star_calls():
    names = _declared_functions()
    for need in ("tma_partition", "tma_induced_subgraph_count", "tma_induced_subgraph_fill", "tma_sage_layer_fwd",
                 "tma_sage_layer_bwd", "tma_average"):
        assert need in names


def test_library_exports_every_declared_symbol(lib):
    for name in _declared_functions():
        assert hasattr(lib, name), f"libtma.so does not export {name}"


def test_binding_lists_the_same_symbols():
    from paper_2305_09887_amd import binding
    assert sorted(binding.EXPORTS) == _declared_functions()


def test_host_side_argument_validation_needs_no_gpu(lib):
    lib.tma_last_error.restype = ctypes.c_char_p
    assert lib.tma_version() >= 100
    # K = 0 is rejected before anything touches a device
    rc = lib.tma_partition(ctypes.c_int64(8), None, ctypes.c_int64(0), ctypes.c_int32(0), ctypes.c_uint64(1), None, None)
    assert rc == -1 and b"K=0" in lib.tma_last_error()
    lib.tma_loss_workspace_bytes.restype = ctypes.c_size_t
    assert lib.tma_loss_workspace_bytes(ctypes.c_int64(1000), ctypes.c_int32(47)) % 256 == 0
    lib.tma_sage_layer_bwd_workspace_bytes.restype = ctypes.c_size_t
    small = lib.tma_sage_layer_bwd_workspace_bytes(ctypes.c_int64(1000), 64, 64, 0, 0)
    large = lib.tma_sage_layer_bwd_workspace_bytes(ctypes.c_int64(1000), 64, 64, 0, 1)
    assert large >= small + 1000 * 64 * 4


def test_extraction_entry_points_reject_bad_arguments_before_touching_a_device(lib):
    """The no-wait and fused forms of the extraction: every refusal below happens in host code."""
    lib.tma_last_error.restype = ctypes.c_char_p
    i64, i32, u64, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_size_t
    fake = ctypes.c_void_p(4096)            # a non-NULL, 256-byte aligned address that is never dereferenced

    def fused(n, K, p, cap_n, cap_e, sizes=fake, ws=fake, ws_bytes=1 << 40):
        return lib.tma_random_subgraph_async(i64(n), fake, fake, i32(K), u64(7), i32(p), fake, fake, fake, fake, fake,
                                             i64(cap_n), i64(cap_e), sizes, ws, sz(ws_bytes), None)

    assert fused(100, 0, 0, 10, 10) < 0 and b"K outside" in lib.tma_last_error()
    assert fused(100, 4, 4, 10, 10) < 0 and b"p outside" in lib.tma_last_error()
    assert fused(100, 4, 1, 10, -1) < 0 and b"cap_nnz_loc" in lib.tma_last_error()
    assert fused(100, 4, 1, 10, 10, sizes=None) < 0 and b"d_sizes_out" in lib.tma_last_error()
    assert fused(100, 4, 1, 101, 10) < 0 and b"cap_n_loc" in lib.tma_last_error()
    assert fused(-1, 4, 1, 0, 0) < 0 and b"n_nodes" in lib.tma_last_error()
    assert fused(100, 4, 1, 10, 10, ws=ctypes.c_void_p(4100)) < 0 and b"aligned" in lib.tma_last_error()
    assert fused(100, 4, 1, 10, 10, ws_bytes=16) < 0 and b"workspace" in lib.tma_last_error()
    rc = lib.tma_induced_subgraph_async(i64(100), fake, fake, None, i32(0), fake, fake, fake, fake, fake, i64(10), i64(10),
                                        fake, fake, sz(1 << 40), None)
    assert rc < 0 and b"part" in lib.tma_last_error()
    lib.tma_gcn_block_bwd_workspace_bytes.restype = sz
    assert lib.tma_gcn_block_bwd_workspace_bytes(i64(10), i64(5), i64(0), 8, 8, 0, 1) == 0      # n_src < n_dst
    assert lib.tma_gcn_block_bwd_workspace_bytes(i64(10), i64(50), i64(200), 8, 8, 0, 1) % 256 == 0


def test_device_count_forms_of_the_sampler_reject_bad_arguments_in_host_code(lib):
    lib.tma_last_error.restype = ctypes.c_char_p
    i64, i32, u64, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_size_t
    fake = ctypes.c_void_p(4096)            # non-NULL, 256-byte aligned, never dereferenced

    def sample(cap_dst, d_n=fake, cap_entries=1000, ws_bytes=1 << 40, fanout=5):
        return lib.tma_neighbor_sample_dev(i64(cap_dst), d_n, fake, i64(5000), fake, fake, i32(fanout), u64(1), fake, fake,
                                           fake, i64(cap_entries), fake, sz(ws_bytes), None)

    assert sample(100, d_n=None) < 0 and b"d_n_dst" in lib.tma_last_error()
    assert sample(100, fanout=0) < 0 and b"fanout" in lib.tma_last_error()
    assert sample(100, cap_entries=499) < 0 and b"room for 499 entries" in lib.tma_last_error()     # capacity rows count
    assert sample(100, ws_bytes=64) < 0 and b"workspace" in lib.tma_last_error()

    def relabel(n, cap_dst, max_items, cap_src, d_n=fake, out=fake, ws_bytes=1 << 40):
        return lib.tma_mfg_relabel_dev(i64(n), i64(cap_dst), d_n, fake, i64(max_items), None, fake, fake, i64(cap_src), out,
                                       fake, sz(ws_bytes), None)

    assert relabel(1000, 10, 50, 60, out=None) < 0 and b"d_n_src_out" in lib.tma_last_error()
    assert relabel(1000, 10, 50, 60, d_n=None) < 0 and b"d_n_dst" in lib.tma_last_error()
    assert relabel(1000, 10, 50, 59) < 0 and b"room for 59 source nodes" in lib.tma_last_error()
    assert relabel(1000, 1001, 0, 1001) < 0 and b"n_dst" in lib.tma_last_error()
    assert relabel(1000, 10, 50, 60, ws_bytes=64) < 0 and b"workspace" in lib.tma_last_error()
    rc = lib.tma_gather_rows_dev(i64(10), None, fake, fake, i64(64), i64(64), fake, i64(64), None)
    assert rc < 0 and b"d_n_rows" in lib.tma_last_error()
    rc = lib.tma_gather_rows_dev(i64(10), fake, fake, fake, i64(32), i64(64), fake, i64(64), None)
    assert rc < 0 and b"pitch" in lib.tma_last_error()


def test_prepared_weight_entry_points_reject_bad_arguments_in_host_code(lib):
    lib.tma_last_error.restype = ctypes.c_char_p
    i64, i32, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    fake = ctypes.c_void_p(4096)
    lib.tma_sage_weights_bf16_bytes.restype = sz
    assert lib.tma_sage_weights_bf16_bytes(i32(128), i32(256)) == 2 * 128 * 256 * 2
    assert lib.tma_sage_weights_bf16_bytes(i32(3), i32(5)) == 256 and lib.tma_sage_weights_bf16_bytes(i32(0), i32(5)) == 0
    assert lib.tma_sage_prepare_weights_bf16(fake, fake, i32(8), i32(8), None, None) < 0 and b"NULL" in lib.tma_last_error()
    assert lib.tma_sage_prepare_weights_bf16(fake, fake, i32(0), i32(8), fake, None) < 0 and b"F_in=0" in lib.tma_last_error()

    def fwd(dtype, wt):
        return lib.tma_sage_layer_fwd_prepared(i64(10), fake, fake, fake, fake, i64(8), i32(8), fake, fake, fake, i32(8), i32(0),
                                               i32(dtype), fake, i64(8), fake, i64(8), wt, None)

    assert fwd(0, fake) < 0 and b"bf16 storage" in lib.tma_last_error()
    assert fwd(1, None) < 0 and b"Wt_bf16" in lib.tma_last_error()
    assert fwd(1, ctypes.c_void_p(4100)) < 0 and b"16-byte aligned" in lib.tma_last_error()


def test_host_generator_reproduces_the_published_vector(lib):
    """tma_mix64 is host code: the library's generator against the published SplitMix64 outputs for seed 1234567
    (the same fixture that pins the oracle's), no GPU needed."""
    lib.tma_mix64.restype = ctypes.c_uint64
    lib.tma_mix64.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
    want = [int(tok, 0) for line in open(os.path.join(ROOT, "tests", "golden", "splitmix64_seed1234567.txt"))
            if not line.startswith("#") for tok in line.split()]
    assert len(want) >= 5
    assert [lib.tma_mix64(1234567, i) for i in range(len(want))] == want


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: `bench.py --gpus N` with N > 1 exits with a message that says so (no GPU needed to see it)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0 and "ONE GPU" in (r.stdout + r.stderr)
