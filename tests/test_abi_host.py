"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes agree with the container layout, and bad arguments give the documented codes."""
import ctypes
import os
import re

import numpy as np
import pytest

import adacomp_workloads as W
from paper_1712_02679_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_1712_02679_amd import build
        build.build()
    return binding.lib()


def test_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "adacomp.h")).read() + open(os.path.join(ROOT, "include", "adacomp_debug.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(adacomp_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_struct_sizes():
    assert ctypes.sizeof(binding.Layer) == 24
    assert binding.PACKET_HEADER.itemsize == 32 and binding.PACKET_LAYER.itemsize == 64


def test_bin_index_constants(L):
    assert binding.adacomp_selftest_binindex() == 0


def test_sizes_follow_the_container_layout(L):
    pad16 = lambda x: (x + 15) // 16 * 16
    for i in range(1, 6):
        t = W.workload(i).table()
        fixed = 32 + 64 * len(t)
        words = 0
        for _, n, T in t:
            wb = 1 if T <= 64 else 2
            nb = -(-n // T)
            fixed += pad16(nb * wb) + pad16(4 * (-(-nb // 64)))
            words += pad16(n * wb)
        assert binding.adacomp_packet_fixed_bytes(t) == fixed
        assert binding.adacomp_packet_bound(t) == fixed + words
        ws = binding.adacomp_workspace_bytes(t)
        assert ws > 2 * W.workload(i).n_total and ws < 2.5 * W.workload(i).n_total + (1 << 20)


def test_workspace_follows_the_element_count_not_the_address_span(L):
    far = [(4096, 50 * 4000 + 7, 50), (2 ** 32 + 4096, 500 * 600 + 13, 500), (2 ** 32 + 2 ** 31, 16384 * 6 + 5, 16384)]
    n_params = sum(n for _, n, _ in far)
    near = []
    off = 0
    for _, n, T in far:
        near.append((off, n, T))
        off += (n + 3) // 4 * 4
    assert binding.adacomp_workspace_bytes(far) == binding.adacomp_workspace_bytes(near) <= 3 * n_params
    assert binding.adacomp_workspace_bytes_batch(far, 4) - binding.adacomp_workspace_bytes_batch(far, 3) <= 2.2 * n_params


def test_bad_tables_are_refused(L):
    assert binding.adacomp_packet_bound([(0, 0, 50)]) == 0           # empty layer
    assert binding.adacomp_packet_bound([(0, 10, 0)]) == 0           # L_T = 0
    assert binding.adacomp_packet_bound([(0, 10, 16385)]) == 0       # L_T above 16K
    assert binding.adacomp_packet_bound([(2, 10, 50)]) == 0          # offset not a multiple of 4
    assert binding.adacomp_packet_bound([(0, 100, 50), (96, 8, 50)]) == 0   # overlap
    assert binding.adacomp_packet_bound([(0, 1 << 31, 50)]) == 0     # layer too long
    assert binding.adacomp_packet_bound([(0, 10, 16384)]) > 0
    assert binding.adacomp_workspace_bytes([]) == 0


def test_error_codes_without_touching_the_gpu(L):
    t = binding.layer_array([(0, 1000, 50)])
    buf = np.zeros(1 << 16, np.uint8)
    base = (buf.ctypes.data + 255) // 256 * 256
    p = ctypes.c_void_p
    # compress on a workspace that was never initialised
    rc = L.adacomp_compress(t, 1, p(base), p(base + 4096), p(base + 8192), 4096, p(base + 16384), 1 << 14, None)
    assert rc == binding.EWORKSPACE
    rc = L.adacomp_compress(t, 1, None, p(base + 4096), p(base + 8192), 4096, p(base + 16384), 1 << 14, None)
    assert rc == binding.EINVAL
    rc = L.adacomp_compress(t, 1, p(base + 4), p(base + 4096), p(base + 8192), 4096, p(base + 16384), 1 << 14, None)
    assert rc == binding.EALIGN
    rc = L.adacomp_compress(t, 1, p(base), p(base), p(base + 8192), 4096, p(base + 16384), 1 << 14, None)
    assert rc == binding.EINVAL                                       # grad aliases residue
    ptrs = (p * 1)(base)
    rc = L.adacomp_unpack_accumulate(t, 1, ptrs, 1, p(base + 4096), p(base + 16384), 1 << 14, None)
    assert rc == binding.EWORKSPACE
    rc = L.adacomp_workspace_init(t, 1, p(base + 16384 + 8), 1 << 14, None)
    assert rc == binding.EALIGN
    rc = L.adacomp_workspace_init(t, 1, p(base + 16384), 16, None)
    assert rc == binding.EWORKSPACE
    assert L.adacomp_workspace_release(p(base)) == binding.EINVAL
    # the lazy pair: same checks as the eager call; a sync needs a registered workspace
    gp, rp, pp = (p * 1)(base), (p * 1)(base + 4096), (p * 1)(base + 8192)
    rc = L.adacomp_compress_batch_lazy(t, 1, 1, gp, rp, pp, 4096, p(base + 16384), 1 << 14, None)
    assert rc == binding.EWORKSPACE
    rc = L.adacomp_compress_batch_lazy(t, 1, 1, gp, gp, pp, 4096, p(base + 16384), 1 << 14, None)
    assert rc == binding.EINVAL
    assert L.adacomp_residue_sync(None, None) == binding.EINVAL
    assert L.adacomp_residue_sync(p(base + 16384), None) == binding.EWORKSPACE
    assert b"adacomp_residue_sync" in L.adacomp_strerror(binding.EPENDING)
    assert b"L_T" in L.adacomp_strerror(binding.EBADLT)


def test_static_entry_point_refusals_need_no_gpu(L):
    """adacomp_compress_static: null pointers, bad tables and tables beyond the static array are
    refused on the host; a table that fits fails loudly without a GPU (no CPU path)."""
    import torch
    buf = np.zeros(1 << 16, np.uint8)
    base = (buf.ctypes.data + 255) // 256 * 256
    p = ctypes.c_void_p
    t = binding.layer_array([(0, 1000, 50)])
    assert L.adacomp_compress_static(t, 1, None, p(base + 4096), p(base + 8192), 4096, None) == binding.EINVAL
    assert L.adacomp_compress_static(None, 1, p(base), p(base + 4096), p(base + 8192), 4096, None) == binding.EINVAL
    if torch.cuda.is_available():
        return   # the rest would enqueue work on host pointers
    bad = binding.layer_array([(0, 1000, 16385)])
    assert L.adacomp_compress_static(bad, 1, p(base), p(base + 4096), p(base + 8192), 4096, None) == binding.EBADLT
    big = W.workload(3).table()
    assert binding.adacomp_workspace_bytes(big) > binding.STATIC_SCRATCH_BYTES
    rc = L.adacomp_compress_static(binding.layer_array(big), len(big), p(base), p(base + 4096), p(base + 8192), 1 << 30, None)
    assert rc == binding.ETOOBIG and b"16 MiB" in L.adacomp_strerror(rc)
    assert L.adacomp_compress_static(t, 1, p(base), p(base + 4096), p(base + 8192), 4096, None) == binding.EHIP


def test_no_cpu_fallback(L):
    """Without a GPU the set-up call fails loudly instead of computing anything on the host."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    t = binding.layer_array([(0, 1000, 50)])
    buf = np.zeros(1 << 16, np.uint8)
    base = (buf.ctypes.data + 255) // 256 * 256
    rc = L.adacomp_workspace_init(t, 1, ctypes.c_void_p(base), 1 << 15, None)
    assert rc == binding.EHIP


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before it touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert out.returncode != 0
    assert "one GPU" in out.stderr and out.stdout.strip() == ""
