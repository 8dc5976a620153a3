"""adacomp_compress_static, the entry point that allocates nothing (its workspace is a static device
array inside the library), against adacomp_compress on a workspace of the caller's and against the
CPU oracle: packet and residue bit for bit, on calls in a row that share the array, the later ones
with smaller layer tables."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import adacomp_workloads as W  # noqa: E402

f32 = np.float32
POISON = 0xCD


def _case(A, oracle_lib, wl, n_steps, seed):
    """n_steps free-running steps of one learner through the static entry point, through
    adacomp_compress and through the oracle."""
    dev = "cuda:0"
    table, n = wl.table(), wl.n_total
    bound = A.adacomp_packet_bound(table)
    ws = torch.zeros(A.adacomp_workspace_bytes(table), dtype=torch.uint8, device=dev)
    A.adacomp_workspace_init(table, ws)
    try:
        R_static = torch.zeros(n, dtype=torch.float32, device=dev)
        R_plain = torch.zeros(n, dtype=torch.float32, device=dev)
        R_cpu = np.zeros(n, f32)
        pk_static = torch.empty(bound + 64, dtype=torch.uint8, device=dev)
        pk_plain = torch.empty(bound + 64, dtype=torch.uint8, device=dev)
        for t in range(n_steps):
            print(f"[no_alloc] {wl.name} step {t}", flush=True)
            g_np = W.gradient(wl, 0, t, seed=seed)
            g = torch.from_numpy(g_np).to(dev)
            pk_static.fill_(POISON)
            pk_plain.fill_(POISON)
            A.adacomp_compress_static(table, g, R_static, pk_static, packet_capacity=bound)
            A.adacomp_compress(table, g, R_plain, pk_plain, ws, packet_capacity=bound)
            torch.cuda.synchronize()
            want = oracle_lib.compress(table, g_np, R_cpu)
            assert torch.equal(pk_static, pk_plain), f"{wl.name} step {t}: packet differs from adacomp_compress"
            assert torch.equal(R_static.view(torch.int32), R_plain.view(torch.int32)), f"{wl.name} step {t}: residue"
            got = pk_static.cpu().numpy()
            assert np.array_equal(got[:want.size], want), f"{wl.name} step {t}: packet differs from the oracle"
            assert np.all(got[want.size:] == POISON)
            assert np.array_equal(R_static.cpu().numpy().view(np.uint32), R_cpu.view(np.uint32))
    finally:
        A.adacomp_workspace_release(ws)


def test_static_scratch_entry_point(oracle_lib):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1712_02679_amd as A
    from paper_1712_02679_amd import binding
    # the char-LSTM table (3.3 M elements, about 7 MB of the 16 MiB array), then the smaller CIFAR-CNN
    # table (two word widths), then a tiny one, then the first again: every change of table rewrites
    # the tile tables over what the previous call left in the array
    big = W.workload(4)
    _case(A, oracle_lib, big, 2, seed=5)
    _case(A, oracle_lib, W.workload(2), 3, seed=6)
    _case(A, oracle_lib, W.custom("tiny", [("a", 777, 50), ("b", 1301, 500), ("c", 5, 16384)]), 2, seed=7)
    _case(A, oracle_lib, big, 1, seed=8)
    # a table that does not fit the array is refused before anything is enqueued
    wl3 = W.workload(3)
    assert A.adacomp_workspace_bytes(wl3.table()) > binding.STATIC_SCRATCH_BYTES
    g = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    r = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    p = torch.zeros(A.adacomp_packet_fixed_bytes(wl3.table()), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(A.AdacompError) as e:
        A.adacomp_compress_static(wl3.table(), g, r, p)
    assert e.value.code == binding.ETOOBIG
    # and the array still serves the next call
    _case(A, oracle_lib, W.workload(1), 2, seed=9)


def test_static_scratch_entry_point_in_a_hip_graph(oracle_lib):
    """What the entry point is for: once its static array holds the tile tables of a layer table (one
    call outside the capture), a call only launches kernels, so it can be captured in a HIP graph.  The
    graph is replayed several times with eager work and synchronisations in between; every replay is
    checked against the free-running oracle."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1712_02679_amd as A
    dev = "cuda:0"
    wl = W.workload(2)
    table, n = wl.table(), wl.n_total
    bound = A.adacomp_packet_bound(table)
    g_in = torch.zeros(n, dtype=torch.float32, device=dev)
    R = torch.zeros(n, dtype=torch.float32, device=dev)
    pk = torch.empty(bound + 64, dtype=torch.uint8, device=dev)
    # eager neighbour on a workspace of its own, run between the replays
    ws = torch.zeros(A.adacomp_workspace_bytes(table), dtype=torch.uint8, device=dev)
    A.adacomp_workspace_init(table, ws)
    R2 = torch.zeros(n, dtype=torch.float32, device=dev)
    pk2 = torch.empty(bound, dtype=torch.uint8, device=dev)
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):   # outside the capture: writes the tile tables into the static array
            A.adacomp_compress_static(table, g_in, R, pk, packet_capacity=bound)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            A.adacomp_compress_static(table, g_in, R, pk, packet_capacity=bound)
        R.zero_()
        R_cpu = np.zeros(n, f32)
        for t in range(4):
            print(f"[no_alloc] graph replay {t}", flush=True)
            g_np = W.gradient(wl, 0, t, seed=31)
            g_in.copy_(torch.from_numpy(g_np))
            pk.fill_(POISON)
            graph.replay()
            torch.cuda.synchronize()
            want = oracle_lib.compress(table, g_np, R_cpu)
            got = pk.cpu().numpy()
            assert np.array_equal(got[:want.size], want), f"replay {t}: packet differs from the oracle"
            assert np.all(got[want.size:] == POISON)
            assert np.array_equal(R.cpu().numpy().view(np.uint32), R_cpu.view(np.uint32)), f"replay {t}: residue"
            A.adacomp_compress(table, g_in, R2, pk2, ws)
            torch.cuda.synchronize()
    finally:
        A.adacomp_workspace_release(ws)
