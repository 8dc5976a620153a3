"""GPU parity: libadacomp (HIP kernels, through the C ABI) against the CPU oracle, element by
element, on the five benchmark workloads and on edge cases.  Needs an MI355X."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import adacomp_workloads as W  # noqa: E402

f32 = np.float32
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_harness
    return gpu_harness


def _rand(seed, n, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(f32)


# ------------------------------------------------------------------------------------------------
# the five workloads
# ------------------------------------------------------------------------------------------------
def test_workload1_fc_all_steps(H, oracle_lib):
    wl = W.workload(1)
    stats = H.run_parity(oracle_lib, wl, wl.n_learners, wl.n_steps)
    per_bin = [s[2] / 794 for s in stats]
    assert 50 < per_bin[0] < 60 and per_bin[-1] < per_bin[0]   # more is sent while residues are small


def test_workload1_step_locked(H, oracle_lib):
    wl = W.workload(1)
    H.run_parity(oracle_lib, wl, 1, 3, step_locked=True)


def test_workload2_cifar_cnn_all_steps(H, oracle_lib):
    wl = W.workload(2)
    H.run_parity(oracle_lib, wl, wl.n_learners, wl.n_steps)


def test_workload4_char_lstm_single_calls(H, oracle_lib):
    wl = W.workload(4)
    H.run_parity(oracle_lib, wl, wl.n_learners, 3)   # 8 learners, one adacomp_compress call each, g_max compared


def test_workload4_as_configured(H, oracle_lib):
    """The char-LSTM table exactly as configured: 8 learners x 50 free-running steps through
    adacomp_compress_batch and adacomp_unpack_accumulate, in the launch configuration bench.py times
    (no g_max vector kept); every packet, residue and 8-packet sum of every step against the oracle."""
    wl = W.workload(4)
    assert (wl.n_learners, wl.n_steps) == (8, 50)
    H.run_parity(oracle_lib, wl, wl.n_learners, wl.n_steps, batch=True, check_gmax=False, threads=16, oracle_threads=8)


def test_workload2_long_run(H, oracle_lib):
    """Five times the configured number of steps, free-running: residues, packets and sums stay
    bit-equal to the oracle's (a single differing bit would feed back through the residue)."""
    wl = W.workload(2)
    H.run_parity(oracle_lib, wl, wl.n_learners, 100, batch=True, check_gmax=False)


def test_workload3_resnet50_full_size(H, oracle_lib):
    wl = W.workload(3)
    H.run_parity(oracle_lib, wl, 2, 3, check_gmax=True)                # full layer table, 2 learners x 3 steps


def test_workload5_speech_dnn_full_size(H, oracle_lib):
    """Full 125 M-element layer table in the launch configuration bench.py times: two learners,
    two free-running steps, every element compared; then a 16-packet unpack."""
    import gpu_harness as G
    import packet_format as pf
    wl = W.workload(5)
    table, n_total = wl.table(), wl.n_total
    mask = G.layer_mask(table, n_total)
    gpu = G.GpuSide(table, n_total, 2)
    R_cpu = [np.zeros(n_total, f32) for _ in range(2)]
    cpu_packets = []
    try:
        for t in range(2):
            cpu_packets = []
            for k in range(2):
                tag = f"speech_dnn step {t} learner {k}"
                G.say(tag)
                g = W.gradient(wl, k, t, threads=16)
                want = oracle_lib.compress(table, g, R_cpu[k])
                got = gpu.compress(k, g)
                G.compare_packet(got, want, gpu.capacity, tag)
                G.compare_residue(gpu.residue[k].cpu().numpy(), R_cpu[k], mask, 1.0, tag)
                cpu_packets.append(want)
        G.say("speech_dnn unpack of 16 (two distinct packets, repeated)")
        order = [k % 2 for k in range(16)]
        gpu.dense.fill_(float("nan"))
        import paper_1712_02679_amd as A
        A.adacomp_unpack_accumulate(table, [gpu.packets[k] for k in order], gpu.dense, gpu.ws)
        torch.cuda.synchronize()
        got = gpu.dense.cpu().numpy()
        want = oracle_lib.unpack_accumulate(table, [cpu_packets[k] for k in order], n_total)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    finally:
        gpu.close()


# ------------------------------------------------------------------------------------------------
# edge cases
# ------------------------------------------------------------------------------------------------
def test_worked_example_on_gpu(H, oracle_lib):
    vals = {}
    for line in open(os.path.join(GOLDEN, "worked_example_T4.txt")):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            vals[k] = v
    R0, dW = np.array(vals["residue"], f32), np.array(vals["dW"], f32)
    wl = W.custom("worked", [("l", 16, 4)])
    import gpu_harness as G
    import packet_format as pf
    gpu = G.GpuSide(wl.table(), 16, 1, keep_gmax=True)
    try:
        gpu.residue[0].copy_(torch.from_numpy(R0))
        buf = gpu.compress(0, dW)
        h, layers = pf.parse(buf[:int(pf.header(buf)["total_bytes"])])
        assert layers[0]["words"].tolist() == [int(v) for v in vals["words"]]
        assert layers[0]["counts"].tolist() == [int(v) for v in vals["counts"]]
        assert layers[0]["rec"]["scale"] == f32(vals["scale"][0])
        assert np.array_equal(gpu.residue[0].cpu().numpy(), np.array(vals["residue_new"], f32))
        assert np.array_equal(gpu.gmax(), np.array(vals["gmax"], f32))
        assert np.array_equal(gpu.unpack([0]), np.array(vals["decoded"], f32))
    finally:
        gpu.close()


EDGE_TABLES = {
    "LT1": [("a", 1003, 1)],
    "LT2_LT3": [("a", 4099, 2), ("b", 10001, 3)],
    "LT7_straddles_float4": [("a", 12345, 7)],
    "LT64_LT65_word_width": [("a", 64 * 130 + 5, 64), ("b", 65 * 130 + 5, 65)],
    "LT50_ragged_many_chunks": [("a", 50 * 64 * 9 + 17, 50)],
    "LT500_ragged": [("a", 500 * 131 + 216, 500)],
    "LT4096_LT4097": [("a", 3 * 4096 + 9, 4096), ("b", 3 * 4097 + 1, 4097)],
    "LT5000_LT8192": [("a", 5000 * 5 + 3, 5000), ("b", 8192 * 3, 8192)],
    "LT16384_and_odd_16383": [("a", 16384 * 3 + 5, 16384), ("b", 16383 * 2 + 7, 16383)],
    # bin lengths whose tiles start at every 4-byte position of a 16-byte slot: odd lengths below and above
    # 4096 (groups of four bins per tile / single unaligned bins), twice an odd number above 8192, and the
    # two lengths whose unaligned tiles do not fit their tile class with the misalignment added
    "odd_bin_lengths": [("a", 1025 * 13 + 3, 1025), ("b", 3001 * 9 + 2, 3001), ("c", 4097 * 9 + 5, 4097), ("d", 5001 * 7 + 1, 5001),
                        ("e", 8194 * 5 + 3, 8194), ("f", 16381 * 5 + 2, 16381), ("g", 16382 * 4 + 1, 16382), ("h", 16383 * 5, 16383)],
    "tiny_layers": [("a", 1, 500), ("b", 2, 50), ("c", 3, 1), ("d", 5, 16384), ("e", 63, 64)],
    "many_layers_300": [(f"l{i}", 1 + (i * 37) % 211, (1, 3, 50, 64, 65, 500)[i % 6]) for i in range(300)],
    "mixed_with_gaps": [("a", 4801, 50), ("b", 102402, 50), ("c", 786433, 500), ("d", 1923, 500), ("e", 777, 9)],
}


@pytest.mark.parametrize("name", sorted(EDGE_TABLES))
def test_edge_tables(H, oracle_lib, name):
    wl = W.custom(name, EDGE_TABLES[name], dist="normal_outliers")
    H.run_parity(oracle_lib, wl, 3, 4, seed=7, label=name)


@pytest.fixture
def three_launch_compress():
    """Small tables fold the scan into the placement kernel; this sends them down the path of the
    large ones (separate scan launch) for the duration of a test."""
    import paper_1712_02679_amd as A
    A.adacomp_tuning_fold_scan(False)
    yield
    A.adacomp_tuning_fold_scan(True)


@pytest.mark.parametrize("name", sorted(EDGE_TABLES))
def test_edge_tables_with_separate_scan_launch(H, oracle_lib, three_launch_compress, name):
    wl = W.custom(name, EDGE_TABLES[name], dist="normal_outliers")
    H.run_parity(oracle_lib, wl, 3, 3, seed=8, label=name + ", separate scan", batch=True)
    H.run_lazy_parity(oracle_lib, wl, 2, 3, 2, seed=8, label="lazy " + name + ", separate scan")


@pytest.fixture
def word_by_word_placement():
    """Tables with short bins and a separate scan launch correct the residue tile by tile in the
    placement kernel; this sends them down the word-by-word placement of the other tables."""
    import paper_1712_02679_amd as A
    A.adacomp_tuning_place_tiled(False)
    yield
    A.adacomp_tuning_place_tiled(True)


@pytest.mark.parametrize("name", sorted(EDGE_TABLES))
def test_edge_tables_with_word_by_word_placement(H, oracle_lib, three_launch_compress, word_by_word_placement, name):
    wl = W.custom(name, EDGE_TABLES[name], dist="normal_outliers")
    H.run_parity(oracle_lib, wl, 3, 3, seed=18, label=name + ", separate scan, word-by-word placement", batch=True)


def test_tiled_placement_alignment_and_density(H, oracle_lib, three_launch_compress):
    """The tile-by-tile placement on layers that start at every 16-byte position inside a 64-byte line,
    with ragged ends, dense and sparse tiles side by side (short and long bins in one table), all
    elements sent, and a truncated packet; single and batched calls, free-running against the oracle."""
    layers = [("a", 50 * 90 + 7, 50), ("b", 4 + 64 * 70, 64), ("c", 8 + 13 * 33 + 1, 13), ("d", 12 + 500 * 9, 500),
              ("e", 7 * 641 + 3, 7), ("f", 16384 + 5, 16384), ("g", 3 * 1500 + 2, 3), ("h", 1 * 4100, 1)]
    wl = W.custom("tiled_alignment", layers, dist="normal_outliers")
    H.run_parity(oracle_lib, wl, 3, 4, seed=21, batch=True)
    H.run_parity(oracle_lib, wl, 2, 3, seed=22)
    # every element sent (equal magnitudes): every line of every tile is rewritten
    n = wl.n_total
    same = lambda k, t: np.where((np.arange(n) + k + t) % 3 == 0, -0.5, 0.5).astype(f32)
    H.run_parity(oracle_lib, wl, 2, 2, grads=same, label="tiled_alignment all sent", batch=True)


def test_scan_paths_can_alternate(H, oracle_lib):
    """The folded and the separate scan leave the same state behind: calls on one workspace may
    alternate between them, also while lazy corrections wait."""
    import gpu_harness as G
    import paper_1712_02679_amd as A
    wl = W.custom("alternate", [("a", 50 * 300 + 7, 50), ("b", 500 * 70 + 11, 500), ("c", 9000, 4500)], dist="normal_outliers")
    table, n = wl.table(), wl.n_total
    mask = G.layer_mask(table, n)
    gpu = G.GpuSide(table, n, 2, batch=True)
    R_cpu = [np.zeros(n, f32) for _ in range(2)]
    try:
        for t in range(8):
            A.adacomp_tuning_fold_scan(t % 2 == 0)
            grads = [W.gradient(wl, k, t, seed=12) for k in range(2)]
            g_dev = [torch.from_numpy(x).to(G.DEV) for x in grads]
            lazy = t % 4 < 3                           # three lazy calls, then an eager one after a sync
            if lazy:
                A.adacomp_compress_batch_lazy(table, g_dev, gpu.residue, gpu.packets, gpu.ws, packet_capacity=gpu.capacity)
            else:
                A.adacomp_residue_sync(gpu.ws)
                A.adacomp_compress_batch(table, g_dev, gpu.residue, gpu.packets, gpu.ws, packet_capacity=gpu.capacity)
            torch.cuda.synchronize()
            for k in range(2):
                want = oracle_lib.compress(table, grads[k], R_cpu[k])
                assert np.array_equal(gpu.packets[k].cpu().numpy()[:want.size], want), f"step {t} learner {k}"
                if not lazy:
                    G.compare_residue(gpu.residue[k].cpu().numpy(), R_cpu[k], mask, 1.0, f"alternate step {t} learner {k}")
    finally:
        A.adacomp_tuning_fold_scan(True)
        gpu.close()


def test_layers_in_any_order_with_gaps(H, oracle_lib):
    """The layer table need not follow the buffer: layers listed out of address order, with large
    holes between them and in front of the first; nothing outside the layers is touched."""
    wl = W.custom_placed("scattered", [("c", 500 * 70 + 13, 500, 400000), ("a", 50 * 130 + 7, 50, 1024),
                                       ("d", 9000, 4500, 120000), ("b", 64 * 66 + 1, 64, 64000),
                                       ("e", 777, 9, 300000)], dist="normal_outliers")
    H.run_parity(oracle_lib, wl, 3, 3, seed=21, label="scattered layers")
    H.run_parity(oracle_lib, wl, 3, 2, seed=22, label="scattered layers, batched", batch=True)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_layer_tables(H, oracle_lib, seed):
    """Forty seeded random layer tables each (1-8 layers, bin lengths from 1 to 16384 with the
    awkward ones in between, layers from one element to 600 k, 1-33 learners, single or batched
    calls, unpack with and without runs of tiles), two free-running steps per table."""
    import paper_1712_02679_amd as A
    rng = np.random.default_rng(seed)
    lts = [1, 2, 3, 5, 7, 16, 49, 50, 63, 64, 65, 100, 255, 256, 257, 499, 500, 1000, 2048, 4095, 4096, 4097,
           5000, 8191, 8192, 12000, 16383, 16384]
    try:
        for case in range(40):
            layers = []
            for i in range(int(rng.integers(1, 9))):
                T = int(rng.choice(lts))
                kind = int(rng.integers(0, 4))
                if kind == 0:
                    n = int(rng.integers(1, 3 * T + 2))
                elif kind == 1:
                    n = int(T * rng.integers(1, 200) + rng.integers(0, T))
                elif kind == 2:
                    n = int(rng.integers(1, 300000))
                else:
                    n = int(T * 64 * rng.integers(1, 6) + rng.integers(0, 64 * T))
                layers.append((f"l{i}", max(1, min(n, 600000)), T))
            wl = W.custom(f"random{seed}_{case}", layers, dist=str(rng.choice(["normal", "normal_outliers", "laplace"])))
            n_learners = int(rng.choice([1, 2, 3, 5, 17, 33]))
            batch = bool(rng.integers(0, 2))
            A.adacomp_tuning_unpack_min_groups(1 if rng.integers(0, 2) else 0)
            H.run_parity(oracle_lib, wl, n_learners, 2, seed=int(rng.integers(0, 1000)), batch=batch, check_gmax=False,
                         label=f"random table {seed}/{case} {layers}")
    finally:
        A.adacomp_tuning_unpack_min_groups(0)


# ------------------------------------------------------------------------------------------------
# batched compress: several learners per launch
# ------------------------------------------------------------------------------------------------
def test_batch_workload2(H, oracle_lib):
    wl = W.workload(2)
    H.run_parity(oracle_lib, wl, wl.n_learners, 6, batch=True)


def test_batch_workload3_all_learners_all_steps(H, oracle_lib):
    """ResNet-50 table as configured: 8 learners, 10 free-running steps, one batched call per step."""
    wl = W.workload(3)
    H.run_parity(oracle_lib, wl, wl.n_learners, wl.n_steps, batch=True, check_gmax=False, threads=16)


@pytest.mark.parametrize("name", ["mixed_with_gaps", "LT16384_and_odd_16383", "tiny_layers", "LT64_LT65_word_width"])
def test_batch_edge_tables(H, oracle_lib, name):
    wl = W.custom(name, EDGE_TABLES[name], dist="normal_outliers")
    H.run_parity(oracle_lib, wl, 5, 3, seed=11, label="batch " + name, batch=True)


def test_batch_more_learners_than_one_launch_holds(H, oracle_lib):
    wl = W.custom("batch40", [("a", 50 * 40 + 7, 50), ("b", 500 * 12 + 11, 500)])
    H.run_parity(oracle_lib, wl, 40, 2, seed=3, batch=True, check_gmax=False)


def test_workload5_as_configured(H, oracle_lib):
    """The speech-DNN table exactly as configured and as bench.py times it: 16 learners of the
    125 M-element table, 10 free-running steps of adacomp_compress_batch (no g_max vector kept) with a
    16-packet adacomp_unpack_accumulate after each; every packet, residue and sum of every step against
    the oracle (one oracle call per learner and host thread)."""
    wl = W.workload(5)
    assert (wl.n_learners, wl.n_steps) == (16, 10)
    H.run_parity(oracle_lib, wl, wl.n_learners, wl.n_steps, batch=True, check_gmax=False, threads=16, oracle_threads=16)


def test_batch_workload5_full_size_sixteen_learners(H, oracle_lib):
    """The launch configuration bench.py times: 16 learners of the 125 M-element table in one
    adacomp_compress_batch call.  Learners 0 and 15 are compared with the oracle element by
    element; all 16 packets must equal what 16 single adacomp_compress calls produce."""
    import gpu_harness as G
    import paper_1712_02679_amd as A
    wl = W.workload(5)
    table, n_total = wl.table(), wl.n_total
    mask = G.layer_mask(table, n_total)
    n = 16
    gpu = G.GpuSide(table, n_total, n, batch=True)
    try:
        grads = [torch.from_numpy(W.gradient(wl, k, 0, threads=16)).to(G.DEV) for k in range(n)]
        for p in gpu.packets:
            p.fill_(G.POISON)
        A.adacomp_compress_batch(table, grads, gpu.residue, gpu.packets, gpu.ws)
        torch.cuda.synchronize()
        for k in (0, 15):
            G.say(f"speech_dnn batch learner {k} vs oracle")
            R = np.zeros(n_total, f32)
            want = oracle_lib.compress(table, grads[k].cpu().numpy(), R)
            G.compare_packet(gpu.packets[k].cpu().numpy(), want, gpu.capacity, f"batch learner {k}")
            G.compare_residue(gpu.residue[k].cpu().numpy(), R, mask, 1.0, f"batch learner {k}")
        single = G.GpuSide(table, n_total, 1)
        try:
            for k in range(n):
                G.say(f"speech_dnn batch learner {k} vs single call")
                single.residue[0].zero_()
                single.packets[0].fill_(G.POISON)
                A.adacomp_compress(table, grads[k], single.residue[0], single.packets[0], single.ws)
                torch.cuda.synchronize()
                assert torch.equal(single.packets[0], gpu.packets[k]), k
                assert torch.equal(single.residue[0].view(torch.int32), gpu.residue[k].view(torch.int32)), k
        finally:
            single.close()
    finally:
        gpu.close()


# ------------------------------------------------------------------------------------------------
# the paper's own stress-test bin lengths on the CIFAR10-CNN table
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("conv_lt,fc_lt", [(800, 8000), (5000, 5000)])
def test_paper_stress_bin_lengths(H, oracle_lib, conv_lt, fc_lt):
    """Fig. 2(a): L_T = 800 for convolutional and 8000 for fully connected layers; section
    "Robustness of the AdaComp Technique": L_T = 5000 everywhere.  4 learners x 5 free-running steps."""
    wl = W.with_bin_lengths(W.workload(2), conv_lt, fc_lt)
    H.run_parity(oracle_lib, wl, 4, 5, batch=True)


@pytest.mark.parametrize("lt", [200, 300])
def test_paper_local_selection_bin_lengths(H, oracle_lib, lt):
    """Section "Robustness of the AdaComp Technique": local selection (bin maxima only) at the bin
    lengths of its ablation, 200 and 300, 4 learners x 5 free-running steps."""
    wl = W.with_bin_lengths(W.workload(2), lt, lt)
    H.run_parity(oracle_lib, wl, 4, 5, batch=True, rule=2)


# ------------------------------------------------------------------------------------------------
# selection variants: the printed compare alone, local selection, other soft-threshold factors
# ------------------------------------------------------------------------------------------------
# ------------------------------------------------------------------------------------------------
# lazy residue: the corrections of a call are applied by the next call, or by adacomp_residue_sync
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("sync_every", [0, 1, 3])
def test_lazy_workload2(H, oracle_lib, sync_every):
    wl = W.workload(2)
    H.run_lazy_parity(oracle_lib, wl, wl.n_learners, 7, sync_every)


@pytest.mark.parametrize("name", sorted(EDGE_TABLES))
def test_lazy_edge_tables(H, oracle_lib, name):
    wl = W.custom(name, EDGE_TABLES[name], dist="normal_outliers")
    H.run_lazy_parity(oracle_lib, wl, 3, 5, 2, seed=17, label="lazy " + name)


def test_lazy_more_learners_than_one_launch_holds(H, oracle_lib):
    wl = W.custom("lazy40", [("a", 50 * 40 + 7, 50), ("b", 500 * 12 + 11, 500)])
    H.run_lazy_parity(oracle_lib, wl, 40, 3, 0, seed=3)


def test_lazy_workload3_and_workload5(H, oracle_lib):
    """The two large tables (short bins with both tile classes; the table bench.py times, with one
    streaming launch per learner), four free-running lazy steps with a sync in the middle."""
    wl = W.workload(3)
    H.run_lazy_parity(oracle_lib, wl, 4, 4, 2, threads=16, oracle_threads=4)
    wl = W.workload(5)
    H.run_lazy_parity(oracle_lib, wl, 4, 4, 2, threads=16, oracle_threads=4)


def test_lazy_bookkeeping(H, oracle_lib):
    """While corrections wait, every compress call but the lazy one with the same residue buffers is
    refused and enqueues nothing; a sync with nothing waiting does nothing; after the sync the eager
    calls go on from the same residue the eager calls alone would have reached."""
    import gpu_harness as G
    import paper_1712_02679_amd as A
    wl = W.custom("lazy_books", [("a", 50 * 300 + 7, 50), ("b", 500 * 70 + 11, 500)])
    table, n = wl.table(), wl.n_total
    mask = G.layer_mask(table, n)
    lazy, eager = G.GpuSide(table, n, 2, batch=True), G.GpuSide(table, n, 2, batch=True)
    try:
        A.adacomp_residue_sync(lazy.ws)                       # nothing waits: no-op
        other = [torch.zeros_like(r) for r in lazy.residue]
        for t in range(4):
            g = [torch.from_numpy(W.gradient(wl, k, t, seed=5)).to(G.DEV) for k in range(2)]
            A.adacomp_compress_batch_lazy(table, g, lazy.residue, lazy.packets, lazy.ws)
            A.adacomp_compress_batch(table, g, eager.residue, eager.packets, eager.ws)
            torch.cuda.synchronize()
            before = [r.clone() for r in lazy.residue], [p.clone() for p in lazy.packets]
            for call in (lambda: A.adacomp_compress_batch(table, g, lazy.residue, lazy.packets, lazy.ws),
                         lambda: A.adacomp_compress(table, g[0], lazy.residue[0], lazy.packets[0], lazy.ws),
                         lambda: A.adacomp_compress_variant(table, g, lazy.residue, lazy.packets, lazy.ws, rule=1),
                         lambda: A.adacomp_compress_batch_lazy(table, g, other, lazy.packets, lazy.ws),
                         lambda: A.adacomp_compress_batch_lazy(table, g, lazy.residue[::-1], lazy.packets, lazy.ws),
                         lambda: A.adacomp_compress_batch_lazy(table, g[:1], lazy.residue[:1], lazy.packets[:1], lazy.ws)):
                with pytest.raises(A.AdacompError) as e:
                    call()
                assert e.value.code == A.binding.EPENDING
            torch.cuda.synchronize()
            for k in range(2):
                assert torch.equal(before[0][k], lazy.residue[k]) and torch.equal(before[1][k], lazy.packets[k])
                assert torch.equal(lazy.packets[k], eager.packets[k]), f"step {t} learner {k}"
        A.adacomp_residue_sync(lazy.ws)
        A.adacomp_residue_sync(lazy.ws)                       # twice: the second finds nothing
        torch.cuda.synchronize()
        for k in range(2):
            assert torch.equal(lazy.residue[k], eager.residue[k])
        g = [torch.from_numpy(W.gradient(wl, k, 9, seed=5)).to(G.DEV) for k in range(2)]
        A.adacomp_compress_batch(table, g, lazy.residue, lazy.packets, lazy.ws)   # accepted again
        A.adacomp_compress_batch(table, g, eager.residue, eager.packets, eager.ws)
        torch.cuda.synchronize()
        for k in range(2):
            assert torch.equal(lazy.residue[k], eager.residue[k]) and torch.equal(lazy.packets[k], eager.packets[k])
        assert mask.any()
    finally:
        lazy.close()
        eager.close()


def test_variant_workload5_eight_learners(H, oracle_lib):
    """The selection variants at the size and learner count where the streaming kernel is launched
    once per learner with fewer workgroups resident per compute unit: 8 learners of the 125 M-element
    table, one step, soft-threshold factor 2.5, every packet, residue and the sum against the oracle."""
    wl = W.workload(5)
    stats = H.run_parity(oracle_lib, wl, 8, 1, batch=True, rule=0, soft_factor=2.5, check_gmax=False,
                         threads=16, oracle_threads=8, label="variant factor 2.5 at full size")
    assert all(s[2] > 0 for s in stats)


@pytest.mark.parametrize("rule,factor", [(1, 2.0), (2, 2.0), (0, 1.5), (0, 3.0), (0, 1.0), (1, 2.5), (0, 2.75)])
def test_variants_workload2(H, oracle_lib, rule, factor):
    wl = W.workload(2)
    stats = H.run_parity(oracle_lib, wl, 2, 5, batch=True, rule=rule, soft_factor=factor,
                         label=f"variant rule {rule} factor {factor}")
    assert all(s[2] > 0 for s in stats)


@pytest.mark.parametrize("rule,factor", [(1, 2.0), (2, 2.0), (0, 1.5)])
def test_variants_edge_tables_with_zeros(H, oracle_lib, rule, factor):
    """Zero stretches and ties: the printed compare sends the zeros of an all-zero bin."""
    wl = W.custom("varz", [("a", 50 * 90 + 11, 50), ("b", 500 * 21 + 3, 500), ("c", 64 * 3 + 1, 64), ("d", 5000, 4097)])
    n = wl.n_total

    def grads(k, t):
        g = np.round(_rand(300 * k + t, n) * 2).astype(f32) / 4
        g[(np.arange(n) // 700) % 3 == 0] = 0
        return g
    H.run_parity(oracle_lib, wl, 2, 4, grads=grads, batch=True, rule=rule, soft_factor=factor, label="variant zeros")


def test_variant_default_equals_compress(H):
    """rule 0 with factor 2 through the variant entry point is adacomp_compress bit for bit, and bad
    rules / factors are refused."""
    import gpu_harness as G
    import paper_1712_02679_amd as A
    wl = W.workload(1)
    table, n = wl.table(), wl.n_total
    a, b = G.GpuSide(table, n, 1), G.GpuSide(table, n, 1, batch=True)
    try:
        for t in range(3):
            g = W.gradient(wl, 0, t)
            pa = a.compress(0, g)
            gt = torch.from_numpy(g).to(G.DEV)
            b.packets[0].fill_(G.POISON)
            A.adacomp_compress_variant(table, [gt], b.residue, b.packets, b.ws, rule=0, soft_factor=2.0)
            torch.cuda.synchronize()
            assert np.array_equal(pa, b.packets[0].cpu().numpy())
            assert torch.equal(a.residue[0], b.residue[0])
        for rule, factor in [(3, 2.0), (0, 0.5), (0, 17.0), (0, float("nan"))]:
            with pytest.raises(A.AdacompError) as e:
                A.adacomp_compress_variant(table, [gt], b.residue, b.packets, b.ws, rule=rule, soft_factor=factor)
            assert e.value.code == -1
    finally:
        a.close()
        b.close()


# ------------------------------------------------------------------------------------------------
# unpack + average + optimizer step in one pass
# ------------------------------------------------------------------------------------------------
def _update_case(oracle_lib, wl, n_learners, n_steps, kind, with_dense, seed=0, threads=1, grads_fn=None):
    import gpu_harness as G
    import paper_1712_02679_amd as A
    table, n = wl.table(), wl.n_total
    mask = G.layer_mask(table, n)
    gpu = G.GpuSide(table, n, n_learners, batch=True)
    rng = np.random.default_rng(seed)
    w_cpu = rng.standard_normal(n).astype(f32)
    s1_cpu = np.zeros(n, f32)
    s2_cpu = np.zeros(n, f32)
    w_gpu, s1_gpu, s2_gpu = (torch.from_numpy(x.copy()).to(G.DEV) for x in (w_cpu, s1_cpu, s2_cpu))
    R_cpu = [np.zeros(n, f32) for _ in range(n_learners)]
    lr, mu, b1, b2, eps = 0.05, 0.9, 0.9, 0.999, 1e-8
    try:
        for t in range(n_steps):
            G.say(f"{wl.name} update kind {kind} step {t}")
            grads = [grads_fn(k, t) if grads_fn else W.gradient(wl, k, t, seed=seed, threads=threads) for k in range(n_learners)]
            gpu.compress_batch(grads)
            if threads > 1:  # learners are independent: one oracle call per host thread
                from concurrent.futures import ThreadPoolExecutor
                with ThreadPoolExecutor(min(threads, n_learners)) as pool:
                    pk_cpu = list(pool.map(lambda k: oracle_lib.compress(table, grads[k], R_cpu[k]), range(n_learners)))
            else:
                pk_cpu = [oracle_lib.compress(table, grads[k], R_cpu[k]) for k in range(n_learners)]
            dense_cpu = oracle_lib.unpack_accumulate(table, pk_cpu, n)
            dense_cpu[~mask] = 0
            bias1, bias2 = float(f32(1 - b1 ** (t + 1))), float(f32(1 - b2 ** (t + 1)))
            if kind == 1:
                oracle_lib.update_sgd(table, dense_cpu, n_learners, w_cpu, s1_cpu, lr, mu)
            else:
                oracle_lib.update_adam(table, dense_cpu, n_learners, w_cpu, s1_cpu, s2_cpu, lr, b1, b2, eps, bias1, bias2)
            gpu.dense.fill_(float("nan"))
            A.adacomp_unpack_update(table, gpu.packets, gpu.dense if with_dense else None, w_gpu, s1_gpu,
                                    s2_gpu if kind == 2 else None, gpu.ws, kind, lr, momentum=mu, beta1=b1,
                                    beta2=b2, eps=eps, bias1=bias1, bias2=bias2)
            torch.cuda.synchronize()
            for name, got, want in (("weights", w_gpu, w_cpu), ("state1", s1_gpu, s1_cpu), ("state2", s2_gpu, s2_cpu)):
                got = got.cpu().numpy()
                assert np.array_equal(got[~mask], want[~mask]), f"{name}: touched outside the layers"
                if not np.array_equal(got[mask].view(np.uint32), want[mask].view(np.uint32)):
                    rel = np.abs(got[mask].astype(np.float64) - want[mask]) / np.maximum(np.abs(want[mask]), 1e-30)
                    raise AssertionError(f"{name} step {t}: not bit-equal, max relative difference {rel.max():.3e}")
            if with_dense:
                got = gpu.dense.cpu().numpy()
                assert np.array_equal(got[mask].view(np.uint32), dense_cpu[mask].view(np.uint32))
                assert np.isnan(got[~mask]).all()
    finally:
        gpu.close()


@pytest.mark.parametrize("kind,with_dense", [(1, False), (1, True), (2, False), (2, True)])
def test_unpack_update_workload2(H, oracle_lib, kind, with_dense):
    _update_case(oracle_lib, W.workload(2), 4, 6, kind, with_dense)


def test_unpack_update_full_size_tables(H, oracle_lib):
    """The launch configurations bench.py times: Adam on the 125 M-element table with 16 packets
    (single tiles, 16-bit kernel) and SGD on the ResNet-50 table with 8 packets (one launch per
    word width), each one step from zero residues, every element against the oracle."""
    _update_case(oracle_lib, W.workload(5), 16, 1, 2, False, threads=16)
    _update_case(oracle_lib, W.workload(3), 8, 1, 1, True, threads=16)


@pytest.mark.parametrize("kind", [1, 2])
def test_unpack_update_edge_table(H, oracle_lib, kind):
    wl = W.custom("upd_edge", EDGE_TABLES["mixed_with_gaps"] + [("z", 16383 * 2 + 7, 16383)], dist="normal_outliers")
    _update_case(oracle_lib, wl, 3, 3, kind, False, seed=5)


@pytest.mark.parametrize("kind,with_dense", [(1, False), (1, True), (2, True)])
def test_unpack_update_odd_bin_lengths(H, oracle_lib, kind, with_dense):
    """The optimizer epilogue on tiles that start at every 4-byte position of a 16-byte slot."""
    wl = W.custom("upd_odd", EDGE_TABLES["odd_bin_lengths"], dist="normal_outliers")
    _update_case(oracle_lib, wl, 3, 2, kind, with_dense, seed=15)


def test_unpack_update_many_learners_and_errors(H, oracle_lib):
    """70 learners: two launches, the step is applied once by the last; dense_out is then required."""
    import gpu_harness as G
    import paper_1712_02679_amd as A
    wl = W.custom("upd70", [("a", 50 * 40 + 7, 50), ("b", 500 * 12 + 11, 500)])
    _update_case(oracle_lib, wl, 70, 2, 1, True, seed=2)
    table, n = wl.table(), wl.n_total
    gpu = G.GpuSide(table, n, 70, batch=True)
    try:
        w = torch.zeros(n, device=G.DEV)
        s1 = torch.zeros(n, device=G.DEV)
        with pytest.raises(A.AdacompError) as e:      # no dense_out with more than 64 learners
            A.adacomp_unpack_update(table, gpu.packets, None, w, s1, None, gpu.ws, 1, 0.1, momentum=0.9)
        assert e.value.code == -1
        with pytest.raises(A.AdacompError):           # Adam without its second state
            A.adacomp_unpack_update(table, gpu.packets[:2], None, w, s1, None, gpu.ws, 2, 0.1)
        with pytest.raises(A.AdacompError):           # unknown optimizer
            A.adacomp_unpack_update(table, gpu.packets[:2], None, w, s1, None, gpu.ws, 3, 0.1)
        with pytest.raises(A.AdacompError):           # aliasing state
            A.adacomp_unpack_update(table, gpu.packets[:2], None, w, w, None, gpu.ws, 1, 0.1)
    finally:
        gpu.close()


# ------------------------------------------------------------------------------------------------
# unpack with runs of tiles per workgroup (large tables do this by default; here the threshold is
# lowered so that every small table does, including the shortened runs at the end of the table)
# ------------------------------------------------------------------------------------------------
@pytest.fixture
def grouped_unpack_tiles():
    import paper_1712_02679_amd as A
    A.adacomp_tuning_unpack_min_groups(1)
    yield
    A.adacomp_tuning_unpack_min_groups(0)


GROUPED_TABLES = dict(EDGE_TABLES)
GROUPED_TABLES["LT500_many_tiles"] = [("a", 500 * 64 * 40 + 333, 500), ("b", 3000 * 64 * 3 + 5, 3000)]
GROUPED_TABLES["LT16384_many_slices"] = [("a", 16384 * 30 + 4100, 16384), ("b", 4097 * 70, 4097)]


@pytest.mark.parametrize("name", sorted(GROUPED_TABLES))
def test_grouped_unpack_tables(H, oracle_lib, grouped_unpack_tiles, name):
    wl = W.custom(name, GROUPED_TABLES[name], dist="normal_outliers")
    H.run_parity(oracle_lib, wl, 3, 2, seed=17, label="grouped unpack " + name, batch=True, check_gmax=False)


def test_grouped_unpack_many_learners(H, oracle_lib, grouped_unpack_tiles):
    """More than 16 learners (the tables are rebuilt per tile) and more than 64 (a second launch
    that accumulates)."""
    wl = W.custom("grp70", [("a", 50 * 200 + 7, 50), ("b", 500 * 150 + 11, 500), ("c", 9000 * 3 + 1, 9000)])
    H.run_parity(oracle_lib, wl, 20, 2, seed=4, batch=True, check_gmax=False)
    H.run_parity(oracle_lib, wl, 70, 1, seed=5, batch=True, check_gmax=False)


@pytest.mark.parametrize("kind", [1, 2])
def test_grouped_unpack_update(H, oracle_lib, grouped_unpack_tiles, kind):
    wl = W.custom("grp_upd", GROUPED_TABLES["LT500_many_tiles"] + [("z", 16383 * 2 + 7, 16383), ("y", 777, 9)], dist="normal_outliers")
    _update_case(oracle_lib, wl, 3, 2, kind, True, seed=6)
    _update_case(oracle_lib, wl, 18, 1, kind, False, seed=7)


@pytest.mark.parametrize("fold", [True, False])
def test_scale_when_the_float64_sum_of_gmax_is_not_exact(H, oracle_lib, fold):
    """The layer scale is a float64 sum of float32 values, taken bin after bin by the oracle and in a
    tree by the kernels (per tile, then over tiles: by k_scan, or inside the placement kernel for small
    tables).  The orders agree bit for bit while the sum is exact in float64; here it is not: the
    g_max values of a layer span 45 binary orders of magnitude over 20 000 bins.  The stated bar
    then applies: every index, sign, count and the layout bit-equal, each scale within 1e-6 relative,
    the residue within 1e-6 max(|G|, scale).  Both scan paths are run; how many scales were bit-equal
    is printed."""
    import gpu_harness as G
    import packet_format as pf
    import paper_1712_02679_amd as A
    T1, nb1, T2, nb2 = 50, 20000, 500, 900
    layers = [("wide50", T1 * nb1, T1), ("wide500", T2 * nb2 + 123, T2)]
    wl = W.custom("wide_gmax", layers)
    table, n = wl.table(), wl.n_total
    mask = G.layer_mask(table, n)
    rng = np.random.default_rng(4242)
    g = rng.standard_normal(n).astype(f32)
    for off, cnt, T in table:   # one magnitude per bin, log-uniform over 2^-40 .. 2^5
        nb = -(-cnt // T)
        mag = np.exp2(rng.uniform(-40.0, 5.0, nb)).astype(f32)
        g[off:off + cnt] *= np.repeat(mag, T)[:cnt]
    A.adacomp_tuning_fold_scan(fold)
    gpu = G.GpuSide(table, n, 1, batch=True)
    try:
        R_cpu = np.zeros(n, f32)
        want = oracle_lib.compress(table, g, R_cpu)
        got = gpu.compress_batch([g])[0]
        exact = G.compare_packet(got, want, gpu.capacity, "wide g_max", strict=False)
        h, recs = pf.parse(want, check=False)
        scale_hint = max(float(r["rec"]["scale"]) for r in recs)
        same_r = G.compare_residue(gpu.residue[0].cpu().numpy(), R_cpu, mask, scale_hint, "wide g_max", strict=False)
        gh, grecs = pf.parse(got[:want.size], check=False)
        eq = sum(float(a["rec"]["scale"]) == float(b["rec"]["scale"]) for a, b in zip(grecs, recs))
        print(f"wide g_max, fold={fold}: {eq} of {len(recs)} scales bit-equal to the oracle's, packet exact={exact}, residue exact={same_r}")
        # the float64 sum really is inexact here: summing the oracle's own g_max values in another
        # order changes the float64 result for at least one layer
        inexact = 0
        for off, cnt, T in table:
            G0 = g[off:off + cnt]
            gm = np.abs(np.pad(G0, (0, (-cnt) % T))).reshape(-1, T).max(axis=1).astype(np.float64)
            fwd, rev = 0.0, 0.0
            for v in gm:
                fwd += v
            for v in gm[::-1]:
                rev += v
            inexact += fwd != rev
        assert inexact >= 1
    finally:
        gpu.close()
        A.adacomp_tuning_fold_scan(True)


def test_ties_and_zeros(H, oracle_lib):
    """Coarse dyadic grid: many equal magnitudes, exact cancellations to +-0, all-zero bins."""
    wl = W.custom("ties", [("a", 50 * 300 + 11, 50), ("b", 500 * 40 + 3, 500)])
    n = wl.n_total

    def grads(k, t):
        g = np.round(_rand(100 * k + t, n) * 2).astype(f32) / 4
        g[(np.arange(n) // 1000) % 3 == 0] = 0          # whole zero stretches
        if t == 2:
            g = -grads(k, 1) - grads(k, 0) + f32(0.0)  # pushes many G to exact zero
        return g.astype(f32)
    H.run_parity(oracle_lib, wl, 2, 4, grads=grads, label="ties")


def _subnormal_case():
    """Layers whose values are all subnormal, a layer that mixes subnormal and ordinary values, and
    a layer of very large ones."""
    wl = W.custom("subnormal", [("a", 50 * 90 + 7, 50), ("b", 500 * 30 + 11, 500), ("c", 64 * 40, 64), ("d", 500 * 20, 500)])
    n = wl.n_total
    lay = wl.layers
    tiny = float(np.finfo(f32).tiny)

    def grads(k, t):
        g = _rand(1000 * k + t, n)
        out = np.zeros(n, f32)
        a, b, c, d = (slice(l.elem_offset, l.elem_offset + l.n_elems) for l in lay)
        out[a] = (g[a].astype(np.float64) * tiny * 2.0 ** -8).astype(f32)    # all subnormal
        out[b] = (g[b].astype(np.float64) * tiny * 2.0 ** -3).astype(f32)    # subnormal, a few reach the normal range
        mixed = g[c].copy()
        mixed[::3] = (mixed[::3].astype(np.float64) * tiny * 0.01).astype(f32)
        out[c] = mixed
        out[d] = g[d] * f32(1e30)
        return out
    g0 = grads(0, 0)
    assert np.count_nonzero((np.abs(g0) < tiny) & (g0 != 0)) > 10000    # the inputs really are subnormal
    return wl, grads


def test_subnormal_and_large_magnitudes(H, oracle_lib):
    """Nothing on the path flushes subnormal numbers (G, g_max, the scale, the residue, the adds of the
    unpacked sum, the optimizer steps), and magnitudes up to 1e30 pass through unharmed."""
    wl, grads = _subnormal_case()
    H.run_parity(oracle_lib, wl, 5, 4, grads=grads, label="subnormal")
    H.run_parity(oracle_lib, wl, 20, 2, grads=grads, label="subnormal, batched", batch=True, check_gmax=False)
    _update_case(oracle_lib, wl, 3, 2, 1, True, grads_fn=grads)
    _update_case(oracle_lib, wl, 3, 2, 2, False, grads_fn=grads)


@pytest.mark.parametrize("fold", [True, False])
def test_non_finite_inputs_are_memory_safe(H, fold):
    """NaN and infinities are outside the method (the results are unspecified), but the calls stay
    inside their buffers: the packet is a well-formed container no longer than the bound, nothing is
    written behind it or outside the layers, and the packet can be unpacked.  With the folded scan and
    with the separate scan launch (tile-by-tile placement for this table's short bins)."""
    import gpu_harness as G
    import packet_format as pf
    import paper_1712_02679_amd as A
    A.adacomp_tuning_fold_scan(fold)
    try:
        _non_finite_case(G, pf)
    finally:
        A.adacomp_tuning_fold_scan(True)


def _non_finite_case(G, pf):
    wl = W.custom("nonfinite", [("a", 50 * 90 + 7, 50), ("b", 500 * 20 + 11, 500), ("c", 16384 + 9, 16384)], dist="normal_outliers")
    table, n = wl.table(), wl.n_total
    mask = G.layer_mask(table, n)
    gpu = G.GpuSide(table, n, 1)
    try:
        rng = np.random.default_rng(404)
        for t in range(3):
            g = W.gradient(wl, 0, t, seed=404)
            bad = rng.choice(n, 400, replace=False)
            g[bad[:150]] = np.nan
            g[bad[150:275]] = np.inf
            g[bad[275:]] = -np.inf
            buf = gpu.compress(0, g)
            h = pf.header(buf)
            total = int(h["total_bytes"])
            assert int(h["status"]) == 0 and total <= gpu.bound
            assert np.all(buf[total:] == G.POISON)
            pf.parse(buf[:total])                     # every structural invariant of the container
            assert np.all(gpu.residue[0].cpu().numpy()[~mask] == 0)
            dense = gpu.unpack([0])
            assert np.isnan(dense[~mask]).all()
    finally:
        gpu.close()


def test_all_zero_and_all_selected(H, oracle_lib):
    wl = W.custom("extremes", [("a", 50 * 70, 50), ("b", 500 * 9 + 100, 500)])
    n = wl.n_total

    def grads(k, t):
        if t == 0:
            return np.zeros(n, f32)                      # nothing to send, scale 0
        sign = np.where(np.random.default_rng(t).random(n) < 0.5, -1, 1).astype(f32)
        return sign * f32(0.125)                         # every element is a bin maximum: all sent
    stats = H.run_parity(oracle_lib, wl, 1, 2, grads=grads, label="extremes")
    assert stats[0][2] == 0 and stats[1][2] == wl.n_params
    import paper_1712_02679_amd as A
    assert stats[1][3] == A.adacomp_packet_bound(wl.table())


@pytest.mark.parametrize("batch", [False, True])
def test_all_selected_every_bin_length(H, oracle_lib, batch):
    """Every element sent, for every kind of tile and word: bins of 1, 7, 64 (8-bit words, up to 64
    words per bin), 65, 500, 4096 (a tile per bin), 4097 and 16384 (bins cut into slices on unpack,
    thousands of words per bin), with three learners whose signs differ, so that the unpacked sum
    meets every address three times."""
    import paper_1712_02679_amd as A
    wl = W.custom("all_sent", [("a", 1000, 1), ("b", 7 * 300 + 3, 7), ("c", 64 * 70, 64), ("d", 65 * 70 + 1, 65),
                               ("e", 500 * 20 + 250, 500), ("f", 4096 * 3, 4096), ("g", 4097 * 2 + 5, 4097),
                               ("h", 16384 * 2 + 100, 16384)])
    n = wl.n_total

    def grads(k, t):
        sign = np.where(np.random.default_rng(10 * k + t).random(n) < 0.5, -1, 1).astype(f32)
        return sign * f32(0.25)
    stats = H.run_parity(oracle_lib, wl, 3, 2, grads=grads, label="all sent", batch=batch, check_gmax=False)
    assert all(st[2] == wl.n_params for st in stats)                       # every element, every learner and step
    assert stats[0][3] == A.adacomp_packet_bound(wl.table())


@pytest.mark.parametrize("fold", [True, False])
def test_truncated_packet(H, oracle_lib, fold):
    """Capacity below the need: status = truncated, total_bytes = the need, the words that fit are
    the oracle's, nothing is written past the capacity, residue updated as if all had been sent.
    With the folded scan (word-by-word placement) and with the separate scan launch, where this
    table's short bins take the tile-by-tile placement."""
    import gpu_harness as G
    import packet_format as pf
    import paper_1712_02679_amd as A
    A.adacomp_tuning_fold_scan(fold)
    try:
        _truncated_packet_case(oracle_lib, G, pf, A)
    finally:
        A.adacomp_tuning_fold_scan(True)


def _truncated_packet_case(oracle_lib, G, pf, A):
    wl = W.custom("trunc", [("a", 50 * 200, 50), ("b", 500 * 100, 500)])
    table, n = wl.table(), wl.n_total
    g = W.gradient(wl, 0, 0)
    R = np.zeros(n, f32)
    want = oracle_lib.compress(table, g, R)
    fixed = A.adacomp_packet_fixed_bytes(table)
    cap = fixed + (want.size - fixed) // 2 // 16 * 16 + 6
    gpu = G.GpuSide(table, n, 1, capacity=cap)
    try:
        buf = gpu.compress(0, g)
        h = pf.header(buf)
        assert h["status"] == 1 and h["total_bytes"] == want.size
        assert np.all(buf[cap:] == G.POISON)
        same = buf[:cap] == want[:cap]
        same[8:12] = True                                 # the status word itself
        assert np.all(same)
        assert np.array_equal(gpu.residue[0].cpu().numpy(), R)
        # a truncated packet contributes nothing to unpack
        assert np.all(gpu.unpack([0]) == 0)
    finally:
        gpu.close()
    with pytest.raises(A.AdacompError) as e:
        G.GpuSide(table, n, 1, capacity=fixed - 16).compress(0, g)
    assert e.value.code == -4


@pytest.mark.parametrize("T", [50, 500])
def test_unpack_bins_past_total_bytes_contribute_nothing(H, oracle_lib, T):
    """A packet whose chunk offset points past its own total_bytes: the bins of that chunk are
    dropped for that learner, everything else is summed as usual, and no word is read from beyond
    total_bytes (the altered offset still points inside the allocated buffer, which is as long as
    the packet bound, so this holds whatever the kernel does)."""
    import gpu_harness as G
    import packet_format as pf
    wl = W.custom("past_end", [("a", T * 64 * 3 + 7, T)])
    table, n = wl.table(), wl.n_total
    gpu = G.GpuSide(table, n, 3)
    try:
        cpu_packets = []
        for k in range(3):
            g = W.gradient(wl, k, 0)
            cpu_packets.append(oracle_lib.compress(table, g, np.zeros(n, f32)))
            gpu.compress(k, g)
        h, layers = pf.parse(cpu_packets[1])
        word_bytes = int(layers[0]["rec"]["word_bits"]) // 8
        cho = int(layers[0]["rec"]["chunks_offset"])
        past = int(h["total_bytes"]) // word_bytes + 1000              # in words, counted from the layer's first word
        assert (int(layers[0]["rec"]["words_offset"]) + (past + 64 * T) * word_bytes) < gpu.capacity
        altered = torch.tensor(np.array([past], "<u4").view(np.uint8), device=G.DEV)
        gpu.packets[1][cho + 4:cho + 8] = altered                      # chunk 1 of learner 1
        got = gpu.unpack([0, 1, 2])
        want = oracle_lib.unpack_accumulate(table, cpu_packets, n)
        without = oracle_lib.unpack_accumulate(table, [cpu_packets[0], cpu_packets[2]], n)
        lo, hi = 64 * T, 128 * T
        want[lo:hi] = without[lo:hi]
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    finally:
        gpu.close()


def test_many_learners(H, oracle_lib):
    """0, 1, 17 and 70 learners: empty sum, learner groups of 16 in LDS, more than one launch of 64."""
    import gpu_harness as G
    wl = W.custom("many", [("a", 50 * 100 + 7, 50), ("b", 500 * 30 + 11, 500)])
    table, n = wl.table(), wl.n_total
    mask = G.layer_mask(table, n)
    gpu = G.GpuSide(table, n, 70)
    cpu_packets = []
    try:
        for k in range(70):
            g = _rand(k, n, 10.0 ** ((k % 7) - 3))
            cpu_packets.append(oracle_lib.compress(table, g, np.zeros(n, f32)))
            gpu.compress(k, g)
        for count in (0, 1, 17, 64, 70):
            G.say(f"many learners: {count}")
            got = gpu.unpack(list(range(count)))
            want = oracle_lib.unpack_accumulate(table, cpu_packets[:count], n)
            assert np.array_equal(got[mask].view(np.uint32), want[mask].view(np.uint32)), count
    finally:
        gpu.close()


def test_deterministic_reruns(H):
    """Same inputs twice give byte-identical packets, residues and dense sums (no atomics on floats,
    integer scans only)."""
    import gpu_harness as G
    wl = W.workload(2)
    table, n = wl.table(), wl.n_total
    outs = []
    for rep in range(2):
        gpu = G.GpuSide(table, n, 2)
        try:
            bufs = []
            for t in range(3):
                for k in range(2):
                    bufs.append(gpu.compress(k, W.gradient(wl, k, t)).copy())
            outs.append((bufs, [r.cpu().numpy() for r in gpu.residue], gpu.unpack([0, 1])))
        finally:
            gpu.close()
    for a, b in zip(outs[0][0], outs[1][0]):
        assert np.array_equal(a, b)
    for a, b in zip(outs[0][1], outs[1][1]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(outs[0][2].view(np.uint32), outs[1][2].view(np.uint32))


def test_hip_graph_capture_and_replay(H, oracle_lib):
    """compress_batch + unpack only launch kernels on the caller's stream (no allocation, copy or
    synchronisation), so they can be captured in a HIP graph.  The graph is replayed several times
    with eager work and synchronisations in between, and every replay is checked against the
    free-running oracle."""
    import gpu_harness as G
    import paper_1712_02679_amd as A
    wl = W.workload(2)
    table, n, nl = wl.table(), wl.n_total, 3
    mask = G.layer_mask(table, n)
    gpu = G.GpuSide(table, n, nl, batch=True)
    other = G.GpuSide(table, n, 1)
    try:
        static_g = [torch.zeros(n, dtype=torch.float32, device=G.DEV) for _ in range(nl)]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                       # warm-up outside capture
            A.adacomp_compress_batch(table, static_g, gpu.residue, gpu.packets, gpu.ws)
            A.adacomp_unpack_accumulate(table, gpu.packets, gpu.dense, gpu.ws)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            A.adacomp_compress_batch(table, static_g, gpu.residue, gpu.packets, gpu.ws)
            A.adacomp_unpack_accumulate(table, gpu.packets, gpu.dense, gpu.ws)
        for r in gpu.residue:
            r.zero_()
        R_cpu = [np.zeros(n, f32) for _ in range(nl)]
        for t in range(5):
            G.say(f"graph replay {t}")
            grads = [W.gradient(wl, k, t) for k in range(nl)]
            for k in range(nl):
                static_g[k].copy_(torch.from_numpy(grads[k]))
            for p in gpu.packets:
                p.fill_(G.POISON)
            graph.replay()
            torch.cuda.synchronize()
            want = [oracle_lib.compress(table, grads[k], R_cpu[k]) for k in range(nl)]
            for k in range(nl):
                G.compare_packet(gpu.packets[k].cpu().numpy(), want[k], gpu.capacity, f"replay {t} learner {k}")
                G.compare_residue(gpu.residue[k].cpu().numpy(), R_cpu[k], mask, 1.0, f"replay {t} learner {k}")
            dense = oracle_lib.unpack_accumulate(table, want, n)
            assert np.array_equal(gpu.dense.cpu().numpy()[mask].view(np.uint32), dense[mask].view(np.uint32))
            # eager work of the same library on other buffers between the replays
            other.compress(0, grads[0])
            other.unpack([0])
    finally:
        gpu.close()
        other.close()


def test_hip_graph_replay_of_the_lazy_call(H, oracle_lib):
    """A graph holds the kernels of the call that was captured: a lazy call captured while
    corrections wait (here: after a first lazy call, on zero gradients) applies the previous replay's
    corrections at every replay.  Packets and sums against the oracle at every replay, residues after
    the sync that follows the last one."""
    import gpu_harness as G
    import paper_1712_02679_amd as A
    wl = W.workload(2)
    table, n, nl = wl.table(), wl.n_total, 3
    mask = G.layer_mask(table, n)
    gpu = G.GpuSide(table, n, nl, batch=True)
    other = G.GpuSide(table, n, 1)
    try:
        static_g = [torch.zeros(n, dtype=torch.float32, device=G.DEV) for _ in range(nl)]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                       # first lazy call, outside capture: nothing is sent
            A.adacomp_compress_batch_lazy(table, static_g, gpu.residue, gpu.packets, gpu.ws)
            A.adacomp_unpack_accumulate(table, gpu.packets, gpu.dense, gpu.ws)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            A.adacomp_compress_batch_lazy(table, static_g, gpu.residue, gpu.packets, gpu.ws)
            A.adacomp_unpack_accumulate(table, gpu.packets, gpu.dense, gpu.ws)
        R_cpu = [np.zeros(n, f32) for _ in range(nl)]
        for t in range(5):
            G.say(f"lazy graph replay {t}")
            grads = [W.gradient(wl, k, t) for k in range(nl)]
            for k in range(nl):
                static_g[k].copy_(torch.from_numpy(grads[k]))
            for p in gpu.packets:
                p.fill_(G.POISON)
            graph.replay()
            torch.cuda.synchronize()
            want = [oracle_lib.compress(table, grads[k], R_cpu[k]) for k in range(nl)]
            for k in range(nl):
                G.compare_packet(gpu.packets[k].cpu().numpy(), want[k], gpu.capacity, f"lazy replay {t} learner {k}")
            dense = oracle_lib.unpack_accumulate(table, want, n)
            assert np.array_equal(gpu.dense.cpu().numpy()[mask].view(np.uint32), dense[mask].view(np.uint32))
            other.compress(0, grads[0])                      # eager work on other buffers between the replays
            other.unpack([0])
        A.adacomp_residue_sync(gpu.ws)
        torch.cuda.synchronize()
        for k in range(nl):
            G.compare_residue(gpu.residue[k].cpu().numpy(), R_cpu[k], mask, 1.0, f"lazy replays, learner {k}, after the sync")
    finally:
        gpu.close()
        other.close()


def test_two_streams_two_workspaces(H, oracle_lib):
    """Calls on different streams with different workspaces do not interact: two learners are
    compressed concurrently, each on a stream of its own, for several steps with no synchronisation
    in between, and each gives exactly what the oracle gives."""
    import gpu_harness as G
    import paper_1712_02679_amd as A
    wl = W.workload(4)
    table, n = wl.table(), wl.n_total
    sides = [G.GpuSide(table, n, 1), G.GpuSide(table, n, 1)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    steps = 4
    try:
        grads = [[torch.from_numpy(W.gradient(wl, k, t)).to(G.DEV) for t in range(steps)] for k in range(2)]
        packets = [[torch.full((sides[k].capacity,), G.POISON, dtype=torch.uint8, device=G.DEV) for _ in range(steps)] for k in range(2)]
        torch.cuda.synchronize()
        for t in range(steps):
            for k in range(2):
                with torch.cuda.stream(streams[k]):
                    A.adacomp_compress(table, grads[k][t], sides[k].residue[0], packets[k][t], sides[k].ws)
        torch.cuda.synchronize()
        for k in range(2):
            R = np.zeros(n, f32)
            for t in range(steps):
                want = oracle_lib.compress(table, grads[k][t].cpu().numpy(), R)
                G.compare_packet(packets[k][t].cpu().numpy(), want, sides[k].capacity, f"stream {k} step {t}")
            assert np.array_equal(sides[k].residue[0].cpu().numpy().view(np.uint32), R.view(np.uint32))
    finally:
        for s_ in sides:
            s_.close()


def test_two_host_threads_two_workspaces(H, oracle_lib):
    """Two host threads call the library at the same time, each with its own stream, workspace and
    learners (one through the eager calls, one through the lazy ones), while workspaces are
    registered and released on a third: the host-side books are locked, and each thread gets exactly
    what the oracle gives."""
    import threading
    import gpu_harness as G
    import paper_1712_02679_amd as A
    wl = W.workload(2)
    table, n, nl, steps = wl.table(), wl.n_total, 2, 12
    sides = [G.GpuSide(table, n, nl, batch=True) for _ in range(2)]
    grads_np = [[[W.gradient(wl, 2 * w + k, t, seed=90) for k in range(nl)] for t in range(steps)] for w in range(2)]
    grads = [[[torch.from_numpy(g).to(G.DEV) for g in step] for step in per] for per in grads_np]
    packets = [[[torch.full((sides[w].capacity,), G.POISON, dtype=torch.uint8, device=G.DEV) for _ in range(nl)]
                for _ in range(steps)] for w in range(2)]
    torch.cuda.synchronize()
    errors, stop = [], threading.Event()

    def worker(w):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for t in range(steps):
                    call = A.adacomp_compress_batch if w == 0 else A.adacomp_compress_batch_lazy
                    call(table, grads[w][t], sides[w].residue, packets[w][t], sides[w].ws)
                    A.adacomp_unpack_accumulate(table, packets[w][t], sides[w].dense, sides[w].ws)
                if w == 1:
                    A.adacomp_residue_sync(sides[w].ws)
            stream.synchronize()
        except Exception as e:   # reported by the main thread
            errors.append((w, repr(e)))

    def churn():
        other = [(0, 5000, 50), (5000, 7001, 500)]
        try:
            while not stop.is_set():
                ws = torch.zeros(A.adacomp_workspace_bytes(other), dtype=torch.uint8, device=G.DEV)
                A.adacomp_workspace_init(other, ws)
                A.adacomp_workspace_release(ws)
        except Exception as e:
            errors.append(("churn", repr(e)))

    try:
        threads = [threading.Thread(target=worker, args=(w,)) for w in range(2)]
        extra = threading.Thread(target=churn)
        extra.start()
        for th in threads:
            th.start()
        for th in threads:
            th.join()
        stop.set()
        extra.join()
        torch.cuda.synchronize()
        assert not errors, errors
        mask = G.layer_mask(table, n)
        for w in range(2):
            R = [np.zeros(n, f32) for _ in range(nl)]
            want = None
            for t in range(steps):
                want = [oracle_lib.compress(table, grads_np[w][t][k], R[k]) for k in range(nl)]
                for k in range(nl):
                    G.compare_packet(packets[w][t][k].cpu().numpy(), want[k], sides[w].capacity, f"thread {w} step {t} learner {k}")
            for k in range(nl):
                assert np.array_equal(sides[w].residue[k].cpu().numpy().view(np.uint32), R[k].view(np.uint32)), f"thread {w} residue {k}"
            dense = oracle_lib.unpack_accumulate(table, want, n)
            assert np.array_equal(sides[w].dense.cpu().numpy()[mask].view(np.uint32), dense[mask].view(np.uint32))
    finally:
        stop.set()
        for s_ in sides:
            s_.close()


def test_checkpoint_resume(H, oracle_lib):
    """The residue is the only learner state: copying it out and back resumes identically."""
    import gpu_harness as G
    wl = W.workload(1)
    table, n = wl.table(), wl.n_total
    a = G.GpuSide(table, n, 1)
    b = G.GpuSide(table, n, 1)
    try:
        for t in range(2):
            a.compress(0, W.gradient(wl, 0, t))
        b.residue[0].copy_(a.residue[0].cpu().to(G.DEV))     # "checkpoint" through host memory
        pa = a.compress(0, W.gradient(wl, 0, 2))
        pb = b.compress(0, W.gradient(wl, 0, 2))
        assert np.array_equal(pa, pb)
    finally:
        a.close()
        b.close()


def test_caller_written_in_c(H):
    """The C ABI from a caller that is not Python: tests/c_driver/abi_roundtrip (C++ and the HIP
    runtime only, built beforehand by the build entry point) runs batched and single compress
    calls, unpack and the fused SGD step on a four-layer table and compares every byte with the
    oracle linked into it."""
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_driver", "abi_roundtrip")
    assert os.path.exists(exe), "build it first: python -c 'import __graft_entry__ as g; g.build()'"
    res = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "c caller ok" in res.stdout


def test_library_called_before_torch_is_imported(H):
    """A process that touches the binding before it imports torch must end up with one HIP runtime
    (the binding pulls torch in before it loads the library): set-up and a compress call work."""
    import subprocess
    import sys
    code = (
        "import paper_1712_02679_amd as A\n"
        "A.adacomp_tuning_fold_scan(True)\n"            # loads the library
        "import torch\n"
        "t = [(0, 50 * 40 + 7, 50), (2008, 500 * 12 + 11, 500)]\n"
        "n = 2008 + 6011\n"
        "ws = torch.zeros(A.adacomp_workspace_bytes(t), dtype=torch.uint8, device='cuda')\n"
        "A.adacomp_workspace_init(t, ws)\n"
        "g = torch.randn(n, device='cuda'); r = torch.zeros(n, device='cuda')\n"
        "p = torch.zeros(A.adacomp_packet_bound(t), dtype=torch.uint8, device='cuda')\n"
        "A.adacomp_compress(t, g, r, p, ws)\n"
        "torch.cuda.synchronize()\n"
        "h, _ = A.read_packet_summary(p)\n"
        "assert int(h['n_selected']) > 0\n"
        "print('ok')\n")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and "ok" in out.stdout, out.stderr[-2000:]


def test_copy_kernel(H):
    import paper_1712_02679_amd as A
    for n in (1, 5, 1024, 1 << 20, (1 << 22) + 3):
        src = torch.arange(n, dtype=torch.float32, device="cuda:0")
        dst = torch.full((n + 4,), -1.0, dtype=torch.float32, device="cuda:0")
        A.adacomp_copy_f32(dst, src, n)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and torch.all(dst[n:] == -1.0)


def test_calibration_kernels(H):
    """The bare triad and fill that bench.py measures the hot kernels against do what they say
    (x <- x + y as single float32 additions, x <- value), on whole and ragged numbers of tiles, and
    touch nothing beyond n."""
    import paper_1712_02679_amd as A
    for n in (4, 4096, 4096 * 64, 4096 * 130 + 8, (1 << 22) + 4092):
        x0 = torch.randn(n + 8, dtype=torch.float32, device="cuda:0")
        y = torch.randn(n + 8, dtype=torch.float32, device="cuda:0")
        x = x0.clone()
        A.adacomp_triad_f32(x, y, n)
        torch.cuda.synchronize()
        assert torch.equal(x[:n], x0[:n] + y[:n]) and torch.equal(x[n:], x0[n:])
        for resident in (3, 4, 6, 8):       # the same kernel with fewer workgroups per compute unit
            x.copy_(x0)
            A.adacomp_triad_resident_f32(x, y, resident, n)
            torch.cuda.synchronize()
            assert torch.equal(x[:n], x0[:n] + y[:n]) and torch.equal(x[n:], x0[n:])
        A.adacomp_fill_f32(x, 2.5, n)
        torch.cuda.synchronize()
        assert torch.all(x[:n] == 2.5) and torch.equal(x[n:], x0[n:])
    with pytest.raises(A.AdacompError):
        A.adacomp_triad_f32(x, y, 6)          # not a multiple of 4
    with pytest.raises(A.AdacompError):
        A.adacomp_triad_f32(x, x, 8)          # in place on itself
    for resident in (0, 2, 9):
        with pytest.raises(A.AdacompError):
            A.adacomp_triad_resident_f32(x, y, resident, 8)
