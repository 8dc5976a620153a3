"""Shared driver of the GPU parity tests: runs the same seeded inputs through libadacomp (via the
C ABI binding) and through the CPU oracle, and compares element by element.

Bars: packets bit-identical in indices, signs, counts and
layout; float32 scale within 1e-6 relative; residue within 1e-6 * max(|G|, scale) absolute.
Because every float32 step is a single correctly rounded addition and the float64 sum of g_max
is exact for these inputs, bit equality is expected throughout and is what the comparisons
assert first; the tolerance form is the fallback that tells a genuine mismatch from a last-bit
difference in the scale.
"""
import os
import sys

import numpy as np
import torch

import adacomp_workloads as W
import packet_format as pf
import paper_1712_02679_amd as A

DEV = "cuda:0"
POISON = 0xCD


_PROGRESS = None


def say(msg):
    """Names the case about to run: on stdout (pytest shows it with -s or on failure) and, flushed, in
    a progress log that a test runner which captures stdout does not hide (in the directory
    ADACOMP_TEST_LOG_DIR names, else in the temporary directory)."""
    global _PROGRESS
    print(f"[parity] {msg}", flush=True)
    try:
        if _PROGRESS is None:
            import tempfile
            d = os.environ.get("ADACOMP_TEST_LOG_DIR") or ""
            if not os.path.isdir(d):
                d = tempfile.gettempdir()
            _PROGRESS = open(os.path.join(d, "parity_progress.log"), "a", buffering=1)
        if _PROGRESS:
            _PROGRESS.write(msg + "\n")
            _PROGRESS.flush()
    except OSError:
        _PROGRESS = False


class GpuSide:
    """Device buffers of n learners for one layer table."""

    def __init__(self, table, n_total, n_learners, capacity=None, batch=False, keep_gmax=False):
        """keep_gmax: have compress store the g_max vector (a diagnostic that the timed path leaves
        off); only the cases that compare it switch it on, and close() switches it off again."""
        self.table, self.n_total = table, n_total
        ws_bytes = A.adacomp_workspace_bytes_batch(table, n_learners) if batch else A.adacomp_workspace_bytes(table)
        self.ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=DEV)
        A.adacomp_workspace_init(table, self.ws)
        self.keep_gmax = bool(keep_gmax)
        A.adacomp_debug_keep_gmax(self.keep_gmax)
        self.bound = A.adacomp_packet_bound(table)
        self.capacity = self.bound if capacity is None else capacity
        self.residue = [torch.zeros(n_total, dtype=torch.float32, device=DEV) for _ in range(n_learners)]
        self.packets = [torch.full((self.capacity + 64,), POISON, dtype=torch.uint8, device=DEV)
                        for _ in range(n_learners)]
        self.dense = torch.full((n_total,), float("nan"), dtype=torch.float32, device=DEV)

    def compress(self, k, grad_np):
        g = torch.from_numpy(grad_np).to(DEV)
        self.packets[k].fill_(POISON)
        A.adacomp_compress(self.table, g, self.residue[k], self.packets[k], self.ws,
                           packet_capacity=self.capacity)
        torch.cuda.synchronize()
        return self.packets[k].cpu().numpy()

    def compress_batch(self, grads_np, rule=0, soft_factor=2.0):
        """One adacomp_compress_batch (or _variant) call over all learners; returns their packet buffers."""
        g = [torch.from_numpy(x).to(DEV) for x in grads_np]
        for p in self.packets:
            p.fill_(POISON)
        if rule == 0 and soft_factor == 2.0:
            A.adacomp_compress_batch(self.table, g, self.residue, self.packets, self.ws, packet_capacity=self.capacity)
        else:
            A.adacomp_compress_variant(self.table, g, self.residue, self.packets, self.ws, rule=rule,
                                       soft_factor=soft_factor, packet_capacity=self.capacity)
        torch.cuda.synchronize()
        return [p.cpu().numpy() for p in self.packets]

    def unpack(self, ks):
        self.dense.fill_(float("nan"))
        A.adacomp_unpack_accumulate(self.table, [self.packets[k] for k in ks], self.dense, self.ws)
        torch.cuda.synchronize()
        return self.dense.cpu().numpy()

    def gmax(self, learner=0):
        assert self.keep_gmax, "this GpuSide was made without keep_gmax"
        off, n, stride = A.adacomp_workspace_gmax(self.table)
        off += stride * learner
        return self.ws[off:off + 4 * n].cpu().numpy().view(np.float32)

    def close(self):
        A.adacomp_debug_keep_gmax(False)
        A.adacomp_workspace_release(self.ws)


def layer_mask(table, n_total):
    m = np.zeros(n_total, bool)
    for off, n, _ in table:
        m[off:off + n] = True
    return m


def compare_packet(got_buf, want, capacity, tag, strict=True):
    """got_buf: device packet buffer (with poison tail); want: oracle packet bytes.
    Everything but the scales must be bit-equal and the scales within 1e-6 relative.  strict: the
    scales must be bit-equal too (what every case expects whose float64 sum of g_max is exact);
    otherwise the return value says whether they were."""
    h = pf.header(got_buf)
    assert int(h["total_bytes"]) == want.size, f"{tag}: total_bytes {int(h['total_bytes'])} != oracle {want.size}"
    got = got_buf[:want.size]
    if not np.array_equal(got, want):
        # locate the difference for the report; then decide whether it is only a scale's last bits
        gh, gl = pf.parse(got, check=False)
        wh, wl = pf.parse(want, check=False)
        masked_g, masked_w = got.copy(), want.copy()
        for li in range(int(wh["n_layers"])):
            lo = 32 + 64 * li + 28
            masked_g[lo:lo + 4] = 0
            masked_w[lo:lo + 4] = 0
            sg, sw = float(gl[li]["rec"]["scale"]), float(wl[li]["rec"]["scale"])
            assert abs(sg - sw) <= 1e-6 * abs(sw), f"{tag}: layer {li} scale {sg!r} vs oracle {sw!r}"
        bad = np.flatnonzero(masked_g != masked_w)
        assert bad.size == 0, f"{tag}: packet differs from the oracle at byte {bad[0]} ({bad.size} bytes differ)"
        if strict:
            raise AssertionError(f"{tag}: packet equal except for the last bits of a scale "
                                 "(inside the 1e-6 bar, but bit equality was expected)")
        assert np.all(got_buf[want.size:] == POISON), f"{tag}: bytes after total_bytes were written"
        return False
    # nothing written past the packet end / past the capacity
    tail = got_buf[want.size:]
    assert np.all(tail == POISON), f"{tag}: bytes after total_bytes were written"
    pf.parse(got)  # structural invariants of the container
    return True


def compare_residue(got, want, mask, scale_hint, tag, strict=True):
    """mask: the elements that belong to a layer, or None when all do (no copies are made then)."""
    if mask is None:
        mask = slice(None)
    if np.array_equal(got[mask].view(np.uint32), want[mask].view(np.uint32)):
        return True
    d = np.abs(got[mask].astype(np.float64) - want[mask])
    tol = 1e-6 * np.maximum(np.abs(want[mask]), scale_hint)
    worst = int(np.argmax(d - tol))
    assert np.all(d <= tol), f"{tag}: residue differs beyond 1e-6 at masked index {worst}: {got[mask][worst]} vs {want[mask][worst]}"
    if strict:
        raise AssertionError(f"{tag}: residue within 1e-6 but not bit-equal (max diff {d.max():.3e})")
    return False


def run_parity(oracle_lib, wl, n_learners, n_steps, seed=0, step_locked=False, grads=None,
               check_gmax=True, unpack_every_step=True, threads=8, label=None, batch=False, rule=0, soft_factor=2.0,
               oracle_threads=1):
    """Free-running (default) or step-locked comparison of GPU and oracle over several steps.
    grads: optional callable (learner, step) -> numpy float32 array overriding the generator.
    oracle_threads > 1 (batched runs without the g_max check): the oracle's calls of one step, one per
    learner, run on that many host threads (the learners are independent)."""
    label = label or wl.name
    assert batch or (rule == 0 and soft_factor == 2.0), "variants go through the batched entry point"
    table, n_total = wl.table(), wl.n_total
    mask = layer_mask(table, n_total)
    if mask.all():
        mask = None   # a table without gaps: whole arrays are compared
    gpu = GpuSide(table, n_total, n_learners, batch=batch, keep_gmax=check_gmax)
    R_cpu = [np.zeros(n_total, np.float32) for _ in range(n_learners)]
    stats = []
    try:
        for t in range(n_steps):
            cpu_packets = []
            if batch:   # all learners in one adacomp_compress_batch call, compared one by one below
                say(f"{label} step {t} batch of {n_learners}")
                all_g = [grads(k, t) if grads else W.gradient(wl, k, t, seed=seed, threads=threads)
                         for k in range(n_learners)]
                if step_locked:
                    for k in range(n_learners):
                        gpu.residue[k].copy_(torch.from_numpy(R_cpu[k]))
                batch_bufs = gpu.compress_batch(all_g, rule, soft_factor)
                wants = None
                if oracle_threads > 1 and not check_gmax:
                    from concurrent.futures import ThreadPoolExecutor
                    with ThreadPoolExecutor(min(oracle_threads, n_learners)) as pool:
                        wants = list(pool.map(lambda k: oracle_lib.compress(table, all_g[k], R_cpu[k], rule=rule,
                                                                            soft_factor=soft_factor), range(n_learners)))
            for k in range(n_learners):
                tag = f"{label} step {t} learner {k}"
                say(tag)
                g = all_g[k] if batch else (grads(k, t) if grads else W.gradient(wl, k, t, seed=seed, threads=threads))
                if step_locked and not batch:
                    gpu.residue[k].copy_(torch.from_numpy(R_cpu[k]))
                R_before = R_cpu[k].copy() if check_gmax else None
                if batch and wants is not None:
                    want = wants[k]
                else:
                    want = oracle_lib.compress(table, g, R_cpu[k], rule=rule, soft_factor=soft_factor)
                got_buf = batch_bufs[k] if batch else gpu.compress(k, g)
                if check_gmax:
                    G = R_before + g
                    expect = np.concatenate([
                        np.abs(np.pad(G[off:off + n], (0, (-n) % T))).reshape(-1, T).max(axis=1)
                        for off, n, T in table])
                    assert np.array_equal(gpu.gmax(k if batch else 0).view(np.uint32), expect.view(np.uint32)), f"{tag}: g_max"
                compare_packet(got_buf, want, gpu.capacity, tag)
                h, layers = pf.parse(want, check=False)
                scale_hint = max(float(l["rec"]["scale"]) for l in layers)
                r_host = gpu.residue[k].cpu().numpy()
                compare_residue(r_host, R_cpu[k], mask, scale_hint, tag)
                # gaps between layers are never written
                assert mask is None or np.all(r_host[~mask] == 0)
                cpu_packets.append(want)
                stats.append((t, k, int(h["n_selected"]), want.size))
            if unpack_every_step or t == n_steps - 1:
                say(f"{label} step {t} unpack of {n_learners}")
                got = gpu.unpack(list(range(n_learners)))
                want = oracle_lib.unpack_accumulate(table, cpu_packets, n_total)
                sel = slice(None) if mask is None else mask
                assert np.array_equal(got[sel].view(np.uint32), want[sel].view(np.uint32)), \
                    f"{label} step {t}: dense sum differs"
                assert mask is None or np.isnan(got[~mask]).all(), f"{label}: unpack wrote outside the layers"
    finally:
        gpu.close()
    return stats


def run_lazy_parity(oracle_lib, wl, n_learners, n_steps, sync_every, seed=0, threads=8, oracle_threads=1, label=None):
    """adacomp_compress_batch_lazy against the oracle, free-running.  Every step: every packet and
    the 16-packet sum, and the residue as the call leaves it (G everywhere: the corrections wait).
    After every sync_every-th step and after the last one: adacomp_residue_sync, then the residue
    against the oracle's (0: only after the last step)."""
    from concurrent.futures import ThreadPoolExecutor
    label = label or ("lazy " + wl.name)
    table, n_total = wl.table(), wl.n_total
    mask = layer_mask(table, n_total)
    gpu = GpuSide(table, n_total, n_learners, batch=True)
    R_cpu = [np.zeros(n_total, np.float32) for _ in range(n_learners)]
    try:
        for t in range(n_steps):
            say(f"{label} step {t} lazy batch of {n_learners}")
            all_g = [W.gradient(wl, k, t, seed=seed, threads=threads) for k in range(n_learners)]
            G_want = [R_cpu[k] + all_g[k] for k in range(n_learners)]   # float32: what pack() accumulates
            g_dev = [torch.from_numpy(x).to(DEV) for x in all_g]
            for p in gpu.packets:
                p.fill_(POISON)
            A.adacomp_compress_batch_lazy(table, g_dev, gpu.residue, gpu.packets, gpu.ws, packet_capacity=gpu.capacity)
            torch.cuda.synchronize()
            with ThreadPoolExecutor(max(1, min(oracle_threads, n_learners))) as pool:
                wants = list(pool.map(lambda k: oracle_lib.compress(table, all_g[k], R_cpu[k]), range(n_learners)))
            for k in range(n_learners):
                tag = f"{label} step {t} learner {k}"
                say(tag)
                compare_packet(gpu.packets[k].cpu().numpy(), wants[k], gpu.capacity, tag)
                got_r = gpu.residue[k].cpu().numpy()
                assert np.array_equal(got_r[mask].view(np.uint32), G_want[k][mask].view(np.uint32)), \
                    f"{tag}: before the sync the residue is G"
            say(f"{label} step {t} unpack of {n_learners}")
            got = gpu.unpack(list(range(n_learners)))
            want = oracle_lib.unpack_accumulate(table, wants, n_total)
            assert np.array_equal(got[mask].view(np.uint32), want[mask].view(np.uint32)), f"{label} step {t}: dense sum differs"
            if (sync_every and (t + 1) % sync_every == 0) or t == n_steps - 1:
                say(f"{label} step {t} residue sync")
                A.adacomp_residue_sync(gpu.ws)
                torch.cuda.synchronize()
                for k in range(n_learners):
                    h, layers = pf.parse(wants[k], check=False)
                    scale_hint = max(float(l["rec"]["scale"]) for l in layers)
                    got_r = gpu.residue[k].cpu().numpy()
                    compare_residue(got_r, R_cpu[k], mask, scale_hint, f"{label} step {t} learner {k} after the sync")
                    assert np.all(got_r[~mask] == 0)
    finally:
        gpu.close()
