"""ctypes binding of libadacomp's C ABI (include/adacomp.h): argument marshalling only.

Every step of the method runs in the HIP kernels behind these calls.  PyTorch tensors are used as
device buffers and for the current HIP stream; nothing is computed with torch.  There is no CPU
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import functools
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadacomp.so")

OK, EINVAL, EBADLT, EALIGN, ENOSPC, EHIP, EWORKSPACE, EPENDING, ETOOBIG = 0, -1, -2, -3, -4, -5, -6, -7, -8
STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = [
    "adacomp_packet_bound", "adacomp_packet_fixed_bytes", "adacomp_workspace_bytes",
    "adacomp_workspace_bytes_batch", "adacomp_workspace_init", "adacomp_workspace_release",
    "adacomp_compress", "adacomp_compress_static", "adacomp_compress_batch", "adacomp_compress_variant",
    "adacomp_compress_batch_lazy", "adacomp_residue_sync",
    "adacomp_unpack_accumulate", "adacomp_unpack_update", "adacomp_strerror", "adacomp_workspace_gmax", "adacomp_debug_keep_gmax",
    "adacomp_copy_f32", "adacomp_triad_f32", "adacomp_triad_resident_f32", "adacomp_fill_f32",
    "adacomp_selftest_binindex", "adacomp_tuning_unpack_min_groups", "adacomp_tuning_fold_scan", "adacomp_tuning_place_tiled", "adacomp_timing_enable", "adacomp_timing_read",
]

PACKET_HEADER = np.dtype([("magic", "<u4"), ("version", "<u4"), ("status", "<u4"), ("n_layers", "<u4"),
                          ("total_bytes", "<u8"), ("n_selected", "<u8")])
PACKET_LAYER = np.dtype([("elem_offset", "<u8"), ("n_elems", "<u8"), ("L_T", "<u4"), ("n_bins", "<u4"),
                         ("word_bits", "<u4"), ("scale", "<f4"), ("n_selected", "<u8"),
                         ("counts_offset", "<u8"), ("chunks_offset", "<u8"), ("words_offset", "<u8")])


class Layer(ctypes.Structure):
    _fields_ = [("elem_offset", ctypes.c_uint64), ("n_elems", ctypes.c_uint64),
                ("L_T", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class Optimizer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_uint32), ("lr", ctypes.c_float), ("momentum", ctypes.c_float),
                ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("bias1", ctypes.c_float), ("bias2", ctypes.c_float)]


OPT_SGD_MOMENTUM, OPT_ADAM = 1, 2


class AdacompError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libadacomp: {msg} ({code})")
        self.code = code


_lib = None


def lib():
    """Loads libadacomp.so (built beforehand by ``__graft_entry__.build()``); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1712_02679_amd.build` "
                               "(there is no CPU fallback)")
        # PyTorch brings its own copy of the HIP runtime; it has to be in the process before the
        # library is, or the two end up with different runtimes and the first call that touches
        # the device fails with ADACOMP_EHIP.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        LP, u32, sz, vp = ctypes.POINTER(Layer), ctypes.c_uint32, ctypes.c_size_t, ctypes.c_void_p
        for name in ("adacomp_packet_bound", "adacomp_packet_fixed_bytes", "adacomp_workspace_bytes"):
            getattr(L, name).restype = sz
            getattr(L, name).argtypes = [LP, u32]
        L.adacomp_workspace_bytes_batch.restype = sz
        L.adacomp_workspace_bytes_batch.argtypes = [LP, u32, u32]
        L.adacomp_compress_batch.argtypes = [LP, u32, u32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                             ctypes.POINTER(vp), sz, vp, sz, vp]
        L.adacomp_compress_batch_lazy.argtypes = L.adacomp_compress_batch.argtypes
        L.adacomp_residue_sync.argtypes = [vp, vp]
        L.adacomp_compress_variant.argtypes = [LP, u32, u32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                               ctypes.POINTER(vp), sz, u32, ctypes.c_float, vp, sz, vp]
        L.adacomp_workspace_init.argtypes = [LP, u32, vp, sz, vp]
        L.adacomp_workspace_release.argtypes = [vp]
        L.adacomp_compress.argtypes = [LP, u32, vp, vp, vp, sz, vp, sz, vp]
        L.adacomp_compress_static.argtypes = [LP, u32, vp, vp, vp, sz, vp]
        L.adacomp_unpack_accumulate.argtypes = [LP, u32, ctypes.POINTER(vp), u32, vp, vp, sz, vp]
        L.adacomp_unpack_update.argtypes = [LP, u32, ctypes.POINTER(vp), u32, vp, vp, vp, vp,
                                            ctypes.POINTER(Optimizer), vp, sz, vp]
        L.adacomp_strerror.restype = ctypes.c_char_p
        L.adacomp_strerror.argtypes = [ctypes.c_int]
        L.adacomp_workspace_gmax.argtypes = [LP, u32, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.adacomp_debug_keep_gmax.argtypes = [ctypes.c_int]
        L.adacomp_copy_f32.argtypes = [vp, vp, sz, vp]
        L.adacomp_triad_f32.argtypes = [vp, vp, sz, vp]
        L.adacomp_triad_resident_f32.argtypes = [vp, vp, sz, ctypes.c_uint32, vp]
        L.adacomp_fill_f32.argtypes = [vp, ctypes.c_float, sz, vp]
        L.adacomp_tuning_unpack_min_groups.argtypes = [ctypes.c_uint32]
        L.adacomp_tuning_fold_scan.argtypes = [ctypes.c_int]
        L.adacomp_tuning_place_tiled.argtypes = [ctypes.c_int]
        L.adacomp_timing_enable.argtypes = [ctypes.c_int]
        L.adacomp_timing_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_uint64),
                                          ctypes.POINTER(ctypes.c_uint64)]
        _lib = L
    return _lib


def _check(rc):
    if rc != OK:
        raise AdacompError(rc, lib().adacomp_strerror(rc).decode())


@functools.lru_cache(maxsize=32)
def _layer_array(key):
    arr = (Layer * max(1, len(key)))()
    for i, (off, n, lt) in enumerate(key):
        arr[i].elem_offset, arr[i].n_elems, arr[i].L_T, arr[i].reserved = int(off), int(n), int(lt), 0
    return arr


def layer_array(layers):
    """[(elem_offset, n_elems, L_T)] -> ctypes array of adacomp_layer_t (kept for tables seen before:
    the library only reads it)."""
    return _layer_array(tuple(map(tuple, layers)))


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def adacomp_packet_bound(layers) -> int:
    return int(lib().adacomp_packet_bound(layer_array(layers), len(layers)))


def adacomp_packet_fixed_bytes(layers) -> int:
    return int(lib().adacomp_packet_fixed_bytes(layer_array(layers), len(layers)))


def adacomp_workspace_bytes(layers) -> int:
    return int(lib().adacomp_workspace_bytes(layer_array(layers), len(layers)))


def adacomp_workspace_bytes_batch(layers, n_learners) -> int:
    return int(lib().adacomp_workspace_bytes_batch(layer_array(layers), len(layers), int(n_learners)))


def adacomp_workspace_init(layers, workspace):
    _check(lib().adacomp_workspace_init(layer_array(layers), len(layers), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream()))


def adacomp_workspace_release(workspace):
    _check(lib().adacomp_workspace_release(_ptr(workspace)))


def adacomp_compress(layers, grad, residue, packet_out, workspace, packet_capacity=None):
    """grad, residue: float32 CUDA tensors; packet_out, workspace: uint8 CUDA tensors."""
    cap = packet_out.numel() if packet_capacity is None else int(packet_capacity)
    _check(lib().adacomp_compress(layer_array(layers), len(layers), _ptr(grad), _ptr(residue),
                                  _ptr(packet_out), cap, _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream()))


def adacomp_compress_static(layers, grad, residue, packet_out, packet_capacity=None):
    """adacomp_compress on the library's own static scratch array: no workspace, nothing allocated."""
    cap = packet_out.numel() if packet_capacity is None else int(packet_capacity)
    _check(lib().adacomp_compress_static(layer_array(layers), len(layers), _ptr(grad), _ptr(residue),
                                         _ptr(packet_out), cap, _stream()))


def adacomp_compress_batch(layers, grads, residues, packets_out, workspace, packet_capacity=None):
    """grads, residues: lists of float32 CUDA tensors; packets_out: list of uint8 CUDA tensors."""
    n = len(grads)
    cap = min(p.numel() for p in packets_out) if packet_capacity is None else int(packet_capacity)
    vp = ctypes.c_void_p
    g = (vp * n)(*[t.data_ptr() for t in grads])
    r = (vp * n)(*[t.data_ptr() for t in residues])
    p = (vp * n)(*[t.data_ptr() for t in packets_out])
    _check(lib().adacomp_compress_batch(layer_array(layers), len(layers), n, g, r, p, cap, _ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream()))


def adacomp_compress_batch_lazy(layers, grads, residues, packets_out, workspace, packet_capacity=None):
    """adacomp_compress_batch with the residue corrections left waiting in the workspace: the next
    call on it is this one with the same residue tensors, or adacomp_residue_sync."""
    n = len(grads)
    cap = min(p.numel() for p in packets_out) if packet_capacity is None else int(packet_capacity)
    vp = ctypes.c_void_p
    g = (vp * n)(*[t.data_ptr() for t in grads])
    r = (vp * n)(*[t.data_ptr() for t in residues])
    p = (vp * n)(*[t.data_ptr() for t in packets_out])
    _check(lib().adacomp_compress_batch_lazy(layer_array(layers), len(layers), n, g, r, p, cap, _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream()))


def adacomp_residue_sync(workspace):
    """Writes the residue corrections that the last lazy call on this workspace left waiting."""
    _check(lib().adacomp_residue_sync(_ptr(workspace), _stream()))


RULE_ADACOMP, RULE_PRINTED_COMPARE, RULE_LOCAL_SELECTION = 0, 1, 2


def adacomp_compress_variant(layers, grads, residues, packets_out, workspace, rule=RULE_ADACOMP, soft_factor=2.0,
                             packet_capacity=None):
    """adacomp_compress_batch with another selection rule or soft-threshold factor."""
    n = len(grads)
    cap = min(p.numel() for p in packets_out) if packet_capacity is None else int(packet_capacity)
    vp = ctypes.c_void_p
    g = (vp * n)(*[t.data_ptr() for t in grads])
    r = (vp * n)(*[t.data_ptr() for t in residues])
    p = (vp * n)(*[t.data_ptr() for t in packets_out])
    _check(lib().adacomp_compress_variant(layer_array(layers), len(layers), n, g, r, p, cap, int(rule),
                                          ctypes.c_float(soft_factor), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream()))


def adacomp_unpack_accumulate(layers, packets, dense_out, workspace):
    """packets: list of uint8 CUDA tensors (one per learner)."""
    ptrs = (ctypes.c_void_p * max(1, len(packets)))(*[p.data_ptr() for p in packets])
    _check(lib().adacomp_unpack_accumulate(layer_array(layers), len(layers), ptrs, len(packets),
                                           _ptr(dense_out), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream()))


def adacomp_unpack_update(layers, packets, dense_out, weights, state1, state2, workspace, kind, lr, momentum=0.0,
                          beta1=0.9, beta2=0.999, eps=1e-8, bias1=1.0, bias2=1.0):
    """unpack + average + one optimizer step; dense_out and state2 may be None."""
    ptrs = (ctypes.c_void_p * max(1, len(packets)))(*[p.data_ptr() for p in packets])
    opt = Optimizer(int(kind), lr, momentum, beta1, beta2, eps, bias1, bias2)
    null = ctypes.c_void_p(None)
    _check(lib().adacomp_unpack_update(layer_array(layers), len(layers), ptrs, len(packets),
                                       _ptr(dense_out) if dense_out is not None else null, _ptr(weights),
                                       _ptr(state1), _ptr(state2) if state2 is not None else null,
                                       ctypes.byref(opt), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream()))


def adacomp_workspace_gmax(layers):
    off, n, stride = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().adacomp_workspace_gmax(layer_array(layers), len(layers), ctypes.byref(off), ctypes.byref(n),
                                        ctypes.byref(stride)))
    return off.value, n.value, stride.value


def adacomp_debug_keep_gmax(on: bool):
    _check(lib().adacomp_debug_keep_gmax(1 if on else 0))


def adacomp_copy_f32(dst, src, n=None):
    _check(lib().adacomp_copy_f32(_ptr(dst), _ptr(src), dst.numel() if n is None else int(n), _stream()))


def adacomp_triad_f32(x, y, n=None):
    """x <- x + y in place with the access pattern of the streaming pass of compress (12 B per element)."""
    _check(lib().adacomp_triad_f32(_ptr(x), _ptr(y), x.numel() if n is None else int(n), _stream()))


def adacomp_triad_resident_f32(x, y, workgroups_per_cu, n=None):
    """The same triad with at most workgroups_per_cu (3 .. 8) workgroups resident per compute unit."""
    _check(lib().adacomp_triad_resident_f32(_ptr(x), _ptr(y), x.numel() if n is None else int(n),
                                            int(workgroups_per_cu), _stream()))


def adacomp_fill_f32(x, value=0.0, n=None):
    """x <- value with streaming 16-byte stores (4 B per element)."""
    _check(lib().adacomp_fill_f32(_ptr(x), ctypes.c_float(value), x.numel() if n is None else int(n), _stream()))


def adacomp_selftest_binindex() -> int:
    return int(lib().adacomp_selftest_binindex())


def adacomp_tuning_unpack_min_groups(n_groups: int):
    """Workspaces initialised afterwards group unpack tiles only while n_groups workgroups remain; 0: default."""
    _check(lib().adacomp_tuning_unpack_min_groups(int(n_groups)))


def adacomp_tuning_fold_scan(enable: bool):
    """False: small tables take the three-launch compress path of the large ones; True: the default."""
    _check(lib().adacomp_tuning_fold_scan(1 if enable else 0))


def adacomp_tuning_place_tiled(enable: bool):
    """False: tables with short bins take the word-by-word placement of the others; True: the default."""
    _check(lib().adacomp_tuning_place_tiled(1 if enable else 0))


def adacomp_timing_enable(every: int):
    """0: off; k > 0: record every k-th launch of the streaming kernel."""
    _check(lib().adacomp_timing_enable(int(every)))


def adacomp_timing_read():
    ms, n, k = ctypes.c_double(), ctypes.c_uint64(), ctypes.c_uint64()
    _check(lib().adacomp_timing_read(ctypes.byref(ms), ctypes.byref(n), ctypes.byref(k)))
    return ms.value, n.value, k.value


def read_packet_summary(packet):
    """Header and layer records of a packet tensor as numpy records (one small D2H copy)."""
    head = packet[:32].cpu().numpy().view(PACKET_HEADER)[0]
    n = int(head["n_layers"])
    recs = packet[32:32 + 64 * n].cpu().numpy().view(PACKET_LAYER)
    return head, recs
