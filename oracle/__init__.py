"""ctypes access to the CPU oracle (``adacomp_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` import
this package.  It never imports the GPU package and the GPU package never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adacomp_oracle.c")
_LIB = os.path.join(_HERE, "libadacomp_oracle.so")

RULE_UNION, RULE_LITERAL, RULE_LS = 0, 1, 2


def build(extra_defines=(), out=None) -> str:
    """Compile the oracle with gcc.  No value-changing options: -O2, contraction off."""
    out = out or _LIB
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           "-shared", "-fPIC", *[f"-D{d}" for d in extra_defines], "-o", out, _SRC, "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return out


class _Layer(ctypes.Structure):
    _fields_ = [("elem_offset", ctypes.c_uint64), ("n_elems", ctypes.c_uint64),
                ("L_T", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


def _layer_array(layers):
    arr = (_Layer * len(layers))()
    for i, (off, n, lt) in enumerate(layers):
        arr[i].elem_offset, arr[i].n_elems, arr[i].L_T, arr[i].reserved = int(off), int(n), int(lt), 0
    return arr


class Oracle:
    """Thin wrapper: marshals numpy arrays into the C functions, nothing else."""

    def __init__(self, lib_path: str | None = None):
        path = lib_path or _LIB
        if not os.path.exists(path) or (lib_path is None and os.path.getmtime(path) < os.path.getmtime(_SRC)):
            build(out=path)
        self.lib = ctypes.CDLL(path)
        L = self.lib
        fp = ctypes.POINTER(ctypes.c_float)
        L.adacomp_oracle_pack_layer.restype = ctypes.c_longlong
        L.adacomp_oracle_pack_layer.argtypes = [fp, fp, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int,
                                                ctypes.c_float, fp, fp, fp, fp, ctypes.POINTER(ctypes.c_uint8), fp]
        L.adacomp_oracle_packet_bound.restype = ctypes.c_size_t
        L.adacomp_oracle_packet_bound.argtypes = [ctypes.POINTER(_Layer), ctypes.c_uint32]
        L.adacomp_oracle_compress.restype = ctypes.c_longlong
        L.adacomp_oracle_compress.argtypes = [ctypes.POINTER(_Layer), ctypes.c_uint32, fp, fp,
                                              ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float]
        L.adacomp_oracle_unpack_accumulate.restype = ctypes.c_int
        L.adacomp_oracle_unpack_accumulate.argtypes = [ctypes.POINTER(_Layer), ctypes.c_uint32,
                                                       ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint32, fp]

        cf = ctypes.c_float
        L.adacomp_oracle_update_sgd.restype = ctypes.c_int
        L.adacomp_oracle_update_sgd.argtypes = [ctypes.POINTER(_Layer), ctypes.c_uint32, fp, ctypes.c_uint32, fp, fp, cf, cf]
        L.adacomp_oracle_update_adam.restype = ctypes.c_int
        L.adacomp_oracle_update_adam.argtypes = [ctypes.POINTER(_Layer), ctypes.c_uint32, fp, ctypes.c_uint32, fp, fp, fp,
                                                 cf, cf, cf, cf, cf, cf]

    @staticmethod
    def _f(a):
        assert a.dtype == np.float32 and a.flags.c_contiguous
        return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))

    def pack_layer(self, residue, dW, T, rule=RULE_UNION, soft_factor=2.0):
        """One layer of Algorithm 2.  Returns a dict of every intermediate value."""
        residue = np.ascontiguousarray(residue, dtype=np.float32)
        dW = np.ascontiguousarray(dW, dtype=np.float32)
        n = residue.size
        n_bins = (n + T - 1) // T
        G = np.empty(n, np.float32)
        H = np.empty(n, np.float32)
        gmax = np.empty(n_bins, np.float32)
        scale = np.zeros(1, np.float32)
        sel = np.empty(n, np.uint8)
        R_new = np.empty(n, np.float32)
        rc = self.lib.adacomp_oracle_pack_layer(self._f(residue), self._f(dW), n, T, rule, soft_factor, self._f(G),
                                                self._f(H), self._f(gmax), self._f(scale),
                                                sel.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                                self._f(R_new))
        if rc < 0:
            raise ValueError(f"adacomp_oracle_pack_layer failed: {rc}")
        return {"G": G, "H": H, "gmax": gmax, "scale": scale[0], "selected": sel.astype(bool),
                "residue": R_new, "n_selected": int(rc)}

    def packet_bound(self, layers) -> int:
        return int(self.lib.adacomp_oracle_packet_bound(_layer_array(layers), len(layers)))

    def compress(self, layers, grad, residue, capacity=None, rule=RULE_UNION, soft_factor=2.0):
        """pack() over a layer table; ``residue`` (numpy float32) is updated in place.
        Returns the packet as a uint8 array of exactly total_bytes.  Raises on error codes."""
        assert grad.dtype == np.float32 and residue.dtype == np.float32
        assert grad.flags.c_contiguous and residue.flags.c_contiguous
        cap = self.packet_bound(layers) if capacity is None else int(capacity)
        if cap == 0:
            raise OracleError(self.lib.adacomp_oracle_compress(
                _layer_array(layers), len(layers), self._f(grad), self._f(residue), None, 0, rule, soft_factor))
        buf = np.zeros(cap, np.uint8)
        rc = self.lib.adacomp_oracle_compress(_layer_array(layers), len(layers), self._f(grad),
                                              self._f(residue), buf.ctypes.data, cap, rule, soft_factor)
        if rc < 0:
            raise OracleError(rc)
        return buf[:rc].copy()

    def unpack_accumulate(self, layers, packets, n_total):
        """Sum of the decoded packets, learner 0 first; returns a float32 array of n_total
        elements (elements outside every layer keep the fill value NaN)."""
        dense = np.full(n_total, np.nan, np.float32)
        keep = [np.ascontiguousarray(p, dtype=np.uint8) for p in packets]
        ptrs = (ctypes.c_void_p * max(1, len(keep)))(*[p.ctypes.data for p in keep])
        rc = self.lib.adacomp_oracle_unpack_accumulate(_layer_array(layers), len(layers), ptrs,
                                                       len(keep), self._f(dense))
        if rc != 0:
            raise OracleError(rc)
        return dense


    def update_sgd(self, layers, dense_sum, n_learners, weights, momentum_buf, lr, momentum):
        """averageGradients + SGD-with-momentum step, in place on weights and momentum_buf."""
        rc = self.lib.adacomp_oracle_update_sgd(_layer_array(layers), len(layers), self._f(dense_sum), n_learners,
                                                self._f(weights), self._f(momentum_buf), lr, momentum)
        if rc != 0:
            raise OracleError(rc)

    def update_adam(self, layers, dense_sum, n_learners, weights, m_buf, v_buf, lr, beta1, beta2, eps, bias1, bias2):
        """averageGradients + Adam step, in place on weights, m_buf and v_buf."""
        rc = self.lib.adacomp_oracle_update_adam(_layer_array(layers), len(layers), self._f(dense_sum), n_learners,
                                                 self._f(weights), self._f(m_buf), self._f(v_buf), lr, beta1, beta2,
                                                 eps, bias1, bias2)
        if rc != 0:
            raise OracleError(rc)


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle error {code}")
        self.code = int(code)
