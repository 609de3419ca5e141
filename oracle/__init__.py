"""ctypes wrapper around the CPU oracle (oracle/spdnn_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library and its Python binding never
import this package, and this package never imports them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spdnn_oracle.cpp")
_LIB = os.path.join(_HERE, "libspdnn_oracle.so")
_lib = None

FRAGILE_EPS = 1e-4   # rows whose largest pre-activation is this close to zero are "fragile"


def build(force: bool = True) -> str:
    """Compile the oracle with g++ (single-threaded, -O2, hardware FMA)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-mfma", "-std=c++17", "-fPIC", "-shared", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build(force=True)
        lib = ctypes.CDLL(_LIB)
        pp_i = ctypes.POINTER(ctypes.c_void_p)
        for name in ("spdnn_oracle_infer", "spdnn_oracle_infer_f64"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_int32, ctypes.c_int32, pp_i, pp_i, ctypes.c_void_p,
                           ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double, ctypes.c_void_p]
        for name in ("spdnn_oracle_infer_csr", "spdnn_oracle_infer_csr_f64"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_int32, ctypes.c_int32, pp_i, pp_i, pp_i, ctypes.c_void_p,
                           ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double, ctypes.c_void_p]
        _lib = lib
    return _lib


class OracleResult:
    """n_active, active_rows (ascending original ids), Y (rows of Y_L for those
    ids), active_per_layer[l] = rows active on entry to layer l (entry L = final),
    fragile_layer[r] (first layer with |max pre-activation| < eps, else -1),
    layers_evaluated."""

    def __init__(self, n_active, active_rows, Y, active_per_layer, fragile_layer, layers_evaluated):
        self.n_active = n_active
        self.active_rows = active_rows
        self.Y = Y
        self.active_per_layer = active_per_layer
        self.fragile_layer = fragile_layer
        self.layers_evaluated = layers_evaluated


def infer(idx, val, bias, Y0, no_skip=False, f64=False, want_Y=True, fragile_eps=FRAGILE_EPS, ptr=None):
    """Run the oracle.

    idx: list of L int32 arrays [N, 32] (an entry may be None for a layer no
    active row reaches); val: list of L float32 arrays [N, 32]; bias: float32
    [N]; Y0: [batch, N] float32 (float64 if f64).  With ptr (list of L int32
    arrays [N+1]) the layers are general: neuron j of layer l owns entries
    ptr[l][j] .. ptr[l][j+1]-1 of the flat arrays idx[l] / val[l].  Returns
    OracleResult.
    """
    lib = _load()
    L = len(idx)
    assert len(val) == L and (ptr is None or len(ptr) == L)
    bias = np.ascontiguousarray(bias, dtype=np.float32)
    N = int(bias.shape[0])
    ft = np.float64 if f64 else np.float32
    Y0 = np.ascontiguousarray(Y0, dtype=ft)
    batch = int(Y0.shape[0])
    assert Y0.shape == (batch, N)
    keep = []
    ip = (ctypes.c_void_p * max(L, 1))()
    vp = (ctypes.c_void_p * max(L, 1))()
    pp = (ctypes.c_void_p * max(L, 1))()
    for l in range(L):
        if idx[l] is None:
            ip[l] = None
            vp[l] = None
            pp[l] = None
            continue
        a = np.ascontiguousarray(idx[l], dtype=np.int32)
        v = np.ascontiguousarray(val[l], dtype=np.float32)
        if ptr is None:
            assert a.shape == (N, 32) and v.shape == (N, 32), "layer %d: expected [N,32]" % l
        else:
            q = np.ascontiguousarray(ptr[l], dtype=np.int32)
            assert q.shape == (N + 1,) and q[0] == 0 and (np.diff(q) >= 0).all(), "layer %d: bad ptr" % l
            assert a.shape == (int(q[N]),) and v.shape == a.shape, "layer %d: expected ptr[N] entries" % l
            keep.append(q)
            pp[l] = q.ctypes.data
        if a.size and (a.min() < 0 or a.max() >= N):
            raise ValueError("layer %d: column index outside [0, N)" % l)
        keep.append((a, v))
        ip[l] = a.ctypes.data
        vp[l] = v.ctypes.data
    n_active = np.zeros(1, dtype=np.int32)
    rows = np.zeros(max(batch, 1), dtype=np.int32)
    Y = np.zeros((max(batch, 1), N), dtype=ft) if want_Y else None
    apl = np.zeros(L + 1, dtype=np.int32)
    frag = np.zeros(max(batch, 1), dtype=np.int32)
    nev = np.zeros(1, dtype=np.int32)
    if ptr is None:
        fn = lib.spdnn_oracle_infer_f64 if f64 else lib.spdnn_oracle_infer
        head = (N, L, ip, vp)
    else:
        fn = lib.spdnn_oracle_infer_csr_f64 if f64 else lib.spdnn_oracle_infer_csr
        head = (N, L, pp, ip, vp)
    rc = fn(*head, bias.ctypes.data, Y0.ctypes.data, batch, 1 if no_skip else 0,
            n_active.ctypes.data, rows.ctypes.data, Y.ctypes.data if want_Y else None,
            apl.ctypes.data, frag.ctypes.data, float(fragile_eps), nev.ctypes.data)
    if rc == -2:
        raise RuntimeError("oracle: an active row reached a layer whose weights were not provided")
    if rc != 0:
        raise RuntimeError("oracle: bad arguments (rc=%d)" % rc)
    n = int(n_active[0])
    return OracleResult(n, rows[:n].copy(), Y[:n].copy() if want_Y else None, apl, frag[:batch].copy(),
                        int(nev[0]))
