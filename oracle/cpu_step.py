"""ctypes wrapper of cpu_step.c, the plain C/OpenMP baseline of one MoE decode layer step.

TEST / BENCHMARK INFRASTRUCTURE ONLY (like everything under oracle/): used by the benchmark's
CPU-baseline leg and by a CPU test that checks it against moei_oracle.  The product never loads it.
"""
from __future__ import annotations

import ctypes as C
import os
import shutil
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "cpu_step.c")
LIB = os.path.join(_HERE, "libcpu_step.so")
_lib = None


def build() -> str:
    """gcc -O2 -fopenmp: scalar loops, no fast-math (the sums keep their written order)."""
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        raise RuntimeError("no C compiler for oracle/cpu_step.c")
    cmd = [cc, "-O2", "-fopenmp", "-fPIC", "-shared", "-std=gnu11", "-Wall", SRC, "-o", LIB + ".tmp", "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("gcc failed:\n" + r.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
            build()
        _lib = C.CDLL(LIB)
        _lib.cpu_decode_step.restype = C.c_int
        _lib.cpu_threads_available.restype = C.c_int
    return _lib


def threads_available() -> int:
    return int(lib().cpu_threads_available())


def _ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def pointer_table(triples) -> np.ndarray:
    """[n][3] addresses of (W_gate, W_up, W_down) arrays; the arrays must stay alive."""
    out = np.zeros((len(triples), 3), dtype=np.uint64)
    for i, t in enumerate(triples):
        for j in range(3):
            out[i, j] = _ptr(t[j])
    return out


def decode_step(traces, eam, layer, W_r, bias, x, experts_tab, shared_tab, H, I, k, renorm, eps, resident, threads=1):
    """One layer step; ``eam`` (int64 [L][E]) is updated in place.  Weights are fp32 or uint16
    (bf16 bit patterns); ``experts_tab`` / ``shared_tab`` come from ``pointer_table``."""
    traces = np.ascontiguousarray(traces, dtype=np.int32)
    N = traces.shape[0]
    L, E = eam.shape
    assert eam.dtype == np.int64 and eam.flags["C_CONTIGUOUS"]
    bf = 1 if W_r.dtype == np.uint16 else 0
    assert x.dtype == W_r.dtype
    LE = L * E
    idx = np.zeros(k, dtype=np.int32)
    w = np.zeros(k, dtype=np.float64)
    best, n_pf, n_ev = C.c_int32(-1), C.c_int32(0), C.c_int32(0)
    sim = C.c_double(0.0)
    P, V = np.zeros(LE), np.zeros(LE)
    pf, ev = np.zeros(LE, dtype=np.int32), np.zeros(LE, dtype=np.int32)
    y = np.zeros(H, dtype=np.float64)
    res = np.ascontiguousarray(np.asarray(resident).reshape(-1).astype(np.uint8))
    bias32 = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    n_shared = 0 if shared_tab is None else int(shared_tab.shape[0])
    rc = lib().cpu_decode_step(
        C.c_void_p(_ptr(traces) if N else 0), N, L, E, C.c_void_p(_ptr(eam)), layer, C.c_void_p(_ptr(W_r)),
        C.c_void_p(_ptr(bias32) if bias32 is not None else 0), C.c_void_p(_ptr(x)), H, I, bf, k, int(bool(renorm)),
        C.c_double(eps), C.c_void_p(_ptr(experts_tab)), C.c_void_p(_ptr(shared_tab) if n_shared else 0), n_shared,
        C.c_void_p(_ptr(res)), threads, C.c_void_p(_ptr(idx)), C.c_void_p(_ptr(w)), C.byref(best), C.byref(sim),
        C.c_void_p(_ptr(P)), C.c_void_p(_ptr(V)), C.c_void_p(_ptr(pf)), C.byref(n_pf), C.c_void_p(_ptr(ev)),
        C.byref(n_ev), C.c_void_p(_ptr(y)))
    if rc != 0:
        raise RuntimeError(f"cpu_decode_step failed with code {rc}")
    return dict(idx=idx, w=w, best=best.value, sim=sim.value, P=P.reshape(L, E), V=V.reshape(L, E),
                pf_order=pf[:n_pf.value].tolist(), ev_order=ev[:n_ev.value].tolist(), y=y)
