"""ctypes front end of the fp64 log-domain CPU oracle (lfmmi_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
cpu_baseline leg of the benchmark. Nothing in the product package imports it,
and it imports nothing from the product package.

    forward_backward(graph, logits, lengths, leak) -> (logz[B], gamma[B,T,P])
    loss(num_graphs, den_graph, logits, lengths, leak) -> (objf[B], grad[B,T,P])

`graph` is a dict of plain arrays (num_states, num_pdfs, src, dst, pdf, logw,
init_prob, final_prob). Eq. 2: objf = log P(X|G_num) - log P(X|G_den);
Eq. 3: grad = gamma_num - gamma_den.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lfmmi_oracle.c")
_LIB = os.path.join(_HERE, "liblfmmi_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (OpenMP over sequences)."""
    if force or not os.path.exists(_LIB) or \
            os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.lfmmi_oracle_forward_backward.restype = ctypes.c_int
        lib.lfmmi_oracle_forward_backward.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_long, i32p, i32p, i32p, f32p,
            f32p, f32p, ctypes.c_double, ctypes.c_int, ctypes.c_int, f32p, i32p,
            f64p, f64p, f64p, ctypes.c_int]
        lib.lfmmi_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads():
    return int(_load().lfmmi_oracle_max_threads())


def _p(arr, ctype):
    return arr.ctypes.data_as(ctypes.POINTER(ctype))


def forward_backward(graph, logits, lengths, leak, want_gamma=True,
                     num_threads=0, return_bwd_total=False):
    """log Z per sequence and pdf occupancies gamma = d logZ / d logits."""
    lib = _load()
    src = np.ascontiguousarray(graph["src"], dtype=np.int32)
    dst = np.ascontiguousarray(graph["dst"], dtype=np.int32)
    pdf = np.ascontiguousarray(graph["pdf"], dtype=np.int32)
    logw = np.ascontiguousarray(graph["logw"], dtype=np.float32)
    pi = np.ascontiguousarray(graph["init_prob"], dtype=np.float32)
    fin = np.ascontiguousarray(graph["final_prob"], dtype=np.float32)
    x = np.ascontiguousarray(logits, dtype=np.float32)
    lens = np.ascontiguousarray(lengths, dtype=np.int32)
    B, T, P = x.shape
    S = int(graph["num_states"])
    if int(graph["num_pdfs"]) != P or len(lens) != B:
        raise ValueError("shape mismatch")
    if len(pi) != S or len(fin) != S:
        raise ValueError("init/final length mismatch")
    logz = np.zeros(B, dtype=np.float64)
    logz_b = np.zeros(B, dtype=np.float64)
    gamma = np.zeros((B, T, P), dtype=np.float64) if want_gamma else None
    rc = lib.lfmmi_oracle_forward_backward(
        S, P, len(src), _p(src, ctypes.c_int), _p(dst, ctypes.c_int),
        _p(pdf, ctypes.c_int), _p(logw, ctypes.c_float), _p(pi, ctypes.c_float),
        _p(fin, ctypes.c_float), float(leak), B, T, _p(x, ctypes.c_float),
        _p(lens, ctypes.c_int), _p(logz, ctypes.c_double),
        _p(logz_b, ctypes.c_double),
        _p(gamma, ctypes.c_double) if want_gamma else None, int(num_threads))
    if rc != 0:
        raise RuntimeError("oracle failed with code %d" % rc)
    if return_bwd_total:
        return logz, gamma, logz_b
    return logz, gamma


def forward_backward_per_utt(graphs, logits, lengths, leak, want_gamma=True):
    """One graph per sequence (numerators): graphs[b] goes with logits[b]."""
    B, T, P = logits.shape
    logz = np.zeros(B, dtype=np.float64)
    gamma = np.zeros((B, T, P), dtype=np.float64) if want_gamma else None
    for b in range(B):
        lz, g = forward_backward(graphs[b], logits[b:b + 1], lengths[b:b + 1],
                                 leak, want_gamma)
        logz[b] = lz[0]
        if want_gamma:
            gamma[b] = g[0]
    return logz, gamma


def loss(num_graphs, den_graph, logits, lengths, leak):
    """Eq. 2 and Eq. 3: (logZ_num - logZ_den, gamma_num - gamma_den), plus the
    two log-likelihood vectors for separate comparison."""
    lz_n, g_n = forward_backward_per_utt(num_graphs, logits, lengths, leak)
    lz_d, g_d = forward_backward(den_graph, logits, lengths, leak)
    return lz_n - lz_d, g_n - g_d, lz_n, lz_d
