"""The C form of the attention oracle (oracle/attention_ref.c) -- TEST INFRASTRUCTURE.

Same definition as OracleTree.attention, written as plain loops in C and spread over threads by
requested node, so that benchmark-sized trees can be checked on every output row and timed as
the CPU baseline.  The tree (nodes, decoding of bf16 / e4m3 bits to fp64) stays the Python
OracleTree; this module hands the fp64 pieces of every root-to-node path to the C routine,
which materialises each branch contiguously and evaluates fp64 attention on it.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "attention_ref.c")
LIB_PATH = os.path.join(HERE, "libspex_oracle.so")

_lib = None


def build(verbose: bool = False) -> str:
    """Compile the C oracle (always recompiles); returns the path of the shared library."""
    cmd = ["gcc", "-O3", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           SOURCE, "-o", LIB_PATH, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stderr)
    return LIB_PATH


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH) or os.path.getmtime(LIB_PATH) < os.path.getmtime(SOURCE):
            build()
        lib = ctypes.CDLL(LIB_PATH)
        lib.spex_oracle_attention.restype = ctypes.c_int
        lib.spex_oracle_attention.argtypes = [
            ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def attention(tree, leaves: Sequence[int], q_lens: Optional[Sequence[int]], q: np.ndarray,
              sm_scale: float, draft_masks: Optional[Sequence[int]] = None, threads: int = 0):
    """out [rows, Hq, D], lse [rows, Hq] and a dict {materialise_s, attention_s (thread-seconds,
    summed over threads), threads} for the requested nodes of an OracleTree."""
    lib = load()
    n = len(leaves)
    if q_lens is None:
        q_lens = [1] * n
    q = np.ascontiguousarray(q, dtype=np.float64)
    rows = int(sum(q_lens))
    assert q.shape == (rows, tree.Hq, tree.D)
    indptr = [0]
    k_ptrs, v_ptrs, toks, keep = [], [], [], []
    for leaf in leaves:
        for u in tree.path(leaf):
            for a, b in zip(tree.K[u], tree.V[u]):
                if a is None:
                    raise ValueError(f"node {u} holds tokens without values")
                a = np.ascontiguousarray(a, dtype=np.float64)
                b = np.ascontiguousarray(b, dtype=np.float64)
                keep.append((a, b))
                k_ptrs.append(a.ctypes.data)
                v_ptrs.append(b.ctypes.data)
                toks.append(a.shape[0])
        indptr.append(len(toks))
    indptr = np.asarray(indptr, dtype=np.int64)
    k_ptrs = np.asarray(k_ptrs, dtype=np.uint64)
    v_ptrs = np.asarray(v_ptrs, dtype=np.uint64)
    toks = np.asarray(toks, dtype=np.int64)
    ql = np.asarray(q_lens, dtype=np.int32)
    q_off = np.concatenate([[0], np.cumsum(ql[:-1], dtype=np.int64)]).astype(np.int64) if n else \
        np.zeros(0, dtype=np.int64)
    masks = None
    if draft_masks is not None:
        masks = np.asarray([int(m) for m in draft_masks], dtype=np.uint32)
        assert masks.shape == (rows,)
    out = np.zeros((rows, tree.Hq, tree.D))
    lse = np.zeros((rows, tree.Hq))
    seconds = np.zeros(2)
    used = ctypes.c_int32(0)

    def ptr(a):
        return None if a is None else a.ctypes.data

    rc = lib.spex_oracle_attention(n, ptr(indptr), ptr(k_ptrs), ptr(v_ptrs), ptr(toks), ptr(ql),
                                   ptr(q_off), ptr(q), ptr(masks), tree.Hq, tree.Hkv, tree.D,
                                   float(sm_scale), ptr(out), ptr(lse), int(threads), ptr(seconds),
                                   ctypes.byref(used))
    if rc > 0:
        raise ValueError(f"requested node {leaves[rc - 1]}: every query needs at least one visible "
                         "token, and masks may only name the request's drafts")
    if rc < 0:
        raise RuntimeError(f"spex_oracle_attention failed ({rc})")
    return out, lse, dict(materialise_s=float(seconds[0]), attention_s=float(seconds[1]),
                          threads=int(used.value))
