"""TEST INFRASTRUCTURE ONLY -- ctypes front end of the fp64 attention oracle.

Compiles ``tree_attention_oracle.c`` with gcc on first use (the checker is plain
C with OpenMP over (query, head)) and exposes it as ``tree_attention``.
The computation follows the definition in Section 3.1 of the paper:
softmax(q K^T / sqrt(d)) V over exactly the tokens on the query's tree path.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tree_attention_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_tree_attention.so")
_handle = None


def library_path() -> str:
    return _LIB


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc, -O2, OpenMP). Returns the path of the shared object."""
    global _handle
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        _handle = None
    return _LIB


def _lib():
    global _handle
    if _handle is None:
        build()
        h = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f32p = ctypes.POINTER(ctypes.c_float)
        h.oracle_tree_attention.restype = ctypes.c_int
        h.oracle_tree_attention.argtypes = [
            f32p, f32p, f32p, ctypes.POINTER(ctypes.c_double),
            i32p, i32p, i32p, ctypes.c_int32, i32p, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_int32, i32p,
        ]
        h.oracle_tree_attention_extents.restype = ctypes.c_int
        h.oracle_tree_attention_extents.argtypes = [
            f32p, f32p, f32p, ctypes.POINTER(ctypes.c_double),
            i32p, i32p, i32p, i32p, ctypes.c_int32, i32p, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_int32, i32p,
        ]
        _handle = h
    return _handle


def _as_f32(x) -> np.ndarray:
    """float32 numpy view of a numpy array or a torch tensor (bf16 widens exactly)."""
    if hasattr(x, "detach"):
        x = x.detach().to("cpu").float().numpy()
    x = np.asarray(x)
    if x.dtype == np.float64:
        y = x.astype(np.float32)
        if not np.array_equal(y.astype(np.float64), x):
            raise ValueError("oracle inputs must be exactly representable in float32")
        x = y
    return np.ascontiguousarray(x, dtype=np.float32)


def _as_i32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=np.int32)


def tree_attention(Q, K, V, node_tok_begin, node_tok_len, node_parent, query_node,
                   scale: float | None = None, nthreads: int = 0, return_threads: bool = False):
    """O[j,h,:] = softmax(scale * Q[j,h] . K[path(j), h//G]) V[path(j), h//G] in fp64.

    Q: [nq,Hq,d]; K, V: [ntok,Hkv,d] (numpy float32/float64 or torch tensors);
    returns a float64 array [nq,Hq,d].  scale defaults to 1/sqrt(d).
    """
    q, k, v = _as_f32(Q), _as_f32(K), _as_f32(V)
    nq, Hq, d = q.shape
    ntok, Hkv, d2 = k.shape
    assert v.shape == k.shape and d2 == d
    nb, nl, npar, qn = map(_as_i32, (node_tok_begin, node_tok_len, node_parent, query_node))
    assert qn.shape[0] == nq
    if scale is None:
        scale = 1.0 / float(np.sqrt(d))
    out = np.zeros((nq, Hq, d), dtype=np.float64)
    used = ctypes.c_int32(0)
    i32p = ctypes.POINTER(ctypes.c_int32)
    f32p = ctypes.POINTER(ctypes.c_float)
    rc = _lib().oracle_tree_attention(
        q.ctypes.data_as(f32p), k.ctypes.data_as(f32p), v.ctypes.data_as(f32p),
        out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        nb.ctypes.data_as(i32p), nl.ctypes.data_as(i32p), npar.ctypes.data_as(i32p), nb.shape[0],
        qn.ctypes.data_as(i32p), nq, ntok, Hq, Hkv, d, float(scale), int(nthreads), ctypes.byref(used))
    if rc != 0:
        raise ValueError(f"oracle_tree_attention failed with code {rc}")
    if return_threads:
        return out, int(used.value)
    return out


def tree_attention_paged(Q, K, V, node_page_ptr, page_ids, page_size, node_tok_len, node_parent, query_node,
                         scale: float | None = None, nthreads: int = 0):
    """The same attention over a paged pool: K, V are [n_pool_pages * page_size, Hkv, d] and token t of node u
    is row page_ids[node_page_ptr[u] + t // page_size] * page_size + t % page_size (Section 4.2).  Every page
    becomes one extent of the node, in order; nothing is merged or moved."""
    q, k, v = _as_f32(Q), _as_f32(K), _as_f32(V)
    nq, Hq, d = q.shape
    ntok, Hkv, _ = k.shape
    pp, pg, nl, npar, qn = map(_as_i32, (node_page_ptr, page_ids, node_tok_len, node_parent, query_node))
    P = int(page_size)
    ext_ptr, ext_begin, ext_len = [0], [], []
    for u in range(nl.shape[0]):
        left, i = int(nl[u]), 0
        while left > 0:
            ext_begin.append(int(pg[pp[u] + i]) * P)
            ext_len.append(min(P, left))
            left -= P
            i += 1
        ext_ptr.append(len(ext_len))
    ep, eb, el = map(_as_i32, (ext_ptr, ext_begin if ext_begin else [0], ext_len if ext_len else [0]))
    if scale is None:
        scale = 1.0 / float(np.sqrt(d))
    out = np.zeros((nq, Hq, d), dtype=np.float64)
    i32p = ctypes.POINTER(ctypes.c_int32)
    f32p = ctypes.POINTER(ctypes.c_float)
    rc = _lib().oracle_tree_attention_extents(
        q.ctypes.data_as(f32p), k.ctypes.data_as(f32p), v.ctypes.data_as(f32p),
        out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        ep.ctypes.data_as(i32p), eb.ctypes.data_as(i32p), el.ctypes.data_as(i32p), npar.ctypes.data_as(i32p),
        nl.shape[0], qn.ctypes.data_as(i32p), nq, ntok, Hq, Hkv, d, float(scale), int(nthreads), None)
    if rc != 0:
        raise ValueError(f"oracle_tree_attention_extents failed with code {rc}")
    return out
