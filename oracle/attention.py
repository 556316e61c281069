"""ctypes front end of the fp64 definition oracle (attention_oracle.c).

TEST INFRASTRUCTURE ONLY.  Evaluates Eq. 1-2 of the paper per (request, query
head) over the request's concatenated root-to-leaf context (Sec. 4.1).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attention_oracle.c")
_LIB = os.path.join(_HERE, "libcodec_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.codec_oracle_decode_attention.restype = ctypes.c_int
        lib.codec_oracle_decode_attention.argtypes = [
            ctypes.c_int32, i32p, i32p, ctypes.c_int32, i32p, i32p, i32p, ctypes.c_int32,
            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
            u16p, u16p, u16p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_int64, i32p, i32p, i32p, ctypes.POINTER(ctypes.c_uint32), f64p, f64p, ctypes.c_int32]
        lib.codec_oracle_decode16.restype = ctypes.c_double
        lib.codec_oracle_decode16.argtypes = [ctypes.c_uint16, ctypes.c_int32]
        lib.codec_oracle_max_threads.restype = ctypes.c_int32
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def decode16(bits: int, dtype: int) -> float:
    return float(_load().codec_oracle_decode16(int(bits), int(dtype)))


def max_threads() -> int:
    return int(_load().codec_oracle_max_threads())


def decode_attention(parent, node_len, req_node, node_page_off, page_ids, page_size,
                     h_q, h_kv, d, dtype, scale, q_bits, k_bits, v_bits,
                     page_stride, token_stride, head_stride,
                     sel=None, nthreads: int = 0, req_mask_off=None, req_mask=None):
    """Returns (out [n, d] float64, lse [n] float64).

    ``sel``: optional list of (request, query head) pairs; default all pairs,
    request-major, reshaped by the caller as [B, h_q, d].
    ``req_mask_off`` [B + 1], ``req_mask`` (uint32 words): per-request visibility over the tokens of the
    request's last node (Sec. 4.1); a request without words sees everything.
    """
    lib = _load()
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    node_len = np.ascontiguousarray(node_len, dtype=np.int32)
    req_node = np.ascontiguousarray(req_node, dtype=np.int32)
    node_page_off = np.ascontiguousarray(node_page_off, dtype=np.int32)
    page_ids = np.ascontiguousarray(page_ids, dtype=np.int32)
    q_bits = np.ascontiguousarray(q_bits, dtype=np.uint16)
    k_bits = np.ascontiguousarray(k_bits, dtype=np.uint16)
    v_bits = np.ascontiguousarray(v_bits, dtype=np.uint16)
    b = req_node.shape[0]
    if sel is None:
        n = b * h_q
        sr = sh = None
    else:
        sel = np.asarray(sel, dtype=np.int32).reshape(-1, 2)
        n = sel.shape[0]
        sr = np.ascontiguousarray(sel[:, 0])
        sh = np.ascontiguousarray(sel[:, 1])
    mo = mw = None
    if req_mask_off is not None:
        mo = np.ascontiguousarray(req_mask_off, dtype=np.int32)
        mw = np.ascontiguousarray(req_mask, dtype=np.uint32)
        if mw.size == 0:
            mw = np.zeros(1, dtype=np.uint32)
    out = np.zeros((n, d), dtype=np.float64)
    lse = np.zeros(n, dtype=np.float64)
    rc = lib.codec_oracle_decode_attention(
        parent.shape[0], _p(parent, ctypes.c_int32), _p(node_len, ctypes.c_int32),
        b, _p(req_node, ctypes.c_int32), _p(node_page_off, ctypes.c_int32),
        _p(page_ids, ctypes.c_int32), page_size, h_q, h_kv, d, dtype, float(scale),
        _p(q_bits, ctypes.c_uint16), _p(k_bits, ctypes.c_uint16), _p(v_bits, ctypes.c_uint16),
        page_stride, token_stride, head_stride,
        n, _p(sr, ctypes.c_int32) if sr is not None else None,
        _p(sh, ctypes.c_int32) if sh is not None else None,
        _p(mo, ctypes.c_int32) if mo is not None else None,
        _p(mw, ctypes.c_uint32) if mw is not None else None,
        _p(out, ctypes.c_double), _p(lse, ctypes.c_double), nthreads)
    if rc != 0:
        raise ValueError(f"oracle rejected the forest (status {rc})")
    return out, lse


def decode_attention_workload(w, sel=None, nthreads: int = 0):
    """Run the oracle on a ``workloads.Workload``; full output comes back as [B, h_q, d]."""
    f, h, p = w.forest, w.head, w.paged
    out, lse = decode_attention(f.parent, f.node_len, f.req_node, p.node_page_off, p.page_ids,
                                p.page_size, h.num_q_heads, h.num_kv_heads, h.head_dim, h.dtype,
                                h.scale, w.q_bits(), w.k_bits(), w.v_bits(),
                                p.page_stride, p.token_stride, p.head_stride, sel, nthreads,
                                getattr(f, "req_mask_off", None), getattr(f, "req_mask", None))
    if sel is None:
        out = out.reshape(f.num_requests, h.num_q_heads, h.head_dim)
        lse = lse.reshape(f.num_requests, h.num_q_heads)
    return out, lse
