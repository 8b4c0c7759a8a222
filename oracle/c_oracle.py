"""Build and call the plain C oracle (decode_block_c.c) through ctypes.

TEST INFRASTRUCTURE ONLY (tests, smoke check, bench cpu_baseline leg).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "decode_block_c.c")
_LIB = os.path.join(_HERE, "liboracle_decode_block.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc (-O3, OpenMP, strict IEEE arithmetic)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.cfo_decode_block.argtypes = [u16p] * 5 + [ctypes.c_int] * 7 + [ctypes.c_double] + [f64p] * 5
        lib.cfo_decode_block.restype = ctypes.c_int
        lib.cfo_num_threads.restype = ctypes.c_int
        lib.cfo_set_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().cfo_num_threads())


def set_num_threads(n: int) -> None:
    _load().cfo_set_num_threads(int(n))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16
    return a, a.view(np.uint16).ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def decode_block(x, w_qkv, w_o, k_cache, v_cache, pos, n_q_heads, n_kv_heads, head_dim, rope_base):
    """Same contract as oracle.decode_block.decode_block; inputs must be fp16 arrays."""
    lib = _load()
    B, D = x.shape
    nq, nkv, d = int(n_q_heads), int(n_kv_heads), int(head_dim)
    max_seq = k_cache.shape[2]
    assert w_qkv.shape == (D, (nq + 2 * nkv) * d) and w_o.shape == (nq * d, D)
    assert k_cache.shape == (B, nkv, max_seq, d) and v_cache.shape == k_cache.shape
    keep = [_u16(a) for a in (x, w_qkv, w_o, k_cache, v_cache)]
    out = np.empty((B, D)); q_rot = np.empty((B, nq, d)); k_rot = np.empty((B, nkv, d))
    v_new = np.empty((B, nkv, d)); attn = np.empty((B, nq, d))
    f64p = ctypes.POINTER(ctypes.c_double)
    rc = lib.cfo_decode_block(*[k[1] for k in keep], B, D, nq, nkv, d, max_seq, int(pos), float(rope_base),
                              *[a.ctypes.data_as(f64p) for a in (out, q_rot, k_rot, v_new, attn)])
    if rc != 0:
        raise ValueError("cfo_decode_block rejected its arguments")
    return {"out": out, "q_rot": q_rot, "k_rot": k_rot, "v_new": v_new, "attn": attn}


def decode_layer(x, gamma, eps, w_qkv, w_o, k_cache, v_cache, pos, n_q_heads, n_kv_heads, head_dim, rope_base):
    """Same contract as oracle.decode_block.decode_layer; inputs must be fp16 arrays."""
    lib = _load()
    B, D = x.shape
    nq, nkv, d = int(n_q_heads), int(n_kv_heads), int(head_dim)
    max_seq = k_cache.shape[2]
    assert gamma.shape == (D,)
    assert w_qkv.shape == (D, (nq + 2 * nkv) * d) and w_o.shape == (nq * d, D)
    assert k_cache.shape == (B, nkv, max_seq, d) and v_cache.shape == k_cache.shape
    kx, kg = _u16(x), _u16(gamma)
    keep = [_u16(a) for a in (w_qkv, w_o, k_cache, v_cache)]
    out = np.empty((B, D)); q_rot = np.empty((B, nq, d)); k_rot = np.empty((B, nkv, d))
    v_new = np.empty((B, nkv, d)); attn = np.empty((B, nq, d))
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.cfo_decode_layer.restype = ctypes.c_int
    rc = lib.cfo_decode_layer(kx[1], kg[1], ctypes.c_double(float(eps)), *[k[1] for k in keep], B, D, nq, nkv, d, max_seq,
                              int(pos), ctypes.c_double(float(rope_base)),
                              *[a.ctypes.data_as(f64p) for a in (out, q_rot, k_rot, v_new, attn)])
    if rc != 0:
        raise ValueError("cfo_decode_layer rejected its arguments")
    return {"out": out, "q_rot": q_rot, "k_rot": k_rot, "v_new": v_new, "attn": attn}
