"""ctypes access to the CPU oracle (``bitsnap_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It knows nothing about the HIP library and imports nothing from it.
Inputs and outputs are flat numpy arrays; bf16/fp16 values travel as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bitsnap_oracle.c")
_LIB = os.path.join(_HERE, "libbitsnap_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -O2 only, no fast-math, no FMA contraction."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = C.CDLL(_LIB)
    p = C.c_void_p
    i64 = C.c_int64
    L.oracle_encode_sparse.argtypes = [p, p, i64, p, p]
    L.oracle_encode_sparse.restype = i64
    L.oracle_encode_sparse_naive.argtypes = [p, p, i64, p, p]
    L.oracle_encode_sparse_naive.restype = i64
    L.oracle_tile_offsets.argtypes = [p, i64, i64, p]
    L.oracle_tile_offsets.restype = None
    L.oracle_decode_sparse.argtypes = [p, p, p, i64, p]
    L.oracle_encode_sparse_ex.argtypes = [p, p, i64, C.c_int, p, p, p]
    L.oracle_encode_sparse_ex.restype = i64
    L.oracle_decode_sparse_ex.argtypes = [p, p, p, i64, C.c_int, p]
    L.oracle_decode_sparse_ex.restype = None
    L.oracle_encode_sparse32_ex.argtypes = [p, p, i64, C.c_int, p, p, p]
    L.oracle_encode_sparse32_ex.restype = i64
    L.oracle_decode_sparse32_ex.argtypes = [p, p, p, i64, C.c_int, p]
    L.oracle_decode_sparse32_ex.restype = None
    L.oracle_decode_sparse.restype = None
    L.oracle_norm_quantile.argtypes = [C.c_int, C.c_int]
    L.oracle_norm_quantile.restype = C.c_double
    L.oracle_cluster_fit.argtypes = [p, i64, p, p]
    L.oracle_cluster_fit.restype = None
    L.oracle_cluster_edges.argtypes = [C.c_float, C.c_float, C.c_int, p]
    L.oracle_cluster_edges.restype = None
    L.oracle_quantize_cluster.argtypes = [p, i64, i64, C.c_int, p, p, p, p, p]
    L.oracle_quantize_cluster.restype = None
    L.oracle_dequantize_cluster.argtypes = [p, p, p, i64, i64, C.c_int, p]
    L.oracle_dequantize_cluster.restype = None
    L.oracle_quantize_cluster_ex.argtypes = [p, i64, i64, C.c_int, p, p, C.c_int, p, p, p, p]
    L.oracle_quantize_cluster_ex.restype = None
    L.oracle_dequantize_cluster_ex.argtypes = [p, p, p, i64, i64, C.c_int, p, C.c_int, p]
    L.oracle_dequantize_cluster_ex.restype = None
    L.oracle_code_qmap_bruteforce.argtypes = [C.c_float, C.c_float, C.c_float, p, p]
    L.oracle_code_qmap_bruteforce.restype = C.c_int
    L.oracle_code_bruteforce.argtypes = [C.c_float, C.c_float, C.c_float, p]
    L.oracle_code_bruteforce.restype = C.c_int
    _lib = L
    return L


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16 and a.ndim == 1
    return a


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32 and a.ndim == 1
    return a


# ---------------------------------------------------------------------------------------------
# sparse path
# ---------------------------------------------------------------------------------------------
def encode_sparse(cur, base) -> Tuple[np.ndarray, np.ndarray, int]:
    """-> (mask[ceil(n/8)] uint8, payload[n_c] uint16, n_c)."""
    cur, base = _u16(cur), _u16(base)
    n = cur.size
    assert base.size == n
    mask = np.empty((n + 7) // 8, np.uint8)
    payload = np.empty(max(n, 1), np.uint16)
    nc = _load().oracle_encode_sparse(_ptr(cur), _ptr(base), n, _ptr(mask), _ptr(payload))
    return mask, payload[:nc].copy(), int(nc)


def encode_sparse_ex(cur, base, delta: bool = False, new_base=None) -> Tuple[np.ndarray, np.ndarray, int]:
    """Extended form: delta payload (cur XOR base) and / or a copy of cur into new_base (a uint16 array, which
    may be `base` itself).  -> (mask, payload[n_c], n_c)."""
    cur = _u16(cur)
    n = cur.size
    assert base.dtype == np.uint16 and base.flags.c_contiguous and base.size == n
    if new_base is not None:
        assert new_base.dtype == np.uint16 and new_base.flags.c_contiguous and new_base.size == n
    mask = np.empty((n + 7) // 8, np.uint8)
    payload = np.empty(max(n, 1), np.uint16)
    nc = _load().oracle_encode_sparse_ex(_ptr(cur), _ptr(base), n, int(bool(delta)), _ptr(mask), _ptr(payload),
                                         None if new_base is None else _ptr(new_base))
    return mask, payload[:nc].copy(), int(nc)


def decode_sparse_ex(base, mask, payload, delta: bool = False) -> np.ndarray:
    base, payload = _u16(base), _u16(payload)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    n = base.size
    out = np.empty(max(n, 1), np.uint16)
    pay = payload if payload.size else np.zeros(1, np.uint16)
    _load().oracle_decode_sparse_ex(_ptr(base), _ptr(mask), _ptr(pay), n, int(bool(delta)), _ptr(out))
    return out[:n].copy()


def _u32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint32 and a.ndim == 1
    return a


def encode_sparse32(cur, base, delta: bool = False, new_base=None) -> Tuple[np.ndarray, np.ndarray, int]:
    """32-bit elements (bit patterns as uint32).  -> (mask[ceil(n/8)], payload[n_c] uint32, n_c)."""
    cur = _u32(cur)
    n = cur.size
    assert base.dtype == np.uint32 and base.flags.c_contiguous and base.size == n
    if new_base is not None:
        assert new_base.dtype == np.uint32 and new_base.flags.c_contiguous and new_base.size == n
    mask = np.empty((n + 7) // 8, np.uint8)
    payload = np.empty(max(n, 1), np.uint32)
    nc = _load().oracle_encode_sparse32_ex(_ptr(cur), _ptr(base), n, int(bool(delta)), _ptr(mask), _ptr(payload),
                                           None if new_base is None else _ptr(new_base))
    return mask, payload[:nc].copy(), int(nc)


def decode_sparse32(base, mask, payload, delta: bool = False) -> np.ndarray:
    base, payload = _u32(base), _u32(payload)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    n = base.size
    out = np.empty(max(n, 1), np.uint32)
    pay = payload if payload.size else np.zeros(1, np.uint32)
    _load().oracle_decode_sparse32_ex(_ptr(base), _ptr(mask), _ptr(pay), n, int(bool(delta)), _ptr(out))
    return out[:n].copy()


def encode_sparse_naive(cur, base) -> Tuple[np.ndarray, np.ndarray, int]:
    cur, base = _u16(cur), _u16(base)
    n = cur.size
    flags = np.empty(max(n, 1), np.uint8)
    payload = np.empty(max(n, 1), np.uint16)
    nc = _load().oracle_encode_sparse_naive(_ptr(cur), _ptr(base), n, _ptr(flags), _ptr(payload))
    return flags[:n].copy(), payload[:nc].copy(), int(nc)


def tile_offsets(mask, n: int, tile: int) -> np.ndarray:
    """-> uint64[ceil(n/tile)+1]; entry t counts set bits before element t*tile."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    ntiles = (n + tile - 1) // tile
    off = np.zeros(ntiles + 1, np.uint64)
    _load().oracle_tile_offsets(_ptr(mask), n, tile, _ptr(off))
    return off


def decode_sparse(base, mask, payload) -> np.ndarray:
    base = _u16(base)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    payload = np.ascontiguousarray(payload, dtype=np.uint16)
    out = np.empty(base.size, np.uint16)
    _load().oracle_decode_sparse(_ptr(base), _ptr(mask), _ptr(payload), base.size, _ptr(out))
    return out


# ---------------------------------------------------------------------------------------------
# cluster path
# ---------------------------------------------------------------------------------------------
def norm_quantile(k: int, m: int) -> float:
    return float(_load().oracle_norm_quantile(k, m))


def cluster_fit(x) -> Tuple[np.float32, np.float32]:
    x = _f32(x)
    mu = C.c_float()
    sg = C.c_float()
    _load().oracle_cluster_fit(_ptr(x), x.size, C.byref(mu), C.byref(sg))
    return np.float32(mu.value), np.float32(sg.value)


def cluster_edges(mu, sigma, m: int) -> np.ndarray:
    e = np.zeros(16, np.float32)
    _load().oracle_cluster_edges(C.c_float(float(mu)), C.c_float(float(sigma)), m, _ptr(e))
    return e[: m - 1].copy()


def n_groups(n: int, G: int) -> int:
    if n <= 0:
        return 0
    if G <= 0 or G > n:
        G = n
    return (n + G - 1) // G


def quantize_cluster(x, G: int = 4096, m: int = 16, fit_in=None):
    """-> dict(codes uint8[n], labels uint8[ceil(n/2)], params f32[groups,m,2] = (S,b),
    fit f32[groups, 2+m-1] = (mu, sigma, e_1..e_{m-1}))."""
    x = _f32(x)
    n = x.size
    g = n_groups(n, G)
    codes = np.zeros(n, np.uint8)
    labels = np.zeros((n + 1) // 2, np.uint8)
    params = np.zeros((g, m, 2), np.float32)
    fit = np.zeros((g, 2 + m - 1), np.float32)
    fi = None
    if fit_in is not None:
        fi = np.ascontiguousarray(fit_in, dtype=np.float32).reshape(g, 2)
    _load().oracle_quantize_cluster(_ptr(x), n, G, m, _ptr(fi), _ptr(codes), _ptr(labels), _ptr(params), _ptr(fit))
    return dict(codes=codes, labels=labels, params=params, fit=fit)


def dequantize_cluster(codes, labels, params, n: int, G: int = 4096, m: int = 16) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    labels = np.ascontiguousarray(labels, dtype=np.uint8)
    params = np.ascontiguousarray(params, dtype=np.float32)
    out = np.zeros(n, np.float32)
    _load().oracle_dequantize_cluster(_ptr(codes), _ptr(labels), _ptr(params), n, G, m, _ptr(out))
    return out


def _qmap(qmap) -> Optional[np.ndarray]:
    if qmap is None:
        return None
    q = np.ascontiguousarray(qmap, dtype=np.float32)
    assert q.shape == (256,)
    return q


def quantize_cluster_ex(x, G: int = 4096, m: int = 16, fit_in=None, qmap=None, cluster_major: bool = False):
    """Format variants: a 256-entry map Q (None = linear) and / or cluster-major codes.  Same dict as quantize_cluster."""
    x = _f32(x)
    n = x.size
    g = n_groups(n, G)
    codes = np.zeros(n, np.uint8)
    labels = np.zeros((n + 1) // 2, np.uint8)
    params = np.zeros((g, m, 2), np.float32)
    fit = np.zeros((g, 2 + m - 1), np.float32)
    fi = None
    if fit_in is not None:
        fi = np.ascontiguousarray(fit_in, dtype=np.float32).reshape(g, 2)
    _load().oracle_quantize_cluster_ex(_ptr(x), n, G, m, _ptr(fi), _ptr(_qmap(qmap)), int(bool(cluster_major)),
                                       _ptr(codes), _ptr(labels), _ptr(params), _ptr(fit))
    return dict(codes=codes, labels=labels, params=params, fit=fit)


def dequantize_cluster_ex(codes, labels, params, n: int, G: int = 4096, m: int = 16, qmap=None,
                          cluster_major: bool = False) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    labels = np.ascontiguousarray(labels, dtype=np.uint8)
    params = np.ascontiguousarray(params, dtype=np.float32)
    out = np.zeros(n, np.float32)
    _load().oracle_dequantize_cluster_ex(_ptr(codes), _ptr(labels), _ptr(params), n, G, m, _ptr(_qmap(qmap)),
                                         int(bool(cluster_major)), _ptr(out))
    return out


def code_qmap_bruteforce(x, b, S, qmap) -> Tuple[int, float]:
    gap = C.c_double()
    q = _qmap(qmap)
    j = _load().oracle_code_qmap_bruteforce(C.c_float(float(x)), C.c_float(float(b)), C.c_float(float(S)), _ptr(q),
                                            C.byref(gap))
    return int(j), float(gap.value)


def code_bruteforce(x, b, S) -> Tuple[int, float]:
    gap = C.c_double()
    j = _load().oracle_code_bruteforce(C.c_float(float(x)), C.c_float(float(b)), C.c_float(float(S)), C.byref(gap))
    return int(j), float(gap.value)


def unpack_labels(labels, n: int) -> np.ndarray:
    """uint4 pairs -> one uint8 label per element (layout helper for tests, no codec arithmetic)."""
    labels = np.ascontiguousarray(labels, dtype=np.uint8)
    out = np.empty(labels.size * 2, np.uint8)
    out[0::2] = labels & 15
    out[1::2] = labels >> 4
    return out[:n]
