"""ctypes binding of libbitsnap.so: same names as the C ABI (include/bitsnap.h), argument
marshalling only.  Tensors are torch tensors on the MI355X; torch supplies device memory and the
current HIP stream, every step of the codecs runs in the library's kernels.

There is no fallback: if the library has not been built (``python -m paper_2511_12376_amd.build``)
or cannot be loaded, every entry point raises ``BitsnapError``.
"""
from __future__ import annotations

import ctypes as C
import os
from types import SimpleNamespace
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbitsnap.so")

SYMBOLS = (
    "bitsnap_version", "bitsnap_error_string", "bitsnap_debug_stream_copy", "bitsnap_debug_stream_mix",
    "bitsnap_sparse_tile_elems", "bitsnap_sparse_tile_elems_for", "bitsnap_sparse_mask_bytes",
    "bitsnap_sparse_workspace_bytes", "bitsnap_sparse_workspace_bytes_for",
    "bitsnap_encode_sparse", "bitsnap_decode_sparse", "bitsnap_encode_sparse_ex", "bitsnap_decode_sparse_ex",
    "bitsnap_encode_sparse_batched_ex", "bitsnap_decode_sparse_batched_ex", "bitsnap_debug_set_spin_limit",
    "bitsnap_cluster_groups", "bitsnap_cluster_param_bytes", "bitsnap_cluster_label_bytes",
    "bitsnap_cluster_fit_floats", "bitsnap_cluster_workspace_bytes", "bitsnap_cluster_z",
    "bitsnap_quantize_cluster", "bitsnap_dequantize_cluster",
    "bitsnap_quantize_cluster_ex", "bitsnap_dequantize_cluster_ex", "bitsnap_cluster_workspace_bytes_ex",
    "bitsnap_quantize_cluster_batched_ex", "bitsnap_dequantize_cluster_batched_ex",
    "bitsnap_cluster_chunk_elems", "bitsnap_cluster_batch_workspace_bytes",
    "bitsnap_quantize_cluster_batched", "bitsnap_dequantize_cluster_batched",
    "bitsnap_sparse_batch_workspace_bytes", "bitsnap_encode_sparse_batched", "bitsnap_decode_sparse_batched",
    "bitsnap_encode_sparse_static",
)


class BitsnapError(RuntimeError):
    pass


_lib = None


def lib():
    """The loaded library.  Raises BitsnapError when it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise BitsnapError(f"{LIB_PATH} not found: build it with `python -m paper_2511_12376_amd.build`")
    try:
        L = C.CDLL(LIB_PATH)
    except OSError as e:  # e.g. no HIP runtime on this machine
        raise BitsnapError(f"cannot load {LIB_PATH}: {e}") from e
    p, i64, sz, i = C.c_void_p, C.c_int64, C.c_size_t, C.c_int
    L.bitsnap_version.argtypes, L.bitsnap_version.restype = [], i
    L.bitsnap_error_string.argtypes, L.bitsnap_error_string.restype = [i], C.c_char_p
    L.bitsnap_debug_stream_copy.argtypes, L.bitsnap_debug_stream_copy.restype = [p, p, i64, p], i
    L.bitsnap_debug_stream_mix.argtypes, L.bitsnap_debug_stream_mix.restype = [p, p, p, i64, i, p], i
    L.bitsnap_sparse_tile_elems.argtypes, L.bitsnap_sparse_tile_elems.restype = [], sz
    L.bitsnap_sparse_mask_bytes.argtypes, L.bitsnap_sparse_mask_bytes.restype = [i64], sz
    L.bitsnap_sparse_workspace_bytes.argtypes, L.bitsnap_sparse_workspace_bytes.restype = [i64], sz
    L.bitsnap_encode_sparse.argtypes = [p, p, i64, i, p, p, i64, p, p, p, sz, p]
    L.bitsnap_encode_sparse.restype = i
    L.bitsnap_encode_sparse_static.argtypes = [p, p, i64, i, p, p, i64, p, p, p]
    L.bitsnap_encode_sparse_static.restype = i
    L.bitsnap_decode_sparse.argtypes = [p, p, p, i64, i64, i, p, p, p, sz, p]
    L.bitsnap_decode_sparse.restype = i
    L.bitsnap_encode_sparse_ex.argtypes = [p, p, i64, i, C.c_uint32, p, p, i64, p, p, p, p, sz, p]
    L.bitsnap_encode_sparse_ex.restype = i
    L.bitsnap_decode_sparse_ex.argtypes = [p, p, p, i64, i64, i, C.c_uint32, p, p, p, p, sz, p]
    L.bitsnap_decode_sparse_ex.restype = i
    L.bitsnap_encode_sparse_batched_ex.argtypes = [p, i64, i64, i, C.c_uint32, p, sz, p]
    L.bitsnap_encode_sparse_batched_ex.restype = i
    L.bitsnap_decode_sparse_batched_ex.argtypes = [p, i64, i64, i, C.c_uint32, p, sz, p]
    L.bitsnap_decode_sparse_batched_ex.restype = i
    L.bitsnap_sparse_tile_elems_for.argtypes, L.bitsnap_sparse_tile_elems_for.restype = [i], sz
    L.bitsnap_sparse_workspace_bytes_for.argtypes, L.bitsnap_sparse_workspace_bytes_for.restype = [i64, i], sz
    L.bitsnap_debug_set_spin_limit.argtypes, L.bitsnap_debug_set_spin_limit.restype = [C.c_uint32], None
    L.bitsnap_cluster_groups.argtypes, L.bitsnap_cluster_groups.restype = [i64, i64], sz
    L.bitsnap_cluster_param_bytes.argtypes, L.bitsnap_cluster_param_bytes.restype = [i64, i64, i], sz
    L.bitsnap_cluster_label_bytes.argtypes, L.bitsnap_cluster_label_bytes.restype = [i64], sz
    L.bitsnap_cluster_fit_floats.argtypes, L.bitsnap_cluster_fit_floats.restype = [i64, i64, i], sz
    L.bitsnap_cluster_workspace_bytes.argtypes, L.bitsnap_cluster_workspace_bytes.restype = [i64, i64, i], sz
    L.bitsnap_cluster_z.argtypes, L.bitsnap_cluster_z.restype = [i, i], C.c_double
    L.bitsnap_quantize_cluster_batched_ex.argtypes = [p, i64, i64, i64, i, C.c_uint32, p, p, p, sz, p]
    L.bitsnap_quantize_cluster_batched_ex.restype = i
    L.bitsnap_dequantize_cluster_batched_ex.argtypes = [p, i64, i64, i64, i, C.c_uint32, p, p, sz, p]
    L.bitsnap_dequantize_cluster_batched_ex.restype = i
    L.bitsnap_cluster_chunk_elems.argtypes, L.bitsnap_cluster_chunk_elems.restype = [], sz
    L.bitsnap_cluster_batch_workspace_bytes.argtypes = [i64, i64, i64, C.c_uint32]
    L.bitsnap_cluster_batch_workspace_bytes.restype = sz
    L.bitsnap_quantize_cluster_ex.argtypes = [p, i64, i64, i, C.c_uint32, p, p, p, p, p, p, p, p, sz, p]
    L.bitsnap_quantize_cluster_ex.restype = i
    L.bitsnap_dequantize_cluster_ex.argtypes = [p, p, p, i64, i64, i, C.c_uint32, p, p, p, sz, p]
    L.bitsnap_dequantize_cluster_ex.restype = i
    L.bitsnap_cluster_workspace_bytes_ex.argtypes = [i64, i64, i, C.c_uint32]
    L.bitsnap_cluster_workspace_bytes_ex.restype = sz
    L.bitsnap_quantize_cluster.argtypes = [p, i64, i64, i, p, p, p, p, p, p, p, sz, p]
    L.bitsnap_quantize_cluster.restype = i
    L.bitsnap_dequantize_cluster.argtypes = [p, p, p, i64, i64, i, p, p]
    L.bitsnap_dequantize_cluster.restype = i
    L.bitsnap_sparse_batch_workspace_bytes.argtypes, L.bitsnap_sparse_batch_workspace_bytes.restype = [i64], sz
    L.bitsnap_encode_sparse_batched.argtypes = [p, i64, i64, p, sz, p]
    L.bitsnap_encode_sparse_batched.restype = i
    L.bitsnap_decode_sparse_batched.argtypes = [p, i64, i64, p, sz, p]
    L.bitsnap_decode_sparse_batched.restype = i
    L.bitsnap_quantize_cluster_batched.argtypes = [p, i64, i64, i64, i, p, p]
    L.bitsnap_quantize_cluster_batched.restype = i
    L.bitsnap_dequantize_cluster_batched.argtypes = [p, i64, i64, i64, i, p]
    L.bitsnap_dequantize_cluster_batched.restype = i
    _lib = L
    return L


def _check(rc: int, what: str):
    if rc != 0:
        raise BitsnapError(f"{what}: {lib().bitsnap_error_string(rc).decode()} ({rc})")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


# ----------------------------------------------------------------------------------------------
# size helpers (host)
# ----------------------------------------------------------------------------------------------
def version() -> int:
    return lib().bitsnap_version()


def sparse_tile_elems(elem_bytes: int = 2) -> int:
    return lib().bitsnap_sparse_tile_elems() if elem_bytes == 2 else lib().bitsnap_sparse_tile_elems_for(elem_bytes)


def sparse_mask_bytes(n: int) -> int:
    return lib().bitsnap_sparse_mask_bytes(n)


def sparse_workspace_bytes(n: int, elem_bytes: int = 2) -> int:
    if elem_bytes == 2:
        return lib().bitsnap_sparse_workspace_bytes(n)
    return lib().bitsnap_sparse_workspace_bytes_for(n, elem_bytes)


def cluster_groups(n: int, group: int) -> int:
    return lib().bitsnap_cluster_groups(n, group)


def cluster_param_bytes(n: int, group: int, m: int) -> int:
    return lib().bitsnap_cluster_param_bytes(n, group, m)


def cluster_label_bytes(n: int) -> int:
    return lib().bitsnap_cluster_label_bytes(n)


def cluster_fit_floats(n: int, group: int, m: int) -> int:
    return lib().bitsnap_cluster_fit_floats(n, group, m)


def cluster_workspace_bytes(n: int, group: int, m: int) -> int:
    return lib().bitsnap_cluster_workspace_bytes(n, group, m)


def cluster_z(k: int, m: int) -> float:
    return lib().bitsnap_cluster_z(k, m)


def debug_set_spin_limit(polls: int) -> None:
    lib().bitsnap_debug_set_spin_limit(polls)


def debug_stream_copy(dst, src, stream=None) -> None:
    """dst <- src with the library's plain copy kernel (same byte size, multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().bitsnap_debug_stream_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "bitsnap_debug_stream_copy")


def debug_stream_mix(wide, small_bytes, small_halves, to_small: bool, stream=None) -> None:
    """Streaming traffic with the cluster codecs' byte mix (wide: fp32 [n]; bytes [n]; halves [n/2])."""
    n = wide.numel()
    assert small_bytes.numel() == n and small_halves.numel() * 2 == n
    _check(lib().bitsnap_debug_stream_mix(_ptr(wide), _ptr(small_bytes), _ptr(small_halves), n, int(bool(to_small)),
                                          _stream(stream)), "bitsnap_debug_stream_mix")


def new_sparse_workspace(n: int, device, elem_bytes: int = 2):
    """A zeroed workspace good for tensors of up to n elements (reusable across calls)."""
    import torch
    return torch.zeros(sparse_workspace_bytes(n, elem_bytes), dtype=torch.uint8, device=device)


# ----------------------------------------------------------------------------------------------
# the four codecs.  Raw forms take every buffer; the caller allocates.
# ----------------------------------------------------------------------------------------------
SPARSE_DELTA = 1  # BITSNAP_SPARSE_DELTA
SPARSE_OFFSETS = 2  # BITSNAP_SPARSE_OFFSETS (batched decode)
CLUSTER_MAJOR = 1  # BITSNAP_CLUSTER_MAJOR


def encode_sparse_raw(cur, base, n: int, mask, payload, payload_capacity: int, tile_offsets, n_changed,
                      workspace, stream=None, *, flags: int = 0, new_base=None, elem_bytes: int = 2) -> None:
    """flags == 0 and new_base is None: bitsnap_encode_sparse; otherwise bitsnap_encode_sparse_ex."""
    wsb = workspace.numel() * workspace.element_size()
    if flags == 0 and new_base is None:
        rc = lib().bitsnap_encode_sparse(_ptr(cur), _ptr(base), n, elem_bytes, _ptr(mask), _ptr(payload), payload_capacity,
                                         _ptr(tile_offsets), _ptr(n_changed), _ptr(workspace), wsb, _stream(stream))
        _check(rc, "bitsnap_encode_sparse")
    else:
        rc = lib().bitsnap_encode_sparse_ex(_ptr(cur), _ptr(base), n, elem_bytes, flags, _ptr(mask), _ptr(payload),
                                            payload_capacity, _ptr(tile_offsets), _ptr(n_changed), _ptr(new_base),
                                            _ptr(workspace), wsb, _stream(stream))
        _check(rc, "bitsnap_encode_sparse_ex")


STATIC_MAX_TILES = 16384  # BITSNAP_STATIC_MAX_TILES


def encode_sparse_static_raw(cur, base, n: int, mask, payload, payload_capacity: int, tile_offsets, n_changed,
                             stream=None, *, elem_bytes: int = 2) -> None:
    """bitsnap_encode_sparse_static: the encoder with the library's own scan buffer (no workspace, no allocation)."""
    rc = lib().bitsnap_encode_sparse_static(_ptr(cur), _ptr(base), n, elem_bytes, _ptr(mask), _ptr(payload),
                                            payload_capacity, _ptr(tile_offsets), _ptr(n_changed), _stream(stream))
    _check(rc, "bitsnap_encode_sparse_static")


def decode_sparse_raw(base, mask, payload, payload_elems: int, n: int, out, n_changed, workspace, stream=None, *,
                      flags: int = 0, elem_bytes: int = 2, tile_offsets=None) -> None:
    """tile_offsets: the encoder's array for this tensor; the decoder then skips its counting pass."""
    wsb = workspace.numel() * workspace.element_size()
    if flags == 0 and tile_offsets is None:
        rc = lib().bitsnap_decode_sparse(_ptr(base), _ptr(mask), _ptr(payload), payload_elems, n, elem_bytes, _ptr(out),
                                         _ptr(n_changed), _ptr(workspace), wsb, _stream(stream))
        _check(rc, "bitsnap_decode_sparse")
    else:
        rc = lib().bitsnap_decode_sparse_ex(_ptr(base), _ptr(mask), _ptr(payload), payload_elems, n, elem_bytes, flags,
                                            _ptr(tile_offsets), _ptr(out), _ptr(n_changed), _ptr(workspace), wsb,
                                            _stream(stream))
        _check(rc, "bitsnap_decode_sparse_ex")


def quantize_cluster_raw(x, n: int, group: int, m: int, codes, labels, params, fit_out=None, fit_in=None,
                         status=None, workspace=None, stream=None) -> None:
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().bitsnap_quantize_cluster(_ptr(x), n, group, m, _ptr(codes), _ptr(labels), _ptr(params),
                                        _ptr(fit_out), _ptr(fit_in), _ptr(status), _ptr(workspace), wb,
                                        _stream(stream))
    _check(rc, "bitsnap_quantize_cluster")


def dequantize_cluster_raw(codes, labels, params, n: int, group: int, m: int, out, stream=None) -> None:
    rc = lib().bitsnap_dequantize_cluster(_ptr(codes), _ptr(labels), _ptr(params), n, group, m, _ptr(out),
                                          _stream(stream))
    _check(rc, "bitsnap_dequantize_cluster")


def cluster_workspace_bytes_ex(n: int, group: int, m: int, flags: int) -> int:
    return lib().bitsnap_cluster_workspace_bytes_ex(n, group, m, flags)


def quantize_cluster_ex_raw(x, n: int, group: int, m: int, flags: int, qmap, codes, labels, params, fit_out=None,
                            fit_in=None, status=None, workspace=None, stream=None) -> None:
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().bitsnap_quantize_cluster_ex(_ptr(x), n, group, m, flags, _ptr(qmap), _ptr(codes), _ptr(labels),
                                           _ptr(params), _ptr(fit_out), _ptr(fit_in), _ptr(status), _ptr(workspace), wb,
                                           _stream(stream))
    _check(rc, "bitsnap_quantize_cluster_ex")


def dequantize_cluster_ex_raw(codes, labels, params, n: int, group: int, m: int, flags: int, qmap, out,
                              workspace=None, stream=None) -> None:
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().bitsnap_dequantize_cluster_ex(_ptr(codes), _ptr(labels), _ptr(params), n, group, m, flags, _ptr(qmap),
                                             _ptr(out), _ptr(workspace), wb, _stream(stream))
    _check(rc, "bitsnap_dequantize_cluster_ex")


# ----------------------------------------------------------------------------------------------
# convenience forms: allocate the outputs with torch, then call the raw form
# ----------------------------------------------------------------------------------------------
def _flat_elems(t):
    """Flat view of a contiguous device tensor of 2-byte or 4-byte elements."""
    assert t.is_cuda and t.is_contiguous() and t.element_size() in (2, 4), "need a contiguous 16- or 32-bit device tensor"
    return t.reshape(-1)


def encode_sparse(cur, base, *, capacity: Optional[int] = None, want_offsets: bool = False, workspace=None,
                  stream=None, delta: bool = False, new_base=None):
    """-> namespace(mask uint8[mask_bytes], payload int16[capacity], n_changed uint64-as-int64[1] (device),
    tile_offsets int32[tiles] or None, workspace).  Nothing is synchronised.
    delta: the payload holds cur XOR base; new_base: 16-bit tensor that receives a copy of cur (may be base)."""
    import torch
    cur, base = _flat_elems(cur), _flat_elems(base)
    n = cur.numel()
    eb = cur.element_size()
    assert base.numel() == n and base.element_size() == eb
    dev = cur.device
    capacity = n if capacity is None else capacity
    mask = torch.empty(sparse_mask_bytes(n), dtype=torch.uint8, device=dev)
    payload = torch.empty(max(capacity, 1), dtype=torch.int16 if eb == 2 else torch.int32, device=dev)
    n_changed = torch.empty(1, dtype=torch.int64, device=dev)
    tiles = (n + sparse_tile_elems(eb) - 1) // sparse_tile_elems(eb)
    offs = torch.empty(max(tiles, 1), dtype=torch.int32, device=dev) if want_offsets else None
    if workspace is None:
        workspace = new_sparse_workspace(n, dev, eb)
    encode_sparse_raw(cur, base, n, mask, payload, capacity, offs, n_changed, workspace, stream,
                      flags=SPARSE_DELTA if delta else 0, new_base=None if new_base is None else _flat_elems(new_base),
                      elem_bytes=eb)
    return SimpleNamespace(mask=mask, payload=payload, n_changed=n_changed, tile_offsets=offs, workspace=workspace,
                           n=n, capacity=capacity)


def decode_sparse(base, mask, payload, payload_elems: int, *, out=None, workspace=None, stream=None,
                  delta: bool = False, tile_offsets=None):
    """-> (out, n_changed[1] device).  ``out`` defaults to a new tensor like ``base``.  tile_offsets: the encoder's
    (encode_sparse(..., want_offsets=True)); the decoder then runs one kernel instead of three."""
    import torch
    base_f = _flat_elems(base)
    n = base_f.numel()
    if out is None:
        out = torch.empty_like(base)
    out_f = _flat_elems(out)
    n_changed = torch.empty(1, dtype=torch.int64, device=base.device)
    eb = base_f.element_size()
    if workspace is None:
        workspace = new_sparse_workspace(n, base.device, eb)
    decode_sparse_raw(base_f, mask, payload, payload_elems, n, out_f, n_changed, workspace, stream,
                      flags=SPARSE_DELTA if delta else 0, elem_bytes=eb, tile_offsets=tile_offsets)
    return out, n_changed


def quantize_cluster(x, group: int = 4096, m: int = 16, *, fit_in=None, want_fit: bool = True, stream=None):
    """-> namespace(codes uint8[n], labels uint8[ceil(n/2)], params f32[groups,m,2], fit f32[groups,m+1] or None,
    status int32[1])."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dtype == torch.float32
    xf = x.reshape(-1)
    n = xf.numel()
    dev = x.device
    g = cluster_groups(n, group)
    codes = torch.empty(max(n, 1), dtype=torch.uint8, device=dev)[:n]
    labels = torch.empty(max(cluster_label_bytes(n), 1), dtype=torch.uint8, device=dev)[:cluster_label_bytes(n)]
    params = torch.empty((max(g, 1), m, 2), dtype=torch.float32, device=dev)[:g]
    fit = torch.empty((max(g, 1), m + 1), dtype=torch.float32, device=dev)[:g] if want_fit else None
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    wsb = cluster_workspace_bytes(n, group, m)
    ws = torch.zeros(wsb, dtype=torch.uint8, device=dev) if wsb else None
    quantize_cluster_raw(xf, n, group, m, codes, labels, params, fit, fit_in, status, ws, stream)
    return SimpleNamespace(codes=codes, labels=labels, params=params, fit=fit, status=status, n=n, group=group, m=m)


def quantize_cluster_ex(x, group: int = 4096, m: int = 16, *, qmap=None, cluster_major: bool = False, fit_in=None,
                        want_fit: bool = True, stream=None):
    """quantize_cluster with the format options: qmap = device fp32[256] table (None: linear map), cluster_major =
    codes stored cluster by cluster inside each group.  Same namespace as quantize_cluster."""
    import torch
    assert x.is_cuda and x.is_contiguous() and x.dtype == torch.float32
    xf = x.reshape(-1)
    n = xf.numel()
    dev = x.device
    g = cluster_groups(n, group)
    codes = torch.empty(max(n, 1), dtype=torch.uint8, device=dev)[:n]
    labels = torch.empty(max(cluster_label_bytes(n), 1), dtype=torch.uint8, device=dev)[:cluster_label_bytes(n)]
    params = torch.empty((max(g, 1), m, 2), dtype=torch.float32, device=dev)[:g]
    fit = torch.empty((max(g, 1), m + 1), dtype=torch.float32, device=dev)[:g] if want_fit else None
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    flags = CLUSTER_MAJOR if cluster_major else 0
    wsb = cluster_workspace_bytes_ex(n, group, m, flags)
    ws = torch.zeros(wsb, dtype=torch.uint8, device=dev) if wsb else None
    quantize_cluster_ex_raw(xf, n, group, m, flags, qmap, codes, labels, params, fit, fit_in, status, ws, stream)
    return SimpleNamespace(codes=codes, labels=labels, params=params, fit=fit, status=status, n=n, group=group, m=m,
                           workspace=ws)


def dequantize_cluster_ex(codes, labels, params, n: int, group: int = 4096, m: int = 16, *, qmap=None,
                          cluster_major: bool = False, out=None, workspace=None, stream=None):
    import torch
    if out is None:
        out = torch.empty(max(n, 1), dtype=torch.float32, device=codes.device)[:n]
    flags = CLUSTER_MAJOR if cluster_major else 0
    if workspace is None:
        wsb = cluster_workspace_bytes_ex(n, group, m, flags)
        workspace = torch.zeros(wsb, dtype=torch.uint8, device=codes.device) if wsb else None
    dequantize_cluster_ex_raw(codes, labels, params, n, group, m, flags, qmap, out, workspace, stream)
    return out


def dequantize_cluster(codes, labels, params, n: int, group: int = 4096, m: int = 16, *, out=None, stream=None):
    import torch
    if out is None:
        out = torch.empty(max(n, 1), dtype=torch.float32, device=codes.device)[:n]
    dequantize_cluster_raw(codes, labels, params, n, group, m, out, stream)
    return out


# ----------------------------------------------------------------------------------------------
# batched forms: the caller-side list of tensors becomes a device array of items
# ----------------------------------------------------------------------------------------------
def cluster_items(values, codes, labels, params, group: int, fit_out=None, fit_in=None):
    """Device array of bitsnap_cluster_item (8 x int64 per tensor) for lists of torch tensors.
    ``values`` holds x (quantize) or out (dequantize).  -> (items int64[count, 8], total_groups); with group = 0
    (one group per tensor, for the *_batched_ex calls) the numbering counts chunks instead of groups."""
    import torch
    rows, first = [], 0
    for k, v in enumerate(values):
        n = v.numel()
        assert n > 0
        rows.append([v.data_ptr(), codes[k].data_ptr(), labels[k].data_ptr(), params[k].data_ptr(),
                     0 if fit_out is None else fit_out[k].data_ptr(), 0 if fit_in is None else fit_in[k].data_ptr(),
                     n, first])
        first += cluster_groups(n, group) if group > 0 else (n + cluster_chunk_elems() - 1) // cluster_chunk_elems()
    items = torch.tensor(rows, dtype=torch.int64).to(values[0].device)
    return items, first


def quantize_cluster_batched(items, total_groups: int, group: int, m: int, status=None, stream=None) -> None:
    rc = lib().bitsnap_quantize_cluster_batched(_ptr(items), items.shape[0], total_groups, group, m, _ptr(status),
                                                _stream(stream))
    _check(rc, "bitsnap_quantize_cluster_batched")


def dequantize_cluster_batched(items, total_groups: int, group: int, m: int, stream=None) -> None:
    rc = lib().bitsnap_dequantize_cluster_batched(_ptr(items), items.shape[0], total_groups, group, m, _stream(stream))
    _check(rc, "bitsnap_dequantize_cluster_batched")


def cluster_chunk_elems() -> int:
    return lib().bitsnap_cluster_chunk_elems()


def cluster_batch_workspace_bytes(total_groups: int, count: int, group: int, flags: int = 0) -> int:
    return lib().bitsnap_cluster_batch_workspace_bytes(total_groups, count, group, flags)


def quantize_cluster_batched_ex(items, total_groups: int, group: int, m: int, *, qmap=None, cluster_major: bool = False,
                                status=None, workspace=None, stream=None) -> None:
    """group = 0: one group per tensor; build the items with cluster_items(..., group=0), which then counts chunks."""
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().bitsnap_quantize_cluster_batched_ex(_ptr(items), items.shape[0], total_groups, group, m,
                                                   CLUSTER_MAJOR if cluster_major else 0, _ptr(qmap), _ptr(status),
                                                   _ptr(workspace), wb, _stream(stream))
    _check(rc, "bitsnap_quantize_cluster_batched_ex")


def dequantize_cluster_batched_ex(items, total_groups: int, group: int, m: int, *, qmap=None, cluster_major: bool = False,
                                  workspace=None, stream=None) -> None:
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().bitsnap_dequantize_cluster_batched_ex(_ptr(items), items.shape[0], total_groups, group, m,
                                                     CLUSTER_MAJOR if cluster_major else 0, _ptr(qmap), _ptr(workspace), wb,
                                                     _stream(stream))
    _check(rc, "bitsnap_dequantize_cluster_batched_ex")


def sparse_batch_workspace_bytes(total_tiles: int) -> int:
    return lib().bitsnap_sparse_batch_workspace_bytes(total_tiles)


def sparse_items(n_list, *, src=None, base=None, mask=None, payload=None, out=None, n_changed=None,
                 tile_offsets=None, capacity=None, elem_bytes: int = 2):
    """Device array of bitsnap_sparse_item (10 x int64 per tensor) from parallel lists of torch tensors
    (None where a field is unused).  -> (items int64[count, 10], total_tiles)."""
    import torch
    T = sparse_tile_elems(elem_bytes)
    rows, first = [], 0
    ptr = lambda lst, k: 0 if lst is None or lst[k] is None else lst[k].data_ptr()
    for k, n in enumerate(n_list):
        assert n > 0
        rows.append([ptr(src, k), ptr(base, k), ptr(mask, k), ptr(payload, k), ptr(out, k), ptr(n_changed, k),
                     ptr(tile_offsets, k), n, n if capacity is None else capacity[k], first])
        first += (n + T - 1) // T
    dev = next(l[0].device for l in (src, base, mask, payload, out) if l is not None)
    return torch.tensor(rows, dtype=torch.int64).to(dev), first


def encode_sparse_batched(items, total_tiles: int, workspace, stream=None, *, flags: Optional[int] = None,
                          elem_bytes: int = 2) -> None:
    """flags None: bitsnap_encode_sparse_batched; an int: the _ex form (an item's `out` is then its new_base)."""
    wsb = workspace.numel() * workspace.element_size()
    if flags is None and elem_bytes == 2:
        rc = lib().bitsnap_encode_sparse_batched(_ptr(items), items.shape[0], total_tiles, _ptr(workspace), wsb,
                                                 _stream(stream))
        _check(rc, "bitsnap_encode_sparse_batched")
    else:
        rc = lib().bitsnap_encode_sparse_batched_ex(_ptr(items), items.shape[0], total_tiles, elem_bytes, flags or 0,
                                                    _ptr(workspace), wsb, _stream(stream))
        _check(rc, "bitsnap_encode_sparse_batched_ex")


def decode_sparse_batched(items, total_tiles: int, workspace, stream=None, *, flags: Optional[int] = None,
                          elem_bytes: int = 2) -> None:
    wsb = workspace.numel() * workspace.element_size()
    if flags is None and elem_bytes == 2:
        rc = lib().bitsnap_decode_sparse_batched(_ptr(items), items.shape[0], total_tiles, _ptr(workspace), wsb,
                                                 _stream(stream))
        _check(rc, "bitsnap_decode_sparse_batched")
    else:
        rc = lib().bitsnap_decode_sparse_batched_ex(_ptr(items), items.shape[0], total_tiles, elem_bytes, flags or 0,
                                                    _ptr(workspace), wsb, _stream(stream))
        _check(rc, "bitsnap_decode_sparse_batched_ex")
