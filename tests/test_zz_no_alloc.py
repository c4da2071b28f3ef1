"""GPU: bitsnap_encode_sparse_static (the encoder with the library's own scan buffer, for callers that cannot
allocate) against bitsnap_encode_sparse with a caller-supplied workspace, bit for bit, through the C ABI."""
import numpy as np
import pytest
import torch

from gpu_util import DEV, announce, to_np, u16_to_dev
from paper_2511_12376_amd import binding as B

pytestmark = pytest.mark.gpu

T = B.sparse_tile_elems()


def _pair(n, p, seed):
    rng = np.random.default_rng(seed)
    base = rng.integers(0, 1 << 16, n, dtype=np.uint16)
    cur = base.copy()
    sel = rng.random(n) < p
    cur[sel] ^= rng.integers(1, 1 << 16, n, dtype=np.uint16)[sel]
    return cur, base


def _outputs(n):
    tiles = max((n + T - 1) // T, 1)
    return dict(mask=torch.full((max(B.sparse_mask_bytes(n), 16),), 0xA5, dtype=torch.uint8, device=DEV),
                payload=torch.full((max(n, 8),), -1, dtype=torch.int16, device=DEV),
                offsets=torch.full((tiles,), -1, dtype=torch.int32, device=DEV),
                count=torch.full((1,), -1, dtype=torch.int64, device=DEV))


def _both(n, p, seed):
    """The same tensor through both entry points; every output must be the same, byte for byte."""
    cur_h, base_h = _pair(n, p, seed)
    cur, base = u16_to_dev(cur_h), u16_to_dev(base_h)
    ref, got = _outputs(n), _outputs(n)
    ws = B.new_sparse_workspace(n, DEV)
    B.encode_sparse_raw(cur, base, n, ref["mask"], ref["payload"], n, ref["offsets"], ref["count"], ws)
    B.encode_sparse_static_raw(cur, base, n, got["mask"], got["payload"], n, got["offsets"], got["count"])
    torch.cuda.synchronize()
    nc = int(ref["count"].item())
    assert nc == int(np.count_nonzero(cur_h != base_h))
    assert int(got["count"].item()) == nc
    mb = B.sparse_mask_bytes(n)
    assert np.array_equal(to_np(got["mask"])[:mb], to_np(ref["mask"])[:mb])
    assert np.array_equal(to_np(got["payload"])[:nc], to_np(ref["payload"])[:nc])
    assert not (to_np(got["payload"])[nc:max(n, 8)] != -1).any() or n == 0      # nothing beyond the changed values
    tiles = (n + T - 1) // T
    assert np.array_equal(to_np(got["offsets"])[:tiles], to_np(ref["offsets"])[:tiles])
    return nc


def test_static_encoder_equals_workspace_encoder_two_calls_in_a_row():
    announce("static sparse encoder: 5 tiles + tail, then a smaller tensor")
    assert _both(5 * T + 4321, 0.3, 11) > 0
    assert _both(2 * T - 77, 0.06, 12) > 0       # the array still holds the first call's scan words
    assert _both(1000, 1.0, 13) == 1000
    assert _both(0, 0.5, 14) == 0


def test_static_encoder_32_bit_elements_and_many_calls():
    announce("static sparse encoder: 4-byte elements, 20 calls")
    rng = np.random.default_rng(5)
    for k in range(20):
        n = int(rng.integers(1, 6 * T))
        _both(n, float(rng.random()), 100 + k)
    n = 3 * B.sparse_tile_elems(4) + 99
    a = torch.from_numpy(rng.integers(-2**31, 2**31 - 1, n, dtype=np.int64).astype(np.int32)).to(DEV)
    b = a ^ (torch.rand(n, device=DEV) < 0.2).to(torch.int32)
    ref, got = _outputs(2 * n), _outputs(2 * n)
    ws = B.new_sparse_workspace(n, DEV, 4)
    B.encode_sparse_raw(a, b, n, ref["mask"], ref["payload"], n, None, ref["count"], ws, elem_bytes=4)
    B.encode_sparse_static_raw(a, b, n, got["mask"], got["payload"], n, None, got["count"], elem_bytes=4)
    torch.cuda.synchronize()
    nc = int(ref["count"].item())
    assert int(got["count"].item()) == nc == int((a != b).sum().item())
    assert np.array_equal(to_np(got["mask"])[:B.sparse_mask_bytes(n)], to_np(ref["mask"])[:B.sparse_mask_bytes(n)])
    assert np.array_equal(to_np(got["payload"])[:2 * nc], to_np(ref["payload"])[:2 * nc])


def test_static_encoder_rejects_what_its_buffer_cannot_serve():
    announce("static sparse encoder: size limit")
    L = B.lib()
    n = (B.STATIC_MAX_TILES + 1) * T
    one = torch.zeros(16, dtype=torch.uint8, device=DEV)
    rc = L.bitsnap_encode_sparse_static(one.data_ptr(), one.data_ptr(), n, 2, one.data_ptr(), one.data_ptr(), 0, None,
                                        one.data_ptr(), None)
    assert rc == -7 and b"BITSNAP_STATIC_MAX_TILES" in L.bitsnap_error_string(rc)
    assert L.bitsnap_encode_sparse_static(one.data_ptr(), one.data_ptr(), -1, 2, one.data_ptr(), one.data_ptr(), 0, None,
                                          one.data_ptr(), None) == -2
    torch.cuda.synchronize()
