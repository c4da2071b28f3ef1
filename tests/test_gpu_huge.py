"""GPU parity at sizes beyond 2^31 and 2^32 elements in ONE tensor: every index, offset and count that is 32-bit in
ordinary tests has to be 64-bit here.  The oracle checks sampled regions (it cannot walk four billion elements in
seconds); the whole result is checked through properties written with torch operations: the mask is the packed
comparison, the payload is the selection of the changed values, the round trip is lossless.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, announce, to_np
from paper_2511_12376_amd import binding as B

pytestmark = pytest.mark.gpu

N_SPARSE = (1 << 32) + 8 * 12345 + 3          # more than 2^32 elements, ragged last tile and last mask byte


def _packed(changed, n):
    """uint8[ceil(n/8)]: bit t of byte j = changed[8j + t] (torch only)."""
    pad = (-n) % 8
    c = torch.cat([changed, torch.zeros(pad, dtype=torch.bool, device=changed.device)]) if pad else changed
    w = torch.tensor([1, 2, 4, 8, 16, 32, 64, 128], dtype=torch.uint8, device=changed.device)
    out = torch.empty(c.numel() // 8, dtype=torch.uint8, device=changed.device)
    step = 1 << 28                                                         # bytes per piece: bounds the temporaries
    for lo in range(0, out.numel(), step):
        hi = min(out.numel(), lo + step)
        out[lo:hi] = (c[8 * lo:8 * hi].view(-1, 8).to(torch.uint8) * w).sum(dim=1, dtype=torch.int32).to(torch.uint8)
    return out


@pytest.mark.parametrize("dense", [False, True])
def test_sparse_pair_beyond_two_to_the_32_elements(dense):
    announce("huge sparse", N_SPARSE, "all changed" if dense else "1 % changed")
    n = N_SPARSE
    g = torch.Generator(device=DEV)
    g.manual_seed(77)
    base = torch.randint(-32768, 32767, (n,), dtype=torch.int16, device=DEV, generator=g)
    if dense:
        cur = base ^ 1                                                     # every element changed: n_c = n > 2^32
    else:
        flip = torch.rand(n, device=DEV, generator=g) < 0.01
        cur = torch.where(flip, base ^ 0x0101, base)
        del flip
    enc = B.encode_sparse(cur.view(torch.bfloat16), base.view(torch.bfloat16))
    torch.cuda.synchronize()
    changed = cur != base
    nc = int(changed.sum().item())
    assert int(enc.n_changed.item()) == nc and (nc == n if dense else 0 < nc < n // 50)
    mask = enc.mask[: (n + 7) // 8]
    assert torch.equal(mask, _packed(changed, n))
    pos = 0                                                                # torch's own selection, in pieces below 2^31
    for lo_ in range(0, n, 1 << 28):
        sel = cur[lo_:lo_ + (1 << 28)][changed[lo_:lo_ + (1 << 28)]]
        assert torch.equal(enc.payload[pos:pos + sel.numel()], sel), lo_
        pos += sel.numel()
    assert pos == nc
    # the last 200 000 elements (all beyond 2^32) against the oracle, mask bytes and payload tail
    lo = (n - 200_000) // 8 * 8
    o_mask, o_pay, o_nc = oracle.encode_sparse(to_np(cur[lo:]).view(np.uint16), to_np(base[lo:]).view(np.uint16))
    assert np.array_equal(to_np(mask[lo // 8:]), o_mask)
    assert np.array_equal(to_np(enc.payload[nc - o_nc:nc]).view(np.uint16), o_pay)
    del changed
    out, cnt = B.decode_sparse(base.view(torch.bfloat16), enc.mask, enc.payload, n, workspace=enc.workspace)
    torch.cuda.synchronize()
    assert int(cnt.item()) == nc and torch.equal(out.view(torch.int16), cur)
    # tile offsets are 32-bit: not available at this size
    with pytest.raises(B.BitsnapError):
        B.encode_sparse(cur.view(torch.bfloat16), base.view(torch.bfloat16), want_offsets=True)


def test_cluster_pair_beyond_two_to_the_31_elements():
    n = (1 << 31) + 3 * 4096 + 77
    announce("huge cluster", n)
    g = torch.Generator(device=DEV)
    g.manual_seed(78)
    x = torch.empty(n, dtype=torch.float32, device=DEV)
    step = 1 << 28
    for lo in range(0, n, step):
        x[lo:lo + step].normal_(0.0, 1e-3, generator=g)
    q = B.quantize_cluster(x, 4096, 16)
    xh = B.dequantize_cluster(q.codes, q.labels, q.params, n, 4096, 16)
    torch.cuda.synchronize()
    assert int(q.status.item()) == 0
    groups = (n + 4095) // 4096
    rng = np.random.default_rng(79)
    for gi in [0, groups - 1, groups - 2, groups - 3, groups - 4, (1 << 19) - 1, 1 << 19] + list(rng.integers(0, groups, 12)):
        lo, hi = int(gi) * 4096, min(n, int(gi) * 4096 + 4096)
        xs = to_np(x[lo:hi])
        o = oracle.quantize_cluster(xs, 4096, 16, fit_in=to_np(q.fit[gi, :2]).reshape(1, 2).copy())
        assert np.array_equal(to_np(q.codes[lo:hi]), o["codes"]), gi
        assert np.array_equal(to_np(q.labels[lo // 2:(hi + 1) // 2]), o["labels"]), gi
        assert np.array_equal(to_np(q.params[gi]), o["params"][0]), gi
        o_fit = oracle.quantize_cluster(xs, 4096, 16)["fit"]
        assert np.allclose(to_np(q.fit[gi]), o_fit[0], rtol=1e-6, atol=0)
        assert np.array_equal(to_np(xh[lo:hi]), oracle.dequantize_cluster(o["codes"], o["labels"], o["params"], hi - lo, 4096, 16)), gi
    # every element is within half a code step of its cluster's range (a property that holds at any size)
    err = (xh - x).abs_()
    assert float(err.max().item()) <= 1e-3 * 12 / 255


def _pieces(n, step=1 << 28):
    return [(lo, min(n, lo + step)) for lo in range(0, n, step)]


def test_whole_tensor_group_beyond_two_to_the_31_elements():
    """group = 0 on 2^31 + 12 365 elements: 524 292 chunks in 2049 slices, one fit, one cluster-major arrangement."""
    n = (1 << 31) + 3 * 4096 + 77
    announce("huge whole-tensor group", n)
    g = torch.Generator(device=DEV)
    g.manual_seed(80)
    x = torch.empty(n, dtype=torch.float32, device=DEV)
    for lo, hi in _pieces(n):
        x[lo:hi].normal_(2e-4, 1e-3, generator=g)
    q = B.quantize_cluster(x, 0, 16)
    torch.cuda.synchronize()
    assert int(q.status.item()) == 0
    # the fit against torch's fp64 reductions
    mean = sum(float(x[lo:hi].double().sum().item()) for lo, hi in _pieces(n)) / n
    var = sum(float(((x[lo:hi].double() - mean) ** 2).sum().item()) for lo, hi in _pieces(n)) / n
    fit = to_np(q.fit)[0]
    assert abs(fit[0] - mean) <= 1e-6 * max(abs(mean), var ** 0.5) and abs(fit[1] - var ** 0.5) <= 1e-6 * var ** 0.5
    assert np.array_equal(fit[2:], oracle.cluster_edges(fit[0], fit[1], 16))
    # labels = number of edges <= x (torch.bucketize), (S, b) = range of every cluster
    edges = torch.from_numpy(fit[2:].copy()).to(DEV)
    lab = torch.empty(n, dtype=torch.uint8, device=DEV)
    for lo, hi in _pieces(n):
        lab[lo:hi] = torch.bucketize(x[lo:hi], edges, right=True).to(torch.uint8)
    packed = q.labels
    assert torch.equal(packed[: n // 2], lab[0:n - 1:2] | (lab[1:n:2] << 4)) and int(packed[n // 2].item()) == int(lab[n - 1].item())
    params = to_np(q.params)[0]
    lows, highs = [], []
    for c in range(16):
        mn = min(float(x[lo:hi][lab[lo:hi] == c].min().item()) for lo, hi in _pieces(n))
        mx = max(float(x[lo:hi][lab[lo:hi] == c].max().item()) for lo, hi in _pieces(n))
        assert params[c, 1] == np.float32(mn) and params[c, 0] == np.float32(mx) - np.float32(mn), c
        lows.append(mn), highs.append(mx)
    # codes of sampled stretches through the oracle: a small tensor that holds the stretch and every cluster's two
    # extremes has the same (S, b), so its codes for the stretch are the whole tensor's
    ends = np.array(lows + highs, np.float32)
    xh = B.dequantize_cluster(q.codes, q.labels, q.params, n, 0, 16)
    torch.cuda.synchronize()
    for lo in (0, 123_456 * 4096, (1 << 31) - 2048, n - 5000):
        xs = np.concatenate([to_np(x[lo:lo + 5000]), ends])
        o = oracle.quantize_cluster(xs, 0, 16, fit_in=fit[:2].reshape(1, 2).copy())
        assert np.array_equal(o["params"][0], params)
        assert np.array_equal(to_np(q.codes[lo:lo + 5000]), o["codes"][:5000]), lo
        assert np.array_equal(to_np(xh[lo:lo + 5000]),
                              oracle.dequantize_cluster(o["codes"], o["labels"], o["params"], xs.size, 0, 16)[:5000]), lo
    # cluster-major codes: cluster c's run is the selection of its members' codes, in element order
    qm = B.quantize_cluster_ex(x, 0, 16, cluster_major=True)
    torch.cuda.synchronize()
    assert torch.equal(qm.labels, q.labels) and torch.equal(qm.params, q.params)
    pos = 0
    for c in range(16):
        for lo, hi in _pieces(n):
            sel = q.codes[lo:hi][lab[lo:hi] == c]
            assert torch.equal(qm.codes[pos:pos + sel.numel()], sel), (c, lo)
            pos += sel.numel()
    assert pos == n
    back = B.dequantize_cluster_ex(qm.codes, qm.labels, qm.params, n, 0, 16, cluster_major=True, workspace=qm.workspace)
    torch.cuda.synchronize()
    assert torch.equal(back, xh)
