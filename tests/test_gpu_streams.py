"""Calls on two streams at once, each with its own workspace: the library keeps no state that two calls could share
(besides host-side caches behind a lock), so results must be those of the calls made one after the other."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, announce, f32_to_dev, to_np, u16_to_dev
from paper_2511_12376_amd import binding as B

pytestmark = pytest.mark.gpu


def test_two_streams_side_by_side():
    announce("two streams")
    rng = np.random.default_rng(5)
    T = B.sparse_tile_elems()
    sizes = [40 * T + 123, 33 * T + 7]
    pairs = []
    for n in sizes:
        base = rng.integers(0, 1 << 16, n, dtype=np.uint16)
        cur = base.copy()
        sel = rng.random(n) < 0.4
        cur[sel] ^= rng.integers(1, 1 << 16, n, dtype=np.uint16)[sel]
        pairs.append((cur, base))
    xs = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    dev = [dict(cur=u16_to_dev(c), base=u16_to_dev(b), x=f32_to_dev(x)) for (c, b), x in zip(pairs, xs)]
    bufs = []
    for d, n in zip(dev, sizes):
        bufs.append(dict(mask=torch.zeros(B.sparse_mask_bytes(n), dtype=torch.uint8, device=DEV),
                         payload=torch.zeros(n, dtype=torch.int16, device=DEV),
                         cnt=torch.zeros(1, dtype=torch.int64, device=DEV),
                         ws=B.new_sparse_workspace(n, DEV),
                         out=torch.zeros(n, dtype=torch.int16, device=DEV),
                         codes=torch.zeros(n, dtype=torch.uint8, device=DEV),
                         labels=torch.zeros((n + 1) // 2, dtype=torch.uint8, device=DEV),
                         params=torch.zeros(B.cluster_groups(n, 4096), 16, 2, dtype=torch.float32, device=DEV),
                         fit=torch.zeros(B.cluster_groups(n, 4096), 17, dtype=torch.float32, device=DEV),
                         xh=torch.zeros(n, dtype=torch.float32, device=DEV)))
    torch.cuda.synchronize()
    for rep in range(3):                       # alternate the streams so that their kernels overlap
        for k in (0, 1):
            d, b, n, s = dev[k], bufs[k], sizes[k], streams[k]
            B.encode_sparse_raw(d["cur"], d["base"], n, b["mask"], b["payload"], n, None, b["cnt"], b["ws"], s)
            B.quantize_cluster_raw(d["x"], n, 4096, 16, b["codes"], b["labels"], b["params"], b["fit"], None, None, None, s)
            B.decode_sparse_raw(d["base"], b["mask"], b["payload"], n, n, b["out"], None, b["ws"], s)
            B.dequantize_cluster_raw(b["codes"], b["labels"], b["params"], n, 4096, 16, b["xh"], s)
    torch.cuda.synchronize()
    for k in (0, 1):
        cur, base = pairs[k]
        b, n = bufs[k], sizes[k]
        o_mask, o_pay, o_nc = oracle.encode_sparse(cur, base)
        assert int(b["cnt"].item()) == o_nc
        assert np.array_equal(to_np(b["mask"])[: o_mask.size], o_mask)
        assert np.array_equal(to_np(b["payload"]).view(np.uint16)[:o_nc], o_pay)
        assert np.array_equal(to_np(b["out"]).view(np.uint16), cur)
        o = oracle.quantize_cluster(xs[k], 4096, 16, fit_in=to_np(b["fit"])[:, :2].copy())
        assert np.array_equal(to_np(b["codes"]), o["codes"]) and np.array_equal(to_np(b["labels"]), o["labels"])
        assert np.array_equal(to_np(b["params"]), o["params"])
        assert np.array_equal(to_np(b["xh"]), oracle.dequantize_cluster(o["codes"], o["labels"], o["params"], n, 4096, 16))
