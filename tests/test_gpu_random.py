"""GPU parity on seeded random cases: sizes, change patterns, value scales and option combinations drawn at random
(the other GPU test files walk fixed lists).  Everything is compared with the oracle bit for bit; the cluster fit is
handed to the oracle as in the other cluster tests."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, announce, f32_to_dev, to_np
from paper_2511_12376_amd import binding as B
from paper_2511_12376_amd import synth

pytestmark = pytest.mark.gpu


def _changes(rng, n):
    """A change mask with one of several structures: independent, bursts, a stride, a prefix, nothing, everything."""
    kind = rng.integers(0, 6)
    if kind == 0:
        return rng.random(n) < rng.choice([0.001, 0.05, 0.3, 0.7, 0.95])
    if kind == 1:
        sel = np.zeros(n, bool)
        for _ in range(int(rng.integers(1, 20))):
            lo = int(rng.integers(0, max(n, 1)))
            sel[lo:lo + int(rng.integers(1, 5000))] = True
        return sel
    if kind == 2:
        sel = np.zeros(n, bool)
        sel[int(rng.integers(0, 7))::int(rng.integers(2, 70))] = True
        return sel
    if kind == 3:
        sel = np.zeros(n, bool)
        sel[:int(rng.integers(0, n + 1))] = True
        return sel
    return np.full(n, kind == 5)


@pytest.mark.parametrize("seed", range(100))
def test_sparse_pair_on_random_cases(seed):
    rng = np.random.default_rng(1000 + seed)
    wide = bool(rng.integers(0, 2))
    tile = B.sparse_tile_elems(4 if wide else 2)
    n = int(rng.choice([rng.integers(0, 300), rng.integers(0, 3 * tile), rng.integers(0, 12 * tile)]))
    delta, refresh = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    announce("random sparse", seed, n, "4-byte" if wide else "2-byte", delta, refresh)
    dt, tdt = (np.uint32, torch.int32) if wide else (np.uint16, torch.int16)
    bits = 32 if wide else 16
    base = rng.integers(0, 1 << bits, n, dtype=np.uint64).astype(dt)
    cur = base.copy()
    sel = _changes(rng, n)
    cur[sel] ^= rng.integers(1, 1 << bits, n, dtype=np.uint64).astype(dt)[sel]
    enc_o = oracle.encode_sparse32 if wide else oracle.encode_sparse_ex
    dec_o = oracle.decode_sparse32 if wide else oracle.decode_sparse_ex
    o_mask, o_pay, o_nc = enc_o(cur, base, delta=delta)
    to_dev = lambda a: torch.from_numpy(a.view(np.int32 if wide else np.int16)).to(DEV)
    cur_d, base_d = to_dev(cur), to_dev(base)
    new_base = torch.zeros(max(n, 1), dtype=tdt, device=DEV)[:n] if refresh else None
    enc = B.encode_sparse(cur_d, base_d, delta=delta, new_base=new_base)
    torch.cuda.synchronize()
    assert int(enc.n_changed.item()) == o_nc
    assert np.array_equal(to_np(enc.mask)[: o_mask.size], o_mask) and not to_np(enc.mask)[o_mask.size:].any()
    assert np.array_equal(to_np(enc.payload).view(dt)[:o_nc], o_pay)
    if refresh:
        assert np.array_equal(to_np(new_base).view(dt), cur)
    out, cnt = B.decode_sparse(base_d, enc.mask, enc.payload, n, workspace=enc.workspace, delta=delta)
    torch.cuda.synchronize()
    assert int(cnt.item()) == o_nc and np.array_equal(to_np(out).view(dt), cur)
    assert np.array_equal(dec_o(base, o_mask, o_pay, delta=delta), cur)


@pytest.mark.parametrize("seed", range(100))
def test_cluster_pair_on_random_cases(seed):
    rng = np.random.default_rng(2000 + seed)
    G = int(rng.choice([256, 512, 1024, 2048, 4096, 0, 2 * int(rng.integers(1, 5000)), 4096 * int(rng.integers(2, 40)) + 2 * int(rng.integers(0, 2048))]))
    n = int(rng.choice([rng.integers(1, 5000), rng.integers(1, 200_000), rng.integers(1, 1_500_000)]))
    m = int(rng.choice([16, 16, 16, rng.integers(1, 17)]))
    kind = [None, None, "normal", "square", "steps", "linear"][int(rng.integers(0, 6))]
    major = bool(rng.integers(0, 2))
    announce("random cluster", seed, n, G, m, kind, major)
    shape = int(rng.integers(0, 4))
    x = rng.standard_normal(n) * 10.0 ** rng.integers(-9, 3)
    if shape == 1:
        x = x + rng.standard_normal() * np.abs(x).mean() * 10.0 ** rng.integers(0, 4)     # a mean far from zero
    elif shape == 2:
        x = x * x                                                                        # one-sided, like Adam's second moment
    elif shape == 3:
        x[rng.random(n) < 0.01] *= 1e3                                                   # outliers
    x = x.astype(np.float32)
    Q = None if kind is None else synth.qmap_table(kind)
    Qd = None if Q is None else f32_to_dev(Q)
    q = B.quantize_cluster_ex(f32_to_dev(x), G, m, qmap=Qd, cluster_major=major)
    torch.cuda.synchronize()
    assert int(q.status.item()) == 0
    fit = to_np(q.fit)
    o_fit = oracle.quantize_cluster(x, G, m)["fit"]
    sg = np.maximum(o_fit[:, 1].astype(np.float64), 1e-45)
    assert np.all(np.abs(fit[:, 1] - o_fit[:, 1]) <= 1e-6 * sg)
    assert np.all(np.abs(fit[:, 0] - o_fit[:, 0]) <= 1e-6 * np.maximum(np.abs(o_fit[:, 0]), sg))
    o = oracle.quantize_cluster_ex(x, G, m, fit_in=fit[:, :2].copy(), qmap=Q, cluster_major=major)
    assert np.array_equal(to_np(q.labels), o["labels"]) and np.array_equal(to_np(q.params), o["params"])
    assert np.array_equal(to_np(q.codes), o["codes"])
    xh = B.dequantize_cluster_ex(q.codes, q.labels, q.params, n, G, m, qmap=Qd, cluster_major=major, workspace=q.workspace)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(xh), oracle.dequantize_cluster_ex(o["codes"], o["labels"], o["params"], n, G, m, qmap=Q,
                                                                  cluster_major=major))
