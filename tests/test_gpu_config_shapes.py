"""GPU parity at the full shapes of the other synthetic checkpoints, in the launch configuration the benchmark
times (single-tensor calls and one batched call over several tensors): the GPT-2-XL token embedding
(50257 x 1600: the last tile, the last group and the mask's last byte are all partial), a k/v slice of the
tensor-parallel Llama-2-70B rank (128 x 8192), the Llama-2-13B embedding with changes in whole 4096-element runs
(tiles are empty or hold several fully changed runs).  The oracle recomputes sampled tiles and groups one by one,
the ragged ends always among them; totals are checked through properties that hold at any size."""
import math

import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, announce, to_np
from paper_2511_12376_amd import binding as B
from paper_2511_12376_amd import synth

pytestmark = pytest.mark.gpu

T = B.sparse_tile_elems()
G, M = 4096, 16

# (config, tensor index, changed fraction) -> the tensor's name, for the test ids
CASES = [(1, 0, 0.01), (1, 0, 0.2), (4, 3, 0.06), (4, 4, 0.06), (3, 0, 0.06)]


def _name(case):
    c, t, p = case
    return f"config{c}-{synth.config(c).tensors[t][0]}-p{p}"


def _check_sparse_tile(enc, cur16, base16, n, offs, t):
    lo, hi = t * T, min((t + 1) * T, n)
    c = cur16[lo:hi].cpu().numpy().view(np.uint16)
    b = base16[lo:hi].cpu().numpy().view(np.uint16)
    o_mask, o_pay, o_nc = oracle.encode_sparse(c, b)
    assert np.array_equal(to_np(enc["mask"][lo // 8:lo // 8 + o_mask.size]), o_mask)
    assert np.array_equal(to_np(enc["payload"][offs[t]:offs[t] + o_nc]).view(np.uint16), o_pay)
    return o_nc


@pytest.mark.parametrize("case", CASES, ids=_name)
def test_sparse_pair_at_full_shape(case):
    c, t, p = case
    cfg = synth.config(c, p=p)
    announce("config shape sparse", _name(case))
    d = synth.make_tensor_torch(cfg, t, DEV, want=("base", "cur"))
    n = d["cur"].numel()
    assert n == math.prod(cfg.tensors[t][1])
    ntiles = (n + T - 1) // T
    enc = dict(mask=torch.full((B.sparse_mask_bytes(n),), 0xA5, dtype=torch.uint8, device=DEV),
               payload=torch.empty(n, dtype=torch.int16, device=DEV),
               offsets=torch.empty(ntiles, dtype=torch.int32, device=DEV),
               count=torch.zeros(1, dtype=torch.int64, device=DEV))
    ws = B.new_sparse_workspace(n, DEV)
    B.encode_sparse_raw(d["cur"], d["base"], n, enc["mask"], enc["payload"], n, enc["offsets"], enc["count"], ws)
    out = torch.empty_like(d["cur"])
    cnt = torch.zeros(1, dtype=torch.int64, device=DEV)
    B.decode_sparse_raw(d["base"], enc["mask"], enc["payload"], n, n, out, cnt, ws)
    torch.cuda.synchronize()
    cur16, base16 = d["cur"].view(torch.int16), d["base"].view(torch.int16)
    changed = cur16 != base16
    nc = int(enc["count"].item())
    assert nc == int(changed.sum().item()) == int(cnt.item())
    assert torch.equal(out.view(torch.int16), cur16)                                   # lossless at any size
    assert not to_np(enc["mask"][(n + 7) // 8:]).any()                                 # padding bytes are zero
    pad = torch.zeros(ntiles * T - n, dtype=torch.bool, device=DEV)
    per_tile = torch.cat([changed, pad]).view(ntiles, T).sum(dim=1).cpu().numpy()
    offs = to_np(enc["offsets"]).view(np.uint32).astype(np.int64)
    assert np.array_equal(offs, np.concatenate([[0], np.cumsum(per_tile)[:-1]]))
    rng = np.random.default_rng(c * 100 + t)
    picks = {0, ntiles - 1, max(ntiles - 2, 0)} | set(int(v) for v in rng.integers(0, ntiles, 24))
    if cfg.recipe == "runs":                                                           # the fullest tiles as well
        picks |= set(int(v) for v in np.argsort(per_tile)[-3:])
    for tile in sorted(picks):
        assert _check_sparse_tile(enc, cur16, base16, n, offs, tile) == per_tile[tile]


@pytest.mark.parametrize("case", CASES[:1] + CASES[2:3], ids=_name)
def test_cluster_pair_at_full_shape(case):
    c, t, p = case
    cfg = synth.config(c, p=p)
    announce("config shape cluster", _name(case))
    d = synth.make_tensor_torch(cfg, t, DEV, want=("base", "cur", "m", "v"))
    for key in ("m", "v"):
        x = d[key]
        n = x.numel()
        q = B.quantize_cluster(x, G, M)
        xh = B.dequantize_cluster(q.codes, q.labels, q.params, n, G, M)
        torch.cuda.synchronize()
        assert int(q.status.item()) == 0
        groups = (n + G - 1) // G
        rng = np.random.default_rng(7 + t)
        for g in sorted({0, groups - 1, max(groups - 2, 0)} | set(int(v) for v in rng.integers(0, groups, 24))):
            lo, hi = g * G, min((g + 1) * G, n)
            xs = to_np(x[lo:hi])
            fit_g = to_np(q.fit[g])
            o = oracle.quantize_cluster(xs, G, M)
            assert abs(float(fit_g[1]) - float(o["fit"][0, 1])) <= 1e-6 * float(o["fit"][0, 1])
            assert abs(float(fit_g[0]) - float(o["fit"][0, 0])) <= 1e-6 * max(abs(float(o["fit"][0, 0])), float(o["fit"][0, 1]))
            if not np.array_equal(fit_g[:2], o["fit"][0, :2]):
                o = oracle.quantize_cluster(xs, G, M, fit_in=fit_g[:2].copy())
            assert np.array_equal(fit_g, o["fit"][0])
            assert np.array_equal(to_np(q.params[g]), o["params"][0])
            assert np.array_equal(to_np(q.codes[lo:hi]), o["codes"])
            assert np.array_equal(to_np(q.labels[lo // 2:(hi + 1) // 2]), o["labels"])
            assert np.array_equal(to_np(xh[lo:hi]),
                                  oracle.dequantize_cluster(o["codes"], o["labels"], o["params"], hi - lo, G, M))
        # the error bound of the method on the whole tensor (fp32 rounding of q*step + b at the cluster's magnitude)
        lab = torch.stack([q.labels & 15, q.labels >> 4], dim=1).reshape(-1)[:n].long()
        grp = torch.arange(n, device=DEV) // G
        S = q.params[:, :, 0].reshape(-1)[grp * M + lab].double()
        b = q.params[:, :, 1].reshape(-1)[grp * M + lab].double()
        err = (xh.double() - x.double()).abs()
        assert bool((err <= S / 510 * (1 + 1e-5) + 5e-7 * torch.maximum(b.abs(), (b + S).abs())).all())


def test_batched_pass_over_a_layer_of_the_gpt2_xl_shape():
    """One batched call per operation over the embeddings and the first layer of the GPT-2-XL list (14 tensors
    from 1600 to 80 M elements, most of them not multiples of the tile or the group): every tensor must equal the
    single-tensor call, bit for bit."""
    announce("config shape batched")
    cfg = synth.config(1, p=0.06)
    idx = list(range(14))
    ds = [synth.make_tensor_torch(cfg, t, DEV, want=("base", "cur", "m")) for t in idx]
    sizes = [d["cur"].numel() for d in ds]
    masks = [torch.empty(B.sparse_mask_bytes(n), dtype=torch.uint8, device=DEV) for n in sizes]
    pays = [torch.empty(n, dtype=torch.int16, device=DEV) for n in sizes]
    cnts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    outs = [torch.empty(n, dtype=torch.bfloat16, device=DEV) for n in sizes]
    items, tiles = B.sparse_items(sizes, src=[d["cur"] for d in ds], base=[d["base"] for d in ds], mask=masks,
                                  payload=pays, n_changed=cnts)
    ws = torch.zeros(B.sparse_batch_workspace_bytes(tiles), dtype=torch.uint8, device=DEV)
    B.encode_sparse_batched(items, tiles, ws)
    ditems, _ = B.sparse_items(sizes, base=[d["base"] for d in ds], mask=masks, payload=pays, out=outs)
    B.decode_sparse_batched(ditems, tiles, ws)
    codes = [torch.empty(n, dtype=torch.uint8, device=DEV) for n in sizes]
    labels = [torch.empty((n + 1) // 2, dtype=torch.uint8, device=DEV) for n in sizes]
    params = [torch.empty(B.cluster_groups(n, G), M, 2, dtype=torch.float32, device=DEV) for n in sizes]
    qitems, groups = B.cluster_items([d["m"] for d in ds], codes, labels, params, G)
    B.quantize_cluster_batched(qitems, groups, G, M)
    deq = [torch.empty(n, dtype=torch.float32, device=DEV) for n in sizes]
    dqitems, _ = B.cluster_items(deq, codes, labels, params, G)
    B.dequantize_cluster_batched(dqitems, groups, G, M)
    torch.cuda.synchronize()
    for k, d in enumerate(ds):
        n = sizes[k]
        one = B.encode_sparse(d["cur"], d["base"])
        q1 = B.quantize_cluster(d["m"], G, M)
        x1 = B.dequantize_cluster(q1.codes, q1.labels, q1.params, n, G, M)
        torch.cuda.synchronize()
        nc = int(one.n_changed.item())
        assert int(cnts[k].item()) == nc
        assert torch.equal(masks[k], one.mask) and torch.equal(pays[k][:nc], one.payload[:nc])
        assert torch.equal(outs[k].view(torch.int16), d["cur"].view(torch.int16))
        assert torch.equal(codes[k], q1.codes) and torch.equal(labels[k], q1.labels)
        assert torch.equal(params[k], q1.params) and torch.equal(deq[k], x1)
