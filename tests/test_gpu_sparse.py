"""GPU parity: encode_sparse / decode_sparse through the C ABI against the CPU oracle, element by
element, bit-exact (masks, offsets, payloads, counts, round trips)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, announce, dev_to_u16, to_np, u16_to_dev
from paper_2511_12376_amd import binding as B
from paper_2511_12376_amd import synth

pytestmark = pytest.mark.gpu

T = B.sparse_tile_elems()
SIZES = [0, 1, 7, 8, 9, 63, 64, 65, 511, 512, 513, 4095, 4096, 4097, 8191, 8193, T - 1, T, T + 1, 2 * T - 1, 2 * T, 3 * T + 777, 1_000_003]


def _pair(n, p, seed):
    rng = np.random.default_rng(seed)
    base = rng.integers(0, 1 << 16, n, dtype=np.uint16)
    cur = base.copy()
    sel = rng.random(n) < p
    cur[sel] ^= rng.integers(1, 1 << 16, n, dtype=np.uint16)[sel]
    return cur, base


def _check_encode(cur, base, ws=None, capacity=None):
    n = cur.size
    o_mask, o_pay, o_nc = oracle.encode_sparse(cur, base)
    enc = B.encode_sparse(u16_to_dev(cur), u16_to_dev(base), want_offsets=True, workspace=ws, capacity=capacity)
    torch.cuda.synchronize()
    nc = int(enc.n_changed.item())
    assert nc == o_nc
    mask = to_np(enc.mask)
    nb = (n + 7) // 8
    assert np.array_equal(mask[:nb], o_mask)
    assert not mask[nb:].any()                                    # padding bytes are zero
    cap = n if capacity is None else capacity
    k = min(nc, cap)
    assert np.array_equal(to_np(enc.payload).view(np.uint16)[:k], o_pay[:k])
    ntiles = (n + T - 1) // T
    offs = oracle.tile_offsets(o_mask, n, T)
    assert np.array_equal(to_np(enc.tile_offsets).view(np.uint32)[:ntiles], offs[:ntiles].astype(np.uint32))
    return enc, o_mask, o_pay, o_nc


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("p", [0.0, 0.06, 0.5, 1.0])
def test_encode_decode_match_oracle(n, p):
    announce("sparse", n, p)
    cur, base = _pair(n, p, 31 * n + int(100 * p))
    enc, o_mask, o_pay, o_nc = _check_encode(cur, base)
    # decode the GPU's own output and the oracle's output; both must give cur back
    out, nch = B.decode_sparse(u16_to_dev(base), enc.mask, enc.payload, o_nc)
    torch.cuda.synchronize()
    assert int(nch.item()) == o_nc
    assert np.array_equal(dev_to_u16(out), cur)
    o_out = oracle.decode_sparse(base, o_mask, o_pay)
    mask_d = torch.zeros(max(B.sparse_mask_bytes(n), 16), dtype=torch.uint8, device=DEV)
    mask_d[: o_mask.size] = torch.from_numpy(o_mask).to(DEV)
    pay_d = torch.from_numpy(np.concatenate([o_pay, np.zeros(8, np.uint16)]).view(np.int16)).to(DEV)
    out2, _ = B.decode_sparse(u16_to_dev(base), mask_d, pay_d, o_nc)
    torch.cuda.synchronize()
    assert np.array_equal(dev_to_u16(out2), o_out)


@pytest.mark.parametrize("tiles", [8, 9, 10, 511, 1376, 2048, 2049, 4095, 4096, 4097])
@pytest.mark.parametrize("elem_bytes", [2, 4])
def test_decode_on_both_sides_of_its_launch_plans(tiles, elem_bytes):
    """A single tensor is decoded by one launch up to 8 tiles, by two (counting kernel + merge that adds up the
    tile counts itself) up to 4096, by three beyond; with the encoder's tile offsets by one launch up to 2048
    tiles and as without them beyond; the last tile is ragged, the changed fraction differs from tile to tile, and
    the decoder runs on the oracle's bytes, also in place."""
    announce("sparse decode launch plans", tiles, elem_bytes)
    te = B.sparse_tile_elems(elem_bytes)
    n = (tiles - 1) * te + 4097
    rng = np.random.default_rng(7000 + 10 * tiles + elem_bytes)
    dt = np.uint16 if elem_bytes == 2 else np.uint32
    base = rng.integers(0, 1 << 16, n, dtype=np.uint16).astype(dt)
    if elem_bytes == 4:
        base |= rng.integers(0, 1 << 16, n, dtype=np.uint32).astype(dt) << 16
    cur = base.copy()
    p_tile = rng.choice([0.0, 0.01, 0.3, 1.0], size=tiles)          # a different changed fraction in every tile
    sel = rng.random(n) < np.repeat(p_tile, te)[:n]
    cur[sel] ^= dt(1)
    if elem_bytes == 2:
        o_mask, o_pay, o_nc = oracle.encode_sparse(cur, base)
        o_out = oracle.decode_sparse(base, o_mask, o_pay)
    else:
        o_mask, o_pay, o_nc = oracle.encode_sparse32(cur, base)
        o_out = oracle.decode_sparse32(base, o_mask, o_pay)
    assert o_nc == int(sel.sum()) and np.array_equal(o_out, cur)
    tdt = torch.int16 if elem_bytes == 2 else torch.int32
    as_dev = lambda a: torch.from_numpy(a.view(np.int16 if elem_bytes == 2 else np.int32)).to(DEV)
    mask_d = torch.zeros(max(B.sparse_mask_bytes(n), 16), dtype=torch.uint8, device=DEV)
    mask_d[: o_mask.size] = torch.from_numpy(o_mask).to(DEV)
    pay_d = as_dev(np.concatenate([o_pay, np.zeros(8, dt)]))
    base_d = as_dev(base)
    out, cnt = B.decode_sparse(base_d, mask_d, pay_d, o_nc)
    torch.cuda.synchronize()
    assert int(cnt.item()) == o_nc
    assert np.array_equal(to_np(out).view(dt), cur)
    inplace = base_d.clone()
    out2, cnt2 = B.decode_sparse(inplace, mask_d, pay_d, o_nc, out=inplace)
    torch.cuda.synchronize()
    assert int(cnt2.item()) == o_nc and np.array_equal(to_np(inplace).view(dt), cur)
    offs = oracle.tile_offsets(o_mask, n, te)[:tiles].astype(np.uint32)
    out3, cnt3 = B.decode_sparse(base_d, mask_d, pay_d, o_nc, tile_offsets=torch.from_numpy(offs.view(np.int32)).to(DEV))
    torch.cuda.synchronize()
    assert int(cnt3.item()) == o_nc and np.array_equal(to_np(out3).view(dt), cur)


@pytest.mark.parametrize("tiles", [9, 1377, 4099])
@pytest.mark.parametrize("elem_bytes", [2, 4])
def test_decode_leaves_nothing_the_encoders_scan_could_read_as_written(tiles, elem_bytes):
    """Decode and encode share a workspace.  The encoder's scan takes a 64-bit word for written only if its two
    top bits are set and its tag equals the call's; whatever the decoder keeps there (tile offsets, tile counts,
    the segments' places) must keep those two bits clear, also for tiles whose every element changed, where the
    places are largest, and for an odd number of tiles, where the places do not start on the counts' last word.
    An encode that follows with the same workspace, at whatever tag, matches the oracle."""
    announce("sparse decode leaves scan words unwritten", tiles, elem_bytes)
    te = B.sparse_tile_elems(elem_bytes)
    n = (tiles - 1) * te + te // 2 + 3
    rng = np.random.default_rng(7100 + tiles + elem_bytes)
    dt = np.uint16 if elem_bytes == 2 else np.uint32
    base = rng.integers(0, 1 << 16, n, dtype=np.uint16).astype(dt)
    cur = base ^ dt(1)                                              # every element changed
    cur[rng.integers(0, n, n // 50)] ^= dt(1)                       # ... but for a few
    as_dev = lambda a: torch.from_numpy(a.view(np.int16 if elem_bytes == 2 else np.int32)).to(DEV)
    o_mask, o_pay, o_nc = (oracle.encode_sparse if elem_bytes == 2 else oracle.encode_sparse32)(cur, base)
    ws = B.new_sparse_workspace(n, DEV, elem_bytes)
    mask_d = torch.zeros(max(B.sparse_mask_bytes(n), 16), dtype=torch.uint8, device=DEV)
    mask_d[: o_mask.size] = torch.from_numpy(o_mask).to(DEV)
    pay_d = as_dev(np.concatenate([o_pay, np.zeros(8, dt)]))
    out, cnt = B.decode_sparse(as_dev(base), mask_d, pay_d, o_nc, workspace=ws)
    torch.cuda.synchronize()
    assert int(cnt.item()) == o_nc and np.array_equal(to_np(out).view(dt), cur)
    words = to_np(ws[256:256 + (ws.numel() - 256) // 8 * 8]).view(np.uint64)
    assert words.any() and not (words >> np.uint64(62)).any()
    hdr = ws[:16].view(torch.int32)
    tags = sorted({int(w >> np.uint64(40)) for w in words[words != 0][-400:]})
    for tag in tags[:3] + tags[-3:]:
        B.decode_sparse(as_dev(base), mask_d, pay_d, o_nc, workspace=ws)
        torch.cuda.synchronize()
        hdr[2] = tag                                                # the tag some word of the decode happens to carry
        torch.cuda.synchronize()
        enc = B.encode_sparse(as_dev(cur), as_dev(base), workspace=ws)
        torch.cuda.synchronize()
        assert int(enc.n_changed.item()) == o_nc
        assert np.array_equal(to_np(enc.mask)[: o_mask.size], o_mask)
        assert np.array_equal(to_np(enc.payload).view(dt)[:o_nc], o_pay)


def test_decode_in_place_and_special_patterns():
    announce("sparse in-place / -0 / NaN")
    pats = np.array([0x0000, 0x8000, 0x7FC1, 0x7FC2, 0x7F80, 0x0001], np.uint16)
    base = np.tile(np.repeat(pats, len(pats)), 300)
    cur = np.tile(np.tile(pats, len(pats)), 300)
    enc, _, _, nc = _check_encode(cur, base)
    assert nc == 300 * len(pats) * (len(pats) - 1)
    buf = u16_to_dev(base)
    B.decode_sparse(buf, enc.mask, enc.payload, nc, out=buf)     # patch the base in place
    torch.cuda.synchronize()
    assert np.array_equal(dev_to_u16(buf), cur)


def test_config0_every_tensor_with_one_workspace():
    cfg = synth.config(0)
    ws = B.new_sparse_workspace(max(np.prod(s) for _, s in cfg.tensors), DEV)
    for t in range(len(cfg.tensors)):
        announce("sparse config0 tensor", t)
        d = synth.make_tensor_np(cfg, t)
        enc, _, _, nc = _check_encode(d["cur"], d["base"], ws=ws)
        assert nc == d["n_changed"]
        out, _ = B.decode_sparse(u16_to_dev(d["base"]), enc.mask, enc.payload, nc, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(dev_to_u16(out), d["cur"])


def test_clustered_runs_config3_shape():
    announce("sparse config3 runs")
    d = synth.make_tensor_np(synth.config(3), 2, n_limit=5_000_000 + 13)
    enc, _, _, nc = _check_encode(d["cur"], d["base"])
    out, _ = B.decode_sparse(u16_to_dev(d["base"]), enc.mask, enc.payload, nc)
    torch.cuda.synchronize()
    assert np.array_equal(dev_to_u16(out), d["cur"])


def test_payload_capacity_overflow_is_reported_not_written():
    announce("sparse capacity overflow")
    n = 3 * T + 100
    cur, base = _pair(n, 0.5, 5)
    cap = 1000
    o_mask, o_pay, o_nc = oracle.encode_sparse(cur, base)
    assert o_nc > cap
    guard = torch.full((cap + 64,), 0x5A5A, dtype=torch.int16, device=DEV)
    mask = torch.empty(B.sparse_mask_bytes(n), dtype=torch.uint8, device=DEV)
    nch = torch.zeros(1, dtype=torch.int64, device=DEV)
    ws = B.new_sparse_workspace(n, DEV)
    B.encode_sparse_raw(u16_to_dev(cur), u16_to_dev(base), n, mask, guard, cap, None, nch, ws)
    torch.cuda.synchronize()
    assert int(nch.item()) == o_nc                                # the true count: overflow is visible
    g = to_np(guard).view(np.uint16)
    assert np.array_equal(g[:cap], o_pay[:cap]) and np.all(g[cap:] == 0x5A5A)
    assert np.array_equal(to_np(mask)[: o_mask.size], o_mask)
    # decode with too few payload elements stays in bounds: surplus elements read as 0
    out, _ = B.decode_sparse(u16_to_dev(base), mask, guard, cap, workspace=ws)
    torch.cuda.synchronize()
    got = dev_to_u16(out)
    bits = np.unpackbits(o_mask, bitorder="little")[:n].astype(bool)
    rank = np.cumsum(bits) - 1
    ok = ~bits | (rank < cap)
    assert np.array_equal(got[ok], cur[ok]) and not got[~ok].any()


def test_workspace_reuse_and_epoch_wrap():
    announce("sparse workspace reuse / epoch wrap")
    nmax = 40 * T
    ws = B.new_sparse_workspace(nmax, DEV)
    hdr = ws[:16].view(torch.int32)
    rng = np.random.default_rng(0)
    for it in range(12):
        if it == 4:
            torch.cuda.synchronize()
            hdr[2] = (1 << 22) - 3                                 # two calls before the 22-bit tag wraps
            torch.cuda.synchronize()
        n = int(rng.integers(1, nmax))
        cur, base = _pair(n, 0.3, 900 + it)
        _check_encode(cur, base, ws=ws)
    torch.cuda.synchronize()
    h = to_np(hdr)
    assert h[0] == 0 and h[1] == 0 and h[3] == 0                   # ticket, done, error are reset
    assert 0 < h[2] < 16                                           # the tag wrapped and started again


def test_spin_limit_knob_needs_its_opt_in(monkeypatch):
    """Without BITSNAP_DEBUG_KNOBS=1 in the environment the test knob does nothing: an encode of 2000 tiles
    after set_spin_limit(1) is as good as any other."""
    announce("sparse spin-limit knob without opt-in")
    monkeypatch.delenv("BITSNAP_DEBUG_KNOBS", raising=False)
    n = 2000 * T
    cur, base = _pair(n, 0.2, 78)
    try:
        B.debug_set_spin_limit(1)
        enc = B.encode_sparse(u16_to_dev(cur), u16_to_dev(base))
        torch.cuda.synchronize()
    finally:
        B.debug_set_spin_limit(0)
    assert int(enc.n_changed.item()) == oracle.encode_sparse(cur, base)[2]


def test_give_up_path_reports_and_recovers(monkeypatch):
    """With a spin limit of one poll, workgroups that have to wait give up.  The call must still
    finish, report the failure through n_changed, and leave the workspace usable."""
    announce("sparse give-up path")
    monkeypatch.setenv("BITSNAP_DEBUG_KNOBS", "1")
    n = 2000 * T
    cur, base = _pair(n, 0.2, 77)
    ws = B.new_sparse_workspace(n, DEV)
    cur_d, base_d = u16_to_dev(cur), u16_to_dev(base)
    try:
        B.debug_set_spin_limit(1)
        enc = B.encode_sparse(cur_d, base_d, workspace=ws)
        torch.cuda.synchronize()
        nc = int(enc.n_changed.item())
    finally:
        B.debug_set_spin_limit(0)
    o_mask, o_pay, o_nc = oracle.encode_sparse(cur, base)
    assert nc == o_nc or nc == -1                                  # UINT64_MAX read as int64
    enc = B.encode_sparse(cur_d, base_d, workspace=ws)             # the same workspace, normal limit
    torch.cuda.synchronize()
    assert int(enc.n_changed.item()) == o_nc
    assert np.array_equal(to_np(enc.payload).view(np.uint16)[:o_nc], o_pay)


def test_full_size_tensor_sampled_tiles():
    """Llama-2-7B's largest tensor shape (32000 x 4096), in the launch configuration the benchmark
    times.  The oracle recomputes sampled tiles one by one; totals are checked through properties
    that hold at any size."""
    announce("sparse full size sampled")
    cfg = synth.config(1, p=0.06)                                  # Bernoulli recipe, cheap to generate
    n = 32000 * 4096
    d = synth.make_tensor_torch(synth.Config(9, "big", "bernoulli", 0.06, 0, (("w", (n,)),)), 0, DEV, want=("base", "cur"))
    enc = B.encode_sparse(d["cur"], d["base"], want_offsets=True)
    out, nch = B.decode_sparse(d["base"], enc.mask, enc.payload, n, workspace=enc.workspace)
    torch.cuda.synchronize()
    nc = int(enc.n_changed.item())
    changed = d["cur"].view(torch.int16) != d["base"].view(torch.int16)
    assert nc == int(changed.sum().item()) == int(nch.item())
    assert torch.equal(out.view(torch.int16), d["cur"].view(torch.int16))
    offs = to_np(enc.tile_offsets).view(np.uint32).astype(np.int64)
    ntiles = n // T
    per_tile = changed.view(ntiles, T).sum(dim=1).cpu().numpy()
    assert np.array_equal(offs, np.concatenate([[0], np.cumsum(per_tile)[:-1]]))
    rng = np.random.default_rng(1)
    cur16, base16 = d["cur"].view(torch.int16), d["base"].view(torch.int16)
    for t in [0, 1, ntiles - 1] + list(rng.integers(0, ntiles, 40)):
        lo = t * T
        c = cur16[lo:lo + T].cpu().numpy().view(np.uint16)
        b = base16[lo:lo + T].cpu().numpy().view(np.uint16)
        o_mask, o_pay, o_nc = oracle.encode_sparse(c, b)
        assert np.array_equal(to_np(enc.mask[lo // 8:(lo + T) // 8]), o_mask)
        assert np.array_equal(to_np(enc.payload[offs[t]:offs[t] + o_nc]).view(np.uint16), o_pay)


def test_batched_equals_oracle_per_tensor():
    """One launch over a list of tensors: the scan restarts at each tensor, every item gets exactly
    the oracle's mask, payload, count and offsets, and the batched decode gives every tensor back."""
    announce("sparse batched")
    sizes = [1, T, T + 1, 5 * T + 77, 9, 3 * T, 200_003, 8, 40 * T - 1, 65]
    ps = [1.0, 0.06, 0.5, 0.7, 0.0, 1.0, 0.06, 0.5, 0.3, 0.2]
    pairs = [_pair(n, p, 4000 + i) for i, (n, p) in enumerate(zip(sizes, ps))]
    cur = [u16_to_dev(c) for c, _ in pairs]
    base = [u16_to_dev(b) for _, b in pairs]
    mask = [torch.full((B.sparse_mask_bytes(n),), 0xEE, dtype=torch.uint8, device=DEV) for n in sizes]
    payload = [torch.zeros(n + 8, dtype=torch.int16, device=DEV) for n in sizes]
    counts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    offs = [torch.zeros((n + T - 1) // T, dtype=torch.int32, device=DEV) for n in sizes]
    items, total = B.sparse_items(sizes, src=cur, base=base, mask=mask, payload=payload, n_changed=counts, tile_offsets=offs)
    ws = torch.zeros(B.sparse_batch_workspace_bytes(total), dtype=torch.uint8, device=DEV)
    for rep in range(2):                                           # twice: the workspace must come back clean
        B.encode_sparse_batched(items, total, ws)
    out = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for n in sizes]
    dcounts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    ditems, dtotal = B.sparse_items(sizes, base=base, mask=mask, payload=payload, out=out, n_changed=dcounts)
    assert dtotal == total
    B.decode_sparse_batched(ditems, total, ws)
    torch.cuda.synchronize()
    for k, (c, b) in enumerate(pairs):
        o_mask, o_pay, o_nc = oracle.encode_sparse(c, b)
        assert int(counts[k].item()) == o_nc == int(dcounts[k].item())
        m = to_np(mask[k])
        assert np.array_equal(m[: o_mask.size], o_mask) and not m[o_mask.size:].any()
        assert np.array_equal(to_np(payload[k]).view(np.uint16)[:o_nc], o_pay)
        o_off = oracle.tile_offsets(o_mask, sizes[k], T)
        assert np.array_equal(to_np(offs[k]).view(np.uint32), o_off[:-1].astype(np.uint32))
        assert np.array_equal(dev_to_u16(out[k]), c)
    # the same workspace still serves a single-tensor call
    enc = B.encode_sparse(cur[3], base[3], workspace=ws)
    torch.cuda.synchronize()
    assert int(enc.n_changed.item()) == int(counts[3].item())


def test_full_size_batched_pass_sampled():
    """The launch configuration the benchmark reports: ONE batched launch over a list of 7B-shaped tensors
    (the 131 M-element embedding, 16.8 M and 45 M matrices, 4096-element norms between them), Adam-recipe
    change pattern.  Whole tensors are checked through properties on the device; the oracle recomputes
    sampled tiles of every tensor."""
    announce("sparse full size batched")
    cfg = synth.config(2)
    picks = [0, 1, 2, 3, 5, 8, 9, 4]                               # embedding, attention and MLP matrices, norms
    data = [synth.make_tensor_torch(cfg, t, DEV, adam_steps=12, want=("base", "cur")) for t in picks]
    sizes = [d["cur"].numel() for d in data]
    cur, base = [d["cur"] for d in data], [d["base"] for d in data]
    mask = [torch.empty(B.sparse_mask_bytes(n), dtype=torch.uint8, device=DEV) for n in sizes]
    payload = [torch.empty(n, dtype=torch.int16, device=DEV) for n in sizes]
    counts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    offs = [torch.zeros((n + T - 1) // T, dtype=torch.int32, device=DEV) for n in sizes]
    items, total = B.sparse_items(sizes, src=cur, base=base, mask=mask, payload=payload, n_changed=counts, tile_offsets=offs)
    ws = torch.zeros(B.sparse_batch_workspace_bytes(total), dtype=torch.uint8, device=DEV)
    B.encode_sparse_batched(items, total, ws)
    out = [torch.empty(n, dtype=torch.bfloat16, device=DEV) for n in sizes]
    dcounts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    ditems, _ = B.sparse_items(sizes, base=base, mask=mask, payload=payload, out=out, n_changed=dcounts)
    B.decode_sparse_batched(ditems, total, ws)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for k, n in enumerate(sizes):
        c16, b16 = cur[k].view(torch.int16), base[k].view(torch.int16)
        changed = c16 != b16
        nc = int(changed.sum().item())
        assert nc == int(counts[k].item()) == int(dcounts[k].item())
        assert 0 < nc < n
        assert torch.equal(out[k].view(torch.int16), c16)          # lossless at full size
        assert torch.equal(payload[k][:nc], c16[changed])          # the changed values, in index order
        ntiles = (n + T - 1) // T
        o = to_np(offs[k]).view(np.uint32).astype(np.int64)
        for t in sorted(set([0, ntiles - 1] + list(rng.integers(0, ntiles, 6)))):
            lo, hi = t * T, min(n, (t + 1) * T)
            o_mask, o_pay, o_nc = oracle.encode_sparse(c16[lo:hi].cpu().numpy().view(np.uint16), b16[lo:hi].cpu().numpy().view(np.uint16))
            assert np.array_equal(to_np(mask[k][lo // 8:lo // 8 + o_mask.size]), o_mask)
            assert np.array_equal(to_np(payload[k][o[t]:o[t] + o_nc]).view(np.uint16), o_pay)


@pytest.mark.parametrize("n", [0, 1, 9, 4097, T - 1, T, 2 * T + 5, 3 * T + 777, 1_000_003])
@pytest.mark.parametrize("p", [0.0, 0.06, 0.7, 1.0])
def test_delta_payload_and_new_base_match_oracle(n, p):
    """The extended entry points: payload = non-zero elements of cur XOR base, and a copy of cur into the
    next base, into a fresh buffer and in place over the base buffer."""
    announce("sparse delta payload / new base", n, p)
    cur, base = _pair(n, p, 9000 + n)
    for delta in (True, False):
        o_mask, o_pay, o_nc = oracle.encode_sparse_ex(cur, base, delta=delta)
        cur_d, base_d = u16_to_dev(cur), u16_to_dev(base)
        fresh = torch.full((max(n, 1),), 0x5A5A, dtype=torch.int16, device=DEV)[:n]
        enc = B.encode_sparse(cur_d, base_d, delta=delta, new_base=fresh, want_offsets=True)
        torch.cuda.synchronize()
        assert int(enc.n_changed.item()) == o_nc
        assert np.array_equal(to_np(enc.mask)[: o_mask.size], o_mask)
        assert np.array_equal(to_np(enc.payload).view(np.uint16)[:o_nc], o_pay)
        assert np.array_equal(to_np(fresh).view(np.uint16), cur)
        assert np.array_equal(dev_to_u16(base_d), base)            # the base itself was left alone
        out, nch = B.decode_sparse(base_d, enc.mask, enc.payload, o_nc, delta=delta, workspace=enc.workspace)
        torch.cuda.synchronize()
        assert int(nch.item()) == o_nc and np.array_equal(dev_to_u16(out), cur)
        assert np.array_equal(dev_to_u16(out), oracle.decode_sparse_ex(base, o_mask, o_pay, delta=delta))
        # in place: the base buffer becomes cur, the encoding is still the one against the old base
        enc2 = B.encode_sparse(cur_d, base_d, delta=delta, new_base=base_d, workspace=enc.workspace)
        torch.cuda.synchronize()
        assert int(enc2.n_changed.item()) == o_nc
        assert np.array_equal(to_np(enc2.mask)[: o_mask.size], o_mask)
        assert np.array_equal(to_np(enc2.payload).view(np.uint16)[:o_nc], o_pay)
        assert np.array_equal(dev_to_u16(base_d), cur)


def test_batched_delta_payload_and_new_base():
    announce("sparse batched delta / new base")
    sizes = [1, T, T + 1, 5 * T + 77, 9, 200_003, 40 * T - 1]
    ps = [1.0, 0.06, 0.5, 0.7, 0.0, 0.06, 0.3]
    pairs = [_pair(n, p, 7000 + i) for i, (n, p) in enumerate(zip(sizes, ps))]
    cur = [u16_to_dev(c) for c, _ in pairs]
    base = [u16_to_dev(b) for _, b in pairs]
    mask = [torch.zeros(B.sparse_mask_bytes(n), dtype=torch.uint8, device=DEV) for n in sizes]
    payload = [torch.zeros(n + 8, dtype=torch.int16, device=DEV) for n in sizes]
    counts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    # every second tensor refreshes its base in place, one gets a fresh copy, the others none
    new_base = [base[k] if k % 2 == 0 else None for k in range(len(sizes))]
    new_base[3] = torch.zeros(sizes[3], dtype=torch.bfloat16, device=DEV)
    items, total = B.sparse_items(sizes, src=cur, base=base, mask=mask, payload=payload, n_changed=counts, out=new_base)
    ws = torch.zeros(B.sparse_batch_workspace_bytes(total), dtype=torch.uint8, device=DEV)
    B.encode_sparse_batched(items, total, ws, flags=B.SPARSE_DELTA)
    torch.cuda.synchronize()
    old_base = [u16_to_dev(b) for _, b in pairs]
    out = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for n in sizes]
    ditems, _ = B.sparse_items(sizes, base=old_base, mask=mask, payload=payload, out=out)
    B.decode_sparse_batched(ditems, total, ws, flags=B.SPARSE_DELTA)
    torch.cuda.synchronize()
    for k, (c, b) in enumerate(pairs):
        o_mask, o_pay, o_nc = oracle.encode_sparse_ex(c, b, delta=True)
        assert int(counts[k].item()) == o_nc
        assert np.array_equal(to_np(mask[k])[: o_mask.size], o_mask)
        assert np.array_equal(to_np(payload[k]).view(np.uint16)[:o_nc], o_pay)
        assert np.array_equal(dev_to_u16(out[k]), c)
        if new_base[k] is not None:
            assert np.array_equal(dev_to_u16(new_base[k]), c)
        else:
            assert np.array_equal(dev_to_u16(base[k]), b)
    # the plain batched call ignores `out` in the encoder
    base2 = [u16_to_dev(b) for _, b in pairs]
    guard = [torch.full((n,), 0x1234, dtype=torch.int16, device=DEV) for n in sizes]
    items2, _ = B.sparse_items(sizes, src=cur, base=base2, mask=mask, payload=payload, n_changed=counts, out=guard)
    B.encode_sparse_batched(items2, total, ws)
    torch.cuda.synchronize()
    assert all(bool((g == 0x1234).all()) for g in guard)


# 32-bit elements -----------------------------------------------------------------------------
T4 = B.sparse_tile_elems(4)


def _pair32(n, p, seed):
    rng = np.random.default_rng(seed)
    base = rng.integers(0, 1 << 32, n, dtype=np.uint32)
    cur = base.copy()
    sel = rng.random(n) < p
    kind = rng.integers(0, 3, n)                                   # low half only, high half only, both
    x = np.where(kind == 0, rng.integers(1, 1 << 16, n), np.where(kind == 1, rng.integers(1, 1 << 16, n) << 16,
                 rng.integers(1, 1 << 32, n))).astype(np.uint32)
    cur[sel] ^= x[sel]
    return cur, base


def _u32_to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int32)).to(DEV)


def _dev_to_u32(t):
    return t.contiguous().view(torch.int32).cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("n", [0, 1, 7, 9, 4097, T4 - 1, T4, T4 + 1, 2 * T4 + 5, 3 * T4 + 777, 1_000_003])
@pytest.mark.parametrize("p", [0.0, 0.06, 0.7, 1.0])
def test_32_bit_elements_match_oracle(n, p):
    """fp32 states through the same entry points (elem_bytes = 4): mask, offsets, payload, count, round trip,
    value and delta payloads, the copy into the next base."""
    announce("sparse 32-bit elements", n, p)
    cur, base = _pair32(n, p, 12000 + n)
    cur_d, base_d = _u32_to_dev(cur), _u32_to_dev(base)
    for delta in (False, True):
        o_mask, o_pay, o_nc = oracle.encode_sparse32(cur, base, delta=delta)
        fresh = torch.full((max(n, 1),), 0x5A5A5A5A, dtype=torch.int32, device=DEV)[:n]
        enc = B.encode_sparse(cur_d, base_d, delta=delta, new_base=fresh, want_offsets=True)
        torch.cuda.synchronize()
        assert int(enc.n_changed.item()) == o_nc
        mask = to_np(enc.mask)
        assert np.array_equal(mask[: o_mask.size], o_mask) and not mask[o_mask.size:].any()
        assert np.array_equal(_dev_to_u32(enc.payload)[:o_nc], o_pay)
        ntiles = (n + T4 - 1) // T4
        offs = oracle.tile_offsets(o_mask, n, T4)
        assert np.array_equal(to_np(enc.tile_offsets).view(np.uint32)[:ntiles], offs[:ntiles].astype(np.uint32))
        assert np.array_equal(_dev_to_u32(fresh), cur)
        out, nch = B.decode_sparse(base_d, enc.mask, enc.payload, o_nc, delta=delta, workspace=enc.workspace)
        torch.cuda.synchronize()
        assert int(nch.item()) == o_nc and np.array_equal(_dev_to_u32(out), cur)
    # in place: decode over the base buffer, and a payload buffer that is too small
    patched = base_d.clone()
    enc = B.encode_sparse(cur_d, base_d)
    B.decode_sparse(patched, enc.mask, enc.payload, int(enc.n_changed.item()), out=patched, workspace=enc.workspace)
    torch.cuda.synchronize()
    assert np.array_equal(_dev_to_u32(patched), cur)
    o_mask, o_pay, o_nc = oracle.encode_sparse32(cur, base)
    if o_nc > 3:
        cap = o_nc // 2
        small = B.encode_sparse(cur_d, base_d, capacity=cap)
        torch.cuda.synchronize()
        assert int(small.n_changed.item()) == o_nc
        assert np.array_equal(_dev_to_u32(small.payload)[:cap], o_pay[:cap])


def test_32_bit_elements_batched():
    announce("sparse 32-bit batched")
    sizes = [1, T4, T4 + 1, 5 * T4 + 77, 9, 200_003, 40 * T4 - 1]
    ps = [1.0, 0.06, 0.5, 0.7, 0.0, 0.06, 0.3]
    pairs = [_pair32(n, p, 13000 + i) for i, (n, p) in enumerate(zip(sizes, ps))]
    cur = [_u32_to_dev(c) for c, _ in pairs]
    base = [_u32_to_dev(b) for _, b in pairs]
    mask = [torch.zeros(B.sparse_mask_bytes(n), dtype=torch.uint8, device=DEV) for n in sizes]
    payload = [torch.zeros(n + 8, dtype=torch.int32, device=DEV) for n in sizes]
    counts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    offs = [torch.zeros((n + T4 - 1) // T4, dtype=torch.int32, device=DEV) for n in sizes]
    items, total = B.sparse_items(sizes, src=cur, base=base, mask=mask, payload=payload, n_changed=counts,
                                  tile_offsets=offs, elem_bytes=4)
    ws = torch.zeros(B.sparse_batch_workspace_bytes(total), dtype=torch.uint8, device=DEV)
    for flags in (0, B.SPARSE_DELTA):
        B.encode_sparse_batched(items, total, ws, flags=flags, elem_bytes=4)
        out = [torch.zeros(n, dtype=torch.int32, device=DEV) for n in sizes]
        ditems, _ = B.sparse_items(sizes, base=base, mask=mask, payload=payload, out=out, elem_bytes=4)
        B.decode_sparse_batched(ditems, total, ws, flags=flags, elem_bytes=4)
        torch.cuda.synchronize()
        for k, (c, b) in enumerate(pairs):
            o_mask, o_pay, o_nc = oracle.encode_sparse32(c, b, delta=bool(flags))
            assert int(counts[k].item()) == o_nc
            assert np.array_equal(to_np(mask[k])[: o_mask.size], o_mask)
            assert np.array_equal(_dev_to_u32(payload[k])[:o_nc], o_pay)
            o_off = oracle.tile_offsets(o_mask, sizes[k], T4)
            assert np.array_equal(to_np(offs[k]).view(np.uint32), o_off[:-1].astype(np.uint32))
            assert np.array_equal(_dev_to_u32(out[k]), c)


@pytest.mark.parametrize("n", [1, 9, 4097, T - 1, T, T + 1, 2 * T + 5, 7 * T + 777, 1_000_003])
@pytest.mark.parametrize("p", [0.0, 0.06, 0.7, 1.0])
def test_decode_with_the_encoders_tile_offsets(n, p):
    """Given the encoder's tile offsets the decoder skips its counting pass; the result and the reported count are
    the same.  Also with the delta payload, with 4-byte elements, and with a payload buffer larger than the count."""
    announce("decode with offsets", n, p)
    cur, base = _pair(n, p, 7000 + n % 997)
    for delta in (False, True):
        enc = B.encode_sparse(u16_to_dev(cur), u16_to_dev(base), want_offsets=True, delta=delta)
        out, cnt = B.decode_sparse(u16_to_dev(base), enc.mask, enc.payload, n, workspace=enc.workspace, delta=delta,
                                   tile_offsets=enc.tile_offsets)
        torch.cuda.synchronize()
        assert np.array_equal(dev_to_u16(out), cur)
        assert int(cnt.item()) == int(enc.n_changed.item()) == int((cur != base).sum())
    T4_ = B.sparse_tile_elems(4)
    rng = np.random.default_rng(n)
    b32 = rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32)
    c32 = b32.copy()
    sel = rng.random(n) < p
    c32[sel] ^= rng.integers(1, 1 << 32, n, dtype=np.uint64).astype(np.uint32)[sel]
    to32 = lambda a: torch.from_numpy(a.view(np.int32)).to(DEV)
    enc = B.encode_sparse(to32(c32), to32(b32), want_offsets=True)
    assert enc.tile_offsets.numel() == max((n + T4_ - 1) // T4_, 1)
    out, cnt = B.decode_sparse(to32(b32), enc.mask, enc.payload, n, workspace=enc.workspace, tile_offsets=enc.tile_offsets)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(out).view(np.uint32), c32) and int(cnt.item()) == int(sel.sum())


def test_batched_decode_with_tile_offsets():
    announce("batched decode with offsets")
    sizes = [1, T, T + 1, 5 * T + 77, 9, 3 * T, 200_003, 8, 40 * T - 1, 65]
    ps = [1.0, 0.06, 0.5, 0.7, 0.0, 1.0, 0.06, 0.5, 0.3, 0.2]
    pairs = [_pair(n, p, 4100 + i) for i, (n, p) in enumerate(zip(sizes, ps))]
    cur = [u16_to_dev(c) for c, _ in pairs]
    base = [u16_to_dev(b) for _, b in pairs]
    mask = [torch.zeros(B.sparse_mask_bytes(n), dtype=torch.uint8, device=DEV) for n in sizes]
    payload = [torch.zeros(n + 8, dtype=torch.int16, device=DEV) for n in sizes]
    counts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    offs = [torch.zeros((n + T - 1) // T, dtype=torch.int32, device=DEV) for n in sizes]
    items, total = B.sparse_items(sizes, src=cur, base=base, mask=mask, payload=payload, n_changed=counts, tile_offsets=offs)
    ws = torch.zeros(B.sparse_batch_workspace_bytes(total), dtype=torch.uint8, device=DEV)
    B.encode_sparse_batched(items, total, ws)
    out = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for n in sizes]
    dcounts = [torch.full((1,), -1, dtype=torch.int64, device=DEV) for _ in sizes]
    ditems, _ = B.sparse_items(sizes, base=base, mask=mask, payload=payload, out=out, n_changed=dcounts, tile_offsets=offs)
    B.decode_sparse_batched(ditems, total, ws, flags=B.SPARSE_OFFSETS)
    torch.cuda.synchronize()
    for k, (c, b) in enumerate(pairs):
        assert np.array_equal(dev_to_u16(out[k]), c), k
        assert int(dcounts[k].item()) == int(counts[k].item()) == int((c != b).sum()), k
    # the workspace was not touched by that decode: an encode right after it is fine
    B.encode_sparse_batched(items, total, ws)
    torch.cuda.synchronize()
    assert int(counts[3].item()) == int((pairs[3][0] != pairs[3][1]).sum())


@pytest.mark.parametrize("elem_bytes", [2, 4])
def test_batched_scan_restarts_at_every_place_of_the_scanning_waves_window(elem_bytes):
    """The scanning wave adds up the tiles' counts 64 at a time (four such windows per round) and restarts at the
    first tile of every tensor.  Lists whose tensors are 1, 2, 62 ... 257 tiles long put those restarts at the
    first and the last lane of a window, several into one window, and none into others; single-tensor calls of the
    same lengths cover windows that end with the tensor.  Counts, offsets and payloads are the oracle's."""
    announce(f"sparse scan windows, {elem_bytes}-byte elements")
    Te = B.sparse_tile_elems(elem_bytes)
    tiles = [1, 1, 1, 2, 59, 1, 63, 1, 64, 65, 1, 1, 127, 128, 1, 255, 256, 257, 1, 62, 2, 1]
    sizes = [t * Te - (k * 997) % (Te - 1) for k, t in enumerate(tiles)]      # ragged last tiles, tile counts as listed
    assert [(n + Te - 1) // Te for n in sizes] == tiles
    mk = _pair if elem_bytes == 2 else _pair32
    pairs = [mk(n, [0.3, 0.0, 1.0, 0.06][k % 4], 9100 + k) for k, n in enumerate(sizes)]
    up = u16_to_dev if elem_bytes == 2 else _u32_to_dev
    dt = torch.int16 if elem_bytes == 2 else torch.int32
    view = np.uint16 if elem_bytes == 2 else np.uint32
    cur = [up(c) for c, _ in pairs]
    base = [up(b) for _, b in pairs]
    mask = [torch.full((B.sparse_mask_bytes(n),), 0xEE, dtype=torch.uint8, device=DEV) for n in sizes]
    payload = [torch.zeros(n + 8, dtype=dt, device=DEV) for n in sizes]
    counts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    offs = [torch.zeros(t, dtype=torch.int32, device=DEV) for t in tiles]
    items, total = B.sparse_items(sizes, src=cur, base=base, mask=mask, payload=payload, n_changed=counts, tile_offsets=offs,
                                  elem_bytes=elem_bytes)
    assert total == sum(tiles)
    ws = torch.zeros(B.sparse_batch_workspace_bytes(total), dtype=torch.uint8, device=DEV)
    B.encode_sparse_batched(items, total, ws, flags=None if elem_bytes == 2 else 0, elem_bytes=elem_bytes)
    torch.cuda.synchronize()
    enc_fn = oracle.encode_sparse if elem_bytes == 2 else oracle.encode_sparse32
    expected = []
    for k, (c, b) in enumerate(pairs):
        o_mask, o_pay, o_nc = enc_fn(c, b)[:3]
        expected.append((o_mask, o_pay, o_nc))
        assert int(counts[k].item()) == o_nc, (k, tiles[k])
        assert np.array_equal(to_np(mask[k])[: o_mask.size], o_mask)
        assert np.array_equal(to_np(payload[k]).view(view)[:o_nc], o_pay), (k, tiles[k])
        o_off = oracle.tile_offsets(o_mask, sizes[k], Te)
        assert np.array_equal(to_np(offs[k]).view(np.uint32), o_off[:-1].astype(np.uint32)), (k, tiles[k])
    # one call per tensor with the same workspace: every window ends with the tensor
    for k in (3, 6, 8, 9, 13, 16, 17):
        pay = torch.zeros(sizes[k] + 8, dtype=dt, device=DEV)
        msk = torch.zeros(B.sparse_mask_bytes(sizes[k]), dtype=torch.uint8, device=DEV)
        nc = torch.zeros(1, dtype=torch.int64, device=DEV)
        off = torch.zeros(tiles[k], dtype=torch.int32, device=DEV)
        B.encode_sparse_raw(cur[k], base[k], sizes[k], msk, pay, sizes[k] + 8, off, nc, ws, elem_bytes=elem_bytes)
        torch.cuda.synchronize()
        o_mask, o_pay, o_nc = expected[k]
        assert int(nc.item()) == o_nc
        assert np.array_equal(to_np(pay).view(view)[:o_nc], o_pay)
        assert np.array_equal(to_np(off).view(np.uint32), oracle.tile_offsets(o_mask, sizes[k], Te)[:-1].astype(np.uint32))
