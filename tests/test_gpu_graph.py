"""GPU: the batched checkpoint pass captured in a HIP graph.  The library launches kernels only (no
allocation, no memset, its scan state renews itself from call to call), so a captured pass can be
replayed; every replay is compared with the oracle after the inputs were changed eagerly in between."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, announce, dev_to_u16, f32_to_dev, to_np, u16_to_dev
from paper_2511_12376_amd import binding as B

pytestmark = pytest.mark.gpu


def test_batched_pass_replays_from_a_graph():
    announce("graph replay of the batched pass")
    T = B.sparse_tile_elems()
    rng = np.random.default_rng(31)
    sizes = [3 * T + 5, 4096, 70_001, T]
    base_np = [rng.integers(0, 1 << 16, n, dtype=np.uint16) for n in sizes]
    cur = [u16_to_dev(b) for b in base_np]                        # rewritten before every replay
    base = [u16_to_dev(b) for b in base_np]
    xs = [f32_to_dev(np.zeros(n, np.float32)) for n in sizes]     # rewritten before every replay
    mask = [torch.zeros(B.sparse_mask_bytes(n), dtype=torch.uint8, device=DEV) for n in sizes]
    payload = [torch.zeros(n, dtype=torch.int16, device=DEV) for n in sizes]
    counts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    out = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for n in sizes]
    codes = [torch.zeros(n, dtype=torch.uint8, device=DEV) for n in sizes]
    labels = [torch.zeros((n + 1) // 2, dtype=torch.uint8, device=DEV) for n in sizes]
    params = [torch.zeros(B.cluster_groups(n, 4096), 16, 2, dtype=torch.float32, device=DEV) for n in sizes]
    fits = [torch.zeros(B.cluster_groups(n, 4096), 17, dtype=torch.float32, device=DEV) for n in sizes]
    deq = [torch.zeros(n, dtype=torch.float32, device=DEV) for n in sizes]
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    e_items, total = B.sparse_items(sizes, src=cur, base=base, mask=mask, payload=payload, n_changed=counts)
    d_items, _ = B.sparse_items(sizes, base=base, mask=mask, payload=payload, out=out)
    q_items, groups = B.cluster_items(xs, codes, labels, params, 4096, fit_out=fits)
    dq_items, _ = B.cluster_items(deq, codes, labels, params, 4096)
    ws = torch.zeros(B.sparse_batch_workspace_bytes(total), dtype=torch.uint8, device=DEV)

    def one_pass():
        B.encode_sparse_batched(e_items, total, ws)
        B.quantize_cluster_batched(q_items, groups, 4096, 16, status)
        B.decode_sparse_batched(d_items, total, ws)
        B.dequantize_cluster_batched(dq_items, groups, 4096, 16)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_pass()                                                # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        one_pass()
    for rep in range(4):
        cur_np, x_np = [], []
        for k, n in enumerate(sizes):                             # eager work between the replays: new inputs
            c = base_np[k].copy()
            sel = rng.random(n) < (0.05 + 0.3 * rep)
            c[sel] ^= rng.integers(1, 1 << 16, n, dtype=np.uint16)[sel]
            cur_np.append(c)
            cur[k].copy_(u16_to_dev(c))
            x = (rng.standard_normal(n) * 10.0 ** rng.integers(-5, 0)).astype(np.float32)
            x_np.append(x)
            xs[k].copy_(f32_to_dev(x))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        for k, n in enumerate(sizes):
            o_mask, o_pay, o_nc = oracle.encode_sparse(cur_np[k], base_np[k])
            assert int(counts[k].item()) == o_nc, (rep, k)
            assert np.array_equal(to_np(mask[k])[: o_mask.size], o_mask)
            assert np.array_equal(to_np(payload[k]).view(np.uint16)[:o_nc], o_pay)
            assert np.array_equal(dev_to_u16(out[k]), cur_np[k])
            o = oracle.quantize_cluster(x_np[k], 4096, 16, fit_in=to_np(fits[k])[:, :2].copy())
            assert np.array_equal(to_np(codes[k]), o["codes"]) and np.array_equal(to_np(labels[k]), o["labels"])
            assert np.array_equal(to_np(params[k]).reshape(-1, 16, 2), o["params"])
            assert np.array_equal(to_np(deq[k]), oracle.dequantize_cluster(o["codes"], o["labels"], o["params"], n, 4096, 16))


def test_one_group_per_tensor_pass_replays_from_a_graph():
    """The multi-pass kernels over a list of tensors (group = 0), with a table and cluster-major codes, and the sparse
    decode that takes the encoder's tile offsets: nine, four and one kernel launches, nothing else."""
    announce("graph replay of the whole-tensor-group pass")
    from paper_2511_12376_amd import synth
    T = B.sparse_tile_elems()
    rng = np.random.default_rng(32)
    sizes = [300 * 4096 + 5, 4096, 70_001, 3]
    Q = synth.qmap_table("normal")
    Qd = f32_to_dev(Q)
    xs = [f32_to_dev(np.zeros(n, np.float32)) for n in sizes]
    codes = [torch.zeros(n, dtype=torch.uint8, device=DEV) for n in sizes]
    labels = [torch.zeros((n + 1) // 2, dtype=torch.uint8, device=DEV) for n in sizes]
    params = [torch.zeros(1, 16, 2, dtype=torch.float32, device=DEV) for n in sizes]
    fits = [torch.zeros(1, 17, dtype=torch.float32, device=DEV) for n in sizes]
    deq = [torch.zeros(n, dtype=torch.float32, device=DEV) for n in sizes]
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    q_items, chunks = B.cluster_items(xs, codes, labels, params, 0, fit_out=fits)
    dq_items, _ = B.cluster_items(deq, codes, labels, params, 0)
    cws = torch.zeros(B.cluster_batch_workspace_bytes(chunks, len(sizes), 0, B.CLUSTER_MAJOR), dtype=torch.uint8, device=DEV)
    base_np = [rng.integers(0, 1 << 16, n, dtype=np.uint16) for n in sizes]
    cur = [u16_to_dev(b) for b in base_np]
    base = [u16_to_dev(b) for b in base_np]
    mask = [torch.zeros(B.sparse_mask_bytes(n), dtype=torch.uint8, device=DEV) for n in sizes]
    payload = [torch.zeros(n, dtype=torch.int16, device=DEV) for n in sizes]
    counts = [torch.zeros(1, dtype=torch.int64, device=DEV) for _ in sizes]
    offs = [torch.zeros((n + T - 1) // T, dtype=torch.int32, device=DEV) for n in sizes]
    out = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for n in sizes]
    e_items, total = B.sparse_items(sizes, src=cur, base=base, mask=mask, payload=payload, n_changed=counts, tile_offsets=offs)
    d_items, _ = B.sparse_items(sizes, base=base, mask=mask, payload=payload, out=out, tile_offsets=offs)
    ws = torch.zeros(B.sparse_batch_workspace_bytes(total), dtype=torch.uint8, device=DEV)

    def one_pass():
        B.quantize_cluster_batched_ex(q_items, chunks, 0, 16, qmap=Qd, cluster_major=True, status=status, workspace=cws)
        B.dequantize_cluster_batched_ex(dq_items, chunks, 0, 16, qmap=Qd, cluster_major=True, workspace=cws)
        B.encode_sparse_batched(e_items, total, ws)
        B.decode_sparse_batched(d_items, total, ws, flags=B.SPARSE_OFFSETS)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_pass()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        one_pass()
    for rep in range(3):
        x_np, cur_np = [], []
        for k, n in enumerate(sizes):
            x = (rng.standard_normal(n) * 10.0 ** rng.integers(-5, 0)).astype(np.float32)
            x_np.append(x)
            xs[k].copy_(f32_to_dev(x))
            c = base_np[k].copy()
            sel = rng.random(n) < (0.1 + 0.4 * rep)
            c[sel] ^= rng.integers(1, 1 << 16, n, dtype=np.uint16)[sel]
            cur_np.append(c)
            cur[k].copy_(u16_to_dev(c))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        for k, n in enumerate(sizes):
            o = oracle.quantize_cluster_ex(x_np[k], 0, 16, fit_in=to_np(fits[k])[:, :2].copy(), qmap=Q, cluster_major=True)
            assert np.array_equal(to_np(codes[k]), o["codes"]) and np.array_equal(to_np(labels[k]), o["labels"]), (rep, k)
            assert np.array_equal(to_np(params[k]), o["params"])
            assert np.array_equal(to_np(deq[k]), oracle.dequantize_cluster_ex(o["codes"], o["labels"], o["params"], n, 0, 16,
                                                                              qmap=Q, cluster_major=True))
            assert int(counts[k].item()) == int((cur_np[k] != base_np[k]).sum())
            assert np.array_equal(dev_to_u16(out[k]), cur_np[k])
