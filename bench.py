#!/usr/bin/env python3
"""Benchmark of the BitSnap codec hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic checkpoint that is already resident
in HBM: encode_sparse of every bf16 weight tensor against its base, quantize_cluster of the fp32
master weights and both Adam moments, then decode_sparse and dequantize_cluster of everything
that was just produced.  Two ways of issuing it are timed: "batched" (the *_batched entry points:
one launch per operation and state, 8 launches per step) and "per-tensor" (one call per tensor,
2328 launches per step).  --mode picks the one reported as `value`; the other is listed beside it.  The default workload is the Llama-2-7B-shaped checkpoint (291 tensors,
6.74 G parameters, 14 bytes of state per parameter) whose next checkpoint comes from 100
simulated Adam steps.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--limit-tensors N]
                    [--no-cpu-baseline]

Prints ONE JSON line.  `value` is GB/s of input state: (bytes encoded + bytes decoded) / time.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
GROUP, M = 4096, 16


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--p", type=float, default=None, help="change fraction for the Bernoulli configs")
    ap.add_argument("--limit-tensors", type=int, default=0, help="only the first N tensors (debugging)")
    ap.add_argument("--adam-steps", type=int, default=None)
    ap.add_argument("--mode", choices=["batched", "per-tensor"], default="batched",
                    help="which entry points the reported step uses; the other mode is timed too and reported beside it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="only the step: skip the figures reported under extras")
    ap.add_argument("--cpu-sample-tensors", type=int, default=4)
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every tensor is an independent unit; a multi-GPU job runs "
              "one such process per rank on its own shard, with no communication).  Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2511_12376_amd import binding as B
    from paper_2511_12376_amd import synth

    L = B.lib()                      # raises if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = synth.config(args.config, p=args.p)
    tensors = list(range(len(cfg.tensors)))
    if args.limit_tensors:
        tensors = tensors[: args.limit_tensors]
    sizes = [math.prod(cfg.tensors[t][1]) for t in tensors]
    n_total, n_max = sum(sizes), max(sizes)

    # ------------------------------------------------------------------ inputs, resident in HBM
    t0 = time.time()
    inputs = []
    for t in tensors:
        d = synth.make_tensor_torch(cfg, t, dev, adam_steps=args.adam_steps)
        inputs.append(d)
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    # ------------------------------------------------------------------ outputs
    u8, i16, f32, i64 = torch.uint8, torch.int16, torch.float32, torch.int64
    ws = B.new_sparse_workspace(n_max, dev)
    enc = []
    for n in sizes:
        g = B.cluster_groups(n, GROUP)
        e = dict(mask=torch.empty(B.sparse_mask_bytes(n), dtype=u8, device=dev),
                 payload=torch.empty(n, dtype=i16, device=dev),
                 n_changed=torch.zeros(1, dtype=i64, device=dev),
                 q=[dict(codes=torch.empty(n, dtype=u8, device=dev),
                         labels=torch.empty((n + 1) // 2, dtype=u8, device=dev),
                         params=torch.empty(g * M * 2, dtype=f32, device=dev)) for _ in range(3)])
        enc.append(e)
    RING = 4
    dec_ring = [torch.empty(n_max, dtype=torch.bfloat16, device=dev) for _ in range(RING)]
    deq_ring = [torch.empty(n_max, dtype=f32, device=dev) for _ in range(RING)]
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    dec_count = torch.zeros(1, dtype=i64, device=dev)

    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream or None
    ws_bytes = ws.numel()

    # pre-marshalled argument lists: the timed loop is nothing but the C-ABI calls
    calls = {"encode_sparse": [], "quantize_cluster": [], "decode_sparse": [], "dequantize_cluster": []}
    for i, (d, e, n) in enumerate(zip(inputs, enc, sizes)):
        calls["encode_sparse"].append((d["cur"].data_ptr(), d["base"].data_ptr(), n, 2, e["mask"].data_ptr(),
                                       e["payload"].data_ptr(), n, None, e["n_changed"].data_ptr(), ws.data_ptr(),
                                       ws_bytes, sp))
        calls["decode_sparse"].append((d["base"].data_ptr(), e["mask"].data_ptr(), e["payload"].data_ptr(), n, n, 2,
                                       dec_ring[i % RING].data_ptr(), dec_count.data_ptr(), ws.data_ptr(), ws_bytes, sp))
        for j, key in enumerate(("master", "m", "v")):
            q = e["q"][j]
            calls["quantize_cluster"].append((d[key].data_ptr(), n, GROUP, M, q["codes"].data_ptr(),
                                              q["labels"].data_ptr(), q["params"].data_ptr(), None, None,
                                              status.data_ptr(), None, 0, sp))
            calls["dequantize_cluster"].append((q["codes"].data_ptr(), q["labels"].data_ptr(), q["params"].data_ptr(),
                                                n, GROUP, M, deq_ring[(3 * i + j) % RING].data_ptr(), sp))
    # batched form: device item arrays; decoded outputs go to arenas that the three states share
    T = B.sparse_tile_elems()
    dec_arena = torch.empty(n_total, dtype=torch.bfloat16, device=dev)
    deq_arena = torch.empty(n_total, dtype=f32, device=dev)
    starts = [0]
    for n in sizes:
        starts.append(starts[-1] + n)
    dec_out = [dec_arena[starts[i]:starts[i + 1]] for i in range(len(sizes))]
    deq_out = [deq_arena[starts[i]:starts[i + 1]] for i in range(len(sizes))]
    enc_items, total_tiles = B.sparse_items(sizes, src=[d["cur"] for d in inputs], base=[d["base"] for d in inputs],
                                            mask=[e["mask"] for e in enc], payload=[e["payload"] for e in enc],
                                            n_changed=[e["n_changed"] for e in enc])
    dec_items, _ = B.sparse_items(sizes, base=[d["base"] for d in inputs], mask=[e["mask"] for e in enc],
                                  payload=[e["payload"] for e in enc], out=dec_out)
    bws = torch.zeros(B.sparse_batch_workspace_bytes(total_tiles), dtype=u8, device=dev)
    q_items, dq_items, total_groups = [], [], 0
    for j, key in enumerate(("master", "m", "v")):
        qi, total_groups = B.cluster_items([d[key] for d in inputs], [e["q"][j]["codes"] for e in enc],
                                           [e["q"][j]["labels"] for e in enc], [e["q"][j]["params"] for e in enc], GROUP)
        di, _ = B.cluster_items(deq_out, [e["q"][j]["codes"] for e in enc], [e["q"][j]["labels"] for e in enc],
                                [e["q"][j]["params"] for e in enc], GROUP)
        q_items.append(qi)
        dq_items.append(di)
    bcalls = {
        "encode_sparse": [(L.bitsnap_encode_sparse_batched, (enc_items.data_ptr(), len(sizes), total_tiles, bws.data_ptr(), bws.numel(), sp))],
        "quantize_cluster": [(L.bitsnap_quantize_cluster_batched, (qi.data_ptr(), len(sizes), total_groups, GROUP, M, status.data_ptr(), sp)) for qi in q_items],
        "decode_sparse": [(L.bitsnap_decode_sparse_batched, (dec_items.data_ptr(), len(sizes), total_tiles, bws.data_ptr(), bws.numel(), sp))],
        "dequantize_cluster": [(L.bitsnap_dequantize_cluster_batched, (di.data_ptr(), len(sizes), total_groups, GROUP, M, sp)) for di in dq_items],
    }

    fns = {"encode_sparse": L.bitsnap_encode_sparse, "quantize_cluster": L.bitsnap_quantize_cluster,
           "decode_sparse": L.bitsnap_decode_sparse, "dequantize_cluster": L.bitsnap_dequantize_cluster}
    order = ["encode_sparse", "quantize_cluster", "decode_sparse", "dequantize_cluster"]

    def run_step(mode, events=None):
        for k, op in enumerate(order):
            if events is not None:
                events[k].record(stream)
            if mode == "batched":
                for fn, a in bcalls[op]:
                    rc = fn(*a)
                    if rc != 0:
                        raise RuntimeError(f"{op} (batched): {L.bitsnap_error_string(rc).decode()}")
            else:
                fn = fns[op]
                for a in calls[op]:
                    rc = fn(*a)
                    if rc != 0:
                        raise RuntimeError(f"{op}: {L.bitsnap_error_string(rc).decode()}")
        if events is not None:
            events[len(order)].record(stream)

    def time_mode(mode):
        for _ in range(args.warmup):
            run_step(mode)
        torch.cuda.synchronize()
        # the timed region: exactly --steps steps between two synchronisations
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(order) + 1)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s_ in range(args.steps):
            run_step(mode, ev[s_])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        op_ms = {op: sum(ev[s_][k].elapsed_time(ev[s_][k + 1]) for s_ in range(args.steps)) / args.steps
                 for k, op in enumerate(order)}
        return wall * 1e3 / args.steps, op_ms

    other = "per-tensor" if args.mode == "batched" else "batched"
    other_ms, other_op_ms = time_mode(other)
    ms_per_step, op_ms = time_mode(args.mode)
    n_launch = {op: (len(bcalls[op]) if args.mode == "batched" else len(calls[op])) for op in order}

    # what a dependency-free streaming copy sustains on this machine (context for the fractions below,
    # and the kernel the HBM byte counters are calibrated against: it reads and writes cal_bytes)
    cal_bytes = min(1 << 30, n_max * 4) // (1 << 20) * (1 << 20)
    copy_gbps = None
    if cal_bytes > 0:
        cal_src = deq_ring[0].view(torch.uint8)[:cal_bytes]
        cal_dst = deq_ring[1].view(torch.uint8)[:cal_bytes]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for it in range(2):
            e0.record(stream)
            for _ in range(5):
                B.debug_stream_copy(cal_dst, cal_src)
            e1.record(stream)
            torch.cuda.synchronize()
        copy_gbps = 5 * 2 * cal_bytes / (e0.elapsed_time(e1) * 1e-3) / 1e9

    mix_ceiling, extras = None, {}
    state_bytes_of = {"encode_sparse": 2 * n_total, "decode_sparse": 2 * n_total,
                      "quantize_cluster": 12 * n_total, "dequantize_cluster": 12 * n_total}
    if not args.no_extras:
        # what the memory system leaves to win for the cluster codecs: the same bytes in the same pattern, no arithmetic
        mix_n = min(n_max, 1 << 28) // 4096 * 4096
        mix_ceiling = None
        if mix_n > 0:
            mix_b = torch.empty(mix_n, dtype=u8, device=dev)
            mix_h = torch.empty(mix_n // 2, dtype=u8, device=dev)
            mix_w = deq_ring[2][:mix_n]
            mix_ceiling = {}
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for name, to_small in (("quantize_cluster", True), ("dequantize_cluster", False)):
                for it in range(2):
                    e0.record(stream)
                    for _ in range(5):
                        B.debug_stream_mix(mix_w, mix_b, mix_h, to_small)
                    e1.record(stream)
                    torch.cuda.synchronize()
                mix_ceiling[name] = round(5 * 5.5 * mix_n / (e0.elapsed_time(e1) * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
            del mix_b, mix_h

        # ------------------------------------------------------------------ beside the step: one fit per tensor
        # (group = 0, Algorithm 2 as the paper states it) on the first-moment state, one call per tensor;
        # three passes over the tensor instead of one, codes and labels into the same buffers
        gws = torch.empty(max(B.cluster_workspace_bytes(n, 0, M) for n in sizes), dtype=u8, device=dev)
        gparams = torch.empty(M * 2, dtype=f32, device=dev)
        gcalls = [(d["m"].data_ptr(), n, 0, M, e["q"][1]["codes"].data_ptr(), e["q"][1]["labels"].data_ptr(),
                   gparams.data_ptr(), None, None, status.data_ptr(), gws.data_ptr(), gws.numel(), sp)
                  for d, e, n in zip(inputs, enc, sizes)]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for it in range(2):
            e0.record(stream)
            for a in gcalls:
                rc = L.bitsnap_quantize_cluster(*a)
                assert rc == 0, rc
            e1.record(stream)
            torch.cuda.synchronize()
        whole_ms = e0.elapsed_time(e1)
        whole_alg = 3 * 4 * n_total + n_total + (n_total + 1) // 2 + len(sizes) * M * 8
        extras = {"quantize_whole_tensor_fit": {
            "what": "group = 0 (one fit per tensor), first-moment state, one call per tensor, 3 passes over x",
            "ms": round(whole_ms, 3), "api_calls": len(gcalls), "state_GBps": round(4 * n_total / whole_ms / 1e6, 1),
            "hbm_GBps": round(whole_alg / whole_ms / 1e6, 1), "hbm_frac": round(whole_alg / whole_ms / 1e6 / HBM_PEAK_GBS, 4)}}
        del gws
        # the same through one batched call for the whole state (the passes then stream over the list of tensors)
        lparams = [torch.empty(1, M, 2, dtype=f32, device=dev) for _ in sizes]
        litems, lchunks = B.cluster_items([d["m"] for d in inputs], [e["q"][1]["codes"] for e in enc],
                                          [e["q"][1]["labels"] for e in enc], lparams, 0)
        lws = torch.zeros(B.cluster_batch_workspace_bytes(lchunks, len(sizes), 0, 0), dtype=u8, device=dev)
        for it in range(2):
            e0.record(stream)
            B.quantize_cluster_batched_ex(litems, lchunks, 0, M, status=status, workspace=lws)
            e1.record(stream)
            torch.cuda.synchronize()
        list_ms = e0.elapsed_time(e1)
        extras["quantize_whole_tensor_fit"]["batched"] = {
            "ms": round(list_ms, 3), "api_calls": 1, "hbm_GBps": round(whole_alg / list_ms / 1e6, 1),
            "hbm_frac": round(whole_alg / list_ms / 1e6 / HBM_PEAK_GBS, 4)}
        del lws, lparams, litems
        # steady state on the single largest tensor: each op alone, five calls in a row
        big = max(range(len(sizes)), key=lambda i: sizes[i])
        nb = sizes[big]
        largest_ms = {}
        for op in order:
            call = calls[op][big if op.endswith("sparse") else 3 * big]
            fn = getattr(L, "bitsnap_" + op)
            for it in range(2):
                e0.record(stream)
                for _ in range(5):
                    fn(*call)
                e1.record(stream)
                torch.cuda.synchronize()
            largest_ms[op] = e0.elapsed_time(e1) / 5
        nc_big = int(enc[big]["n_changed"].item())
        big_alg = {"encode_sparse": 4 * nb + (nb + 7) // 8 + 2 * nc_big, "decode_sparse": 4 * nb + (nb + 7) // 8 + 2 * nc_big,
                   "quantize_cluster": 5 * nb + (nb + 1) // 2 + B.cluster_groups(nb, GROUP) * M * 8,
                   "dequantize_cluster": 5 * nb + (nb + 1) // 2 + B.cluster_groups(nb, GROUP) * M * 8}
        extras["largest_tensor"] = {"elements": nb, "ops": {op: {"ms": round(largest_ms[op], 4),
                                    "hbm_frac": round(big_alg[op] / largest_ms[op] / 1e6 / HBM_PEAK_GBS, 4)} for op in order}}
        # the sparse encoder's options: delta payload (cur XOR base) and a copy of cur into the next base (here: the
        # decode arena), one batched launch; afterwards the plain encoder restores the value payload
        ex_items, _ = B.sparse_items(sizes, src=[d["cur"] for d in inputs], base=[d["base"] for d in inputs],
                                     mask=[e["mask"] for e in enc], payload=[e["payload"] for e in enc],
                                     n_changed=[e["n_changed"] for e in enc], out=dec_out)
        for it in range(2):
            e0.record(stream)
            rc = L.bitsnap_encode_sparse_batched_ex(ex_items.data_ptr(), len(sizes), total_tiles, 2, B.SPARSE_DELTA,
                                                    bws.data_ptr(), bws.numel(), sp)
            assert rc == 0, rc
            e1.record(stream)
            torch.cuda.synchronize()
        ex_ms = e0.elapsed_time(e1)
        assert all(torch.equal(o.view(i16), d["cur"].view(i16)) for o, d in list(zip(dec_out, inputs))[:4])
        ex_nc = sum(int(e["n_changed"].item()) for e in enc)
        ex_alg = 6 * n_total + sum((n + 7) // 8 for n in sizes) + 2 * ex_nc
        extras["encode_sparse_delta_payload_and_new_base"] = {
            "what": "batched, payload = cur XOR base, cur also copied into a second buffer (the next base)",
            "ms": round(ex_ms, 3), "hbm_GBps": round(ex_alg / ex_ms / 1e6, 1),
            "hbm_frac": round(ex_alg / ex_ms / 1e6 / HBM_PEAK_GBS, 4)}
        fn, a = bcalls["encode_sparse"][0]
        fn(*a)
        torch.cuda.synchronize()

        # decode given the encoder's tile offsets (4 bytes per 32768 elements kept with the mask): no counting
        # pass over the mask, one launch for the whole list
        T2 = B.sparse_tile_elems(2)
        offs = [torch.empty((n + T2 - 1) // T2, dtype=torch.int32, device=dev) for n in sizes]
        o_enc_items, _ = B.sparse_items(sizes, src=[d["cur"] for d in inputs], base=[d["base"] for d in inputs],
                                        mask=[e["mask"] for e in enc], payload=[e["payload"] for e in enc],
                                        n_changed=[e["n_changed"] for e in enc], tile_offsets=offs)
        B.encode_sparse_batched(o_enc_items, total_tiles, bws)
        o_dec_items, _ = B.sparse_items(sizes, base=[d["base"] for d in inputs], mask=[e["mask"] for e in enc],
                                        payload=[e["payload"] for e in enc], out=dec_out, tile_offsets=offs)
        for it in range(2):
            e0.record(stream)
            B.decode_sparse_batched(o_dec_items, total_tiles, bws, flags=B.SPARSE_OFFSETS)
            e1.record(stream)
            torch.cuda.synchronize()
        od_ms = e0.elapsed_time(e1)
        assert all(torch.equal(o.view(i16), d["cur"].view(i16)) for o, d in list(zip(dec_out, inputs))[:4])
        od_alg = 4 * n_total + sum((n + 7) // 8 for n in sizes) + 2 * ex_nc
        extras["decode_sparse_with_encoder_tile_offsets"] = {
            "what": "batched decode that reads the encoder's tile_offsets instead of counting the mask first",
            "ms": round(od_ms, 3), "hbm_frac": round(od_alg / od_ms / 1e6 / HBM_PEAK_GBS, 4)}
        del offs, o_enc_items, o_dec_items

        # the sparse codec on 4-byte elements: the largest tensor's fp32 master weights against a copy in which
        # 30 % of the elements have their lowest mantissa bit flipped (one call each, the steady state of a big tensor)
        m32 = inputs[big]["master"].view(torch.int32)
        g32 = torch.Generator(device=dev)
        g32.manual_seed(synth.seed_for(cfg.index, 9999))
        b32 = m32 ^ (torch.rand(nb, device=dev, generator=g32) < 0.3).to(torch.int32)
        e32 = B.encode_sparse(m32, b32)
        o32, _ = B.decode_sparse(b32, e32.mask, e32.payload, nb, workspace=e32.workspace)
        torch.cuda.synchronize()
        nc32 = int(e32.n_changed.item())
        assert torch.equal(o32, m32) and nc32 == int((m32 != b32).sum().item())
        alg32 = 8 * nb + (nb + 7) // 8 + 4 * nc32
        row32 = {"elements": nb, "changed_fraction": round(nc32 / nb, 4)}
        for name, fn32 in (("encode", lambda: B.encode_sparse_raw(m32, b32, nb, e32.mask, e32.payload, nb, None, e32.n_changed,
                                                                  e32.workspace, elem_bytes=4)),
                           ("decode", lambda: B.decode_sparse_raw(b32, e32.mask, e32.payload, nb, nb, o32, None,
                                                                  e32.workspace, elem_bytes=4))):
            for it in range(2):
                e0.record(stream)
                for _ in range(5):
                    fn32()
                e1.record(stream)
                torch.cuda.synchronize()
            ms32 = e0.elapsed_time(e1) / 5
            row32[name] = {"ms": round(ms32, 4), "hbm_frac": round(alg32 / ms32 / 1e6 / HBM_PEAK_GBS, 4)}
        extras["sparse_32_bit_elements"] = row32
        del m32, b32, e32, o32

        # the cluster pair's format variants on the largest tensor's first Adam moment: a non-linear 256-entry map
        # (bisection in LDS per element) and cluster-major codes (a stable 16-way partition inside the wave)
        xq = inputs[big]["m"].reshape(-1)
        qtab = torch.from_numpy(synth.qmap_table("normal")).to(dev)
        valg = 5 * nb + (nb + 1) // 2 + B.cluster_groups(nb, GROUP) * M * 8
        rows_v = {}
        for label, tab, major in (("cluster-major codes", None, True), ("table map", qtab, False),
                                  ("table map, cluster-major codes", qtab, True)):
            qv = B.quantize_cluster_ex(xq, GROUP, M, qmap=tab, cluster_major=major)
            ov = torch.empty(nb, dtype=torch.float32, device=dev)
            fl = B.CLUSTER_MAJOR if major else 0
            row = {}
            for name, fnv in (("quantize", lambda: B.quantize_cluster_ex_raw(xq, nb, GROUP, M, fl, tab, qv.codes, qv.labels,
                                                                             qv.params, None, None, qv.status)),
                              ("dequantize", lambda: B.dequantize_cluster_ex_raw(qv.codes, qv.labels, qv.params, nb, GROUP, M,
                                                                                 fl, tab, ov))):
                for it in range(2):
                    e0.record(stream)
                    for _ in range(5):
                        fnv()
                    e1.record(stream)
                    torch.cuda.synchronize()
                msv = e0.elapsed_time(e1) / 5
                row[name] = {"ms": round(msv, 4), "hbm_frac": round(valg / msv / 1e6 / HBM_PEAK_GBS, 4)}
            rows_v[label] = row
            del qv, ov
        # the paper's own formulation on the same tensor: one fit and one cluster-major arrangement for the whole tensor
        wsz = B.cluster_workspace_bytes_ex(nb, 0, M, B.CLUSTER_MAJOR)
        wsv = torch.zeros(wsz, dtype=u8, device=dev)
        qv = B.quantize_cluster_ex(xq, 0, M, qmap=qtab, cluster_major=True)
        ov = torch.empty(nb, dtype=torch.float32, device=dev)
        row = {}
        for name, fnv in (("quantize", lambda: B.quantize_cluster_ex_raw(xq, nb, 0, M, B.CLUSTER_MAJOR, qtab, qv.codes, qv.labels,
                                                                         qv.params, None, None, qv.status, wsv)),
                          ("dequantize", lambda: B.dequantize_cluster_ex_raw(qv.codes, qv.labels, qv.params, nb, 0, M,
                                                                             B.CLUSTER_MAJOR, qtab, ov, wsv))):
            for it in range(2):
                e0.record(stream)
                for _ in range(3):
                    fnv()
                e1.record(stream)
                torch.cuda.synchronize()
            row[name] = {"ms": round(e0.elapsed_time(e1) / 3, 4)}
        rows_v["table map, cluster-major codes, one group per tensor"] = row
        del qv, ov, wsv

        # and over the whole first-moment state in one batched launch (table map + cluster-major codes); the plain
        # batched call afterwards restores that state's element-order codes
        alg_state = 5 * n_total + sum((n + 1) // 2 for n in sizes) + total_groups * M * 8
        row_b = {}
        for name, fnb in (("quantize", lambda: B.quantize_cluster_batched_ex(q_items[1], total_groups, GROUP, M, qmap=qtab,
                                                                             cluster_major=True, status=status)),
                          ("dequantize", lambda: B.dequantize_cluster_batched_ex(dq_items[1], total_groups, GROUP, M,
                                                                                 qmap=qtab, cluster_major=True))):
            for it in range(2):
                e0.record(stream)
                fnb()
                e1.record(stream)
                torch.cuda.synchronize()
            msb = e0.elapsed_time(e1)
            row_b[name] = {"ms": round(msb, 3), "hbm_frac": round(alg_state / msb / 1e6 / HBM_PEAK_GBS, 4)}
        fn, a = bcalls["quantize_cluster"][1]
        fn(*a)
        torch.cuda.synchronize()
        extras["cluster_format_variants"] = {"elements": nb, "rows": rows_v,
                                             "batched_first_moment_state_table_map_cluster_major": row_b}

        # the one-call-per-tensor step again, captured once in a HIP graph and replayed: what is left of it when
        # the host no longer issues 2328 calls per step
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        ssp = side.cuda_stream
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for op in order:
                fn = fns[op]
                for a in calls[op]:
                    rc = fn(*(a[:-1] + (ssp,)))
                    assert rc == 0, rc
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        t_g = time.time()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.time() - t_g) / 3 * 1e3
        extras["per_tensor_step_replayed_from_graph"] = {"ms_per_step": round(graph_ms, 3),
                                                         "value_GBps": round(sum(state_bytes_of.values()) / graph_ms / 1e6, 1),
                                                         "kernel_nodes": sum(len(calls[op]) for op in order)}
        del graph

        # quantisation error on these synthetic Adam states, next to plain min-max 8-bit (one cluster): the
        # comparison the paper's evaluation makes on trained states (its table of MRE and MSE against naive
        # 8-bit quantisation); torch only computes the two error measures
        def quality(x, group, m, tab=None):
            q = B.quantize_cluster_ex(x, group, m, qmap=tab)
            xh = B.dequantize_cluster_ex(q.codes, q.labels, q.params, x.numel(), group, m, qmap=tab, workspace=q.workspace)
            err = (xh.double() - x.double())
            nz = x != 0
            return {"MSE": float((err * err).mean().item()),
                    "MRE": float((err[nz].abs() / x[nz].double().abs()).mean().item())}
        sample = min(range(len(sizes)), key=lambda i: abs(sizes[i] - 11008 * 4096))
        extras["quantisation_error_synthetic"] = {
            "tensor": cfg.tensors[tensors[sample]][0], "elements": sizes[sample],
            "rows": {f"{state} {label}": quality(inputs[sample][key], group, m, tab)
                     for state, key in (("adam1", "m"), ("adam2", "v"))
                     for label, group, m, tab in (("16 clusters per 4096-element group", GROUP, M, None),
                                                  ("16 clusters per 4096-element group, levels dense in mid-range", GROUP, M, qtab),
                                                  ("16 clusters per tensor", 0, M, None),
                                                  ("naive 8-bit (1 cluster per tensor)", 0, 1, None),
                                                  ("1 cluster per tensor, levels dense in mid-range", 0, 1, qtab))}}
        # the step's own codes of that state, for whoever looks at the buffers afterwards
        for a in (c for k, c in enumerate(calls["quantize_cluster"]) if k % 3 == 1):
            L.bitsnap_quantize_cluster(*a)
        torch.cuda.synchronize()


    # ------------------------------------------------------------------ accounting
    n_changed = sum(int(e["n_changed"].item()) for e in enc)
    assert int(status.item()) == 0
    p = n_changed / n_total
    groups = sum(B.cluster_groups(n, GROUP) for n in sizes)
    state_bytes = {"encode_sparse": 2 * n_total, "decode_sparse": 2 * n_total,
                   "quantize_cluster": 12 * n_total, "dequantize_cluster": 12 * n_total}
    mask_bytes = sum((n + 7) // 8 for n in sizes)
    sparse_alg = 4 * n_total + mask_bytes + 2 * n_changed           # cur + base (or base + out) + mask + payload
    cluster_alg = 3 * (4 * n_total + n_total + (n_total + 1) // 2 + groups * M * 8)
    alg_bytes = {"encode_sparse": sparse_alg, "decode_sparse": sparse_alg,
                 "quantize_cluster": cluster_alg, "dequantize_cluster": cluster_alg}
    ops = {}
    for op in order:
        sec = op_ms[op] * 1e-3
        ops[op] = {"ms": round(op_ms[op], 3), "api_calls": n_launch[op],
                   "state_GBps": round(state_bytes[op] / sec / 1e9, 1),
                   "hbm_GBps": round(alg_bytes[op] / sec / 1e9, 1),
                   "hbm_frac": round(alg_bytes[op] / sec / 1e9 / HBM_PEAK_GBS, 4)}
    total_state = sum(state_bytes.values())
    value = total_state / (ms_per_step * 1e-3) / 1e9

    dominant = max(order, key=lambda op: op_ms[op])
    bt = "_batched" if args.mode == "batched" else ""
    kernel_name = {"encode_sparse": "encode_sparse_kernel", "decode_sparse": "decode_sparse_kernel",
                   "quantize_cluster": f"quantize_cluster{bt}_kernel<16>",
                   "dequantize_cluster": f"dequantize_cluster{bt}_kernel<16>"}
    launches = len(bcalls[dominant]) if args.mode == "batched" else len(calls[dominant])
    roofline = {"bound": "hbm", "kernel": kernel_name[dominant],
                "achieved": round(alg_bytes[dominant] / (op_ms[dominant] * 1e-3) / 1e9, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(alg_bytes[dominant] / (op_ms[dominant] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "traffic": read_traffic(kernel_name[dominant]),
                "launches_per_step": launches,
                "avg_launch_us": round(op_ms[dominant] * 1e3 / launches, 2),
                "algorithmic_bytes_per_launch": round(alg_bytes[dominant] / launches)}

    out = {"metric": "checkpoint encode/decode GB/s (input state) and % of HBM peak",
           "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "u16 compare + f32 (f64 group statistics)", "data": "synthetic",
           "mode": args.mode,
           "other_mode": {"mode": other, "ms_per_step": round(other_ms, 3),
                          "value": round(total_state / (other_ms * 1e-3) / 1e9, 1),
                          "op_ms": {op: round(other_op_ms[op], 3) for op in order}},
           "config": {"workload": f"configs[{cfg.index}] {cfg.name}-shaped checkpoint: {len(tensors)} tensors, "
                                  f"{n_total} params, bf16 weights vs base + fp32 master/m/v, tensor by tensor",
                      "recipe": cfg.recipe, "changed_fraction": round(p, 4), "group": GROUP, "clusters": M,
                      "state_bytes_per_step": total_state, "generation_s": round(gen_s, 1)},
           "hbm_frac_of_peak": {op: ops[op]["hbm_frac"] for op in order},
           "copy_kernel_GBps": None if copy_gbps is None else round(copy_gbps, 1), "copy_kernel_bytes_each_way": cal_bytes,
           "streaming_ceiling_frac_of_peak": mix_ceiling,
           "ops": ops, "extras": extras, "roofline": roofline}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inputs, sizes, args.cpu_sample_tensors, cfg)
    print(json.dumps(out), flush=True)


def read_traffic(kernel):
    """HBM bytes per launch of the dominant kernel from the committed counter summary, if present:
    a line 'traffic_bytes_per_launch <kernel> <bytes>' in profiles/hbm_traffic_llama2_7b.txt."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_llama2_7b.txt")
    try:
        with open(path) as f:
            for line in f:
                w = line.split()
                if len(w) == 3 and w[0] == "traffic_bytes_per_launch" and w[1] == kernel:
                    return float(w[2])
    except OSError:
        pass
    return None


def cpu_baseline(inputs, sizes, k, cfg):
    """The CPU oracle, as it stands, single thread, on a bounded sample of the same workload: the
    same four operations on the first `k` 2-D tensors after the embeddings."""
    import numpy as np
    import torch

    import oracle

    pick = [i for i, n in enumerate(sizes) if 4_000_000 <= n <= 20_000_000][:k]
    if not pick:
        pick = list(range(min(k, len(sizes))))
    host = []
    for i in pick:
        d = inputs[i]
        host.append(dict(cur=d["cur"].view(torch.int16).cpu().numpy().view(np.uint16),
                         base=d["base"].view(torch.int16).cpu().numpy().view(np.uint16),
                         states=[d[key].cpu().numpy() for key in ("master", "m", "v")]))
    state = 0
    t0 = time.perf_counter()
    for h in host:
        n = h["cur"].size
        mask, payload, nc = oracle.encode_sparse(h["cur"], h["base"])
        oracle.decode_sparse(h["base"], mask, payload)
        for x in h["states"]:
            q = oracle.quantize_cluster(x, GROUP, M)
            oracle.dequantize_cluster(q["codes"], q["labels"], q["params"], n, GROUP, M)
        state += 2 * 14 * n
    sec = time.perf_counter() - t0
    return {"value": round(state / sec / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{len(pick)} tensors of configs[{cfg.index}] ({sum(sizes[i] for i in pick)} params: "
                      f"{', '.join(cfg.tensors[i][0] for i in pick)}), all four operations, {round(sec, 1)} s"}


if __name__ == "__main__":
    main()
