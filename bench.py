#!/usr/bin/env python3
"""Benchmark of the BitSnap codec hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic checkpoint that is already resident
in HBM: encode_sparse of every bf16 weight tensor against its base, quantize_cluster of every fp32
state the configuration has (master weights where it has them, both Adam moments), then
decode_sparse and dequantize_cluster of everything that was just produced.  Two ways of issuing it
are timed: "batched" (the *_batched entry points: one launch per operation, state and batch of
tensors) and "per-tensor" (one call per tensor).  --mode picks the one reported as `value`; the
other is listed beside it.

The default workload is configs[2], the Llama-2-7B-shaped checkpoint (291 tensors, 6.74 G
parameters, 14 bytes of state per parameter) whose next checkpoint comes from 100 simulated Adam
steps.  --config 1 (GPT-2-XL shape, --p sets the changed fraction), 3 (Llama-2-13B shape, changes
in 4096-element runs, weights + both moments) and 4 (one tensor-parallel rank's slice of
Llama-2-70B, 16 bytes of state per parameter resident) run the other checkpoints; the compressed
checkpoint stays resident, decoded tensors go to a bounded, reused region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C] [--p P] [--mode batched|per-tensor]
                    [--batch-elems N] [--limit-tensors N] [--no-extras] [--no-cpu-baseline]

Prints ONE JSON line.  `value` is GB/s of input state: (bytes encoded + bytes decoded) / time.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
GROUP, M = 4096, 16
ORDER = ["encode_sparse", "quantize_cluster", "decode_sparse", "dequantize_cluster"]
# the fp32 states each configuration quantises
STATES = {0: ("m", "v"), 1: ("m", "v"), 2: ("master", "m", "v"), 3: ("m", "v"), 4: ("master", "m", "v")}
# elements per batched launch where the whole list would not leave room for the decoded arenas
DEFAULT_BATCH_ELEMS = {3: 1 << 30, 4: 1 << 30}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--p", type=float, default=None, help="change fraction for the Bernoulli / runs configs")
    ap.add_argument("--limit-tensors", type=int, default=0, help="only the first N tensors (debugging)")
    ap.add_argument("--adam-steps", type=int, default=None)
    ap.add_argument("--mode", choices=["batched", "per-tensor"], default="batched",
                    help="which entry points the reported step uses; the other mode is timed too and reported beside it")
    ap.add_argument("--batch-elems", type=int, default=None,
                    help="batched mode: at most this many elements per launch (0 = the whole list in one launch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="only the step: skip the figures reported under extras")
    ap.add_argument("--cpu-sample-tensors", type=int, default=4)
    return ap.parse_args()


def med(xs):
    return statistics.median(xs)


def progress(*what):
    """A line on stderr per finished stage: a run under a profiler can take minutes between two of them."""
    print("[bench]", *what, file=sys.stderr, flush=True)


def timed(fn, stream, reps=5, rounds=2):
    """ms per call of fn(): `rounds` rounds of `reps` calls between two events, the last round counts."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(rounds):
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every tensor is an independent unit; a multi-GPU job runs "
              "one such process per rank on its own shard, with no communication).  Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2511_12376_amd import binding as B
    from paper_2511_12376_amd import synth

    L = B.lib()                      # raises if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = synth.config(args.config, p=args.p)
    states = STATES[cfg.index]
    S = len(states)
    tensors = list(range(len(cfg.tensors)))
    if args.limit_tensors:
        tensors = tensors[: args.limit_tensors]
    sizes = [math.prod(cfg.tensors[t][1]) for t in tensors]
    n_total, n_max = sum(sizes), max(sizes)
    count = len(sizes)

    # ------------------------------------------------------------------ inputs, resident in HBM
    t0 = time.time()
    def gen_progress(s, steps):
        torch.cuda.synchronize()
        progress(f"simulated Adam step {s} of {steps}")
    inputs = synth.make_checkpoint_torch(cfg, dev, tensors, adam_steps=args.adam_steps, want=("base", "cur") + states,
                                         on_step=gen_progress)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    gen_s = time.time() - t0
    progress(f"inputs generated in {gen_s:.1f} s")

    # ------------------------------------------------------------------ the compressed checkpoint (stays resident)
    u8, i16, f32, i64 = torch.uint8, torch.int16, torch.float32, torch.int64
    ws = B.new_sparse_workspace(n_max, dev)
    enc = []
    for n in sizes:
        g = B.cluster_groups(n, GROUP)
        enc.append(dict(mask=torch.empty(B.sparse_mask_bytes(n), dtype=u8, device=dev),
                        payload=torch.empty(n, dtype=i16, device=dev),
                        n_changed=torch.zeros(1, dtype=i64, device=dev),
                        q=[dict(codes=torch.empty(n, dtype=u8, device=dev),
                                labels=torch.empty((n + 1) // 2, dtype=u8, device=dev),
                                params=torch.empty(g * M * 2, dtype=f32, device=dev)) for _ in range(S)]))
    # decoded tensors: a ring of largest-tensor-sized buffers (per-tensor calls) ...
    RING = 4
    dec_ring = [torch.empty(n_max, dtype=torch.bfloat16, device=dev) for _ in range(RING)]
    deq_ring = [torch.empty(n_max, dtype=f32, device=dev) for _ in range(RING)]
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    dec_count = torch.zeros(1, dtype=i64, device=dev)

    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream or None
    ws_bytes = ws.numel()

    # pre-marshalled argument lists: the timed loop is nothing but the C-ABI calls
    calls = {op: [] for op in ORDER}
    for i, (d, e, n) in enumerate(zip(inputs, enc, sizes)):
        calls["encode_sparse"].append((d["cur"].data_ptr(), d["base"].data_ptr(), n, 2, e["mask"].data_ptr(),
                                       e["payload"].data_ptr(), n, None, e["n_changed"].data_ptr(), ws.data_ptr(),
                                       ws_bytes, sp))
        calls["decode_sparse"].append((d["base"].data_ptr(), e["mask"].data_ptr(), e["payload"].data_ptr(), n, n, 2,
                                       dec_ring[i % RING].data_ptr(), dec_count.data_ptr(), ws.data_ptr(), ws_bytes, sp))
        for j, key in enumerate(states):
            q = e["q"][j]
            calls["quantize_cluster"].append((d[key].data_ptr(), n, GROUP, M, q["codes"].data_ptr(),
                                              q["labels"].data_ptr(), q["params"].data_ptr(), None, None,
                                              status.data_ptr(), None, 0, sp))
            calls["dequantize_cluster"].append((q["codes"].data_ptr(), q["labels"].data_ptr(), q["params"].data_ptr(),
                                                n, GROUP, M, deq_ring[(S * i + j) % RING].data_ptr(), sp))

    # ... and, for the batched calls, two arenas the size of the largest batch, used in turn by the
    # batches and shared by the states.  A batch is a run of consecutive tensors of at most
    # batch_elems elements (the whole list where that fits beside everything else).
    batch_elems = args.batch_elems if args.batch_elems is not None else DEFAULT_BATCH_ELEMS.get(cfg.index, 0)
    batches, lo, acc = [], 0, 0
    for i, n in enumerate(sizes):
        if batch_elems and acc and acc + n > batch_elems:
            batches.append((lo, i))
            lo, acc = i, 0
        acc += n
    batches.append((lo, count))
    arena_elems = max(sum(sizes[a:b]) for a, b in batches)
    n_arenas = 1 if len(batches) == 1 else 2
    dec_arena = [torch.empty(arena_elems, dtype=torch.bfloat16, device=dev) for _ in range(n_arenas)]
    deq_arena = [torch.empty(arena_elems, dtype=f32, device=dev) for _ in range(n_arenas)]
    bcalls = {op: [] for op in ORDER}
    max_tiles, q_items_of_state, dq_items_of_state, dec_out_all, deq_out_all = 0, [[] for _ in states], [[] for _ in states], [], []
    keep = []  # the device item arrays must outlive the calls that use them
    for bi, (a, b) in enumerate(batches):
        bs = sizes[a:b]
        starts = [0]
        for n in bs:
            starts.append(starts[-1] + n)
        dec_out = [dec_arena[bi % n_arenas][starts[k]:starts[k + 1]] for k in range(len(bs))]
        deq_out = [deq_arena[bi % n_arenas][starts[k]:starts[k + 1]] for k in range(len(bs))]
        dec_out_all += dec_out
        deq_out_all += deq_out
        enc_items, tiles = B.sparse_items(bs, src=[d["cur"] for d in inputs[a:b]], base=[d["base"] for d in inputs[a:b]],
                                          mask=[e["mask"] for e in enc[a:b]], payload=[e["payload"] for e in enc[a:b]],
                                          n_changed=[e["n_changed"] for e in enc[a:b]])
        dec_items, _ = B.sparse_items(bs, base=[d["base"] for d in inputs[a:b]], mask=[e["mask"] for e in enc[a:b]],
                                      payload=[e["payload"] for e in enc[a:b]], out=dec_out)
        max_tiles = max(max_tiles, tiles)
        keep += [enc_items, dec_items]
        bcalls["encode_sparse"].append(("s", L.bitsnap_encode_sparse_batched, enc_items, len(bs), tiles))
        bcalls["decode_sparse"].append(("s", L.bitsnap_decode_sparse_batched, dec_items, len(bs), tiles))
        for j, key in enumerate(states):
            qi, groups_b = B.cluster_items([d[key] for d in inputs[a:b]], [e["q"][j]["codes"] for e in enc[a:b]],
                                           [e["q"][j]["labels"] for e in enc[a:b]], [e["q"][j]["params"] for e in enc[a:b]], GROUP)
            di, _ = B.cluster_items(deq_out, [e["q"][j]["codes"] for e in enc[a:b]], [e["q"][j]["labels"] for e in enc[a:b]],
                                    [e["q"][j]["params"] for e in enc[a:b]], GROUP)
            keep += [qi, di]
            q_items_of_state[j].append((qi, groups_b))
            dq_items_of_state[j].append((di, groups_b))
            bcalls["quantize_cluster"].append(("q", L.bitsnap_quantize_cluster_batched, qi, len(bs), groups_b))
            bcalls["dequantize_cluster"].append(("d", L.bitsnap_dequantize_cluster_batched, di, len(bs), groups_b))
    bws = torch.zeros(B.sparse_batch_workspace_bytes(max_tiles), dtype=u8, device=dev)
    for op in ORDER:
        marshalled = []
        for kind, fn, items, cnt, units in bcalls[op]:
            if kind == "s":
                marshalled.append((fn, (items.data_ptr(), cnt, units, bws.data_ptr(), bws.numel(), sp)))
            elif kind == "q":
                marshalled.append((fn, (items.data_ptr(), cnt, units, GROUP, M, status.data_ptr(), sp)))
            else:
                marshalled.append((fn, (items.data_ptr(), cnt, units, GROUP, M, sp)))
        bcalls[op] = marshalled

    fns = {op: getattr(L, "bitsnap_" + op) for op in ORDER}

    def run_step(mode, events=None):
        for k, op in enumerate(ORDER):
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
            events[len(ORDER)].record(stream)

    def time_mode(mode):
        for _ in range(args.warmup):
            run_step(mode)
        torch.cuda.synchronize()
        # the timed region: exactly --steps steps between two synchronisations
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(ORDER) + 1)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s_ in range(args.steps):
            run_step(mode, ev[s_])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        per_step = {op: [ev[s_][k].elapsed_time(ev[s_][k + 1]) for s_ in range(args.steps)] for k, op in enumerate(ORDER)}
        per_step["step"] = [ev[s_][0].elapsed_time(ev[s_][len(ORDER)]) for s_ in range(args.steps)]
        return wall * 1e3 / args.steps, per_step

    other = "per-tensor" if args.mode == "batched" else "batched"
    other_ms, other_per_step = time_mode(other)
    progress(f"{other} mode timed: {other_ms:.3f} ms per step")
    ms_per_step, per_step = time_mode(args.mode)
    progress(f"{args.mode} mode timed: {ms_per_step:.3f} ms per step")
    op_ms = {op: sum(per_step[op]) / args.steps for op in ORDER}
    n_launch = {op: (len(bcalls[op]) if args.mode == "batched" else len(calls[op])) for op in ORDER}

    # what a dependency-free streaming copy sustains on this machine (context for the fractions below,
    # and the kernel the HBM byte counters are calibrated against: it reads and writes cal_bytes)
    cal_bytes = min(1 << 30, n_max * 4) // (1 << 20) * (1 << 20)
    copy_gbps = None
    if cal_bytes > 0:
        cal_src = deq_ring[0].view(torch.uint8)[:cal_bytes]
        cal_dst = deq_ring[1].view(torch.uint8)[:cal_bytes]
        copy_gbps = 2 * cal_bytes / (timed(lambda: B.debug_stream_copy(cal_dst, cal_src), stream) * 1e-3) / 1e9

    # ------------------------------------------------------------------ accounting
    n_changed = sum(int(e["n_changed"].item()) for e in enc)
    assert int(status.item()) == 0
    p = n_changed / n_total
    groups = sum(B.cluster_groups(n, GROUP) for n in sizes)
    state_bytes = {"encode_sparse": 2 * n_total, "decode_sparse": 2 * n_total,
                   "quantize_cluster": 4 * S * n_total, "dequantize_cluster": 4 * S * n_total}
    mask_bytes = sum((n + 7) // 8 for n in sizes)
    sparse_alg = 4 * n_total + mask_bytes + 2 * n_changed           # cur + base (or base + out) + mask + payload
    cluster_alg = S * (4 * n_total + n_total + sum((n + 1) // 2 for n in sizes) + groups * M * 8)
    alg_bytes = {"encode_sparse": sparse_alg, "decode_sparse": sparse_alg,
                 "quantize_cluster": cluster_alg, "dequantize_cluster": cluster_alg}

    def op_rows(ms_lists, launches):
        rows = {}
        for op in ORDER:
            mean = sum(ms_lists[op]) / len(ms_lists[op])
            rows[op] = {"ms": round(mean, 3), "ms_median": round(med(ms_lists[op]), 3), "ms_min": round(min(ms_lists[op]), 3),
                        "api_calls": launches[op], "state_GBps": round(state_bytes[op] / mean / 1e6, 1),
                        "hbm_GBps": round(alg_bytes[op] / mean / 1e6, 1),
                        "hbm_frac": round(alg_bytes[op] / mean / 1e6 / HBM_PEAK_GBS, 4),
                        "algorithmic_bytes": int(round(alg_bytes[op]))}
        return rows

    ops = op_rows(per_step, n_launch)
    other_launch = {op: (len(calls[op]) if args.mode == "batched" else len(bcalls[op])) for op in ORDER}
    other_ops = op_rows(other_per_step, other_launch)
    total_state = sum(state_bytes.values())
    value = total_state / (ms_per_step * 1e-3) / 1e9

    extras = {}
    mix_ceiling = None
    if not args.no_extras:
        ctx = dict(args=args, torch=torch, B=B, L=L, synth=synth, cfg=cfg, dev=dev, stream=stream, sp=sp, inputs=inputs, enc=enc,
                   sizes=sizes, tensors=tensors, states=states, calls=calls, bcalls=bcalls, fns=fns, status=status, ws=ws, bws=bws,
                   dec_out=dec_out_all, deq_out=deq_out_all, deq_ring=deq_ring, dec_ring=dec_ring, batches=batches,
                   q_items=q_items_of_state, dq_items=dq_items_of_state, n_total=n_total, n_max=n_max,
                   state_bytes=state_bytes, p=p)
        mix_ceiling = streaming_ceiling(ctx)
        extras["low_change_fraction"] = low_p_extra(ctx)
        progress("low changed fraction row done")
        if cfg.index == 2 and len(batches) == 1:
            extras.update(config2_extras(ctx))
            progress("extras done")

    dominant = max(ORDER, key=lambda op: op_ms[op])
    batched = args.mode == "batched"
    kernel_name = {"encode_sparse": f"encode_sparse_kernel<{str(batched).lower()}, false, 2, false>",
                   # after its counting kernel; a single tensor of up to 2048 tiles (nearly all of them) takes the form
                   # of the merge that adds up the tile counts itself (source 3), a list the scanned offsets (source 0)
                   "decode_sparse": "decode_merge_kernel<true, false, 0, 2>" if batched else "decode_merge_kernel<false, false, 3, 2>",
                   "quantize_cluster": "quantize_cluster_batched_kernel<16>" if batched else "quantize_cluster_kernel<16>",
                   "dequantize_cluster": "dequantize_cluster_batched_parts_kernel<8>" if batched else "dequantize_cluster_parts_kernel<8>"}
    launches = n_launch[dominant]
    traffic, traffic_src = read_traffic(cfg, p, kernel_name[dominant], args.mode)
    if args.limit_tensors or args.batch_elems is not None:   # the committed counter readings are of the whole workload
        traffic, traffic_src = None, None
    roofline = {"bound": "hbm", "kernel": kernel_name[dominant],
                "achieved": round(alg_bytes[dominant] / (op_ms[dominant] * 1e-3) / 1e9, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(alg_bytes[dominant] / (op_ms[dominant] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_src,
                "launches_per_step": launches,
                "avg_launch_us": round(op_ms[dominant] * 1e3 / launches, 2),
                "algorithmic_bytes_per_launch": round(alg_bytes[dominant] / launches)}

    resident = torch.cuda.memory_allocated() / 1e9
    out = {"metric": "checkpoint encode/decode GB/s (input state) and % of HBM peak",
           "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "u16 compare + f32 (f64 group statistics)", "data": "synthetic",
           "mode": args.mode,
           "step_ms": {"median": round(med(per_step["step"]), 3), "min": round(min(per_step["step"]), 3)},
           "other_mode": {"mode": other, "ms_per_step": round(other_ms, 3),
                          "value": round(total_state / (other_ms * 1e-3) / 1e9, 1),
                          "step_ms": {"median": round(med(other_per_step["step"]), 3), "min": round(min(other_per_step["step"]), 3)},
                          "op_ms": {op: other_ops[op]["ms"] for op in ORDER},
                          "hbm_frac_of_peak": {op: other_ops[op]["hbm_frac"] for op in ORDER},
                          "api_calls": other_launch},
           "config": {"workload": f"configs[{cfg.index}] {cfg.name}-shaped checkpoint: {count} tensors, "
                                  f"{n_total} params, bf16 weights vs base + fp32 {'/'.join(states)}, tensor by tensor",
                      "recipe": cfg.recipe, "changed_fraction": round(p, 4), "group": GROUP, "clusters": M,
                      "states_quantised": list(states), "state_bytes_per_step": total_state,
                      "batched_launch_batches": len(batches), "batch_elems_limit": batch_elems or None,
                      "resident_GB": round(resident, 1), "generation_s": round(gen_s, 1)},
           "hbm_frac_of_peak": {op: ops[op]["hbm_frac"] for op in ORDER},
           "copy_kernel_GBps": None if copy_gbps is None else round(copy_gbps, 1), "copy_kernel_bytes_each_way": cal_bytes,
           "streaming_ceiling_frac_of_peak": mix_ceiling,
           "ops": ops, "extras": extras, "roofline": roofline}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inputs, sizes, states, args.cpu_sample_tensors, cfg)
        progress("cpu baseline done")
    print(json.dumps(out), flush=True)


def streaming_ceiling(c):
    """What the memory system leaves to win for the cluster codecs: the same bytes in the same pattern, no arithmetic."""
    torch, B = c["torch"], c["B"]
    mix_n = min(c["n_max"], 1 << 28) // 4096 * 4096
    if mix_n <= 0:
        return None
    mix_b = torch.empty(mix_n, dtype=torch.uint8, device=c["dev"])
    mix_h = torch.empty(mix_n // 2, dtype=torch.uint8, device=c["dev"])
    mix_w = c["deq_ring"][2][:mix_n]
    res = {}
    for name, to_small in (("quantize_cluster", True), ("dequantize_cluster", False)):
        ms = timed(lambda: B.debug_stream_mix(mix_w, mix_b, mix_h, to_small), c["stream"])
        res[name] = round(5.5 * mix_n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    return res


def low_p_extra(c, p_low=0.06):
    """The sparse pair at the changed fraction the paper works in (a few per cent) on this checkpoint's own
    tensors: a second `cur` in which a Bernoulli(p_low) subset of the base has its lowest bit flipped.  Only the
    weights are touched; the step's own encoded weights are restored afterwards."""
    torch, B, L = c["torch"], c["B"], c["L"]
    if c["cfg"].recipe != "adam" and abs(c["p"] - p_low) < 0.02:
        return {"skipped": "the step itself runs at this changed fraction"}
    sizes, inputs, enc, stream, sp = c["sizes"], c["inputs"], c["enc"], c["stream"], c["sp"]
    gen = torch.Generator(device=c["dev"])
    gen.manual_seed(c["synth"].seed_for(c["cfg"].index, 7777))
    low = [(d["base"].view(torch.int16) ^ (torch.rand(n, device=c["dev"], generator=gen) < p_low).to(torch.int16))
           for d, n in zip(inputs, sizes)]
    rows = {}
    enc_ms, dec_ms = [], []
    for (a, b), (dfn, dargs) in zip(c["batches"], c["bcalls"]["decode_sparse"]):
        items, tiles = B.sparse_items(sizes[a:b], src=low[a:b], base=[d["base"] for d in inputs[a:b]],
                                      mask=[e["mask"] for e in enc[a:b]], payload=[e["payload"] for e in enc[a:b]],
                                      n_changed=[e["n_changed"] for e in enc[a:b]])
        bw = c["bws"]
        enc_ms.append(timed(lambda: B.encode_sparse_batched(items, tiles, bw), stream, reps=3))
        dec_ms.append(timed(lambda: dfn(*dargs), stream, reps=3))
    torch.cuda.synchronize()
    nc = sum(int(e["n_changed"].item()) for e in enc)
    n_total = c["n_total"]
    alg = 4 * n_total + sum((n + 7) // 8 for n in sizes) + 2 * nc
    for name, ms in (("encode_sparse", sum(enc_ms)), ("decode_sparse", sum(dec_ms))):
        rows[name + "_batched"] = {"ms": round(ms, 3), "state_GBps": round(2 * n_total / ms / 1e6, 1),
                                   "hbm_frac": round(alg / ms / 1e6 / HBM_PEAK_GBS, 4)}
    # the largest tensor alone, one call per op
    big = max(range(len(sizes)), key=lambda i: sizes[i])
    nb, e, d = sizes[big], enc[big], inputs[big]
    ws = c["ws"]
    ms_e = timed(lambda: L.bitsnap_encode_sparse(low[big].data_ptr(), d["base"].data_ptr(), nb, 2, e["mask"].data_ptr(),
                                                 e["payload"].data_ptr(), nb, None, e["n_changed"].data_ptr(), ws.data_ptr(),
                                                 ws.numel(), sp), stream)
    ms_d = timed(lambda: L.bitsnap_decode_sparse(*c["calls"]["decode_sparse"][big]), stream)
    torch.cuda.synchronize()
    ncb = int(e["n_changed"].item())
    assert torch.equal(c["dec_ring"][big % len(c["dec_ring"])][:nb].view(torch.int16), low[big])
    algb = 4 * nb + (nb + 7) // 8 + 2 * ncb
    rows["largest_tensor"] = {"elements": nb, "encode_sparse": {"ms": round(ms_e, 4), "hbm_frac": round(algb / ms_e / 1e6 / HBM_PEAK_GBS, 4)},
                              "decode_sparse": {"ms": round(ms_d, 4), "hbm_frac": round(algb / ms_d / 1e6 / HBM_PEAK_GBS, 4)}}
    del low
    for fn, a in c["bcalls"]["encode_sparse"]:     # the step's own masks and payloads again
        fn(*a)
    torch.cuda.synchronize()
    return {"what": f"weights of this checkpoint with a Bernoulli({p_low}) subset of the base changed (lowest bit flipped)",
            "changed_fraction": round(nc / n_total, 4), "compression_ratio": round(2 * n_total / (alg - 4 * n_total), 2), **rows}


def config2_extras(c):
    """Figures reported beside the step on the 7B-shaped checkpoint: the paper's own formulation (one fit per tensor),
    the format options, 4-byte elements, a graph replay of the per-tensor step, synthetic quantisation error."""
    torch, B, L, synth, cfg, dev, stream, sp = c["torch"], c["B"], c["L"], c["synth"], c["cfg"], c["dev"], c["stream"], c["sp"]
    inputs, enc, sizes, status, calls, bcalls, fns = c["inputs"], c["enc"], c["sizes"], c["status"], c["calls"], c["bcalls"], c["fns"]
    dec_out, n_total, tensors = c["dec_out"], c["n_total"], c["tensors"]
    u8, i16, f32 = torch.uint8, torch.int16, torch.float32
    bws = c["bws"]
    total_tiles = bcalls["encode_sparse"][0][1][2]
    q_items = [x[0][0] for x in c["q_items"]]
    dq_items = [x[0][0] for x in c["dq_items"]]
    total_groups = c["q_items"][0][0][1]
    extras = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    # ------------------------------------------------------------------ one fit per tensor
    # (group = 0, Algorithm 2 as the paper states it) on the first-moment state, one call per tensor;
    # three passes over the tensor instead of one, codes and labels into the same buffers
    gws = torch.empty(max(B.cluster_workspace_bytes(n, 0, M) for n in sizes), dtype=u8, device=dev)
    gparams = torch.empty(M * 2, dtype=f32, device=dev)
    gcalls = [(d["m"].data_ptr(), n, 0, M, e["q"][1]["codes"].data_ptr(), e["q"][1]["labels"].data_ptr(),
               gparams.data_ptr(), None, None, status.data_ptr(), gws.data_ptr(), gws.numel(), sp)
              for d, e, n in zip(inputs, enc, sizes)]

    def whole():
        for a in gcalls:
            rc = L.bitsnap_quantize_cluster(*a)
            assert rc == 0, rc
    whole_ms = timed(whole, stream, reps=1)
    whole_alg = 3 * 4 * n_total + n_total + (n_total + 1) // 2 + len(sizes) * M * 8
    extras["quantize_whole_tensor_fit"] = {
        "what": "group = 0 (one fit per tensor), first-moment state, one call per tensor, 3 passes over x",
        "ms": round(whole_ms, 3), "api_calls": len(gcalls), "state_GBps": round(4 * n_total / whole_ms / 1e6, 1),
        "hbm_GBps": round(whole_alg / whole_ms / 1e6, 1), "hbm_frac": round(whole_alg / whole_ms / 1e6 / HBM_PEAK_GBS, 4)}
    del gws
    # the same through one batched call for the whole state (the passes then stream over the list of tensors)
    lparams = [torch.empty(1, M, 2, dtype=f32, device=dev) for _ in sizes]
    litems, lchunks = B.cluster_items([d["m"] for d in inputs], [e["q"][1]["codes"] for e in enc],
                                      [e["q"][1]["labels"] for e in enc], lparams, 0)
    lws = torch.zeros(B.cluster_batch_workspace_bytes(lchunks, len(sizes), 0, 0), dtype=u8, device=dev)
    list_ms = timed(lambda: B.quantize_cluster_batched_ex(litems, lchunks, 0, M, status=status, workspace=lws), stream, reps=1)
    extras["quantize_whole_tensor_fit"]["batched"] = {
        "ms": round(list_ms, 3), "api_calls": 1, "hbm_GBps": round(whole_alg / list_ms / 1e6, 1),
        "hbm_frac": round(whole_alg / list_ms / 1e6 / HBM_PEAK_GBS, 4)}
    del lws, lparams, litems
    # steady state on the single largest tensor: each op alone, five calls in a row
    big = max(range(len(sizes)), key=lambda i: sizes[i])
    nb = sizes[big]
    largest_ms = {}
    for op in ORDER:
        call = calls[op][big if op.endswith("sparse") else 3 * big]
        fn = fns[op]
        largest_ms[op] = timed(lambda: fn(*call), stream)
    nc_big = int(enc[big]["n_changed"].item())
    big_alg = {"encode_sparse": 4 * nb + (nb + 7) // 8 + 2 * nc_big, "decode_sparse": 4 * nb + (nb + 7) // 8 + 2 * nc_big,
               "quantize_cluster": 5 * nb + (nb + 1) // 2 + B.cluster_groups(nb, GROUP) * M * 8,
               "dequantize_cluster": 5 * nb + (nb + 1) // 2 + B.cluster_groups(nb, GROUP) * M * 8}
    extras["largest_tensor"] = {"elements": nb, "ops": {op: {"ms": round(largest_ms[op], 4),
                                "hbm_frac": round(big_alg[op] / largest_ms[op] / 1e6 / HBM_PEAK_GBS, 4)} for op in ORDER}}
    # the sparse encoder's options: delta payload (cur XOR base) and a copy of cur into the next base (here: the
    # decode arena), one batched launch; afterwards the plain encoder restores the value payload
    ex_items, _ = B.sparse_items(sizes, src=[d["cur"] for d in inputs], base=[d["base"] for d in inputs],
                                 mask=[e["mask"] for e in enc], payload=[e["payload"] for e in enc],
                                 n_changed=[e["n_changed"] for e in enc], out=dec_out)

    def ex_call():
        rc = L.bitsnap_encode_sparse_batched_ex(ex_items.data_ptr(), len(sizes), total_tiles, 2, B.SPARSE_DELTA,
                                                bws.data_ptr(), bws.numel(), sp)
        assert rc == 0, rc
    ex_ms = timed(ex_call, stream, reps=1)
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
    od_ms = timed(lambda: B.decode_sparse_batched(o_dec_items, total_tiles, bws, flags=B.SPARSE_OFFSETS), stream, reps=1)
    assert all(torch.equal(o.view(i16), d["cur"].view(i16)) for o, d in list(zip(dec_out, inputs))[:4])
    od_alg = 4 * n_total + sum((n + 7) // 8 for n in sizes) + 2 * ex_nc
    extras["decode_sparse_with_encoder_tile_offsets"] = {
        "what": "batched decode that is given the encoder's tile_offsets (the library reads them instead of counting the mask "
                "for lists of up to 2048 tiles, where that is faster; a longer list decodes as without them)",
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
        ms32 = timed(fn32, stream)
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
            msv = timed(fnv, stream)
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
        row[name] = {"ms": round(timed(fnv, stream, reps=3), 4)}
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
        msb = timed(fnb, stream, reps=1)
        row_b[name] = {"ms": round(msb, 3), "hbm_frac": round(alg_state / msb / 1e6 / HBM_PEAK_GBS, 4)}
    fn, a = bcalls["quantize_cluster"][1]
    fn(*a)
    torch.cuda.synchronize()
    extras["cluster_format_variants"] = {"elements": nb, "rows": rows_v,
                                         "batched_first_moment_state_table_map_cluster_major": row_b}

    # the one-call-per-tensor step again, captured once in a HIP graph and replayed: what is left of it when
    # the host no longer issues one call per tensor and operation
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    ssp = side.cuda_stream
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for op in ORDER:
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
                                                     "value_GBps": round(sum(c["state_bytes"].values()) / graph_ms / 1e6, 1),
                                                     "kernel_nodes": sum(len(calls[op]) for op in ORDER)}
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
    for a in (x for k, x in enumerate(calls["quantize_cluster"]) if k % 3 == 1):
        L.bitsnap_quantize_cluster(*a)
    torch.cuda.synchronize()
    return extras


def traffic_file(cfg, p):
    tag = cfg.name.replace("-", "_")
    if cfg.recipe != "adam":
        tag += "_p%03d" % round(100 * (cfg.p if cfg.p else p))
    return os.path.join(ROOT, "profiles", f"hbm_traffic_{tag}.txt")


def read_traffic(cfg, p, kernel, mode):
    """HBM bytes per launch of the dominant kernel from the committed counter summary of this workload, if there
    is one: a line 'traffic_bytes_per_launch <mode> <kernel> <bytes>' in profiles/hbm_traffic_<workload>.txt (kernel
    names contain blanks; the line is split at its first two and its last one).  -> (bytes or None, where from)."""
    path = traffic_file(cfg, p)
    try:
        with open(path) as f:
            for line in f:
                if not line.startswith("traffic_bytes_per_launch "):
                    continue
                _, md, rest = line.rstrip("\n").split(" ", 2)
                name, _, num = rest.rpartition(" ")
                if md == mode and name == kernel:
                    return float(num), "rocprofv3 FETCH_SIZE + WRITE_SIZE, " + os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def cpu_baseline(inputs, sizes, states, k, cfg):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the same four operations on 2-D
    tensors after the embeddings.  Two legs: one thread on `k` tensors, then three tensors per thread on as many
    threads as this box gives one GPU's job (the oracle is plain C behind ctypes, which releases the
    interpreter lock for the duration of a call; nothing in the oracle changes)."""
    import numpy as np
    import torch
    from concurrent.futures import ThreadPoolExecutor

    import oracle

    cores_total = os.cpu_count() or 1
    threads = max(1, min(16, cores_total))
    pick = [i for i, n in enumerate(sizes) if 2_000_000 <= n <= 30_000_000]
    if not pick:
        pick = list(range(len(sizes)))
    pick_one, pick_all = pick[:k], pick[:3 * threads]

    def to_host(i):
        d = inputs[i]
        return dict(cur=d["cur"].view(torch.int16).cpu().numpy().view(np.uint16),
                    base=d["base"].view(torch.int16).cpu().numpy().view(np.uint16),
                    states=[d[key].cpu().numpy() for key in states])

    def work(h, op_s):
        n = h["cur"].size
        t0 = time.perf_counter()
        mask, payload, _ = oracle.encode_sparse(h["cur"], h["base"])
        t1 = time.perf_counter()
        oracle.decode_sparse(h["base"], mask, payload)
        t2 = time.perf_counter()
        tq = td = 0.0
        for x in h["states"]:
            a = time.perf_counter()
            q = oracle.quantize_cluster(x, GROUP, M)
            b = time.perf_counter()
            oracle.dequantize_cluster(q["codes"], q["labels"], q["params"], n, GROUP, M)
            tq, td = tq + b - a, td + time.perf_counter() - b
        for op, s in zip(ORDER, (t1 - t0, tq, t2 - t1, td)):
            op_s[op] = op_s.get(op, 0.0) + s
        return 2 * (2 + 4 * len(states)) * n

    host = {i: to_host(i) for i in sorted(set(pick_one) | set(pick_all))}
    op_s = {}
    t0 = time.perf_counter()
    state_one = sum(work(host[i], op_s) for i in pick_one)
    sec_one = time.perf_counter() - t0
    n_one = sum(sizes[i] for i in pick_one)
    per_op_one = {op: round((2 if op.endswith("sparse") else 4 * len(states)) * n_one / op_s[op] / 1e9, 4) for op in ORDER}

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as pool:
        state_all = sum(pool.map(lambda i: work(host[i], {}), pick_all))
    sec_all = time.perf_counter() - t0
    used = min(threads, len(pick_all))
    return {"value": round(state_all / sec_all / 1e9, 4), "unit": "GB/s", "cores": used, "cores_total": cores_total,
            "kind": "oracle",
            "sample": f"{len(pick_all)} tensors of configs[{cfg.index}] ({sum(sizes[i] for i in pick_all)} params, one at a time per thread, "
                      f"{used} threads), all four operations, {round(sec_all, 1)} s",
            "one_core": {"value": round(state_one / sec_one / 1e9, 4), "unit": "GB/s", "cores": 1,
                         "state_GBps_per_op": per_op_one,
                         "sample": f"{len(pick_one)} tensors ({n_one} params: "
                                   f"{', '.join(cfg.tensors[i][0] for i in pick_one)}), {round(sec_one, 1)} s"}}


if __name__ == "__main__":
    main()
