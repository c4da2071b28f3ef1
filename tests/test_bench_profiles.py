"""The counter summaries under profiles/ are what bench.py quotes as roofline.traffic: every workload the
bench can run has one, and every line bench.py looks up is there and plausible (host logic only, no GPU)."""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2511_12376_amd import synth  # noqa: E402

WORKLOADS = [(1, 0.01), (1, 0.06), (1, 0.2), (2, None), (3, None), (4, None)]
KERNELS = {
    "batched": ["encode_sparse_kernel<true, false, 2, false>", "decode_merge_kernel<true, false, 0, 2>",
                "quantize_cluster_batched_kernel<16>", "dequantize_cluster_batched_parts_kernel<8>"],
    "per-tensor": ["encode_sparse_kernel<false, false, 2, false>", "decode_merge_kernel<false, false, 3, 2>",
                   "quantize_cluster_kernel<16>", "dequantize_cluster_parts_kernel<8>"],
}


@pytest.mark.parametrize("index,p", WORKLOADS)
def test_every_workload_has_its_counter_summary(index, p):
    cfg = synth.config(index, p=p)
    path = bench.traffic_file(cfg, cfg.p if cfg.p else 0.7095)
    assert os.path.exists(path), path
    trace = path.replace("hbm_traffic_", "kernel_trace_")
    assert os.path.exists(trace), trace
    text = open(path).read()
    assert "rocprofv3 --pmc FETCH_SIZE" in text and "rocprofv3 --pmc WRITE_SIZE" in text   # the commands are in the file
    n_total = sum(__import__("math").prod(shape) for _, shape in cfg.tensors)
    for mode, names in KERNELS.items():
        for name in names:
            traffic, src = bench.read_traffic(cfg, cfg.p if cfg.p else 0.7095, name, mode)
            assert traffic is not None and traffic > 0, (mode, name)
            assert src and os.path.basename(path) in src
            if mode == "batched":   # a launch moves between 4 and 8 bytes per element it covers, and covers at most the whole state
                assert traffic <= 8 * n_total


def test_unknown_kernel_or_workload_gives_no_number():
    cfg = synth.config(2)
    assert bench.read_traffic(cfg, 0.7095, "no_such_kernel<1>", "batched") == (None, None)
    cfg1 = synth.config(1, p=0.5)   # no summary was made at this changed fraction
    assert bench.read_traffic(cfg1, 0.5, KERNELS["batched"][0], "batched") == (None, None)
