"""Pins for the oracle's format variants of the cluster path (paper: "Cluster Based Quantization for Optimizer
States"): Eq. qmap-distance with a general 256-entry map Q, T^D = Q(T^Q)*S + b, and the cluster-major arrangement
of the codes in Eq. decluster.  Reference values come from brute force, from numpy routines that are the textbook
form of a step (stable sort by key, nearest entry of a sorted table through its midpoints), from closed forms on
hand-made inputs, and from the error bound of a nearest-level code.
"""
import numpy as np
import pytest

import oracle
from paper_2511_12376_amd import synth

KINDS = ["linear", "square", "normal", "steps"]


def _states(seed, n, scale=1e-3):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(n) * scale).astype(np.float32)


# ---------------------------------------------------------------------------------------------
# Eq. decluster: cluster-major codes
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("G,n", [(4096, 3 * 4096 + 517), (1000, 4321), (0, 5000), (256, 256)])
def test_cluster_major_is_a_stable_sort_by_label_inside_each_group(G, n):
    x = _states(1, n)
    a = oracle.quantize_cluster(x, G, 16)
    b = oracle.quantize_cluster_ex(x, G, 16, cluster_major=True)
    assert np.array_equal(a["labels"], b["labels"]) and np.array_equal(a["params"], b["params"])
    lab = oracle.unpack_labels(a["labels"], n)
    g = G if 0 < G <= n else n
    for lo in range(0, n, g):
        hi = min(n, lo + g)
        order = np.argsort(lab[lo:hi], kind="stable")
        assert np.array_equal(b["codes"][lo:hi], a["codes"][lo:hi][order])


def test_cluster_major_on_a_hand_made_group():
    # two clusters split at the mean: (mu, sigma) given, m = 2, so label = (x >= mu)
    x = np.array([5.0, -1.0, 7.0, -3.0, 6.0, -2.0], np.float32)
    fit = np.array([[0.0, 1.0]], np.float32)
    a = oracle.quantize_cluster_ex(x, 0, 2, fit_in=fit)
    b = oracle.quantize_cluster_ex(x, 0, 2, fit_in=fit, cluster_major=True)
    assert list(oracle.unpack_labels(a["labels"], 6)) == [1, 0, 1, 0, 1, 0]
    # cluster 0 = (-1, -3, -2): b = -3, S = 2 -> codes 255, 0, 127.5 -> 128 (tie to even); cluster 1 = (5, 7, 6)
    assert list(a["codes"]) == [0, 255, 255, 0, 128, 128]
    assert list(b["codes"]) == [255, 0, 128, 0, 255, 128]
    out = oracle.dequantize_cluster_ex(b["codes"], b["labels"], b["params"], 6, 0, 2, cluster_major=True)
    assert out[0] == 5.0 and out[1] == -1.0 and out[2] == 7.0 and out[3] == -3.0
    assert abs(out[4] - 6.0) < 2.0 / 255 and abs(out[5] + 2.0) < 2.0 / 255


@pytest.mark.parametrize("G,n,m", [(4096, 2 * 4096 + 100, 16), (512, 5000, 7), (0, 3000, 16), (1024, 1024, 1)])
def test_decluster_returns_every_value_to_its_position(G, n, m):
    x = _states(2, n)
    a = oracle.quantize_cluster(x, G, m)
    b = oracle.quantize_cluster_ex(x, G, m, cluster_major=True)
    want = oracle.dequantize_cluster(a["codes"], a["labels"], a["params"], n, G, m)
    got = oracle.dequantize_cluster_ex(b["codes"], b["labels"], b["params"], n, G, m, cluster_major=True)
    assert np.array_equal(got, want)
    # and the plain arrangement through the extended call is the plain call
    assert np.array_equal(oracle.dequantize_cluster_ex(a["codes"], a["labels"], a["params"], n, G, m), want)


# ---------------------------------------------------------------------------------------------
# Eq. qmap-distance with a table
# ---------------------------------------------------------------------------------------------
def _nearest_by_midpoints(Q, t):
    """Nearest entry of a sorted table: count the midpoints below t (numpy), lowest index among equal entries."""
    Q = Q.astype(np.float64)
    idx = np.searchsorted((Q[:-1] + Q[1:]) / 2, t, side="left")   # a tie at a midpoint goes to the lower entry
    first = np.searchsorted(Q, Q[idx], side="left")               # repeated entries: the first of them
    return first


@pytest.mark.parametrize("kind", KINDS)
def test_table_codes_are_the_nearest_entries(kind):
    Q = synth.qmap_table(kind)
    n = 6000
    x = _states(3, n)
    q = oracle.quantize_cluster_ex(x, 4096, 16, qmap=Q)
    lab = oracle.unpack_labels(q["labels"], n)
    grp = np.arange(n) // 4096
    S = q["params"][grp, lab, 0].astype(np.float64)
    b = q["params"][grp, lab, 1].astype(np.float64)
    ok = S > 0
    t = np.where(ok, (x.astype(np.float64) - b) / np.where(ok, S, 1.0), 0.0)
    want = _nearest_by_midpoints(Q, t)
    Qd = Q.astype(np.float64)
    d_got, d_want = np.abs(Qd[q["codes"]] - t), np.abs(Qd[want] - t)
    differ = q["codes"] != want
    # where the two differ, t sits within fp32 rounding of a midpoint (both entries equally near)
    assert np.all(np.abs(d_got[differ] - d_want[differ]) < 4e-7)
    assert np.count_nonzero(differ) < n // 200
    assert np.all(q["codes"][~ok] == 0)
    # and never a farther entry than any other
    assert np.all(d_got <= np.abs(Qd[None, :] - t[:, None]).min(axis=1) + 4e-7)


@pytest.mark.parametrize("kind", ["square", "normal"])
def test_table_codes_against_exhaustive_search(kind):
    Q = synth.qmap_table(kind)
    rng = np.random.default_rng(5)
    for trial in range(10):
        n = int(rng.integers(1, 65))
        x = (rng.standard_normal(n) * 10.0 ** rng.integers(-8, 2)).astype(np.float32)
        q = oracle.quantize_cluster_ex(x, 0, 4, qmap=Q)
        lab = oracle.unpack_labels(q["labels"], n)
        for i in range(n):
            S, b = q["params"][0, lab[i]]
            j, gap = oracle.code_qmap_bruteforce(x[i], b, S, Q)
            assert q["codes"][i] == j or gap < 4e-7, (i, x[i], j, q["codes"][i], gap)


def test_linear_table_reproduces_the_linear_codes():
    n = 20000
    x = _states(6, n)
    a = oracle.quantize_cluster(x, 4096, 16)
    b = oracle.quantize_cluster_ex(x, 4096, 16, qmap=synth.qmap_table("linear"))
    differ = a["codes"] != b["codes"]
    assert np.count_nonzero(differ) < n // 500          # only positions within rounding of j + 1/2
    assert np.all(np.abs(a["codes"][differ].astype(int) - b["codes"][differ].astype(int)) == 1)
    lab = oracle.unpack_labels(a["labels"], n)
    grp = np.arange(n) // 4096
    S, bb = a["params"][grp, lab, 0].astype(np.float64), a["params"][grp, lab, 1].astype(np.float64)
    pos = (x[differ].astype(np.float64) - bb[differ]) / S[differ] * 255
    assert np.all(np.abs(pos - np.floor(pos) - 0.5) < 1e-3)


def test_exact_ties_and_repeated_entries_take_the_lowest_index():
    # one cluster, b = 0, S = 1 (a power of two: t = x exactly)
    Q = np.linspace(0, 1, 256).astype(np.float32)
    Q[:] = 1.0
    Q[0], Q[1], Q[2], Q[3], Q[4] = 0.0, 0.25, 0.25, 0.75, 0.75      # repeated entries; the rest is 1.0
    x = np.array([0.0, 1.0, 0.5, 0.25, 0.125, 0.75, 0.875, 0.3], np.float32)
    q = oracle.quantize_cluster_ex(x, 0, 1, qmap=Q)
    assert q["params"][0, 0, 0] == 1.0 and q["params"][0, 0, 1] == 0.0
    #            0.0 1.0 0.5(tie 0.25|0.75) 0.25 0.125(tie 0|0.25) 0.75 0.875(tie 0.75|1) 0.3
    assert list(q["codes"]) == [0, 5, 1, 1, 0, 3, 3, 1]


@pytest.mark.parametrize("kind", KINDS)
def test_table_dequantisation_error_is_within_half_a_gap(kind):
    Q = synth.qmap_table(kind)
    n = 3 * 4096 + 11
    x = _states(7, n)
    q = oracle.quantize_cluster_ex(x, 4096, 16, qmap=Q, cluster_major=True)
    xh = oracle.dequantize_cluster_ex(q["codes"], q["labels"], q["params"], n, 4096, 16, qmap=Q, cluster_major=True)
    e = oracle.quantize_cluster_ex(x, 4096, 16, qmap=Q)                 # element order, to look codes up by position
    lab = oracle.unpack_labels(q["labels"], n)
    grp = np.arange(n) // 4096
    S = q["params"][grp, lab, 0].astype(np.float64)
    Qd = Q.astype(np.float64)
    levels = np.unique(Qd)                                              # distinct levels (a table may repeat entries)
    c = np.searchsorted(levels, Qd[e["codes"].astype(int)])
    up = np.where(c < levels.size - 1, levels[np.minimum(c + 1, levels.size - 1)] - levels[c], 0.0)
    dn = np.where(c > 0, levels[c] - levels[np.maximum(c - 1, 0)], 0.0)
    half_gap = np.maximum(up, dn) / 2
    err = np.abs(xh.astype(np.float64) - x.astype(np.float64))
    assert np.all(err <= half_gap * S * (1 + 1e-5) + 4e-7 * S + 2 * np.spacing(np.abs(x)).astype(np.float64))
    # closed form on the ends of every cluster's range: the minimum comes back exactly (Q[0] = 0)
    for g in range(4):
        xs, ls = x[g * 4096:(g + 1) * 4096], lab[g * 4096:(g + 1) * 4096]
        for cl in np.unique(ls):
            i = g * 4096 + np.flatnonzero(ls == cl)[np.argmin(xs[ls == cl])]
            assert xh[i] == x[i]


def test_table_dequantise_on_hand_made_inputs():
    Q = np.zeros(256, np.float32)
    Q[1], Q[2], Q[255] = 0.5, 0.75, 1.0
    params = np.array([[[8.0, -1.0], [2.0, 100.0]]], np.float32)            # (S, b)
    codes = np.array([0, 1, 255, 2], np.uint8)
    labels = np.array([0 | (0 << 4), 1 | (1 << 4)], np.uint8)
    out = oracle.dequantize_cluster_ex(codes, labels, params, 4, 0, 2, qmap=Q)
    assert list(out) == [-1.0, 3.0, 102.0, 101.5]
    # cluster-major: cluster 0 holds elements 0 and 1, cluster 1 elements 2 and 3 -> the same order here; now interleave
    labels = np.array([0 | (1 << 4), 0 | (1 << 4)], np.uint8)               # labels 0, 1, 0, 1
    out = oracle.dequantize_cluster_ex(codes, labels, params, 4, 0, 2, qmap=Q, cluster_major=True)
    # cluster 0's codes are (0, 1), cluster 1's are (255, 2); element order 0:c0[0], 1:c1[0], 2:c0[1], 3:c1[1]
    assert list(out) == [-1.0, 102.0, 3.0, 101.5]
