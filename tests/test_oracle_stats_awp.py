"""Pins for the CPU oracle's per-layer statistics and AWP rule (no GPU)."""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- statistics
def test_closed_forms():
    # constant layers: |W| = |c| * sqrt(n), exactly representable for n = 4^k, c = 2^-3
    sizes = [4 ** k for k in range(0, 9)]
    off = workloads.offsets_from_sizes(sizes)
    w = np.full(int(off[-1]), -0.125, dtype=np.float32)
    st = oracle.stats(w, off)
    for l, n in enumerate(sizes):
        assert st[l, 0] == n / 64.0
        assert st[l, 1] == 0.125 * math.sqrt(n) == 0.125 * 2 ** int(math.log2(n) / 2)
        assert st[l, 2] == 0.125
    # 3-4-5 and 5-12-13 triangles, single non-zero element, empty layer
    w = np.array([3, -4, 5, 12, 0, 0, -7, 0], dtype=np.float32)
    off = np.array([0, 2, 4, 4, 8], dtype=np.int64)
    st = oracle.stats(w, off)
    assert st.tolist() == [[25.0, 5.0, 4.0], [169.0, 13.0, 12.0], [0.0, 0.0, 0.0],
                           [49.0, 7.0, 7.0]]


def test_matches_numpy_and_torch_float64_norms():
    ws = workloads.make_weight_set("tiny")
    off, w = ws.layer_offsets, ws.weights
    st = oracle.stats(w, off)
    for l in range(ws.n_layers):
        seg = w[off[l]:off[l + 1]]
        ref = np.linalg.norm(seg.astype(np.float64))
        tref = torch.linalg.vector_norm(torch.from_numpy(seg), dtype=torch.float64).item()
        assert st[l, 1] == pytest.approx(ref, rel=1e-14)
        assert st[l, 1] == pytest.approx(tref, rel=1e-14)
        assert st[l, 0] == pytest.approx(float(np.sum(seg.astype(np.float64) ** 2)), rel=1e-14)
        assert st[l, 0] == pytest.approx(math.fsum(float(x) * float(x) for x in seg), rel=1e-14)
        assert st[l, 2] == float(np.max(np.abs(seg)))
        assert st[l, 1] == math.sqrt(st[l, 0])


def test_he_normal_statistical_sanity():
    # E[sum w^2] = n * 2 / fan_in = 2 * out_channels; relative sd = sqrt(2/n)
    shapes = workloads.alexnet_shapes()[:5]
    w = workloads.he_normal_weights(shapes, seed=1)
    off = workloads.offsets_from_sizes(workloads.layer_sizes(shapes))
    st = oracle.stats(w, off)
    for l, (o, i, kh, kw) in enumerate(shapes):
        n = o * i * kh * kw
        assert st[l, 0] == pytest.approx(2.0 * o, rel=6 * math.sqrt(2.0 / n))


def test_squares_are_taken_in_double():
    # float32 squares would overflow / underflow; double ones must not
    w = np.array([3e38, 3e38, 1e-30, 1e-30], dtype=np.float32)
    st = oracle.stats(w, np.array([0, 2, 4], dtype=np.int64))
    assert st[0, 1] == pytest.approx(float(np.float32(3e38)) * math.sqrt(2), rel=1e-15)
    assert st[1, 1] == pytest.approx(float(np.float32(1e-30)) * math.sqrt(2), rel=1e-15)


def test_nan_and_inf():
    w = np.array([1.0, np.nan, 2.0, np.inf, -3.0, 1.0], dtype=np.float32)
    st = oracle.stats(w, np.array([0, 3, 5, 6], dtype=np.int64))
    assert np.isnan(st[0]).all()
    assert st[1, 0] == np.inf and st[1, 1] == np.inf and st[1, 2] == np.inf
    assert st[2].tolist() == [1.0, 1.0, 1.0]


# ---------------------------------------------------------------- AWP rule
def run(norms, T, interval, n_bits=8, init_bits=8):
    """norms: [steps][layers]; returns bits, counters, bytes after every step."""
    norms = np.asarray(norms, dtype=np.float64)
    st = oracle.AwpState(norms.shape[1], init_bits)
    hist = []
    for row in norms:
        b = oracle.awp_update(st, row, T, interval, n_bits)
        hist.append((st.bits.copy(), st.counter.copy(), b))
    return hist


def test_constant_norm_upgrades_every_interval_until_32_bits():
    # delta = 0 < T = 0.5 on every batch after the first; INTERVAL = 3
    hist = run([[2.0]] * 16, T=0.5, interval=3)
    bits = [int(h[0][0]) for h in hist]
    # batch 0 only records the norm; batches 1..3 count to 3 -> +8 bits, etc.
    assert bits == [8, 8, 8, 16, 16, 16, 24, 24, 24, 32, 32, 32, 32, 32, 32, 32]
    assert [int(h[2][0]) for h in hist] == [1, 1, 1, 2, 2, 2, 3, 3, 3, 4, 4, 4, 4, 4, 4, 4]
    assert [int(h[1][0]) for h in hist] == [0, 1, 2, 0, 1, 2, 0, 1, 2, 0, 1, 2, 0, 1, 2, 0]


def test_paper_thresholds_never_fire_on_growing_norms():
    facts = json.load(open(os.path.join(GOLDEN, "paper_facts.json")))["awp_parameters"]
    norms = [[1.0 + 0.01 * s, 5.0 * 1.001 ** s] for s in range(50)]
    for net in ("alexnet", "vgg", "resnet"):
        hist = run(norms, T=facts["T"][net], interval=2, n_bits=facts["N"],
                   init_bits=facts["initial_bits"])
        assert all(h[0].tolist() == [8, 8] and h[1].tolist() == [0, 0] for h in hist)


def test_counter_is_cumulative_not_consecutive():
    # relative changes: -10%, +5%, -10%, +5%, -10% ... with T = -0.05, INTERVAL = 3
    norms, v = [[1.0]], 1.0
    for s in range(8):
        v *= 0.9 if s % 2 == 0 else 1.05
        norms.append([v])
    hist = run(norms, T=-0.05, interval=3)
    assert [int(h[1][0]) for h in hist] == [0, 1, 1, 2, 2, 0, 0, 1, 1]
    assert [int(h[0][0]) for h in hist] == [8, 8, 8, 8, 8, 16, 16, 16, 16]


def test_signed_comparison_and_strictness():
    # delta == T exactly does not count (strict <); |delta| is not used
    hist = run([[4.0], [2.0], [1.0], [4.0]], T=-0.5, interval=1)
    assert [int(h[0][0]) for h in hist] == [8, 8, 8, 8]
    hist = run([[4.0], [1.0], [8.0]], T=-0.5, interval=1)
    assert [int(h[0][0]) for h in hist] == [8, 16, 16]


def test_bits_to_bytes_rounds_up():
    facts = json.load(open(os.path.join(GOLDEN, "paper_facts.json")))["bits_to_bytes"]
    for bits, want in ((8, 1), (facts["bits"], facts["bytes"]), (16, 2), (17, 3), (24, 3),
                       (25, 4), (32, 4), (1, 1), (9, 2)):
        st = oracle.AwpState(1, init_bits=bits)
        assert oracle.awp_update(st, [1.0], T=0.0, interval=5)[0] == want


def test_non_byte_step_and_layers_independent():
    # N = 6 bits per upgrade: 8 -> 14 -> 20 -> 26 -> 32 bits = 1, 2, 3, 4, 4 bytes
    norms = [[1.0, 1.0]] + [[1.0, 2.0 ** (s + 1)] for s in range(5)]
    hist = run(norms, T=0.5, interval=1, n_bits=6)
    assert [int(h[0][0]) for h in hist] == [8, 14, 20, 26, 32, 32]
    assert [int(h[2][0]) for h in hist] == [1, 2, 3, 4, 4, 4]
    assert all(int(h[0][1]) == 8 for h in hist)      # layer 1 doubles every batch: delta = 1 >= T


def test_zero_previous_norm():
    hist = run([[0.0], [0.0], [1.0], [1.0]], T=0.5, interval=1)
    # 0 -> 0: delta = 0 < T counts; 0 -> 1: delta = +inf does not; 1 -> 1 counts
    assert [int(h[0][0]) for h in hist] == [8, 16, 16, 24]


# ---------------------------------------------------------------- layer groups
def test_group_norms():
    shapes = workloads.paper_resnet34_shapes()[:9]
    w = workloads.he_normal_weights(shapes, seed=4)
    off = workloads.offsets_from_sizes(workloads.layer_sizes(shapes))
    L = len(shapes)
    # one group over everything is the norm of the whole vector (library routine)
    g_all = oracle.group_norms(w, off, [0, L])
    assert g_all[0] == pytest.approx(np.linalg.norm(w.astype(np.float64)), rel=1e-12)
    # one group per layer reproduces the per-layer norms exactly
    per_layer = oracle.group_norms(w, off, np.arange(L + 1))
    assert per_layer.tolist() == oracle.stats(w, off)[:, 1].tolist()
    # blocks of two layers: Pythagoras over the members, an empty group gives 0
    grp = [0, 1, 3, 3, 5, 7, 9]
    got = oracle.group_norms(w, off, grp)
    st = oracle.stats(w, off)
    for g in range(len(grp) - 1):
        members = st[grp[g]:grp[g + 1], 0]
        assert got[g] == pytest.approx(math.sqrt(float(members.sum())), rel=1e-12, abs=0.0)
    assert got[2] == 0.0
    # 3-4-5 across two layers
    w2 = np.array([3.0, 0.0, 4.0], dtype=np.float32)
    assert oracle.group_norms(w2, np.array([0, 1, 3]), [0, 2])[0] == 5.0
