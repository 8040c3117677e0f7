"""awp_layer_stats_noalloc (the entry point for callers that cannot allocate device
memory) against awp_layer_stats and against the oracle, through the C ABI.

Two calls in a row share the library's fixed scratch array, the second on a
smaller input: stale partials of the first call must not leak into the second.
Collected last (file name), so a failure here hides no other test.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu

STATS_RTOL = 1e-10     # same bar as the other statistics tests (required: 1e-5)


@pytest.fixture(scope="module")
def adt():
    import paper_2004_02297_amd as m
    m.load_library()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_against_both(adt, w, off):
    dw = dev(w)
    L = len(off) - 1
    ref = adt.awp_layer_stats(dw, off)
    out = torch.full((L, 3), -7.0, dtype=torch.float64, device="cuda")
    adt.awp_layer_stats_noalloc(dw, off, out)
    torch.cuda.synchronize()
    got, want = out.cpu().numpy(), ref.cpu().numpy()
    assert got.tobytes() == want.tobytes(), "differs from awp_layer_stats"
    exp = oracle.stats(w, off)
    np.testing.assert_allclose(got, exp, rtol=STATS_RTOL, atol=0.0)
    np.testing.assert_array_equal(got[:, 2], exp[:, 2])        # largest magnitude: exact
    return got


def test_two_calls_in_a_row_second_one_smaller(adt):
    big = workloads.make_weight_set("resnet50")                # 54 layers, 3,139 tiles
    first = check_against_both(adt, big.weights, big.layer_offsets)
    sizes = [5, 0, 8193, 4097, 1, 30000, 8192]                 # ragged, fewer tiles
    off, _, w = workloads.ragged_case(sizes, [1] * len(sizes), seed=41, he=True)
    second = check_against_both(adt, w, off)
    assert second[1].tolist() == [0.0, 0.0, 0.0]               # the empty layer
    # and the big one again: same bits as the first time
    again = check_against_both(adt, big.weights, big.layer_offsets)
    assert again.tobytes() == first.tobytes()


def test_no_device_memory_is_taken(adt):
    ws = workloads.make_weight_set("alexnet")
    dw = dev(ws.weights)
    out = torch.empty((ws.n_layers, 3), dtype=torch.float64, device="cuda")
    adt.awp_layer_stats_noalloc(dw, ws.layer_offsets, out)     # first call: address lookup
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(5):
        adt.awp_layer_stats_noalloc(dw, ws.layer_offsets, out)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
    np.testing.assert_allclose(out.cpu().numpy(), oracle.stats(ws.weights, ws.layer_offsets),
                               rtol=STATS_RTOL, atol=0.0)


def test_non_default_stream_and_nan(adt):
    sizes = [100, 9000, 17]
    off, _, w = workloads.ragged_case(sizes, [1, 1, 1], seed=42, he=True)
    w = w.copy()
    w[int(off[1]) + 5] = np.nan
    dw = dev(w)
    out = torch.empty((3, 3), dtype=torch.float64, device="cuda")
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        adt.awp_layer_stats_noalloc(dw, off, out)
    s.synchronize()
    got, exp = out.cpu().numpy(), oracle.stats(w, off)
    assert np.isnan(got[1]).all() and np.isnan(exp[1]).all()
    np.testing.assert_allclose(got[[0, 2]], exp[[0, 2]], rtol=STATS_RTOL, atol=0.0)


def test_sizes_beyond_the_fixed_scratch_are_refused(adt):
    lib = adt.load_library()
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: the limits are checked first
    ERANGE, EINVAL = -5, -1
    max_tiles = 131072

    def ptr(a):
        return a.ctypes.data_as(ctypes.c_void_p)

    too_many = np.array([0, 8192 * max_tiles + 1], dtype=np.int64)
    assert lib.awp_layer_stats_noalloc(fake, ptr(too_many), 1, fake, None) == ERANGE
    assert b"exceed the fixed scratch" in lib.adt_last_error()
    layers = np.arange(130, dtype=np.int64)                       # 129 layers of one weight
    assert lib.awp_layer_stats_noalloc(fake, ptr(layers), 129, fake, None) == ERANGE
    assert b"at most 128 layers" in lib.adt_last_error()
    assert lib.awp_layer_stats_noalloc(fake, ptr(layers), 2, None, None) == EINVAL
    # empty work succeeds without touching the GPU
    empty = np.array([0], dtype=np.int64)
    assert lib.awp_layer_stats_noalloc(None, ptr(empty), 0, None, None) == 0
