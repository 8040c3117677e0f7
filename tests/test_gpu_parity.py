"""GPU parity: libadt (through its C ABI) against the CPU oracle, bit for bit.

Pack streams and unpacked words must be identical to the oracle's; statistics
must agree to 1e-5 relative (the stated bar) and are checked to 1e-10: both
sides add exact double-precision squares, in different orders; the oracle's
index-order sum of n terms carries a rounding error of about sqrt(n) * 2^-53
(1e-12 at n = 1e8), the kernels' tree-shaped sum less.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu

STATS_RTOL_BAR = 1e-5      # the required tolerance
STATS_RTOL = 1e-10         # what the kernels are expected to reach
MASK = {1: 0xFF000000, 2: 0xFFFF0000, 3: 0xFFFFFF00, 4: 0xFFFFFFFF}


@pytest.fixture(scope="module")
def adt():
    import paper_2004_02297_amd as m
    m.load_library()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_pack_unpack(adt, w, off, rb, w_shift=0, p_shift=0):
    """Pack + unpack on the GPU with guard bytes around both outputs and the
    given misalignment of the base pointers (w_shift in elements, p_shift in
    bytes); compare with the oracle."""
    n = int(off[-1])
    size = oracle.packed_size(off, rb)
    exp_stream = oracle.pack(w, off, rb)
    exp_back = oracle.unpack(exp_stream, off, rb)

    guard = 64
    wbuf = torch.zeros(n + w_shift + 8, dtype=torch.float32, device="cuda")
    wview = wbuf[w_shift:w_shift + n]
    wview.copy_(torch.from_numpy(w))
    pbuf = torch.full((size + p_shift + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
    pview = pbuf[guard + p_shift:guard + p_shift + size]
    adt.adt_pack(wview, off, rb, out=pview)
    got = pbuf.cpu().numpy()
    lo, hi = guard + p_shift, guard + p_shift + size
    assert np.all(got[:lo] == 0xA5) and np.all(got[hi:] == 0xA5), "pack wrote outside its stream"
    assert np.array_equal(got[lo:hi], exp_stream), "packed stream differs from the oracle"

    obuf = torch.full((n + w_shift + 2 * guard,), float("nan"), dtype=torch.float32, device="cuda")
    obuf.view(torch.int32).fill_(0x5A5A5A5A)
    oview = obuf[guard + w_shift:guard + w_shift + n]
    adt.adt_unpack(pview, off, rb, out=oview)
    gotw = obuf.view(torch.int32).cpu().numpy().view(np.uint32)
    lo, hi = guard + w_shift, guard + w_shift + n
    assert np.all(gotw[:lo] == 0x5A5A5A5A) and np.all(gotw[hi:] == 0x5A5A5A5A), \
        "unpack wrote outside its output"
    assert np.array_equal(gotw[lo:hi], exp_back.view(np.uint32)), "unpacked words differ"
    # what is unique: the closed form the oracle is pinned to
    u = w.view(np.uint32)
    for l in range(len(rb)):
        seg = slice(int(off[l]), int(off[l + 1]))
        assert np.array_equal(gotw[lo:hi][seg], u[seg] & np.uint32(MASK[int(rb[l])]))


def check_pack_unpack_fused(adt, w, off, rb, w_shift=0, p_shift=0):
    """adt_pack_unpack with guard bytes and misaligned bases against the oracle."""
    n = int(off[-1])
    exp_stream = oracle.pack(w, off, rb)
    exp_back = oracle.unpack(exp_stream, off, rb)
    size, guard = exp_stream.size, 64
    wbuf = torch.zeros(n + w_shift + 8, dtype=torch.float32, device="cuda")
    wview = wbuf[w_shift:w_shift + n]
    wview.copy_(torch.from_numpy(w))
    pbuf = torch.full((size + p_shift + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
    obuf = torch.zeros(n + w_shift + 2 * guard, dtype=torch.float32, device="cuda")
    obuf.view(torch.int32).fill_(0x5A5A5A5A)
    adt.adt_pack_unpack(wview, off, rb, out=pbuf[guard + p_shift:guard + p_shift + size],
                        weights_out=obuf[guard + w_shift:guard + w_shift + n])
    got = pbuf.cpu().numpy()
    lo, hi = guard + p_shift, guard + p_shift + size
    assert np.all(got[:lo] == 0xA5) and np.all(got[hi:] == 0xA5)
    assert np.array_equal(got[lo:hi], exp_stream)
    gotw = obuf.view(torch.int32).cpu().numpy().view(np.uint32)
    lo, hi = guard + w_shift, guard + w_shift + n
    assert np.all(gotw[:lo] == 0x5A5A5A5A) and np.all(gotw[hi:] == 0x5A5A5A5A)
    assert np.array_equal(gotw[lo:hi], exp_back.view(np.uint32))


def check_stats(adt, w, off, rtol=STATS_RTOL):
    exp = oracle.stats(w, off)
    got = adt.awp_layer_stats(dev(w), off).cpu().numpy()
    assert got.shape == exp.shape
    assert STATS_RTOL <= STATS_RTOL_BAR
    nan = np.isnan(exp)
    assert np.array_equal(np.isnan(got), nan)
    np.testing.assert_allclose(got[~nan], exp[~nan], rtol=rtol, atol=0.0)
    np.testing.assert_array_equal(got[:, 2][~nan[:, 2]], exp[:, 2][~nan[:, 2]])   # absmax exact
    return got


# ------------------------------------------------------------------ configs
def test_tiny_config(adt):
    ws = workloads.make_weight_set("tiny")
    rb = workloads.config_bytes("tiny")
    assert adt.adt_packed_size(ws.layer_offsets, rb) == 35168
    check_pack_unpack(adt, ws.weights, ws.layer_offsets, rb)
    check_stats(adt, ws.weights, ws.layer_offsets)


@pytest.mark.parametrize("name,variant", [
    ("alexnet", "default"), ("resnet50", "default"),
    ("vgg16", "all2"), ("vgg16", "all3"), ("vgg16", "mixed"),
    ("paper_alexnet", "default"), ("paper_vgga", "default"), ("paper_resnet34", "default"),
])
def test_full_size_configs(adt, name, variant):
    ws = workloads.make_weight_set(name)
    rb = workloads.config_bytes(name, variant)
    off, w = ws.layer_offsets, ws.weights
    exp_stream = oracle.pack(w, off, rb)
    dw = dev(w)
    packed = adt.adt_pack(dw, off, rb)
    assert packed.numel() == exp_stream.size
    assert np.array_equal(packed.cpu().numpy(), exp_stream)
    back = adt.adt_unpack(packed, off, rb)
    exp_back = oracle.unpack(exp_stream, off, rb)
    assert np.array_equal(back.view(torch.int32).cpu().numpy(), exp_back.view(np.int32))
    # pack and truncate in one kernel: same stream, same words
    packed2, back2 = adt.adt_pack_unpack(dw, off, rb)
    assert torch.equal(packed2, packed)
    assert torch.equal(back2.view(torch.int32), back.view(torch.int32))
    del packed, back, packed2, back2
    if variant in ("default", "all2"):
        check_stats(adt, w, off)


def test_alexnet_hundred_passes_stay_identical(adt):
    ws = workloads.make_weight_set("alexnet")
    rb = workloads.config_bytes("alexnet")
    off = ws.layer_offsets
    dw = dev(ws.weights)
    first_p = adt.adt_pack(dw, off, rb)
    first_w = adt.adt_unpack(first_p, off, rb)
    p = torch.empty_like(first_p)
    w2 = torch.empty_like(first_w)
    for _ in range(100):
        adt.adt_pack(dw, off, rb, out=p)
        adt.adt_unpack(p, off, rb, out=w2)
    assert torch.equal(p, first_p)
    assert torch.equal(w2.view(torch.int32), first_w.view(torch.int32))
    assert np.array_equal(first_p.cpu().numpy(), oracle.pack(ws.weights, off, rb))


# ------------------------------------------------------------------ ragged / edge cases
@pytest.mark.parametrize("w_shift,p_shift", [(0, 0), (1, 0), (0, 1), (3, 7), (2, 13), (1, 15)])
def test_alignment_sweep(adt, w_shift, p_shift):
    off, rb, w = workloads.alignment_sweep_case()
    check_pack_unpack(adt, w, off, rb, w_shift, p_shift)
    check_pack_unpack_fused(adt, w, off, rb, w_shift, p_shift)


@pytest.mark.parametrize("r", [1, 2, 3, 4])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 63, 64, 65, 1023, 1024, 1025, 4095, 4096, 4097,
                               8192 + 17, 3 * 4096])
def test_single_layer_sizes(adt, n, r):
    off, rb, w = workloads.ragged_case([n], [r], seed=100 + n)
    for p_shift in (0, 5):
        check_pack_unpack(adt, w, off, rb, 0, p_shift)


def test_special_values(adt):
    w = np.tile(workloads.special_values(), 40)
    for r in (1, 2, 3, 4):
        off, rb, _ = workloads.ragged_case([w.size], [r], seed=0)
        check_pack_unpack(adt, w, off, rb)


def test_empty_inputs(adt):
    z = torch.zeros(0, dtype=torch.float32, device="cuda")
    off = np.array([0], dtype=np.int64)
    assert adt.adt_pack(z, off, np.zeros(0, np.uint8)).numel() == 0
    off = np.array([0, 0, 0], dtype=np.int64)
    rb = np.array([1, 3], dtype=np.uint8)
    p = adt.adt_pack(z, off, rb)
    assert p.numel() == 0
    assert adt.adt_unpack(p, off, rb).numel() == 0
    st = adt.awp_layer_stats(z, off).cpu().numpy()
    assert st.tolist() == [[0.0, 0.0, 0.0], [0.0, 0.0, 0.0]]


def test_many_layers_use_the_device_table(adt):
    rng = np.random.default_rng(77)
    sizes = rng.integers(0, 9000, size=300)
    sizes[::17] = 0
    rb = rng.integers(1, 5, size=300).astype(np.uint8)
    off, rb, w = workloads.ragged_case(sizes, rb, seed=78)
    for _ in range(6):     # more calls than ring slots
        check_pack_unpack(adt, w, off, rb, 1, 3)
    check_pack_unpack_fused(adt, w, off, rb, 1, 3)
    off2, _, w2 = workloads.ragged_case(sizes, rb, seed=79, he=True)
    for _ in range(6):
        check_stats(adt, w2, off2)


def test_back_to_back_calls_with_different_large_tables(adt):
    """Twelve pack / unpack / statistics calls with twelve different tables of more
    than 128 layers, queued without waiting for the GPU in between: a table handed
    to a launch must stay intact until that launch has read it, however quickly the
    following calls come."""
    cases = []
    for k in range(12):
        rng = np.random.default_rng(900 + k)
        L = int(rng.integers(130, 400))
        sizes = rng.integers(0, 6000, size=L)
        rb = rng.integers(1, 5, size=L).astype(np.uint8)
        off, rb, w = workloads.ragged_case(sizes, rb, seed=950 + k, he=True)
        n, size = int(off[-1]), oracle.packed_size(off, rb)
        cases.append(dict(off=off, rb=rb, w=w, dw=dev(w), n=n, size=size,
                          p=torch.zeros(size, dtype=torch.uint8, device="cuda"),
                          back=torch.zeros(n, dtype=torch.float32, device="cuda"),
                          st=torch.zeros((len(rb), 3), dtype=torch.float64, device="cuda")))
    torch.cuda.synchronize()
    for c in cases:                       # nothing here waits for the GPU
        adt.awp_layer_stats(c["dw"], c["off"], out=c["st"])
        adt.adt_pack(c["dw"], c["off"], c["rb"], out=c["p"])
        adt.adt_unpack(c["p"], c["off"], c["rb"], out=c["back"])
    torch.cuda.synchronize()
    for k, c in enumerate(cases):
        exp = oracle.pack(c["w"], c["off"], c["rb"])
        assert np.array_equal(c["p"].cpu().numpy(), exp), k
        assert np.array_equal(c["back"].view(torch.int32).cpu().numpy(),
                              oracle.unpack(exp, c["off"], c["rb"]).view(np.int32)), k
        est = oracle.stats(c["w"], c["off"])
        got = c["st"].cpu().numpy()
        np.testing.assert_allclose(got, est, rtol=STATS_RTOL, atol=0.0)
        np.testing.assert_array_equal(got[:, 2], est[:, 2])


# ------------------------------------------------------------------ exhaustive bit patterns
def test_all_bit_patterns_on_gpu(adt):
    """Every 32-bit word, every byte count: unpack(pack(w)) equals the mask
    closed form (checked on the device), and one slice is compared with the
    oracle element by element."""
    chunk = 1 << 28
    off = np.array([0, chunk], dtype=np.int64)
    for r in (1, 2, 3, 4):
        rb = np.array([r], dtype=np.uint8)
        mask = MASK[r] - (1 << 32)            # as a signed 32-bit value
        p = torch.empty(chunk * r, dtype=torch.uint8, device="cuda")
        back = torch.empty(chunk, dtype=torch.float32, device="cuda")
        for c in range(16):
            words = torch.arange(c * chunk - (1 << 31), (c + 1) * chunk - (1 << 31),
                                 dtype=torch.int64, device="cuda").to(torch.int32)
            adt.adt_pack(words.view(torch.float32), off, rb, out=p)
            adt.adt_unpack(p, off, rb, out=back)
            assert torch.equal(back.view(torch.int32), words & mask), (r, c)
            if c == 5:
                n = 1 << 22
                hw = words[:n].cpu().numpy().view(np.float32)
                o1 = np.array([0, n], dtype=np.int64)
                assert np.array_equal(p[:n * r].cpu().numpy(), oracle.pack(hw, o1, rb))
            del words


# ------------------------------------------------------------------ statistics
def test_stats_ragged_and_special(adt):
    sizes = [0, 1, 2, 3, 5, 255, 256, 257, 16383, 16384, 16385, 0, 40000, 7]
    off, _, w = workloads.ragged_case(sizes, [1] * len(sizes), seed=5, he=True)
    check_stats(adt, w, off)
    w2 = w.copy()
    w2[int(off[4])] = np.nan          # layer 4 gets a NaN
    w2[int(off[8]) + 9] = np.inf      # layer 8 an infinity
    w2[int(off[12]) + 123] = -3e38    # layer 12 a huge value (no float32 overflow allowed)
    got = check_stats(adt, w2, off)
    assert np.isnan(got[4]).all() and got[8, 1] == np.inf and np.isfinite(got[12]).all()


def test_stats_misaligned_base_and_determinism(adt):
    ws = workloads.make_weight_set("resnet50")
    off = ws.layer_offsets
    buf = torch.zeros(ws.n_weights + 4, dtype=torch.float32, device="cuda")
    exp = oracle.stats(ws.weights, off)
    outs = []
    for shift in (0, 1, 3):
        v = buf[shift:shift + ws.n_weights]
        v.copy_(torch.from_numpy(ws.weights))
        outs.append(adt.awp_layer_stats(v, off).cpu().numpy())
        np.testing.assert_allclose(outs[-1], exp, rtol=STATS_RTOL)
    again = adt.awp_layer_stats(buf[3:3 + ws.n_weights], off).cpu().numpy()
    assert again.tobytes() == outs[-1].tobytes()       # run-to-run identical
    assert outs[0].tobytes() == outs[1].tobytes()      # independent of base alignment


@pytest.mark.parametrize("kernel", ["pack_kernel", "pack_unpack_kernel"])
@pytest.mark.parametrize("waves,extra_lds", [(1, 0), (1, 9216), (4, 20480)])
def test_launch_shapes_of_pack_give_the_same_bytes(adt, kernel, waves, extra_lds):
    off, rb, w = workloads.alignment_sweep_case()
    sizes = [1, 1023, 1024, 1025, 4095, 4096, 4097, 0, 20000, 3]
    off2, rb2, w2 = workloads.ragged_case(sizes, [1, 2, 3, 4, 3, 2, 1, 4, 3, 2], seed=61)
    try:
        adt.adt_launch_shape(kernel, waves, extra_lds)
        for o, r, x in ((off, rb, w), (off2, rb2, w2)):
            check_pack_unpack(adt, x, o, r, 1, 5)
            check_pack_unpack_fused(adt, x, o, r, 3, 11)
    finally:
        adt.adt_launch_shape(kernel, 0)
    with pytest.raises(adt.AdtError):
        adt.adt_launch_shape("pack_kernel", 2)
    with pytest.raises(adt.AdtError):
        adt.adt_launch_shape("unpack_kernel", 4)
    with pytest.raises(adt.AdtError):
        adt.adt_launch_shape("stats_final_kernel", 4)


@pytest.mark.parametrize("kernel", ["pack_kernel", "pack_unpack_kernel"])
def test_stream_store_kind_does_not_change_the_bytes(adt, kernel):
    """Ordinary and nontemporal stream stores (chosen by the stream's size against a
    limit) write the same bytes, aligned or not."""
    off, rb, w = workloads.alignment_sweep_case()
    old = adt.adt_stream_cache_limit(kernel)
    try:
        for limit in (0, 1 << 60):
            adt.adt_stream_cache_limit(kernel, limit)
            check_pack_unpack(adt, w, off, rb, 0, 0)
            check_pack_unpack(adt, w, off, rb, 1, 9)
            check_pack_unpack_fused(adt, w, off, rb, 0, 0)
            check_pack_unpack_fused(adt, w, off, rb, 2, 5)
    finally:
        adt.adt_stream_cache_limit(kernel, old)
    with pytest.raises(adt.AdtError):
        adt.adt_stream_cache_limit("unpack_kernel", 0)


# ------------------------------------------------------------------ streams
def test_statistics_calls_on_two_streams_share_the_scratch_safely(adt):
    """awp_layer_stats keeps one scratch buffer per device; calls on different
    streams are ordered against each other by the library."""
    a = workloads.make_weight_set("alexnet")
    b = workloads.make_weight_set("resnet50")
    da, db = dev(a.weights), dev(b.weights)
    ea, eb = oracle.stats(a.weights, a.layer_offsets), oracle.stats(b.weights, b.layer_offsets)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    outs = []
    for _ in range(6):
        with torch.cuda.stream(s1):
            outs.append((adt.awp_layer_stats(da, a.layer_offsets), ea))
        with torch.cuda.stream(s2):
            outs.append((adt.awp_layer_stats(db, b.layer_offsets), eb))
    torch.cuda.synchronize()
    for got, exp in outs:
        np.testing.assert_allclose(got.cpu().numpy(), exp, rtol=STATS_RTOL, atol=0.0)



def test_non_default_stream(adt):
    ws = workloads.make_weight_set("tiny")
    rb = workloads.config_bytes("tiny")
    dw = dev(ws.weights)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        p = adt.adt_pack(dw, ws.layer_offsets, rb)
        b = adt.adt_unpack(p, ws.layer_offsets, rb)
        st = adt.awp_layer_stats(dw, ws.layer_offsets)
    s.synchronize()
    exp = oracle.pack(ws.weights, ws.layer_offsets, rb)
    assert np.array_equal(p.cpu().numpy(), exp)
    assert np.array_equal(b.view(torch.int32).cpu().numpy(),
                          oracle.unpack(exp, ws.layer_offsets, rb).view(np.int32))
    np.testing.assert_allclose(st.cpu().numpy(), oracle.stats(ws.weights, ws.layer_offsets),
                               rtol=STATS_RTOL)


# ------------------------------------------------------------------ ablation variants
@pytest.mark.parametrize("variant", ["naive", "vec_direct", "per_layer"])
def test_ablation_variants_give_the_same_bytes(adt, variant):
    v = {"naive": adt.ABLATION_NAIVE, "vec_direct": adt.ABLATION_VEC_DIRECT,
         "per_layer": adt.ABLATION_PER_LAYER}[variant]
    if variant == "vec_direct":       # needs 4-byte aligned layer starts
        sizes = [16, 4096, 4100, 8, 0, 20000, 12, 1028, 4]
        off, rb, w = workloads.ragged_case(sizes, [1, 2, 3, 4, 1, 3, 1, 2, 3], seed=31)
        w = np.concatenate([w, np.zeros(3, np.float32)])
        off = off.copy(); off[-1] += 3                 # ragged tail inside the last layer
    elif variant == "naive":          # at most 128 layers
        sizes = [1, 0, 2, 3, 5, 15, 17, 255, 256, 257, 4095, 4097, 1023, 7, 9000, 31, 33, 1, 1, 12289]
        off, rb, w = workloads.ragged_case(sizes, [1, 3, 1, 3, 2, 4, 1, 2, 3, 4] * 2, seed=32)
    else:
        off, rb, w = workloads.alignment_sweep_case()
    exp = oracle.pack(w, off, rb)
    dw = dev(w)
    p = torch.full((exp.size + 32,), 0xA5, dtype=torch.uint8, device="cuda")
    adt.adt_ablation(v, False, dw, off, rb, p[:exp.size] if exp.size else p)
    got = p.cpu().numpy()
    assert np.array_equal(got[:exp.size], exp) and np.all(got[exp.size:] == 0xA5)
    if variant != "vec_direct":
        back = torch.zeros_like(dw)
        adt.adt_ablation(v, True, back, off, rb, p)
        assert np.array_equal(back.view(torch.int32).cpu().numpy(),
                              oracle.unpack(exp, off, rb).view(np.int32))


# ------------------------------------------------------------------ 16-bit unpack
@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
@pytest.mark.parametrize("elem_shift,p_shift", [(0, 0), (1, 3), (4, 16), (8, 5)])
def test_unpack16_ragged(adt, fmt, elem_shift, p_shift):
    off, rb, w = workloads.alignment_sweep_case()
    w = w.copy()
    w[::7] = workloads.he_normal_weights([(1, 50, 1, 1)], seed=3)[0]     # some ordinary values too
    stream = oracle.pack(w, off, rb)
    exp = oracle.unpack16(stream, off, rb, fmt)
    n, guard = int(off[-1]), 32
    pbuf = torch.zeros(stream.size + p_shift + 16, dtype=torch.uint8, device="cuda")
    pview = pbuf[p_shift:p_shift + stream.size]
    pview.copy_(torch.from_numpy(stream))
    dtype = torch.bfloat16 if fmt == "bf16" else torch.float16
    obuf = torch.zeros(n + elem_shift + 2 * guard, dtype=dtype, device="cuda")
    obuf.view(torch.int16).fill_(0x5A5A)
    adt.adt_unpack16(pview, off, rb, fmt, out=obuf[guard + elem_shift:guard + elem_shift + n])
    got = obuf.view(torch.int16).cpu().numpy().view(np.uint16)
    lo, hi = guard + elem_shift, guard + elem_shift + n
    assert np.all(got[:lo] == 0x5A5A) and np.all(got[hi:] == 0x5A5A)
    got = got[lo:hi]
    assert np.array_equal(got, exp)                 # NaNs included: both sides give 0x7E00 | sign


@pytest.mark.parametrize("fmt", ["bf16", "fp16"])
def test_unpack16_full_size(adt, fmt):
    ws = workloads.make_weight_set("alexnet")
    rb = workloads.config_bytes("alexnet")
    stream = oracle.pack(ws.weights, ws.layer_offsets, rb)
    got = adt.adt_unpack16(dev(stream), ws.layer_offsets, rb, fmt)
    assert np.array_equal(got.view(torch.int16).cpu().numpy().view(np.uint16),
                          oracle.unpack16(stream, ws.layer_offsets, rb, fmt))


# ------------------------------------------------------------------ beyond 4 GiB
def test_offsets_beyond_four_gib(adt):
    """Element and byte offsets that do not fit 32 bits: 1.2 G weights (4.8 GB of
    FP32) in three layers; the stream of the middle layer starts beyond 2^32
    bytes.  Checked against the mask closed form on the device for every
    weight, and against the oracle on slices around each layer boundary."""
    sizes = [(1 << 30) + 4097, 3, (1 << 27) + 11]
    rb = np.array([4, 1, 3], dtype=np.uint8)
    off = workloads.offsets_from_sizes(sizes)
    N = int(off[-1])
    g = torch.Generator(device="cuda")
    g.manual_seed(123)
    w = torch.randint(-(1 << 31), (1 << 31) - 1, (N,), generator=g, device="cuda",
                      dtype=torch.int64).to(torch.int32)
    wf = w.view(torch.float32)
    size = adt.adt_packed_size(off, rb)
    assert size > (1 << 32)
    packed = adt.adt_pack(wf, off, rb)
    back = adt.adt_unpack(packed, off, rb)
    fused_p, fused_w = adt.adt_pack_unpack(wf, off, rb)
    assert torch.equal(fused_p, packed)
    pos = 0
    for l, n in enumerate(sizes):
        r = int(rb[l])
        mask = MASK[r] - (1 << 32)
        seg = slice(int(off[l]), int(off[l + 1]))
        assert torch.equal(back[seg].view(torch.int32), w[seg] & mask), l
        assert torch.equal(fused_w[seg].view(torch.int32), w[seg] & mask), l
        # oracle on the first and last 5000 weights of the layer
        for a, b in ((0, min(n, 5000)), (max(0, n - 5000), n)):
            hw = w[seg][a:b].cpu().numpy().view(np.float32)
            o1 = np.array([0, b - a], dtype=np.int64)
            exp = oracle.pack(hw, o1, rb[l:l + 1])
            got = packed[pos + a * r:pos + b * r].cpu().numpy()
            assert np.array_equal(got, exp), (l, a, b)
        pos += n * r
    assert pos == size
    del packed, back, fused_p, fused_w
    # statistics over the same layers (values as floats may be NaN/Inf: use finite data)
    w.copy_((torch.randn(N, generator=g, device="cuda") * 0.01).view(torch.int32))
    st = adt.awp_layer_stats(wf, off).cpu().numpy()
    for l in range(3):
        seg = wf[int(off[l]):int(off[l + 1])].double()
        ref = float(torch.sum(seg * seg))
        assert st[l, 0] == pytest.approx(ref, rel=1e-10)
        assert st[l, 2] == float(seg.abs().max())


# ------------------------------------------------------------------ seeded random tables
@pytest.mark.parametrize("seed", range(12))
def test_random_layer_tables(adt, seed):
    """Random numbers of layers, sizes (skewed towards tile boundaries), byte
    counts and base misalignments; every entry point against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    L = int(rng.integers(1, 40))
    kinds = rng.integers(0, 5, size=L)
    sizes = np.where(kinds == 0, rng.integers(0, 8, size=L),
             np.where(kinds == 1, 1024 * rng.integers(1, 9, size=L) + rng.integers(-2, 3, size=L),
             np.where(kinds == 2, 4096 * rng.integers(1, 5, size=L) + rng.integers(-2, 3, size=L),
             np.where(kinds == 3, rng.integers(1, 30000, size=L), 8192 + rng.integers(-1, 2, size=L)))))
    sizes = np.maximum(sizes, 0)
    rbytes = rng.integers(1, 5, size=L).astype(np.uint8)
    off, rb, w = workloads.ragged_case(sizes, rbytes, seed=2000 + seed)
    w_shift, p_shift = int(rng.integers(0, 4)), int(rng.integers(0, 16))
    check_pack_unpack(adt, w, off, rb, w_shift, p_shift)
    check_pack_unpack_fused(adt, w, off, rb, w_shift, p_shift)
    if int(off[-1]):
        stream = oracle.pack(w, off, rb)
        for fmt in ("bf16", "fp16"):
            got = adt.adt_unpack16(dev(stream), off, rb, fmt)
            got = got.view(torch.int16).cpu().numpy().view(np.uint16)
            exp = oracle.unpack16(stream, off, rb, fmt)
            assert np.array_equal(got, exp), fmt
    _, _, wn = workloads.ragged_case(sizes, rbytes, seed=3000 + seed, he=True)
    check_stats(adt, wn, off)
