"""Plan path (awp_adt_step) against the oracle and against the three-call path.

The plan runs statistics, the AWP rule, pack and unpack of one batch without a
host round trip and speculates on unchanged byte counts; whatever the rule
decides, its outputs must equal the sequential definition: this batch's norms
choose this batch's byte counts.  Parameters here make byte counts change often
so that the redo path runs many times.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def adt():
    import paper_2004_02297_amd as m
    m.load_library()
    return m


def run_trajectory(adt, sizes, steps, T, interval, n_bits, init_bits, seed, w_shift=0,
                   p_shift=0, truncated=True, groups=None, out_dtype=torch.float32):
    rng = np.random.default_rng(seed)
    off = workloads.offsets_from_sizes(sizes)
    L, N = len(sizes), int(off[-1])
    hw = (rng.standard_normal(N).astype(np.float32) * np.float32(0.05))
    wbuf = torch.zeros(N + w_shift + 4, dtype=torch.float32, device="cuda")
    w = wbuf[w_shift:w_shift + N]
    pbuf = torch.full((4 * N + p_shift + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    packed = pbuf[p_shift:p_shift + 4 * N]
    obuf = torch.zeros(N + w_shift + 4, dtype=out_dtype, device="cuda")
    out = obuf[w_shift:w_shift + N] if truncated else None

    grp = np.arange(L + 1, dtype=np.int32) if groups is None else np.asarray(groups, np.int32)
    G = grp.size - 1
    ib = None if init_bits is None else np.full(G, init_bits, np.int32)
    plan = adt.AwpPlan(off, T, interval, n_bits, init_bits=ib, group_offsets=groups)
    ost = oracle.AwpState(G, 8 if init_bits is None else init_bits)
    n_changes = 0
    prev = None
    for step in range(steps):
        if step:
            scale = 1.0 + rng.choice([-0.05, -0.01, 0.0, 0.01, 0.05], size=L)
            for l in range(L):
                hw[off[l]:off[l + 1]] *= np.float32(scale[l])
            hw += rng.standard_normal(N).astype(np.float32) * np.float32(1e-4)
        w.copy_(torch.from_numpy(hw))
        plan.step(w, packed, out)
        got = plan.read()

        o_stats = oracle.stats(hw, off)
        np.testing.assert_allclose(got["stats"], o_stats, rtol=1e-10, atol=0.0)
        np.testing.assert_array_equal(got["stats"][:, 2], o_stats[:, 2])
        if groups is None:
            orb = oracle.awp_update(ost, o_stats[:, 1], T, interval, n_bits)
        else:
            gb = oracle.awp_update(ost, oracle.group_norms(hw, off, grp), T, interval, n_bits)
            orb = np.repeat(gb, np.diff(grp)).astype(np.uint8)
            # the three-call route through the host helpers agrees as well
            hb = adt.awp_expand_group_bytes(gb, grp)
            assert np.array_equal(hb, orb)
            np.testing.assert_allclose(adt.awp_group_norms(got["stats"], grp),
                                       oracle.group_norms(hw, off, grp), rtol=1e-10)
        assert np.array_equal(got["bytes"], orb), f"step {step}"
        assert np.array_equal(got["bits"], ost.bits) and np.array_equal(got["counter"], ost.counter)
        exp_stream = oracle.pack(hw, off, orb)
        assert got["packed_size"] == exp_stream.size
        hp = pbuf.cpu().numpy()
        assert np.array_equal(hp[p_shift:p_shift + exp_stream.size], exp_stream), f"step {step}"
        assert np.all(hp[:p_shift] == 0xA5) and np.all(hp[p_shift + 4 * N:] == 0xA5)
        if truncated and out_dtype == torch.float32:
            exp_w = oracle.unpack(exp_stream, off, orb)
            assert np.array_equal(out.view(torch.int32).cpu().numpy(), exp_w.view(np.int32)), \
                f"step {step}"
        elif truncated:
            fmt = "bf16" if out_dtype == torch.bfloat16 else "fp16"
            exp16 = oracle.unpack16(exp_stream, off, orb, fmt)
            assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16), exp16), \
                f"step {step}"
        # the three-call path gives the same stream
        p3 = adt.adt_pack(w, off, orb)
        assert torch.equal(p3, packed[:exp_stream.size])
        if prev is not None and not np.array_equal(prev, orb):
            n_changes += 1
        prev = orb
    plan.close()
    return n_changes


def test_plan_matches_oracle_with_frequent_changes(adt):
    sizes = [1, 0, 5, 4095, 4096, 4097, 17, 12289, 1023, 30000, 3, 8192]
    n = run_trajectory(adt, sizes, steps=24, T=0.0, interval=2, n_bits=8, init_bits=None, seed=1)
    assert n >= 5      # the redo path really ran


def test_plan_misaligned_buffers_and_odd_bit_steps(adt):
    sizes = [7, 4097, 1, 2049, 0, 10001, 333]
    n = run_trajectory(adt, sizes, steps=16, T=0.02, interval=1, n_bits=3, init_bits=5, seed=2,
                       w_shift=1, p_shift=5)
    assert n >= 4


def test_plan_without_truncated_copy(adt):
    n = run_trajectory(adt, [5000, 64, 4096], steps=8, T=0.0, interval=1, n_bits=8,
                       init_bits=None, seed=3, truncated=False)
    assert n >= 1


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float16])
def test_plan_with_16_bit_truncated_weights(adt, out_dtype):
    sizes = [5, 4097, 1, 2049, 0, 10001, 333, 8192]
    n = run_trajectory(adt, sizes, steps=12, T=0.0, interval=1, n_bits=8, init_bits=None,
                       seed=7, w_shift=1, p_shift=3, out_dtype=out_dtype)
    assert n >= 2


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("shift", [0, 1, 2, 4, 8])
def test_plan_16_bit_output_on_and_off_the_16_byte_grid(adt, out_dtype, shift):
    """A full wave tile of 16-bit words that starts on the 16-byte grid is stored
    16 bytes per lane (neighbouring lanes trade halves of two chunks), any other
    tile 8 bytes or less per lane.  Layer sizes that are multiples of 8 put every
    tile on the grid at shifts 0 and 8 and off it at 1, 2 and 4; every byte count
    and the special values (NaNs, infinities, subnormals) take both routes."""
    sizes = [8192, 1024, 6144, 8, 3072, 1000, 2048, 4096 + 16, 5120]
    off = workloads.offsets_from_sizes(sizes)
    L, N = len(sizes), int(off[-1])
    rb = (np.arange(L) % 4 + 1).astype(np.uint8)
    hw = workloads.random_bit_patterns(N, seed=77 + shift)
    sp = workloads.special_values()
    for l in range(L):                          # special values at the head and inside each layer
        n = min(sp.size, sizes[l])
        hw[off[l]:off[l] + n] = sp[:n]
        if sizes[l] > 1024 + sp.size:
            hw[off[l] + 1024:off[l] + 1024 + sp.size] = sp
    w = torch.from_numpy(hw).cuda()
    packed = torch.empty(4 * N, dtype=torch.uint8, device="cuda")
    guard = 64
    obuf = torch.zeros(N + shift + 2 * guard, dtype=out_dtype, device="cuda")
    obuf.view(torch.int16).fill_(0x5A5A)
    out = obuf[guard + shift:guard + shift + N]
    plan = adt.AwpPlan(off, -1.0, 1000, 8, init_bits=rb.astype(np.int32) * 8)
    plan.step(w, packed, out)
    got = plan.read()
    assert np.array_equal(got["bytes"], rb)
    exp = oracle.pack(hw, off, rb)
    assert np.array_equal(packed[:exp.size].cpu().numpy(), exp)
    fmt = "bf16" if out_dtype == torch.bfloat16 else "fp16"
    all16 = obuf.view(torch.int16).cpu().numpy().view(np.uint16)
    lo, hi = guard + shift, guard + shift + N
    assert np.all(all16[:lo] == 0x5A5A) and np.all(all16[hi:] == 0x5A5A)
    assert np.array_equal(all16[lo:hi], oracle.unpack16(exp, off, rb, fmt))
    # the separate 16-bit unpack takes the same two routes
    obuf.view(torch.int16).fill_(0x5A5A)
    adt.adt_unpack16(packed[:exp.size], off, rb, fmt, out=out)
    all16 = obuf.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.all(all16[:lo] == 0x5A5A) and np.all(all16[hi:] == 0x5A5A)
    assert np.array_equal(all16[lo:hi], oracle.unpack16(exp, off, rb, fmt))
    plan.close()


def test_plan_many_layers(adt):
    rng = np.random.default_rng(9)
    sizes = rng.integers(0, 3000, size=2500).tolist()     # rule kernel loops over 1024-layer chunks
    n = run_trajectory(adt, sizes, steps=6, T=0.0, interval=1, n_bits=8, init_bits=None, seed=4)
    assert n >= 1


def test_plan_with_layer_groups(adt):
    # groups of uneven length, an empty group and single-layer groups
    sizes = [300, 4096, 5000, 1, 7000, 64, 8192, 33, 2, 9000, 12]
    groups = [0, 1, 3, 3, 6, 7, 10, 11]
    n = run_trajectory(adt, sizes, steps=20, T=0.0, interval=2, n_bits=8, init_bits=None,
                       seed=5, groups=groups)
    assert n >= 4


def test_plan_resnet34_block_groups_full_size(adt):
    ws = workloads.make_weight_set("paper_resnet34")
    off, N, L = ws.layer_offsets, ws.n_weights, ws.n_layers
    grp = workloads.paper_resnet34_group_offsets()
    w = torch.from_numpy(ws.weights).cuda()
    packed = torch.empty(4 * N, dtype=torch.uint8, device="cuda")
    out = torch.empty_like(w)
    start = (np.arange(grp.size - 1) % 4 + 1).astype(np.int32) * 8     # 1,2,3,4 bytes per block
    plan = adt.AwpPlan(off, -2e-5, 2000, 8, init_bits=start, group_offsets=grp)
    plan.step(w, packed, out)
    plan.step(w, packed, out)
    got = plan.read()
    rb = np.repeat((start // 8).astype(np.uint8), np.diff(grp))
    assert np.array_equal(got["bytes"], rb) and np.array_equal(got["bits"], start)
    exp = oracle.pack(ws.weights, off, rb)
    assert got["packed_size"] == exp.size
    assert np.array_equal(packed[:exp.size].cpu().numpy(), exp)
    assert np.array_equal(out.view(torch.int32).cpu().numpy(),
                          oracle.unpack(exp, off, rb).view(np.int32))
    plan.close()


@pytest.mark.parametrize("variant,out_dtype", [
    ("all2", torch.float32), ("all3", torch.float32), ("all4", torch.float32),
    ("mixed", torch.float32), ("all3", torch.bfloat16), ("mixed", torch.float16),
    ("all2", None), ("mixed", None), ("all4", None),
])
def test_plan_full_size_vgg16(adt, variant, out_dtype):
    """The whole pass on the VGG-16-shaped set at every byte assignment the
    measurements use, with the default (nontemporal) stream stores; out_dtype None:
    statistics, rule and stream only, no truncated copy (the side that sends)."""
    ws = workloads.make_weight_set("vgg16")
    off, N, L = ws.layer_offsets, ws.n_weights, ws.n_layers
    rb = workloads.config_bytes("vgg16", variant)
    size = oracle.packed_size(off, rb)
    w = torch.from_numpy(ws.weights).cuda()
    packed = torch.empty(4 * N, dtype=torch.uint8, device="cuda")
    out = None if out_dtype is None else torch.empty(N, dtype=out_dtype, device="cuda")
    plan = adt.AwpPlan(off, -2e-3, 4000, 8, init_bits=rb.astype(np.int32) * 8)
    for _ in range(3):
        plan.step(w, packed, out)
    got = plan.read()
    assert np.array_equal(got["bytes"], rb)
    np.testing.assert_allclose(got["stats"], oracle.stats(ws.weights, off), rtol=1e-10)
    exp = oracle.pack(ws.weights, off, rb)
    assert got["packed_size"] == exp.size == size
    assert np.array_equal(packed[:exp.size].cpu().numpy(), exp)
    if out_dtype is None:
        pass
    elif out_dtype == torch.float32:
        assert np.array_equal(out.view(torch.int32).cpu().numpy(),
                              oracle.unpack(exp, off, rb).view(np.int32))
    else:
        fmt = "bf16" if out_dtype == torch.bfloat16 else "fp16"
        assert np.array_equal(out.view(torch.int16).cpu().numpy().view(np.uint16),
                              oracle.unpack16(exp, off, rb, fmt))
    plan.close()


def test_plan_full_size_stream_crosses_the_cache_limit_inside_a_redo(adt):
    """VGG-16-shaped weights whose norms shrink every batch, so that with T = 0 and
    INTERVAL = 1 every layer gains a byte per batch: 1 -> 2 -> 3 -> 4 bytes.  The
    stream grows from 132 MiB to 528 MiB.  With the limit of the cache-friendly
    stream stores set to 280 MiB, the batch that takes the stream from 264 to
    396 MiB crosses it inside the redo pass (the speculative pass of that batch
    still ran below the limit)."""
    ws = workloads.make_weight_set("vgg16")
    off, N, L = ws.layer_offsets, ws.n_weights, ws.n_layers
    limit = 280 << 20
    old = adt.adt_stream_cache_limit("fused_kernel", limit)
    try:
        hw = ws.weights.copy()
        w = torch.from_numpy(hw).cuda()
        packed = torch.empty(4 * N, dtype=torch.uint8, device="cuda")
        out = torch.empty_like(w)
        plan = adt.AwpPlan(off, 0.0, 1, 8)
        ost = oracle.AwpState(L, 8)
        sizes = []
        for step in range(5):
            if step:
                hw *= np.float32(0.99)
                w.copy_(torch.from_numpy(hw))
            plan.step(w, packed, out)
            got = plan.read()
            o_stats = oracle.stats(hw, off)
            orb = oracle.awp_update(ost, o_stats[:, 1], 0.0, 1, 8)
            assert np.array_equal(got["bytes"], orb), step
            exp = oracle.pack(hw, off, orb)
            assert got["packed_size"] == exp.size
            assert np.array_equal(packed[:exp.size].cpu().numpy(), exp), step
            assert np.array_equal(out.view(torch.int32).cpu().numpy(),
                                  oracle.unpack(exp, off, orb).view(np.int32)), step
            sizes.append(exp.size)
    finally:
        adt.adt_stream_cache_limit("fused_kernel", old)
    assert sizes == [N, 2 * N, 3 * N, 4 * N, 4 * N]
    assert sizes[1] <= limit < sizes[2]
    plan.close()


def test_plan_cache_limit_flips_between_batches_small(adt):
    """The same flip on a small ragged set, with the limit lowered so that the
    stream crosses it back and forth: the bytes never depend on the store kind."""
    old = adt.adt_stream_cache_limit("fused_kernel")
    try:
        for limit in (0, 60000, 1 << 60):
            adt.adt_stream_cache_limit("fused_kernel", limit)
            n = run_trajectory(adt, [5000, 4097, 1, 12289, 0, 3000], steps=10, T=0.0, interval=1,
                               n_bits=8, init_bits=None, seed=11, w_shift=1, p_shift=7)
            assert n >= 3
    finally:
        adt.adt_stream_cache_limit("fused_kernel", old)


@pytest.mark.parametrize("waves,extra_lds", [(1, 0), (1, 12288), (4, 0), (4, 24576)])
def test_plan_launch_shapes_give_identical_results(adt, waves, extra_lds):
    """Every launch shape of the fused kernel (1 or 4 wavefronts per block, with or
    without an occupancy cap) gives the oracle's bytes and the default shape's
    statistics bit for bit."""
    sizes = [1, 0, 5, 4095, 4096, 4097, 17, 12289, 1023, 30000, 3, 8192, 1025, 2049, 3073]
    off = workloads.offsets_from_sizes(sizes)
    N = int(off[-1])
    hw = workloads.ragged_case(sizes, [1] * len(sizes), seed=77, he=True)[2]
    w = torch.from_numpy(hw).cuda()
    packed = torch.empty(4 * N, dtype=torch.uint8, device="cuda")
    out = torch.empty_like(w)
    ref = adt.AwpPlan(off, 0.0, 1, 8)
    ref.step(w, packed, out)
    want = ref.read()["stats"]
    ref.close()
    try:
        adt.adt_launch_shape("fused_kernel", waves, extra_lds)
        n = run_trajectory(adt, sizes, steps=8, T=0.0, interval=1, n_bits=8, init_bits=None,
                           seed=12, w_shift=1, p_shift=3)
        assert n >= 2
        plan = adt.AwpPlan(off, 0.0, 1, 8)
        plan.step(w, packed, out)
        assert plan.read()["stats"].tobytes() == want.tobytes()
        plan.close()
    finally:
        adt.adt_launch_shape("fused_kernel", 0)


def test_plan_more_layers_than_the_redo_table_holds(adt):
    """Beyond 1024 layers the stream offsets are rebuilt by a kernel of their own."""
    rng = np.random.default_rng(19)
    sizes = rng.integers(0, 400, size=5000).tolist()
    n = run_trajectory(adt, sizes, steps=5, T=0.0, interval=1, n_bits=8, init_bits=None, seed=14)
    assert n >= 1


def test_plan_with_only_empty_layers(adt):
    off = np.zeros(4, dtype=np.int64)
    plan = adt.AwpPlan(off, 0.0, 1, 8)
    z = torch.zeros(0, dtype=torch.float32, device="cuda")
    p = torch.zeros(0, dtype=torch.uint8, device="cuda")
    for _ in range(3):
        plan.step(z, p, None)
    got = plan.read()
    # zero norms: delta = 0, not below T = 0, nothing is ever counted
    assert got["bits"].tolist() == [8, 8, 8] and got["counter"].tolist() == [0, 0, 0]
    assert got["packed_size"] == 0 and got["stats"].tolist() == [[0.0] * 3] * 3
    assert plan.get_state()["batches_seen"] == 1
    plan.close()


def test_plan_argument_checks(adt):
    off = np.array([0, 100], dtype=np.int64)
    plan = adt.AwpPlan(off, 0.0, 1)
    w = torch.zeros(100, device="cuda")
    with pytest.raises(adt.AdtError):
        plan.step(w, torch.zeros(399, dtype=torch.uint8, device="cuda"))
    with pytest.raises(adt.AdtError):
        adt.AwpPlan(off, 0.0, 0)
    with pytest.raises(adt.AdtError):
        adt.AwpPlan(off, 0.0, 1, init_bits=np.array([33], np.int32))
    plan.close()


def test_plan_step_replayed_from_a_hip_graph(adt):
    """awp_adt_step allocates nothing and never waits for the GPU, so a whole
    pass can be captured once and replayed.  Every replay (with eager work and
    synchronisation in between) must equal an eager plan fed the same weights."""
    sizes = [5000, 4096, 77, 12289, 1, 9000]
    off = workloads.offsets_from_sizes(sizes)
    N, L = int(off[-1]), len(sizes)
    rng = np.random.default_rng(21)
    hw = rng.standard_normal(N).astype(np.float32) * np.float32(0.05)
    w = torch.from_numpy(hw).cuda()
    pe, pg = (torch.zeros(4 * N, dtype=torch.uint8, device="cuda") for _ in range(2))
    oe, og = (torch.zeros(N, dtype=torch.float32, device="cuda") for _ in range(2))
    eager = adt.AwpPlan(off, 0.0, 2, 8)
    graphed = adt.AwpPlan(off, 0.0, 2, 8)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            graphed.step(w, pg, og)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # capturing enqueued nothing; even the plan's first batch (which only
    # records norms) comes from the graph
    changes = 0
    prev = None
    for it in range(10):
        if it:
            scale = torch.from_numpy((1.0 + rng.choice([-0.05, 0.0, 0.05], size=N))
                                     .astype(np.float32))
            w.mul_(scale.cuda())                  # eager work between replays
        torch.cuda.synchronize()
        eager.step(w, pe, oe)
        g.replay()
        torch.cuda.synchronize()
        se, sg = eager.read(), graphed.read()
        for k in ("bits", "counter", "bytes"):
            assert np.array_equal(se[k], sg[k]), (it, k)
        assert se["packed_size"] == sg["packed_size"]
        assert se["stats"].tobytes() == sg["stats"].tobytes()
        n = se["packed_size"]
        assert torch.equal(pe[:n], pg[:n]) and torch.equal(oe.view(torch.int32), og.view(torch.int32))
        exp = oracle.pack(w.cpu().numpy(), off, se["bytes"])
        assert np.array_equal(pg[:n].cpu().numpy(), exp)
        if prev is not None and not np.array_equal(prev, se["bytes"]):
            changes += 1
        prev = se["bytes"]
    assert changes >= 2
    eager.close()
    graphed.close()


def test_launch_timing_stays_out_of_a_captured_graph(adt):
    """With launch timing switched on, a step captured into a graph is recorded as
    ordinary launches (timing events inside a capture would never complete); the
    replays are correct and adt_timing_read returns without blocking."""
    sizes = [5000, 4096, 77]
    off = workloads.offsets_from_sizes(sizes)
    N = int(off[-1])
    hw = workloads.ragged_case(sizes, [1] * 3, seed=5, he=True)[2]
    w = torch.from_numpy(hw).cuda()
    p = torch.zeros(4 * N, dtype=torch.uint8, device="cuda")
    o = torch.zeros(N, dtype=torch.float32, device="cuda")
    plan = adt.AwpPlan(off, -1.0, 5, 8, init_bits=np.full(3, 16, np.int32))
    torch.cuda.synchronize()
    adt.adt_timing_enable(True, 16)
    adt.adt_timing_read()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            plan.step(w, p, o)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert all(v["launches"] == 0 for v in adt.adt_timing_read().values())
    for _ in range(3):
        g.replay()
        torch.cuda.synchronize()
    plan.step(w, p, o)                       # an eager step is timed as usual
    torch.cuda.synchronize()
    t = adt.adt_timing_read()
    adt.adt_timing_enable(False)
    assert t["fused_kernel"]["launches"] == 1 and t["final_rule_kernel"]["launches"] == 1
    rb = np.full(3, 2, np.uint8)
    exp = oracle.pack(hw, off, rb)
    assert np.array_equal(p[:exp.size].cpu().numpy(), exp)
    assert np.array_equal(o.view(torch.int32).cpu().numpy(), oracle.unpack(exp, off, rb).view(np.int32))
    plan.close()


def count_redo_launches(adt, fn):
    """Run fn() with launch timing on; returns {kernel name: launches}."""
    adt.adt_timing_enable(True, 4096)
    adt.adt_timing_read()
    fn()
    torch.cuda.synchronize()
    t = adt.adt_timing_read()
    adt.adt_timing_enable(False)
    return {k: v["launches"] for k, v in t.items()}


@pytest.mark.parametrize("sync_every_step", [True, False])
def test_plan_leaves_the_redo_launch_out_only_when_nothing_can_change(adt, sync_every_step):
    """With INTERVAL = 6 and every batch counting, a layer's byte count moves on
    batches 7, 13, 19, ... (the first batch only records norms).  The library may
    leave the redo launch out while the host can prove, from the counter status
    the device publishes, that no counter can reach INTERVAL; every step still has
    to equal the oracle, with the host running ahead of the device or not."""
    sizes = [5000, 4096, 1, 0, 9000, 12289]
    off = workloads.offsets_from_sizes(sizes)
    L, N = len(sizes), int(off[-1])
    rng = np.random.default_rng(61)
    hw = rng.standard_normal(N).astype(np.float32) * np.float32(0.05)
    steps, interval = 40, 6
    ws = [torch.from_numpy(hw * np.float32(0.99) ** i).cuda() for i in range(steps)]   # norms shrink
    ps = [torch.full((4 * N,), 0xA5, dtype=torch.uint8, device="cuda") for _ in range(steps)]
    outs = [torch.zeros(N, dtype=torch.float32, device="cuda") for _ in range(steps)]
    plan = adt.AwpPlan(off, 0.0, interval, 8)

    def run():
        for i in range(steps):
            plan.step(ws[i], ps[i], outs[i])
            if sync_every_step:
                torch.cuda.synchronize()

    launches = count_redo_launches(adt, run)
    assert launches["fused_kernel"] == steps
    # a final reduction rides with the next batch while nothing can move, and is a launch of
    # its own next to every redo pass
    assert launches["redo_kernel"] <= launches["final_rule_kernel"] <= steps
    ost = oracle.AwpState(L, 8)
    changes, prev = 0, None
    for i in range(steps):
        hwi = ws[i].cpu().numpy()
        orb = oracle.awp_update(ost, oracle.stats(hwi, off)[:, 1], 0.0, interval, 8)
        exp = oracle.pack(hwi, off, orb)
        assert np.array_equal(ps[i][:exp.size].cpu().numpy(), exp), i
        assert np.array_equal(outs[i].view(torch.int32).cpu().numpy(),
                              oracle.unpack(exp, off, orb).view(np.int32)), i
        if prev is not None and not np.array_equal(prev, orb):
            changes += 1
        prev = orb
    got = plan.read()
    assert np.array_equal(got["bytes"], prev) and np.array_equal(got["counter"], ost.counter)
    assert changes == 3                                  # 8 -> 16 -> 24 -> 32 bits
    assert changes <= launches["redo_kernel"] <= steps
    if sync_every_step:
        # the host sees a fresh status word before every step: redo only where a counter stands at
        # INTERVAL - 1 or, the word being one batch old, may stand there: two batches in six
        assert launches["redo_kernel"] <= 14
    plan.close()


def test_plan_state_does_not_depend_on_where_the_final_reduction_ran(adt):
    """While no byte count can move, a batch's final reduction and rule ride at the
    head of the next batch's fused kernel; awp_plan_read launches them on their own
    if they have not run yet.  Both routes give the same bits: a plan that is read
    after every step and one that is read only at the end agree bit for bit in
    state and statistics, and with the oracle in counters and byte counts."""
    sizes = [300000, 4096, 1, 0, 70000, 12289, 1500000]     # several sub-blocks per big layer
    groups = [0, 1, 3, 5, 7]
    off = workloads.offsets_from_sizes(sizes)
    L, N = len(sizes), int(off[-1])
    grp = np.asarray(groups, np.int32)
    rng = np.random.default_rng(71)
    hw = rng.standard_normal(N).astype(np.float32) * np.float32(0.05)
    steps = 9
    ws = [torch.from_numpy(hw * np.float32(1.0 + 0.01 * ((i * 7) % 5 - 2))).cuda() for i in range(steps)]
    pa, pb = (torch.zeros(4 * N, dtype=torch.uint8, device="cuda") for _ in range(2))
    oa, ob = (torch.zeros(N, dtype=torch.float32, device="cuda") for _ in range(2))
    a = adt.AwpPlan(off, 0.0, 500, 8, group_offsets=groups)
    b = adt.AwpPlan(off, 0.0, 500, 8, group_offsets=groups)

    def run_b():
        for i in range(steps):
            b.step(ws[i], pb, ob)
    launches = count_redo_launches(adt, run_b)
    # the first batch's reduction rides with the second batch, and so on; only the last one is
    # launched on its own (by the read below), and no redo pass at all
    assert launches["fused_kernel"] == steps and launches["redo_kernel"] == 0
    assert launches["final_rule_kernel"] == 0
    ost = oracle.AwpState(len(groups) - 1, 8)
    for i in range(steps):
        a.step(ws[i], pa, oa)
        sa = a.read()
        hwi = ws[i].cpu().numpy()
        gb = oracle.awp_update(ost, oracle.group_norms(hwi, off, grp), 0.0, 500, 8)
        assert np.array_equal(sa["bytes"], np.repeat(gb, np.diff(grp))) and np.array_equal(sa["counter"], ost.counter)
        np.testing.assert_allclose(sa["stats"], oracle.stats(hwi, off), rtol=1e-10, atol=0.0)
    sb = b.read()
    for k in ("bits", "counter", "bytes"):
        assert np.array_equal(sa[k], sb[k]), k
    assert sa["stats"].tobytes() == sb["stats"].tobytes()
    assert a.get_state()["l2_prev"].tobytes() == b.get_state()["l2_prev"].tobytes()
    assert sa["counter"].max() >= 3                        # batches did count
    n = sa["packed_size"]
    assert n == sb["packed_size"] and torch.equal(pa[:n], pb[:n])
    assert torch.equal(oa.view(torch.int32), ob.view(torch.int32))
    a.close()
    b.close()


@pytest.mark.parametrize("big", [8_400_000, 40_000_000])
def test_carried_reduction_of_one_big_layer(adt, big):
    """A layer of many sub-blocks in a small plan (one slice per chunk) and in a
    medium one (three slices per chunk): every batch's reduction is carried by the
    next batch's kernel; state and statistics of the last batch against the oracle."""
    sizes = [5000, big, 70000]
    off = workloads.offsets_from_sizes(sizes)
    N = int(off[-1])
    rng = np.random.default_rng(73)
    hw = rng.standard_normal(N).astype(np.float32) * np.float32(0.05)
    w = torch.from_numpy(hw).cuda()
    packed = torch.zeros(4 * N, dtype=torch.uint8, device="cuda")
    out = torch.zeros(N, dtype=torch.float32, device="cuda")
    plan = adt.AwpPlan(off, 0.0, 300, 8)
    ost = oracle.AwpState(3, 8)
    steps = 5
    for i in range(steps):
        if i:
            w.mul_(0.98)
        plan.step(w, packed, out)
    for i in range(steps):                       # the oracle follows the same weights
        hwi = (torch.from_numpy(hw) * 1.0)
        for _ in range(i):
            hwi.mul_(0.98)
        hwi = hwi.numpy()
        orb = oracle.awp_update(ost, oracle.stats(hwi, off)[:, 1], 0.0, 300, 8)
    got = plan.read()
    assert np.array_equal(got["counter"], ost.counter) and got["counter"].tolist() == [4, 4, 4]
    assert np.array_equal(got["bytes"], orb)
    np.testing.assert_allclose(got["stats"], oracle.stats(hwi, off), rtol=1e-10, atol=0.0)
    assert np.array_equal(out.view(torch.int32).cpu().numpy(),
                          oracle.unpack(oracle.pack(hwi, off, orb), off, orb).view(np.int32))
    plan.close()


@pytest.mark.parametrize("seed", range(24))
def test_plan_random_configurations_against_the_oracle(adt, seed):
    """Random layer sizes, groups, AWP parameters and output formats; the state is read,
    flushed or left alone at random between steps, so that carried reductions, reductions
    launched by a read and in-order steps with a redo pass follow each other in every
    order.  Whenever the state is read it must equal the oracle's, and the stream and the
    truncated weights of every step must equal the oracle's for that step."""
    rng = np.random.default_rng(1000 + seed)
    L = int(rng.integers(1, 12))
    sizes = [int(x) for x in rng.choice([0, 1, 63, 1024, 4097, 30000, 262144, 700001], size=L)]
    if sum(sizes) == 0:
        sizes[0] = 5000
    cuts = sorted(set(int(c) for c in rng.integers(0, L + 1, size=int(rng.integers(0, 4)))) | {0, L})
    groups = cuts if rng.random() < 0.5 else list(range(L + 1))
    grp = np.asarray(groups, np.int32)
    G = grp.size - 1
    interval = int(rng.choice([1, 2, 3, 7, 50]))
    n_bits = int(rng.choice([3, 8, 8, 16]))
    T = float(rng.choice([0.0, -0.005, 0.02]))
    init = int(rng.choice([5, 8, 8, 16]))
    out_dtype = [torch.float32, torch.float32, torch.bfloat16, torch.float16][int(rng.integers(0, 4))]
    off = workloads.offsets_from_sizes(sizes)
    N = int(off[-1])
    hw = rng.standard_normal(N).astype(np.float32) * np.float32(0.05)
    w = torch.from_numpy(hw).cuda()
    steps = 14
    packed = [torch.full((4 * N + 8,), 0xA5, dtype=torch.uint8, device="cuda") for _ in range(steps)]
    outs = [torch.zeros(N, dtype=out_dtype, device="cuda") for _ in range(steps)]
    plan = adt.AwpPlan(off, T, interval, n_bits, init_bits=np.full(G, init, np.int32), group_offsets=groups)
    ost = oracle.AwpState(G, init)
    history = []
    for i in range(steps):
        if i:
            hw = hw * np.float32(rng.choice([0.9, 0.97, 1.0, 1.01, 1.1]))
            w.copy_(torch.from_numpy(hw))
        plan.step(w, packed[i], outs[i])
        gb = oracle.awp_update(ost, oracle.group_norms(hw, off, grp), T, interval, n_bits)
        orb = np.repeat(gb, np.diff(grp)).astype(np.uint8)
        history.append((hw.copy(), orb))
        action = rng.integers(0, 4)
        if action == 0:
            got = plan.read()
            assert np.array_equal(got["bytes"], orb), (seed, i)
            assert np.array_equal(got["bits"], ost.bits) and np.array_equal(got["counter"], ost.counter)
            np.testing.assert_allclose(got["stats"], oracle.stats(hw, off), rtol=1e-10, atol=0.0)
        elif action == 1:
            plan.flush()
        elif action == 2:
            torch.cuda.synchronize()
    got = plan.read()
    assert np.array_equal(got["bits"], ost.bits) and np.array_equal(got["counter"], ost.counter)
    for i, (hwi, orb) in enumerate(history):
        exp = oracle.pack(hwi, off, orb)
        hp = packed[i].cpu().numpy()
        assert np.array_equal(hp[:exp.size], exp), (seed, i)
        assert np.all(hp[4 * N:] == 0xA5)
        if out_dtype == torch.float32:
            assert np.array_equal(outs[i].view(torch.int32).cpu().numpy(),
                                  oracle.unpack(exp, off, orb).view(np.int32)), (seed, i)
        else:
            fmt = "bf16" if out_dtype == torch.bfloat16 else "fp16"
            assert np.array_equal(outs[i].view(torch.int16).cpu().numpy().view(np.uint16),
                                  oracle.unpack16(exp, off, orb, fmt)), (seed, i)
    plan.close()


def test_two_plans_on_two_streams_do_not_disturb_each_other(adt):
    """Two plans with different layer sets and parameters step on streams of their
    own, interleaved and without any wait in between; every step of each must equal
    the oracle's.  Everything a plan's step touches belongs to that plan."""
    rng = np.random.default_rng(77)
    cfg = [dict(sizes=[30000, 5, 262144, 4097, 700001], T=0.0, interval=2, n_bits=8, init=8,
                dtype=torch.float32),
           dict(sizes=[1024, 500000, 63, 131072], T=-0.005, interval=50, n_bits=16, init=16,
                dtype=torch.bfloat16)]
    steps = 10
    runs = []
    for c in cfg:
        off = workloads.offsets_from_sizes(c["sizes"])
        N, L = int(off[-1]), len(c["sizes"])
        hw = rng.standard_normal(N).astype(np.float32) * np.float32(0.05)
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            w = torch.from_numpy(hw).cuda()
            packed = [torch.full((4 * N,), 0xA5, dtype=torch.uint8, device="cuda") for _ in range(steps)]
            outs = [torch.zeros(N, dtype=c["dtype"], device="cuda") for _ in range(steps)]
        runs.append(dict(c=c, off=off, N=N, L=L, hw=hw, w=w, packed=packed, outs=outs, stream=stream,
                         plan=adt.AwpPlan(off, c["T"], c["interval"], c["n_bits"],
                                          init_bits=np.full(L, c["init"], np.int32)),
                         ost=oracle.AwpState(L, c["init"]), history=[]))
    torch.cuda.synchronize()
    for i in range(steps):
        for r in runs:
            c = r["c"]
            if i:
                r["hw"] = r["hw"] * np.float32(rng.choice([0.9, 0.97, 1.01, 1.1]))
            with torch.cuda.stream(r["stream"]):
                r["w"].copy_(torch.from_numpy(r["hw"]), non_blocking=False)
                r["plan"].step(r["w"], r["packed"][i], r["outs"][i])
            orb = oracle.awp_update(r["ost"], oracle.stats(r["hw"], r["off"])[:, 1], c["T"],
                                    c["interval"], c["n_bits"])
            r["history"].append((r["hw"].copy(), orb))
    for r in runs:
        got = r["plan"].read()
        assert np.array_equal(got["bits"], r["ost"].bits)
        assert np.array_equal(got["counter"], r["ost"].counter)
        for i, (hwi, orb) in enumerate(r["history"]):
            exp = oracle.pack(hwi, r["off"], orb)
            assert np.array_equal(r["packed"][i][:exp.size].cpu().numpy(), exp), i
            if r["c"]["dtype"] == torch.float32:
                assert np.array_equal(r["outs"][i].view(torch.int32).cpu().numpy(),
                                      oracle.unpack(exp, r["off"], orb).view(np.int32)), i
            else:
                assert np.array_equal(r["outs"][i].view(torch.int16).cpu().numpy().view(np.uint16),
                                      oracle.unpack16(exp, r["off"], orb, "bf16")), i
        r["plan"].close()


def test_carried_reduction_with_many_layers_and_changing_output_formats(adt):
    """3000 small layers (thousands of carried sub-blocks, tile search beyond the
    pivots, redo tables beyond LDS size) while nothing can move, the truncated
    weights asked for as FP32, bfloat16, binary16 or not at all from step to step:
    the state at the end and every step's stream against the oracle."""
    rng = np.random.default_rng(74)
    sizes = [int(x) for x in rng.integers(0, 6000, size=3000)]
    off = workloads.offsets_from_sizes(sizes)
    L, N = len(sizes), int(off[-1])
    hw = rng.standard_normal(N).astype(np.float32) * np.float32(0.05)
    w = torch.from_numpy(hw).cuda()
    steps = 6
    packed = [torch.zeros(4 * N, dtype=torch.uint8, device="cuda") for _ in range(steps)]
    outs = [torch.zeros(N, dtype=torch.float32, device="cuda"),
            torch.zeros(N, dtype=torch.bfloat16, device="cuda"),
            None,
            torch.zeros(N, dtype=torch.float16, device="cuda"),
            torch.zeros(N, dtype=torch.float32, device="cuda"),
            None]
    plan = adt.AwpPlan(off, 0.0, 1000, 8, init_bits=np.full(L, 16, np.int32))
    ost = oracle.AwpState(L, 16)
    hist = []
    for i in range(steps):
        if i:
            hw = hw * np.float32(0.97)
            w.copy_(torch.from_numpy(hw))
        plan.step(w, packed[i], outs[i])
        orb = oracle.awp_update(ost, oracle.stats(hw, off)[:, 1], 0.0, 1000, 8)
        hist.append((hw.copy(), orb))
    got = plan.read()
    assert np.array_equal(got["bits"], ost.bits) and np.array_equal(got["counter"], ost.counter)
    assert got["counter"].max() == steps - 1
    np.testing.assert_allclose(got["stats"], oracle.stats(hw, off), rtol=1e-10, atol=0.0)
    for i, (hwi, orb) in enumerate(hist):
        exp = oracle.pack(hwi, off, orb)
        assert np.array_equal(packed[i][:exp.size].cpu().numpy(), exp), i
        o = outs[i]
        if o is None:
            continue
        if o.dtype == torch.float32:
            assert np.array_equal(o.view(torch.int32).cpu().numpy(), oracle.unpack(exp, off, orb).view(np.int32)), i
        else:
            fmt = "bf16" if o.dtype == torch.bfloat16 else "fp16"
            assert np.array_equal(o.view(torch.int16).cpu().numpy().view(np.uint16),
                                  oracle.unpack16(exp, off, orb, fmt)), i
    plan.close()


def test_capture_refuses_a_plan_whose_last_batch_is_not_reduced_yet(adt):
    """An eager step may leave its final reduction to the next step; a step captured
    then would freeze that reduction into the graph.  The library refuses; after
    awp_plan_read the capture goes through and replays match the eager path."""
    sizes = [20000, 4096, 3000]
    off = workloads.offsets_from_sizes(sizes)
    N = int(off[-1])
    rng = np.random.default_rng(72)
    w = torch.from_numpy(rng.standard_normal(N).astype(np.float32) * np.float32(0.05)).cuda()
    packed = torch.zeros(4 * N, dtype=torch.uint8, device="cuda")
    out = torch.zeros(N, dtype=torch.float32, device="cuda")
    plan = adt.AwpPlan(off, 0.0, 500, 8)
    eager = adt.AwpPlan(off, 0.0, 500, 8)
    plan.step(w, packed, out)
    eager.step(w, packed, out)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    refused = False
    with torch.cuda.stream(side):
        try:
            with torch.cuda.graph(g, stream=side):
                try:
                    plan.step(w, packed, out)
                except adt.AdtError as err:
                    refused = "awp_plan_read" in str(err)
        except Exception:
            pass                                 # an empty capture may be refused by the runtime itself
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert refused
    plan.read()
    g = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            plan.step(w, packed, out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for it in range(4):
        w.mul_(0.99)
        torch.cuda.synchronize()
        g.replay()
        eager.step(w, packed, out)
        torch.cuda.synchronize()
        sg, se = plan.read(), eager.read()
        for k in ("bits", "counter", "bytes"):
            assert np.array_equal(sg[k], se[k]), (it, k)
        assert sg["stats"].tobytes() == se["stats"].tobytes()
    assert se["counter"].tolist() == [4, 4, 4]
    plan.close()
    eager.close()


def test_plan_resumed_next_to_a_change_runs_the_redo_pass(adt):
    """State restored with a counter one short of INTERVAL: the very next batch
    changes the byte count, so the first step after set_state must not leave
    the redo launch out."""
    sizes = [6000, 4096, 3000]
    off = workloads.offsets_from_sizes(sizes)
    N = int(off[-1])
    rng = np.random.default_rng(62)
    hw = rng.standard_normal(N).astype(np.float32) * np.float32(0.05)
    interval = 1000
    plan = adt.AwpPlan(off, 0.0, interval, 8)
    w = torch.from_numpy(hw).cuda()
    packed = torch.zeros(4 * N, dtype=torch.uint8, device="cuda")
    out = torch.zeros(N, dtype=torch.float32, device="cuda")
    for _ in range(3):
        plan.step(w, packed, out)
    norms = oracle.stats(hw, off)[:, 1]
    plan.set_state({"bits": np.array([8, 16, 8], np.int32),
                    "counter": np.array([interval - 1, 5, interval - 2], np.int32),
                    "l2_prev": norms * 2.0, "batches_seen": 1})     # this batch's norms are smaller: counts
    plan.step(w, packed, out)
    got = plan.read()
    assert got["bits"].tolist() == [16, 16, 8] and got["counter"].tolist() == [0, 6, interval - 1]
    rb = np.array([2, 2, 1], np.uint8)
    exp = oracle.pack(hw, off, rb)
    assert got["packed_size"] == exp.size
    assert np.array_equal(packed[:exp.size].cpu().numpy(), exp)
    assert np.array_equal(out.view(torch.int32).cpu().numpy(), oracle.unpack(exp, off, rb).view(np.int32))
    plan.step(w, packed, out)                # same weights again
    got = plan.read()
    assert got["counter"].tolist() == [0, 6, interval - 1]      # equal norms do not count with T = 0
    plan.close()


def test_plan_checkpoint_and_resume(adt):
    """A plan rebuilt from get_state() continues exactly like the original."""
    sizes = [3000, 4096, 17, 9000, 5000]
    groups = [0, 2, 3, 5]
    off = workloads.offsets_from_sizes(sizes)
    N = int(off[-1])
    rng = np.random.default_rng(33)
    hw = rng.standard_normal(N).astype(np.float32) * np.float32(0.05)
    w = torch.from_numpy(hw).cuda()
    pa, pb = (torch.zeros(4 * N, dtype=torch.uint8, device="cuda") for _ in range(2))
    oa, ob = (torch.zeros(N, dtype=torch.float32, device="cuda") for _ in range(2))
    a = adt.AwpPlan(off, 0.0, 2, 8, group_offsets=groups)
    fresh = adt.AwpPlan(off, 0.0, 2, 8, group_offsets=groups).get_state()
    assert fresh["batches_seen"] == 0 and fresh["bits"].tolist() == [8, 8, 8]

    def advance():
        scale = torch.from_numpy((1.0 + rng.choice([-0.05, 0.0, 0.05], size=N)).astype(np.float32))
        w.mul_(scale.cuda())

    for _ in range(7):
        a.step(w, pa, oa)
        advance()
    saved = a.get_state()
    assert saved["batches_seen"] == 1 and saved["bits"].max() > 8
    b = adt.AwpPlan(off, 0.0, 2, 8, group_offsets=groups)
    b.set_state(saved)
    for it in range(8):
        a.step(w, pa, oa)
        b.step(w, pb, ob)
        sa, sb = a.read(), b.read()
        for k in ("bits", "counter", "bytes"):
            assert np.array_equal(sa[k], sb[k]), (it, k)
        n = sa["packed_size"]
        assert n == sb["packed_size"] and torch.equal(pa[:n], pb[:n])
        assert torch.equal(oa.view(torch.int32), ob.view(torch.int32))
        ga, gb = a.get_state(), b.get_state()
        assert ga["l2_prev"].tobytes() == gb["l2_prev"].tobytes()
        advance()
    with pytest.raises(adt.AdtError):
        b.set_state({"bits": np.array([8, 40, 8]), "counter": np.zeros(3), "l2_prev": np.zeros(3),
                     "batches_seen": 1})
    a.close()
    b.close()
