"""Pins for the CPU oracle's Bitpack / Bitunpack (no GPU).

Every check compares the oracle with something that is not the oracle: the
IEEE-754 encoding of hand-worked examples, the closed form "clear the low
8*(4-r) bits" over all 2^32 words, library routines (bfloat16 widening,
memcpy), an independent numpy byte-slicing formulation, and invariants.
"""
import json
import os
import struct
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
MASK = {1: 0xFF000000, 2: 0xFFFF0000, 3: 0xFFFFFF00, 4: 0xFFFFFFFF}


def one_layer(n, r):
    return np.array([0, n], dtype=np.int64), np.array([r], dtype=np.uint8)


def roundtrip(w, off, rb):
    return oracle.unpack(oracle.pack(w, off, rb), off, rb)


# ---------------------------------------------------------------- worked examples
def test_worked_examples_from_ieee754():
    ex = json.load(open(os.path.join(GOLDEN, "worked_examples.json")))["examples"]
    for e in ex:
        word = int(e["word"], 16)
        # the fixture's word really is the encoding of its value (struct, not oracle)
        assert struct.unpack("<I", struct.pack("<f", float(e["value"])))[0] == word
        w = np.array([word], dtype=np.uint32).view(np.float32)
        off, rb = one_layer(1, e["r"])
        stream = oracle.pack(w, off, rb)
        assert [f"{b:02X}" for b in stream] == e["stream"], e
        back = oracle.unpack(stream, off, rb)
        assert int(back.view(np.uint32)[0]) == int(e["kept"], 16), e
        expect = float(e["value_after"])
        assert back[0] == np.float32(expect) and np.signbit(back[0]) == np.signbit(expect), e


def test_format_field_widths_of_section_v_a():
    """r bytes keep exactly sign + exponent + mantissa bits of the r*8-bit
    format the paper lists; every other bit comes back zero."""
    facts = json.load(open(os.path.join(GOLDEN, "paper_facts.json")))
    w = workloads.random_bit_patterns(1 << 16, seed=7)
    u = w.view(np.uint32)
    for fmt in facts["transfer_formats"]["formats"]:
        r = fmt["bits"] // 8
        kept_bits = fmt["sign"] + fmt["exponent"] + fmt["mantissa"]
        assert kept_bits == fmt["bits"]
        off, rb = one_layer(w.size, r)
        back = roundtrip(w, off, rb).view(np.uint32)
        # IEEE-754 binary32 layout: sign bit 31, exponent bits 30..23, mantissa 22..0
        sign = (back >> 31) & 1
        expo = (back >> 23) & 0xFF
        mant = back & 0x7FFFFF
        assert np.array_equal(sign, (u >> 31) & 1)
        lost_exp = 8 - fmt["exponent"]
        assert np.array_equal(expo, (((u >> 23) & 0xFF) >> lost_exp) << lost_exp)
        lost_man = 23 - fmt["mantissa"]
        assert np.array_equal(mant, ((u & 0x7FFFFF) >> lost_man) << lost_man)
    # 8-bit format: exponent's lowest bit is lost, so +inf becomes 2^127
    off, rb = one_layer(1, 1)
    inf = np.array([np.inf], dtype=np.float32)
    assert roundtrip(inf, off, rb)[0] == np.float32(2.0 ** 127)


def test_figure2_size_and_order():
    facts = json.load(open(os.path.join(GOLDEN, "paper_facts.json")))["figure2"]
    n, r = facts["weights"], facts["round_to"]
    # weights A..H with distinguishable bytes X3 X2 X1 X0
    words = np.array([(0xA0 + i) << 24 | (0xB0 + i) << 16 | (0xC0 + i) << 8 | (0xD0 + i)
                      for i in range(n)], dtype=np.uint32)
    off, rb = one_layer(n, r)
    stream = oracle.pack(words.view(np.float32), off, rb)
    assert stream.size * 8 == facts["stored_bits"]
    for i in range(n):  # element i occupies bytes [3i, 3i+3): bytes 1..3 of the word
        assert set(stream[3 * i:3 * i + 3].tolist()) == {0xA0 + i, 0xB0 + i, 0xC0 + i}
        assert 0xD0 + i not in stream.tolist()


# ---------------------------------------------------------------- exhaustive closed form
def _exhaustive_chunk(args):
    start, count = args
    u = np.arange(start, start + count, dtype=np.uint64).astype(np.uint32)
    w = u.view(np.float32)
    bad = 0
    for r in (1, 2, 3, 4):
        off, rb = one_layer(count, r)
        back = roundtrip(w, off, rb).view(np.uint32)
        bad += int(np.count_nonzero(back != (u & np.uint32(MASK[r]))))
    return bad


def test_all_bit_patterns_match_mask_closed_form():
    """unpack(pack(w, r)) == bits(w) & (0xFFFFFFFF << 8(4-r)) for ALL 2^32 words."""
    chunk = 1 << 24
    jobs = [(s, chunk) for s in range(0, 1 << 32, chunk)]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        bad = sum(ex.map(_exhaustive_chunk, jobs))
    assert bad == 0


# ---------------------------------------------------------------- library routines
def test_four_bytes_is_memcpy_and_identity():
    w = workloads.random_bit_patterns(100003, seed=1)
    off, rb = one_layer(w.size, 4)
    stream = oracle.pack(w, off, rb)
    assert stream.tobytes() == w.tobytes()
    assert roundtrip(w, off, rb).tobytes() == w.tobytes()


def test_two_bytes_is_bfloat16_by_truncation():
    w = workloads.he_normal_weights(workloads.tiny_shapes(), seed=0)
    off, rb = one_layer(w.size, 2)
    stream = oracle.pack(w, off, rb)
    as_bf16 = torch.from_numpy(stream.copy()).view(torch.bfloat16)
    widened = as_bf16.float().numpy()            # exact library widening
    assert widened.tobytes() == oracle.unpack(stream, off, rb).tobytes()
    hi16 = (torch.from_numpy(w.copy()).view(torch.int32) >> 16).to(torch.int16).numpy()
    assert stream.view(np.int16).tobytes() == hi16.tobytes()


@pytest.mark.parametrize("r", [1, 2, 3, 4])
def test_stream_equals_numpy_byte_slicing(r):
    """Independent formulation: the last r bytes of each little-endian word."""
    w = workloads.random_bit_patterns(4099, seed=20 + r)
    off, rb = one_layer(w.size, r)
    expect = w.view(np.uint8).reshape(-1, 4)[:, 4 - r:].reshape(-1)
    assert np.array_equal(oracle.pack(w, off, rb), expect)
    # and the inverse, by placing the bytes back into zeroed words
    words = np.zeros((w.size, 4), dtype=np.uint8)
    words[:, 4 - r:] = expect.reshape(-1, r)
    assert oracle.unpack(expect, off, rb).tobytes() == words.tobytes()


# ---------------------------------------------------------------- layout across layers
def test_layers_concatenate_without_padding():
    off, rb, w = workloads.alignment_sweep_case()
    stream = oracle.pack(w, off, rb)
    sizes = np.diff(off)
    assert stream.size == int(np.sum(sizes * rb)) == oracle.packed_size(off, rb)
    parts, pos = [], 0
    for l in range(len(rb)):
        o1, r1 = one_layer(int(sizes[l]), int(rb[l]))
        part = oracle.pack(w[off[l]:off[l + 1]], o1, r1)
        assert np.array_equal(part, stream[pos:pos + part.size])
        pos += part.size
        parts.append(part)
    assert pos == stream.size
    # every start offset modulo 16 occurs, so the GPU alignment paths get inputs
    starts = np.concatenate([[0], np.cumsum(sizes * rb)[:-1]])
    pairs = {(int(r), int(s % 16)) for r, s, n in zip(rb, starts, sizes) if n > 0}
    assert pairs >= {(r, s) for r in (1, 2, 3, 4) for s in range(16)}
    back = oracle.unpack(stream, off, rb).view(np.uint32)
    for l in range(len(rb)):
        seg = slice(off[l], off[l + 1])
        assert np.array_equal(back[seg], w.view(np.uint32)[seg] & np.uint32(MASK[int(rb[l])]))


def test_tiny_config_size():
    ws = workloads.make_weight_set("tiny")
    rb = workloads.config_bytes("tiny")
    assert ws.n_weights == 10160
    assert oracle.packed_size(ws.layer_offsets, rb) == 35168
    assert oracle.pack(ws.weights, ws.layer_offsets, rb).size == 35168


def test_empty_inputs():
    off = np.array([0], dtype=np.int64)
    assert oracle.pack(np.zeros(0, np.float32), off, np.zeros(0, np.uint8)).size == 0
    off = np.array([0, 0, 0], dtype=np.int64)
    rb = np.array([1, 3], dtype=np.uint8)
    assert oracle.pack(np.zeros(0, np.float32), off, rb).size == 0
    assert oracle.unpack(np.zeros(0, np.uint8), off, rb).size == 0


# ---------------------------------------------------------------- invariants
def test_invariants():
    w = np.concatenate([workloads.random_bit_patterns(50000, seed=3),
                        workloads.special_values()])
    u = w.view(np.uint32)
    for r in (1, 2, 3, 4):
        off, rb = one_layer(w.size, r)
        stream = oracle.pack(w, off, rb)
        q = oracle.unpack(stream, off, rb)
        qu = q.view(np.uint32)
        assert np.array_equal(qu >> 31, u >> 31)                        # sign kept
        assert np.all((qu & 0x7FFFFFFF) <= (u & 0x7FFFFFFF))            # magnitude never grows
        assert np.all(qu & np.uint32(~MASK[r] & 0xFFFFFFFF) == 0)       # zero fill
        assert roundtrip(q, off, rb).tobytes() == q.tobytes()           # idempotent
        assert np.array_equal(oracle.pack(q, off, rb), stream)          # pack(unpack(P)) == P
        for r1 in range(1, r):                                          # coarser after finer
            o1, b1 = one_layer(w.size, r1)
            assert roundtrip(q, o1, b1).tobytes() == roundtrip(w, o1, b1).tobytes()


def test_relative_error_bounds_for_normal_numbers():
    w = workloads.he_normal_weights(workloads.alexnet_shapes()[:2], seed=9)
    w = w[np.abs(w) >= np.finfo(np.float32).tiny].astype(np.float64)
    w32 = w.astype(np.float32)
    for r, bound in ((2, 2.0 ** -7), (3, 2.0 ** -15)):
        off, rb = one_layer(w32.size, r)
        q = roundtrip(w32, off, rb).astype(np.float64)
        rel = (np.abs(w) - np.abs(q)) / np.abs(w)
        assert rel.min() >= 0.0 and rel.max() < bound
        assert rel.max() > bound / 4          # the bound is nearly attained
    off, rb = one_layer(w32.size, 1)
    q = np.abs(roundtrip(w32, off, rb).astype(np.float64))
    assert np.all(q <= np.abs(w)) and np.all(q > np.abs(w) / 4)


def test_special_values_documented_behaviour():
    def rt(word, r):
        off, rb = one_layer(1, r)
        return int(roundtrip(np.array([word], np.uint32).view(np.float32), off, rb)
                   .view(np.uint32)[0])
    assert rt(0x7F800001, 2) == 0x7F800000     # NaN with payload in dropped bits -> +inf
    assert rt(0x7F8000FF, 3) == 0x7F800000
    assert rt(0x7FC00000, 2) == 0x7FC00000     # quiet NaN survives at 2 bytes
    assert rt(0x7FC00000, 1) == 0x7F000000     # ... but not at 1 byte
    assert rt(0x80000000, 1) == 0x80000000     # -0 stays -0
    assert rt(0x007FFFFF, 2) == 0x007F0000     # denormal keeps its high mantissa bits
    assert rt(0x0000FFFF, 2) == 0x00000000


def test_invalid_tables_rejected():
    w = np.zeros(4, np.float32)
    with pytest.raises(ValueError):
        oracle.pack(w, np.array([0, 4]), np.array([5], np.uint8))
    with pytest.raises(ValueError):
        oracle.pack(w, np.array([0, 4]), np.array([0], np.uint8))
    with pytest.raises(ValueError):
        oracle.pack(w, np.array([0, 5, 4]), np.array([1, 1], np.uint8))
    with pytest.raises(ValueError):
        oracle.pack(w, np.array([1, 4]), np.array([1], np.uint8))


# ---------------------------------------------------------------- property test
from hypothesis import given, settings, strategies as st  # noqa: E402


@settings(max_examples=60, deadline=None)
@given(st.lists(st.tuples(st.integers(0, 40), st.integers(1, 4)), min_size=0, max_size=8),
       st.integers(0, 2 ** 32 - 1))
def test_random_tables_round_trip_is_the_mask(layers, seed):
    sizes = [n for n, _ in layers]
    rb = np.array([r for _, r in layers], dtype=np.uint8)
    off = workloads.offsets_from_sizes(sizes)
    w = workloads.random_bit_patterns(int(off[-1]), seed)
    stream = oracle.pack(w, off, rb)
    assert stream.size == sum(n * r for n, r in layers)
    back = oracle.unpack(stream, off, rb).view(np.uint32)
    u = w.view(np.uint32)
    pos = 0
    for l, (n, r) in enumerate(layers):
        seg = slice(int(off[l]), int(off[l + 1]))
        assert np.array_equal(back[seg], u[seg] & np.uint32(MASK[r]))
        # element i of the layer sits at stream bytes [pos + i r, pos + (i + 1) r)
        img = u[seg].astype("<u4").view(np.uint8).reshape(-1, 4)[:, 4 - r:]
        assert np.array_equal(stream[pos:pos + n * r].reshape(-1, r), img)
        pos += n * r
