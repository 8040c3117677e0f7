"""Pins for the oracle's 16-bit unpack (no GPU)."""
import struct

import numpy as np
import pytest
import torch

import oracle
import workloads


def one_layer(n, r):
    return np.array([0, n], dtype=np.int64), np.array([r], dtype=np.uint8)


@pytest.mark.parametrize("r", [1, 2, 3, 4])
def test_bf16_is_the_two_byte_stream_of_the_same_weights(r):
    """The top 16 bits of what r bytes give back are what 2 bytes (1 byte for
    r = 1) would have kept: an identity between two different pack calls."""
    w = np.concatenate([workloads.random_bit_patterns(20000, seed=40 + r),
                        workloads.special_values()])
    off, rb = one_layer(w.size, r)
    got = oracle.unpack16(oracle.pack(w, off, rb), off, rb, "bf16")
    o2, b2 = one_layer(w.size, min(r, 2))
    coarse = oracle.unpack(oracle.pack(w, o2, b2), o2, b2)
    assert np.array_equal(got, (coarse.view(np.uint32) >> 16).astype(np.uint16))
    if r >= 2:
        assert got.tobytes() == oracle.pack(w, o2, b2).tobytes()
    # widening the bf16 result (library routine) gives back the 2-byte round trip
    wide = torch.from_numpy(got.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    assert wide.tobytes() == coarse.tobytes()


def test_fp16_hand_examples():
    def conv(value, r):
        w = np.array([value], dtype=np.float32)
        off, rb = one_layer(1, r)
        return int(oracle.unpack16(oracle.pack(w, off, rb), off, rb, "fp16")[0])
    assert conv(1.0, 4) == 0x3C00
    assert conv(-2.5, 2) == 0xC100
    assert conv(65504.0, 4) == 0x7BFF            # largest finite binary16
    assert conv(65520.0, 4) == 0x7C00            # rounds up past the largest: infinity
    assert conv(65519.0, 4) == 0x7BFF
    assert conv(2.0 ** -24, 4) == 0x0001         # smallest subnormal
    assert conv(2.0 ** -25, 4) == 0x0000         # tie, rounds to even (zero)
    assert conv(2.0 ** -25 * 1.5, 4) == 0x0001
    assert conv(1.0 + 2.0 ** -11, 4) == 0x3C00   # tie to even (down)
    assert conv(1.0 + 3 * 2.0 ** -11, 4) == 0x3C02   # tie to even (up)
    assert conv(0.1, 2) == 0x2E60                # 0.1 cut to 2 bytes is 0.099609375, exact in binary16
    assert struct.unpack("<e", struct.pack("<H", 0x2E60))[0] == 0.099609375
    assert conv(1.0, 1) == 0x3800                # 1 byte gives 0.5
    assert conv(float("inf"), 1) == 0x7C00       # 2^127 overflows binary16
    assert conv(-0.0, 3) == 0x8000
    assert conv(float("inf"), 4) == 0x7C00 and conv(float("-inf"), 2) == 0xFC00


def test_fp16_nan_rule():
    """A NaN becomes the quiet NaN 0x7E00 with the word's sign, whatever its payload;
    a NaN whose payload lies only in the dropped bytes has become an infinity before."""
    def conv_bits(bits, r):
        w = np.array([bits], dtype=np.uint32).view(np.float32)
        off, rb = one_layer(1, r)
        return int(oracle.unpack16(oracle.pack(w, off, rb), off, rb, "fp16")[0])
    assert conv_bits(0x7FC00000, 4) == 0x7E00            # the usual quiet NaN
    assert conv_bits(0xFFC00000, 4) == 0xFE00            # its negative
    assert conv_bits(0x7F800001, 4) == 0x7E00            # signalling, payload in the lowest bit
    assert conv_bits(0xFF800001, 4) == 0xFE00
    assert conv_bits(0x7FFFFFFF, 2) == 0x7E00            # payload survives the cut to 2 bytes
    assert conv_bits(0x7F800001, 3) == 0x7C00            # payload cut away: an infinity, not a NaN
    assert conv_bits(0xFF80FF00, 2) == 0xFC00


def test_fp16_matches_torch_conversion():
    ws = workloads.make_weight_set("tiny")
    rb = workloads.config_bytes("tiny")
    stream = oracle.pack(ws.weights, ws.layer_offsets, rb)
    got = oracle.unpack16(stream, ws.layer_offsets, rb, "fp16")
    back = oracle.unpack(stream, ws.layer_offsets, rb)
    ref = torch.from_numpy(back).half().view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)
    w = workloads.random_bit_patterns(100000, seed=50)
    off, r4 = one_layer(w.size, 4)
    got = oracle.unpack16(oracle.pack(w, off, r4), off, r4, "fp16")
    ref = torch.from_numpy(w.copy()).half().view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(w)
    assert nan.sum() > 100
    assert np.array_equal(got[~nan], ref[~nan])           # torch's NaN payloads are its own
    sign = (w.view(np.uint32)[nan] >> 16).astype(np.uint16) & 0x8000
    assert np.array_equal(got[nan], sign | 0x7E00)
