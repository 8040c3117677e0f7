#!/usr/bin/env python3
"""Writes tests/golden/tiny_case.bin: the Tiny weight set (3 layers, 10,160
He-normal weights, seed 0, bytes per layer 2, 3, 4) with what the CPU oracle
computes from it.  Calls only workloads.py (inputs) and oracle/ (expected
values); nothing here comes from the GPU library.  Read by the C client of
tests/test_gpu_c_client.py.

Layout (little endian): "ADTT", int32 n_layers, int64 layer_offsets[L+1],
uint8 bytes_per_layer[L] zero-padded to a multiple of 8, int64 packed_size,
float32 weights[N], uint8 stream[packed_size] zero-padded to a multiple of 8,
float32 unpacked[N], float64 stats[L][3].
"""
import os
import struct
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle      # noqa: E402
import workloads   # noqa: E402


def pad8(b: bytes) -> bytes:
    return b + b"\0" * (-len(b) % 8)


def main() -> None:
    ws = workloads.make_weight_set("tiny")
    rb = workloads.config_bytes("tiny")
    off = ws.layer_offsets
    stream = oracle.pack(ws.weights, off, rb)
    unpacked = oracle.unpack(stream, off, rb)
    stats = oracle.stats(ws.weights, off)
    blob = b"ADTT" + struct.pack("<i", ws.n_layers) + off.astype("<i8").tobytes()
    blob += pad8(rb.astype(np.uint8).tobytes()) + struct.pack("<q", stream.size)
    blob += ws.weights.astype("<f4").tobytes() + pad8(stream.tobytes())
    blob += unpacked.astype("<f4").tobytes() + stats.astype("<f8").tobytes()
    path = os.path.join(HERE, "tiny_case.bin")
    with open(path, "wb") as f:
        f.write(blob)
    print("wrote %s: %d bytes, %d weights, %d stream bytes" % (path, len(blob), ws.n_weights, stream.size))


if __name__ == "__main__":
    main()
