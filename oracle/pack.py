"""CPU oracle for the stage-boundary packing of a sparse tensor (C, F) into one contiguous buffer.

TEST INFRASTRUCTURE ONLY; the product never imports this.

Sec. III-B (last paragraph): what crosses a stage boundary is the coordinate matrix and the feature matrix of the
sparse tensor.  The paper gives no wire format; the one taken here (little-endian, all sections 256-byte aligned):

    bytes 0..3    "SPCF"            bytes 4..7    uint32 version = 1
    bytes 8..15   int64  n (rows)   bytes 16..19  int32 channels     bytes 20..23 int32 dtype (0 fp32, 1 bf16)
    bytes 24..27  int32 tensor stride             bytes 28..31  0
    bytes 32..39  int64 offset of the coordinates (= 256)
    bytes 40..47  int64 offset of the features    (= 256 + n*16 rounded up to 256)
    bytes 48..55  int64 total bytes               (= features offset + n*channels*element size rounded up to 256)
    bytes 56..255 0
    coordinates: int32 [n][4] rows (b, x, y, z);  features: [n][channels] row-major;  padding bytes are 0.

Written with numpy array slicing only.  Pinned by tests/test_oracle_pins.py (an independent struct.unpack parse
of the header, round trips, sizes).
"""
from __future__ import annotations

import numpy as np

HEADER_BYTES = 256
ALIGN = 256
ELT = {0: 4, 1: 2}


def _up(v: int) -> int:
    return (v + ALIGN - 1) // ALIGN * ALIGN


def packed_bytes(n: int, channels: int, dtype: int) -> int:
    return HEADER_BYTES + _up(16 * n) + _up(n * channels * ELT[dtype])


def pack(coords, feats_bits, dtype: int, tensor_stride: int) -> np.ndarray:
    """coords int32 [n][4]; feats_bits: float32 [n][c] (dtype 0) or uint16 bf16 bit patterns [n][c] (dtype 1).
    Returns the packed buffer as uint8."""
    coords = np.ascontiguousarray(coords, np.int32)
    feats_bits = np.ascontiguousarray(feats_bits, np.float32 if dtype == 0 else np.uint16)
    n, c = feats_bits.shape
    assert coords.shape == (n, 4)
    f_off = HEADER_BYTES + _up(16 * n)
    total = packed_bytes(n, c, dtype)
    buf = np.zeros(total, np.uint8)
    buf[0:4] = np.frombuffer(b"SPCF", np.uint8)
    buf[4:8] = np.array([1], "<u4").view(np.uint8)
    buf[8:16] = np.array([n], "<i8").view(np.uint8)
    buf[16:28] = np.array([c, dtype, tensor_stride], "<i4").view(np.uint8)
    buf[32:56] = np.array([HEADER_BYTES, f_off, total], "<i8").view(np.uint8)
    buf[HEADER_BYTES:HEADER_BYTES + 16 * n] = coords.view(np.uint8).reshape(-1)
    buf[f_off:f_off + n * c * ELT[dtype]] = feats_bits.view(np.uint8).reshape(-1)
    return buf


def unpack(buf):
    """Returns (coords int32 [n][4], feats (float32 or uint16 bits) [n][c], dtype, tensor_stride)."""
    buf = np.ascontiguousarray(buf, np.uint8)
    if bytes(buf[0:4]) != b"SPCF" or int(buf[4:8].view("<u4")[0]) != 1:
        raise ValueError("not a packed sparse tensor")
    n = int(buf[8:16].view("<i8")[0])
    c, dtype, ts = (int(v) for v in buf[16:28].view("<i4"))
    c_off, f_off, total = (int(v) for v in buf[32:56].view("<i8"))
    if total != len(buf) or total != packed_bytes(n, c, dtype):
        raise ValueError("size fields do not match the buffer")
    coords = buf[c_off:c_off + 16 * n].view(np.int32).reshape(n, 4).copy()
    raw = buf[f_off:f_off + n * c * ELT[dtype]]
    feats = raw.view(np.float32 if dtype == 0 else np.uint16).reshape(n, c).copy()
    return coords, feats, dtype, ts
