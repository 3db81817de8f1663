import struct

import numpy as np


def f32_bits(x):
    """binary32 bits of a double, rounded once by the hardware conversion (RNE, overflow -> inf)."""
    with np.errstate(over="ignore"):
        return int(np.array([x], dtype=np.float64).astype(np.float32).view(np.uint32)[0])


def bits_f32(b):
    return struct.unpack("<f", struct.pack("<I", int(b) & 0xFFFFFFFF))[0]


def fp16_bits(x):
    return int(np.float16(x).view(np.uint16))


def bf16_bits(x):
    b = f32_bits(x)
    assert b & 0xFFFF == 0, "value not representable in bf16"
    return b >> 16


def e5m2_bits(x):
    b = fp16_bits(x)
    assert b & 0xFF == 0, "value not representable in e5m2"
    return b >> 8


ENCODERS = {"fp16": fp16_bits, "bf16": bf16_bits, "e5m2": e5m2_bits, "tf32": f32_bits}     # (a TF32 operand is a binary32 word)
