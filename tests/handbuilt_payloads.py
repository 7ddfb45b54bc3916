"""Payloads typed in by hand for the decoders (2 tokens x 64 channels: four packet groups, INT8 size 128 bytes),
with what a decoder has to make of them.  Used by the oracle's pins and by the GPU parity tests; no code of
either side had a part in these bytes.

Layout of a packed page: header (one 4-bit code per group, even group in the low nibble), then the packet bodies
in group order, zero padding to a multiple of 16 bytes.  Scale 0.5, so a code q decodes to q / 2 exactly."""
import numpy as np

N, D, SCALE = 2, 64, 0.5

_G0 = bytes([254] + [0] * 31)          # width 8: u0 = 254 (delta +127), the rest 0 -> token 0, channels 0..31 = 127
_G1 = bytes([0x01, 0, 0, 0])           # width 1: u0 = 1 (delta -1)                -> token 0, channels 32..63 = 126
_G2 = bytes([0, 0, 0, 0])              # width 1: all 0                            -> token 1, channels 0..31 = 0
_G3 = bytes([0, 0, 0, 0x80])           # width 1: u31 = 1 (delta -1 at channel 63) -> token 1, channel 63 = -1


def _pad(b, n16=None):
    n = (len(b) + 15) // 16 * 16 if n16 is None else n16 * 16
    return b + bytes(n - len(b))


def _values(tok0_hi, tok1_last=-1):
    q = np.zeros((N, D), np.float32)
    q[0, :32] = 127
    q[0, 32:] = tok0_hi
    q[1, 63] = tok1_last
    return (q * SCALE).astype(np.float16)


# (name, mode, payload, decodes?, expected FP16 values or None)
CASES = [
    ("literal packets only, mode 3", 3, _pad(bytes([0x18, 0x11]) + _G0 + _G1 + _G2 + _G3), True, _values(126)),
    ("literal packets only, mode 2", 2, _pad(bytes([0x18, 0x11]) + _G0 + _G1 + _G2 + _G3), True, _values(126)),
    ("a zero-run packet, mode 3", 3, _pad(bytes([0x08, 0x11]) + _G0 + _G2 + _G3), True, _values(127)),
    ("a zero-run packet in a mode-2 page", 2, _pad(bytes([0x08, 0x11]) + _G0 + _G2 + _G3), False, None),
    ("a run packet of ones, mode 3", 3, _pad(bytes([0x98, 0x11]) + _G0 + bytes([1]) + _G2 + _G3), True, _values(126 - np.arange(32))),
    ("a run packet in a mode-2 page", 2, _pad(bytes([0x98, 0x11]) + _G0 + bytes([1]) + _G2 + _G3), False, None),
    ("code 10 where an 8 would make the sizes fit", 3, _pad(bytes([0x1A, 0x11]) + _G0 + _G1 + _G2 + _G3), False, None),
    ("code 15 where an 8 would make the sizes fit", 3, _pad(bytes([0x1F, 0x11]) + _G0 + _G1 + _G2 + _G3), False, None),
    ("sixteen bytes more than the packets need", 3, _pad(bytes([0x18, 0x11]) + _G0 + _G1 + _G2 + _G3, 4), False, None),
    ("sixteen bytes fewer than the packets need", 3, _pad(bytes([0x18, 0x11]) + _G0 + _G1 + _G2 + _G3)[:32], False, None),
    ("packed page of 112 bytes: the largest valid one", 3, _pad(bytes([0x88, 0x56]) + _G0 + bytes(32) + bytes(24) + bytes(20)), True,
     np.concatenate([np.full(64, 63.5), np.zeros(64)]).astype(np.float16).reshape(N, D)),
    ("packed page as large as its INT8 form", 3, _pad(bytes([0x88, 0x78]) + _G0 + bytes(32) + bytes(32) + bytes(28)), False, None),
    ("packed page larger than its INT8 form", 3, _pad(bytes([0x88, 0x88]) + _G0 + bytes(32) + bytes(32) + bytes(32)), False, None),
    ("the first payload labelled mode 4: no delta step", 4, _pad(bytes([0x18, 0x11]) + _G0 + _G1 + _G2 + _G3), True,
     np.array([63.5] + [0.0] * 31 + [-0.5] + [0.0] * 31 + [0.0] * 63 + [-0.5], np.float16).reshape(N, D)),
    ("the first payload labelled mode 5, which 2-token pages do not have", 5, _pad(bytes([0x18, 0x11]) + _G0 + _G1 + _G2 + _G3), False, None),
    ("the first payload labelled mode 6", 6, _pad(bytes([0x18, 0x11]) + _G0 + _G1 + _G2 + _G3), False, None),
    # mode 1: the 128 codes as they are (two's complement), scale 0.5
    ("INT8 page", 1, bytes([127, 0x81, 1, 0xFF] + [0] * 124), True,
     np.array([63.5, -63.5, 0.5, -0.5] + [0.0] * 124, np.float16).reshape(N, D)),
    ("INT8 page with sixteen bytes too many", 1, bytes([127, 0x81, 1, 0xFF] + [0] * 140), False, None),
    ("INT8 page with sixteen bytes too few", 1, bytes([127, 0x81, 1, 0xFF] + [0] * 108), False, None),
    # mode 0: the FP16 bit patterns, little-endian (0x3C00 = 1.0, 0xC000 = -2.0, 0x7E00 = a NaN)
    ("raw page", 0, bytes([0x00, 0x3C, 0x00, 0xC0, 0x00, 0x7E] + [0] * 250), True,
     np.array([0x3C00, 0xC000, 0x7E00] + [0] * 125, np.uint16).view(np.float16).reshape(N, D)),
    ("raw page with sixteen bytes too many", 0, bytes([0x00, 0x3C] + [0] * 270), False, None),
    ("raw page with sixteen bytes too few", 0, bytes([0x00, 0x3C] + [0] * 238), False, None),
]
for _name, _mode, _pl, _ok, _val in CASES:
    assert len(_pl) % 16 == 0 and (_val is None) == (not _ok)
assert len(CASES[10][2]) == 112 and len(CASES[11][2]) == 128 and len(CASES[12][2]) == 144
