"""Writes kvc1_handworked.json: pages small enough to encode by hand under the KVC-1 reading of
Algorithm 2 (KV-Cache Compression) and Section 3.5.3.  Inputs come from the formulas below; every
expected payload, scale and mode is typed in by hand with the working in its note.  Nothing here
calls the oracle or the GPU library: the fixture pins both from outside.

Run from the repository root: python tests/golden/write_handworked.py
"""
import json
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
cases = []


def hx(a):
    return np.asarray(a, np.float16).view(np.uint16).tobytes().hex()


def add(name, N, d, x, mode, scale_bits, payload_hex, xhat=None, note="", scheme=3):
    assert len(payload_hex) % 32 == 0
    c = dict(name=name, N=N, d=d, scheme=scheme, x_fp16_le_hex=hx(x), mode=mode, scale_bits=scale_bits,
             n16=len(payload_hex) // 32, payload_hex=payload_hex, note=note)
    if xhat is not None:
        c["xhat_bits_prefix"] = xhat
    cases.append(c)


i = np.arange(64)
add("all_zero", 1, 64, np.zeros(64), 3, "00000000", "00" * 16,
    note="amax=0: s=0, both groups zero-run packets, header byte 0x00")
add("all_127", 1, 64, np.full(64, 127.0), 3, "3f800000", "08fe" + "00" * 46,
    note="delta=[127,0,...]: g0 literal w=8 (u0=zigzag(127)=254), g1 zero-run; 1+32=33 -> 48 B")
x = i.astype(np.float64)
x[63] = 127
add("ramp", 1, 64, x, 3, "3f800000", "82" + "a8" + "aa" * 7 + "02" * 31 + "82" + "00" * 7,
    note="g0: u=[0,2,2,...] w=2 -> a8 aa*7; g1: u=[2]*31+[130] w=8; header 0x82; 1+8+32=41 -> 48 B")
add("stride4", 1, 64, -127 + 4 * i, 3, "3f800000", "98" + "fd" + "08" * 31 + "08" + "00" * 14,
    note="g0: u=[253,8,8,...] w=8; g1: all delta=4 -> run packet body 0x08; header 0x98; 1+32+1=34 -> 48 B")
x = np.zeros(64)
x[:31] = 4 * np.arange(31)
x[31] = 127
q = [4 * k for k in range(31)] + [127] + [0] * 32
add("fallback_int8", 1, 64, x, 1, "3f800000", bytes(q).hex(),
    note="g0 w=4 (16 B), g1 starts with delta=-127 -> w=8 (32 B); 1+16+32=49 -> 64 >= 64: stored as plain INT8")
x = np.zeros(64)
x[:4] = [1.0, 0.5, -1.0, 1 / 254]
add("unit_amax", 1, 64, x, 3, "3c010204", "08fe7d82fe" + "00" * 43, xhat=["3c00", "3808", "bc00", "0000"],
    note="amax=1: s=fl32(1/127)=0x3C010204, 1/s=127 exactly; q=[127,64,-127,0]; u=[254,125,130,254,0..]")
x = np.zeros((2, 32))
x[0, :] = 127
x[0, 0] = 63
x[0, 1] = 126
x[1, :] = 5
add("two_rows", 2, 32, x, 3, "3f800000", "47" + "7ebf" + "00" * 26 + "0a" + "00" * 15 + "00" * 3,
    note="rows are differenced along the channel index only: row0 q=[63,126,127,...] u=[126,126,2,0..] w=7 "
         "(126|126<<7|2<<14 = 0xBF7E); row1 q=5 everywhere, first column verbatim: u=[10,0,..] w=4; header 0x47; 1+28+16=45 -> 48 B")
x = np.zeros(64)
x[:3] = [3, -2, 1]
x[40] = 127
add("nodelta_mode4", 1, 64, x, 4, "3f800000", "83" + "9e" + "00" * 11 + "00" * 8 + "fe" + "00" * 23 + "00" * 3, scheme=4,
    note="mode 4 (extension: no delta step): u = zigzag(q) = [6,3,2,0..] -> w=3, 6|3<<3|2<<6 = 0x9E; second group has "
         "u[8] = zigzag(127) = 254 -> w=8; header 0x83; 1+12+32 = 45 -> 48 B")
x = np.zeros((16, 128))
x[0, 0] = 127
x[:, 2:4] = 1
x[5, 9] = -1
add("channel_pairs_mode5", 16, 128, x, 5, "3f800000",
    "18" + "00" * 7 + "09" + "00" * 23 + "fe" + "00" * 31 + "00080000" + "02" + "00" * 11, scheme=5,
    note="mode 5 (extension: groups are channel pairs over the 16 tokens, no delta step): pair p goes to group "
         "(p mod 4)*16 + p div 4, element (t, c) to position (t mod 4)*8 + (t div 4)*2 + (c mod 2). x[0][0]=127: pair 0, "
         "group 0, position 0, u=254 -> w=8; x[5][9]=-1: pair 4, group 1, position 8+2+1=11, u=1 -> w=1, bit 11 = byte 1 "
         "value 0x08; channels 2,3 all 1: pair 1, group 16, 32 equal u=2 -> run packet, body 0x02; every other group "
         "zero-run. Header nibbles 0,1,16 = 8,1,9. 32+32+4+1 = 69 -> 80 B")

x = np.zeros((16, 256))
x[0, 0] = 127
x[15, 77] = -3
x[9, 201] = 3
x[3, 130] = -1
x[:, 252:254] = 2
add("channel_pairs_mode5_d256", 16, 256, x, 5, "3f800000",
    "08" + "00" * 19 + "30" + "00" * 15 + "30" + "00" * 3 + "01" + "00" * 14 + "90" + "00" * 8
    + "fe" + "00" * 31 + "00" * 11 + "a0" + "00" * 5 + "03" + "00" * 6 + "00000001" + "04" + "00" * 3, scheme=5,
    note="mode 5 at d = 256 (extension): 32 channel octets in two runs of W = 16; channel c has octet o = c div 8, pair "
         "j = (c div 2) mod 4, group ((o div 16)*4 + j)*16 + o mod 16; position (t mod 4)*8 + (t div 4)*2 + c mod 2. "
         "x[0][0]=127: o=0 j=0 -> group 0, pos 0, u=254, w=8 (32 B: fe 00..). x[15][77]=-3: o=9 j=2 -> group 41, pos "
         "24+6+1=31, u=5, w=3 (12 B), bits 93..95 = 101b -> byte 11 = 0xA0. x[9][201]=3: o=25 (second run) j=0 -> group "
         "(4+0)*16+9=73, pos 8+4+1=13, u=6, w=3, bits 39..41 = 110b -> byte 5 = 0x03. x[3][130]=-1: o=16 j=1 -> group "
         "(4+1)*16+0=80, pos 24, u=1, w=1 (4 B), bit 24 -> byte 3 = 0x01. channels 252,253 all 2: o=31 j=2 -> group "
         "(4+2)*16+15=111, 32 equal u=4 -> run packet, body 0x04. Header (64 B): nibble of group 0 = 8 (byte 0 low), "
         "41 = 3 (byte 20 high), 73 = 3 (byte 36 high), 80 = 1 (byte 40 low), 111 = 9 (byte 55 high); all other groups "
         "zero-run. 64+32+12+12+4+1 = 125 -> 128 B")

x = np.zeros((16, 64))
x[0, 0] = 127
x[15, 45] = -3
x[9, 33] = 3
x[:, 62:64] = 2
add("channel_pairs_mode5_d64", 16, 64, x, 5, "3f800000",
    "08" + "00" + "03" + "00" * 7 + "30" + "00" * 4 + "90"
    + "fe" + "00" * 31 + "00" * 5 + "03" + "00" * 6 + "00" * 11 + "a0" + "04" + "00" * 7, scheme=5,
    note="mode 5 at d = 64 (extension): 8 channel octets, W = 8, so channel c (octet o = c div 8, pair j = (c div 2) mod 4) "
         "goes to group j*8 + o, position (t mod 4)*8 + (t div 4)*2 + c mod 2; 32 groups, 16 header bytes. x[0][0]=127: group 0, "
         "pos 0, u=254, w=8 (32 B). x[9][33]=3: o=4 j=0 -> group 4, pos 8+4+1=13, u=6, w=3 (12 B), bits 39..41 = 110b -> byte 5 = "
         "0x03. x[15][45]=-3: o=5 j=2 -> group 21, pos 24+6+1=31, u=5, w=3, bits 93..95 = 101b -> byte 11 = 0xA0. channels 62,63 "
         "all 2: o=7 j=3 -> group 31, 32 equal u=4 -> run packet, body 0x04. Header nibbles: group 0 = 8 (byte 0 low), 4 = 3 (byte 2 "
         "low), 21 = 3 (byte 10 high), 31 = 9 (byte 15 high). 16+32+12+12+1 = 73 -> 80 B")

x = np.zeros((3, 32))
x[1:, :] = 127
add("odd_group_count_n3_d32", 3, 32, x, 3, "3f800000",
    "8008" + ("fe" + "00" * 31) * 2 + "00" * 14,
    note="three groups (one per token row), so the header is two bytes and the second one's high nibble is unused: row 0 all "
         "zero -> code 0; rows 1 and 2 all 127 -> delta [127, 0, ...], u0 = 254, w = 8 (32 B each). Header byte 0 = g0 | g1<<4 = "
         "0x80, byte 1 = g2 = 0x08. 2 + 32 + 32 = 66 -> 80 B, below the 96 B of the INT8 form")
x = np.zeros((5, 96))
x[0, 0] = 127
x[2, 32:64] = 3
x[4, 95] = -1
add("short_last_pass_n5_d96", 5, 96, x, 3, "3f800000",
    "08000030" + "03000001" + "fefd" + "00" * 30 + "06" + "00" * 11 + "05" + "00" * 11 + "00000080" + "00" * 12,
    note="480 elements: 15 groups (three per token row of 96 channels), 8 header bytes, the last nibble unused. g0 (row 0, "
         "channels 0-31): q = [127, 0, ...] -> delta [127, -127, 0, ...] -> u = [254, 253, 0, ...], w = 8 (32 B: fe fd 00..). "
         "g7 (row 2, channels 32-63, all 3): delta [3, 0, ...] -> u0 = 6, w = 3 (12 B, byte 0 = 0x06). g8 (row 2, channels 64-95): "
         "delta [-3, 0, ...] -> u0 = 5, w = 3 (byte 0 = 0x05). g14 (row 4, channels 64-95): last element -1 -> position 31, u = 1, "
         "w = 1 (4 B, bit 31 -> byte 3 = 0x80). Header nibbles: g0 = 8 (byte 0 low), g7 = 3 (byte 3 high), g8 = 3 (byte 4 low), "
         "g14 = 1 (byte 7 low). 8 + 32 + 12 + 12 + 4 = 68 -> 80 B")

doc = dict(citation="Algorithm 2 (KV-Cache Compression) and Section 3.5.3 (inverse), under the KVC-1 reading of the "
           "unspecified byte format; worked by hand, not produced by any implementation. The paper prints no numeric example.",
           cases=cases)
with open(os.path.join(HERE, "kvc1_handworked.json"), "w") as f:
    json.dump(doc, f, indent=1)
