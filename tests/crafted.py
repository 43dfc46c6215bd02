"""Hand-assembled NZ streams for rejection tests (bytes written out field by field, no encoder involved)."""
import struct

import numpy as np


def frame_header(codec, raw_bytes, payload, p0, p1, step_bits):
    h = [0x31465A4E, codec, raw_bytes, payload, p0, p1, step_bits]
    x = 0x5A5A5A5A
    for v in h:
        x ^= v
    return struct.pack("<8I", *h, x)


def single_frame_stream(n, chunk, step_bits, frame, seg_syms=256, K=256):
    """64-byte stream header + one offset (pad 16) + the given frame bytes (padded to 16)."""
    assert n <= chunk
    frame = frame + bytes((-len(frame)) % 16)
    total = 64 + 16 + len(frame)
    hdr = struct.pack("<IIQIIIIIIQ", 0x31535A4E, 1, n, chunk, 1, step_bits, seg_syms, K, 0, total) + bytes(16)
    assert len(hdr) == 64
    return np.frombuffer(hdr + struct.pack("<QQ", 80, 0) + frame, np.uint8).copy()


def zero_bit_huffman_stream(n, step_bits, K=256):
    """A HUFFMAN frame that passes every header check (magic, check word, sizes, legal code lengths {1, 1}) but whose
    segment table claims 0 bits for every segment and whose payload ends right after the tables.  No prefix code
    spends fewer than one bit per symbol, so the frame is corrupt."""
    nseg = (n + 255) // 256
    lens = bytes([1, 1, 0, 0])
    segt = bytes(2 * nseg + (2 if nseg & 1 else 0))
    payload = lens + segt
    fr = frame_header(2, 4 * n, len(payload), 2, 256 | (K << 16), step_bits) + payload
    return single_frame_stream(n, n, step_bits, fr, K=K)
