"""Test-side codec of the library's "f6 tiles" (include/smoothrot.h, "Fast prefill path"): encodes INT4 codes
into the byte image sr_pack_f6_tiles / sr_fwht_quant_act_f6 write and decodes such an image back, so that the
tests can compare the library's operands with the oracle's codes.  It restates a storage format of the library,
not arithmetic of the method: the only thing taken from the oracle is the value of a 6-bit E2M3 pattern.
Pinned in tests/test_f6_codec.py (hand-placed codes, round trips)."""
import numpy as np

from oracle import smoothrot_oracle as o


def f6_field(codes) -> np.ndarray:
    """6-bit pattern of code / 8: sign bit, then the magnitude |code| (0..8) in the low 5 bits."""
    c = np.asarray(codes).astype(np.int64)
    assert c.min(initial=0) >= o.QMIN and c.max(initial=0) <= o.QMAX
    return (np.where(c < 0, 32, 0) | np.abs(c)).astype(np.uint8)


def _piece_offsets(R: int, r: int, t: int, g: int):
    return 256 * t + 128 * (g ^ (R & 1)) + 16 * r, 512 + 128 * (g ^ (R & 1)) + 16 * r + 8 * t


def f6_tiles_pack(codes: np.ndarray) -> np.ndarray:
    """[rows, K] codes -> the byte image of their f6 tiles (K % 128 == 0; rows padded with zero
    codes to a multiple of 8).  Block (R, C) = rows 8R..8R+7 x codes 128C..128C+127 is 768 bytes at
    ((C * rows/8) + R) * 768; piece (r, t, g) = codes k = 128C + 64t + 32g + j, j = 0..31, of row
    8R + r as a 192-bit little-endian string (code j in bits 6j..6j+5); its first 16 bytes sit at
    256t + 128(g ^ (R & 1)) + 16r, its last 8 bytes at 512 + 128(g ^ (R & 1)) + 16r + 8t."""
    rows, K = codes.shape
    assert K % 128 == 0
    rb, nc = (rows + 7) // 8, K // 128
    c = np.zeros((rb * 8, K), dtype=np.int64)
    c[:rows] = codes
    f = f6_field(c).reshape(rb, 8, nc, 2, 2, 32)                                  # R, r, C, t, g, j
    bits = ((f[..., None] >> np.arange(6, dtype=np.uint8)) & 1).reshape(rb, 8, nc, 2, 2, 192)
    by = np.packbits(bits, axis=-1, bitorder="little")                            # 24 bytes per piece
    out = np.zeros((nc, rb, 768), dtype=np.uint8)
    for R in range(rb):
        for r in range(8):
            for t in range(2):
                for g in range(2):
                    o16, o8 = _piece_offsets(R, r, t, g)
                    out[:, R, o16:o16 + 16] = by[R, r, :, t, g, :16]
                    out[:, R, o8:o8 + 8] = by[R, r, :, t, g, 16:]
    return out.reshape(-1)


def f6_tiles_unpack(buf: np.ndarray, rows: int, K: int) -> np.ndarray:
    """Inverse of f6_tiles_pack: the 6-bit patterns [rows, K] stored in a tile image."""
    rb, nc = (rows + 7) // 8, K // 128
    img = np.asarray(buf, dtype=np.uint8)[:rb * nc * 768].reshape(nc, rb, 768)
    f = np.zeros((rb, 8, nc, 2, 2, 32), dtype=np.uint8)
    w = (1 << np.arange(6)).astype(np.uint8)
    for R in range(rb):
        for r in range(8):
            for t in range(2):
                for g in range(2):
                    o16, o8 = _piece_offsets(R, r, t, g)
                    by = np.concatenate([img[:, R, o16:o16 + 16], img[:, R, o8:o8 + 8]], axis=1)   # [nc, 24]
                    bits = np.unpackbits(by, axis=-1, bitorder="little").reshape(nc, 32, 6)
                    f[R, r, :, t, g, :] = (bits * w).sum(axis=-1)
    return f.reshape(rb * 8, K)[:rows]


def f6_codes(fields: np.ndarray) -> np.ndarray:
    """6-bit patterns -> the INT4 codes they stand for: 8 * e2m3_value (asserted integral, in range)."""
    v = 8.0 * o.e2m3_value(fields)
    c = np.rint(v)
    assert np.array_equal(c, v) and c.min(initial=0) >= o.QMIN and c.max(initial=0) <= o.QMAX
    return c.astype(np.int8)
