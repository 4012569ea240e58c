"""Pins of the test-side f6-tile codec (tests/f6_codec.py): the format of include/smoothrot.h worked out by hand."""
import numpy as np
import pytest

import f6_codec as fc
import workloads as wl
from oracle import smoothrot_oracle as o


def test_field_and_code_are_inverse_and_range_checked():
    codes = np.arange(-8, 8)
    f = fc.f6_field(codes)
    assert np.array_equal(8.0 * o.e2m3_value(f), codes.astype(np.float64))
    assert np.array_equal(fc.f6_codes(f), codes)
    assert f.max() < 64 and len(set(f.tolist())) == 16
    with pytest.raises(AssertionError):
        fc.f6_field(np.array([8]))
    with pytest.raises(AssertionError):
        fc.f6_codes(np.array([9]))                                        # 9/8 * 8 = 9: not a code


def test_f6_tiles_hand_placed_codes():
    """One code at a time in an otherwise zero [16, 256] matrix: byte offset and bit position worked out
    by hand from the layout's definition."""
    def image(row, k, code):
        c = np.zeros((16, 256), np.int8)
        c[row, k] = code
        return fc.f6_tiles_pack(c)
    img = image(0, 0, 7)                                 # block (R=0, C=0), piece r=0,t=0,g=0, code j=0: byte 0, bits 0-5
    assert img.size == 2 * 2 * 768 and img[0] == 7 and img.sum() == 7
    img = image(0, 1, -8)                                # j=1: bits 6..11 of the string = 0b101000 << 6
    assert img[0] == 0 and img[1] == 40 >> 2 and np.count_nonzero(img) == 1      # 40 << 6 = 0x0A00
    img = image(0, 31, 1)                                # j=31: bits 186..191 -> last byte of the 8-byte tail
    assert img[512 + 7] == 1 << 2 and np.count_nonzero(img) == 1
    img = image(3, 32, 1)                                # g=1 (k=32), r=3, R=0: 16-byte part at 128 + 48
    assert img[128 + 48] == 1 and np.count_nonzero(img) == 1
    img = image(3, 64, 1)                                # t=1: 16-byte part at 256 + 48
    assert img[256 + 48] == 1 and np.count_nonzero(img) == 1
    img = image(8, 0, 1)                                 # R=1: second block of chunk 0; g flips with R & 1
    assert img[768 + 128] == 1 and np.count_nonzero(img) == 1
    img = image(8, 31, 1)                                # R=1 tail: 512 + 128 * (0 ^ 1) + 7
    assert img[768 + 512 + 128 + 7] == 4 and np.count_nonzero(img) == 1
    img = image(0, 64 + 31, 1)                           # t=1 tail shares the 16-byte slot of the t=0 tail: + 8
    assert img[512 + 8 + 7] == 4 and np.count_nonzero(img) == 1
    img = image(5, 32 + 64 + 31, -1)                     # r=5, t=1, g=1: 512 + 128 + 80 + 8, field 33 << 2 in the last byte
    assert img[512 + 128 + 80 + 8 + 7] == (33 << 2) & 255 and np.count_nonzero(img) == 1
    img = image(0, 128, 1)                               # chunk C=1 starts after both row blocks of chunk 0
    assert img[2 * 768] == 1 and np.count_nonzero(img) == 1


@pytest.mark.parametrize("rows,K", [(1, 128), (8, 256), (19, 384), (40, 896)])
def test_f6_tiles_round_trip(rows, K):
    c = wl.random_codes(rows + K, rows, K)
    img = fc.f6_tiles_pack(c)
    assert img.dtype == np.uint8 and img.size == ((rows + 7) // 8) * (K // 128) * 768
    assert np.array_equal(fc.f6_codes(fc.f6_tiles_unpack(img, rows, K)), c)
    # every byte of the image belongs to exactly one piece: flipping any code changes the image
    c2 = c.copy()
    c2[rows - 1, K - 1] = -8 if c[rows - 1, K - 1] != -8 else 7
    assert not np.array_equal(fc.f6_tiles_pack(c2), img)
