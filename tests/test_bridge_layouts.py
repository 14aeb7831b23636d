"""The packed layouts of the min-max containers, as include/twa.h words them, against the test bridge that
spreads stored codes out for the oracle (CPU only).  The GPU tests compare the quantiser's stored bytes with
the oracle's codes THROUGH that bridge, so this pins the layouts the library writes to the header's text."""
from types import SimpleNamespace

import numpy as np
import torch

from oracle.bridge import to_oracle

U8MM, U4MM, U16MM, U2MM, U1MM, U3MM = 4, 5, 6, 7, 8, 9


def _pm(dtype, data, D, bits):
    ab = torch.tensor([[0.5, -1.0]], dtype=torch.float32)
    return SimpleNamespace(dtype=dtype, data=data, scales=ab, D=D, n=data.shape[0], block=bits, gscale=1.0)


def _codes(n, ld, bits, seed):
    return np.random.default_rng(seed).integers(0, 1 << bits, size=(n, ld), dtype=np.int64)


def test_one_two_and_four_bit_fields_run_low_bits_first():
    # element i of a vector sits in byte i*B/8 at bit (i*B) mod 8
    n, ld = 3, 2048
    for dtype, bits in ((U1MM, 1), (U2MM, 2), (U4MM, 4)):
        c = _codes(n, ld, bits, bits)
        raw = np.zeros((n, ld * bits // 8), dtype=np.uint8)
        for i in range(ld):
            raw[:, (i * bits) // 8] |= (c[:, i] << ((i * bits) % 8)).astype(np.uint8)
        po = to_oracle(_pm(dtype, torch.from_numpy(raw), ld, bits), layer_off=[0, ld])
        assert np.array_equal(po.data, c)


def test_three_bit_groups_of_32_elements_in_three_words():
    # element e = 16h + 4k + m of a group: low two bits in word h at bit 2(4k + m), high bit in word 2 at
    # bit 8k + m + 4h; words are little endian, groups follow each other
    n, ld = 2, 2048
    c = _codes(n, ld, 3, 33)
    words = np.zeros((n, ld // 32, 3), dtype=np.uint64)
    for g in range(ld // 32):
        for h in range(2):
            for k in range(4):
                for m in range(4):
                    q = c[:, 32 * g + 16 * h + 4 * k + m].astype(np.uint64)
                    words[:, g, h] |= (q & np.uint64(3)) << np.uint64(2 * (4 * k + m))
                    words[:, g, 2] |= (q >> np.uint64(2)) << np.uint64(8 * k + m + 4 * h)
    raw = words.astype("<u4").reshape(n, -1).view(np.uint8)
    assert raw.shape == (n, ld * 3 // 8)
    po = to_oracle(_pm(U3MM, torch.from_numpy(raw.copy()), ld, 3), layer_off=[0, ld])
    assert np.array_equal(po.data, c)


def test_bytes_and_words_hold_the_code_minus_half_its_range():
    n, ld = 2, 2048
    for dtype, width, B in ((U8MM, 8, 8), (U8MM, 8, 6), (U16MM, 16, 16), (U16MM, 16, 12)):
        c = _codes(n, ld, B, B)
        stored = (c - (1 << (B - 1))).astype(np.int8 if width == 8 else np.int16)
        po = to_oracle(_pm(dtype, torch.from_numpy(stored), ld, B), layer_off=[0, ld])
        assert np.array_equal(po.data, c)
