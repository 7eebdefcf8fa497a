"""Pins of the layout reference encoders (tests/layout_ref.py): the 6-bit e2m3 format as published, the placement
of single codes in the fp6 operand form and in the weight-streaming layout, round trips.  CPU only."""
import numpy as np

import layout_ref


# ---------------------------------------------------------------- fp6 operand form (hardware container of the codes)

def test_e2m3_format_facts():
    """The 6-bit format as published (OCP Microscaling FP6 e2m3): largest value 7.5, smallest
    positive 0.125, 1.0 is exponent field 1 with a zero mantissa, positive patterns order like their values."""
    vals = [layout_ref.e2m3_value(c) for c in range(64)]
    assert max(vals) == 7.5 and min(v for v in vals if v > 0) == 0.125
    assert layout_ref.e2m3_value(0b001000) == 1.0 and layout_ref.e2m3_value(0b101000) == -1.0
    assert vals[:32] == sorted(vals[:32]) and len(set(vals[:32])) == 32
    assert [vals[32 + c] for c in range(32)] == [-v for v in vals[:32]]


def test_codes_are_exact_in_e2m3_and_products_sum_exactly_in_fp32():
    table = layout_ref.e2m3_code_table()
    assert [layout_ref.e2m3_value(c) for c in table] == [q / 8.0 for q in range(16)]
    assert table == tuple(range(16))                # the pattern of q/8 is q: subnormals below 8, exponent field 1 from 8 on
    # q/2 and q/4 would be exact too (any of the three scalings fits the format)
    vals = {layout_ref.e2m3_value(c) for c in range(32)}
    assert all(q / 2.0 in vals and q / 4.0 in vals for q in range(16))
    # worst case of the accumulator: K = 32768 products of (15/8)^2, added one by one in fp32
    step = np.float32(1.875) * np.float32(1.875)
    run = np.cumsum(np.full(32768, step, dtype=np.float32), dtype=np.float32)
    assert run[-1] == np.float32(3.515625 * 32768) and (np.diff(run.astype(np.float64)) == 3.515625).all()
    # and a random row pair: 64 * (fp32 running sum of (qa/8)(qb/8)) is the integer dot product at every step
    rng = np.random.default_rng(11)
    qa, qb = rng.integers(0, 16, 32768), rng.integers(0, 16, 32768)
    run = np.cumsum((qa / 8.0).astype(np.float32) * (qb / 8.0).astype(np.float32), dtype=np.float32)
    np.testing.assert_array_equal(64.0 * run.astype(np.float64), np.cumsum(qa * qb))


def test_fp6_layout_round_trip_and_placement():
    rng = np.random.default_rng(5)
    q = rng.integers(0, 16, (45, 384), dtype=np.uint8)                     # a ragged second row block
    buf = layout_ref.pack_fp6(q)
    assert buf.shape == (64 * 384 * 3 // 4,)
    np.testing.assert_array_equal(layout_ref.unpack_fp6(buf, 45, 384) * 8.0, q)
    # one code alone: row 37 (block 1, r = 5), k = 128 + 64 + 3 (chunk 1, group 2, field 3)
    one = np.zeros((45, 384), dtype=np.uint8)
    one[37, 195] = 9                                                        # 9/8 -> pattern 0b001001
    b1 = layout_ref.pack_fp6(one)
    base = (1 * 2 + 1) * 3072
    where = base + 64 * 5 + 16 * (2 ^ 1) + (6 * 3) // 8                     # bits 18..23 of the string: byte 2, bit 2
    assert np.flatnonzero(b1).tolist() == [where] and b1[where] == 0b001001 << 2
    # a field in the last 8 bytes: field 30 starts at bit 180 = byte 22, bit 4 -> tail byte 6
    one[:] = 0
    one[2, 30] = 15                                                         # 15/8 -> 0b001111
    b2 = layout_ref.pack_fp6(one)
    t = 2048 + 256 * 0 + 8 * 2 + 6
    assert np.flatnonzero(b2).tolist() == [t] and b2[t] == (0b001111 << 4) & 0xFF


def test_decode_layout_is_the_stated_permutation():
    """The weight-streaming layout only moves 16-byte pieces.  Checked three ways: one byte placed by hand,
    the multiset of bytes, and the layout read back as an axis transposition [block, chunk, s, r, 16] ->
    [block, r, chunk, s, 16] (the walk in the reference is loops over rows, chunks and pieces)."""
    rng = np.random.default_rng(11)
    p = rng.integers(0, 256, (40, 192), dtype=np.uint8)                    # 40 rows: a ragged third block; K = 384
    buf = layout_ref.pack_decode16(p)
    assert buf.shape == (48 * 192,)
    back = buf.reshape(3, 3, 4, 16, 16).transpose(0, 3, 1, 2, 4).reshape(48, 192)
    np.testing.assert_array_equal(back[:40], p)
    assert not back[40:].any()
    np.testing.assert_array_equal(np.sort(buf)[-p.size:], np.sort(p.ravel()))
    # row 21 (block 1, r = 5), byte 150 of the row = chunk 2, s = 1, byte 6 of the piece
    one = np.zeros((40, 192), dtype=np.uint8)
    one[21, 150] = 0xA7
    b = layout_ref.pack_decode16(one)
    where = 1 * 16 * 192 + 2 * 1024 + (16 * 1 + 5) * 16 + 6
    assert np.flatnonzero(b).tolist() == [where] and b[where] == 0xA7
