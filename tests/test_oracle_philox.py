"""Pins for the oracle's counter-based dropout generator."""
import os

import numpy as np

from oracle import nmt_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    n = 0
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        out = O.philox4x32_10(np.array(w[:4]), w[4:6])
        assert [int(x) for x in out] == w[6:]
        n += 1
    assert n >= 2


def test_philox_is_a_bijection_on_a_sample():
    # distinct counters under one key never collide
    ctr = np.zeros((4096, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(4096)
    out = O.philox4x32_10(ctr, (7, 9))
    assert len({tuple(r) for r in out.tolist()}) == 4096


def test_dropout_threshold_is_exact():
    assert O.dropout_threshold(0.5) == 32768
    assert O.dropout_threshold(0.0) == 0
    # 0.3 as float32 is slightly above 0.3; ceil(p * 65536)
    assert O.dropout_threshold(0.3) == 19661
    assert O.dropout_threshold(0.1) == 6554


def test_dropout_identity_determinism_and_rate():
    uid = np.arange(8)
    assert O.dropout_keep(0, 3, 1, 0, uid, 16, 64, 0.0).all()
    a = O.dropout_keep(5, 17, 3, 1, uid, 16, 64, 0.3)
    b = O.dropout_keep(5, 17, 3, 1, uid, 16, 64, 0.3)
    assert (a == b).all()
    for other in (O.dropout_keep(6, 17, 3, 1, uid, 16, 64, 0.3), O.dropout_keep(5, 18, 3, 1, uid, 16, 64, 0.3),
                  O.dropout_keep(5, 17, 4, 1, uid, 16, 64, 0.3), O.dropout_keep(5, 17, 3, 2, uid, 16, 64, 0.3)):
        assert (a != other).mean() > 0.2
    big = O.dropout_keep(1, 2, 3, 0, np.arange(64), 32, 512, 0.3)         # ~1e6 draws
    n = big.size
    p_keep = 1.0 - O.dropout_threshold(0.3) / 65536.0
    assert abs(big.mean() - p_keep) < 4.0 * np.sqrt(p_keep * (1 - p_keep) / n)


def test_dropout_mask_independent_of_batch_split_and_padding():
    uid = np.array([10, 11, 12, 13])
    full = O.dropout_keep(9, 33, 2, 0, uid, 12, 40, 0.25).reshape(4, 12, 40)
    part = O.dropout_keep(9, 33, 2, 0, uid[2:], 7, 40, 0.25).reshape(2, 7, 40)
    assert (full[2:, :7] == part).all()


def test_dropout_column_to_word_mapping():
    # column c uses word (c>>1)&3, low half for even c, of counter group c>>3
    keep = O.dropout_keep(3, 5, 7, 2, np.array([4]), 3, 24, 0.4).reshape(3, 24)
    thr = O.dropout_threshold(0.4)
    for t in range(3):
        for c in range(24):
            w = O.philox4x32_10(np.array([c >> 3, 4, (5 << 16) | t, (7 << 8) | 2]), (3, 0))
            u = (int(w[(c >> 1) & 3]) >> (16 * (c & 1))) & 0xFFFF
            assert keep[t, c] == (u >= thr)
