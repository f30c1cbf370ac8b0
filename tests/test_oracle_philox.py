"""Pins for the oracle's random numbers: Philox4x32-10 known answers, the counter/key
layout of a (session, position, step) block, and the map from a word to r in [0,1)."""
import os

import numpy as np
from scipy import stats

from oracle import oracle as O


def _kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers(golden_dir):
    rows = _kat(golden_dir)
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = O.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want


def test_block_layout_is_session_position_step_under_seed():
    seed, step = 0x0123456789ABCDEF, 0xFEDCBA9876543210
    got = O.random_block(seed, step, session=7, position=3)
    want = O.philox4x32_10([7, 3, step & 0xFFFFFFFF, step >> 32], [seed & 0xFFFFFFFF, seed >> 32])
    assert (got == want).all()
    # each of the four coordinates changes the block
    base = O.random_block(1, 2, 3, 4)
    for other in (O.random_block(9, 2, 3, 4), O.random_block(1, 9, 3, 4), O.random_block(1, 2, 9, 4),
                  O.random_block(1, 2, 3, 9), O.random_block(1 << 32 | 1, 2, 3, 4),
                  O.random_block(1, 1 << 32 | 2, 3, 4)):
        assert (base != other).any()


def test_u01_is_top_24_bits():
    assert O.u01(0) == 0.0
    assert O.u01(0xFF) == 0.0
    assert O.u01(0x100) == 2.0 ** -24
    assert O.u01(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    assert O.u01(0x80000000) == 0.5


def test_words_are_uniform_and_blocks_distinct():
    words = np.array([O.random_block(11, step, b, i) for step in range(8) for b in range(64)
                      for i in range(16)], dtype=np.uint32)
    assert len({tuple(w) for w in words.tolist()}) == words.shape[0]
    for col in range(4):
        r = (words[:, col] >> 8).astype(np.float64) / 2 ** 24
        assert abs(r.mean() - 0.5) < 5 * (1 / 12 / r.size) ** 0.5
        counts = np.bincount((words[:, col] >> 24).astype(np.int64), minlength=256)
        assert stats.chisquare(counts).pvalue > 1e-4
    # accept, residual and bonus uniforms of one block must not be tied to one another
    r0 = (words[:, 0] >> 8).astype(np.float64)
    for col in (1, 2):
        rc = (words[:, col] >> 8).astype(np.float64)
        assert abs(np.corrcoef(r0, rc)[0, 1]) < 5 / r0.size ** 0.5
