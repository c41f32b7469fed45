"""Pins for oracle/replay.py: bounded FIFO semantics by brute force."""
from collections import deque

import numpy as np

from oracle import replay


def _rows(lo, n, O=3, A=2):
    base = np.arange(lo, lo + n, dtype=np.float32)
    return dict(obs=np.repeat(base[:, None], O, 1), act=np.repeat(base[:, None] + 0.25, A, 1),
                rew=base + 0.5, done=(base % 2), next_obs=np.repeat(base[:, None] + 0.75, O, 1))


def test_fifo_overwrites_oldest_and_keeps_order():
    cap = 10
    buf = replay.ReplayBuffer(cap, 3, 2)
    model = deque(maxlen=cap)
    slot_of = {}
    lo, cursor = 0, 0
    for n in (4, 3, 5, 1, 10, 13, 25, 2):
        buf.insert(**_rows(lo, n))
        for v in range(lo, lo + n):
            model.append(v)
            slot_of[v] = cursor
            cursor = (cursor + 1) % cap
        lo += n
        assert buf.count == len(model)
        assert buf.cursor == cursor
        # every live transition sits in the slot it was written to; others are gone
        for v in model:
            s, a, r, d, s2 = buf.gather([slot_of[v]])
            assert s[0, 0] == v and a[0, 1] == v + 0.25 and r[0] == v + 0.5 and d[0] == v % 2 and s2[0, 2] == v + 0.75
        assert sorted(buf.rows[:buf.count, 0].tolist()) == sorted(float(v) for v in model)


def test_row_layout_is_obs_act_rew_done_next_obs():
    buf = replay.ReplayBuffer(4, 3, 2)
    buf.insert(**_rows(7, 1))
    assert buf.rows[0].tolist() == [7, 7, 7, 7.25, 7.25, 7.5, 1.0, 7.75, 7.75, 7.75]
