"""Per-agent replay buffer for the oracle (test infrastructure only).

Sec. 1 / App. A of the paper: transitions go into a bounded buffer in
first-in-first-out order, one buffer per agent when data must not mix.
A row is [obs (O), act (A), reward, done, next_obs (O)] in float32.

Pins: tests/test_oracle_replay.py (overwrite order after wrap-around, brute
force against a Python deque).
"""
import numpy as np


class ReplayBuffer:
    def __init__(self, capacity, obs_dim, act_dim):
        self.capacity = int(capacity)
        self.obs_dim = obs_dim
        self.act_dim = act_dim
        self.rows = np.zeros((self.capacity, 2 * obs_dim + act_dim + 2), dtype=np.float32)
        self.cursor = 0
        self.count = 0

    def insert(self, obs, act, rew, done, next_obs):
        """Append n transitions; the oldest are overwritten once full."""
        obs = np.asarray(obs, dtype=np.float32).reshape(-1, self.obs_dim)
        n = obs.shape[0]
        block = np.concatenate([
            obs,
            np.asarray(act, dtype=np.float32).reshape(n, self.act_dim),
            np.asarray(rew, dtype=np.float32).reshape(n, 1),
            np.asarray(done, dtype=np.float32).reshape(n, 1),
            np.asarray(next_obs, dtype=np.float32).reshape(n, self.obs_dim)], axis=1)
        off = 0
        while off < n:                          # contiguous pieces, in arrival order
            seg = min(n - off, self.capacity - self.cursor)
            self.rows[self.cursor:self.cursor + seg] = block[off:off + seg]
            self.cursor = (self.cursor + seg) % self.capacity
            off += seg
        self.count = min(self.count + n, self.capacity)

    def gather(self, idx):
        """Rows at idx, split into (s, a, r, d, s2)."""
        O, A = self.obs_dim, self.act_dim
        r = self.rows[np.asarray(idx)]
        return r[:, :O], r[:, O:O + A], r[:, O + A], r[:, O + A + 1], r[:, O + A + 2:]
