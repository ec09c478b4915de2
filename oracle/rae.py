"""CPU oracle for role-conditioned advantage estimation — TEST INFRASTRUCTURE.

Follows the policy-optimisation loop of Alg. 1 and the RAE equation of Sec. 3:
one exponential-moving-average baseline b[G][p] per game G and role p in {0,1},
initialised to 0; for every finished trajectory, in batch order and for both
roles, first b <- alpha*b + (1-alpha)*R_p, then A_p = R_p - b with the updated
b.  Rewards are zero-sum, R_1 = -R_0.  alpha = 0.95 is the paper's "EMA decay
rate" (hyper-parameter table, App. D).  float64 throughout.
"""
from __future__ import annotations

import numpy as np


class RAE:
    def __init__(self, n_games: int, alpha: float = 0.95):
        self.alpha = float(alpha)
        self.b = np.zeros((n_games, 2), dtype=np.float64)

    def update(self, game_id, r0):
        """Processes trajectories in array order; returns advantages [n, 2]."""
        game_id = np.asarray(game_id)
        r0 = np.asarray(r0, dtype=np.float64)
        adv = np.empty((r0.shape[0], 2), dtype=np.float64)
        for i in range(r0.shape[0]):
            G = int(game_id[i])
            for p in (0, 1):
                R = r0[i] if p == 0 else -r0[i]
                self.b[G, p] = self.alpha * self.b[G, p] + (1.0 - self.alpha) * R
                adv[i, p] = R - self.b[G, p]
        return adv
