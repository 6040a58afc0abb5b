"""Set-based brute-force simulator of H2O (or Lambda-masking) + LESS for tiny inputs.

TEST INFRASTRUCTURE ONLY.  A second, deliberately different statement of the
same semantics as oracle/less_oracle.c, used to pin it:

* it keeps the whole token history and explicit index sets (no slots, no
  in-place replacement, no recursion for the state);
* Eq. 3 is evaluated exactly as printed, without any shift (inputs are tiny);
* H and z are rebuilt at every step from the closed form of Eq. 6, i.e. the
  sum over every pair discarded so far;
* feature maps use numpy matmuls and scipy's erf.

Pure numpy, O(n) scans everywhere: only for small cases.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf


def _gelu(x):
    return x * 0.5 * (1.0 + erf(x / np.sqrt(2.0)))


def phi(q, Wq1, Wq2):
    """Eq. 1."""
    return np.abs(_gelu(_gelu(q @ Wq1) @ Wq2))


def psi(k, Wk1, Wk2, Wk3):
    """Eq. 2."""
    return np.abs(_gelu(_gelu(k @ Wk1) @ Wk2) @ Wk3)


class BruteForceUnit:
    def __init__(self, head_dim, n_heavy, n_recent, W, sparse_denominator=False, policy="h2o",
                 q_per_kv=1):
        """q_per_kv = G > 1: the unit has G query heads sharing keys, values, cache and state;
        then W["Wq1"], W["Wq2"] carry a leading axis G, step() takes q [G,D] and prefill() Q
        [G,P,D], and outputs have the same leading axis."""
        assert policy in ("h2o", "lambda")
        self.policy = policy
        self.G = q_per_kv
        self.D, self.Nh, self.Nr = head_dim, n_heavy, n_recent
        self.W = {k: np.asarray(v, dtype=np.float64) for k, v in W.items()}
        self.sparse_denominator = sparse_denominator
        self.keys, self.values = [], []          # full history, index = position
        self.alive = set()                       # positions in the sparse cache
        self.score = {}                          # position -> accumulated probability
        self.discarded = []                      # positions, in order of eviction

    # Eq. 6: the state is the sum over everything discarded so far
    def state(self):
        R = self.W["Wk3"].shape[0]
        H = np.zeros((R, self.D)); z = np.zeros(R)
        for p in self.discarded:
            g = psi(self.keys[p], self.W["Wk1"], self.W["Wk2"], self.W["Wk3"])
            H += np.outer(g, self.values[p]); z += g
        return H, z

    def prefill(self, Q, K, V):
        Q, K, V = (np.asarray(a, dtype=np.float64) for a in (Q, K, V))
        P = K.shape[0]
        Qs = Q[None] if self.G == 1 else Q
        col = np.zeros(P); outs = []
        for Qg in Qs:                                           # every query head of the unit
            S = Qg @ K.T / np.sqrt(self.D)
            S[np.triu_indices(P, 1)] = -np.inf
            A = np.exp(S - S.max(axis=1, keepdims=True))
            A /= A.sum(axis=1, keepdims=True)
            col += A.sum(axis=0)                                # attention mass from all heads
            outs.append(A @ V)
        self.keys = [K[i] for i in range(P)]; self.values = [V[i] for i in range(P)]
        C = self.Nh + self.Nr
        if P <= C:
            self.alive = set(range(P))
        else:
            recent = set(range(P - self.Nr, P))
            rest = [p for p in range(P) if p not in recent]
            if self.policy == "lambda":
                heavy = set(range(self.Nh))          # the first tokens of the sequence
            else:
                rest.sort(key=lambda p: (col[p], p))
                heavy = set(rest[len(rest) - self.Nh:]) if self.Nh else set()
            self.alive = recent | heavy
            self.discarded = sorted(set(rest) - heavy)
        self.score = {p: col[p] for p in self.alive}
        return outs[0] if self.G == 1 else np.stack(outs)

    def step(self, q, k, v):
        q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
        n = len(self.keys)
        H, z = self.state()
        self.keys.append(k); self.values.append(v)
        members = sorted(self.alive) + [n]                      # K', V' of Eq. 3
        outs = []
        for g in range(self.G):                                 # every query head of the unit
            qg = q if self.G == 1 else q[g]
            Wq1, Wq2 = (self.W["Wq1"], self.W["Wq2"]) if self.G == 1 else (self.W["Wq1"][g], self.W["Wq2"][g])
            f = phi(qg, Wq1, Wq2)
            w = {p: np.exp(qg @ self.keys[p] / np.sqrt(self.D)) for p in members}
            num = f @ H + sum(w[p] * self.values[p] for p in members)
            den_sparse = sum(w[p] for p in members)
            den = f @ z + den_sparse
            outs.append(num / den)
            d = den_sparse if self.sparse_denominator else den
            for p in members:
                self.score[p] = self.score.get(p, 0.0) + w[p] / d
        out = outs[0] if self.G == 1 else np.stack(outs)
        self.alive.add(n)
        evicted = -1
        if len(self.alive) > self.Nh + self.Nr:
            newest = sorted(self.alive)[len(self.alive) - self.Nr:] if self.Nr else []
            cand = [p for p in self.alive if p not in newest]
            if self.policy == "lambda":
                evicted = min(p for p in cand if p >= self.Nh or p == n)
            else:
                evicted = min(cand, key=lambda p: (self.score[p], p))
            self.alive.remove(evicted); del self.score[evicted]
            self.discarded.append(evicted)
        return out, evicted
