"""Plain reference of the partition solver (Sec. 3.2.1, "Partition Optimization Solver").

TEST INFRASTRUCTURE ONLY.  An expert's C intermediate neurons are split into S equal groups so
that, token by token, the activation mass concentrates in few groups.  With the calibration
activations A [B, C], L[b, n] = sum over the neurons of group n of |A[b, c]|, and
K_drop = S - k_in groups expected to be skipped, the objective (Eq. 4) is

    loss(P) = sum_b (sum of the K_drop smallest of L[b, 0..S-1]).

Two-stage heuristic, as described:
  greedy   neurons are ranked by their calibration-wide L1 norm (descending; equal norms by
           ascending index) and each goes to the group with the smallest accumulated norm among
           those that still have room (equal sums: the lower group index);
  anneal   neurons of two different groups are swapped (sizes stay equal); a swap that does
           not raise the loss is kept, one that raises it by D is kept with probability
           exp(-D / temp), temp falling geometrically from t0 to t1 over the steps.

Readings where the text is silent: the proposal stream is a counter-based generator
(splitmix64 of seed + 3*step + {0, 1, 2}) so that both implementations draw the same swaps:
neuron i = r0 mod C, neuron j = r1 mod C, a proposal with both in one group is skipped (it
still consumes its step); the acceptance draw is u = (r2 >> 11) * 2^-53; all sums are
binary64.  The reference recomputes Eq. 4 from scratch for every proposal; the library keeps
the group sums L and updates them per kept swap, so the two agree exactly only where every
sum is exact in binary64 (the exact-equality test uses dyadic activations for that reason) and
to rounding elsewhere.
"""
from __future__ import annotations

import math

import numpy as np

MASK = (1 << 64) - 1


def splitmix64(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & MASK
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


def group_mass(A, group_of, S):
    """L [B, S] in binary64, neurons added in ascending index order."""
    B, C = A.shape
    L = np.zeros((B, S), np.float64)
    for c in range(C):
        L[:, group_of[c]] += np.abs(A[:, c].astype(np.float64))
    return L


def drop_sum(row, k_drop):
    """Sum of the k_drop smallest entries, smallest first."""
    s = 0.0
    for v in sorted(row)[:k_drop]:
        s += v
    return s


def objective(A, group_of, S, k_in):
    L = group_mass(A, group_of, S)
    total = 0.0
    for b in range(A.shape[0]):
        total += drop_sum(L[b].tolist(), S - k_in)
    return total


def greedy(A, S):
    B, C = A.shape
    assert C % S == 0
    norm = [0.0] * C
    for c in range(C):
        s = 0.0
        for b in range(B):
            s += abs(float(A[b, c]))
        norm[c] = s
    order = sorted(range(C), key=lambda c: (-norm[c], c))
    acc = [0.0] * S
    size = [0] * S
    group_of = np.empty(C, np.int32)
    for c in order:
        best = -1
        for n in range(S):
            if size[n] < C // S and (best < 0 or acc[n] < acc[best]):
                best = n
        group_of[c] = best
        acc[best] += norm[c]
        size[best] += 1
    return group_of


def anneal(A, group_of, S, k_in, steps, t0, t1, seed):
    """Returns (group_of, loss).  group_of is not modified in place.

    Written as the definition: the loss of the current and of every proposed partition is Eq. 4
    evaluated from scratch (objective()); nothing is carried from one step to the next but the
    partition itself."""
    C = A.shape[1]
    g = np.array(group_of, np.int32)
    loss = objective(A, g, S, k_in)
    for step in range(steps):
        r0 = splitmix64((seed + 3 * step) & MASK)
        r1 = splitmix64((seed + 3 * step + 1) & MASK)
        r2 = splitmix64((seed + 3 * step + 2) & MASK)
        i, j = r0 % C, r1 % C
        if g[i] == g[j]:
            continue
        temp = t0 * (t1 / t0) ** (step / (steps - 1)) if steps > 1 else t0
        proposal = g.copy()
        proposal[i], proposal[j] = g[j], g[i]
        new_loss = objective(A, proposal, S, k_in)
        delta = new_loss - loss
        u = (r2 >> 11) * (1.0 / 9007199254740992.0)
        if delta <= 0.0 or u < math.exp(-delta / temp):
            g, loss = proposal, new_loss
    return g, loss
