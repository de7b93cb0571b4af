"""CPU oracle of the paper's load-balancing placement -- TEST INFRASTRUCTURE ONLY.

Written from Sec. 7 ("Load Balancing").  Historical expert activation is a matrix A[m][b]: the
fraction of the tokens of batch b that went to expert m.  A placement puts every expert on one
of D devices, the same number E/D on each.  (The objective printed in the paper is garbled; what
the text describes and what is implemented: keep the per-batch device load  sum_m P[m][n] A[m][b]
close to 1/D, under  sum_m P[m][n] = E/D  for every device n.)

* Greedy (Sec. 7.1): experts in descending order of their average historical load; each goes to
  the device with the smallest load so far (the sum of the average loads of its experts); a device
  that holds E/D experts leaves the candidates.
* Anti-correlation (Sec. 7.2): same walk, but the load a device n offers to the current expert a is
  sum over its experts m of (mean_m + 0.5 * S[a][m]),  S = Pearson correlation of the two experts'
  historical activations.
* Evaluation: Max Load = the largest device share over all batches and devices; Avg Max Load = the
  largest device share per batch, averaged over the batches.

Conventions the paper leaves open: equal average loads keep the lower expert id first; equal device
loads go to the lower device id; an expert whose activation never varies has correlation 0 with
everyone; sums run in index order in double precision.  Plain Python loops on purpose.
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple


def mean_load(A: Sequence[Sequence[float]]) -> List[float]:
    out = []
    for row in A:
        s = 0.0
        for v in row:
            s += float(v)
        out.append(s / len(row) if len(row) else 0.0)
    return out


def pearson(A: Sequence[Sequence[float]]) -> List[List[float]]:
    E = len(A)
    B = len(A[0]) if E else 0
    mu = mean_load(A)
    dev = [[float(A[m][b]) - mu[m] for b in range(B)] for m in range(E)]
    ss = []
    for m in range(E):
        s = 0.0
        for b in range(B):
            s += dev[m][b] * dev[m][b]
        ss.append(s)
    S = [[0.0] * E for _ in range(E)]
    for a in range(E):
        for m in range(E):
            if ss[a] > 0.0 and ss[m] > 0.0:
                c = 0.0
                for b in range(B):
                    c += dev[a][b] * dev[m][b]
                S[a][m] = c / math.sqrt(ss[a] * ss[m])
    return S


def _walk(A, n_devices: int, corr_weight: float) -> List[int]:
    E = len(A)
    if n_devices < 1 or E % n_devices != 0:
        raise ValueError("the experts must split evenly over the devices")
    cap = E // n_devices
    mu = mean_load(A)
    S = pearson(A) if corr_weight != 0.0 else None
    order = sorted(range(E), key=lambda m: (-mu[m], m))
    members: List[List[int]] = [[] for _ in range(n_devices)]
    device_of = [-1] * E
    for a in order:
        best, best_load = -1, 0.0
        for n in range(n_devices):
            if len(members[n]) >= cap:
                continue
            load = 0.0
            for m in members[n]:
                load += mu[m] + (corr_weight * S[a][m] if S is not None else 0.0)
            if best < 0 or load < best_load:
                best, best_load = n, load
        members[best].append(a)
        device_of[a] = best
    return device_of


def greedy(A, n_devices: int) -> List[int]:
    return _walk(A, n_devices, 0.0)


def anticorrelation(A, n_devices: int, corr_weight: float = 0.5) -> List[int]:
    return _walk(A, n_devices, corr_weight)


def loads(A, device_of: Sequence[int], n_devices: int) -> Tuple[float, float]:
    """(Max Load, Avg Max Load) of a placement on activation data A."""
    E = len(A)
    B = len(A[0]) if E else 0
    worst, acc = 0.0, 0.0
    for b in range(B):
        dev = [0.0] * n_devices
        for m in range(E):
            dev[device_of[m]] += float(A[m][b])
        mx = max(dev)
        worst = max(worst, mx)
        acc += mx
    return worst, (acc / B if B else 0.0)


def best_max_load(A, n_devices: int) -> float:
    """Smallest possible Max Load over every balanced placement (exhaustive; tiny inputs only)."""
    E = len(A)
    cap = E // n_devices
    best = [float("inf")]
    device_of = [-1] * E
    fill = [0] * n_devices

    def go(m: int) -> None:
        if m == E:
            best[0] = min(best[0], loads(A, device_of, n_devices)[0])
            return
        for n in range(n_devices):
            if fill[n] < cap:
                if fill[n] == 0 and any(fill[q] == 0 for q in range(n)):
                    continue  # devices are interchangeable: open them in order
                fill[n] += 1
                device_of[m] = n
                go(m + 1)
                fill[n] -= 1
        device_of[m] = -1

    go(0)
    return best[0]
