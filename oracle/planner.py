"""Oracle of the decoupled-execution planner (test infrastructure only).

Follows the paper's Section 4.1 ("Modeling TGS" and Algorithm 1), in its order
and notation, in plain Python floats (IEEE double):

  D_{g_d}(b)   = b * D'_{g_d} + alpha_{g_d}           draft time of one token for a batch of b
  V_{g_v,w}(b) = b * V'_{g_v,w} + beta_{g_v,w}        verification time of a window of w drafts
  IL(b)        = max{ w * D(b), V(b) }                time to generate a window in decoupled execution
  P(a, w)      = p^a (1 - p)  for 0 <= a <= w-1,  p^w for a = w
  tau_w        = sum_{a=0}^{w-1} p^a (1-p) (a+1)/2  +  w p^w
  TGS(b)       = tau_w / IL(b)
  Algorithm 1: over every verifier configuration g_v of the given set, every drafter size g_d = 1..g_v
               (which fixes b = ceil((g_d + g_v) B / G)) and every window w = 1..w_max: the (g_d, g_v, w)
               with the largest TGS, the first of equals in that visiting order.

Readings (the text leaves these open; they are listed with the others in the design notes):
  * The side condition printed with P(a, w) names an `n` that appears nowhere else; it is read as w.
  * The printed bound w_max = max{ceil(V'_{g_v,w} / D'_{g_d}), ceil(beta_{g_v,w} / alpha_{g_d})} uses
    the parameters of the very window it bounds.  Here it is evaluated with the parameters of the
    largest profiled window W (the profile is a table over w = 1..W) and clipped to [1, W].
  * tau_w weights a partial accept of `a` drafts by (a+1)/2; the text does not say why.  It is taken
    as printed.

The affine parameters come from an offline profile; `fit_affine` is the ordinary least-squares line
through measured (b, time) points.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Sequence


def accept_prob(p: float, a: int, w: int) -> float:
    """P(a, w): exactly `a` of the w drafts of a window are accepted, each draft with probability p."""
    if not (0 <= a <= w) or w < 1:
        raise ValueError("need 0 <= a <= w, w >= 1")
    return p ** a * (1.0 - p) if a < w else p ** w


def tau(p: float, w: int) -> float:
    """Expected tokens generated per window of w drafts (the paper's tau_w)."""
    if w < 1:
        raise ValueError("w >= 1")
    partial = 0.0
    for a in range(w):
        partial += p ** a * (1.0 - p) * ((a + 1) / 2.0)
    return partial + w * p ** w


@dataclass(frozen=True)
class Affine:
    slope: float        # D' or V'
    icpt: float         # alpha or beta

    def __call__(self, b: float) -> float:
        return b * self.slope + self.icpt


def iteration_latency(w: int, D: Affine, V: Affine, b: float) -> float:
    return max(w * D(b), V(b))


def tgs(p: float, w: int, D: Affine, V: Affine, b: float) -> float:
    return tau(p, w) / iteration_latency(w, D, V, b)


def w_max(D: Affine, V_largest: Affine, W: int) -> int:
    cands = []
    if D.slope > 0:
        cands.append(math.ceil(V_largest.slope / D.slope))
    if D.icpt > 0:
        cands.append(math.ceil(V_largest.icpt / D.icpt))
    m = max(cands) if cands else W
    return max(1, min(W, m))


@dataclass(frozen=True)
class Plan:
    g_d: int
    g_v: int
    w: int
    tgs: float
    b: int


def deployments(B: int, G: int, verifier_configs: Sequence[int]):
    """Every (verifier configuration, drafter size) pair with the per-worker batch it implies, in visiting order:
    configurations as given, drafter sizes ascending."""
    for g_v in verifier_configs:
        for g_d in range(1, g_v + 1):
            yield g_d, g_v, -(-((g_d + g_v) * B) // G)        # ceil((g_d + g_v) B / G)


def plan_decoupled(B: int, G: int, p: float, verifier_configs: Sequence[int],
                   D_of: dict, V_of: dict, W: int) -> Plan:
    """What Algorithm 1 computes.  D_of[g_d] -> Affine for g_d = 1..max(verifier_configs);
    V_of[(g_v, w)] -> Affine for every g_v of verifier_configs and w = 1..W.  Every deployment is expanded
    into the windows 1..w_max worth trying; the candidate with the largest TGS wins (the first among equals,
    in visiting order); with no positive TGS the all-zero plan is returned."""
    candidates = [Plan(g_d, g_v, w, tgs(p, w, D_of[g_d], V_of[(g_v, w)], b), b)
                  for g_d, g_v, b in deployments(B, G, verifier_configs)
                  for w in range(1, w_max(D_of[g_d], V_of[(g_v, W)], W) + 1)]
    best = max(candidates, key=lambda c: c.tgs, default=None)  # max() keeps the first of equal keys
    return best if best is not None and best.tgs > 0.0 else Plan(0, 0, 0, 0.0, 0)


def best_window(p: float, D: Affine, V_of_w: Sequence[Affine], b: float) -> tuple:
    """argmax over w = 1..len(V_of_w) of the decoupled TGS at a given batch (Algorithm 2 evaluates this at
    b = 1 for a request whose acceptance rate p has drifted); the first of equal maxima wins."""
    best_w, best_t = 0, 0.0
    for w in range(1, len(V_of_w) + 1):
        t = tgs(p, w, D, V_of_w[w - 1], b)
        if t > best_t:
            best_w, best_t = w, t
    return best_w, best_t


def fit_affine(bs: Sequence[float], ts: Sequence[float]) -> Affine:
    """Least-squares line t = slope * b + icpt through the measured points."""
    n = len(bs)
    if n < 2 or n != len(ts):
        raise ValueError("need two or more points")
    mb = sum(bs) / n
    mt = sum(ts) / n
    sbb = sum((x - mb) * (x - mb) for x in bs)
    sbt = sum((x - mb) * (y - mt) for x, y in zip(bs, ts))
    if sbb == 0:
        raise ValueError("all batch sizes equal")
    slope = sbt / sbb
    return Affine(slope, mt - slope * mb)
