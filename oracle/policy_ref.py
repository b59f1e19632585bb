"""Reference implementation of the storage policy (test infrastructure only: imported by tests/ and by
bench.py's cpu_baseline leg, never by the product path).

Follows the paper's Design section in its own order and notation, in float64, with plain loops:

  Utility(i) = Freq(i) * (alpha * Quality(i, M_i, R_i) - size(i, M_i, R_i) / Bandwidth)
  marginal utility drop = (Utility(i, m) - Utility(i, n)) / (size(i) * (m - n))
  per storage tier, greedily take the compression choice (evict, full quality, compress) with the
  minimal marginal utility drop until the tier's capacity holds what is left.

Readings taken where the paper is silent or garbled (each repeated where it is used):
  P1  the utility formula is printed with its last parenthesis missing; it closes after the fraction.
  P2  m and n are rates expressed as fractions of the entry's full size, so size(i) * (m - n) is the
      number of bytes the step frees: size(i, m) - size(i, n).
  P3  an evicted entry occupies no space and has utility 0 in that tier.
  P4  an entry starts at the allowed choice with the largest utility (the smallest such choice on ties);
      a stored entry can only move to choices that are not better than the one it is held at.
  P5  a step may go from the current choice to ANY smaller choice or to eviction, not only to the next one;
      taking the minimal drop over all of them walks the upper convex hull of (size, utility), which is
      what makes the greedy reach the optimum of the linear relaxation (the textbook result the paper cites).
  P6  ties: smaller drop first, then the lower entry index, then the larger remaining size.
  P7  tiers are filled in order: what tier t evicts is offered to tier t + 1 with that tier's bandwidth.
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

EVICT = -1


@dataclass
class Entry:
    freq: float
    sizes: Sequence[float]      # bytes of each choice, strictly decreasing (choice 0 = full quality)
    qualities: Sequence[float]  # quality of each choice
    min_choice: int = 0         # choices below this index are no longer available (the entry is stored at it)


def utility(freq: float, alpha: float, quality: float, size: float, bandwidth: float) -> float:
    """Utility of one entry under one choice (Design section, utility definition; reading P1)."""
    return freq * (alpha * quality - size / bandwidth)


def marginal_utility_drop(u_m: float, u_n: float, size_m: float, size_n: float) -> float:
    """Utility lost per byte freed by going from the choice of size size_m to the smaller one (reading P2)."""
    return (u_m - u_n) / (size_m - size_n)


def entry_utilities(e: Entry, alpha: float, bandwidth: float) -> List[float]:
    return [utility(e.freq, alpha, q, s, bandwidth) for q, s in zip(e.qualities, e.sizes)]


def start_choice(e: Entry, u: Sequence[float]) -> int:
    """Reading P4 (and P3: eviction, utility 0, wins unless some allowed choice is strictly better)."""
    best, best_u = EVICT, 0.0
    for j in range(e.min_choice, len(e.sizes)):
        if u[j] > best_u or (u[j] == best_u and best != EVICT):
            best, best_u = j, u[j]  # a later choice is smaller: on ties the smaller one stays
    return best


def solve_tier(entries: Sequence[Entry], alpha: float, bandwidth: float, capacity: float,
               active: Optional[Sequence[bool]] = None) -> Tuple[List[int], float, float]:
    """One storage tier: -> (choice per entry or EVICT, total utility, bytes used).  Entries with
    active[i] == False are not offered to this tier and come back as EVICT."""
    n = len(entries)
    us = [entry_utilities(e, alpha, bandwidth) for e in entries]
    cur = [start_choice(entries[i], us[i]) if (active is None or active[i]) else EVICT for i in range(n)]

    def size_of(i):
        return 0.0 if cur[i] == EVICT else float(entries[i].sizes[cur[i]])

    def util_of(i):
        return 0.0 if cur[i] == EVICT else us[i][cur[i]]

    used = sum(size_of(i) for i in range(n))
    while used > capacity:
        best = None  # (drop, entry, -remaining size, target)
        for i in range(n):
            if cur[i] == EVICT:
                continue
            s_m, u_m = size_of(i), util_of(i)
            targets = [(j, float(entries[i].sizes[j]), us[i][j]) for j in range(cur[i] + 1, len(entries[i].sizes))]
            targets.append((EVICT, 0.0, 0.0))
            for j, s_n, u_n in targets:
                key = (marginal_utility_drop(u_m, u_n, s_m, s_n), i, -s_n)
                if best is None or key < best[0]:
                    best = (key, j)
        if best is None:
            break  # everything is evicted already
        (_, i, _), j = best
        used -= size_of(i)
        cur[i] = j
        used += size_of(i)
        # re-sum to keep `used` free of accumulated rounding: sizes are what decides feasibility
        used = sum(size_of(k) for k in range(n))
    total = 0.0
    for i in range(n):
        total += util_of(i)
    return cur, total, used


def plan(entries: Sequence[Entry], alpha: float, tiers: Sequence[Tuple[float, float]]):
    """Cascade over tiers [(bandwidth, capacity), ...] (reading P7): -> (tier per entry or -1, choice per entry
    or EVICT, total utility)."""
    n = len(entries)
    tier_of, choice_of = [-1] * n, [EVICT] * n
    waiting = [True] * n
    total = 0.0
    for t, (bandwidth, capacity) in enumerate(tiers):
        cur, _, _ = solve_tier(entries, alpha, bandwidth, capacity, active=waiting)
        for i in range(n):
            if waiting[i] and cur[i] != EVICT:
                tier_of[i], choice_of[i], waiting[i] = t, cur[i], False
    for i in range(n):
        if tier_of[i] >= 0:
            total += utility(entries[i].freq, alpha, entries[i].qualities[choice_of[i]], entries[i].sizes[choice_of[i]],
                             tiers[tier_of[i]][0])
    return tier_of, choice_of, total


def brute_force_tier(entries: Sequence[Entry], alpha: float, bandwidth: float, capacity: float):
    """Exact optimum of one tier by enumeration (tiny instances only): -> (best total utility, choices)."""
    us = [entry_utilities(e, alpha, bandwidth) for e in entries]
    options = [[EVICT] + list(range(e.min_choice, len(e.sizes))) for e in entries]
    best_u, best_c = 0.0, [EVICT] * len(entries)
    for combo in itertools.product(*options):
        size = sum(0.0 if j == EVICT else entries[i].sizes[j] for i, j in enumerate(combo))
        if size > capacity:
            continue
        u = sum(0.0 if j == EVICT else us[i][j] for i, j in enumerate(combo))
        if u > best_u:
            best_u, best_c = u, list(combo)
    return best_u, best_c
