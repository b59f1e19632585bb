"""CPU-only pins of the policy oracle (utility, marginal utility drop, greedy per-tier choice; Design section of
the paper).  Pins that are not the oracle itself: a three-entry instance worked by hand, exact optima by
enumeration on tiny instances, the optimum of the linear relaxation from scipy's LP solver (the greedy must reach
it up to the one fractional step, as the textbook result the paper cites says), limits (no capacity, unlimited
capacity), monotonicity in capacity and in frequency, the two printed formulas evaluated literally."""
import numpy as np
import pytest
from scipy.optimize import linprog

from oracle import policy_ref as P

EVICT = P.EVICT


def hand_entries():
    return [P.Entry(2.0, [100, 50, 25], [1.0, 0.9, 0.5]),
            P.Entry(1.0, [80, 40], [1.0, 0.8]),
            P.Entry(1.0, [60, 20], [0.9, 0.1])]


def test_formulas_as_printed():
    # Utility = Freq * (alpha * Quality - size / Bandwidth)
    assert P.utility(3.0, 0.5, 0.8, 200.0, 100.0) == 3.0 * (0.5 * 0.8 - 2.0)
    # marginal utility drop = (U(i,m) - U(i,n)) / (size(i) * (m - n)), m and n as fractions of the full size
    full, m, n = 1000.0, 0.5, 0.125
    assert P.marginal_utility_drop(7.0, 4.0, full * m, full * n) == (7.0 - 4.0) / (full * (m - n))


def test_three_entries_worked_by_hand():
    # alpha = 1, bandwidth = 100.  Utilities: A [0, 0.8, 0.5], B [0.2, 0.4], C [0.3, -0.1].
    # Start (largest utility): A at 50 bytes, B at 40, C at 60 = 150 bytes.
    e = hand_entries()
    assert [round(u, 12) for u in P.entry_utilities(e[0], 1.0, 100.0)] == [0.0, 0.8, 0.5]
    assert [round(u, 12) for u in P.entry_utilities(e[2], 1.0, 100.0)] == [0.3, -0.1]
    c, u, used = P.solve_tier(e, 1.0, 100.0, 1000.0)
    assert c == [1, 1, 0] and used == 150 and abs(u - 1.5) < 1e-12
    # capacity 100: drops A->25B 0.012, A->evict 0.016, B->evict 0.010, C->20B 0.010, C->evict 0.005: C goes
    c, u, used = P.solve_tier(e, 1.0, 100.0, 100.0)
    assert c == [1, 1, EVICT] and used == 90 and abs(u - 1.2) < 1e-12
    # capacity 60: next smallest is B->evict (0.010)
    c, u, used = P.solve_tier(e, 1.0, 100.0, 60.0)
    assert c == [1, EVICT, EVICT] and used == 50 and abs(u - 0.8) < 1e-12
    # capacity 30: A->25B (0.012) before A->evict (0.016)
    c, u, used = P.solve_tier(e, 1.0, 100.0, 30.0)
    assert c == [2, EVICT, EVICT] and used == 25 and abs(u - 0.5) < 1e-12
    c, u, used = P.solve_tier(e, 1.0, 100.0, 0.0)
    assert c == [EVICT] * 3 and used == 0 and u == 0
    for cap, want in ((100.0, 1.2), (60.0, 0.8), (30.0, 0.5)):
        assert abs(P.brute_force_tier(e, 1.0, 100.0, cap)[0] - want) < 1e-12


def random_entries(rng, n, max_choices=4, stored=False):
    out = []
    for _ in range(n):
        k = int(rng.integers(1, max_choices + 1))
        full = float(rng.integers(50, 400))
        rates = np.sort(rng.choice([1.0, 0.53, 0.27, 0.14, 0.07], size=k, replace=False))[::-1]
        sens = rng.uniform(0.2, 3.0)
        q = [float(1.0 - (1.0 - r) ** 2 * rng.uniform(0.0, 0.6) * sens / 3) for r in rates]
        out.append(P.Entry(float(rng.uniform(0.1, 5.0)), [full * r for r in rates], q,
                           int(rng.integers(0, k)) if stored else 0))
    return out


def lp_optimum(entries, alpha, bandwidth, capacity):
    cols, owner = [], []
    for i, e in enumerate(entries):
        for j in range(e.min_choice, len(e.sizes)):
            cols.append((P.utility(e.freq, alpha, e.qualities[j], e.sizes[j], bandwidth), e.sizes[j]))
            owner.append(i)
    A = np.zeros((len(entries) + 1, len(cols)))
    for k, (u, s) in enumerate(cols):
        A[owner[k], k] = 1.0
        A[-1, k] = s
    b = np.concatenate([np.ones(len(entries)), [capacity]])
    res = linprog(-np.array([u for u, _ in cols]), A_ub=A, b_ub=b, bounds=(0, 1), method="highs")
    assert res.status == 0
    return -res.fun


@pytest.mark.parametrize("stored", [False, True])
def test_greedy_against_enumeration_and_the_linear_relaxation(stored):
    rng = np.random.default_rng(7 + stored)
    hits = 0
    for trial in range(150):
        entries = random_entries(rng, int(rng.integers(1, 7)), stored=stored)
        alpha, bw = float(rng.uniform(0.3, 3.0)), float(rng.uniform(100, 2000))
        full = sum(e.sizes[e.min_choice] for e in entries)
        cap = float(rng.uniform(0.0, 1.1)) * full
        c, u, used = P.solve_tier(entries, alpha, bw, cap)
        assert used <= cap + 1e-9
        for i, j in enumerate(c):
            assert j == EVICT or entries[i].min_choice <= j < len(entries[i].sizes)
        opt, _ = P.brute_force_tier(entries, alpha, bw, cap)
        lp = lp_optimum(entries, alpha, bw, cap)
        assert u <= opt + 1e-9 <= lp + 2e-9
        # the greedy is the LP solution with its one fractional step rounded down: the gap is below one entry's range
        spread = max(max(0.0, max(P.entry_utilities(e, alpha, bw)[e.min_choice:])) for e in entries)
        assert lp - u <= spread + 1e-9
        hits += abs(u - opt) < 1e-9
    assert hits > 90  # and it is exactly optimal most of the time on such instances


def test_greedy_plus_the_fractional_step_is_the_lp_optimum():
    # Redo the last step fractionally: utility + drop * (capacity - used) must equal the LP optimum.
    rng = np.random.default_rng(3)
    checked = 0
    for trial in range(120):
        entries = random_entries(rng, int(rng.integers(2, 8)))
        alpha, bw = 1.0, float(rng.uniform(200, 1500))
        c_all, u_all, used_all = P.solve_tier(entries, alpha, bw, float("inf"))
        cap = float(rng.uniform(0.05, 0.95)) * used_all
        c, u, used = P.solve_tier(entries, alpha, bw, cap)
        # find the last step by solving with the capacity just above what the final state freed
        lo, hi = used, used_all
        # the state before the last step is the solution at the smallest capacity that is still > cap
        caps = sorted({P.solve_tier(entries, alpha, bw, x)[2] for x in np.linspace(cap, used_all, 400)})
        before = [x for x in caps if x > cap]
        if not before:
            continue
        c_b, u_b, used_b = P.solve_tier(entries, alpha, bw, before[0])
        if used_b <= cap or used_b == used:
            continue
        drop = (u_b - u) / (used_b - used)
        lp = lp_optimum(entries, alpha, bw, cap)
        assert abs(u + drop * (cap - used) - lp) <= 1e-7 * max(1.0, abs(lp)), trial
        checked += 1
    assert checked > 60


def test_limits_and_monotonicity():
    rng = np.random.default_rng(11)
    for trial in range(40):
        entries = random_entries(rng, 6)
        alpha, bw = 1.5, 800.0
        c_inf, u_inf, used_inf = P.solve_tier(entries, alpha, bw, float("inf"))
        for i, e in enumerate(entries):  # unlimited capacity: every entry sits at its own best choice
            us = P.entry_utilities(e, alpha, bw)
            assert (c_inf[i] == EVICT and max(us) <= 0) or us[c_inf[i]] == max(us)
        assert P.solve_tier(entries, alpha, bw, 0.0)[0] == [EVICT] * 6
        last = -1.0
        for cap in np.linspace(0, used_inf, 15):
            _, u, used = P.solve_tier(entries, alpha, bw, float(cap))
            assert used <= cap + 1e-9 and u >= last - 1e-12
            last = u
        # scaling every frequency by the same factor changes no decision
        scaled = [P.Entry(e.freq * 4.0, e.sizes, e.qualities, e.min_choice) for e in entries]
        cap = 0.4 * used_inf
        assert P.solve_tier(scaled, alpha, bw, cap)[0] == P.solve_tier(entries, alpha, bw, cap)[0]


def test_hotter_copy_of_an_entry_is_never_stored_worse():
    rng = np.random.default_rng(5)
    for trial in range(40):
        base = random_entries(rng, 5)
        twin = P.Entry(base[0].freq * 3.0, base[0].sizes, base[0].qualities)
        entries = base + [twin]
        full = sum(e.sizes[0] for e in entries)
        for frac in (0.2, 0.5, 0.8):
            c, _, _ = P.solve_tier(entries, 1.0, 600.0, frac * full)
            cold, hot = c[0], c[-1]
            rank = lambda j: len(twin.sizes) if j == EVICT else j  # larger = worse
            assert rank(hot) <= rank(cold)


def test_two_tiers_cascade():
    e = hand_entries()
    # DRAM: bandwidth 100, capacity 60 keeps A at 50 B (see above); B and C are offered to the slow tier
    # (bandwidth 50): B [1-1.6, 0.8-0.8] = [-0.6, 0.0] -> evict (no gain); C [0.9-1.2, 0.1-0.4] -> evict.
    tier, choice, total = P.plan(e, 1.0, [(100.0, 60.0), (50.0, 1000.0)])
    assert tier == [0, -1, -1] and choice == [1, EVICT, EVICT] and abs(total - 0.8) < 1e-12
    # with a faster second tier (bandwidth 100) both find room there at their best choices
    tier, choice, total = P.plan(e, 1.0, [(100.0, 60.0), (100.0, 1000.0)])
    assert tier == [0, 1, 1] and choice == [1, 1, 0] and abs(total - 1.5) < 1e-12


def test_stored_entries_cannot_regain_quality():
    e = hand_entries()
    e[0].min_choice = 2  # A is already held at 25 bytes
    c, u, used = P.solve_tier(e, 1.0, 100.0, 1000.0)
    assert c == [2, 1, 0] and used == 125
