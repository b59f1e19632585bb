"""The native storage policy (kvh_policy_* in libkvh.so; host only, runs without a GPU) against the Python oracle:
identical decisions and bit-identical utilities on the hand-worked instance, random instances with one to three
tiers, stored entries, ties, and a sweep of capacities; plus its argument errors."""
import ctypes

import numpy as np
import pytest

from oracle import policy_ref as P


@pytest.fixture(scope="module")
def kvh():
    import os

    from paper_2509_00105_amd import build

    if not os.path.exists(build.LIB):  # host-only code: compiling it needs no GPU
        build.build()
    import paper_2509_00105_amd as m

    m.lib()
    return m


def random_entries(rng, n, max_choices=5, stored=False, ties=False):
    out = []
    for _ in range(n):
        k = int(rng.integers(1, max_choices + 1))
        full = int(rng.integers(1000, 400000))
        rates = np.sort(rng.choice([1.0, 0.53, 0.27, 0.14, 0.07, 0.035], size=k, replace=False))[::-1]
        sizes = [float(max(16, int(full * r) // 16 * 16)) for r in rates]
        sizes = sorted(set(sizes), reverse=True)
        sens = rng.uniform(0.2, 3.0)
        q = [float(1.0 - (1.0 - s / sizes[0]) ** 2 * rng.uniform(0.0, 0.6) * sens / 3) for s in sizes]
        if ties:  # coarse values make equal utilities and equal drops common
            q = [round(x * 4) / 4 for x in q]
        freq = float(rng.integers(1, 4)) if ties else float(rng.uniform(0.0, 5.0))
        out.append(P.Entry(freq, sizes, q, int(rng.integers(0, len(sizes))) if stored else 0))
    return out


def native_plan(kvh, entries, alpha, tiers):
    return kvh.policy_plan([e.freq for e in entries], [e.sizes for e in entries], [e.qualities for e in entries], alpha,
                           tiers, [e.min_choice for e in entries])


def test_scalar_formulas_match(kvh):
    rng = np.random.default_rng(0)
    for _ in range(200):
        f, a, q, s, b = rng.uniform(0, 5), rng.uniform(0, 3), rng.uniform(0, 1), float(rng.integers(1, 10**9)), rng.uniform(1, 1e10)
        assert kvh.policy_utility(f, a, q, s, b) == P.utility(f, a, q, s, b)
        um, un, sn = rng.uniform(-5, 5), rng.uniform(-5, 5), float(rng.integers(0, 10**6))
        assert kvh.policy_marginal_utility_drop(um, un, sn + 64.0, sn) == P.marginal_utility_drop(um, un, sn + 64.0, sn)


def test_hand_worked_instance(kvh):
    e = [P.Entry(2.0, [100, 50, 25], [1.0, 0.9, 0.5]), P.Entry(1.0, [80, 40], [1.0, 0.8]), P.Entry(1.0, [60, 20], [0.9, 0.1])]
    for cap, want in ((1000.0, [1, 1, 0]), (100.0, [1, 1, -1]), (60.0, [1, -1, -1]), (30.0, [2, -1, -1]), (0.0, [-1, -1, -1])):
        tier, choice, total = native_plan(kvh, e, 1.0, [(100.0, cap)])
        assert choice.tolist() == want and tier.tolist() == [0 if c >= 0 else -1 for c in want]
        assert total == P.solve_tier(e, 1.0, 100.0, cap)[1]
    tier, choice, total = native_plan(kvh, e, 1.0, [(100.0, 60.0), (100.0, 1000.0)])
    assert tier.tolist() == [0, 1, 1] and choice.tolist() == [1, 1, 0]


@pytest.mark.parametrize("stored,ties", [(False, False), (True, False), (False, True), (True, True)])
def test_random_instances_match_the_oracle(kvh, stored, ties):
    rng = np.random.default_rng(100 + 2 * stored + ties)
    for trial in range(120):
        entries = random_entries(rng, int(rng.integers(1, 40)), stored=stored, ties=ties)
        alpha = float(rng.choice([0.5, 1.0, 2.0])) if ties else float(rng.uniform(0.2, 3.0))
        full = sum(e.sizes[e.min_choice] for e in entries)
        tiers = []
        for t in range(int(rng.integers(1, 4))):
            bw = float(rng.choice([1e5, 1e6, 4e6])) if ties else float(rng.uniform(5e4, 5e6))
            tiers.append((bw, float(int(rng.uniform(0.0, 0.7) * full))))
        want_tier, want_choice, want_total = P.plan(entries, alpha, tiers)
        tier, choice, total = native_plan(kvh, entries, alpha, tiers)
        assert tier.tolist() == want_tier and choice.tolist() == want_choice, trial
        assert total == want_total, trial


def test_capacity_sweep_and_scale(kvh):
    rng = np.random.default_rng(9)
    entries = random_entries(rng, 300)
    full = sum(e.sizes[0] for e in entries)
    last = -1.0
    for frac in np.linspace(0.0, 1.0, 9):
        cap = float(int(frac * full))
        want = P.solve_tier(entries, 1.0, 1e6, cap)
        tier, choice, total = native_plan(kvh, entries, 1.0, [(1e6, cap)])
        assert choice.tolist() == want[0] and total == want[1]
        used = sum(entries[i].sizes[c] for i, c in enumerate(choice) if c >= 0)
        assert used <= cap and total >= last
        last = total
    # a large instance finishes quickly and stays feasible (the oracle would take minutes here)
    big = random_entries(rng, 20000)
    cap = float(int(0.3 * sum(e.sizes[0] for e in big)))
    tier, choice, total = native_plan(kvh, big, 1.0, [(2e9, cap), (1e9, 2 * cap)])
    for t, limit in ((0, cap), (1, 2 * cap)):
        assert sum(big[i].sizes[choice[i]] for i in np.flatnonzero(tier == t)) <= limit
    assert ((tier >= 0) == (choice >= 0)).all()


def test_argument_errors(kvh):
    L = kvh.lib()
    from paper_2509_00105_amd.binding import POLICY_ENTRY, POLICY_TIER

    ent = np.zeros(1, dtype=POLICY_ENTRY); ent["freq"], ent["n_choices"] = 1.0, 2
    sizes = np.array([64.0, 32.0]); q = np.array([1.0, 0.5])
    tr = np.zeros(1, dtype=POLICY_TIER); tr["bandwidth"], tr["capacity"] = 1e6, 100.0
    to, co = np.zeros(1, np.int32), np.zeros(1, np.int32)

    def call(e=ent, s=sizes, qq=q, n_tot=2, t=tr, alpha=1.0):
        return L.kvh_policy_plan(e.ctypes.data, 1, s.ctypes.data, qq.ctypes.data, n_tot, t.ctypes.data, 1, alpha,
                                 to.ctypes.data, co.ctypes.data, None)

    assert call() == 0 and co[0] == 0
    assert L.kvh_policy_plan(None, 1, sizes.ctypes.data, q.ctypes.data, 2, tr.ctypes.data, 1, 1.0, to.ctypes.data, co.ctypes.data, None) == -1
    assert call(s=np.array([64.0, 64.0])) == -1        # not strictly decreasing
    assert call(s=np.array([64.5, 32.0])) == -1        # not a whole number of bytes
    assert call(s=np.array([64.0, 0.0])) == -1
    assert call(qq=np.array([1.0, np.nan])) == -1
    assert call(alpha=float("inf")) == -1
    bad = ent.copy(); bad["n_choices"] = 3
    assert call(e=bad) == -3
    bad = ent.copy(); bad["min_choice"] = 2
    assert call(e=bad) == -3
    bad = ent.copy(); bad["freq"] = -1.0
    assert call(e=bad) == -1
    bt = tr.copy(); bt["bandwidth"] = 0.0
    assert call(t=bt) == -1
    bt = tr.copy(); bt["capacity"] = -1.0
    assert call(t=bt) == -1
    it = tr.copy(); it["capacity"] = np.inf
    assert call(t=it) == 0
    # two entries whose largest sizes add up to 2^53: occupancy sums would no longer be exact
    two = np.zeros(2, dtype=POLICY_ENTRY); two["freq"], two["n_choices"], two["first"] = 1.0, 1, [0, 1]
    half = np.array([2.0 ** 52, 2.0 ** 52]); qq = np.array([1.0, 1.0])
    to2, co2 = np.zeros(2, np.int32), np.zeros(2, np.int32)
    assert L.kvh_policy_plan(two.ctypes.data, 2, half.ctypes.data, qq.ctypes.data, 2, tr.ctypes.data, 1, 1.0,
                             to2.ctypes.data, co2.ctypes.data, None) == -4
