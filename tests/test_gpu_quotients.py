"""GPU checks of the group-parameter quotients (Sec. 3.2's quantisation: scale = r / L, inv = L / r, correctly rounded
in fp32).  The kernels form them without the division sequence; these tests hold them to the division's bits: once
exhaustively on the device (kvh_selftest_division) and once end to end against the oracle, on groups whose ranges
walk through every binary exponent a finite group can have."""
import numpy as np
import pytest

import kv_inputs as gen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

BF16 = gen.BF16


@pytest.fixture(scope="module")
def kvh():
    import paper_2509_00105_amd as m

    m.lib()
    return m


def test_short_quotients_equal_division_for_every_range(kvh):
    assert kvh.selftest_division() == [0, 0, 0, 0, 0, 0]


def exponent_walk(seed):
    """[rows][128] bf16 bit patterns: row i spans [-a, +a] or [0, a] with a = m * 2^e, e walking from the smallest range
    that is not degenerate (2^-100) down past it and up to the largest whose difference still fits fp32."""
    rng = np.random.default_rng(seed)
    rows = []
    for e in range(-112, 127):
        for one_sided in (False, True):
            m = 1.0 + float(rng.integers(0, 128)) / 128.0          # a bf16 mantissa
            a = np.float32(m * 2.0 ** e)
            u = rng.random(128).astype(np.float32)
            x = (u * a if one_sided else (2 * u - 1) * a).astype(np.float32)
            x[int(rng.integers(128))] = a
            x[int(rng.integers(128))] = 0.0 if one_sided else -a
            rows.append(x)
    return gen._cast_to_bits(np.stack(rows), BF16)


@pytest.mark.parametrize("level", [0, 1, 2])
def test_ranges_of_every_exponent_match_oracle(kvh, level):
    xb = exponent_walk(5 + level)                                   # [G][128]
    G = xb.shape[0]
    Gp = -(-G // 128) * 128
    v = np.zeros((1, G, 128), np.uint16); v[0] = xb                 # V: one group per token
    k = np.zeros((1, 128, Gp), np.uint16); k[0, :, :G] = xb.T       # K: one group per channel
    for name, (a, n, c) in (("groups along tokens", (k, 128, Gp)), ("groups along channels", (v, G, 128))):
        want = oracle.encode(a, a, BF16, level)
        t = torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        blob = kvh.encode(t, t, level)
        torch.cuda.synchronize()
        got = blob.cpu().numpy()
        assert np.array_equal(got, want), "%s level %d: first differing byte %d" % (
            name, level, int(np.flatnonzero(got != want)[0]))
        wk, wv = oracle.decode(want, BF16, 1, n, c, level)
        ok = torch.zeros((1, n, c), dtype=torch.bfloat16, device="cuda"); ov = torch.zeros_like(ok)
        kvh.decode(blob, level, n, ok, ov)
        torch.cuda.synchronize()
        assert np.array_equal(ok.view(torch.int16).cpu().numpy().view(np.uint16), wk), name + " K"
        assert np.array_equal(ov.view(torch.int16).cpu().numpy().view(np.uint16), wv), name + " V"
        # transcoding the 8-bit blob down uses both quotients of both levels
        if level == 0:
            for lo in (1, 2):
                w2 = oracle.transcode(want, BF16, 1, n, c, 0, lo)
                g2 = kvh.transcode(blob, BF16, 1, n, c, 0, lo)
                torch.cuda.synchronize()
                assert np.array_equal(g2.cpu().numpy(), w2), "%s transcode 8 -> %d" % (name, kvh.level_bits(lo))
