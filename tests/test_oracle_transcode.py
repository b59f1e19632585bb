"""CPU-only pins of the oracle's transcode (re-compress a stored entry from rate m to rate n, the step the
paper's greedy policy takes when it lowers an entry's rate; Design section, marginal utility drop).  The
oracle is decode followed by encode.  Pins that do not re-run that composition: a hand-computed ramp, the
statistics that must survive (a group always holds code 0 and code L, which decode to the stored min and
max exactly), the identity m -> m, closeness to a direct encode at the target level, the error bound,
degenerate groups, carried token-dropping words, error paths."""
import struct

import numpy as np
import pytest

import kv_inputs as gen
import oracle

F16, BF16 = gen.F16, gen.BF16
PAIRS = [(a, b) for a in range(3) for b in range(3)]


def unpack_codes(section: np.ndarray, n: int, c: int, bits: int) -> np.ndarray:
    rows = section[: n * c * bits // 8].reshape(n, c * bits // 8)
    per = 8 // bits
    out = np.zeros((n, c), dtype=np.int32)
    for j in range(per):
        out[:, j::per] = (rows >> (bits * j)) & ((1 << bits) - 1)
    return out


def sections(blob, l, n, c, level, lam):
    off = oracle.section_offsets(l, n, c, level, lam)
    bits = oracle.level_bits(level)
    G = (n + 127) // 128
    return {
        "kmeta": blob[off["kmeta"]: off["kmeta"] + G * c * 4],
        "kcodes": unpack_codes(blob[off["kcodes"]:], n, c, bits),
        "vmeta": blob[off["vmeta"]: off["vmeta"] + n * (c // 128) * 4],
        "vcodes": unpack_codes(blob[off["vcodes"]:], n, c, bits),
    }


def test_ramp_worked_by_hand():
    # One token, 128 channels: 0, 2, 4, ..., 252, 255.  At 8 bits r = 255, scale = 1: codes are the values and decode
    # is exact.  At 2 bits t = x * 3/255 crosses .5, 1.5, 2.5 at x = 42.5, 127.5, 212.5 (never at an integer), so
    # codes are 0 for x <= 42, 1 up to 126, 2 up to 212, 3 above; the 2-bit entry decodes to 0, 85, 170, 255.
    x = np.array([2 * j for j in range(127)] + [255], dtype=np.float32)
    for dt, cast in ((F16, lambda a: a.astype(np.float16).view(np.uint16)), (BF16, lambda a: (a.view(np.uint32) >> 16).astype(np.uint16))):
        kb = cast(x).reshape(1, 1, 128)
        b8 = oracle.encode(kb, kb, dt, 0)
        s8 = sections(b8, 1, 1, 128, 0, 0)
        assert list(s8["vcodes"][0]) == [int(t) for t in x]
        b2 = oracle.transcode(b8, dt, 1, 1, 128, 0, 2)
        s2 = sections(b2, 1, 1, 128, 2, 0)
        want = [0 if t <= 42 else 1 if t <= 126 else 2 if t <= 212 else 3 for t in x]
        assert list(s2["vcodes"][0]) == want
        # first code byte: channels 0..3 -> values 0, 2, 4, 6 -> codes 0; channels 20..23 -> 40, 42, 44, 46 -> 0,0,1,1
        off = oracle.section_offsets(1, 1, 128, 2, 0)
        assert b2[off["vcodes"]] == 0x00 and b2[off["vcodes"] + 5] == 0b01010000
        k2, v2 = oracle.decode(b2, dt, 1, 1, 128, 2)
        vals = gen.bits_to_f64(v2[0, 0], dt)
        assert list(vals) == [85.0 * q for q in want]
        # header: same shape, new bits and size
        assert b2[7] == 2 and struct.unpack_from("<Q", b2, 24)[0] == b2.size == oracle.blob_size(1, 1, 128, 2)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_group_statistics_survive_and_codes_stay_close(dt):
    l, n, c = 2, 300, 256  # ragged last K group (44 tokens)
    k, v = gen.make_kv(l, n, c, dt, seed=77 + dt)
    enc = [oracle.encode(k, v, dt, lv) for lv in range(3)]
    for a, b in PAIRS:
        out = oracle.transcode(enc[a], dt, l, n, c, a, b)
        assert out.size == oracle.blob_size(l, n, c, b)
        La, Lb = (1 << oracle.level_bits(a)) - 1, (1 << oracle.level_bits(b)) - 1
        for lam in range(l):
            src, got, direct = sections(enc[a], l, n, c, a, lam), sections(out, l, n, c, b, lam), sections(enc[b], l, n, c, b, lam)
            # min and max of every group are reproduced exactly by decode, so the metadata is unchanged
            assert np.array_equal(got["kmeta"], src["kmeta"]) and np.array_equal(got["vmeta"], src["vmeta"])
            if Lb > La:
                continue  # going up cannot restore what level a lost; only the statistics are checked
            for key in ("kcodes", "vcodes"):
                d = np.abs(got[key] - direct[key])
                # the detour through level a moves a value by at most half a step of a: under one code of b
                assert d.max() <= 1
                assert (d != 0).mean() < 0.75 * Lb / La + 0.01
        if a == b:
            assert np.array_equal(out, enc[a])  # E(D(E(x))) == E(x)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_error_bound_after_transcode(dt):
    l, n, c = 1, 256, 128
    k, v = gen.make_kv(l, n, c, dt, seed=5)
    eps = 2.0 ** -11 if dt == F16 else 2.0 ** -8
    for a, b in [(0, 1), (0, 2), (1, 2)]:
        out = oracle.transcode(oracle.encode(k, v, dt, a), dt, l, n, c, a, b)
        kd, vd = oracle.decode(out, dt, l, n, c, b)
        La, Lb = (1 << oracle.level_bits(a)) - 1, (1 << oracle.level_bits(b)) - 1
        x, y = gen.bits_to_f64(v[0], dt), gen.bits_to_f64(vd[0], dt)
        r = (x.max(axis=1) - x.min(axis=1))[:, None]
        amax = np.abs(x).max(axis=1)[:, None]
        assert np.all(np.abs(x - y) <= r / (2 * La) + r / (2 * Lb) + 3 * eps * amax + 1e-30)
        x, y = gen.bits_to_f64(k[0], dt), gen.bits_to_f64(kd[0], dt)
        for g in range(2):
            xs, ys = x[128 * g: 128 * (g + 1)], y[128 * g: 128 * (g + 1)]
            r = (xs.max(axis=0) - xs.min(axis=0))[None, :]
            amax = np.abs(xs).max(axis=0)[None, :]
            assert np.all(np.abs(xs - ys) <= r / (2 * La) + r / (2 * Lb) + 3 * eps * amax + 1e-30)


def test_chain_keeps_statistics():
    dt, l, n, c = BF16, 1, 200, 128
    k, v = gen.make_kv(l, n, c, dt, seed=9)
    b8 = oracle.encode(k, v, dt, 0)
    b4 = oracle.transcode(b8, dt, l, n, c, 0, 1)
    b2 = oracle.transcode(b4, dt, l, n, c, 1, 2)
    b2d = oracle.transcode(b8, dt, l, n, c, 0, 2)
    s, sd, s8 = sections(b2, l, n, c, 2, 0), sections(b2d, l, n, c, 2, 0), sections(b8, l, n, c, 0, 0)
    assert np.array_equal(s["kmeta"], s8["kmeta"]) and np.array_equal(s["vmeta"], s8["vmeta"])
    assert np.array_equal(sd["kmeta"], s8["kmeta"])
    assert np.abs(s["kcodes"] - sd["kcodes"]).max() <= 1 and np.abs(s["vcodes"] - sd["vcodes"]).max() <= 1
    # going up and down again returns the 2-bit entry
    up = oracle.transcode(b2, dt, l, n, c, 2, 0)
    assert np.array_equal(oracle.transcode(up, dt, l, n, c, 0, 2), b2)
    ku, vu = oracle.decode(up, dt, l, n, c, 0)
    k2, v2 = oracle.decode(b2, dt, l, n, c, 2)
    # the 8-bit entry reproduces the 2-bit entry's values to within half an 8-bit step plus the 16-bit rounding
    a, b = gen.bits_to_f64(vu[0], dt), gen.bits_to_f64(v2[0], dt)
    r = (b.max(axis=1) - b.min(axis=1))[:, None]
    assert np.all(np.abs(a - b) <= r / 510 + 2.0 ** -7 * np.abs(b).max(axis=1)[:, None])


def test_degenerate_group_collapses_to_its_minimum():
    # bf16 values 2^-111 and 2^-110: range 2^-111 < 2^-100 -> degenerate, every element decodes to the minimum, so
    # the re-encoded group stores (mn, mn); a constant group keeps (mn, mn) anyway.
    lo, hi = 0x0800, 0x0880  # bf16 2^-111, 2^-110
    row = np.full((1, 1, 128), lo, dtype=np.uint16)
    row[0, 0, 5] = hi
    b = oracle.encode(row, row, BF16, 0)
    off = oracle.section_offsets(1, 1, 128, 0, 0)
    assert struct.unpack_from("<HH", b, off["vmeta"]) == (lo, hi)
    out = oracle.transcode(b, BF16, 1, 1, 128, 0, 2)
    off2 = oracle.section_offsets(1, 1, 128, 2, 0)
    assert struct.unpack_from("<HH", out, off2["vmeta"]) == (lo, lo)
    assert not out[off2["vcodes"]: off2["vcodes"] + 32].any()
    # K side: each channel is its own one-token group -> constant -> (x, x)
    assert struct.unpack_from("<HH", out, off2["kmeta"] + 4 * 5) == (hi, hi)


def test_token_dropping_words_are_carried():
    dt, l, N, c, sink, window = F16, 2, 400, 128, 3, 130
    k, v = gen.make_kv(l, N, c, dt, seed=3)
    n = oracle.kept_tokens(N, sink, window)
    b = oracle.encode_kept(k, v, dt, sink, window, 0)
    out = oracle.transcode(b, dt, l, n, c, 0, 2)
    assert struct.unpack_from("<III", out, 32) == (N, sink, window) and not out[44:64].any()
    pos = list(range(sink)) + list(range(N - window, N))
    plain = oracle.transcode(oracle.encode(np.ascontiguousarray(k[:, pos]), np.ascontiguousarray(v[:, pos]), dt, 0), dt, l, n, c, 0, 2)
    same = out.copy(); same[32:44] = 0
    assert np.array_equal(same, plain)
    kd = np.zeros((l, N, c), np.uint16); vd = np.zeros_like(kd)
    assert oracle.decode_kept_into(out, dt, l, N, c, sink, window, 2, kd, vd) == 0
    # inconsistent words are refused
    bad = b.copy(); struct.pack_into("<I", bad, 36, sink + 1)
    assert oracle.transcode_rc(bad, dt, l, n, c, 0, 2, np.empty(out.size, np.uint8)) == oracle.E_HEADER


def test_error_paths():
    dt, l, n, c = F16, 1, 130, 128
    k, v = gen.make_kv(l, n, c, dt, seed=1)
    b = oracle.encode(k, v, dt, 1)
    out = np.empty(oracle.blob_size(l, n, c, 2), np.uint8)
    assert oracle.transcode_rc(b, dt, l, n, c, 1, 2, out) == oracle.OK
    assert oracle.transcode_rc(b, dt, l, n, c, 0, 2, out[: 16]) == oracle.E_SIZE
    assert oracle.transcode_rc(b, dt, l, n, c, 1, 2, out[:-1]) == oracle.E_SIZE
    assert oracle.transcode_rc(b[:-1], dt, l, n, c, 1, 2, out) == oracle.E_SIZE
    assert oracle.transcode_rc(b, dt, l, n, c, 1, 4, out) == oracle.E_LEVEL
    assert oracle.transcode_rc(b, dt, l, n, c, -1, 2, out) == oracle.E_LEVEL
    assert oracle.transcode_rc(b, dt, l, n, 100, 1, 2, out) == oracle.E_SHAPE
    assert oracle.transcode_rc(b, BF16, l, n, c, 1, 2, out) == oracle.E_HEADER
    big = np.concatenate([b, np.zeros(oracle.blob_size(l, n, c, 0), np.uint8)])
    assert oracle.transcode_rc(big, dt, l, n, c, 0, 2, out) == oracle.E_HEADER  # stored at level 1, claimed 0


def test_statistics_survive_on_hard_groups():
    # Groups whose range is a few units in the last place of the 16-bit type (large offset, small spread), tiny and
    # huge magnitudes, one-token and ragged K groups: the stored min and max must still come back from decode exactly.
    rng = np.random.default_rng(0)
    for trial in range(120):
        dt = trial % 2
        l, n, c = 1, int(rng.integers(1, 200)), 128
        base = float(rng.choice([0, 1, 100, -1000, 3e4 if dt == F16 else 1e30]))
        spread = float(rng.choice([1e-6, 1e-3, 1, 30])) * (1e28 if base == 1e30 else 1)
        x = (base + spread * rng.standard_normal((2, l, n, c))).astype(np.float32)
        bits = x.astype(np.float16).view(np.uint16) if dt == F16 else oracle.f32_to_t16_array(x, BF16)
        k, v = bits[0], bits[1]
        for a in range(3):
            ea = oracle.encode(k, v, dt, a)
            for b in range(3):
                out = oracle.transcode(ea, dt, l, n, c, a, b)
                s, g = sections(ea, l, n, c, a, 0), sections(out, l, n, c, b, 0)
                assert np.array_equal(s["kmeta"], g["kmeta"]) and np.array_equal(s["vmeta"], g["vmeta"]), (trial, a, b)
                if a == b:
                    assert np.array_equal(out, ea), (trial, a)
