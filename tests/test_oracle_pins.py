"""CPU-only pins of the oracle (oracle/kvh_ref.c) against things other than itself.

The paper (AdaptCache) names its quantisation method and one rate, two bits (Preliminary
Results) but prints no equations, examples or error figures for it, so the pins are: the
hand-computed worked examples under tests/golden/, exact-arithmetic brute force, closed forms
(uniform-quantiser RMS = step / sqrt(12), blob-size closed form), invariants (step-bounded
error, exact endpoints, idempotent re-encoding, monotone error across levels), special cases
(constant groups, identity page table, K/V duality on a transposed tile) and the two 16-bit
float conversions checked exhaustively against numpy and torch.
"""
import json
import math
import os
import struct
from fractions import Fraction

import numpy as np
import pytest

import kv_inputs as gen
import oracle

F16, BF16 = gen.F16, gen.BF16
GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.json")


# ---------------------------------------------------------------------------------------------
# helpers (test-side only)
# ---------------------------------------------------------------------------------------------
def to_bits(x, dt):
    """Exactly representable python floats -> uint16 patterns, without using the oracle."""
    x = np.asarray(x, dtype=np.float32)
    if dt == F16:
        out = x.astype(np.float16)
        assert np.array_equal(out.astype(np.float32), x), "value not exact in fp16"
        return out.view(np.uint16)
    u = x.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "value not exact in bf16"
    return (u >> 16).astype(np.uint16)


def val(bits, dt):
    return gen.bits_to_f64(np.asarray(bits, dtype=np.uint16), dt)


def frac_of(bits, dt):
    return Fraction(float(val(np.uint16(bits), dt)))


def split_blob(blob, l, n, c, level):
    """Parse a blob with the layout closed form typed out here (not via the oracle's helper)."""
    b = {0: 8, 1: 4, 2: 2}[level]
    pad = lambda x: (x + 15) // 16 * 16
    G = -(-n // 128)
    km, cd, vm = pad(G * c * 4), pad(n * c * b // 8), pad(n * (c // 128) * 4)
    assert blob.size == 64 + l * (km + vm + 2 * cd)
    out, p = [], 64
    for _ in range(l):
        kmeta = blob[p:p + G * c * 4].view(np.uint16).reshape(G, c, 2); p += km
        kcodes = blob[p:p + n * c * b // 8].reshape(n, c * b // 8); p += cd
        vmeta = blob[p:p + n * (c // 128) * 4].view(np.uint16).reshape(n, c // 128, 2); p += vm
        vcodes = blob[p:p + n * c * b // 8].reshape(n, c * b // 8); p += cd
        out.append((kmeta, kcodes, vmeta, vcodes))
    return out


def unpack(codes_rows, b):
    """[n][c*b/8] bytes -> [n][c] codes, LSB-first."""
    per = 8 // b
    shifts = (np.arange(per) * b).astype(np.uint8)
    q = (codes_rows[:, :, None] >> shifts[None, None, :]) & ((1 << b) - 1)
    return q.reshape(codes_rows.shape[0], -1)


# ---------------------------------------------------------------------------------------------
# 16-bit float conversions: exhaustive / randomised against independent libraries
# ---------------------------------------------------------------------------------------------
def test_fp16_to_f32_exhaustive_vs_numpy():
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.t16_to_f32_array(allbits, F16)
    want = allbits.view(np.float16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32)[~np.isnan(want)], want.view(np.uint32)[~np.isnan(want)])
    assert np.all(np.isnan(got[np.isnan(want)]))


def test_bf16_to_f32_exhaustive_vs_torch():
    import torch

    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.t16_to_f32_array(allbits, BF16)
    want = torch.from_numpy(allbits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    ok = ~np.isnan(want)
    assert np.array_equal(got.view(np.uint32)[ok], want.view(np.uint32)[ok])
    assert np.all(np.isnan(got[~ok]))


def _f32_samples(dt):
    rng = np.random.default_rng(123)
    rnd = rng.integers(0, 2**32, size=1_000_000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    # every T16 value, its exact midpoint to the next one, and one fp32 ulp either side of the midpoint
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    if dt == F16:
        f = allbits.view(np.float16).astype(np.float64)
    else:
        f = (allbits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    f = np.sort(f[np.isfinite(f)])
    mid = ((f[:-1] + f[1:]) / 2).astype(np.float32)  # midpoints of 16-bit values are exact in fp32
    ties = np.concatenate([mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf)),
                           f.astype(np.float32)])
    edge = np.array([65504.0, 65519.99, 65520.0, 65535.0, 1e10, 2.0**-24, 2.0**-25, 2.0**-25 * 1.0001, 2.0**-26,
                     2.0**-14, 2.0**-14 * (1 - 2.0**-12), 3.38e38, 3.4e38, 0.0, -0.0], dtype=np.float32)
    s = np.concatenate([rnd, ties, edge, -edge])
    return s[~np.isnan(s)]


def test_f32_to_fp16_rne_vs_numpy():
    x = _f32_samples(F16)
    got = oracle.f32_to_t16_array(x, F16)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)


def test_f32_to_bf16_rne_vs_torch():
    import torch

    x = _f32_samples(BF16)
    got = oracle.f32_to_t16_array(x, BF16)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_f32_to_t16_is_nearest_even_in_exact_arithmetic(dt):
    """Independent definition: among all finite T16 values pick the nearest, ties to even mantissa."""
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    v = val(allbits, dt)
    fin = np.isfinite(v) & (allbits != 0x8000)
    grid_bits, grid = allbits[fin], v[fin]
    order = np.argsort(grid, kind="stable")
    grid_bits, grid = grid_bits[order], grid[order]
    rng = np.random.default_rng(7)
    hi = 60000.0 if dt == F16 else 1e30
    xs = np.concatenate([rng.standard_normal(1500) * s for s in (1e-7, 1e-4, 1.0, 300.0, hi / 4)]).astype(np.float32)
    got = oracle.f32_to_t16_array(xs, dt)
    for x, g in zip(xs, got):
        i = int(np.searchsorted(grid, float(x)))
        cands = [j for j in (i - 1, i) if 0 <= j < grid.size]
        fx = Fraction(float(x))
        best = min(cands, key=lambda j: (abs(Fraction(float(grid[j])) - fx), int(grid_bits[j]) & 1))
        if float(grid[best]) == 0.0:   # rounds to zero: the sign of x is kept
            assert int(g) == (0x8000 if x < 0 or (x == 0 and np.signbit(x)) else 0)
        else:
            assert int(g) == int(grid_bits[best]), (x, hex(g), hex(grid_bits[best]))


# ---------------------------------------------------------------------------------------------
# worked examples
# ---------------------------------------------------------------------------------------------
def _example_tensor(values, fill, dt, where):
    """One layer, n = 128 tokens, c = 128 channels, everything = fill except the example group."""
    x = np.full((1, 128, 128), fill, dtype=np.float32)
    if where == "K":   # group = channel 5, along tokens
        x[0, :len(values), 5] = values
    else:              # group = token 3, along channels
        x[0, 3, :len(values)] = values
    return to_bits(x, dt)


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("name,level", [("A_2bit", 2), ("B_4bit", 1)])
def test_worked_examples_A_B(name, level, dt):
    ex = json.load(open(GOLD))[name]
    b = ex["bits"]
    assert oracle.level_bits(level) == b
    vals = ex["values"]
    # scalar steps
    mn, mx = int(to_bits(ex["mn"], dt)), int(to_bits(ex["mx"], dt))
    scale, inv, deg = oracle.group_params(mn, mx, dt, b)
    assert (float(scale), float(inv), deg) == (ex["scale"], ex["inv"], False)
    for x, t, q, d in zip(vals, ex["t"], ex["codes"], ex["decoded"]):
        assert (x - ex["mn"]) * ex["inv"] == t
        assert oracle.quantise(int(to_bits(x, dt)), mn, inv, dt, b) == q
        assert float(val(oracle.dequantise(q, mn, mx, dt, b), dt)) == d
        assert abs(x - d) <= ex["max_abs_error"]
    # through the whole encoder, as a V group (bytes are consecutive in a token row) ...
    kfill = _example_tensor([], ex["fill"], dt, "K")
    v = _example_tensor(vals, ex["fill"], dt, "V")
    blob = oracle.encode(kfill, v, dt, level)
    (kmeta, kcodes, vmeta, vcodes), = split_blob(blob, 1, 128, 128, level)
    assert [hex(x) for x in vcodes[3, :len(ex["first_bytes"])]] == [s.lower() for s in ex["first_bytes"]]
    assert list(val(vmeta[3, 0], dt)) == [ex["mn"], ex["mx"]]
    q = unpack(vcodes, b)
    assert list(q[3, :len(vals)]) == ex["codes"] and np.all(q[3, len(vals):] == ex["fill_code"])
    # ... and as a K group (codes of one channel, one per token row)
    k = _example_tensor(vals, ex["fill"], dt, "K")
    blob = oracle.encode(k, _example_tensor([], ex["fill"], dt, "V"), dt, level)
    (kmeta, kcodes, vmeta, vcodes), = split_blob(blob, 1, 128, 128, level)
    q = unpack(kcodes, b)
    assert list(q[:len(vals), 5]) == ex["codes"] and np.all(q[len(vals):, 5] == ex["fill_code"])
    assert list(val(kmeta[0, 5], dt)) == [ex["mn"], ex["mx"]]
    kd, vd = oracle.decode(blob, dt, 1, 128, 128, level)
    assert list(val(kd[0, :len(vals), 5], dt)) == ex["decoded"]
    assert np.all(val(kd[0, len(vals):, 5], dt) == ex["fill_decoded"])
    # untouched channels are constant groups: lossless
    assert np.all(val(kd[0, :, 6], dt) == ex["fill"]) and np.all(val(vd, dt) == ex["fill"])


@pytest.mark.parametrize("dt", [F16, BF16])
def test_worked_example_C_8bit(dt):
    ex = json.load(open(GOLD))["C_8bit"]
    ramp = np.arange(128, dtype=np.float32)
    v = to_bits(np.tile(ramp, (1, 128, 1)), dt)                 # every token row = 0..127 (V groups)
    k = to_bits(np.tile(ramp[:, None], (1, 1, 128)), dt)        # every channel = 0..127 along tokens (K groups)
    blob = oracle.encode(k, v, dt, 0)
    (kmeta, kcodes, vmeta, vcodes), = split_blob(blob, 1, 128, 128, 0)
    want = np.array([(2 * i * 255 + 127) // (2 * 127) for i in range(128)])  # floor(i*255/127 + 1/2), integers only
    for i, q in ex["spot_codes"].items():
        assert want[int(i)] == q
    assert np.array_equal(vcodes, np.tile(want, (128, 1)))      # 8-bit: bytes are the codes
    assert np.array_equal(kcodes, np.tile(want[:, None], (1, 128)))
    assert np.all(val(kmeta[..., 0], dt) == 0) and np.all(val(kmeta[..., 1], dt) == 127)
    kd, vd = oracle.decode(blob, dt, 1, 128, 128, 0)
    assert np.array_equal(kd[0].T, vd[0])
    if dt == F16:
        for i, x in ex["spot_decoded_fp16"].items():
            assert float(val(vd[0, 0, int(i)], dt)) == x
    assert np.max(np.abs(val(vd[0, 0], dt) - ramp)) <= 0.5 * 127 / 255 * (1 + 2**-10) + 0.5 * (2**-4 if dt == F16 else 0.5)


def test_embedding_offsets_typed_by_hand():
    """Layout pin: l=2, n=130 (ragged), c=256, 4-bit; offsets computed by hand from the layout."""
    l, n, c, level = 2, 130, 256, 1
    # per layer: kmeta 2 groups * 256 ch * 4 B = 2048; codes 130 * 128 B = 16640; vmeta 130 * 2 * 4 = 1040
    per_layer = 2048 + 16640 + 1040 + 16640
    assert oracle.blob_size(l, n, c, level) == 64 + 2 * per_layer == 72800
    k = np.zeros((l, n, c), dtype=np.float32)
    v = np.zeros((l, n, c), dtype=np.float32)
    k[1, 128, 7], k[1, 129, 7] = 1.0, 16.0     # layer 1, token-group 1 (only 2 tokens), channel 7
    v[1, 129, 128:133] = [0.0, 15.0, 7.5, 8.5, 3.0]  # layer 1, last token, channel-group 1
    blob = oracle.encode(to_bits(k, F16), to_bits(v, F16), F16, level)
    base1 = 64 + per_layer
    km = base1 + (1 * 256 + 7) * 4
    assert struct.unpack_from("<ee", blob, km) == (1.0, 16.0)
    kc = base1 + 2048
    assert blob[kc + 128 * 128 + 7 // 2] == 0x00 and blob[kc + 129 * 128 + 7 // 2] == 0xF0  # ch 7 = high nibble
    vm = base1 + 2048 + 16640 + (129 * 2 + 1) * 4
    assert struct.unpack_from("<ee", blob, vm) == (0.0, 15.0)
    vc = base1 + 2048 + 16640 + 1040 + 129 * 128 + 128 // 2
    assert list(blob[vc:vc + 3]) == [0xF0, 0x88, 0x03]
    # everything else in the code sections is zero
    rest = blob.copy()
    rest[:64] = 0
    for off, cnt in ((km, 4), (vm, 4), (kc + 129 * 128 + 3, 1), (vc, 3)):
        rest[off:off + cnt] = 0
    assert not rest.any()


# ---------------------------------------------------------------------------------------------
# header, sizes, levels
# ---------------------------------------------------------------------------------------------
def test_levels_and_blob_size_closed_form():
    assert oracle.num_levels() == 3
    assert [oracle.level_bits(i) for i in (-1, 0, 1, 2, 3, 4)] == [-1, 8, 4, 2, 16, -1]  # 3 = the raw level
    # a 256-token chunk of the 32-layer, 1024-channel shape: 64 + l*(ceil(n/128)*4c + n*4c/128 + 2*n*c*b/8)
    assert [oracle.blob_size(32, 256, 1024, lv) for lv in range(3)] == [17_301_568, 8_912_960, 4_718_656]
    U = 2 * 32 * 256 * 1024 * 2
    ratios = [U / oracle.blob_size(32, 256, 1024, lv) for lv in range(3)]
    assert [round(r, 2) for r in ratios] == [1.94, 3.76, 7.11]
    rng = np.random.default_rng(0)
    for _ in range(200):
        l, n, m, lv = int(rng.integers(1, 9)), int(rng.integers(1, 700)), int(rng.integers(1, 9)), int(rng.integers(0, 3))
        c, b = 128 * m, (8, 4, 2)[lv]
        pad = lambda x: (x + 15) // 16 * 16
        want = 64 + l * (-(-n // 128) * 4 * c + pad(n * 4 * c // 128) + 2 * n * c * b // 8)
        assert oracle.blob_size(l, n, c, lv) == want
    for bad in [(0, 1, 128, 0), (1, 0, 128, 0), (1, 1, 64, 0), (1, 1, 192, 0), (1, 1, 128, 4), (1, 1, 128, -1)]:
        assert oracle.blob_size(*bad) == 0


@pytest.mark.parametrize("dt", [F16, BF16])
def test_header_fields(dt):
    k, v = gen.make_kv(3, 200, 256, dt, 5)
    for level, b in ((0, 8), (1, 4), (2, 2)):
        blob = oracle.encode(k, v, dt, level)
        magic, ver, hdt, hb, l, n, c, gt, gc, total = struct.unpack_from("<4sHBBIIIHHQ", blob, 0)
        assert (magic, ver, hdt, hb, l, n, c, gt, gc, total) == (b"KVH1", 1, dt, b, 3, 200, 256, 128, 128, blob.size)
        assert not blob[32:64].any()
        for lam in range(3):
            so = oracle.section_offsets(3, 200, 256, level, lam)
            assert all(so[s] % 16 == 0 for s in ("kmeta", "kcodes", "vmeta", "vcodes"))


def test_error_paths():
    k, v = gen.make_kv(1, 128, 128, F16, 1)
    good = oracle.encode(k, v, F16, 1)
    blob = np.zeros(good.size, dtype=np.uint8)
    assert oracle.encode_rc(k, v, F16, 4, blob) == oracle.E_LEVEL
    assert oracle.encode_rc(k, v, 2, 1, blob) == oracle.E_ARG
    assert oracle.encode_rc(k[:, :, :64], v[:, :, :64], F16, 1, blob) == oracle.E_SHAPE
    assert oracle.encode_rc(k, v, F16, 1, blob[:-1]) == oracle.E_SIZE
    kd, vd = np.zeros_like(k), np.zeros_like(v)
    assert oracle.decode_into(good, F16, 1, 128, 128, 1, kd, vd) == oracle.OK
    assert oracle.decode_into(good[:-1], F16, 1, 128, 128, 1, kd, vd) == oracle.E_SIZE
    assert oracle.decode_into(good, F16, 1, 128, 128, 2, kd, vd) == oracle.E_HEADER   # level mismatch
    assert oracle.decode_into(good, BF16, 1, 128, 128, 1, kd, vd) == oracle.E_HEADER  # dtype mismatch
    for off in (0, 4, 7, 8, 12, 16, 20, 22, 24):
        bad = good.copy(); bad[off] ^= 1
        assert oracle.decode_into(bad, F16, 1, 128, 128, 1, kd, vd) == oracle.E_HEADER
    kk = k.copy(); kk[0, 3, 9] = 0x7C00  # +inf
    assert oracle.encode_rc(kk, v, F16, 1, blob) == oracle.E_NONFINITE
    kk[0, 3, 9] = 0x7E00  # NaN
    assert oracle.encode_rc(kk, v, F16, 1, blob) == oracle.E_NONFINITE


# ---------------------------------------------------------------------------------------------
# brute force in exact arithmetic
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("level", [1, 2])
def test_codes_are_exact_argmin_on_coarse_grid(level, dt):
    """Values on a coarse dyadic grid, so exact ties occur and must go to the even code."""
    b = oracle.level_bits(level); L = (1 << b) - 1
    rng = np.random.default_rng(level * 10 + dt)
    n_ties = 0
    for trial in range(12):
        n = int(rng.integers(1, 5))
        step = 2.0 ** int(rng.integers(-3, 2))
        x = (rng.integers(-12, 13, size=(1, n, 128)) * step).astype(np.float32)
        kb, vb = to_bits(x, dt), to_bits(x[:, :, ::-1].copy(), dt)
        blob = oracle.encode(kb, vb, dt, level)
        (kmeta, kcodes, vmeta, vcodes), = split_blob(blob, 1, n, 128, level)
        qk, qv = unpack(kcodes, b), unpack(vcodes, b)
        for which, bits_, q in (("K", kb[0], qk), ("V", vb[0], qv)):
            for t in range(n):
                for ch in range(128):
                    grp = bits_[:, ch] if which == "K" else bits_[t, :]
                    fr = [frac_of(g, dt) for g in grp]
                    mn, mx = min(fr), max(fr)
                    r = mx - mn
                    xx = frac_of(bits_[t, ch], dt)
                    if r == 0:
                        assert q[t, ch] == 0
                        continue
                    errs = [abs(xx - (mn + qq * r / L)) for qq in range(L + 1)]
                    best = min(errs)
                    args = [qq for qq in range(L + 1) if errs[qq] == best]
                    if len(args) > 1:
                        n_ties += 1
                        args = [qq for qq in args if qq % 2 == 0]
                    assert [int(q[t, ch])] == args, (which, t, ch)
    assert n_ties > 0


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("level", [0, 1, 2])
def test_codes_are_argmin_on_gaussian_data(level, dt):
    """Random data: the oracle's fp32 code is the exact-arithmetic argmin unless the exact
    position is within 2^-18 of a cell boundary (where one fp32 rounding may decide)."""
    b = oracle.level_bits(level); L = (1 << b) - 1
    kb, vb = gen.make_kv(1, 3, 128, dt, 40 + level)
    blob = oracle.encode(kb, vb, dt, level)
    (kmeta, kcodes, vmeta, vcodes), = split_blob(blob, 1, 3, 128, level)
    qk, qv = unpack(kcodes, b), unpack(vcodes, b)
    for which, bits_, q in (("K", kb[0], qk), ("V", vb[0], qv)):
        for t in range(3):
            for ch in range(128):
                grp = bits_[:, ch] if which == "K" else bits_[t, :]
                fr = [frac_of(g, dt) for g in grp]
                mn, mx = min(fr), max(fr)
                r = mx - mn
                pos = (frac_of(bits_[t, ch], dt) - mn) * L / r          # exact position in [0, L]
                near = int(math.floor(pos + Fraction(1, 2)))
                if abs(pos - math.floor(pos) - Fraction(1, 2)) < Fraction(1, 2**18):
                    assert abs(int(q[t, ch]) - pos) <= Fraction(1, 2) + Fraction(1, 2**18)
                else:
                    assert int(q[t, ch]) == near, (which, t, ch, float(pos))


# ---------------------------------------------------------------------------------------------
# invariants on realistic data
# ---------------------------------------------------------------------------------------------
def _ulp(x, dt):
    """Spacing of the 16-bit grid at |x| (float64 arrays)."""
    p, emin = (10, -14) if dt == F16 else (7, -126)
    e = np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** emin)))
    return 2.0 ** (e - p)


def _group_scales(kmeta, vmeta, n, c, b, dt):
    """Exact (float64) step r / L of every element's group, as [n][c] arrays for K and V."""
    L = (1 << b) - 1
    rk = (val(kmeta[..., 1], dt) - val(kmeta[..., 0], dt)) / L          # [G][c]
    rv = (val(vmeta[..., 1], dt) - val(vmeta[..., 0], dt)) / L          # [n][c/128]
    return np.repeat(rk, 128, axis=0)[:n], np.repeat(rv, 128, axis=1)


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("level", [0, 1, 2])
def test_step_bound_endpoints_and_statistics(level, dt):
    l, n, c = 2, 300, 256   # ragged: the third K token-group holds 44 tokens
    b = oracle.level_bits(level)
    k, v = gen.make_kv(l, n, c, dt, 11)
    blob = oracle.encode(k, v, dt, level)
    kd, vd = oracle.decode(blob, dt, l, n, c, level)
    secs = split_blob(blob, l, n, c, level)
    for lam in range(l):
        kmeta, kcodes, vmeta, vcodes = secs[lam]
        xk, xv = val(k[lam], dt), val(v[lam], dt)
        # statistics are the true min / max of each group (numpy reductions as the independent side)
        for g in range(-(-n // 128)):
            seg = xk[128 * g:128 * g + 128]
            assert np.array_equal(val(kmeta[g, :, 0], dt), seg.min(axis=0))
            assert np.array_equal(val(kmeta[g, :, 1], dt), seg.max(axis=0))
        hv = xv.reshape(n, c // 128, 128)
        assert np.array_equal(val(vmeta[..., 0], dt), hv.min(axis=2))
        assert np.array_equal(val(vmeta[..., 1], dt), hv.max(axis=2))
        sk, sv = _group_scales(kmeta, vmeta, n, c, b, dt)
        for x, xh, s, q in ((xk, val(kd[lam], dt), sk, unpack(kcodes, b)), (xv, val(vd[lam], dt), sv, unpack(vcodes, b))):
            err = np.abs(x - xh)
            assert np.all(err <= s / 2 * (1 + 2.0 ** -10) + _ulp(xh, dt) / 2)
            L = (1 << b) - 1
            # code 0 decodes to the stored min, code L to the stored max
            assert np.all(xh[q == 0] <= x[q == 0]) and np.all(xh[q == L] >= x[q == L])
    # exact endpoints, stated directly: where x equals its group's min or max, decode is exact
    for lam in range(l):
        kmeta, kcodes, vmeta, vcodes = secs[lam]
        xk, xv = val(k[lam], dt), val(v[lam], dt)
        mnk = np.repeat(val(kmeta[..., 0], dt), 128, axis=0)[:n]; mxk = np.repeat(val(kmeta[..., 1], dt), 128, axis=0)[:n]
        mnv = np.repeat(val(vmeta[..., 0], dt), 128, axis=1); mxv = np.repeat(val(vmeta[..., 1], dt), 128, axis=1)
        for x, xh, mn, mx in ((xk, val(kd[lam], dt), mnk, mxk), (xv, val(vd[lam], dt), mnv, mxv)):
            ends = (x == mn) | (x == mx)
            assert ends.sum() >= 2 and np.array_equal(x[ends], xh[ends])
            assert np.all((xh >= mn) & (xh <= mx))


@pytest.mark.parametrize("dt", [F16, BF16])
def test_degenerate_groups_are_lossless(dt):
    x = np.zeros((1, 130, 256), dtype=np.float32)
    x[0, :, :128] = 3.5          # constant everywhere in channel-group 0
    x[0, :, 128:] = -0.0         # negative zeros: canonicalised to +0
    x[0, 5, 130] = 0.0
    kb = to_bits(x, dt)
    for level in range(3):
        blob = oracle.encode(kb, kb, dt, level)
        (kmeta, kcodes, vmeta, vcodes), = split_blob(blob, 1, 130, 256, level)
        assert not kcodes.any() and not vcodes.any()
        assert np.all(kmeta[:, 128:, :] == 0) and np.all(vmeta[:, 1, :] == 0)   # +0 bits, never 0x8000
        kd, vd = oracle.decode(blob, dt, 1, 130, 256, level)
        assert np.array_equal(val(kd, dt), val(kb, dt)) and np.array_equal(val(vd, dt), val(kb, dt))
        assert np.all(kd[0, :, 128:] == 0)
    # bf16 only: a range below 2^-100 is degenerate by definition and decodes to the minimum
    if dt == BF16:
        y = np.full((1, 128, 128), 2.0 ** -120, dtype=np.float32)
        y[0, 0, 0] = 2.0 ** -119
        yb = to_bits(y, dt)
        blob = oracle.encode(yb, yb, dt, 2)
        kd, vd = oracle.decode(blob, dt, 1, 128, 128, 2)
        assert np.all(val(kd, dt) == 2.0 ** -120) and np.all(val(vd, dt) == 2.0 ** -120)
        s, i, deg = oracle.group_params(int(to_bits(2.0 ** -120, dt)), int(to_bits(2.0 ** -119, dt)), dt, 2)
        assert (float(s), float(i), deg) == (0.0, 0.0, True)
        s, i, deg = oracle.group_params(int(to_bits(0.0, dt)), int(to_bits(2.0 ** -100, dt)), dt, 2)
        assert deg is False and float(s) == float(np.float32(2.0 ** -100) / np.float32(3))


def _reencode(blob, dt, l, n, c, level):
    kd, vd = oracle.decode(blob, dt, l, n, c, level)
    return oracle.encode(kd, vd, dt, level)


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("level", [0, 1, 2])
def test_idempotent_reencoding_realistic(level, dt):
    """E(D(E(x))) == E(x) byte for byte on workload-shaped data (with a ragged tail)."""
    l, n, c = 2, 333, 384
    k, v = gen.make_kv(l, n, c, dt, 21)
    blob = oracle.encode(k, v, dt, level)
    again = _reencode(blob, dt, l, n, c, level)
    assert np.array_equal(blob, again)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_idempotent_reencoding_tiny_random(dt):
    rng = np.random.default_rng(99 + dt)
    for trial in range(400):
        n = int(rng.integers(1, 6))
        sig = float(np.exp(rng.normal(0, 3)))
        x = (rng.standard_normal((1, n, 128)) * sig + rng.normal(0, 1) * sig * rng.integers(0, 3)).astype(np.float32)
        kb = gen._cast_to_bits(x, dt)
        for level in range(3):
            blob = oracle.encode(kb, kb, dt, level)
            assert np.array_equal(blob, _reencode(blob, dt, 1, n, 128, level)), (trial, level)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_idempotent_reencoding_adversarial(dt):
    """Power-of-two ranges, two-valued groups, range ~ L ulps, range ~ 1 ulp, tiny max vs wide range."""
    p = 10 if dt == F16 else 7
    groups = []
    for e in (-6, 0, 5):
        base = 2.0 ** e
        groups.append(np.linspace(base, 2 * base, 128))                       # power-of-two range
        groups.append(np.where(np.arange(128) % 2 == 0, base, base * (1 + 2.0 ** -p)))   # two values, 1 ulp apart
        groups.append(base * (1 + np.arange(128) % 4 * 2.0 ** -p))            # range = 3 ulps
        groups.append(base * (1 + np.arange(128) % 16 * 2.0 ** -p))           # range = 15 ulps
        groups.append(base * (1 + np.arange(128) * 2.0 ** -p))                # range = 127 ulps
        groups.append(np.concatenate([[-base * 1000, base * 2.0 ** -9], np.linspace(-base * 1000, 0, 126)]))  # |mx| << r
        groups.append(np.concatenate([[-base, base], np.linspace(-base, base, 126)]))
    x = np.stack(groups).astype(np.float32)                  # [G][128]
    xb = gen._cast_to_bits(x, dt)
    G = xb.shape[0]
    v = xb.reshape(1, G, 128)                                # V: each row one group
    k = np.zeros((1, 128, 128), dtype=np.uint16)
    k[0, :, :G] = xb.T                                       # K: each channel one group
    for level in range(3):
        bk = oracle.encode(k, k, dt, level)
        assert np.array_equal(bk, _reencode(bk, dt, 1, 128, 128, level)), ("K", level)
        bv = oracle.encode(v, v, dt, level)
        assert np.array_equal(bv, _reencode(bv, dt, 1, G, 128, level)), ("V", level)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_error_is_monotone_across_levels(dt):
    l, n, c = 2, 256, 256
    k, v = gen.make_kv(l, n, c, dt, 31)
    rms, mxe = [], []
    for level in range(3):
        kd, vd = oracle.decode(oracle.encode(k, v, dt, level), dt, l, n, c, level)
        e = np.concatenate([(val(kd, dt) - val(k, dt)).ravel(), (val(vd, dt) - val(v, dt)).ravel()])
        rms.append(float(np.sqrt(np.mean(e * e)))); mxe.append(float(np.abs(e).max()))
    assert rms[0] <= rms[1] <= rms[2] and mxe[0] <= mxe[1] <= mxe[2]
    assert rms[2] > 3 * rms[1] > 9 * rms[0] * (0.2 if dt == BF16 else 1.0)


@pytest.mark.parametrize("level", [0, 1])
def test_rms_error_matches_uniform_quantiser_closed_form(level):
    """fp16 Gaussian data: RMS of (x - x_hat) / step tends to 1 / sqrt(12)."""
    l, n, c, dt = 2, 512, 256, F16
    b = oracle.level_bits(level)
    k, v = gen.make_kv(l, n, c, dt, 41)
    blob = oracle.encode(k, v, dt, level)
    kd, vd = oracle.decode(blob, dt, l, n, c, level)
    secs = split_blob(blob, l, n, c, level)
    z = []
    for lam in range(l):
        kmeta, _, vmeta, _ = secs[lam]
        sk, sv = _group_scales(kmeta, vmeta, n, c, b, dt)
        z.append(((val(kd[lam], dt) - val(k[lam], dt)) / sk).ravel())
        z.append(((val(vd[lam], dt) - val(v[lam], dt)) / sv).ravel())
    z = np.concatenate(z)
    assert abs(float(np.sqrt(np.mean(z * z))) * math.sqrt(12) - 1.0) < 0.05


# ---------------------------------------------------------------------------------------------
# special cases
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("level", [0, 1, 2])
def test_k_v_duality_on_transposed_tile(level, dt):
    """n = c = 128 and V = K^T: K group (channel j) and V group (token j) hold the same values."""
    k, _ = gen.make_kv(1, 128, 128, dt, 51)
    v = np.ascontiguousarray(k.transpose(0, 2, 1))
    blob = oracle.encode(k, v, dt, level)
    (kmeta, kcodes, vmeta, vcodes), = split_blob(blob, 1, 128, 128, level)
    b = oracle.level_bits(level)
    assert np.array_equal(kmeta[0], vmeta[:, 0])
    assert np.array_equal(unpack(kcodes, b), unpack(vcodes, b).T)
    kd, vd = oracle.decode(blob, dt, 1, 128, 128, level)
    assert np.array_equal(kd[0], vd[0].T)


@pytest.mark.parametrize("level", [0, 2])
def test_paged_scatter_special_cases(level):
    dt, l, n, c, bt = BF16, 2, 200, 128, 16
    k, v = gen.make_kv(l, n, c, dt, 61)
    blob = oracle.encode(k, v, dt, level)
    kc, vc = oracle.decode(blob, dt, l, n, c, level)
    P = -(-n // bt)
    # identity table == contiguous decode
    kp = np.zeros((l, P, bt, c), dtype=np.uint16); vp = np.zeros_like(kp)
    assert oracle.decode_into(blob, dt, l, n, c, level, kp, vp, 0, np.arange(P, dtype=np.int32), bt) == 0
    assert np.array_equal(kp.reshape(l, P * bt, c)[:, :n], kc) and np.array_equal(vp.reshape(l, P * bt, c)[:, :n], vc)
    assert not kp.reshape(l, P * bt, c)[:, n:].any()
    # random permutation in a larger pool, shifted start; inverse gather == contiguous decode
    rng = np.random.default_rng(3)
    pool, t0 = 40, 32
    table = rng.permutation(pool).astype(np.int32)[: (t0 + n + bt - 1) // bt]
    kp = np.full((l, pool, bt, c), 0xABCD, dtype=np.uint16); vp = np.full_like(kp, 0xABCD)
    assert oracle.decode_into(blob, dt, l, n, c, level, kp, vp, t0, table, bt) == 0
    s = np.arange(t0, t0 + n)
    assert np.array_equal(kp[:, table[s // bt], s % bt], kc) and np.array_equal(vp[:, table[s // bt], s % bt], vc)
    touched = np.zeros((pool, bt), dtype=bool); touched[table[s // bt], s % bt] = True
    assert np.all(kp[:, ~touched] == 0xABCD) and np.all(vp[:, ~touched] == 0xABCD)


def test_chunks_are_independent():
    """Encoding tokens [a, b) alone equals the corresponding slice semantics: decode(encode(slice)) == slice decode."""
    dt, l, n, c = F16, 2, 512, 128
    k, v = gen.make_kv(l, n, c, dt, 71)
    whole_k, whole_v = oracle.decode(oracle.encode(k, v, dt, 1), dt, l, n, c, 1)
    for t0 in (0, 256):
        bk = oracle.encode(k[:, t0:t0 + 256], v[:, t0:t0 + 256], dt, 1)   # strided views of the big tensor
        ck, cv = oracle.decode(bk, dt, l, 256, c, 1)
        assert np.array_equal(ck, whole_k[:, t0:t0 + 256]) and np.array_equal(cv, whole_v[:, t0:t0 + 256])


@pytest.mark.parametrize("dt", [F16, BF16])
def test_dequantise_rounds_once_in_fp32_then_once_to_t16(dt):
    """Reconstruction = T16_rne(f32_rne(q * scale + mn)) with the product NOT rounded on its own.

    The exact value q * scale + mn is formed with Fractions; whenever it fits a float64 exactly,
    numpy's float64 -> float32 cast is the single fp32 rounding, and numpy / torch give the final
    16-bit rounding.  A separately rounded product differs on some of these cases.
    """
    import torch

    rng = np.random.default_rng(5 + dt)
    checked = differs_from_unfused = 0
    for trial in range(300):
        sig = float(np.exp(rng.normal(0, 2)))
        pair = gen._cast_to_bits(np.sort(rng.standard_normal(2) * sig).astype(np.float32), dt)
        mn, mx = int(pair[0]), int(pair[1])
        if mn == mx:
            continue
        for b in (8, 4, 2):
            L = (1 << b) - 1
            scale, inv, deg = oracle.group_params(mn, mx, dt, b)
            assert not deg
            # scale itself: one correctly rounded fp32 division of the fp32 difference
            r32 = np.float32(float(val(np.uint16(mx), dt))) - np.float32(float(val(np.uint16(mn), dt)))
            r_exact = Fraction(float(r32)) / L
            assert abs(Fraction(float(scale)) - r_exact) <= abs(Fraction(float(np.spacing(scale)))) / 2
            fmn = frac_of(mn, dt)
            for q in range(1, L):
                exact = q * Fraction(float(scale)) + fmn
                as64 = float(exact)
                if Fraction(as64) != exact:
                    continue
                y32 = np.float32(as64)
                if dt == F16:
                    want = int(np.array(y32).astype(np.float16).view(np.uint16))
                else:
                    want = int(torch.tensor(float(y32), dtype=torch.float32).to(torch.bfloat16).view(torch.int16).item()) & 0xFFFF
                assert oracle.dequantise(q, mn, mx, dt, b) == want, (hex(mn), hex(mx), b, q)
                checked += 1
                unfused = np.float32(np.float32(q) * scale) + np.float32(float(val(np.uint16(mn), dt)))
                differs_from_unfused += int(unfused != y32)
    assert checked > 10000 and differs_from_unfused > 0
