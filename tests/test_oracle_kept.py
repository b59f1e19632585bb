"""CPU-only pins of the oracle's token-dropping functions (the paper's second compression method:
keep the beginning and the end of an entry; Introduction and the fixed-rate token-dropping baseline of
Preliminary Results).  The paper gives no definition, so the pins are: hand-typed kept positions,
equality with an explicit numpy gather followed by the ordinary (already pinned) encoder, the
degenerate case sink + window >= N, scatter checks against numpy indexing, and header checks."""
import struct

import numpy as np
import pytest

import kv_inputs as gen
import oracle

F16, BF16 = gen.F16, gen.BF16


def kept_positions(N, sink, window):
    if sink + window >= N:
        return list(range(N))
    return list(range(sink)) + list(range(N - window, N))


def test_kept_positions_typed_by_hand():
    assert kept_positions(10, 2, 3) == [0, 1, 7, 8, 9]
    assert oracle.kept_tokens(10, 2, 3) == 5
    assert oracle.kept_tokens(10, 0, 3) == 3 and oracle.kept_tokens(10, 4, 0) == 4
    assert oracle.kept_tokens(10, 6, 6) == 10 and oracle.kept_tokens(10, 10, 0) == 10
    assert oracle.kept_tokens(10, 0, 0) == 0 and oracle.kept_tokens(0, 1, 1) == 0 and oracle.kept_tokens(5, -1, 3) == 0
    # a 5-token entry of distinct constant rows, sink 1 + window 2: rows 0, 3, 4 come back at their places
    x = np.repeat(np.arange(1, 6, dtype=np.float32)[None, :, None], 128, axis=2)
    kb = x.astype(np.float16).view(np.uint16)
    blob = oracle.encode_kept(kb, kb, F16, 1, 2, 2)
    out = np.full((1, 5, 128), 0x7777, dtype=np.uint16); outv = out.copy()
    assert oracle.decode_kept_into(blob, F16, 1, 5, 128, 1, 2, 2, out, outv) == 0
    kvals = out.view(np.float16)[0, :, 0].astype(np.float64)
    vvals = outv.view(np.float16)[0, :, 0].astype(np.float64)
    assert list(out[0, 1:3, 0]) == [0x7777, 0x7777] and list(outv[0, 1:3, 0]) == [0x7777, 0x7777]
    # V groups (one token's channels) are constant: exact.  K groups (one channel over the three kept tokens) span
    # 1..5: with 2 bits the step is 4/3, 4.0 sits at 2.25 steps -> code 2 -> fp16(1 + 2 * 4/3) = 3.666015625
    assert list(vvals[[0, 3, 4]]) == [1.0, 4.0, 5.0]
    assert list(kvals[[0, 3, 4]]) == [1.0, 3.666015625, 5.0]


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("N,sink,window", [(300, 4, 124), (515, 128, 200), (130, 1, 1), (64, 100, 100), (200, 0, 37)])
def test_encode_kept_is_gather_then_encode(N, sink, window, dt):
    l, c = 2, 256
    k, v = gen.make_kv(l, N, c, dt, seed=N + sink)
    pos = kept_positions(N, sink, window)
    for level in range(3):
        blob = oracle.encode_kept(k, v, dt, sink, window, level)
        plain = oracle.encode(np.ascontiguousarray(k[:, pos]), np.ascontiguousarray(v[:, pos]), dt, level)
        assert blob.size == plain.size == oracle.blob_size(l, len(pos), c, level)
        assert struct.unpack_from("<III", blob, 32) == (N, sink, window) and not blob[44:64].any()
        assert struct.unpack_from("<I", blob, 12)[0] == len(pos)
        same = blob.copy(); same[32:44] = 0
        assert np.array_equal(same, plain)


@pytest.mark.parametrize("compact", [False, True])
def test_decode_kept_scatters_to_the_right_rows(compact):
    dt, l, N, c, sink, window, level = BF16, 2, 300, 128, 5, 70, 1
    k, v = gen.make_kv(l, N, c, dt, seed=3)
    pos = np.array(kept_positions(N, sink, window))
    blob = oracle.encode_kept(k, v, dt, sink, window, level)
    plain = blob.copy(); plain[32:44] = 0
    wk, wv = oracle.decode(plain, dt, l, len(pos), c, level)
    t0 = 16
    kd = np.full((l, t0 + N + 3, c), 0xBEEF, dtype=np.uint16); vd = kd.copy()
    assert oracle.decode_kept_into(blob, dt, l, N, c, sink, window, level, kd, vd, t0, compact) == 0
    rows = t0 + (np.arange(len(pos)) if compact else pos)
    assert np.array_equal(kd[:, rows], wk) and np.array_equal(vd[:, rows], wv)
    mask = np.ones(kd.shape[1], dtype=bool); mask[rows] = False
    assert np.all(kd[:, mask] == 0xBEEF) and np.all(vd[:, mask] == 0xBEEF)
    # paged, original positions
    bt, pool = 16, 40
    table = np.random.default_rng(0).permutation(pool).astype(np.int32)[: -(-(t0 + N) // bt)]
    kp = np.full((l, pool, bt, c), 0xBEEF, dtype=np.uint16); vp = kp.copy()
    assert oracle.decode_kept_into(blob, dt, l, N, c, sink, window, level, kp, vp, t0, compact, table, bt) == 0
    assert np.array_equal(kp[:, table[rows // bt], rows % bt], wk) and np.array_equal(vp[:, table[rows // bt], rows % bt], wv)


def test_kept_header_is_checked():
    dt, l, N, c = F16, 1, 200, 128
    k, v = gen.make_kv(l, N, c, dt, seed=5)
    blob = oracle.encode_kept(k, v, dt, 8, 56, 0)
    kd = np.zeros((l, N, c), dtype=np.uint16); vd = kd.copy()
    assert oracle.decode_kept_into(blob, dt, l, N, c, 8, 56, 0, kd, vd) == oracle.OK
    assert oracle.decode_kept_into(blob, dt, l, N, c, 56, 8, 0, kd, vd) == oracle.E_HEADER       # same count, other split
    assert oracle.decode_kept_into(blob, dt, l, N + 1, c, 8, 56, 0, kd, vd) == oracle.E_HEADER
    assert oracle.decode_into(blob, dt, l, 64, c, 0, kd, vd) == oracle.E_HEADER                   # not a plain blob
    plain = oracle.encode(k[:, :64], v[:, :64], dt, 0)
    assert oracle.decode_kept_into(plain, dt, l, N, c, 8, 56, 0, kd, vd) == oracle.E_HEADER       # not a dropped blob
    assert oracle.decode_kept_into(blob, dt, l, N, c, 8, 56, 1, kd, vd) == oracle.E_HEADER
