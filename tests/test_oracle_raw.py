"""CPU pins of the oracle's raw level (level 3: an entry stored in full quality, the third of the choices the
paper's greedy step has per entry — evict, store in full quality, compress; Design section).  The level is a
plain definition — rows stored as they are — so the pins are that definition written out with numpy: byte
offsets typed by hand, every 16-bit pattern surviving, and the composed calls (paged decode, token dropping,
transcode) equal to the same numpy gather / scatter / the quantised calls on the stored rows."""
import struct

import numpy as np
import pytest

import kv_inputs as gen
import oracle

F16, BF16 = gen.F16, gen.BF16
RAW = 3


def test_level_table_and_size():
    assert oracle.level_bits(RAW) == 16 and oracle.num_levels() == 3      # three quantised levels; 3 is the raw one
    for l, n, c in [(1, 1, 128), (2, 5, 128), (3, 130, 384), (32, 256, 1024)]:
        assert oracle.blob_size(l, n, c, RAW) == 64 + l * 2 * n * c * 2
    assert oracle.blob_size(1, 1, 64, RAW) == 0 and oracle.blob_size(0, 1, 128, RAW) == 0
    off = oracle.section_offsets(2, 5, 128, RAW, 1)
    per_layer = 2 * 5 * 128 * 2
    assert (off["kmeta"], off["kcodes"], off["vmeta"], off["vcodes"], off["row_bytes"]) == \
           (64 + per_layer, 64 + per_layer, 64 + per_layer + 5 * 128 * 2, 64 + per_layer + 5 * 128 * 2, 256)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_rows_are_stored_as_they_are(dt):
    l, n, c = 3, 7, 256
    k, v = gen.make_kv(l, n, c, dt, seed=31)
    blob = oracle.encode(k, v, dt, RAW)
    assert blob.size == 64 + l * 2 * n * c * 2
    # header: magic, version 1, dtype, bits = 16, l, n, c, group sizes, total bytes, zero drop words
    assert bytes(blob[:4]) == b"KVH1" and struct.unpack_from("<HBB", blob, 4) == (1, dt, 16)
    assert struct.unpack_from("<IIIHHQ", blob, 8) == (l, n, c, 128, 128, blob.size)
    assert not blob[32:64].any()
    # body: per layer the K rows, then the V rows, little-endian 16-bit values
    body = blob[64:].view("<u2").reshape(l, 2, n, c)
    assert np.array_equal(body[:, 0], k) and np.array_equal(body[:, 1], v)
    # one value by a hand-typed offset: layer 2, V, token 4, channel 9
    o = 64 + 2 * (2 * n * c * 2) + n * c * 2 + (4 * c + 9) * 2
    assert int(blob[o]) | int(blob[o + 1]) << 8 == int(v[2, 4, 9])
    dk, dv = oracle.decode(blob, dt, l, n, c, RAW)
    assert np.array_equal(dk, k) and np.array_equal(dv, v)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_every_bit_pattern_survives(dt):
    """All 65,536 patterns, infinities, NaNs and -0 included: the raw level has no finiteness precondition."""
    allbits = np.arange(65536, dtype=np.uint16).reshape(1, 512, 128)
    other = allbits[:, ::-1].copy()
    blob = oracle.encode(allbits, other, dt, RAW)                  # strict: would raise on any error status
    dk, dv = oracle.decode(blob, dt, 1, 512, 128, RAW)
    assert np.array_equal(dk, allbits) and np.array_equal(dv, other)


def test_strided_views_offsets_and_page_tables():
    dt, l, n, c, bt = BF16, 2, 37, 128, 4
    big_k, big_v = gen.make_kv(l, 64, 2 * c, dt, seed=32)
    k, v = big_k[:, 5:5 + n, c:], big_v[:, 5:5 + n, c:]              # token and channel offsets, non-dense strides
    blob = oracle.encode(k, v, dt, RAW)
    assert np.array_equal(blob[64:].view("<u2").reshape(l, 2, n, c)[:, 0], k)
    # contiguous destination at a token offset
    dk = np.full((l, 50, c), 7, np.uint16); dv = dk.copy()
    assert oracle.decode_into(blob, dt, l, n, c, RAW, dk, dv, dst_token0=9) == 0
    assert np.array_equal(dk[:, 9:9 + n], k) and (dk[:, :9] == 7).all() and (dk[:, 9 + n:] == 7).all()
    # paged destination through a permuted table, logical offset 2
    P = -(-(n + 2) // bt)
    table = np.random.default_rng(0).permutation(P + 2).astype(np.int32)[:P]
    pk = np.zeros((l, P + 2, bt, c), np.uint16); pv = np.zeros_like(pk)
    assert oracle.decode_into(blob, dt, l, n, c, RAW, pk, pv, dst_token0=2, page_table=table, block_tokens=bt) == 0
    for t in range(n):
        s = t + 2
        assert np.array_equal(pk[:, table[s // bt], s % bt], k[:, t]) and np.array_equal(pv[:, table[s // bt], s % bt], v[:, t])
    assert pk.astype(bool).sum() <= k.astype(bool).sum()


def test_errors_and_header_checks():
    dt, l, n, c = F16, 1, 3, 128
    k, v = gen.make_kv(l, n, c, dt, seed=33)
    blob = oracle.encode(k, v, dt, RAW)
    dk = np.zeros((l, n, c), np.uint16); dv = dk.copy()
    assert oracle.decode_into(blob, dt, l, n, c, 0, dk, dv) == -7          # a raw blob is not an 8-bit one
    assert oracle.decode_into(blob, BF16, l, n, c, RAW, dk, dv) == -7      # wrong dtype in the header
    assert oracle.decode_into(blob, dt, l, n - 1, c, RAW, dk, dv) == -7    # wrong token count
    q = oracle.encode(k, v, dt, 0)
    big = np.concatenate([q, np.zeros(blob.size, np.uint8)])
    assert oracle.decode_into(big, dt, l, n, c, RAW, dk, dv) == -7         # a quantised blob is not a raw one
    assert not dk.any() and not dv.any()
    assert oracle.encode_rc(k, v, dt, 4, np.zeros(1 << 16, np.uint8)) == -2
    assert oracle.encode_rc(k, v, dt, RAW, np.zeros(blob.size - 1, np.uint8)) == -4


def test_token_dropping_at_the_raw_level_is_a_pure_gather():
    """Dropping without quantisation: the kept rows, unchanged, and back at their positions on decode."""
    dt, l, N, c, sink, window = F16, 2, 40, 128, 3, 10
    k, v = gen.make_kv(l, N, c, dt, seed=34)
    blob = oracle.encode_kept(k, v, dt, sink, window, RAW)
    kept = list(range(sink)) + list(range(N - window, N))
    assert struct.unpack_from("<III", blob, 32) == (N, sink, window) and struct.unpack_from("<I", blob, 12) == (len(kept),)
    body = blob[64:].view("<u2").reshape(l, 2, len(kept), c)
    assert np.array_equal(body[:, 0], k[:, kept]) and np.array_equal(body[:, 1], v[:, kept])
    dk = np.full((l, N, c), 9, np.uint16); dv = dk.copy()
    assert oracle.decode_kept_into(blob, dt, l, N, c, sink, window, RAW, dk, dv) == 0
    assert np.array_equal(dk[:, kept], k[:, kept]) and (dk[:, sink:N - window] == 9).all()


@pytest.mark.parametrize("level", [0, 1, 2])
def test_transcode_to_and_from_the_raw_level(level):
    """raw -> b is the quantised encode of the stored rows; b -> raw stores what the decoder reconstructs;
    raw -> raw is the identity."""
    dt, l, n, c = BF16, 2, 200, 256
    k, v = gen.make_kv(l, n, c, dt, seed=35)
    raw = oracle.encode(k, v, dt, RAW)
    assert np.array_equal(oracle.transcode(raw, dt, l, n, c, RAW, level), oracle.encode(k, v, dt, level))
    assert np.array_equal(oracle.transcode(raw, dt, l, n, c, RAW, RAW), raw)
    q = oracle.encode(k, v, dt, level)
    dk, dv = oracle.decode(q, dt, l, n, c, level)
    assert np.array_equal(oracle.transcode(q, dt, l, n, c, level, RAW), oracle.encode(dk, dv, dt, RAW))
