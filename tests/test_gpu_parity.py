"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar: blobs (header, metadata, packed codes, padding) byte-for-byte equal; reconstructed values
compared as raw 16-bit patterns.  The contractual tolerance on reconstructed values is 1 ulp of
the output dtype; both sides take every decision in fp32 with the same operation order, so the
tests assert the stronger bit equality and only fall back to reporting the ulp distance in the
failure message.
"""
import numpy as np
import pytest

import kv_inputs as gen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

F16, BF16 = gen.F16, gen.BF16
TDT = {F16: torch.float16, BF16: torch.bfloat16}


@pytest.fixture(scope="module")
def kvh():
    import paper_2509_00105_amd as m

    m.lib()
    return m


def to_dev(bits: np.ndarray, dt: int):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(TDT[dt])


def to_host(t) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def assert_same_bits(got: np.ndarray, want: np.ndarray, dt: int, what: str):
    if np.array_equal(got, want):
        return
    bad = np.argwhere(got != want)
    g, w = gen.bits_to_f64(got[got != want], dt), gen.bits_to_f64(want[got != want], dt)
    raise AssertionError("%s: %d of %d elements differ; first at %s: got %r want %r (max |diff| %g)"
                         % (what, bad.shape[0], got.size, tuple(bad[0]), g[0], w[0], np.max(np.abs(g - w))))


def assert_same_blob(got: np.ndarray, want: np.ndarray, what: str):
    assert got.size == want.size, (what, got.size, want.size)
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        raise AssertionError("%s: %d of %d blob bytes differ; first at offset %d: got 0x%02x want 0x%02x"
                             % (what, bad.size, got.size, bad[0], got[bad[0]], want[bad[0]]))


SHAPES = [
    (1, 1, 128),      # a single token: one-element K groups (all degenerate)
    (2, 300, 256),    # ragged: the third K token-group holds 44 tokens; half-filled strip
    (3, 130, 384),    # c not a power of two; vmeta needs padding (130 * 3 * 4 = 1560 bytes)
    (2, 257, 1024),   # two full strips, one token past two groups
    (1, 515, 640),    # second strip a quarter full; several tiles and a tail
    (1, 64, 2048),    # four strips
]


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("level", [0, 1, 2])
@pytest.mark.parametrize("shape", SHAPES)
def test_encode_and_decode_match_oracle(kvh, shape, level, dt):
    l, n, c = shape
    k, v = gen.make_kv(l, n, c, dt, seed=100 + l + n + c)
    want_blob = oracle.encode(k, v, dt, level)
    want_k, want_v = oracle.decode(want_blob, dt, l, n, c, level)

    kd, vd = to_dev(k, dt), to_dev(v, dt)
    assert kvh.blob_size(l, n, c, level) == want_blob.size
    blob = kvh.encode(kd, vd, level)
    torch.cuda.synchronize()
    assert_same_blob(blob.cpu().numpy(), want_blob, "encode %s level %d" % (shape, level))

    # decode the ORACLE's blob, so a decoder fault cannot hide behind an encoder fault
    out_k = torch.full((l, n, c), 7.0, dtype=TDT[dt], device="cuda")
    out_v = torch.full((l, n, c), 7.0, dtype=TDT[dt], device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode(torch.from_numpy(want_blob).cuda(), level, n, out_k, out_v, status=status)
    torch.cuda.synchronize()
    assert status.item() == 0
    assert_same_bits(to_host(out_k), want_k, dt, "decode K %s level %d" % (shape, level))
    assert_same_bits(to_host(out_v), want_v, dt, "decode V %s level %d" % (shape, level))


@pytest.mark.parametrize("dt", [F16, BF16])
def test_special_values_match_oracle(kvh, dt):
    """Constant groups, signed zeros, subnormals, 1-ulp ranges, tiny max against a wide range, ties."""
    p = 10 if dt == F16 else 7
    tiny = 2.0 ** -24 if dt == F16 else 2.0 ** -133
    rows = []
    for base in (2.0 ** -6, 1.0, 32.0):
        rows += [np.full(128, base), np.linspace(base, 2 * base, 128),
                 np.where(np.arange(128) % 2 == 0, base, base * (1 + 2.0 ** -p)),
                 base * (1 + np.arange(128) % 4 * 2.0 ** -p), base * (1 + np.arange(128) * 2.0 ** -p),
                 np.concatenate([[-base * 1000, base * 2.0 ** -9], np.linspace(-base * 1000, 0, 126)]),
                 np.concatenate([[-1.0, 2.0], np.tile([-0.5, 0.25, 0.5, 1.25], 32)[:126]]) * base,
                 np.concatenate([[0.0, 15.0], np.tile([7.5, 8.5, 3.0, 0.5, 1.5, 2.5], 21)]) * base]
    rows += [np.zeros(128), -np.zeros(128), np.where(np.arange(128) % 2 == 0, 0.0, -0.0),
             np.arange(128) * tiny, (np.arange(128) - 64) * tiny, np.where(np.arange(128) < 3, tiny, 0.0)]
    x = np.stack(rows).astype(np.float64)
    G = x.shape[0]
    xb = gen._cast_to_bits(x.astype(np.float32), dt)
    if dt == BF16:  # float32 cannot hold 2^-133 multiples exactly above its own subnormal grid: build the bits directly
        xb[-3] = np.arange(128).astype(np.uint16)                      # bf16 subnormals 0 .. 127 * 2^-133
        xb[-2] = np.where(np.arange(128) < 64, 0x8000 | (64 - np.arange(128)), np.arange(128) - 64).astype(np.uint16)
        xb[-1] = np.where(np.arange(128) < 3, 1, 0).astype(np.uint16)
    v = np.ascontiguousarray(np.broadcast_to(xb[None], (2, G, 128)))
    k = np.zeros((2, 128, 128), dtype=np.uint16)
    k[:, :, :G] = xb.T[None]
    for level in range(3):
        for name, (a, b_), n in (("groups along tokens", (k, k), 128), ("groups along channels", (v, v), G)):
            want_blob = oracle.encode(a, b_, dt, level)
            blob = kvh.encode(to_dev(a, dt), to_dev(b_, dt), level)
            torch.cuda.synchronize()
            assert_same_blob(blob.cpu().numpy(), want_blob, "%s level %d" % (name, level))
            wk, wv = oracle.decode(want_blob, dt, 2, n, 128, level)
            ok = torch.zeros((2, n, 128), dtype=TDT[dt], device="cuda"); ov = torch.zeros_like(ok)
            kvh.decode(blob, level, n, ok, ov)
            torch.cuda.synchronize()
            assert_same_bits(to_host(ok), wk, dt, name + " K"); assert_same_bits(to_host(ov), wv, dt, name + " V")


@pytest.mark.parametrize("level", [0, 1, 2])
def test_worked_examples_on_gpu(kvh, level):
    """The hand-computed 2-bit example, scaled copies of it, through the HIP path."""
    x = np.full((1, 128, 128), 0.25, dtype=np.float32)
    x[0, 3, :4] = [-1.0, -0.5, 0.25, 2.0]
    kb = gen._cast_to_bits(x, F16)
    blob = kvh.encode(to_dev(kb, F16), to_dev(kb, F16), level)
    torch.cuda.synchronize()
    assert_same_blob(blob.cpu().numpy(), oracle.encode(kb, kb, F16, level), "worked example")
    if level == 2:
        so = oracle.section_offsets(1, 128, 128, 2, 0)
        assert blob[so["vcodes"] + 3 * so["row_bytes"]].item() == 0xD0


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("level", [0, 2])
def test_paged_decode_matches_oracle(kvh, level, dt):
    l, n, c, bt, pool, t0 = 2, 333, 256, 16, 40, 48
    k, v = gen.make_kv(l, n, c, dt, seed=7)
    blob = oracle.encode(k, v, dt, level)
    rng = np.random.default_rng(1)
    table = rng.permutation(pool).astype(np.int32)[: -(-(t0 + n) // bt)]
    wk = np.full((l, pool, bt, c), 0x1234, dtype=np.uint16); wv = np.full_like(wk, 0x1234)
    assert oracle.decode_into(blob, dt, l, n, c, level, wk, wv, t0, table, bt) == 0
    gk, gv = to_dev(np.full_like(wk, 0x1234), dt), to_dev(np.full_like(wk, 0x1234), dt)
    kvh.decode(torch.from_numpy(blob).cuda(), level, n, gk, gv, dst_token0=t0,
               page_table=torch.from_numpy(table).cuda(), block_tokens=bt)
    torch.cuda.synchronize()
    assert_same_bits(to_host(gk), wk, dt, "paged K"); assert_same_bits(to_host(gv), wv, dt, "paged V")


def test_paged_decode_with_odd_block_size(kvh):
    l, n, c, bt, dt, level = 1, 100, 128, 12, F16, 1
    k, v = gen.make_kv(l, n, c, dt, seed=8)
    blob = oracle.encode(k, v, dt, level)
    table = np.random.default_rng(2).permutation(12).astype(np.int32)
    wk = np.zeros((l, 12, bt, c), dtype=np.uint16); wv = np.zeros_like(wk)
    assert oracle.decode_into(blob, dt, l, n, c, level, wk, wv, 5, table, bt) == 0
    gk, gv = to_dev(np.zeros_like(wk), dt), to_dev(np.zeros_like(wk), dt)
    kvh.decode(torch.from_numpy(blob).cuda(), level, n, gk, gv, 5, torch.from_numpy(table).cuda(), bt)
    torch.cuda.synchronize()
    assert_same_bits(to_host(gk), wk, dt, "K"); assert_same_bits(to_host(gv), wv, dt, "V")


def test_contiguous_decode_at_token_offset_and_strided_views(kvh):
    """Chunks of one long entry: encode from a strided slice, decode back at dst_token0."""
    dt, l, N, c, chunk = BF16, 2, 640, 256, 256
    k, v = gen.make_kv(l, N, c, dt, seed=9)
    kv = torch.stack([to_dev(k, dt), to_dev(v, dt)])          # [2][l][N][c], K and V halves of one tensor
    out = torch.zeros_like(kv)
    for t0, level in ((0, 0), (256, 2), (512, 1)):
        n = min(chunk, N - t0)
        want = oracle.encode(k[:, t0:t0 + n], v[:, t0:t0 + n], dt, level)
        blob = kvh.encode(kv[0][:, t0:], kv[1][:, t0:], level, n_tokens=n)
        torch.cuda.synchronize()
        assert_same_blob(blob.cpu().numpy(), want, "chunk at %d" % t0)
        kvh.decode(blob, level, n, out[0], out[1], dst_token0=t0)
        wk, wv = oracle.decode(want, dt, l, n, c, level)
        torch.cuda.synchronize()
        assert_same_bits(to_host(out[0][:, t0:t0 + n]), wk, dt, "K"); assert_same_bits(to_host(out[1][:, t0:t0 + n]), wv, dt, "V")


def test_chunked_and_batched_encode_match_per_chunk_oracle(kvh):
    dt, l, N, c, chunk = F16, 2, 900, 256, 256     # 4 chunks, the last holds 132 tokens
    k, v = gen.make_kv(l, N, c, dt, seed=10)
    kd, vd = to_dev(k, dt), to_dev(v, dt)
    levels = [2, 0, 1, 2]
    sizes = [kvh.blob_size(l, min(chunk, N - i * chunk), c, lv) for i, lv in enumerate(levels)]
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    want = [oracle.encode(k[:, i * chunk:(i + 1) * chunk], v[:, i * chunk:(i + 1) * chunk], dt, lv) for i, lv in enumerate(levels)]

    blobs = torch.zeros(int(sum(sizes)), dtype=torch.uint8, device="cuda")
    kvh.encode_chunked(kd, vd, chunk, levels, blobs, offs)
    torch.cuda.synchronize()
    assert_same_blob(blobs.cpu().numpy(), np.concatenate(want), "encode_chunked")

    blobs2 = torch.zeros_like(blobs)
    items = kvh.make_enc_items([blobs2.data_ptr() + int(o) for o in offs], [i * chunk for i in range(4)],
                               [min(chunk, N - i * chunk) for i in range(4)], levels, "cuda")
    kvh.encode_batch(items, 4, chunk, kd, vd)
    torch.cuda.synchronize()
    assert_same_blob(blobs2.cpu().numpy(), np.concatenate(want), "encode_batch")

    # and back: one batched decode of the four mixed-level blobs into a contiguous tensor
    ok, ov = torch.zeros_like(kd), torch.zeros_like(vd)
    status = torch.zeros(4, dtype=torch.int32, device="cuda")
    ditems = kvh.make_dec_items([blobs2.data_ptr() + int(o) for o in offs], [min(chunk, N - i * chunk) for i in range(4)],
                                levels, [i * chunk for i in range(4)], [0] * 4, "cuda")
    kvh.decode_batch(ditems, 4, chunk, ok, ov, status=status)
    torch.cuda.synchronize()
    assert not status.any()
    # the chunked form: the same host arrays as descriptors, at a token offset, contiguous and paged
    base, bt = 32, 16
    sk = torch.zeros((l, base + N + 7, c), dtype=torch.float16, device="cuda"); sv = torch.zeros_like(sk)
    status.zero_()
    kvh.decode_chunked(blobs2, offs, levels, chunk, N, sk, sv, dst_token0=base, status=status)
    n_pages = -(-(base + N) // bt)
    perm = np.random.default_rng(12).permutation(n_pages).astype(np.int32)
    pk = torch.zeros((l, n_pages, bt, c), dtype=torch.float16, device="cuda"); pv = torch.zeros_like(pk)
    kvh.decode_chunked(blobs2, offs, levels, chunk, N, pk, pv, dst_token0=base, page_table=torch.from_numpy(perm).cuda(),
                       block_tokens=bt, status=status)
    torch.cuda.synchronize()
    assert not status.any()
    inv = torch.from_numpy(perm.astype(np.int64)).cuda()
    gk, gv = pk[:, inv].reshape(l, -1, c), pv[:, inv].reshape(l, -1, c)
    for i, lv in enumerate(levels):
        n = min(chunk, N - i * chunk)
        wk, wv = oracle.decode(want[i], dt, l, n, c, lv)
        assert_same_bits(to_host(ok[:, i * chunk:i * chunk + n]), wk, dt, "K chunk %d" % i)
        assert_same_bits(to_host(ov[:, i * chunk:i * chunk + n]), wv, dt, "V chunk %d" % i)
        for what, tk, tv in (("streamed", sk, sv), ("streamed paged", gk, gv)):
            assert_same_bits(to_host(tk[:, base + i * chunk:base + i * chunk + n]), wk, dt, "%s K chunk %d" % (what, i))
            assert_same_bits(to_host(tv[:, base + i * chunk:base + i * chunk + n]), wv, dt, "%s V chunk %d" % (what, i))
    assert not sk[:, :base].any() and not sk[:, base + N:].any()
    with pytest.raises(kvh.KVHError):
        kvh.decode_chunked(blobs2, offs, [2, 0, 1, 4], chunk, N, sk, sv)       # a level out of range: nothing launched
    with pytest.raises(kvh.KVHError):
        kvh.decode_chunked(blobs2, offs[:3], levels[:3], 320, N, sk, sv)        # chunk not a multiple of 128


def test_header_mismatch_sets_status_and_writes_nothing(kvh):
    dt, l, n, c = F16, 2, 200, 256
    k, v = gen.make_kv(l, n, c, dt, seed=11)
    blob = torch.from_numpy(oracle.encode(k, v, dt, 1)).cuda()
    ok = torch.full((l, n, c), 5.0, dtype=torch.float16, device="cuda"); ov = ok.clone()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode(blob, 2, n, ok, ov, status=status)          # stored at level 1, asked for level 2 (smaller reads)
    torch.cuda.synchronize()
    assert status.item() == 1 and bool((ok == 5.0).all()) and bool((ov == 5.0).all())
    status.zero_()
    kvh.decode(blob, 1, n - 1, ok, ov, status=status)      # wrong token count
    torch.cuda.synchronize()
    assert status.item() == 1 and bool((ok == 5.0).all())
    bad = blob.clone(); bad[0] = 0                         # broken magic
    kvh.decode(bad, 1, n, ok, ov, status=None)             # no status buffer: still writes nothing
    torch.cuda.synchronize()
    assert bool((ok == 5.0).all()) and bool((ov == 5.0).all())
    status.zero_()
    kvh.decode(blob, 1, n, ok, ov, status=status)
    torch.cuda.synchronize()
    assert status.item() == 0 and not bool((ok == 5.0).all())


def test_idempotent_reencoding_on_gpu(kvh):
    """E(D(E(x))) == E(x) byte for byte, entirely through the HIP path."""
    for dt in (F16, BF16):
        l, n, c = 2, 333, 384
        k, v = gen.make_kv(l, n, c, dt, seed=21)
        kd, vd = to_dev(k, dt), to_dev(v, dt)
        for level in range(3):
            blob = kvh.encode(kd, vd, level)
            ok, ov = torch.zeros_like(kd), torch.zeros_like(vd)
            kvh.decode(blob, level, n, ok, ov)
            again = kvh.encode(ok, ov, level)
            torch.cuda.synchronize()
            assert torch.equal(blob, again)


# ---------------------------------------------------------------------------------------------
# token dropping (keep the first `sink` and the last `window` tokens, encode them at a level)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("N,sink,window", [(300, 4, 124), (515, 128, 200), (130, 1, 1), (64, 100, 100), (700, 0, 257),
                                           (1000, 130, 0)])
def test_token_dropping_matches_oracle(kvh, N, sink, window, dt):
    l, c = 2, 640
    k, v = gen.make_kv(l, N, c, dt, seed=N + sink + window)
    kd, vd = to_dev(k, dt), to_dev(v, dt)
    n = oracle.kept_tokens(N, sink, window)
    assert kvh.kept_tokens(N, sink, window) == n
    for level in range(3):
        want = oracle.encode_kept(k, v, dt, sink, window, level)
        blob = kvh.encode_kept(kd, vd, sink, window, level)
        torch.cuda.synchronize()
        assert_same_blob(blob.cpu().numpy(), want, "encode_kept N=%d sink=%d window=%d level %d" % (N, sink, window, level))
        for compact in (False, True):
            wk = np.full((l, N + 40, c), 0x5A5A, dtype=np.uint16); wv = wk.copy()
            assert oracle.decode_kept_into(want, dt, l, N, c, sink, window, level, wk, wv, 24, compact) == 0
            gk, gv = to_dev(np.full_like(wk, 0x5A5A), dt), to_dev(np.full_like(wk, 0x5A5A), dt)
            status = torch.zeros(1, dtype=torch.int32, device="cuda")
            kvh.decode_kept(torch.from_numpy(want).cuda(), level, N, sink, window, gk, gv, dst_token0=24, compact=compact,
                            status=status)
            torch.cuda.synchronize()
            assert status.item() == 0
            assert_same_bits(to_host(gk), wk, dt, "decode_kept K compact=%s" % compact)
            assert_same_bits(to_host(gv), wv, dt, "decode_kept V compact=%s" % compact)


def test_token_dropping_paged_and_header_checks(kvh):
    dt, l, N, c, sink, window, level, bt, pool, t0 = BF16, 2, 400, 256, 20, 150, 2, 16, 40, 32
    k, v = gen.make_kv(l, N, c, dt, seed=77)
    want = oracle.encode_kept(k, v, dt, sink, window, level)
    blob = torch.from_numpy(want).cuda()
    table = np.random.default_rng(5).permutation(pool).astype(np.int32)[: -(-(t0 + N) // bt)]
    wk = np.full((l, pool, bt, c), 0x1111, dtype=np.uint16); wv = wk.copy()
    assert oracle.decode_kept_into(want, dt, l, N, c, sink, window, level, wk, wv, t0, False, table, bt) == 0
    gk, gv = to_dev(np.full_like(wk, 0x1111), dt), to_dev(np.full_like(wk, 0x1111), dt)
    kvh.decode_kept(blob, level, N, sink, window, gk, gv, dst_token0=t0, page_table=torch.from_numpy(table).cuda(),
                    block_tokens=bt)
    torch.cuda.synchronize()
    assert_same_bits(to_host(gk), wk, dt, "paged K"); assert_same_bits(to_host(gv), wv, dt, "paged V")
    # a dropped blob is not an ordinary blob, and the split must match
    n = kvh.kept_tokens(N, sink, window)
    ok = torch.full((l, N, c), 3.0, dtype=torch.bfloat16, device="cuda"); ov = ok.clone()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode(blob, level, n, ok, ov, status=status)
    torch.cuda.synchronize()
    assert status.item() == 1 and bool((ok == 3.0).all())
    status.zero_()
    kvh.decode_kept(blob, level, N, window, sink, ok, ov, status=status)
    torch.cuda.synchronize()
    assert status.item() == 1 and bool((ok == 3.0).all()) and bool((ov == 3.0).all())
    plain = torch.from_numpy(oracle.encode(k[:, :n], v[:, :n], dt, level)).cuda()
    status.zero_()
    kvh.decode_kept(plain, level, N, sink, window, ok, ov, status=status)
    torch.cuda.synchronize()
    assert status.item() == 1 and bool((ok == 3.0).all())


def test_token_dropping_batched_with_ordinary_items(kvh):
    """kvh_encode_kept_batch / kvh_decode_kept_batch: several entries with their own (N, sink, window) in one launch,
    an ordinary blob among the decode items, one compact item, one inconsistent item."""
    dt, l, c = BF16, 2, 256
    entries = [(300, 4, 124, 2), (515, 128, 200, 0), (130, 1, 1, 1), (64, 100, 100, 2), (257, 0, 129, 1)]  # N, sink, window, level
    starts = np.concatenate([[0], np.cumsum([e[0] for e in entries])[:-1]])
    total = int(sum(e[0] for e in entries))
    k, v = gen.make_kv(l, total, c, dt, seed=77)
    kd, vd = to_dev(k, dt), to_dev(v, dt)
    kept = [oracle.kept_tokens(N, s, w) for N, s, w, _ in entries]
    sizes = [kvh.blob_size(l, n, c, lv) for n, (_, _, _, lv) in zip(kept, entries)]
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    blobs = torch.zeros(int(sum(sizes)), dtype=torch.uint8, device="cuda")
    ptrs = [blobs.data_ptr() + int(o) for o in offs]
    items = kvh.make_kept_enc_items(ptrs, starts, [e[0] for e in entries], [e[1] for e in entries], [e[2] for e in entries],
                                    [e[3] for e in entries], "cuda")
    kvh.encode_kept_batch(items, len(entries), max(kept), kd, vd)
    torch.cuda.synchronize()
    got = blobs.cpu().numpy()
    wants = []
    for (N, s, w, lv), t0, o, sz in zip(entries, starts, offs, sizes):
        want = oracle.encode_kept(np.ascontiguousarray(k[:, t0:t0 + N]), np.ascontiguousarray(v[:, t0:t0 + N]), dt, s, w, lv)
        assert_same_blob(got[o:o + sz], want, "kept entry at %d" % t0)
        wants.append(want)

    # decode: entries 0..3 back to their places, entry 4 compact behind them, plus an ordinary blob and a bad item
    plain_k, plain_v = gen.make_kv(l, 200, c, dt, seed=78)
    plain = oracle.encode(plain_k, plain_v, dt, 1)
    plain_dev = torch.from_numpy(plain).cuda()
    rows = total + 200 + kept[4]
    wk = np.full((l, rows, c), 0x1111, np.uint16); wv = wk.copy()
    ok = to_dev(wk.copy(), dt); ov = to_dev(wv.copy(), dt)
    d_ptrs, d_n, d_lv, d_t0, d_orig, d_sink, d_win, d_comp = [], [], [], [], [], [], [], []
    for i, ((N, s, w, lv), t0) in enumerate(zip(entries, starts)):
        compact = i == 4
        dst = total + 200 if compact else int(t0)
        assert oracle.decode_kept_into(wants[i], dt, l, N, c, s, w, lv, wk, wv, dst_token0=dst, compact=compact) == 0
        d_ptrs.append(ptrs[i]); d_n.append(kept[i]); d_lv.append(lv); d_t0.append(dst)
        d_orig.append(N); d_sink.append(s); d_win.append(w); d_comp.append(int(compact))
    assert oracle.decode_into(plain, dt, l, 200, c, 1, wk, wv, dst_token0=total) == 0
    d_ptrs.append(plain_dev.data_ptr()); d_n.append(200); d_lv.append(1); d_t0.append(total)
    d_orig.append(0); d_sink.append(0); d_win.append(0); d_comp.append(0)
    # a seventh item whose n_tokens is not what (N, sink, window) keep: status 1, nothing written
    d_ptrs.append(ptrs[0]); d_n.append(kept[0] - 1); d_lv.append(entries[0][3]); d_t0.append(0)
    d_orig.append(entries[0][0]); d_sink.append(entries[0][1]); d_win.append(entries[0][2]); d_comp.append(0)
    ditems = kvh.make_kept_items(d_ptrs, d_n, d_lv, d_t0, [0] * 7, d_orig, d_sink, d_win, d_comp, "cuda")
    status = torch.zeros(7, dtype=torch.int32, device="cuda")
    kvh.decode_kept_batch(ditems, 7, max(d_n), ok, ov, status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0] * 6 + [1]
    assert_same_bits(to_host(ok), wk, dt, "K"); assert_same_bits(to_host(ov), wv, dt, "V")
