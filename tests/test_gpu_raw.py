"""GPU parity of the raw level (level 3: an entry stored in full quality) against the CPU oracle: blobs byte for
byte, decoded rows bit for bit, through the single, batched, chunked, token-dropping and load-path calls."""
import numpy as np
import pytest

import kv_inputs as gen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

F16, BF16 = gen.F16, gen.BF16
TDT = {F16: torch.float16, BF16: torch.bfloat16}
RAW = 3


@pytest.fixture(scope="module")
def kvh():
    import paper_2509_00105_amd as m

    m.lib()
    return m


def to_dev(bits: np.ndarray, dt: int):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(TDT[dt])


def to_host(t) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("shape", [(1, 1, 128), (2, 300, 256), (3, 130, 384), (2, 257, 1024), (1, 515, 640), (1, 64, 2048)])
def test_raw_encode_and_decode_match_oracle(kvh, shape, dt):
    l, n, c = shape
    k, v = gen.make_kv(l, n, c, dt, seed=300 + n)
    assert kvh.level_bits(RAW) == 16 and kvh.blob_size(l, n, c, RAW) == oracle.blob_size(l, n, c, RAW)
    want = oracle.encode(k, v, dt, RAW)
    blob = kvh.encode(to_dev(k, dt), to_dev(v, dt), RAW)
    ok = torch.zeros((l, n, c), dtype=TDT[dt], device="cuda"); ov = torch.zeros_like(ok)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode(torch.from_numpy(want).cuda(), RAW, n, ok, ov, status=status)
    torch.cuda.synchronize()
    assert np.array_equal(blob.cpu().numpy(), want)
    assert status.item() == 0 and np.array_equal(to_host(ok), k) and np.array_equal(to_host(ov), v)


def test_every_bit_pattern_survives_on_the_gpu(kvh):
    allbits = np.arange(65536, dtype=np.uint16).reshape(1, 512, 128)
    other = allbits[:, ::-1].copy()
    for dt in (F16, BF16):
        want = oracle.encode(allbits, other, dt, RAW)
        blob = kvh.encode(to_dev(allbits, dt), to_dev(other, dt), RAW)
        ok = torch.zeros((1, 512, 128), dtype=TDT[dt], device="cuda"); ov = torch.zeros_like(ok)
        kvh.decode(blob, RAW, 512, ok, ov)
        torch.cuda.synchronize()
        assert np.array_equal(blob.cpu().numpy(), want)
        assert np.array_equal(to_host(ok), allbits) and np.array_equal(to_host(ov), other)


def test_raw_items_in_batched_chunked_and_paged_calls(kvh):
    dt, l, N, c, chunk, bt = BF16, 2, 900, 1024, 256, 16
    k, v = gen.make_kv(l, N, c, dt, seed=310)
    kd, vd = to_dev(k, dt), to_dev(v, dt)
    levels = [RAW, 0, RAW, 2]                                   # the last chunk holds 132 tokens
    lens = [min(chunk, N - i * chunk) for i in range(4)]
    sizes = [kvh.blob_size(l, n, c, lv) for n, lv in zip(lens, levels)]
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    want = [oracle.encode(k[:, i * chunk:i * chunk + lens[i]], v[:, i * chunk:i * chunk + lens[i]], dt, lv) for i, lv in enumerate(levels)]
    for how in ("batch", "chunked"):
        blobs = torch.zeros(int(sum(sizes)), dtype=torch.uint8, device="cuda")
        if how == "batch":
            items = kvh.make_enc_items([blobs.data_ptr() + int(o) for o in offs], [i * chunk for i in range(4)], lens, levels, "cuda")
            kvh.encode_batch(items, 4, chunk, kd, vd)
        else:
            kvh.encode_chunked(kd, vd, chunk, levels, blobs, offs)
        torch.cuda.synchronize()
        assert np.array_equal(blobs.cpu().numpy(), np.concatenate(want)), how
    # decode: one batched launch into a paged cache, and the chunked form into a contiguous one
    n_pages = -(-N // bt)
    perm = np.random.default_rng(5).permutation(n_pages).astype(np.int32)
    tab = torch.from_numpy(perm).cuda()
    pk = torch.zeros((l, n_pages, bt, c), dtype=TDT[dt], device="cuda"); pv = torch.zeros_like(pk)
    status = torch.zeros(4, dtype=torch.int32, device="cuda")
    ditems = kvh.make_dec_items([blobs.data_ptr() + int(o) for o in offs], lens, levels, [i * chunk for i in range(4)],
                                [tab.data_ptr()] * 4, "cuda")
    kvh.decode_batch(ditems, 4, chunk, pk, pv, paged=True, block_tokens=bt, status=status)
    ck = torch.zeros((l, N, c), dtype=TDT[dt], device="cuda"); cv = torch.zeros_like(ck)
    kvh.decode_chunked(blobs, offs, levels, chunk, N, ck, cv, status=status)
    torch.cuda.synchronize()
    assert not status.any()
    inv = torch.from_numpy(perm.astype(np.int64)).cuda()
    gk, gv = pk[:, inv].reshape(l, -1, c)[:, :N], pv[:, inv].reshape(l, -1, c)[:, :N]
    for i, lv in enumerate(levels):
        wk, wv = oracle.decode(want[i], dt, l, lens[i], c, lv)
        sl = slice(i * chunk, i * chunk + lens[i])
        for tk, tv in ((gk, gv), (ck, cv)):
            assert np.array_equal(to_host(tk[:, sl]), wk) and np.array_equal(to_host(tv[:, sl]), wv), i
    # a quantised blob decoded as raw (and the other way round) is a header mismatch that writes nothing
    sent = torch.full((l, chunk, c), 5.0, dtype=TDT[dt], device="cuda"); sent2 = sent.clone()
    st1 = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode(blobs[int(offs[0]):int(offs[0]) + sizes[0]], 0, chunk, sent, sent2, status=st1)
    torch.cuda.synchronize()
    assert st1.item() == 1 and bool((sent == 5.0).all()) and bool((sent2 == 5.0).all())


def test_token_dropping_without_quantisation(kvh):
    dt, l, N, c, sink, window = F16, 2, 700, 256, 100, 200
    k, v = gen.make_kv(l, N, c, dt, seed=320)
    want = oracle.encode_kept(k, v, dt, sink, window, RAW)
    blob = kvh.encode_kept(to_dev(k, dt), to_dev(v, dt), sink, window, RAW)
    ok = torch.full((l, N, c), 2.0, dtype=TDT[dt], device="cuda"); ov = ok.clone()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode_kept(blob, RAW, N, sink, window, ok, ov, status=status)
    torch.cuda.synchronize()
    assert np.array_equal(blob.cpu().numpy(), want) and status.item() == 0
    wk = to_host(torch.full((l, N, c), 2.0, dtype=TDT[dt])); wv = wk.copy()
    assert oracle.decode_kept_into(want, dt, l, N, c, sink, window, RAW, wk, wv) == 0
    assert np.array_equal(to_host(ok), wk) and np.array_equal(to_host(ov), wv)


def test_load_path_takes_raw_blobs(kvh):
    dt, l, c = BF16, 4, 256
    lens, levels = [256, 130, 77], [RAW, 1, RAW]
    N = sum(lens)
    k, v = gen.make_kv(l, N, c, dt, seed=330)
    blobs, t0s, t0 = [], [], 0
    wk, wv = np.zeros_like(k), np.zeros_like(v)
    for n, lv in zip(lens, levels):
        b = oracle.encode(np.ascontiguousarray(k[:, t0:t0 + n]), np.ascontiguousarray(v[:, t0:t0 + n]), dt, lv)
        wk[:, t0:t0 + n], wv[:, t0:t0 + n] = oracle.decode(b, dt, l, n, c, lv)
        blobs.append(torch.from_numpy(b).pin_memory()); t0s.append(t0); t0 += n
    staging = torch.empty(2 * (max(b.numel() for b in blobs) + 1536), dtype=torch.uint8, device="cuda")
    ld = kvh.Loader(staging, 2)
    for which in ("loader", "static"):
        ok = torch.zeros((l, N, c), dtype=TDT[dt], device="cuda"); ov = torch.zeros_like(ok)
        status = torch.zeros(3, dtype=torch.int32, device="cuda")
        if which == "loader":
            ld.run(blobs, lens, levels, t0s, ok, ov, status=status)
        else:
            kvh.load_static(blobs, lens, levels, t0s, ok, ov, status=status)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [0, 0, 0]
        assert np.array_equal(to_host(ok), wk) and np.array_equal(to_host(ov), wv), which
    ld.close()


@pytest.mark.parametrize("level", [0, 1, 2])
def test_compressing_a_raw_blob_further_is_an_encode_of_its_rows(kvh, level):
    """The policy lowers a full-quality entry to a quantised level: kvh_encode on a view of the raw blob's rows
    gives, byte for byte, the oracle's transcode raw -> level (decode, then encode); the fused transcode call itself
    refuses the raw level, on the host for a single call and on the device for a batch item."""
    dt, l, n, c = BF16, 3, 300, 512
    k, v = gen.make_kv(l, n, c, dt, seed=340)
    raw = oracle.encode(k, v, dt, RAW)
    want = oracle.transcode(raw, dt, l, n, c, RAW, level)
    raw_dev = torch.from_numpy(raw).cuda()
    rows = raw_dev[64:].view(TDT[dt]).view(l, 2, n, c)          # per layer: K rows, then V rows
    got = kvh.encode(rows[:, 0], rows[:, 1], level)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want)
    with pytest.raises(kvh.KVHError) as e:
        kvh.transcode(raw_dev, dt, l, n, c, RAW, level)
    assert e.value.status == -2
    dst = torch.full((want.size,), 0x77, dtype=torch.uint8, device="cuda")
    items = kvh.make_tc_items([raw_dev.data_ptr()], [dst.data_ptr()], [n], [RAW], [level], "cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.transcode_batch(items, 1, n, dt, l, c, status=status)
    torch.cuda.synchronize()
    assert status.item() == 1 and (dst.cpu().numpy() == 0x77).all()
