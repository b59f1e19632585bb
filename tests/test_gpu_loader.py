"""GPU parity of the load path (kvh_loader_*): blobs in pinned host memory, copied through a ring of device
staging slots and decoded, against the CPU oracle's decode of the same blobs.  Bar: reconstructed values as raw
16-bit patterns, bit for bit.  Blobs are the ORACLE's."""
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


def to_host(t) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def make_entries(dt, l, c, lens, levels, seed):
    """Oracle blobs (pinned) of consecutive pieces of one context, and the oracle's decode of the whole."""
    N = sum(lens)
    k, v = gen.make_kv(l, N, c, dt, seed=seed)
    blobs, want_k, want_v, t0s = [], np.zeros_like(k), np.zeros_like(v), []
    t0 = 0
    for n, lv in zip(lens, levels):
        b = oracle.encode(np.ascontiguousarray(k[:, t0:t0 + n]), np.ascontiguousarray(v[:, t0:t0 + n]), dt, lv)
        dk, dv = oracle.decode(b, dt, l, n, c, lv)
        want_k[:, t0:t0 + n], want_v[:, t0:t0 + n] = dk, dv
        blobs.append(torch.from_numpy(b).pin_memory())
        t0s.append(t0)
        t0 += n
    return blobs, t0s, want_k, want_v, N


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("n_slots", [1, 2, 3])
def test_pipelined_load_matches_oracle(kvh, n_slots, dt):
    l, c = 2, 256
    lens = [256, 130, 256, 1, 384, 77, 256]
    levels = [0, 2, 1, 0, 2, 1, 2]
    blobs, t0s, want_k, want_v, N = make_entries(dt, l, c, lens, levels, seed=60 + n_slots)
    slot = max(b.numel() for b in blobs)
    # slots that hold the largest blob plus the descriptor area: groups of one to a few blobs, several ring turns
    staging = torch.empty(n_slots * (slot + 1536), dtype=torch.uint8, device="cuda")
    ld = kvh.Loader(staging, n_slots)
    assert slot <= ld.slot_bytes < slot + 1536
    ok = torch.full((l, N, c), 3.0, dtype=TDT[dt], device="cuda"); ov = torch.full_like(ok, 3.0)
    status = torch.zeros(len(lens), dtype=torch.int32, device="cuda")
    ld.run(blobs, lens, levels, t0s, ok, ov, status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0] * len(lens)
    assert np.array_equal(to_host(ok), want_k) and np.array_equal(to_host(ov), want_v)
    # a second run on the same loader (slots are reused across runs), in reverse order, into a fresh destination
    ok2 = torch.zeros_like(ok); ov2 = torch.zeros_like(ov)
    ld.run(blobs[::-1], lens[::-1], levels[::-1], t0s[::-1], ok2, ov2, status=status)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(ok2), want_k) and np.array_equal(to_host(ov2), want_v)
    ld.close()


def test_pipelined_load_paged_and_header_mismatch(kvh):
    dt, l, c, bt = BF16, 2, 128, 16
    lens, levels = [64, 48, 80], [1, 0, 2]
    blobs, t0s, want_k, want_v, N = make_entries(dt, l, c, lens, levels, seed=70)
    P = N // bt
    table = np.random.default_rng(1).permutation(P + 3).astype(np.int32)[:P]
    pk = np.zeros((l, P + 3, bt, c), np.uint16); pv = np.zeros_like(pk)
    for lv, b, n, t0 in zip(levels, blobs, lens, t0s):
        assert oracle.decode_into(b.numpy(), dt, l, n, c, lv, pk, pv, dst_token0=t0, page_table=table, block_tokens=bt) == 0
    gk = torch.zeros((l, P + 3, bt, c), dtype=torch.bfloat16, device="cuda"); gv = torch.zeros_like(gk)
    tab = torch.from_numpy(table).cuda()
    staging = torch.empty(2 * (max(b.numel() for b in blobs) + 1536), dtype=torch.uint8, device="cuda")
    ld = kvh.Loader(staging, 2)
    status = torch.zeros(3, dtype=torch.int32, device="cuda")
    ld.run(blobs, lens, levels, t0s, gk, gv, page_tables=[tab] * 3, block_tokens=bt, status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0, 0]
    assert np.array_equal(to_host(gk), pk) and np.array_equal(to_host(gv), pv)
    # item 1 claims the wrong level: it alone reports a mismatch and writes nothing
    gk.zero_(); gv.zero_(); status.zero_()
    wrong = list(levels); wrong[1] = 1
    bigger = [blobs[0], torch.cat([blobs[1], torch.zeros(16, dtype=torch.uint8)]).pin_memory(), blobs[2]]
    ld.run(bigger, lens, wrong, t0s, gk, gv, page_tables=[tab] * 3, block_tokens=bt, status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 1, 0]
    exp_k = pk.copy(); exp_v = pv.copy()
    for s in range(t0s[1], t0s[1] + lens[1]):
        exp_k[:, table[s // bt], s % bt] = 0; exp_v[:, table[s // bt], s % bt] = 0
    assert np.array_equal(to_host(gk), exp_k) and np.array_equal(to_host(gv), exp_v)
    ld.close()


def test_loader_argument_errors(kvh):
    staging = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(kvh.KVHError):
        kvh.Loader(staging, 0)
    with pytest.raises(kvh.KVHError):
        kvh.Loader(staging, 65)
    with pytest.raises(kvh.KVHError):
        kvh.Loader(staging[:32], 2)  # slots smaller than a header
    ld = kvh.Loader(staging, 2)
    k = torch.zeros((1, 256, 128), dtype=torch.float16, device="cuda")
    big = torch.zeros(kvh.blob_size(1, 256, 128, 0), dtype=torch.uint8).pin_memory()
    with pytest.raises(kvh.KVHError):  # a 67,648-byte blob does not fit a 32 KiB slot
        ld.run([big], [256], [0], [0], k, k.clone())
    with pytest.raises(kvh.KVHError):
        ld.run([big], [256], [5], [0], k, k.clone())
    with pytest.raises(ValueError):  # pageable host memory is refused by the binding
        ld.run([torch.zeros(100, dtype=torch.uint8)], [1], [0], [0], k, k.clone())
    # ... and by the library itself (the copy kernel would read it in place)
    import ctypes
    from paper_2509_00105_amd.binding import LOAD_ITEM, _KVView
    pageable = np.zeros(kvh.blob_size(1, 1, 128, 0) + 16, dtype=np.uint8)
    a = np.zeros(1, dtype=LOAD_ITEM)
    a["blob_host"], a["n_tokens"] = (pageable.ctypes.data + 15) & ~15, 1
    view = _KVView(k.data_ptr(), k.data_ptr(), k.stride(0), k.stride(1))
    assert kvh.lib().kvh_loader_run(ld._h, a.ctypes.data, 1, 0, 1, 128, ctypes.byref(view), 16, None, None) == -1
    ld.close()
    torch.cuda.synchronize()


def test_store_path_encode_straight_into_pinned_host_memory(kvh):
    """The store direction needs no staging at all: a blob pointer may be any memory the device can write, so the
    encoder writes its blobs straight into pinned host memory (the DRAM tier).  Byte for byte the oracle's blobs."""
    dt, l, c, chunk = BF16, 2, 1024, 256
    lens, levels = [256, 256, 130], [2, 0, 1]
    N = sum(lens)
    k, v = gen.make_kv(l, N, c, dt, seed=81)
    kd = torch.from_numpy(k.view(np.int16)).cuda().view(torch.bfloat16)
    vd = torch.from_numpy(v.view(np.int16)).cuda().view(torch.bfloat16)
    sizes = [kvh.blob_size(l, n, c, lv) for n, lv in zip(lens, levels)]
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    host = torch.full((int(sum(sizes)),), 0xEE, dtype=torch.uint8).pin_memory()
    t0s = np.concatenate([[0], np.cumsum(lens)[:-1]])
    items = kvh.make_enc_items([host.data_ptr() + int(o) for o in offs], t0s, lens, levels, "cuda")
    kvh.encode_batch(items, 3, chunk, kd, vd)
    torch.cuda.synchronize()
    got = host.numpy()
    for o, s, t0, n, lv in zip(offs, sizes, t0s, lens, levels):
        want = oracle.encode(np.ascontiguousarray(k[:, t0:t0 + n]), np.ascontiguousarray(v[:, t0:t0 + n]), dt, lv)
        assert np.array_equal(got[o:o + s], want), (t0, n, lv)
    # and the fused transcode can demote a blob from HBM straight to the host tier
    dev_blob = torch.from_numpy(got[offs[1]:offs[1] + sizes[1]].copy()).cuda()
    low = torch.empty(kvh.blob_size(l, lens[1], c, 2), dtype=torch.uint8).pin_memory()
    kvh.transcode(dev_blob, torch.bfloat16, l, lens[1], c, 0, 2, out=low)
    torch.cuda.synchronize()
    assert np.array_equal(low.numpy(), oracle.transcode(got[offs[1]:offs[1] + sizes[1]], dt, l, lens[1], c, 0, 2))


def test_loader_takes_token_dropped_blobs(kvh):
    """Ordinary and token-dropped blobs mixed in one run of the loader."""
    dt, l, c = F16, 2, 256
    N, sink, window = 400, 16, 150
    k, v = gen.make_kv(l, N + 256, c, dt, seed=91)
    kept_blob = oracle.encode_kept(np.ascontiguousarray(k[:, :N]), np.ascontiguousarray(v[:, :N]), dt, sink, window, 2)
    plain_blob = oracle.encode(np.ascontiguousarray(k[:, N:]), np.ascontiguousarray(v[:, N:]), dt, 0)
    n_kept = oracle.kept_tokens(N, sink, window)
    wk = np.full((l, N + 256, c), 0x2222, np.uint16); wv = wk.copy()
    assert oracle.decode_kept_into(kept_blob, dt, l, N, c, sink, window, 2, wk, wv) == 0
    assert oracle.decode_into(plain_blob, dt, l, 256, c, 0, wk, wv, dst_token0=N) == 0
    gk = torch.from_numpy(np.full((l, N + 256, c), 0x2222, np.uint16).view(np.int16)).cuda().view(torch.float16)
    gv = gk.clone()
    blobs = [torch.from_numpy(kept_blob).pin_memory(), torch.from_numpy(plain_blob).pin_memory()]
    staging = torch.empty(2 * (max(b.numel() for b in blobs) + 1536), dtype=torch.uint8, device="cuda")
    ld = kvh.Loader(staging, 2)
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    ld.run(blobs, [n_kept, 256], [2, 0], [0, N], gk, gv, status=status, drops=[(N, sink, window, False), None])
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0]
    assert np.array_equal(to_host(gk), wk) and np.array_equal(to_host(gv), wv)
    with pytest.raises(kvh.KVHError):  # n_tokens that is not what the drop words keep
        ld.run(blobs[:1], [n_kept - 1], [2], [0], gk, gv, drops=[(N, sink, window, False)])
    ld.close()


def test_store_then_load_on_one_stream_without_a_sync_between(kvh):
    """Stream order across the two directions: blobs encoded straight into pinned host memory on a stream are
    loaded back by a run enqueued on the same stream right after, with no host synchronisation in between."""
    dt, l, c, chunk = BF16, 4, 1024, 256
    n_chunks = 12
    N = n_chunks * chunk
    levels = [i % 3 for i in range(n_chunks)]
    k, v = gen.make_kv(l, N, c, dt, seed=97)
    kd = torch.from_numpy(k.view(np.int16)).cuda().view(torch.bfloat16)
    vd = torch.from_numpy(v.view(np.int16)).cuda().view(torch.bfloat16)
    sizes = [kvh.blob_size(l, chunk, c, lv) for lv in levels]
    host = [torch.full((s,), 0xEE, dtype=torch.uint8).pin_memory() for s in sizes]
    items = kvh.make_enc_items([h.data_ptr() for h in host], [i * chunk for i in range(n_chunks)], [chunk] * n_chunks,
                               levels, "cuda")
    staging = torch.empty(2 * (2 * max(sizes) + 1536), dtype=torch.uint8, device="cuda")
    ld = kvh.Loader(staging, 2)
    ok = torch.zeros((l, N, c), dtype=torch.bfloat16, device="cuda"); ov = torch.zeros_like(ok)
    status = torch.zeros(n_chunks, dtype=torch.int32, device="cuda")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        kvh.encode_batch(items, n_chunks, chunk, kd, vd, stream=s)
        ld.run(host, [chunk] * n_chunks, levels, [i * chunk for i in range(n_chunks)], ok, ov, status=status, stream=s)
    s.synchronize()
    assert status.cpu().tolist() == [0] * n_chunks
    wk, wv = np.zeros_like(k), np.zeros_like(v)
    for i, lv in enumerate(levels):
        sl = slice(i * chunk, (i + 1) * chunk)
        b = oracle.encode(np.ascontiguousarray(k[:, sl]), np.ascontiguousarray(v[:, sl]), dt, lv)
        assert np.array_equal(host[i].numpy(), b), ("stored blob", i)
        wk[:, sl], wv[:, sl] = oracle.decode(b, dt, l, chunk, c, lv)
    assert np.array_equal(to_host(ok), wk) and np.array_equal(to_host(ov), wv)
    ld.close()
