"""GPU parity at the full sizes of the five workload configurations, in the launch
configuration the benchmark times (batched launches over 256/512-token chunks).

Configs 1, 2 and 3 are compared with the oracle in full (config 3 chunk by chunk: 160 MiB at a
time goes back to the host).  Config 4 sends every 4th chunk plus the first and the last to the
oracle at both levels it runs; config 5 every ragged tail, every 4th chunk, the first and the
last.  Each test prints and asserts the fraction of chunk-levels the oracle saw.  On top of that
come properties that hold at any size: clean status words, exact idempotence of re-encoding on
the device, and agreement between the batched, streamed, contiguous and paged code paths.
"""
import concurrent.futures as cf
import os

import numpy as np
import pytest

import kv_inputs as gen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

F16, BF16 = gen.F16, gen.BF16
THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def kvh():
    import paper_2509_00105_amd as m

    m.lib()
    return m


def bits(t):
    """device 16-bit tensor -> host uint16 array"""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def chunk_plan(kvh, l, N, c, chunk, level_of_chunk):
    spans = [(t0, min(chunk, N - t0)) for t0 in range(0, N, chunk)]
    levels = [level_of_chunk(i) for i in range(len(spans))]
    sizes = [kvh.blob_size(l, n, c, lv) for (_, n), lv in zip(spans, levels)]
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.int64)
    return spans, levels, sizes, offs


def encode_all(kvh, kv, spans, levels, sizes, offs, chunk, token_base=0):
    blobs = torch.empty(int(sum(sizes)), dtype=torch.uint8, device="cuda")
    items = kvh.make_enc_items([blobs.data_ptr() + int(o) for o in offs], [token_base + t0 for t0, _ in spans],
                               [n for _, n in spans], levels, "cuda")
    kvh.encode_batch(items, len(spans), chunk, kv[0], kv[1])
    return blobs


def decode_all(kvh, blobs, spans, levels, offs, chunk, out, token_base=0):
    status = torch.zeros(len(spans), dtype=torch.int32, device="cuda")
    items = kvh.make_dec_items([blobs.data_ptr() + int(o) for o in offs], [n for _, n in spans], levels,
                               [token_base + t0 for t0, _ in spans], [0] * len(spans), "cuda")
    kvh.decode_batch(items, len(spans), chunk, out[0], out[1], status=status)
    torch.cuda.synchronize()
    assert int(status.abs().sum().item()) == 0
    return out


def oracle_check_chunks(kv, out, blobs, picks, spans, levels, sizes, offs, dt, l, c, token_base=0):
    """Copy the picked chunks back and compare blob bytes and decoded bits with the oracle (threaded; one batch of
    chunks on the host at a time).  Returns the number of chunks checked."""
    picks = list(picks)
    for lo in range(0, len(picks), THREADS):
        _oracle_check_batch(kv, out, blobs, picks[lo:lo + THREADS], spans, levels, sizes, offs, dt, l, c, token_base)
    return len(picks)


def _oracle_check_batch(kv, out, blobs, picks, spans, levels, sizes, offs, dt, l, c, token_base):
    jobs = []
    for i in picks:
        t0, n = spans[i]
        src = bits(kv[:, :, token_base + t0:token_base + t0 + n])
        got_blob = blobs[int(offs[i]):int(offs[i]) + sizes[i]].cpu().numpy()
        got_out = bits(out[:, :, token_base + t0:token_base + t0 + n]) if out is not None else None
        jobs.append((i, n, levels[i], src, got_blob, got_out))

    def run(job):
        i, n, level, src, got_blob, got_out = job
        want = oracle.encode(src[0], src[1], dt, level)
        if not np.array_equal(want, got_blob):
            return "chunk %d level %d: blob differs from the oracle" % (i, level)
        if got_out is not None:
            wk, wv = oracle.decode(want, dt, l, n, c, level)
            if not (np.array_equal(wk, got_out[0]) and np.array_equal(wv, got_out[1])):
                return "chunk %d level %d: decoded values differ from the oracle" % (i, level)
        return None

    with cf.ThreadPoolExecutor(max_workers=THREADS) as ex:
        errs = [e for e in ex.map(run, jobs) if e]
    assert not errs, errs


def test_config1_tiny_full_parity_and_invariants(kvh):
    cfg = gen.CONFIGS["tiny"]
    l, N, c, dt, chunk = cfg.l, cfg.n, cfg.c, cfg.dtype, cfg.chunk
    k, v = gen.make_kv(l, N, c, dt, cfg.seed)
    kv = torch.stack([torch.from_numpy(k.view(np.int16)).cuda(), torch.from_numpy(v.view(np.int16)).cuda()]).view(torch.float16)
    errs = []
    for level in range(3):
        spans, levels, sizes, offs = chunk_plan(kvh, l, N, c, chunk, lambda i: level)
        blobs = encode_all(kvh, kv, spans, levels, sizes, offs, chunk)
        out = decode_all(kvh, blobs, spans, levels, offs, chunk, torch.zeros_like(kv))
        oracle_check_chunks(kv, out, blobs, range(len(spans)), spans, levels, sizes, offs, dt, l, c)
        # idempotence, on the device
        again = encode_all(kvh, out, spans, levels, sizes, offs, chunk)
        torch.cuda.synchronize()
        assert torch.equal(blobs, again)
        e = (out.float() - kv.float())
        errs.append((float(e.pow(2).mean().sqrt()), float(e.abs().max())))
    assert errs[0][0] <= errs[1][0] <= errs[2][0] and errs[0][1] <= errs[1][1] <= errs[2][1]


def test_config2_llama3_8b_full_parity_in_bench_configuration(kvh):
    cfg = gen.CONFIGS["llama3_8b_8k"]
    l, N, c, dt, chunk = cfg.l, cfg.n, cfg.c, cfg.dtype, cfg.chunk
    kv = gen.make_kv_device(l, N, c, dt, cfg.seed)
    for level in range(3):
        spans, levels, sizes, offs = chunk_plan(kvh, l, N, c, chunk, lambda i: level)
        blobs = encode_all(kvh, kv, spans, levels, sizes, offs, chunk)
        out = decode_all(kvh, blobs, spans, levels, offs, chunk, torch.zeros_like(kv))
        oracle_check_chunks(kv, out, blobs, range(len(spans)), spans, levels, sizes, offs, dt, l, c)


def test_config3_llama3_70b_full_parity_and_idempotence(kvh):
    cfg = gen.CONFIGS["llama3_70b_32k"]
    l, N, c, dt, chunk = cfg.l, cfg.n, cfg.c, cfg.dtype, cfg.chunk
    kv = gen.make_kv_device(l, N, c, dt, cfg.seed, drift=True)
    out = torch.empty_like(kv)
    n_chunks = N // chunk
    seen = 0
    for level in range(3):
        spans, levels, sizes, offs = chunk_plan(kvh, l, N, c, chunk, lambda i: level)
        blobs = encode_all(kvh, kv, spans, levels, sizes, offs, chunk)
        decode_all(kvh, blobs, spans, levels, offs, chunk, out)
        seen += oracle_check_chunks(kv, out, blobs, range(n_chunks), spans, levels, sizes, offs, dt, l, c)
        print("config 3, %d bits: oracle checked %d of %d chunks (blob bytes and decoded bits)" % (kvh.level_bits(level), n_chunks, n_chunks), flush=True)
        again = encode_all(kvh, out, spans, levels, sizes, offs, chunk)
        torch.cuda.synchronize()
        assert torch.equal(blobs, again), "re-encoding the decoded tensor changed the blobs at level %d" % level
        del blobs, again
    assert seen == 3 * n_chunks  # oracle coverage of config 3: 192 of 192 chunk-levels


def test_config4_long_context_streamed_decode(kvh):
    cfg = gen.CONFIGS["long_7b_128k"]
    l, N, c, dt, chunk = cfg.l, cfg.n, cfg.c, cfg.dtype, cfg.chunk
    kv = gen.make_kv_device(l, N, c, dt, cfg.seed)
    n_chunks = N // chunk
    picks = sorted(set(range(0, n_chunks, 4)) | {n_chunks - 1})
    for level in (0, 2):
        spans, levels, sizes, offs = chunk_plan(kvh, l, N, c, chunk, lambda i: level)
        blobs = torch.empty(int(sum(sizes)), dtype=torch.uint8, device="cuda")
        kvh.encode_chunked(kv[0], kv[1], chunk, levels, blobs, offs)       # one launch per chunk, one stream
        batched = decode_all(kvh, blobs, spans, levels, offs, chunk, torch.empty_like(kv))
        streamed = torch.empty_like(kv)
        status = torch.zeros(n_chunks, dtype=torch.int32, device="cuda")
        kvh.decode_chunked(blobs, offs, levels, chunk, N, streamed[0], streamed[1], status=status)   # host-side descriptors, 32 chunks per launch
        torch.cuda.synchronize()
        assert int(status.abs().sum().item()) == 0
        assert torch.equal(streamed.view(torch.int16), batched.view(torch.int16))
        seen = oracle_check_chunks(kv, streamed, blobs, picks, spans, levels, sizes, offs, dt, l, c)
        print("config 4, %d bits: oracle checked %d of %d chunks (every 4th, first, last)" % (kvh.level_bits(level), seen, n_chunks), flush=True)
        assert seen >= n_chunks // 4 + 1  # oracle coverage of config 4: 129 of 512 chunks at each of its two levels
        del blobs, batched, streamed


def test_config5_mixed_batch_paged_decode(kvh):
    dt, l, c, chunk, bt = BF16, 32, 1024, 256, 16
    lengths = gen.mixed_batch_lengths()
    chunks, tables, n_pages = gen.mixed_batch_plan(lengths, chunk, bt)
    total = int(lengths.sum())
    starts = np.concatenate([[0], np.cumsum(lengths)[:-1]]).astype(np.int64)
    assert 64 == len(lengths) and lengths.min() >= 256 and lengths.max() <= 32768
    kv = gen.make_kv_device(l, total, c, dt, seed=4)                        # all requests back to back
    # encode every chunk of every request at its own level (one launch)
    req = [r for r, _, _, _ in chunks]
    spans = [(int(starts[r] + t0), n) for r, t0, n, _ in chunks]
    levels = [lv for _, _, _, lv in chunks]
    sizes = [kvh.blob_size(l, n, c, lv) for (_, n), lv in zip(spans, levels)]
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.int64)
    blobs = encode_all(kvh, kv, spans, levels, sizes, offs, chunk)
    # paged decode: one launch, each item carries its request's page table
    table_dev = torch.from_numpy(np.concatenate(tables)).cuda()
    table_start = np.concatenate([[0], np.cumsum([len(t) for t in tables])[:-1]])
    paged = torch.zeros((2, l, n_pages, bt, c), dtype=torch.bfloat16, device="cuda")
    status = torch.zeros(len(chunks), dtype=torch.int32, device="cuda")
    items = kvh.make_dec_items([blobs.data_ptr() + int(o) for o in offs], [n for _, n in spans], levels,
                               [t0 for _, t0, _, _ in chunks],
                               [table_dev.data_ptr() + 4 * int(table_start[r]) for r in req], "cuda")
    kvh.decode_batch(items, len(chunks), chunk, paged[0], paged[1], paged=True, block_tokens=bt, status=status)
    torch.cuda.synchronize()
    assert int(status.abs().sum().item()) == 0
    # contiguous decode of the same blobs, then gather the paged cache back into logical order: must agree everywhere
    contiguous = decode_all(kvh, blobs, spans, levels, offs, chunk, torch.empty_like(kv))
    for r in range(len(lengths)):
        n = int(lengths[r])
        tab = torch.from_numpy(tables[r].astype(np.int64)).cuda()
        got = paged[:, :, tab].reshape(2, l, -1, c)[:, :, :n]
        assert torch.equal(got.view(torch.int16), contiguous[:, :, int(starts[r]):int(starts[r]) + n].view(torch.int16)), r
    # no page outside the requests' tokens was written
    used = torch.zeros(n_pages * bt, dtype=torch.bool, device="cuda")
    for r in range(len(lengths)):
        s = torch.arange(int(lengths[r]), device="cuda")
        used[torch.from_numpy(tables[r].astype(np.int64)).cuda()[s // bt] * bt + s % bt] = True
    assert not paged.view(2, l, n_pages * bt, c)[:, :, ~used].any()
    # oracle: every ragged tail (a chunk shorter than 256 tokens), every 4th chunk, the first and the last
    ragged = [i for i, (_, n) in enumerate(spans) if n != chunk]
    picks = sorted(set(ragged) | set(range(0, len(spans), 4)) | {len(spans) - 1})
    seen = oracle_check_chunks(kv, contiguous, blobs, picks, spans, levels, sizes, offs, dt, l, c)
    by_level = [sum(1 for i in picks if levels[i] == lv) for lv in range(3)]
    print("config 5: oracle checked %d of %d chunks (%d ragged tails; %d / %d / %d at 8 / 4 / 2 bits)"
          % (seen, len(spans), len(ragged), by_level[0], by_level[1], by_level[2]), flush=True)
    assert seen >= len(spans) // 4 + len(ragged) // 2 and min(by_level) > 0 and len(ragged) >= 32


def test_config2_transcode_token_dropping_and_load_path_at_full_size(kvh):
    """The widened paths on the benchmark's workload and launch configuration: fused transcode of all 32 chunks
    (sampled chunks against the oracle's decode-then-encode; m -> m is the identity over every byte), token
    dropping of the whole 8192-token entry (sampled layers against the oracle), and the pipelined load path
    (bit-identical to the plain batched decode of the same blobs)."""
    cfg = gen.CONFIGS["llama3_8b_8k"]
    l, N, c, dt, chunk = cfg.l, cfg.n, cfg.c, cfg.dtype, cfg.chunk
    tdt = torch.float16 if dt == F16 else torch.bfloat16
    kv = gen.make_kv_device(l, N, c, dt, cfg.seed)
    n_chunks = N // chunk
    enc = {}
    for level in (0, 1):
        spans, levels, sizes, offs = chunk_plan(kvh, l, N, c, chunk, lambda i: level)
        enc[level] = (encode_all(kvh, kv, spans, levels, sizes, offs, chunk), sizes[0])
    torch.cuda.synchronize()

    # --- transcode ---
    for a, b in ((0, 1), (0, 2), (1, 2), (1, 1)):
        src, size_a = enc[a]
        size_b = kvh.blob_size(l, chunk, c, b)
        dst = torch.zeros(n_chunks * size_b, dtype=torch.uint8, device="cuda")
        status = torch.zeros(n_chunks, dtype=torch.int32, device="cuda")
        items = kvh.make_tc_items([src.data_ptr() + i * size_a for i in range(n_chunks)],
                                  [dst.data_ptr() + i * size_b for i in range(n_chunks)], [chunk] * n_chunks,
                                  [a] * n_chunks, [b] * n_chunks, "cuda")
        kvh.transcode_batch(items, n_chunks, chunk, tdt, l, c, status=status)
        torch.cuda.synchronize()
        assert int(status.abs().sum().item()) == 0
        if a == b:
            assert torch.equal(dst, src)
            continue
        for ci in (0, 13, n_chunks - 1):
            want = oracle.transcode(src[ci * size_a:(ci + 1) * size_a].cpu().numpy(), dt, l, chunk, c, a, b)
            assert np.array_equal(dst[ci * size_b:(ci + 1) * size_b].cpu().numpy(), want), (a, b, ci)

    # --- token dropping: the whole tensor as one entry, half of it kept ---
    sink, window = 128, N // 2 - 128
    n_kept = kvh.kept_tokens(N, sink, window)
    blob = kvh.encode_kept(kv[0], kv[1], sink, window, 2)
    out = torch.zeros_like(kv)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode_kept(blob, 2, N, sink, window, out[0], out[1], status=status)
    torch.cuda.synchronize()
    assert status.item() == 0
    assert not out[:, :, sink:N - window].any()  # dropped rows untouched
    host = bits(kv[:, [0, l - 1]])               # first and last layer through the oracle
    want_blob = oracle.encode_kept(host[0], host[1], dt, sink, window, 2)
    off_g = oracle.section_offsets(l, n_kept, c, 2, l - 1)
    off_w = oracle.section_offsets(2, n_kept, c, 2, 1)
    layer_bytes = (blob.numel() - 64) // l
    got = blob.cpu().numpy()
    assert np.array_equal(got[64:64 + layer_bytes], want_blob[64:64 + layer_bytes])
    assert np.array_equal(got[off_g["kmeta"]:off_g["kmeta"] + layer_bytes], want_blob[off_w["kmeta"]:off_w["kmeta"] + layer_bytes])
    wk = np.zeros((2, N, c), np.uint16); wv = np.zeros_like(wk)
    assert oracle.decode_kept_into(want_blob, dt, 2, N, c, sink, window, 2, wk, wv) == 0
    assert np.array_equal(bits(out[0][[0, l - 1]]), wk) and np.array_equal(bits(out[1][[0, l - 1]]), wv)

    # --- load path: 32 blobs from pinned host memory, two slots of four ---
    src, size = enc[0]
    spans, levels, sizes, offs = chunk_plan(kvh, l, N, c, chunk, lambda i: 0)
    plain = decode_all(kvh, src, spans, levels, offs, chunk, torch.zeros_like(kv))
    host_all = torch.empty(src.numel(), dtype=torch.uint8).pin_memory()
    host_all.copy_(src)
    staging = torch.empty(2 * (4 * size + 1536), dtype=torch.uint8, device="cuda")
    ld = kvh.Loader(staging, 2)
    piped = torch.zeros_like(kv)
    status = torch.zeros(n_chunks, dtype=torch.int32, device="cuda")
    ld.run([host_all[i * size:(i + 1) * size] for i in range(n_chunks)], [chunk] * n_chunks, [0] * n_chunks,
           [i * chunk for i in range(n_chunks)], piped[0], piped[1], status=status)
    torch.cuda.synchronize()
    ld.close()
    assert int(status.abs().sum().item()) == 0
    assert torch.equal(piped.view(torch.int16), plain.view(torch.int16))
