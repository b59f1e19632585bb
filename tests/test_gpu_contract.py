"""GPU tests of what the boundary promises about inputs it cannot vet on the host: batched items that break the
call's own limits are refused as a whole on the device, non-finite input never leads outside the blob, and a
hand-made blob outside the transcoder's domain gets the documented treatment.  Expected bytes come from the oracle.
"""
import numpy as np
import pytest

import kv_inputs as gen
import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

F16, BF16 = gen.F16, gen.BF16
TDT = {F16: torch.float16, BF16: torch.bfloat16}
MISMATCH = 1  # KVH_DEV_HEADER_MISMATCH


@pytest.fixture(scope="module")
def kvh():
    import paper_2509_00105_amd as m

    m.lib()
    return m


def to_dev(bits: np.ndarray, dt: int):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(TDT[dt])


def to_host(t) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def test_encode_batch_skips_an_oversize_item_entirely(kvh):
    """Items 0 and 2 fit max_tokens_per_item = 256; item 1 claims 300 tokens.  Its blob keeps every sentinel byte
    (no header, no partial sections); the neighbours are byte-identical to the oracle."""
    dt, l, N, c = BF16, 2, 900, 1024
    k, v = gen.make_kv(l, N, c, dt, seed=71)
    kd, vd = to_dev(k, dt), to_dev(v, dt)
    t0s, ns, levels = [0, 256, 600], [256, 300, 200], [0, 1, 2]
    sizes = [kvh.blob_size(l, n, c, lv) for n, lv in zip(ns, levels)]
    bufs = [torch.full((s,), 0xA7, dtype=torch.uint8, device="cuda") for s in sizes]
    items = kvh.make_enc_items([b.data_ptr() for b in bufs], t0s, ns, levels, "cuda")
    kvh.encode_batch(items, 3, 256, kd, vd)
    torch.cuda.synchronize()
    assert (bufs[1].cpu().numpy() == 0xA7).all(), "an oversize item wrote into its blob"
    for i in (0, 2):
        want = oracle.encode(k[:, t0s[i]:t0s[i] + ns[i]], v[:, t0s[i]:t0s[i] + ns[i]], dt, levels[i])
        assert np.array_equal(bufs[i].cpu().numpy(), want), i
    # the untouched buffer is no blob: decoding it reports the mismatch and writes nothing
    ok = torch.full((l, 300, c), 3.0, dtype=TDT[dt], device="cuda"); ov = ok.clone()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode(bufs[1], 1, 300, ok, ov, status=status)
    torch.cuda.synchronize()
    assert status.item() == MISMATCH and bool((ok == 3.0).all()) and bool((ov == 3.0).all())
    # the same through the token-dropping batch call: item 1 keeps 300 of 700 tokens against a bound of 256
    bufs = [torch.full((s,), 0xA7, dtype=torch.uint8, device="cuda") for s in sizes]
    kitems = kvh.make_kept_enc_items([b.data_ptr() for b in bufs], [0, 100, 600], [256, 700, 200], [256, 100, 200],
                                     [0, 200, 0], levels, "cuda")
    kvh.encode_kept_batch(kitems, 3, 256, kd, vd)
    torch.cuda.synchronize()
    assert (bufs[1].cpu().numpy() == 0xA7).all()
    assert np.array_equal(bufs[0].cpu().numpy()[64:], oracle.encode(k[:, :256], v[:, :256], dt, 0)[64:])
    assert np.array_equal(bufs[2].cpu().numpy()[64:], oracle.encode(k[:, 600:800], v[:, 600:800], dt, 2)[64:])


@pytest.mark.parametrize("paged", [False, True])
def test_decode_batch_refuses_oversize_and_out_of_range_items(kvh, paged):
    """Four good blobs; the call is made with max_tokens_per_item = 256.  Item 1 holds 300 tokens (a valid blob, but
    longer than the launch covers), item 3 starts at a row index whose end passes 2^31 - 1, item 4 at a negative
    one.  Each gets status 1 and writes nothing; items 0 and 2 are bit-exact."""
    dt, l, c, bt = F16, 2, 1024, 16
    lens, levels = [256, 300, 130, 128, 128], [2, 0, 1, 0, 1]
    rows = 1024
    ks, vs, blobs = [], [], []
    for i, (n, lv) in enumerate(zip(lens, levels)):
        k, v = gen.make_kv(l, n, c, dt, seed=80 + i)
        ks.append(k); vs.append(v)
        blobs.append(torch.from_numpy(oracle.encode(k, v, dt, lv)).cuda())
    dst0 = [0, 256, 576, 2 ** 31 - 100, -16]
    if paged:
        n_pages = rows // bt
        perm = np.random.default_rng(3).permutation(n_pages).astype(np.int32)
        table = torch.from_numpy(perm).cuda()
        ok = torch.full((l, n_pages, bt, c), 7.0, dtype=TDT[dt], device="cuda")
        tables = [table.data_ptr()] * 5
    else:
        ok = torch.full((l, rows, c), 7.0, dtype=TDT[dt], device="cuda")
        tables = [0] * 5
    ov = ok.clone()
    items = kvh.make_dec_items([b.data_ptr() for b in blobs], lens, levels, dst0, tables, "cuda")
    status = torch.zeros(5, dtype=torch.int32, device="cuda")
    kvh.decode_batch(items, 5, 256, ok, ov, paged=paged, block_tokens=bt, status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, MISMATCH, 0, MISMATCH, MISMATCH]
    if paged:
        inv = torch.from_numpy(perm.astype(np.int64)).cuda()
        ok, ov = ok[:, inv].reshape(l, rows, c), ov[:, inv].reshape(l, rows, c)
    written = torch.zeros(rows, dtype=torch.bool, device="cuda")
    for i in (0, 2):
        wk, wv = oracle.decode(blobs[i].cpu().numpy(), dt, l, lens[i], c, levels[i])
        assert np.array_equal(to_host(ok[:, dst0[i]:dst0[i] + lens[i]]), wk), i
        assert np.array_equal(to_host(ov[:, dst0[i]:dst0[i] + lens[i]]), wv), i
        written[dst0[i]:dst0[i] + lens[i]] = True
    assert bool((ok[:, ~written] == 7.0).all()) and bool((ov[:, ~written] == 7.0).all()), "a refused item wrote rows"


def test_decode_kept_batch_refuses_oversize_items(kvh):
    dt, l, c = BF16, 1, 1024
    N, sink, window = 700, 100, 200
    k, v = gen.make_kv(l, N, c, dt, seed=90)
    kept = torch.from_numpy(oracle.encode_kept(k, v, dt, sink, window, 1)).cuda()       # 300 kept tokens
    plain = torch.from_numpy(oracle.encode(k[:, :200], v[:, :200], dt, 0)).cuda()
    ok = torch.full((l, 1024, c), 9.0, dtype=TDT[dt], device="cuda"); ov = ok.clone()
    items = kvh.make_kept_items([kept.data_ptr(), plain.data_ptr()], [300, 200], [1, 0], [0, 800], [0, 0],
                                [N, 0], [sink, 0], [window, 0], [0, 0], "cuda")
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    kvh.decode_kept_batch(items, 2, 256, ok, ov, status=status)                           # 300 > 256: refused
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [MISMATCH, 0]
    assert bool((ok[:, :800] == 9.0).all()) and bool((ov[:, :800] == 9.0).all())
    wk, wv = oracle.decode(plain.cpu().numpy(), dt, l, 200, c, 0)
    assert np.array_equal(to_host(ok[:, 800:1000]), wk) and np.array_equal(to_host(ov[:, 800:1000]), wv)
    status.zero_()
    kvh.decode_kept_batch(items, 2, 300, ok, ov, status=status)                           # the same items fit 300
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0]
    wk = np.zeros((l, N, c), np.uint16); wv = np.zeros_like(wk)
    assert oracle.decode_kept_into(kept.cpu().numpy(), dt, l, N, c, sink, window, 1, wk, wv) == 0
    assert np.array_equal(to_host(ok[:, :sink]), wk[:, :sink]) and np.array_equal(to_host(ov[:, N - window:N]), wv[:, N - window:N])


def test_transcode_batch_refuses_an_oversize_item(kvh):
    dt, l, c = F16, 2, 1024
    lens, pairs = [256, 300, 128], [(0, 2), (0, 1), (1, 2)]
    srcs, wants, outs = [], [], []
    for i, (n, (a, b)) in enumerate(zip(lens, pairs)):
        k, v = gen.make_kv(l, n, c, dt, seed=95 + i)
        s = oracle.encode(k, v, dt, a)
        srcs.append(torch.from_numpy(s).cuda())
        wants.append(oracle.transcode(s, dt, l, n, c, a, b))
        outs.append(torch.full((wants[-1].size,), 0x3C, dtype=torch.uint8, device="cuda"))
    items = kvh.make_tc_items([s.data_ptr() for s in srcs], [o.data_ptr() for o in outs], lens, [a for a, _ in pairs],
                              [b for _, b in pairs], "cuda")
    status = torch.zeros(3, dtype=torch.int32, device="cuda")
    kvh.transcode_batch(items, 3, 256, dt, l, c, status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, MISMATCH, 0]
    assert (outs[1].cpu().numpy() == 0x3C).all(), "an oversize item wrote into its destination"
    for i in (0, 2):
        assert np.array_equal(outs[i].cpu().numpy(), wants[i]), i


@pytest.mark.parametrize("dt", [F16, BF16])
@pytest.mark.parametrize("level", [0, 1, 2])
def test_non_finite_input_stays_inside_the_blob(kvh, level, dt):
    """Non-finite input is a precondition violation with unspecified codes, but the encoder must stay inside the
    blob: guard bytes on both sides intact, header as for finite input, and every 8-channel lane span whose groups
    hold only finite values byte-identical to the oracle's (the oracle refuses non-finite input, so it encodes the
    same tensor with the offending values replaced by zero, which leaves every finite group as it was)."""
    l, n, c = 2, 300, 1024
    rng = np.random.default_rng(200 + level + 10 * dt)
    k, v = gen.make_kv(l, n, c, dt, seed=60 + level)
    pos_inf, neg_inf, nan = (0x7C00, 0xFC00, 0x7E00) if dt == F16 else (0x7F80, 0xFF80, 0x7FC0)
    bad_k = np.zeros((l, n, c), bool); bad_v = np.zeros((l, n, c), bool)
    for bad, x in ((bad_k, k), (bad_v, v)):
        for _ in range(40):
            lam, t, ch = int(rng.integers(l)), int(rng.integers(n)), int(rng.integers(c))
            x[lam, t, ch] = (pos_inf, neg_inf, nan)[int(rng.integers(3))]
            bad[lam, t, ch] = True
    guard = 4096
    size = kvh.blob_size(l, n, c, level)
    buf = torch.full((size + 2 * guard,), 0xEE, dtype=torch.uint8, device="cuda")
    kvh.encode(to_dev(k, dt), to_dev(v, dt), level, blob=buf[guard:guard + size])
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    assert (got[:guard] == 0xEE).all() and (got[guard + size:] == 0xEE).all(), "guard bytes were overwritten"
    got = got[guard:guard + size]
    kz, vz = k.copy(), v.copy()
    kz[bad_k] = 0; vz[bad_v] = 0
    want = oracle.encode(kz, vz, dt, level)
    assert np.array_equal(got[:64], want[:64]), "header"
    b = kvh.level_bits(level)
    span_bytes = 8 * b // 8                                        # bytes of one 8-channel lane span in a code row
    checked = 0
    for lam in range(l):
        off = oracle.section_offsets(l, n, c, level, lam)
        # K: a (token, 8-channel span) is clean when none of the span's channels has a bad value in the token's group
        groups = -(-n // 128)
        bad_group_ch = np.zeros((groups, c), bool)
        for g in range(groups):
            bad_group_ch[g] = bad_k[lam, g * 128:(g + 1) * 128].any(axis=0)
        bad_span = bad_group_ch.reshape(groups, c // 8, 8).any(axis=2)               # [group][span]
        gk = got[off["kcodes"]:off["kcodes"] + n * c * b // 8].reshape(n, c // 8, span_bytes)
        wk = want[off["kcodes"]:off["kcodes"] + n * c * b // 8].reshape(n, c // 8, span_bytes)
        clean = ~bad_span[np.arange(n) // 128]                                        # [token][span]
        assert np.array_equal(gk[clean], wk[clean]), "K codes of finite groups"
        gm = got[off["kmeta"]:off["kmeta"] + groups * c * 4].reshape(groups, c, 4)
        wm = want[off["kmeta"]:off["kmeta"] + groups * c * 4].reshape(groups, c, 4)
        assert np.array_equal(gm[~bad_group_ch], wm[~bad_group_ch]), "K metadata of finite groups"
        # V: a (token, head) group is clean when it holds no bad value
        bad_head = bad_v[lam].reshape(n, c // 128, 128).any(axis=2)
        gv = got[off["vcodes"]:off["vcodes"] + n * c * b // 8].reshape(n, c // 128, 128 * b // 8)
        wv = want[off["vcodes"]:off["vcodes"] + n * c * b // 8].reshape(n, c // 128, 128 * b // 8)
        assert np.array_equal(gv[~bad_head], wv[~bad_head]), "V codes of finite groups"
        gvm = got[off["vmeta"]:off["vmeta"] + n * (c // 128) * 4].reshape(n, c // 128, 4)
        wvm = want[off["vmeta"]:off["vmeta"] + n * (c // 128) * 4].reshape(n, c // 128, 4)
        assert np.array_equal(gvm[~bad_head], wvm[~bad_head]), "V metadata of finite groups"
        checked += int(clean.sum()) + int((~bad_head).sum())
    assert checked > 0.8 * l * n * (c // 8 + c // 128)


@pytest.mark.parametrize("pair", [(0, 1), (0, 2), (1, 2)])
def test_transcode_of_a_blob_outside_its_domain_uses_the_stored_statistics(kvh, pair):
    """The fused transcoder carries group statistics over instead of recomputing them, which is exact for blobs the
    library wrote (every group holds its smallest and largest code).  Pinned here: a hand-made blob B1 in which one
    K group and one V group hold no code 0 and no code L is transcoded as if the stored (min, max) still applied,
    i.e. element for element like blob B2 = B1 with two further elements of those groups set to code 0 and code L —
    and B2, being inside the domain, has the oracle's decode-then-encode as its expected output."""
    a, b = pair
    dt, l, n, c = BF16, 1, 128, 1024
    k, v = gen.make_kv(l, n, c, dt, seed=33)
    base = oracle.encode(k, v, dt, a)
    ba, bb = kvh.level_bits(a), kvh.level_bits(b)
    L = (1 << ba) - 1
    off_a = oracle.section_offsets(l, n, c, a, 0)
    off_b = oracle.section_offsets(l, n, c, b, 0)
    row_a, row_b = c * ba // 8, c * bb // 8

    def codes_of(blob, section, bits, row_bytes, offs):
        raw = blob[offs[section]:offs[section] + n * row_bytes].reshape(n, row_bytes)
        per = 8 // bits
        return np.stack([(raw >> (bits * i)) & ((1 << bits) - 1) for i in range(per)], axis=2).reshape(n, c)

    def put_codes(blob, section, q):
        per = 8 // ba
        qq = q.reshape(n, c // per, per).astype(np.uint8)
        raw = np.zeros((n, c // per), np.uint8)
        for i in range(per):
            raw |= qq[:, :, i] << (ba * i)
        blob[off_a[section]:off_a[section] + n * row_a] = raw.reshape(-1)

    kq, vq = codes_of(base, "kcodes", ba, row_a, off_a), codes_of(base, "vcodes", ba, row_a, off_a)
    kch, vtok, vhead = 517, 77, 3
    mid = max(1, L // 2)
    b1k, b1v = kq.copy(), vq.copy()
    b1k[:, kch] = np.clip(b1k[:, kch], 1, L - 1)                     # K group (channel 517): no 0, no L
    b1v[vtok, vhead * 128:(vhead + 1) * 128] = np.clip(b1v[vtok, vhead * 128:(vhead + 1) * 128], 1, L - 1)
    b2k, b2v = b1k.copy(), b1v.copy()
    b2k[0, kch], b2k[1, kch] = 0, L                                   # back inside the domain
    b2v[vtok, vhead * 128], b2v[vtok, vhead * 128 + 1] = 0, L
    assert mid >= 1
    B1, B2 = base.copy(), base.copy()
    put_codes(B1, "kcodes", b1k); put_codes(B1, "vcodes", b1v)
    put_codes(B2, "kcodes", b2k); put_codes(B2, "vcodes", b2v)
    want2 = oracle.transcode(B2, dt, l, n, c, a, b)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    got1 = kvh.transcode(torch.from_numpy(B1).cuda(), dt, l, n, c, a, b, status=status).cpu().numpy()
    got2 = kvh.transcode(torch.from_numpy(B2).cuda(), dt, l, n, c, a, b, status=status).cpu().numpy()
    torch.cuda.synchronize()
    assert status.item() == 0
    assert np.array_equal(got2, want2), "a blob inside the domain must match the oracle byte for byte"
    # B1: metadata sections equal B2's (the stored statistics are carried over) ...
    for sec, size in (("kmeta", c * 4), ("vmeta", n * (c // 128) * 4)):
        assert np.array_equal(got1[off_b[sec]:off_b[sec] + size], want2[off_b[sec]:off_b[sec] + size]), sec
    # ... and so do all codes except those of the four elements that differ between B1 and B2
    g1k, w2k = codes_of(got1, "kcodes", bb, row_b, off_b), codes_of(want2, "kcodes", bb, row_b, off_b)
    g1v, w2v = codes_of(got1, "vcodes", bb, row_b, off_b), codes_of(want2, "vcodes", bb, row_b, off_b)
    mk = np.ones((n, c), bool); mk[0, kch] = mk[1, kch] = False
    mv = np.ones((n, c), bool); mv[vtok, vhead * 128] = mv[vtok, vhead * 128 + 1] = False
    assert np.array_equal(g1k[mk], w2k[mk]) and np.array_equal(g1v[mv], w2v[mv])
