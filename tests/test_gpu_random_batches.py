"""Randomised GPU parity over the batched entry points: 1-10 random items per launch, ordinary and token-dropped
mixed, random levels, lengths and source offsets; encode_kept_batch and encode_batch, paged decode_kept_batch with
per-item page tables, block sizes and logical offsets (compact or not), transcode_batch to random levels.  Every
blob and every decoded row is compared with the oracle.  Seeded: the cases are the same on every run."""
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


def dev(bits, dt):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(TDT[dt])


def host_bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("case", range(28))
def test_random_batches(kvh, case):
    rng = np.random.default_rng(77000 + case)
    dt = int(rng.integers(0, 2))
    l = int(rng.integers(1, 4))
    c = 128 * int(rng.choice([1, 2, 4, 8, 9]))
    N = int(rng.choice([300, 900, 1500]))
    k, v = gen.make_kv(l, N, c, dt, seed=9000 + case)
    kd, vd = dev(k, dt), dev(v, dt)
    n_items = int(rng.integers(1, 11))
    # ---- items: (t0, orig, sink, window, level); sink == -1 marks an ordinary item
    items = []
    for _ in range(n_items):
        orig = int(rng.integers(1, min(N, 600) + 1))
        t0 = int(rng.integers(0, N - orig + 1))
        level = int(rng.integers(0, 3))
        if rng.random() < 0.5:
            items.append((t0, orig, -1, -1, level))
        else:
            sink = int(rng.integers(0, orig + 1)); window = int(rng.integers(0, orig + 1))
            if sink + window < 1:
                window = 1
            items.append((t0, orig, sink, window, level))
    kept_n = [orig if s < 0 else oracle.kept_tokens(orig, s, w) for (_, orig, s, w, _) in items]
    sizes = [kvh.blob_size(l, n, c, lv) for n, (_, _, _, _, lv) in zip(kept_n, items)]
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.int64)
    want = [oracle.encode(k[:, t0:t0 + orig], v[:, t0:t0 + orig], dt, lv) if s < 0
            else oracle.encode_kept(np.ascontiguousarray(k[:, t0:t0 + orig]), np.ascontiguousarray(v[:, t0:t0 + orig]), dt, s, w, lv)
            for (t0, orig, s, w, lv) in items]

    # ---- encode: ordinary items through encode_batch, all items (ordinary as sink=orig) through encode_kept_batch
    blobs = torch.zeros(int(sum(sizes)), dtype=torch.uint8, device="cuda")
    ptrs = [blobs.data_ptr() + int(o) for o in offs]
    ei = kvh.make_kept_enc_items(ptrs, [it[0] for it in items], [it[1] for it in items],
                                 [it[1] if it[2] < 0 else it[2] for it in items], [0 if it[2] < 0 else it[3] for it in items],
                                 [it[4] for it in items], "cuda")
    kvh.encode_kept_batch(ei, n_items, max(kept_n), kd, vd)
    torch.cuda.synchronize()
    got = blobs.cpu().numpy()
    for i, (o, sz) in enumerate(zip(offs, sizes)):
        w = want[i].copy()
        if items[i][2] < 0:  # encoded as "sink = orig": the header words say (orig, orig, 0) instead of zeros
            assert np.array_equal(got[o + 44:o + sz], w[44:]) and np.array_equal(got[o:o + 32], w[:32]), ("kept-as-plain", case, i)
        else:
            assert np.array_equal(got[o:o + sz], w), ("encode_kept_batch", case, i, items[i])
    plain = [i for i, it in enumerate(items) if it[2] < 0]
    if plain:
        blobs2 = torch.zeros_like(blobs)
        e2 = kvh.make_enc_items([blobs2.data_ptr() + int(offs[i]) for i in plain], [items[i][0] for i in plain],
                                [items[i][1] for i in plain], [items[i][4] for i in plain], "cuda")
        kvh.encode_batch(e2, len(plain), max(items[i][1] for i in plain), kd, vd)
        torch.cuda.synchronize()
        g2 = blobs2.cpu().numpy()
        for i in plain:
            assert np.array_equal(g2[offs[i]:offs[i] + sizes[i]], want[i]), ("encode_batch", case, i, items[i])
    # the reference blobs go to the device for the decode / transcode legs
    ref = torch.from_numpy(np.concatenate(want)).cuda()
    rptr = [ref.data_ptr() + int(o) for o in offs]

    # ---- paged decode of the whole mix
    bt = int(rng.choice([1, 4, 16, 32]))
    compact = [int(rng.integers(0, 2)) for _ in items]
    s0 = [int(rng.integers(0, 2 * bt)) for _ in items]
    span = [(kept_n[i] if (items[i][2] < 0 or compact[i]) else items[i][1]) for i in range(n_items)]
    pages = [(s0[i] + span[i] + bt - 1) // bt for i in range(n_items)]
    P = sum(pages) + 3
    perm = rng.permutation(P).astype(np.int32)
    tabs, at = [], 0
    for p in pages:
        tabs.append(perm[at:at + p].copy()); at += p
    tab_dev = [torch.from_numpy(t).cuda() for t in tabs]
    pk = np.zeros((l, P, bt, c), np.uint16); pv = np.zeros_like(pk)
    for i, (t0, orig, s, w, lv) in enumerate(items):
        if s < 0:
            rc = oracle.decode_into(want[i], dt, l, orig, c, lv, pk, pv, dst_token0=s0[i], page_table=tabs[i], block_tokens=bt)
        else:
            rc = oracle.decode_kept_into(want[i], dt, l, orig, c, s, w, lv, pk, pv, dst_token0=s0[i], compact=bool(compact[i]),
                                         page_table=tabs[i], block_tokens=bt)
        assert rc == 0
    gk = torch.zeros((l, P, bt, c), dtype=TDT[dt], device="cuda"); gv = torch.zeros_like(gk)
    st = torch.zeros(n_items, dtype=torch.int32, device="cuda")
    di = kvh.make_kept_items(rptr, kept_n, [it[4] for it in items], s0, [t.data_ptr() for t in tab_dev],
                             [0 if it[2] < 0 else it[1] for it in items], [0 if it[2] < 0 else it[2] for it in items],
                             [0 if it[2] < 0 else it[3] for it in items], compact, "cuda")
    kvh.decode_kept_batch(di, n_items, max(kept_n), gk, gv, paged=True, block_tokens=bt, status=st)
    torch.cuda.synchronize()
    assert int(st.abs().sum().item()) == 0, ("status", case, st.tolist())
    assert np.array_equal(host_bits(gk), pk) and np.array_equal(host_bits(gv), pv), ("decode_kept_batch", case, bt)

    # ---- transcode every item to a random level
    to = [int(rng.integers(0, 3)) for _ in items]
    osz = [kvh.blob_size(l, kept_n[i], c, to[i]) for i in range(n_items)]
    ooff = np.concatenate([[0], np.cumsum(osz)[:-1]]).astype(np.int64)
    outb = torch.zeros(int(sum(osz)), dtype=torch.uint8, device="cuda")
    ti = kvh.make_tc_items(rptr, [outb.data_ptr() + int(o) for o in ooff], kept_n, [it[4] for it in items], to, "cuda")
    st2 = torch.zeros(n_items, dtype=torch.int32, device="cuda")
    kvh.transcode_batch(ti, n_items, max(kept_n), TDT[dt], l, c, status=st2)
    torch.cuda.synchronize()
    assert int(st2.abs().sum().item()) == 0
    go = outb.cpu().numpy()
    for i in range(n_items):
        w = oracle.transcode(want[i], dt, l, kept_n[i], c, items[i][4], to[i])
        assert np.array_equal(go[ooff[i]:ooff[i] + osz[i]], w), ("transcode_batch", case, i, items[i], to[i])
