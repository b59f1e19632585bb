"""GPU test of kvh_load_static, the allocation-free form of the load path: through the C ABI, its output against
that of kvh_loader_run (the existing entry point it is a variant of) on the same pinned blobs, bit for bit, on two
calls in a row, the second with a smaller input; and against the oracle's decode.  Also: the size limit is an
error, not a fault, and the call allocates no device memory."""
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


def entries(dt, l, c, lens, levels, seed):
    """Oracle blobs (pinned) of consecutive pieces of one context, and the oracle's decode of the whole."""
    N = sum(lens)
    k, v = gen.make_kv(l, N, c, dt, seed=seed)
    blobs, want_k, want_v, t0s, t0 = [], np.zeros_like(k), np.zeros_like(v), [], 0
    for n, lv in zip(lens, levels):
        b = oracle.encode(np.ascontiguousarray(k[:, t0:t0 + n]), np.ascontiguousarray(v[:, t0:t0 + n]), dt, lv)
        dk, dv = oracle.decode(b, dt, l, n, c, lv)
        want_k[:, t0:t0 + n], want_v[:, t0:t0 + n] = dk, dv
        blobs.append(torch.from_numpy(b).pin_memory())
        t0s.append(t0)
        t0 += n
    return blobs, t0s, want_k, want_v, N


def run_both(kvh, dt, l, c, lens, levels, seed, paged_bt=None):
    """The same blobs through kvh_loader_run and kvh_load_static; returns both outputs and the oracle's."""
    blobs, t0s, want_k, want_v, N = entries(dt, l, c, lens, levels, seed)
    staging = torch.empty(2 * (max(b.numel() for b in blobs) + 1536), dtype=torch.uint8, device="cuda")
    shape = (l, N, c)
    tabs = None
    if paged_bt is not None:
        P = -(-N // paged_bt)
        perm = np.random.default_rng(seed).permutation(P).astype(np.int32)
        tab = torch.from_numpy(perm).cuda()
        tabs = [tab] * len(lens)
        shape = (l, P, paged_bt, c)
    outs = []
    for which in ("loader", "static"):
        ok = torch.full(shape, 3.0, dtype=TDT[dt], device="cuda"); ov = torch.full_like(ok, 3.0)
        status = torch.zeros(len(lens), dtype=torch.int32, device="cuda")
        if which == "loader":
            ld = kvh.Loader(staging, 2)
            ld.run(blobs, lens, levels, t0s, ok, ov, page_tables=tabs, block_tokens=paged_bt or 16, status=status)
            torch.cuda.synchronize()
            ld.close()
        else:
            before = torch.cuda.memory_allocated()
            kvh.load_static(blobs, lens, levels, t0s, ok, ov, page_tables=tabs, block_tokens=paged_bt or 16, status=status)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before
        assert status.cpu().tolist() == [0] * len(lens), which
        if paged_bt is not None:
            inv = torch.from_numpy(perm.astype(np.int64)).cuda()
            ok, ov = ok[:, inv].reshape(l, -1, c)[:, :N], ov[:, inv].reshape(l, -1, c)[:, :N]
        outs.append((to_host(ok), to_host(ov)))
    return outs, (want_k, want_v)


def test_static_load_equals_loader_run_twice_second_call_smaller(kvh):
    # first call: seven blobs of mixed levels and lengths, 1.2 MB to 4.3 MB each: several groups through the one slot
    (ld1, st1), want1 = run_both(kvh, BF16, 8, 1024, [256, 130, 256, 1, 384, 77, 256], [0, 2, 1, 0, 2, 1, 2], seed=501)
    assert np.array_equal(st1[0], ld1[0]) and np.array_equal(st1[1], ld1[1])
    assert np.array_equal(st1[0], want1[0]) and np.array_equal(st1[1], want1[1])
    # second call right after it, smaller in every respect: the slot still holds the first call's bytes
    (ld2, st2), want2 = run_both(kvh, F16, 2, 256, [100, 3], [1, 0], seed=502)
    assert np.array_equal(st2[0], ld2[0]) and np.array_equal(st2[1], ld2[1])
    assert np.array_equal(st2[0], want2[0]) and np.array_equal(st2[1], want2[1])


def test_static_load_many_groups_paged_and_dropped(kvh):
    # 24 layers x 256 tokens x 1024 channels at 8 bits = 13 MB per blob: three blobs fill the 40 MiB slot, so eight
    # blobs go through it in three groups
    (ld, st), want = run_both(kvh, BF16, 24, 1024, [256] * 8, [0] * 8, seed=503, paged_bt=16)
    assert np.array_equal(st[0], ld[0]) and np.array_equal(st[1], ld[1])
    assert np.array_equal(st[0], want[0]) and np.array_equal(st[1], want[1])
    # a token-dropped blob next to an ordinary one
    dt, l, c, N, sink, window = F16, 2, 256, 600, 50, 150
    k, v = gen.make_kv(l, N, c, dt, seed=504)
    kept = torch.from_numpy(oracle.encode_kept(k, v, dt, sink, window, 2)).pin_memory()
    plain = torch.from_numpy(oracle.encode(k[:, :128], v[:, :128], dt, 1)).pin_memory()
    ok = torch.zeros((l, 1000, c), dtype=TDT[dt], device="cuda"); ov = torch.zeros_like(ok)
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    kvh.load_static([kept, plain], [200, 128], [2, 1], [0, 700], ok, ov, status=status,
                    drops=[(N, sink, window, False), None])
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0]
    wk = np.zeros((l, 1000, c), np.uint16); wv = np.zeros_like(wk)
    dk = np.zeros((l, N, c), np.uint16); dv = np.zeros_like(dk)
    assert oracle.decode_kept_into(kept.numpy(), dt, l, N, c, sink, window, 2, dk, dv) == 0
    wk[:, :N], wv[:, :N] = dk, dv
    pk, pv = oracle.decode(plain.numpy(), dt, l, 128, c, 1)
    wk[:, 700:828], wv[:, 700:828] = pk, pv
    assert np.array_equal(to_host(ok), wk) and np.array_equal(to_host(ov), wv)


def test_static_load_refuses_what_does_not_fit(kvh):
    dt, l, c = BF16, 80, 1024
    n = 512                                                     # 80 layers x 512 tokens at 8 bits: 86 MB > 40 MiB
    size = kvh.blob_size(l, n, c, 0)
    assert size > (40 << 20)
    big = torch.zeros(size, dtype=torch.uint8).pin_memory()
    ok = torch.zeros((l, n, c), dtype=TDT[dt], device="cuda"); ov = torch.zeros_like(ok)
    with pytest.raises(kvh.KVHError) as e:
        kvh.load_static([big], [n], [0], [0], ok, ov)
    assert e.value.status == -4                                 # KVH_E_SIZE, found before anything is enqueued
    with pytest.raises(kvh.KVHError):
        kvh.load_static([torch.zeros(4096, dtype=torch.uint8).pin_memory()], [128], [5], [0], ok, ov)   # bad level
    torch.cuda.synchronize()
    assert not ok.any() and not ov.any()
