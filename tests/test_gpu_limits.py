"""GPU parity at the edges of the launch geometry: thousands of tiny items in one batched launch (grid z), many
layers with a single token (grid y), a wide channel count (many strips and spans), through encode_batch,
decode_batch and transcode_batch, each against the CPU oracle."""
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


def to_dev(bits, dt):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(TDT[dt])


def to_host(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def test_three_thousand_tiny_items_in_one_launch(kvh):
    dt, l, c, n_items = BF16, 1, 128, 3000
    rng = np.random.default_rng(21)
    lens = rng.integers(1, 4, n_items)
    levels = rng.integers(0, 3, n_items)
    t0s = np.concatenate([[0], np.cumsum(lens)[:-1]])
    N = int(lens.sum())
    k, v = gen.make_kv(l, N, c, dt, seed=21)
    sizes = [kvh.blob_size(l, int(n), c, int(lv)) for n, lv in zip(lens, levels)]
    offs = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.int64)
    want = np.concatenate([oracle.encode(np.ascontiguousarray(k[:, t:t + n]), np.ascontiguousarray(v[:, t:t + n]), dt, int(lv))
                           for t, n, lv in zip(t0s, lens, levels)])
    kd, vd = to_dev(k, dt), to_dev(v, dt)
    blobs = torch.zeros(int(sum(sizes)), dtype=torch.uint8, device="cuda")
    ptrs = [blobs.data_ptr() + int(o) for o in offs]
    kvh.encode_batch(kvh.make_enc_items(ptrs, t0s, lens, levels, "cuda"), n_items, 3, kd, vd)
    torch.cuda.synchronize()
    assert np.array_equal(blobs.cpu().numpy(), want)

    ok, ov = torch.zeros_like(kd), torch.zeros_like(vd)
    status = torch.zeros(n_items, dtype=torch.int32, device="cuda")
    kvh.decode_batch(kvh.make_dec_items(ptrs, lens, levels, t0s, [0] * n_items, "cuda"), n_items, 3, ok, ov, status=status)
    torch.cuda.synchronize()
    assert not status.any()
    wk, wv = np.zeros_like(k), np.zeros_like(v)
    for o, s, t, n, lv in zip(offs, sizes, t0s, lens, levels):
        dk, dv = oracle.decode(want[o:o + s], dt, l, int(n), c, int(lv))
        wk[:, t:t + n], wv[:, t:t + n] = dk, dv
    assert np.array_equal(to_host(ok), wk) and np.array_equal(to_host(ov), wv)

    # every item down to 2 bits in one launch
    out_sizes = [kvh.blob_size(l, int(n), c, 2) for n in lens]
    out_offs = np.concatenate([[0], np.cumsum(out_sizes)[:-1]]).astype(np.int64)
    outs = torch.zeros(int(sum(out_sizes)), dtype=torch.uint8, device="cuda")
    status.zero_()
    items = kvh.make_tc_items(ptrs, [outs.data_ptr() + int(o) for o in out_offs], lens, levels, [2] * n_items, "cuda")
    kvh.transcode_batch(items, n_items, 3, dt, l, c, status=status)
    torch.cuda.synchronize()
    assert not status.any()
    want2 = np.concatenate([oracle.transcode(want[o:o + s], dt, l, int(n), c, int(lv), 2)
                            for o, s, n, lv in zip(offs, sizes, lens, levels)])
    assert np.array_equal(outs.cpu().numpy(), want2)


@pytest.mark.parametrize("dt", [F16, BF16])
def test_many_layers_one_token_and_wide_channels(kvh, dt):
    for l, n, c in ((300, 1, 128), (2, 131, 4224)):   # grid y = 600; 9 strips / 5 spans, the last ones partial
        k, v = gen.make_kv(l, n, c, dt, seed=l + c)
        for level in range(3):
            want = oracle.encode(k, v, dt, level)
            blob = kvh.encode(to_dev(k, dt), to_dev(v, dt), level)
            ok = torch.zeros((l, n, c), dtype=TDT[dt], device="cuda"); ov = torch.zeros_like(ok)
            status = torch.zeros(1, dtype=torch.int32, device="cuda")
            kvh.decode(blob, level, n, ok, ov, status=status)
            low = kvh.transcode(blob, dt, l, n, c, level, 2, status=status)
            torch.cuda.synchronize()
            assert status.item() == 0
            assert np.array_equal(blob.cpu().numpy(), want), (l, n, c, level)
            wk, wv = oracle.decode(want, dt, l, n, c, level)
            assert np.array_equal(to_host(ok), wk) and np.array_equal(to_host(ov), wv), (l, n, c, level)
            assert np.array_equal(low.cpu().numpy(), oracle.transcode(want, dt, l, n, c, level, 2)), (l, n, c, level)


def test_one_long_entry_in_a_single_blob(kvh):
    """40,003 tokens in ONE blob (313 K token-groups, the last one ragged): a long grid in x, 64-bit section offsets."""
    dt, l, n, c, level = F16, 1, 40003, 1024, 2
    k, v = gen.make_kv(l, n, c, dt, seed=4)
    want = oracle.encode(k, v, dt, level)
    blob = kvh.encode(to_dev(k, dt), to_dev(v, dt), level)
    torch.cuda.synchronize()
    assert np.array_equal(blob.cpu().numpy(), want)
    ok = torch.zeros((l, n, c), dtype=TDT[dt], device="cuda"); ov = torch.zeros_like(ok)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode(blob, level, n, ok, ov, status=status)
    low = kvh.transcode(kvh.encode(to_dev(k, dt), to_dev(v, dt), 1), dt, l, n, c, 1, 2, status=status)
    torch.cuda.synchronize()
    assert status.item() == 0
    wk, wv = oracle.decode(want, dt, l, n, c, level)
    assert np.array_equal(to_host(ok), wk) and np.array_equal(to_host(ov), wv)
    assert np.array_equal(low.cpu().numpy(), oracle.transcode(oracle.encode(k, v, dt, 1), dt, l, n, c, 1, 2))


@pytest.mark.parametrize("l,n_big", [(5, 56000), (9, 32000)])
def test_planes_far_apart(kvh, l, n_big):
    """Entries cut out of a tensor whose (layer, K|V) planes lie more than 1 GiB apart in all: the kernels then walk
    the planes in another block order (the encoder in groups of 8 planes, here one or two full groups and a last
    group of 2; the decoder plane by plane), which must not change a byte."""
    dt, n, c, t0 = BF16, 300, 1024, 100
    k, v = gen.make_kv(l, n, c, dt, seed=100 + l)
    kbig = torch.zeros((l, n_big, c), dtype=TDT[dt], device="cuda"); vbig = torch.zeros_like(kbig)
    assert l * kbig.stride(0) * 2 > (1 << 29)
    kbig[:, t0:t0 + n] = to_dev(k, dt); vbig[:, t0:t0 + n] = to_dev(v, dt)
    obig_k = torch.zeros_like(kbig); obig_v = torch.zeros_like(vbig)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    for level in range(4):
        want = oracle.encode(k, v, dt, level)
        blob = kvh.encode(kbig[:, t0:t0 + n], vbig[:, t0:t0 + n], level)
        kvh.decode(blob, level, n, obig_k, obig_v, dst_token0=t0, status=status)
        torch.cuda.synchronize()
        assert status.item() == 0
        assert np.array_equal(blob.cpu().numpy(), want), (l, level)
        wk, wv = oracle.decode(want, dt, l, n, c, level)
        assert np.array_equal(to_host(obig_k[:, t0:t0 + n]), wk) and np.array_equal(to_host(obig_v[:, t0:t0 + n]), wv), (l, level)
    assert not obig_k[:, :t0].any() and not obig_k[:, t0 + n:].any() and not obig_v[:, :t0].any() and not obig_v[:, t0 + n:].any()


def test_long_entry_over_several_layers(kvh):
    """More than 8,192 tokens in one blob of several layers: the encoder then walks the planes two at a time."""
    dt, l, n, c = F16, 3, 8200, 256
    k, v = gen.make_kv(l, n, c, dt, seed=8)
    kd, vd = to_dev(k, dt), to_dev(v, dt)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    for level in range(4):
        want = oracle.encode(k, v, dt, level)
        blob = kvh.encode(kd, vd, level)
        ok = torch.zeros((l, n, c), dtype=TDT[dt], device="cuda"); ov = torch.zeros_like(ok)
        kvh.decode(blob, level, n, ok, ov, status=status)
        torch.cuda.synchronize()
        assert status.item() == 0
        assert np.array_equal(blob.cpu().numpy(), want), level
        wk, wv = oracle.decode(want, dt, l, n, c, level)
        assert np.array_equal(to_host(ok), wk) and np.array_equal(to_host(ov), wv), level
