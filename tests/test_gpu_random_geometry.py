"""Randomised GPU parity over launch geometry: random layer/token/channel counts, padded (strided) source and
destination views, token offsets, random page tables and block sizes, both dtypes, every level, through encode,
decode, token dropping and transcode.  Seeded: the cases are the same on every run."""
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


def padded_device_view(bits, dt, pad_tokens, pad_channels, fill):
    """Device tensor [l][n][c] that is a view into a larger [l][n + pad_tokens][c + pad_channels] allocation."""
    l, n, c = bits.shape
    big = torch.full((l, n + pad_tokens, c + pad_channels), fill, dtype=TDT[dt], device="cuda")
    view = big[:, :n, :c]
    view.copy_(torch.from_numpy(bits.view(np.int16)).cuda().view(TDT[dt]))
    return big, view


def host_bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("case", range(40))
def test_random_geometry(kvh, case):
    rng = np.random.default_rng(1000 + case)
    dt = int(rng.integers(0, 2))
    l = int(rng.integers(1, 5))
    n = int(rng.choice([1, 7, 64, 127, 128, 129, 200, 333, 512, 700]))
    c = 128 * int(rng.choice([1, 2, 3, 4, 5, 8, 9, 12]))
    level = int(rng.integers(0, 3))
    pad_t, pad_c = int(rng.integers(0, 9)), 8 * int(rng.integers(0, 5))
    k, v = gen.make_kv(l, n, c, dt, seed=5000 + case)

    # encode from padded views (token stride c + pad_c, layer stride (n + pad_t) * (c + pad_c))
    _, kd = padded_device_view(k, dt, pad_t, pad_c, 9.0)
    _, vd = padded_device_view(v, dt, pad_t, pad_c, 9.0)
    want = oracle.encode(k, v, dt, level)
    blob = kvh.encode(kd, vd, level)
    torch.cuda.synchronize()
    assert np.array_equal(blob.cpu().numpy(), want), ("encode", dt, l, n, c, level, pad_t, pad_c)

    # decode into a padded destination at a token offset; padding must stay untouched
    t_off = int(rng.integers(0, 20))
    big_k = torch.full((l, t_off + n + pad_t, c + pad_c), 7.0, dtype=TDT[dt], device="cuda")
    big_v = torch.full_like(big_k, 7.0)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    kvh.decode(blob, level, n, big_k[:, :, :c], big_v[:, :, :c], dst_token0=t_off, status=status)
    torch.cuda.synchronize()
    wk, wv = oracle.decode(want, dt, l, n, c, level)
    seven = host_bits(torch.full((1,), 7.0, dtype=TDT[dt]))[0]
    for big, w in ((big_k, wk), (big_v, wv)):
        got = host_bits(big)
        assert status.item() == 0 and np.array_equal(got[:, t_off:t_off + n, :c], w), ("decode", dt, l, n, c, level)
        got[:, t_off:t_off + n, :c] = seven
        assert (got == seven).all(), "decode wrote outside its rows"

    # paged decode with a random block size and table, at a logical offset
    bt = int(rng.choice([1, 3, 16, 32]))
    s0 = int(rng.integers(0, 2 * bt))
    P = (s0 + n + bt - 1) // bt
    table = rng.permutation(P + 2).astype(np.int32)[:P]
    pk = np.zeros((l, P + 2, bt, c), np.uint16); pv = np.zeros_like(pk)
    assert oracle.decode_into(want, dt, l, n, c, level, pk, pv, dst_token0=s0, page_table=table, block_tokens=bt) == 0
    gk = torch.zeros((l, P + 2, bt, c), dtype=TDT[dt], device="cuda"); gv = torch.zeros_like(gk)
    kvh.decode(blob, level, n, gk, gv, dst_token0=s0, page_table=torch.from_numpy(table).cuda(), block_tokens=bt)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(gk), pk) and np.array_equal(host_bits(gv), pv), ("paged", bt, s0)

    # transcode to a random level
    to = int(rng.integers(0, 3))
    low = kvh.transcode(blob, dt, l, n, c, level, to)
    torch.cuda.synchronize()
    assert np.array_equal(low.cpu().numpy(), oracle.transcode(want, dt, l, n, c, level, to)), ("transcode", level, to)

    # token dropping from the padded views
    if n >= 2:
        sink, window = int(rng.integers(0, n)), int(rng.integers(1, n))
        kept = kvh.encode_kept(kd, vd, sink, window, level)
        torch.cuda.synchronize()
        assert np.array_equal(kept.cpu().numpy(), oracle.encode_kept(k, v, dt, sink, window, level)), ("kept", sink, window)
