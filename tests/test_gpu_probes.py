"""GPU checks of the two measurement helpers behind the C ABI (kvh_copy_probe, kvh_stream_probe): they are not part
of the codec, but the benchmark's ceilings rest on them moving exactly the bytes they say."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kvh():
    import paper_2509_00105_amd as m

    m.lib()
    return m


def pattern(n_units, writes):
    """What a pure fill writes: every 16-byte store carries (thread index, 1, 2, 3)."""
    tid = np.arange(n_units * writes, dtype=np.uint32) % 256
    return np.stack([tid, np.full_like(tid, 1), np.full_like(tid, 2), np.full_like(tid, 3)], axis=1).reshape(-1)


def test_copy_probe_copies(kvh):
    src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    kvh.copy_probe(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


def test_stream_probe_moves_what_it_says(kvh):
    units = 256 * 64
    guard = 4096
    for reads, writes in [(0, 1), (1, 1), (1, 2), (1, 8), (2, 1), (8, 1), (1, 0)]:
        src = torch.randint(0, 2 ** 31 - 1, (units * max(reads, 1) * 4,), dtype=torch.int32, device="cuda")
        buf = torch.full((guard + units * max(writes, 1) * 16 + guard,), 0x5A, dtype=torch.uint8, device="cuda")
        dst = buf[guard:guard + units * max(writes, 1) * 16]
        kvh.stream_probe(dst, src, units, reads, writes)
        torch.cuda.synchronize()
        host = buf.cpu().numpy()
        assert (host[:guard] == 0x5A).all() and (host[-guard:] == 0x5A).all(), (reads, writes)
        body = host[guard:-guard]
        if writes == 0:
            assert (body == 0x5A).all()                       # a pure read stores nothing
            continue
        got = body.view(np.uint32)
        want = pattern(units, writes).reshape(-1, writes, 256, 4)      # [group][store j][thread][word]
        s = src.cpu().numpy().view(np.uint32).reshape(-1, max(reads, 1), 256, 4)
        if reads:
            x = np.bitwise_xor.reduce(s, axis=1)              # what the loads of a unit fold to
            # a thread carries its accumulator through the four units it handles (groups 4 b .. 4 b + 3 of block b)
            x = np.bitwise_xor.accumulate(x.reshape(-1, 4, 256, 4), axis=1).reshape(-1, 256, 4)
            want = want ^ x[:, None]
        assert np.array_equal(got, want.reshape(-1)), (reads, writes)
    with pytest.raises(kvh.KVHError):
        kvh.stream_probe(dst, src, 256, 3, 1)                 # not one of the supported mixes
    with pytest.raises(kvh.KVHError):
        kvh.stream_probe(dst, src, 100, 1, 1)                 # not whole groups of 256 units
    with pytest.raises(ValueError):
        kvh.stream_probe(dst[:64], src, 256, 1, 1)            # destination too small
