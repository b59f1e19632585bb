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


def test_time_next_launch_records_the_kernel_itself(kvh):
    """kvh_time_next_launch: the pair is recorded by the next kernel only, its span is positive and no longer than
    what events recorded around the same launch see."""
    k = torch.randn(8, 2048, 1024, device="cuda").to(torch.bfloat16)
    v = torch.randn_like(k)
    blob = kvh.encode(k, v, 0)
    torch.cuda.synchronize()
    s = torch.cuda.current_stream()
    a, b, x, y = (torch.cuda.Event(enable_timing=True) for _ in range(4))
    for e in (a, b, x, y):
        e.record(s)
    torch.cuda.synchronize()
    x.record(s)
    kvh.time_next_launch(a, b)
    kvh.encode(k, v, 0, blob=blob)
    y.record(s)
    torch.cuda.synchronize()
    own, around = a.elapsed_time(b), x.elapsed_time(y)
    assert 0.0 < own <= around * 1.02 + 0.002, (own, around)
    kvh.encode(k, v, 0, blob=blob)          # no pair pending: this launch must leave the events alone
    torch.cuda.synchronize()
    assert a.elapsed_time(b) == own
    assert kvh.lib().kvh_time_next_launch(None, None) == -1
