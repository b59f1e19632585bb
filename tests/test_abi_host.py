"""CPU-only checks of the C-ABI library: it loads, exports every symbol include/kvh.h declares,
its size calculator agrees with the oracle's closed form, and argument errors are reported on
the host before anything is launched (no compute calls here)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "kvh.h")
LIB = os.path.join(ROOT, "paper_2509_00105_amd", "libkvh.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2509_00105_amd import build

        build.build()
    import paper_2509_00105_amd.binding as b

    return b.lib()


def declared_symbols():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(kvh_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert set(names) >= {"kvh_encode", "kvh_decode", "kvh_encode_batch", "kvh_decode_batch", "kvh_encode_chunked",
                          "kvh_blob_size", "kvh_level_bits", "kvh_num_levels", "kvh_strerror", "kvh_copy_probe",
                          "kvh_kept_tokens", "kvh_encode_kept", "kvh_decode_kept", "kvh_transcode", "kvh_transcode_batch",
                          "kvh_loader_create", "kvh_loader_run", "kvh_loader_destroy", "kvh_loader_slot_bytes",
                          "kvh_policy_plan", "kvh_policy_utility", "kvh_policy_marginal_utility_drop",
                          "kvh_encode_kept_batch", "kvh_decode_kept_batch"}
    for n in names:
        assert hasattr(lib, n), n


def test_level_table_and_blob_size_agree_with_oracle(lib):
    assert lib.kvh_num_levels() == oracle.num_levels() == 3
    assert [lib.kvh_level_bits(i) for i in range(-2, 5)] == [oracle.level_bits(i) for i in range(-2, 5)]
    rng = np.random.default_rng(0)
    for _ in range(500):
        l, n, m, lv = int(rng.integers(0, 90)), int(rng.integers(0, 3000)), int(rng.integers(0, 20)), int(rng.integers(-1, 4))
        c = 128 * m + (64 if rng.random() < 0.1 else 0)
        assert lib.kvh_blob_size(l, n, c, lv) == oracle.blob_size(l, n, c, lv), (l, n, c, lv)
    assert lib.kvh_blob_size(32, 256, 1024, 2) == 4_718_656


def test_strerror_covers_every_status(lib):
    seen = {lib.kvh_strerror(s) for s in range(-6, 1)}
    assert len(seen) == 7 and b"unknown status" not in seen
    assert lib.kvh_strerror(-99) == b"unknown status"


def test_argument_errors_are_found_on_the_host(lib):
    """Every call below must be rejected before a launch (fake, suitably aligned pointers)."""
    import torch

    if torch.cuda.is_available():
        pytest.skip("fake device pointers: run only where nothing could be launched")
    from paper_2509_00105_amd.binding import _KVView

    P = 0x10000
    view = _KVView(P, P, 1024 * 256, 1024)
    v = ctypes.byref(view)
    E_ARG, E_LEVEL, E_SHAPE, E_SIZE, E_ALIGN = -1, -2, -3, -4, -5
    big = 1 << 40
    enc = lib.kvh_encode
    assert enc(None, 0, 1, 128, 1024, 0, P, big, None) == E_ARG
    assert enc(v, 0, 1, 128, 1024, 0, None, big, None) == E_ARG
    assert enc(v, 2, 1, 128, 1024, 0, P, big, None) == E_ARG
    assert enc(v, 0, 1, 128, 1024, 4, P, big, None) == E_LEVEL
    assert enc(v, 0, 1, 128, 1024, -1, P, big, None) == E_LEVEL
    assert enc(v, 0, 0, 128, 1024, 0, P, big, None) == E_SHAPE
    assert enc(v, 0, 1, 0, 1024, 0, P, big, None) == E_SHAPE
    assert enc(v, 0, 1, 128, 1000, 0, P, big, None) == E_SHAPE
    assert enc(v, 0, 1, 128, 1024, 0, P, lib.kvh_blob_size(1, 128, 1024, 0) - 1, None) == E_SIZE
    assert enc(v, 0, 1, 128, 1024, 0, P + 8, big, None) == E_ALIGN
    assert enc(ctypes.byref(_KVView(P + 2, P, 1024, 1024)), 0, 1, 128, 1024, 0, P, big, None) == E_ALIGN
    assert enc(ctypes.byref(_KVView(P, P, 1024, 1020)), 0, 1, 128, 1024, 0, P, big, None) == E_ALIGN
    assert enc(ctypes.byref(_KVView(None, P, 1024, 1024)), 0, 1, 128, 1024, 0, P, big, None) == E_ARG

    dec = lib.kvh_decode
    assert dec(None, 0, 1, 128, 1024, 0, v, 0, None, 16, None, None) == E_ARG
    assert dec(P, 0, 1, 128, 1024, 0, None, 0, None, 16, None, None) == E_ARG
    assert dec(P, 0, 1, 128, 1024, 0, v, -1, None, 16, None, None) == E_ARG
    assert dec(P, 0, 1, 128, 1024, 7, v, 0, None, 16, None, None) == E_LEVEL
    assert dec(P, 0, 1, 128, 192, 0, v, 0, None, 16, None, None) == E_SHAPE
    assert dec(P, 0, 1, 128, 1024, 0, v, 0, P, 0, None, None) == E_ARG
    assert dec(P + 4, 0, 1, 128, 1024, 0, v, 0, None, 16, None, None) == E_ALIGN
    assert dec(P, 0, 1, 128, 1024, 0, v, 2**31 - 64, None, 16, None, None) == E_ARG
    assert dec(P, 0, 1, 128, 1024, 0, ctypes.byref(_KVView(P, P, 1024 * 256, 512)), 0, None, 16, None, None) == E_ARG  # rows overlap
    assert lib.kvh_decode_batch(P, 1, 256, 0, 1, 1024, ctypes.byref(_KVView(P, P, 0, 0)), 16, None, None) == E_ARG

    lv = (ctypes.c_int8 * 2)(0, 1)
    off = (ctypes.c_size_t * 2)(0, 1 << 20)
    ch = lib.kvh_encode_chunked
    assert ch(v, 0, 1, 256, 1024, 100, lv, P, off, big, None) == E_SHAPE        # chunk not a multiple of 128
    assert ch(v, 0, 1, 256, 1024, 128, None, P, off, big, None) == E_ARG
    assert ch(v, 0, 1, 256, 1024, 128, (ctypes.c_int8 * 2)(0, 5), P, off, big, None) == E_LEVEL
    assert ch(v, 0, 1, 256, 1024, 128, lv, P, (ctypes.c_size_t * 2)(0, 8), big, None) == E_ALIGN
    assert ch(v, 0, 1, 256, 1024, 128, lv, P, off, (1 << 20) + 100, None) == E_SIZE

    assert lib.kvh_encode_batch(None, 1, 256, 0, 1, 1024, v, None) == E_ARG
    assert lib.kvh_encode_batch(P, 0, 256, 0, 1, 1024, v, None) == E_ARG
    assert lib.kvh_encode_batch(P, 70000, 256, 0, 1, 1024, v, None) == E_ARG
    assert lib.kvh_encode_batch(P, 1, 256, 0, 1, 100, v, None) == E_SHAPE
    assert lib.kvh_decode_batch(None, 1, 256, 0, 1, 1024, v, 16, None, None) == E_ARG
    assert lib.kvh_decode_batch(P, 1, 256, 0, 1, 1024, v, 0, None, None) == E_ARG
    assert lib.kvh_decode_batch(P, 1, 0, 0, 1, 1024, v, 16, None, None) == E_SHAPE

    kept_e, kept_d = lib.kvh_encode_kept, lib.kvh_decode_kept
    assert lib.kvh_kept_tokens(10, 2, 3) == 5 and lib.kvh_kept_tokens(10, 0, 0) == 0 and lib.kvh_kept_tokens(0, 1, 1) == 0
    assert lib.kvh_kept_tokens(10, 2**31 - 1, 2**31 - 1) == 10
    assert kept_e(v, 0, 1, 256, 1024, 0, 0, 0, P, big, None) == E_SHAPE      # nothing kept
    assert kept_e(v, 0, 1, 256, 1024, -1, 8, 0, P, big, None) == E_SHAPE
    assert kept_e(v, 0, 1, 256, 1024, 4, 60, 5, P, big, None) == E_LEVEL
    assert kept_e(v, 0, 1, 256, 1024, 4, 60, 0, P, lib.kvh_blob_size(1, 64, 1024, 0) - 1, None) == E_SIZE
    assert kept_e(v, 0, 1, 256, 1024, 4, 60, 0, P + 4, big, None) == E_ALIGN
    assert kept_d(None, 0, 1, 256, 1024, 4, 60, 0, v, 0, 0, None, 16, None, None) == E_ARG
    assert kept_d(P, 0, 1, 256, 1024, 0, 0, 0, v, 0, 0, None, 16, None, None) == E_SHAPE
    assert kept_d(P, 0, 1, 256, 1024, 4, 60, 0, v, 0, 0, P, 0, None, None) == E_ARG
    assert kept_d(P, 0, 1, 256, 1024, 4, 60, 0, v, 2**31 - 100, 0, None, 16, None, None) == E_ARG

    assert lib.kvh_encode_kept_batch(None, 1, 256, 0, 1, 1024, v, None) == E_ARG
    assert lib.kvh_encode_kept_batch(P, 1, 256, 0, 1, 1000, v, None) == E_SHAPE
    assert lib.kvh_decode_kept_batch(P, 0, 256, 0, 1, 1024, v, 16, None, None) == E_ARG
    assert lib.kvh_decode_kept_batch(P, 1, 256, 0, 1, 1024, v, 0, None, None) == E_ARG

    tc = lib.kvh_transcode
    Q = P + (1 << 30)
    assert tc(None, 0, 1, 128, 1024, 0, 2, Q, big, None, None) == E_ARG
    assert tc(P, 0, 1, 128, 1024, 0, 2, None, big, None, None) == E_ARG
    assert tc(P, 5, 1, 128, 1024, 0, 2, Q, big, None, None) == E_ARG
    assert tc(P, 0, 1, 128, 1024, 3, 2, Q, big, None, None) == E_LEVEL
    assert tc(P, 0, 1, 128, 1024, 0, -1, Q, big, None, None) == E_LEVEL
    assert tc(P, 0, 1, 128, 1024, 0, 3, Q, big, None, None) == E_LEVEL      # the raw level holds rows, not codes
    assert tc(P, 0, 1, 128, 1000, 0, 2, Q, big, None, None) == E_SHAPE
    assert tc(P, 0, 1, 128, 1024, 0, 2, Q, lib.kvh_blob_size(1, 128, 1024, 2) - 1, None, None) == E_SIZE
    assert tc(P + 8, 0, 1, 128, 1024, 0, 2, Q, big, None, None) == E_ALIGN
    assert tc(P, 0, 1, 128, 1024, 0, 2, Q + 8, big, None, None) == E_ALIGN
    assert tc(P, 0, 1, 128, 1024, 0, 2, P + 4096, big, None, None) == E_ARG   # destination inside the source blob
    assert tc(P + 4096, 0, 1, 128, 1024, 0, 2, P, big, None, None) == E_ARG   # source inside the destination blob
    assert lib.kvh_transcode_batch(None, 1, 256, 0, 1, 1024, None, None) == E_ARG
    assert lib.kvh_transcode_batch(P, 0, 256, 0, 1, 1024, None, None) == E_ARG
    assert lib.kvh_transcode_batch(P, 1, 256, 0, 1, 1000, None, None) == E_SHAPE
    h = ctypes.c_void_p()
    assert lib.kvh_loader_create(None, P, 1 << 20, 2) == E_ARG
    assert lib.kvh_loader_create(ctypes.byref(h), None, 1 << 20, 2) == E_ARG and not h
    assert lib.kvh_loader_create(ctypes.byref(h), P, 1 << 20, 0) == E_ARG
    assert lib.kvh_loader_create(ctypes.byref(h), P, 1 << 20, 65) == E_ARG
    assert lib.kvh_loader_create(ctypes.byref(h), P + 8, 1 << 20, 2) == E_ALIGN
    assert lib.kvh_loader_create(ctypes.byref(h), P, 100, 2) == E_SIZE and not h
    assert lib.kvh_loader_run(None, P, 1, 0, 1, 1024, v, 16, None, None) == E_ARG
    assert lib.kvh_loader_destroy(None) == E_ARG
    assert lib.kvh_loader_slot_bytes(None) == 0
    assert lib.kvh_copy_probe(P, P + 4096, 100, None) == E_ALIGN
    assert lib.kvh_copy_probe(None, P, 4096, None) == E_ARG


def test_binding_refuses_host_tensors(lib):
    import torch

    import paper_2509_00105_amd as kvh

    k = torch.zeros((1, 128, 128), dtype=torch.float16)
    with pytest.raises(ValueError):
        kvh.encode(k, k, 0)


def test_transcode_default_output_is_device_memory_for_a_pinned_host_source(monkeypatch):
    """A source blob in pinned host memory reports device "cpu"; the output the binding allocates by default
    must still be memory the kernel can write (the launch itself is mocked: nothing runs)."""
    import torch

    from paper_2509_00105_amd import binding as b

    class FakeTensor:
        def __init__(self, is_cuda, pinned, n=4096):
            self.is_cuda, self._pinned, self._n, self.device = is_cuda, pinned, n, torch.device("cuda" if is_cuda else "cpu")

        def is_pinned(self):
            return self._pinned

        def data_ptr(self):
            return 0x10000

        def numel(self):
            return self._n

    class FakeLib:
        def __init__(self):
            self.calls = []

        def kvh_blob_size(self, l, n, c, level):
            return 4096

        def kvh_transcode(self, *args):
            self.calls.append(args)
            return 0

    fake = FakeLib()
    asked = []

    def fake_empty(size, dtype=None, device=None):
        asked.append(torch.device(device))
        return FakeTensor(torch.device(device).type == "cuda", False, size)

    monkeypatch.setattr(b, "lib", lambda: fake)
    monkeypatch.setattr(b, "_stream_ptr", lambda s: 0)
    monkeypatch.setattr(b.torch, "empty", fake_empty)
    out = b.transcode(FakeTensor(False, True), b.BF16, 1, 128, 128, 0, 1)     # pinned host source
    assert asked[-1].type == "cuda" and out.is_cuda and len(fake.calls) == 1
    out = b.transcode(FakeTensor(True, False), b.BF16, 1, 128, 128, 0, 1)     # device source
    assert asked[-1].type == "cuda" and len(fake.calls) == 2
    with pytest.raises(ValueError):                                           # pageable host source
        b.transcode(FakeTensor(False, False), b.BF16, 1, 128, 128, 0, 1)
    with pytest.raises(ValueError):                                           # pageable host destination
        b.transcode(FakeTensor(True, False), b.BF16, 1, 128, 128, 0, 1, out=FakeTensor(False, False))
    assert len(fake.calls) == 2


def test_bench_traffic_figures_are_those_of_the_committed_profile(lib):
    """bench.py reports HBM traffic per launch from the rocprofv3 summary under profiles/ (counters cannot be read
    inside a run).  The parser must find all nine kernels there, and each figure must be what the table's own
    counter columns give (2.0 x FETCH_SIZE + 1.0 x WRITE_SIZE KiB) and sit within 10 % above the algorithmic bytes."""
    import sys

    sys.path.insert(0, ROOT)
    import bench

    got = bench.profiled_traffic()
    want_keys = {("encode", b) for b in (8, 4, 2)} | {("decode", b) for b in (8, 4, 2)} | \
                {("transcode", 8, 4), ("transcode", 8, 2), ("transcode", 4, 2)}
    assert set(got) == want_keys
    unc = 2 * 32 * 8192 * 1024 * 2
    blob = {b: 32 * lib.kvh_blob_size(32, 256, 1024, lv) for lv, b in enumerate((8, 4, 2))}
    for key, traffic in got.items():
        alg = unc + blob[key[1]] if key[0] != "transcode" else blob[key[1]] + blob[key[2]]
        assert alg <= traffic <= 1.10 * alg, (key, traffic, alg)
    rows = [ln for ln in open(bench.PROFILE_SUMMARY).read().splitlines() if ln.startswith("| enc") or ln.startswith("| dec") or ln.startswith("| transcode")]
    assert len(rows) == 9
    for ln in rows:
        cells = [x.strip() for x in ln.strip("|").split("|")]
        fetch, write, traffic = int(cells[5]), int(cells[6]), int(cells[7])
        assert traffic == (2 * fetch + write) * 1024, cells[0]
    assert bench.profiled_traffic("/nonexistent/file.md") == {}


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asking for more must end with a message, before any GPU work."""
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_binding_records_have_the_layout_of_the_c_structs(tmp_path):
    """The binding marshals descriptors as numpy records; a C program compiled against include/kvh.h prints
    sizeof/offsetof of every struct field and the two must agree name by name."""
    import subprocess

    from paper_2509_00105_amd import binding as b

    records = {"kvh_enc_item": b.ENC_ITEM, "kvh_item": b.DEC_ITEM, "kvh_tc_item": b.TC_ITEM,
               "kvh_load_item": b.LOAD_ITEM, "kvh_kept_enc_item": b.KEPT_ENC_ITEM, "kvh_kept_item": b.KEPT_ITEM,
               "kvh_policy_entry": b.POLICY_ENTRY, "kvh_policy_tier": b.POLICY_TIER}
    lines = ['#include <stddef.h>', '#include <stdio.h>', '#include "kvh.h"', 'int main(void) {']
    for name, dt in records.items():
        lines.append('  printf("%s size %%zu\\n", sizeof(%s));' % (name, name))
        for field in dt.names:
            lines.append('  printf("%s %s %%zu\\n", offsetof(%s, %s));' % (name, field, name, field))
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    seen = 0
    for line in out:
        if not line:
            continue
        name, field, value = line.split()
        dt = records[name]
        if field == "size":
            assert dt.itemsize == int(value), (name, dt.itemsize, value)
        else:
            assert dt.fields[field][1] == int(value), (name, field, dt.fields[field][1], value)
        seen += 1
    assert seen == sum(len(dt.names) + 1 for dt in records.values())
    view = b._KVView
    assert ctypes.sizeof(view) == 32 and [f[0] for f in view._fields_] == ["k", "v", "layer_stride", "token_stride"]
