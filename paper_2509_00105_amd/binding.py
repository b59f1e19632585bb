"""ctypes binding of the C ABI in include/kvh.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkvh.so")

F16, BF16 = 0, 1
_TORCH_DT = {torch.float16: F16, torch.bfloat16: BF16}


class KVHError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, strerror(status)))


class _KVView(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("layer_stride", ctypes.c_int64), ("token_stride", ctypes.c_int64)]


# Device-resident job descriptors, built as structured numpy arrays and uploaded by the caller.
ENC_ITEM = np.dtype([("blob", "<u8"), ("src_token0", "<i8"), ("n_tokens", "<i4"), ("level", "<i4")], align=True)
DEC_ITEM = np.dtype([("blob", "<u8"), ("n_tokens", "<i4"), ("level", "<i4"), ("dst_token0", "<i8"),
                     ("page_table", "<u8")], align=True)
TC_ITEM = np.dtype([("src", "<u8"), ("dst", "<u8"), ("n_tokens", "<i4"), ("level_in", "<i4"), ("level_out", "<i4"),
                    ("reserved", "<i4")], align=True)
LOAD_ITEM = np.dtype([("blob_host", "<u8"), ("n_tokens", "<i4"), ("level", "<i4"), ("dst_token0", "<i8"),
                      ("page_table", "<u8"), ("orig_tokens", "<i4"), ("sink", "<i4"), ("window", "<i4"),
                      ("compact", "<i4")], align=True)  # a HOST array, unlike the others
KEPT_ENC_ITEM = np.dtype([("blob", "<u8"), ("src_token0", "<i8"), ("orig_tokens", "<i4"), ("sink", "<i4"),
                          ("window", "<i4"), ("level", "<i4")], align=True)
KEPT_ITEM = np.dtype([("blob", "<u8"), ("n_tokens", "<i4"), ("level", "<i4"), ("dst_token0", "<i8"), ("page_table", "<u8"),
                      ("orig_tokens", "<i4"), ("sink", "<i4"), ("window", "<i4"), ("compact", "<i4")], align=True)
POLICY_ENTRY = np.dtype([("freq", "<f8"), ("first", "<i4"), ("n_choices", "<i4"), ("min_choice", "<i4"),
                         ("reserved", "<i4")], align=True)
POLICY_TIER = np.dtype([("bandwidth", "<f8"), ("capacity", "<f8")], align=True)
assert POLICY_ENTRY.itemsize == 24 and POLICY_TIER.itemsize == 16
assert ENC_ITEM.itemsize == 24 and DEC_ITEM.itemsize == 32 and TC_ITEM.itemsize == 32 and LOAD_ITEM.itemsize == 48
assert KEPT_ENC_ITEM.itemsize == 32 and KEPT_ITEM.itemsize == 48

_lib = None


def lib() -> ctypes.CDLL:
    """Load libkvh.so (built in-tree by `python -m paper_2509_00105_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libkvh.so is not built: run `python -m paper_2509_00105_amd.build` "
                              "(there is no CPU fallback for the HIP path)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        view = ctypes.POINTER(_KVView)
        L.kvh_num_levels.restype = i32
        L.kvh_num_levels.argtypes = []
        L.kvh_level_bits.restype = i32
        L.kvh_level_bits.argtypes = [i32]
        L.kvh_blob_size.restype = sz
        L.kvh_blob_size.argtypes = [i32, i32, i32, i32]
        L.kvh_encode.restype = i32
        L.kvh_encode.argtypes = [view, i32, i32, i32, i32, i32, vp, sz, vp]
        L.kvh_encode_chunked.restype = i32
        L.kvh_encode_chunked.argtypes = [view, i32, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_int8), vp,
                                         ctypes.POINTER(sz), sz, vp]
        L.kvh_encode_batch.restype = i32
        L.kvh_encode_batch.argtypes = [vp, i32, i32, i32, i32, i32, view, vp]
        L.kvh_decode.restype = i32
        L.kvh_decode.argtypes = [vp, i32, i32, i32, i32, i32, view, i64, vp, i32, vp, vp]
        L.kvh_decode_batch.restype = i32
        L.kvh_decode_batch.argtypes = [vp, i32, i32, i32, i32, i32, view, i32, vp, vp]
        L.kvh_kept_tokens.restype = i32
        L.kvh_kept_tokens.argtypes = [i32, i32, i32]
        L.kvh_encode_kept.restype = i32
        L.kvh_encode_kept.argtypes = [view, i32, i32, i32, i32, i32, i32, i32, vp, sz, vp]
        L.kvh_decode_kept.restype = i32
        L.kvh_decode_kept.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, view, i64, i32, vp, i32, vp, vp]
        L.kvh_encode_kept_batch.restype = i32
        L.kvh_encode_kept_batch.argtypes = [vp, i32, i32, i32, i32, i32, view, vp]
        L.kvh_decode_kept_batch.restype = i32
        L.kvh_decode_kept_batch.argtypes = [vp, i32, i32, i32, i32, i32, view, i32, vp, vp]
        L.kvh_transcode.restype = i32
        L.kvh_transcode.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, sz, vp, vp]
        L.kvh_transcode_batch.restype = i32
        L.kvh_transcode_batch.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp]
        L.kvh_loader_create.restype = i32
        L.kvh_loader_create.argtypes = [ctypes.POINTER(vp), vp, sz, i32]
        L.kvh_loader_slot_bytes.restype = sz
        L.kvh_loader_slot_bytes.argtypes = [vp]
        L.kvh_loader_run.restype = i32
        L.kvh_loader_run.argtypes = [vp, vp, i32, i32, i32, i32, view, i32, vp, vp]
        L.kvh_loader_destroy.restype = i32
        L.kvh_loader_destroy.argtypes = [vp]
        L.kvh_load_static.restype = i32
        L.kvh_load_static.argtypes = [vp, i32, i32, i32, i32, view, i32, vp, vp]
        f64 = ctypes.c_double
        L.kvh_policy_utility.restype = f64
        L.kvh_policy_utility.argtypes = [f64] * 5
        L.kvh_policy_marginal_utility_drop.restype = f64
        L.kvh_policy_marginal_utility_drop.argtypes = [f64] * 4
        L.kvh_policy_plan.restype = i32
        L.kvh_policy_plan.argtypes = [vp, i32, vp, vp, i32, vp, i32, f64, vp, vp, ctypes.POINTER(f64)]
        L.kvh_copy_probe.restype = i32
        L.kvh_copy_probe.argtypes = [vp, vp, sz, vp]
        L.kvh_stream_probe.restype = i32
        L.kvh_stream_probe.argtypes = [vp, vp, sz, i32, i32, vp]
        L.kvh_time_next_launch.restype = i32
        L.kvh_time_next_launch.argtypes = [vp, vp]
        L.kvh_selftest_division.restype = i32
        L.kvh_selftest_division.argtypes = [vp, vp]
        L.kvh_decode_chunked.restype = i32
        L.kvh_decode_chunked.argtypes = [vp, ctypes.POINTER(sz), ctypes.POINTER(ctypes.c_int8), i32, i32, i32, i32, i32,
                                         view, i64, vp, i32, vp, vp]
        L.kvh_strerror.restype = ctypes.c_char_p
        L.kvh_strerror.argtypes = [i32]
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().kvh_strerror(status).decode()


def num_levels() -> int:
    return lib().kvh_num_levels()


def level_bits(level: int) -> int:
    return lib().kvh_level_bits(level)


def blob_size(l: int, n_tokens: int, c: int, level: int) -> int:
    return lib().kvh_blob_size(l, n_tokens, c, level)


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _require_cuda(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("device tensor expected (the HIP path has no CPU fallback)")


def _require_visible(*tensors):
    """Blob buffers may live in HBM or in pinned host memory (both are addressable by the kernels)."""
    for t in tensors:
        if t is not None and not (t.is_cuda or t.is_pinned()):
            raise ValueError("device tensor or pinned host tensor expected (pageable host memory is not visible to the GPU)")


def _view(k: torch.Tensor, v: torch.Tensor, paged: bool = False):
    """kvh_kv_view of K/V tensors [l][tokens][c] (or [l][P][block][c] when paged)."""
    _require_cuda(k, v)
    if k.dtype not in _TORCH_DT or v.dtype != k.dtype:
        raise ValueError("K and V must both be float16 or both bfloat16")
    want = 4 if paged else 3
    if k.dim() != want or v.dim() != want or k.stride() != v.stride() or k.shape != v.shape:
        raise ValueError("K and V must be %d-d with equal shapes and strides" % want)
    if k.stride(-1) != 1:
        raise ValueError("channel stride must be 1")
    if paged and k.stride(1) != k.stride(2) * k.shape[2]:
        raise ValueError("blocks of a paged cache must be densely packed")
    ts = k.stride(2) if paged else k.stride(1)
    return _KVView(k.data_ptr(), v.data_ptr(), k.stride(0), ts), _TORCH_DT[k.dtype]


def _check(rc: int, where: str):
    if rc != 0:
        raise KVHError(rc, where)


def encode(k: torch.Tensor, v: torch.Tensor, level: int, blob: torch.Tensor | None = None, n_tokens: int | None = None,
           stream=None) -> torch.Tensor:
    """kvh_encode: tokens [0, n_tokens) of K/V [l][N][c] -> one blob (uint8 device tensor)."""
    view, dt = _view(k, v)
    l, N, c = k.shape
    n = N if n_tokens is None else n_tokens
    if blob is None:
        size = blob_size(l, n, c, level)
        if size == 0:
            _check(lib().kvh_encode(ctypes.byref(view), dt, l, n, c, level, None, 0, None), "kvh_encode")
        blob = torch.empty(size, dtype=torch.uint8, device=k.device)
    _require_visible(blob)
    _check(lib().kvh_encode(ctypes.byref(view), dt, l, n, c, level, blob.data_ptr(), blob.numel(), _stream_ptr(stream)),
           "kvh_encode")
    return blob


def encode_chunked(k: torch.Tensor, v: torch.Tensor, chunk: int, levels, blobs: torch.Tensor, blob_offsets,
                   stream=None) -> None:
    """kvh_encode_chunked: chunk blobs written at the given byte offsets of `blobs` (host-side descriptors)."""
    view, dt = _view(k, v)
    _require_cuda(blobs)
    l, N, c = k.shape
    lv = np.ascontiguousarray(levels, dtype=np.int8)
    off = np.ascontiguousarray(blob_offsets, dtype=np.uint64)
    n_chunks = -(-N // chunk) if chunk > 0 else 0
    if lv.size != n_chunks or off.size != n_chunks:
        raise ValueError("levels and blob_offsets need ceil(N/chunk) entries")
    _check(lib().kvh_encode_chunked(ctypes.byref(view), dt, l, N, c, chunk,
                                    lv.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)), blobs.data_ptr(),
                                    off.ctypes.data_as(ctypes.POINTER(ctypes.c_size_t)), blobs.numel(),
                                    _stream_ptr(stream)), "kvh_encode_chunked")


def make_enc_items(blob_ptrs, src_token0, n_tokens, levels, device) -> torch.Tensor:
    """Upload an array of kvh_enc_item (argument marshalling; returns a uint8 device tensor)."""
    a = np.zeros(len(blob_ptrs), dtype=ENC_ITEM)
    a["blob"], a["src_token0"], a["n_tokens"], a["level"] = blob_ptrs, src_token0, n_tokens, levels
    return torch.from_numpy(a.view(np.uint8).copy()).to(device)


def make_dec_items(blob_ptrs, n_tokens, levels, dst_token0, page_table_ptrs, device) -> torch.Tensor:
    """Upload an array of kvh_item (argument marshalling; returns a uint8 device tensor)."""
    a = np.zeros(len(blob_ptrs), dtype=DEC_ITEM)
    a["blob"], a["n_tokens"], a["level"], a["dst_token0"], a["page_table"] = \
        blob_ptrs, n_tokens, levels, dst_token0, page_table_ptrs
    return torch.from_numpy(a.view(np.uint8).copy()).to(device)


def encode_batch(items: torch.Tensor, n_items: int, max_tokens_per_item: int, k: torch.Tensor, v: torch.Tensor,
                 stream=None) -> None:
    """kvh_encode_batch: all items in one launch; `items` comes from make_enc_items."""
    view, dt = _view(k, v)
    _require_cuda(items)
    l, _, c = k.shape
    _check(lib().kvh_encode_batch(items.data_ptr(), n_items, max_tokens_per_item, dt, l, c, ctypes.byref(view),
                                  _stream_ptr(stream)), "kvh_encode_batch")


def decode(blob: torch.Tensor, level: int, n_tokens: int, k_dst: torch.Tensor, v_dst: torch.Tensor, dst_token0: int = 0,
           page_table: torch.Tensor | None = None, block_tokens: int = 16, status: torch.Tensor | None = None,
           stream=None) -> None:
    """kvh_decode: one blob -> rows of a contiguous [l][N][c] or paged [l][P][block][c] destination."""
    paged = page_table is not None
    view, dt = _view(k_dst, v_dst, paged)
    _require_cuda(blob, page_table, status)
    if paged and page_table.dtype != torch.int32:
        raise ValueError("page_table must be int32")
    if status is not None and status.dtype != torch.int32:
        raise ValueError("status must be int32")
    l, c = k_dst.shape[0], k_dst.shape[-1]
    _check(lib().kvh_decode(blob.data_ptr(), dt, l, n_tokens, c, level, ctypes.byref(view), dst_token0,
                            page_table.data_ptr() if paged else None, block_tokens,
                            status.data_ptr() if status is not None else None, _stream_ptr(stream)), "kvh_decode")


def decode_chunked(blobs: torch.Tensor, blob_offsets, levels, chunk: int, n_tokens: int, k_dst: torch.Tensor,
                   v_dst: torch.Tensor, dst_token0: int = 0, page_table: torch.Tensor | None = None,
                   block_tokens: int = 16, status: torch.Tensor | None = None, stream=None) -> None:
    """kvh_decode_chunked: an n_tokens entry whose chunk blobs sit at the given byte offsets (host-side descriptors)."""
    paged = page_table is not None
    view, dt = _view(k_dst, v_dst, paged)
    _require_cuda(blobs, page_table, status)
    lv = np.ascontiguousarray(levels, dtype=np.int8)
    off = np.ascontiguousarray(blob_offsets, dtype=np.uint64)
    n_chunks = -(-n_tokens // chunk) if chunk > 0 else 0
    if lv.size != n_chunks or off.size != n_chunks:
        raise ValueError("levels and blob_offsets need ceil(N/chunk) entries")
    if paged and page_table.dtype != torch.int32:
        raise ValueError("page_table must be int32")
    if status is not None and (status.dtype != torch.int32 or status.numel() < n_chunks):
        raise ValueError("status must be int32 with one entry per chunk")
    l, c = k_dst.shape[0], k_dst.shape[-1]
    _check(lib().kvh_decode_chunked(blobs.data_ptr(), off.ctypes.data_as(ctypes.POINTER(ctypes.c_size_t)),
                                    lv.ctypes.data_as(ctypes.POINTER(ctypes.c_int8)), dt, l, n_tokens, c, chunk,
                                    ctypes.byref(view), dst_token0, page_table.data_ptr() if paged else None,
                                    block_tokens, status.data_ptr() if status is not None else None,
                                    _stream_ptr(stream)), "kvh_decode_chunked")


def decode_batch(items: torch.Tensor, n_items: int, max_tokens_per_item: int, k_dst: torch.Tensor,
                 v_dst: torch.Tensor, paged: bool = False, block_tokens: int = 16,
                 status: torch.Tensor | None = None, stream=None) -> None:
    """kvh_decode_batch: all items in one launch; `items` comes from make_dec_items."""
    view, dt = _view(k_dst, v_dst, paged)
    _require_cuda(items, status)
    if status is not None and (status.dtype != torch.int32 or status.numel() < n_items):
        raise ValueError("status must be int32 with one entry per item")
    l, c = k_dst.shape[0], k_dst.shape[-1]
    _check(lib().kvh_decode_batch(items.data_ptr(), n_items, max_tokens_per_item, dt, l, c, ctypes.byref(view),
                                  block_tokens, status.data_ptr() if status is not None else None,
                                  _stream_ptr(stream)), "kvh_decode_batch")


def kept_tokens(N: int, sink: int, window: int) -> int:
    return lib().kvh_kept_tokens(N, sink, window)


def encode_kept(k: torch.Tensor, v: torch.Tensor, sink: int, window: int, level: int,
                blob: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """kvh_encode_kept: keep the first `sink` and last `window` tokens of K/V [l][N][c], encode them."""
    view, dt = _view(k, v)
    l, N, c = k.shape
    if blob is None:
        size = blob_size(l, kept_tokens(N, sink, window), c, level)
        if size == 0:
            _check(lib().kvh_encode_kept(ctypes.byref(view), dt, l, N, c, sink, window, level, None, 0, None), "kvh_encode_kept")
        blob = torch.empty(size, dtype=torch.uint8, device=k.device)
    _require_visible(blob)
    _check(lib().kvh_encode_kept(ctypes.byref(view), dt, l, N, c, sink, window, level, blob.data_ptr(), blob.numel(),
                                 _stream_ptr(stream)), "kvh_encode_kept")
    return blob


def decode_kept(blob: torch.Tensor, level: int, N: int, sink: int, window: int, k_dst: torch.Tensor, v_dst: torch.Tensor,
                dst_token0: int = 0, compact: bool = False, page_table: torch.Tensor | None = None, block_tokens: int = 16,
                status: torch.Tensor | None = None, stream=None) -> None:
    """kvh_decode_kept: a token-dropped blob -> original (or compact) rows of a contiguous or paged destination."""
    paged = page_table is not None
    view, dt = _view(k_dst, v_dst, paged)
    _require_cuda(blob, page_table, status)
    if paged and page_table.dtype != torch.int32:
        raise ValueError("page_table must be int32")
    if status is not None and status.dtype != torch.int32:
        raise ValueError("status must be int32")
    l, c = k_dst.shape[0], k_dst.shape[-1]
    _check(lib().kvh_decode_kept(blob.data_ptr(), dt, l, N, c, sink, window, level, ctypes.byref(view), dst_token0,
                                 int(compact), page_table.data_ptr() if paged else None, block_tokens,
                                 status.data_ptr() if status is not None else None, _stream_ptr(stream)),
           "kvh_decode_kept")


def make_kept_enc_items(blob_ptrs, src_token0, orig_tokens, sinks, windows, levels, device) -> torch.Tensor:
    """Upload an array of kvh_kept_enc_item (argument marshalling; returns a uint8 device tensor)."""
    a = np.zeros(len(blob_ptrs), dtype=KEPT_ENC_ITEM)
    a["blob"], a["src_token0"], a["orig_tokens"], a["sink"], a["window"], a["level"] = \
        blob_ptrs, src_token0, orig_tokens, sinks, windows, levels
    return torch.from_numpy(a.view(np.uint8).copy()).to(device)


def make_kept_items(blob_ptrs, n_tokens, levels, dst_token0, page_table_ptrs, orig_tokens, sinks, windows, compact,
                    device) -> torch.Tensor:
    """Upload an array of kvh_kept_item (argument marshalling; returns a uint8 device tensor)."""
    a = np.zeros(len(blob_ptrs), dtype=KEPT_ITEM)
    a["blob"], a["n_tokens"], a["level"], a["dst_token0"], a["page_table"] = \
        blob_ptrs, n_tokens, levels, dst_token0, page_table_ptrs
    a["orig_tokens"], a["sink"], a["window"], a["compact"] = orig_tokens, sinks, windows, compact
    return torch.from_numpy(a.view(np.uint8).copy()).to(device)


def encode_kept_batch(items: torch.Tensor, n_items: int, max_kept_tokens_per_item: int, k: torch.Tensor,
                      v: torch.Tensor, stream=None) -> None:
    """kvh_encode_kept_batch: all items in one launch; `items` comes from make_kept_enc_items."""
    view, dt = _view(k, v)
    _require_cuda(items)
    l, _, c = k.shape
    _check(lib().kvh_encode_kept_batch(items.data_ptr(), n_items, max_kept_tokens_per_item, dt, l, c,
                                       ctypes.byref(view), _stream_ptr(stream)), "kvh_encode_kept_batch")


def decode_kept_batch(items: torch.Tensor, n_items: int, max_tokens_per_item: int, k_dst: torch.Tensor,
                      v_dst: torch.Tensor, paged: bool = False, block_tokens: int = 16,
                      status: torch.Tensor | None = None, stream=None) -> None:
    """kvh_decode_kept_batch: ordinary and token-dropped blobs in one launch; `items` from make_kept_items."""
    view, dt = _view(k_dst, v_dst, paged)
    _require_cuda(items, status)
    if status is not None and (status.dtype != torch.int32 or status.numel() < n_items):
        raise ValueError("status must be int32 with one entry per item")
    l, c = k_dst.shape[0], k_dst.shape[-1]
    _check(lib().kvh_decode_kept_batch(items.data_ptr(), n_items, max_tokens_per_item, dt, l, c, ctypes.byref(view),
                                       block_tokens, status.data_ptr() if status is not None else None,
                                       _stream_ptr(stream)), "kvh_decode_kept_batch")


def _dt_code(dtype) -> int:
    if dtype in _TORCH_DT:
        return _TORCH_DT[dtype]
    if dtype in (F16, BF16):
        return int(dtype)
    raise ValueError("dtype must be torch.float16, torch.bfloat16, F16 or BF16")


def transcode(blob: torch.Tensor, dtype, l: int, n_tokens: int, c: int, level_in: int, level_out: int,
              out: torch.Tensor | None = None, status: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """kvh_transcode: a blob of n_tokens stored tokens at level_in -> a blob at level_out (uint8 device tensor)."""
    _require_visible(blob, out)
    _require_cuda(status)
    dt = _dt_code(dtype)
    if status is not None and status.dtype != torch.int32:
        raise ValueError("status must be int32")
    if out is None:
        size = blob_size(l, n_tokens, c, level_out)
        if size == 0:
            _check(lib().kvh_transcode(blob.data_ptr(), dt, l, n_tokens, c, level_in, level_out, None, 0, None, None),
                   "kvh_transcode")
        # A source in pinned host memory has device "cpu": the default output still has to be memory the
        # kernel can write, so it goes to the current GPU (pass `out=` to write into the host tier instead).
        out = torch.empty(size, dtype=torch.uint8, device=blob.device if blob.is_cuda else torch.device("cuda"))
        _require_visible(out)
    _check(lib().kvh_transcode(blob.data_ptr(), dt, l, n_tokens, c, level_in, level_out, out.data_ptr(), out.numel(),
                               status.data_ptr() if status is not None else None, _stream_ptr(stream)), "kvh_transcode")
    return out


def make_tc_items(src_ptrs, dst_ptrs, n_tokens, levels_in, levels_out, device) -> torch.Tensor:
    """Upload an array of kvh_tc_item (argument marshalling; returns a uint8 device tensor)."""
    a = np.zeros(len(src_ptrs), dtype=TC_ITEM)
    a["src"], a["dst"], a["n_tokens"], a["level_in"], a["level_out"] = src_ptrs, dst_ptrs, n_tokens, levels_in, levels_out
    return torch.from_numpy(a.view(np.uint8).copy()).to(device)


def transcode_batch(items: torch.Tensor, n_items: int, max_tokens_per_item: int, dtype, l: int, c: int,
                    status: torch.Tensor | None = None, stream=None) -> None:
    """kvh_transcode_batch: all items in one launch; `items` comes from make_tc_items."""
    _require_cuda(items, status)
    if status is not None and (status.dtype != torch.int32 or status.numel() < n_items):
        raise ValueError("status must be int32 with one entry per item")
    _check(lib().kvh_transcode_batch(items.data_ptr(), n_items, max_tokens_per_item, _dt_code(dtype), l, c,
                                     status.data_ptr() if status is not None else None, _stream_ptr(stream)),
           "kvh_transcode_batch")


def _load_items(host_blobs, n_tokens, levels, dst_token0, k_dst, v_dst, page_tables, status, drops):
    """Marshal the HOST array of kvh_load_item shared by Loader.run and load_static."""
    paged = page_tables is not None
    view, dt = _view(k_dst, v_dst, paged)
    _require_cuda(status)
    n = len(host_blobs)
    for b in host_blobs:
        if b.is_cuda or not b.is_pinned() or b.dtype != torch.uint8:
            raise ValueError("host blobs must be pinned uint8 host tensors")
    if status is not None and (status.dtype != torch.int32 or status.numel() < n):
        raise ValueError("status must be int32 with one entry per item")
    a = np.zeros(n, dtype=LOAD_ITEM)
    a["blob_host"] = [b.data_ptr() for b in host_blobs]
    a["n_tokens"], a["level"], a["dst_token0"] = n_tokens, levels, dst_token0
    if drops is not None:
        for i, d in enumerate(drops):
            if d is not None:
                a["orig_tokens"][i], a["sink"][i], a["window"][i], a["compact"][i] = d[0], d[1], d[2], int(d[3])
    if paged:
        for t in page_tables:
            _require_cuda(t)
            if t.dtype != torch.int32:
                raise ValueError("page tables must be int32")
        a["page_table"] = [t.data_ptr() for t in page_tables]
    return view, dt, a


STATIC_SCRATCH_BYTES = 40 << 20  # KVH_STATIC_SCRATCH_BYTES of include/kvh.h


def load_static(host_blobs, n_tokens, levels, dst_token0, k_dst: torch.Tensor, v_dst: torch.Tensor, page_tables=None,
                block_tokens: int = 16, status: torch.Tensor | None = None, stream=None, drops=None) -> None:
    """kvh_load_static: Loader.run without a loader — one staging slot inside the library, nothing allocated.
    The caller keeps `host_blobs` (and page tables) alive until the stream has been synchronised."""
    view, dt, a = _load_items(host_blobs, n_tokens, levels, dst_token0, k_dst, v_dst, page_tables, status, drops)
    l, c = k_dst.shape[0], k_dst.shape[-1]
    _check(lib().kvh_load_static(a.ctypes.data, len(host_blobs), dt, l, c, ctypes.byref(view), block_tokens,
                                 status.data_ptr() if status is not None else None, _stream_ptr(stream)),
           "kvh_load_static")


class Loader:
    """kvh_loader_*: blobs in pinned host memory -> staging slots in `staging` (uint8 device tensor) -> decode."""

    def __init__(self, staging: torch.Tensor, n_slots: int = 2):
        _require_cuda(staging)
        if staging.dtype != torch.uint8 or not staging.is_contiguous():
            raise ValueError("staging must be a contiguous uint8 device tensor")
        self._staging = staging  # keeps the buffer alive as long as the loader
        self._h = ctypes.c_void_p()
        _check(lib().kvh_loader_create(ctypes.byref(self._h), staging.data_ptr(), staging.numel(), n_slots),
               "kvh_loader_create")
        self._keep = None

    @property
    def slot_bytes(self) -> int:
        return lib().kvh_loader_slot_bytes(self._h)

    def run(self, host_blobs, n_tokens, levels, dst_token0, k_dst: torch.Tensor, v_dst: torch.Tensor,
            page_tables=None, block_tokens: int = 16, status: torch.Tensor | None = None, stream=None,
            drops=None) -> None:
        """kvh_loader_run over pinned uint8 host tensors `host_blobs`; page_tables: int32 device tensors or None;
        drops: per blob None (ordinary) or (orig_tokens, sink, window, compact) for a token-dropped one."""
        view, dt, a = _load_items(host_blobs, n_tokens, levels, dst_token0, k_dst, v_dst, page_tables, status, drops)
        n = len(host_blobs)
        l, c = k_dst.shape[0], k_dst.shape[-1]
        self._keep = (host_blobs, page_tables)  # the copies are asynchronous: keep the sources alive
        _check(lib().kvh_loader_run(self._h, a.ctypes.data, n, dt, l, c, ctypes.byref(view), block_tokens,
                                    status.data_ptr() if status is not None else None, _stream_ptr(stream)),
               "kvh_loader_run")

    def close(self) -> None:
        if self._h:
            h, self._h = self._h, ctypes.c_void_p()
            _check(lib().kvh_loader_destroy(h), "kvh_loader_destroy")
        self._keep = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def policy_utility(freq: float, alpha: float, quality: float, size_bytes: float, bandwidth: float) -> float:
    return lib().kvh_policy_utility(freq, alpha, quality, size_bytes, bandwidth)


def policy_marginal_utility_drop(u_m: float, u_n: float, size_m: float, size_n: float) -> float:
    return lib().kvh_policy_marginal_utility_drop(u_m, u_n, size_m, size_n)


def policy_plan(freqs, sizes, qualities, alpha: float, tiers, min_choices=None):
    """kvh_policy_plan.  sizes / qualities: one sequence per entry (choices by decreasing size); tiers: sequence of
    (bandwidth bytes/s, capacity bytes).  -> (tier per entry or -1, choice per entry or -1, total utility)."""
    n = len(freqs)
    ent = np.zeros(n, dtype=POLICY_ENTRY)
    counts = np.array([len(s) for s in sizes], dtype=np.int64)
    ent["freq"] = freqs
    ent["n_choices"] = counts
    ent["first"] = np.concatenate([[0], np.cumsum(counts)[:-1]]) if n else []
    ent["min_choice"] = 0 if min_choices is None else min_choices
    flat_s = np.ascontiguousarray(np.concatenate([np.asarray(s, dtype=np.float64) for s in sizes]))
    flat_q = np.ascontiguousarray(np.concatenate([np.asarray(q, dtype=np.float64) for q in qualities]))
    if flat_q.size != flat_s.size:
        raise ValueError("sizes and qualities must have the same shape")
    tr = np.zeros(len(tiers), dtype=POLICY_TIER)
    tr["bandwidth"] = [t[0] for t in tiers]
    tr["capacity"] = [t[1] for t in tiers]
    tier_out = np.empty(n, dtype=np.int32)
    choice_out = np.empty(n, dtype=np.int32)
    total = ctypes.c_double()
    _check(lib().kvh_policy_plan(ent.ctypes.data, n, flat_s.ctypes.data, flat_q.ctypes.data, int(flat_s.size),
                                 tr.ctypes.data, len(tiers), alpha, tier_out.ctypes.data, choice_out.ctypes.data,
                                 ctypes.byref(total)), "kvh_policy_plan")
    return tier_out, choice_out, total.value


def stream_probe(dst: torch.Tensor, src: torch.Tensor, n_units: int, reads_per_unit: int, writes_per_unit: int,
                 stream=None) -> None:
    """kvh_stream_probe: traffic generator with a chosen read : write mix (no arithmetic)."""
    _require_cuda(dst, src)
    if src.numel() * src.element_size() < n_units * reads_per_unit * 16 or \
            dst.numel() * dst.element_size() < max(16, n_units * writes_per_unit * 16):
        raise ValueError("buffers too small for this many units")
    _check(lib().kvh_stream_probe(dst.data_ptr(), src.data_ptr(), n_units, reads_per_unit, writes_per_unit,
                                  _stream_ptr(stream)), "kvh_stream_probe")


def time_next_launch(start: "torch.cuda.Event", stop: "torch.cuda.Event") -> None:
    """kvh_time_next_launch: the next encode / decode / transcode kernel launched from this thread records `start`
    at its own start and `stop` at its end (events created with enable_timing=True and recorded once before, so
    that they exist; read them with start.elapsed_time(stop) after synchronising)."""
    hs, he = int(start.cuda_event), int(stop.cuda_event)
    if hs == 0 or he == 0:
        raise ValueError("record each event once before handing it over: torch creates an event at its first record")
    _check(lib().kvh_time_next_launch(hs, he), "kvh_time_next_launch")


def selftest_division(stream=None) -> list:
    """kvh_selftest_division: mismatch counts [r/L at 8, 4, 2 bits, L/r at 8, 4, 2 bits] of the short quotient forms
    against fp32 division over every possible group range; all zeros on a device the codec is exact on."""
    out = torch.zeros(6, dtype=torch.int64, device="cuda")
    _check(lib().kvh_selftest_division(out.data_ptr(), _stream_ptr(stream)), "kvh_selftest_division")
    return out.cpu().tolist()


def copy_probe(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """kvh_copy_probe: plain copy kernel used to calibrate counters and the copy-bandwidth ceiling."""
    _require_cuda(dst, src)
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("destination too small")
    _check(lib().kvh_copy_probe(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(stream)), "kvh_copy_probe")
