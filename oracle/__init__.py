"""CPU oracle of the KV-cache level codec — TEST INFRASTRUCTURE ONLY.

`kvh_ref.c` is the definition written out in plain scalar C; this package compiles it with gcc
and exposes it through ctypes on numpy arrays of raw 16-bit patterns.  Only the tests, the
smoke check and the benchmark's cpu_baseline leg may import it; the HIP package never does,
and this package never imports the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvh_ref.c")
_LIB = os.path.join(_HERE, "libkvh_ref.so")

F16, BF16 = 0, 1
OK = 0
E_ARG, E_LEVEL, E_SHAPE, E_SIZE, E_ALIGN, E_HEADER, E_NONFINITE = -1, -2, -3, -4, -5, -7, -8

# -ffp-contract=off: no fused multiply-add except where the source says fmaf.
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    """Compile kvh_ref.c into libkvh_ref.so next to it (gcc, a second or two)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        u16p, u8p, i32p = ctypes.POINTER(ctypes.c_uint16), ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_int32)
        L.kvh_ref_t16_to_f32.restype = ctypes.c_float
        L.kvh_ref_t16_to_f32.argtypes = [ctypes.c_uint16, ctypes.c_int]
        L.kvh_ref_f32_to_t16.restype = ctypes.c_uint16
        L.kvh_ref_f32_to_t16.argtypes = [ctypes.c_float, ctypes.c_int]
        L.kvh_ref_num_levels.restype = ctypes.c_int
        L.kvh_ref_level_bits.restype = ctypes.c_int
        L.kvh_ref_level_bits.argtypes = [ctypes.c_int]
        L.kvh_ref_blob_size.restype = ctypes.c_size_t
        L.kvh_ref_blob_size.argtypes = [ctypes.c_int] * 4
        L.kvh_ref_group_params.restype = ctypes.c_int
        L.kvh_ref_group_params.argtypes = [ctypes.c_uint16, ctypes.c_uint16, ctypes.c_int, ctypes.c_int,
                                           ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float)]
        L.kvh_ref_quantise.restype = ctypes.c_int
        L.kvh_ref_quantise.argtypes = [ctypes.c_uint16, ctypes.c_uint16, ctypes.c_float, ctypes.c_int, ctypes.c_int]
        L.kvh_ref_dequantise.restype = ctypes.c_uint16
        L.kvh_ref_dequantise.argtypes = [ctypes.c_int, ctypes.c_uint16, ctypes.c_uint16, ctypes.c_int, ctypes.c_int]
        L.kvh_ref_encode.restype = ctypes.c_int
        L.kvh_ref_encode.argtypes = [u16p, u16p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int, ctypes.c_int, ctypes.c_int, u8p, ctypes.c_size_t]
        L.kvh_ref_decode.restype = ctypes.c_int
        L.kvh_ref_decode.argtypes = [u8p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int, u16p, u16p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                     i32p, ctypes.c_int]
        L.kvh_ref_section_offsets.restype = ctypes.c_int
        L.kvh_ref_section_offsets.argtypes = [ctypes.c_int] * 5 + [ctypes.POINTER(ctypes.c_uint64)]
        L.kvh_ref_t16_to_f32_array.restype = None
        L.kvh_ref_t16_to_f32_array.argtypes = [u16p, ctypes.POINTER(ctypes.c_float), ctypes.c_size_t, ctypes.c_int]
        L.kvh_ref_f32_to_t16_array.restype = None
        L.kvh_ref_f32_to_t16_array.argtypes = [ctypes.POINTER(ctypes.c_float), u16p, ctypes.c_size_t, ctypes.c_int]
        L.kvh_ref_kept_tokens.restype = ctypes.c_int
        L.kvh_ref_kept_tokens.argtypes = [ctypes.c_int] * 3
        L.kvh_ref_encode_kept.restype = ctypes.c_int
        L.kvh_ref_encode_kept.argtypes = [u16p, u16p, ctypes.c_int64, ctypes.c_int64] + [ctypes.c_int] * 7 + [u8p, ctypes.c_size_t]
        L.kvh_ref_decode_kept.restype = ctypes.c_int
        L.kvh_ref_decode_kept.argtypes = [u8p, ctypes.c_size_t] + [ctypes.c_int] * 7 + [u16p, u16p, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_int64, ctypes.c_int, i32p, ctypes.c_int]
        L.kvh_ref_transcode.restype = ctypes.c_int
        L.kvh_ref_transcode.argtypes = [u8p, ctypes.c_size_t] + [ctypes.c_int] * 6 + [u8p, ctypes.c_size_t]
        _lib = L
    return _lib


def _u16p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _u8p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def _check_view(a: np.ndarray, l: int, n: int, c: int):
    if a.dtype != np.uint16 or a.ndim != 3 or a.shape[0] != l or a.shape[1] < n or a.shape[2] != c:
        raise ValueError("expected uint16 [l][>=n][c], got %s %s" % (a.dtype, a.shape))
    if a.strides[2] != 2 or a.strides[0] % 2 or a.strides[1] % 2:
        raise ValueError("channel stride must be 1 element")
    return a.strides[0] // 2, a.strides[1] // 2


def level_bits(level: int) -> int:
    return lib().kvh_ref_level_bits(level)


def num_levels() -> int:
    return lib().kvh_ref_num_levels()


def blob_size(l: int, n: int, c: int, level: int) -> int:
    return lib().kvh_ref_blob_size(l, n, c, level)


def t16_to_f32(bits: int, dt: int) -> float:
    return lib().kvh_ref_t16_to_f32(bits, dt)


def f32_to_t16(x: float, dt: int) -> int:
    return lib().kvh_ref_f32_to_t16(x, dt)


def t16_to_f32_array(bits: np.ndarray, dt: int) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float32)
    lib().kvh_ref_t16_to_f32_array(_u16p(bits), out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), bits.size, dt)
    return out


def f32_to_t16_array(x: np.ndarray, dt: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().kvh_ref_f32_to_t16_array(x.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), _u16p(out), x.size, dt)
    return out


def group_params(mn_bits: int, mx_bits: int, dt: int, bits: int):
    """-> (scale, inv, degenerate) as numpy float32 scalars and a bool."""
    s, i = ctypes.c_float(), ctypes.c_float()
    deg = lib().kvh_ref_group_params(mn_bits, mx_bits, dt, bits, ctypes.byref(s), ctypes.byref(i))
    return np.float32(s.value), np.float32(i.value), bool(deg)


def quantise(x_bits: int, mn_bits: int, inv, dt: int, bits: int) -> int:
    return lib().kvh_ref_quantise(x_bits, mn_bits, float(inv), dt, bits)


def dequantise(q: int, mn_bits: int, mx_bits: int, dt: int, bits: int) -> int:
    return lib().kvh_ref_dequantise(q, mn_bits, mx_bits, dt, bits)


def encode(k: np.ndarray, v: np.ndarray, dt: int, level: int, n: int | None = None, strict: bool = True) -> np.ndarray:
    """Encode uint16 [l][n][c] K and V (same strides) into one blob (uint8 array)."""
    l, n_all, c = k.shape
    n = n_all if n is None else n
    ls, ts = _check_view(k, l, n, c)
    if _check_view(v, l, n, c) != (ls, ts):
        raise ValueError("K and V must share strides")
    size = blob_size(l, n, c, level)
    if size == 0:
        raise ValueError("bad level or shape (l=%d n=%d c=%d level=%d)" % (l, n, c, level))
    blob = np.empty(size, dtype=np.uint8)
    rc = lib().kvh_ref_encode(_u16p(k), _u16p(v), ls, ts, dt, l, n, c, level, _u8p(blob), size)
    if rc != OK and (strict or rc != E_NONFINITE):
        raise RuntimeError("kvh_ref_encode failed: %d" % rc)
    return blob


def encode_rc(k, v, dt, level, blob: np.ndarray, n=None) -> int:
    """Raw status-returning form (for error-path tests)."""
    l, n_all, c = k.shape
    n = n_all if n is None else n
    ls, ts = k.strides[0] // 2, k.strides[1] // 2
    return lib().kvh_ref_encode(_u16p(k), _u16p(v), ls, ts, dt, l, n, c, level, _u8p(blob), blob.size)


def decode_into(blob: np.ndarray, dt: int, l: int, n: int, c: int, level: int, kdst: np.ndarray, vdst: np.ndarray,
                dst_token0: int = 0, page_table: np.ndarray | None = None, block_tokens: int = 16) -> int:
    """Decode into caller-provided uint16 destinations; returns the status code.

    Contiguous: kdst/vdst are [l][tokens][c].  Paged: [l][P][block_tokens][c] plus an int32 table.
    """
    if kdst.dtype != np.uint16 or vdst.dtype != np.uint16 or kdst.strides != vdst.strides:
        raise ValueError("destinations must be uint16 with equal strides")
    if page_table is None:
        ls, ts = kdst.strides[0] // 2, kdst.strides[1] // 2
        pt = None
    else:
        if kdst.ndim != 4 or kdst.shape[2] != block_tokens:
            raise ValueError("paged destination must be [l][P][block_tokens][c]")
        ls, ts = kdst.strides[0] // 2, kdst.strides[2] // 2
        if kdst.strides[1] != kdst.strides[2] * block_tokens:
            raise ValueError("blocks must be densely packed")
        page_table = np.ascontiguousarray(page_table, dtype=np.int32)
        pt = page_table.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    return lib().kvh_ref_decode(_u8p(blob), blob.size, dt, l, n, c, level, _u16p(kdst), _u16p(vdst), ls, ts,
                                dst_token0, pt, block_tokens)


def decode(blob: np.ndarray, dt: int, l: int, n: int, c: int, level: int):
    """Decode a blob into fresh contiguous uint16 [l][n][c] K and V."""
    k = np.zeros((l, n, c), dtype=np.uint16)
    v = np.zeros((l, n, c), dtype=np.uint16)
    rc = decode_into(blob, dt, l, n, c, level, k, v)
    if rc != OK:
        raise RuntimeError("kvh_ref_decode failed: %d" % rc)
    return k, v


def section_offsets(l: int, n: int, c: int, level: int, lam: int):
    """-> dict of byte offsets of layer lam's kmeta/kcodes/vmeta/vcodes and the packed row size."""
    out = (ctypes.c_uint64 * 5)()
    rc = lib().kvh_ref_section_offsets(l, n, c, level, lam, out)
    if rc != OK:
        raise ValueError("bad arguments: %d" % rc)
    return {"kmeta": out[0], "kcodes": out[1], "vmeta": out[2], "vcodes": out[3], "row_bytes": out[4]}


def kept_tokens(N: int, sink: int, window: int) -> int:
    return lib().kvh_ref_kept_tokens(N, sink, window)


def encode_kept(k: np.ndarray, v: np.ndarray, dt: int, sink: int, window: int, level: int) -> np.ndarray:
    """Token dropping: keep the first `sink` and last `window` tokens of uint16 [l][N][c] K/V, encode them."""
    l, N, c = k.shape
    ls, ts = _check_view(k, l, N, c)
    if _check_view(v, l, N, c) != (ls, ts):
        raise ValueError("K and V must share strides")
    n = kept_tokens(N, sink, window)
    size = blob_size(l, n, c, level) if n > 0 else 0
    if size == 0:
        raise ValueError("bad arguments")
    blob = np.empty(size, dtype=np.uint8)
    rc = lib().kvh_ref_encode_kept(_u16p(k), _u16p(v), ls, ts, dt, l, N, c, sink, window, level, _u8p(blob), size)
    if rc != OK:
        raise RuntimeError("kvh_ref_encode_kept failed: %d" % rc)
    return blob


def decode_kept_into(blob: np.ndarray, dt: int, l: int, N: int, c: int, sink: int, window: int, level: int,
                     kdst: np.ndarray, vdst: np.ndarray, dst_token0: int = 0, compact: bool = False,
                     page_table: np.ndarray | None = None, block_tokens: int = 16) -> int:
    """Decode a token-dropped blob into caller-provided destinations (contiguous or paged); returns the status."""
    if kdst.dtype != np.uint16 or vdst.dtype != np.uint16 or kdst.strides != vdst.strides:
        raise ValueError("destinations must be uint16 with equal strides")
    if page_table is None:
        ls, ts, pt = kdst.strides[0] // 2, kdst.strides[1] // 2, None
    else:
        ls, ts = kdst.strides[0] // 2, kdst.strides[2] // 2
        page_table = np.ascontiguousarray(page_table, dtype=np.int32)
        pt = page_table.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    return lib().kvh_ref_decode_kept(_u8p(blob), blob.size, dt, l, N, c, sink, window, level, _u16p(kdst), _u16p(vdst),
                                     ls, ts, dst_token0, int(compact), pt, block_tokens)


def transcode_rc(blob: np.ndarray, dt: int, l: int, n: int, c: int, level_in: int, level_out: int, out: np.ndarray) -> int:
    """Raw status-returning form of transcode."""
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    return lib().kvh_ref_transcode(_u8p(blob), blob.size, dt, l, n, c, level_in, level_out, _u8p(out), out.size)


def transcode(blob: np.ndarray, dt: int, l: int, n: int, c: int, level_in: int, level_out: int) -> np.ndarray:
    """Re-compress a blob of n stored tokens from level_in to level_out: decode, then encode."""
    size = blob_size(l, n, c, level_out)
    if size == 0:
        raise ValueError("bad level or shape")
    out = np.empty(size, dtype=np.uint8)
    rc = transcode_rc(blob, dt, l, n, c, level_in, level_out, out)
    if rc != OK:
        raise RuntimeError("kvh_ref_transcode failed: %d" % rc)
    return out
