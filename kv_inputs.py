"""Seeded synthetic KV-cache inputs shared by the tests, the smoke check and the benchmark.

This module only *generates inputs*: random KV tensors shaped like the paper's workloads
(Llama-3.1-8B-Instruct KV on long contexts, Preliminary Results / Evaluation setup), request
length mixes, per-chunk level draws and page tables.  It holds none of the codec's arithmetic
(no statistics, no quantisation, no packing, no blob layout) and is imported by both the CPU
oracle's tests and the HIP path's tests, which otherwise share nothing.

Value recipe (the paper's contexts and model weights are not available, so these stand in for
them by shape and by the well-known structure of KV tensors: a wide spread of per-channel
scales and a few outlier channels):

    for every (K|V, layer):   sigma_ch = exp(z_ch), z_ch ~ N(0, 1)
                              ceil(0.01 * c) outlier channels (drawn without replacement)
                              get sigma_ch *= 10
    x[t, ch] = sigma_ch * N(0, 1)            (fp32, then ONE round-to-nearest-even cast to fp16/bf16)

Optional rotary-like drift (K only):  x[t, ch] += 2 * sigma_ch * sin(theta_ch * t + phi_ch),
theta_ch = 10000 ** (-2 * floor((ch mod 128) / 2) / 128),  phi_ch ~ U[0, 2*pi).

Tensors are returned as raw 16-bit patterns (numpy uint16 / torch int16 views) so that neither
consumer depends on how the other interprets a float.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

F16 = 0   # IEEE binary16
BF16 = 1  # bfloat16

DTYPE_NAMES = {F16: "fp16", BF16: "bf16"}


def _cast_to_bits(x32: np.ndarray, dtype: int) -> np.ndarray:
    """fp32 ndarray -> uint16 bit patterns of the 16-bit type, one RNE rounding."""
    if dtype == F16:
        return x32.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        import torch

        t = torch.from_numpy(np.ascontiguousarray(x32)).to(torch.bfloat16)
        return t.view(torch.int16).numpy().view(np.uint16)
    raise ValueError("dtype must be F16 (0) or BF16 (1)")


def bits_to_f64(bits: np.ndarray, dtype: int) -> np.ndarray:
    """uint16 bit patterns -> float64 values (exact); for error reports, not for the codec."""
    bits = np.array(bits, dtype=np.uint16)  # a contiguous copy that keeps the shape (0-d included)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError("dtype must be F16 (0) or BF16 (1)")


def _channel_sigma(rng: np.random.Generator, c: int) -> np.ndarray:
    sigma = np.exp(rng.standard_normal(c)).astype(np.float32)
    n_out = int(math.ceil(0.01 * c))
    out = rng.choice(c, size=n_out, replace=False)
    sigma[out] *= 10.0
    return sigma


def _drift(rng: np.random.Generator, sigma: np.ndarray, n: int, c: int, token0: int) -> np.ndarray:
    ch = np.arange(c)
    theta = 10000.0 ** (-2.0 * np.floor((ch % 128) / 2.0) / 128.0)
    phi = rng.uniform(0.0, 2.0 * math.pi, size=c)
    t = np.arange(token0, token0 + n, dtype=np.float64)[:, None]
    return (2.0 * sigma[None, :].astype(np.float64) * np.sin(theta[None, :] * t + phi[None, :])).astype(np.float32)


def make_kv(l: int, n: int, c: int, dtype: int, seed: int, drift: bool = False):
    """Host generator.  Returns (k_bits, v_bits), each uint16 [l][n][c], C-contiguous."""
    rng = np.random.default_rng(seed)
    k = np.empty((l, n, c), dtype=np.uint16)
    v = np.empty((l, n, c), dtype=np.uint16)
    for which, dst in ((0, k), (1, v)):
        for lam in range(l):
            sigma = _channel_sigma(rng, c)
            x = rng.standard_normal((n, c), dtype=np.float32) * sigma[None, :]
            if drift and which == 0:
                x = x + _drift(rng, sigma, n, c, 0)
            dst[lam] = _cast_to_bits(x, dtype)
    return k, v


def make_kv_device(l: int, n: int, c: int, dtype: int, seed: int, device="cuda", drift: bool = False):
    """Device generator for the configurations too large to build on the host.

    Returns one torch tensor [2][l][n][c] of the 16-bit dtype on `device` (index 0 = K, 1 = V).
    Parity tests copy the bytes they check back to the host, so the two generators need not
    agree with each other.
    """
    import torch

    tdt = torch.float16 if dtype == F16 else torch.bfloat16
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    kv = torch.empty((2, l, n, c), dtype=tdt, device=device)
    n_out = int(math.ceil(0.01 * c))
    ch = torch.arange(c, device=device)
    theta = 10000.0 ** (-2.0 * torch.floor((ch % 128) / 2.0) / 128.0)
    step = 8192
    for which in range(2):
        for lam in range(l):
            sigma = torch.exp(torch.randn(c, generator=g, device=device))
            out = torch.randperm(c, generator=g, device=device)[:n_out]
            sigma[out] *= 10.0
            phi = torch.rand(c, generator=g, device=device) * (2.0 * math.pi)
            for t0 in range(0, n, step):
                m = min(step, n - t0)
                x = torch.randn((m, c), generator=g, device=device) * sigma[None, :]
                if drift and which == 0:
                    t = torch.arange(t0, t0 + m, device=device, dtype=torch.float32)[:, None]
                    x = x + 2.0 * sigma[None, :] * torch.sin(theta[None, :] * t + phi[None, :])
                kv[which, lam, t0:t0 + m] = x.to(tdt)
    return kv


# --------------------------------------------------------------------------------------------
# The five workload configurations (shape, dtype, chunking, seed).
# --------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class KVConfig:
    name: str
    l: int
    n: int
    c: int
    dtype: int
    chunk: int
    seed: int
    drift: bool = False


CONFIGS = {
    "tiny": KVConfig("tiny_4x1024x1024_fp16", 4, 1024, 1024, F16, 256, 0),
    "llama3_8b_8k": KVConfig("llama3_8b_32x8192x1024_bf16", 32, 8192, 1024, BF16, 256, 1),
    "llama3_70b_32k": KVConfig("llama3_70b_80x32768x1024_bf16", 80, 32768, 1024, BF16, 512, 2, drift=True),
    "long_7b_128k": KVConfig("long7b_32x131072x1024_fp16", 32, 131072, 1024, F16, 256, 3),
}


def mixed_batch_lengths(n_requests: int = 64, mean: float = 4096.0, sigma: float = 0.8,
                        lo: int = 256, hi: int = 32768, seed: int = 4) -> np.ndarray:
    """Request lengths: lognormal with ARITHMETIC mean `mean` (mu = ln(mean) - sigma^2/2), clipped."""
    rng = np.random.default_rng(seed)
    mu = math.log(mean) - 0.5 * sigma * sigma
    ln = np.exp(rng.normal(mu, sigma, size=n_requests))
    return np.clip(np.rint(ln), lo, hi).astype(np.int64)


def mixed_batch_plan(lengths: np.ndarray, chunk: int = 256, block_tokens: int = 16,
                     n_levels: int = 3, seed: int = 4):
    """Per-request chunking, a uniformly random level per chunk and one random page permutation.

    Returns (chunks, page_tables, n_pages) where chunks is a list of
    (request, token0, n_tokens, level) and page_tables[r] is the int32 slice of physical block
    ids owned by request r (ceil(len/block_tokens) entries, all distinct across requests).
    """
    rng = np.random.default_rng(seed + 1000)
    pages_per_req = [int(-(-int(n) // block_tokens)) for n in lengths]
    n_pages = int(sum(pages_per_req))
    perm = rng.permutation(n_pages).astype(np.int32)
    page_tables, p0 = [], 0
    for p in pages_per_req:
        page_tables.append(perm[p0:p0 + p].copy())
        p0 += p
    chunks = []
    for r, n in enumerate(lengths):
        n = int(n)
        for t0 in range(0, n, chunk):
            chunks.append((r, t0, min(chunk, n - t0), int(rng.integers(0, n_levels))))
    return chunks, page_tables, n_pages
