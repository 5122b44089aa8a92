"""Seeded synthetic inputs for the FC-layer GEMM tests and benchmark.

This module only *makes data*: bf16 bit patterns in numpy uint16 arrays.  It
holds none of the matrix-multiply arithmetic and imports neither the GPU
library nor the CPU oracle; both sides are handed the same arrays.

The generator is counter based: element number n of stream `seed` is a pure
function of (seed, n), so any slice can be regenerated alone.  SplitMix64
hashes (seed, n) to two 32-bit uniforms, Box-Muller turns them into one
standard normal (fp64), the value is scaled, narrowed to fp32 and rounded to
bf16 with round-to-nearest-even.  Magnitudes below 2^-120 are replaced by zero
so that no input is subnormal in bf16.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_MASK64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        x = (x + np.uint64(0x9E3779B97F4A7C15)) & _MASK64
        z = x
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK64
        return z ^ (z >> np.uint64(31))


def _hash_stream(seed: int, count: int, start: int = 0) -> np.ndarray:
    n = np.arange(start, start + count, dtype=np.uint64)
    s = _splitmix64(np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))[0]
    with np.errstate(over="ignore"):
        return _splitmix64(n ^ s)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern, round to nearest even.  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit pattern -> fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_chunk(seed: int, start: int, cnt: int, sigma: float) -> np.ndarray:
    h = _hash_stream(seed, cnt, start)
    u1 = ((h >> np.uint64(32)).astype(np.float64) + 1.0) / 4294967296.0   # (0, 1]
    u2 = (h & np.uint64(0xFFFFFFFF)).astype(np.float64) / 4294967296.0    # [0, 1)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    v = (z * sigma).astype(np.float32)
    v[np.abs(v) < np.float32(2.0 ** -120)] = 0.0
    return f32_to_bf16_bits(v)


def _workers(workers):
    if workers is None:
        try:
            workers = len(os.sched_getaffinity(0))
        except AttributeError:  # pragma: no cover
            workers = os.cpu_count() or 1
        workers = max(1, min(16, workers))
    return workers


def _in_chunks(total: int, chunk: int, workers, work) -> None:
    """work(start, count) over [0, total) in pieces of `chunk`, on a thread pool."""
    starts = list(range(0, total, chunk))
    workers = _workers(workers)
    if workers == 1 or len(starts) <= 1:
        for st in starts:
            work(st, min(chunk, total - st))
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(lambda st: work(st, min(chunk, total - st)), starts))


def normal_bf16(seed: int, shape, sigma: float = 1.0, chunk: int = 1 << 20, workers: int | None = None) -> np.ndarray:
    """N(0, sigma^2) samples as bf16 bits, shape `shape`, row-major element numbering.

    The result does not depend on `chunk` or `workers` (element n is a function of (seed, n)).
    """
    shape = tuple(int(s) for s in shape)
    total = int(np.prod(shape)) if shape else 1
    out = np.empty(total, dtype=np.uint16)

    def work(start, cnt):
        out[start:start + cnt] = _normal_chunk(seed, start, cnt, sigma)

    _in_chunks(total, chunk, workers, work)
    return out.reshape(shape)


def integer_bf16(seed: int, shape, lo: int = -4, hi: int = 4, chunk: int = 1 << 20, workers: int | None = None) -> np.ndarray:
    """Uniform integers in [lo, hi] (inclusive) as bf16 bits; |values| <= 256 are exact in bf16.

    The result does not depend on `chunk` or `workers` (element n is a function of (seed, n))."""
    if max(abs(lo), abs(hi)) > 256:
        raise ValueError("integers beyond 256 are not all exact in bf16")
    shape = tuple(int(s) for s in shape)
    total = int(np.prod(shape)) if shape else 1
    out = np.empty(total, dtype=np.uint16)
    span = np.uint64(hi - lo + 1)

    def work(start, cnt):
        h = _hash_stream(seed, cnt, start)
        v = ((h >> np.uint64(11)) % span).astype(np.int64) + lo
        out[start:start + cnt] = f32_to_bf16_bits(v.astype(np.float32))

    _in_chunks(total, chunk, workers, work)
    return out.reshape(shape)


def transpose_bits(a: np.ndarray) -> np.ndarray:
    """Exact transpose of a 2-D array of bit patterns (a copy, row-major)."""
    return np.ascontiguousarray(a.T)


# ---------------------------------------------------------------------------
# Workloads (shapes and value distributions of the benchmark configurations).
# Each entry: name, op, M, N, K in the GEMM sense for the op's natural mode.
# ---------------------------------------------------------------------------

BASE_SEED = 2502081450000


def fc_layer_gemms(tokens: int, d_in: int, d_out: int, tag: str):
    """The three GEMMs of one FC layer W[d_in, d_out] on `tokens` tokens, natural modes."""
    return [
        dict(name=f"{tag}.fwd", op="fwd", layout="NN", M=tokens, N=d_out, K=d_in),
        dict(name=f"{tag}.bwd_data", op="bwd_data", layout="NT", M=tokens, N=d_in, K=d_out),
        dict(name=f"{tag}.bwd_weight", op="bwd_weight", layout="TN", M=d_in, N=d_out, K=tokens),
    ]


def workload(name: str):
    """List of GEMMs (dicts) making up one pass of a named workload."""
    if name == "tiny_mlp":            # 1024 tokens, hidden 512
        return fc_layer_gemms(1024, 512, 2048, "fc1") + fc_layer_gemms(1024, 2048, 512, "fc2")
    if name == "gpt5b_layer":         # 2048 tokens, hidden 4096, unsharded layer
        return (fc_layer_gemms(2048, 4096, 12288, "qkv") + fc_layer_gemms(2048, 4096, 4096, "attn_out")
                + fc_layer_gemms(2048, 4096, 16384, "fc1") + fc_layer_gemms(2048, 16384, 4096, "fc2"))
    if name == "gpt80b_shard":        # hidden 8192, 4096 tokens, Gx=4, Gy=2
        return fc_layer_gemms(4096, 2048, 16384, "fc1") + fc_layer_gemms(4096, 16384, 2048, "fc2")
    if name == "gpt320b_skinny":      # hidden 16384, 2048 tokens, Gx=8, Gy=8
        return fc_layer_gemms(2048, 2048, 8192, "fc1") + fc_layer_gemms(2048, 8192, 2048, "fc2")
    raise ValueError(f"unknown workload {name!r}")


def fc_layer_tensors(tokens: int, d_in: int, d_out: int, seed: int):
    """X ~ N(0,1) [tokens,d_in], W ~ N(0,0.02^2) [d_in,d_out], dY ~ N(0,1) [tokens,d_out]."""
    return dict(
        X=normal_bf16(seed + 0, (tokens, d_in), 1.0),
        W=normal_bf16(seed + 1, (d_in, d_out), 0.02),
        dY=normal_bf16(seed + 2, (tokens, d_out), 1.0),
    )


def operands_for(op: str, layout: str, t: dict):
    """First and second operand of `op`, stored the way `layout` wants them.

    t holds the cached buffers X[tokens,in], W[in,out], dY[tokens,out].  In the natural
    mode of each op (fwd NN: X, W; bwd_data NT: dY, W; bwd_weight TN: X, dY) the cached
    buffers are returned untouched; any other mode gets an exact transposed copy.
    """
    if op == "fwd":            # C[T,out] = X . W      first is [M,K], second is [K,N]
        first, first_is_mk, second, second_is_kn = t["X"], True, t["W"], True
    elif op == "bwd_data":     # C[T,in] = dY . W^T    first is [M,K], second is [N,K]
        first, first_is_mk, second, second_is_kn = t["dY"], True, t["W"], False
    elif op == "bwd_weight":   # C[in,out] = X^T . dY  first is [K,M], second is [K,N]
        first, first_is_mk, second, second_is_kn = t["X"], False, t["dY"], True
    else:
        raise ValueError(op)
    if layout not in ("NN", "NT", "TN"):
        raise ValueError(layout)
    want_first_mk = layout != "TN"
    want_second_kn = layout != "NT"
    a = first if first_is_mk == want_first_mk else transpose_bits(first)
    b = second if second_is_kn == want_second_kn else transpose_bits(second)
    return a, b
