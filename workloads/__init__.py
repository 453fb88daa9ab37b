"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and shapes them; it contains none of
the quantiser's arithmetic (no rotation construction, no codebook, no
quantisation).  Both the CPU oracle's tests and the GPU library's tests take
their inputs from here, so that the two sides see the same arrays.

All draws use numpy's default_rng (PCG64) seeded with an explicit integer
list, on the host.  Large row sets are produced in chunks of CHUNK rows with
seed [seed, stream, chunk_index], so any chunk can be regenerated alone.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

CHUNK = 65536


@dataclass(frozen=True)
class Config:
    name: str
    kind: str  # "mse" or "prod"
    bits: int  # total bit-width b; prod uses bits-1 for the MSE stage
    d: int
    n: int  # vectors per group
    n_groups: int  # KV heads (1 for ANN)
    nq: int  # queries in total
    q_per_group: int
    in_dtype: str  # "f32" or "bf16"
    unit_norm: bool
    topk: int
    seed_x: int
    seed_q: int
    seed_pi: int
    seed_s: int
    d_hi: int = 0  # > 0: that many outlier channels form a second instance with bits + 1 (Sec. 4.3)

    @property
    def bits_mse(self) -> int:
        return self.bits if self.kind == "mse" else self.bits - 1


CONFIGS = {
    "C1": Config("C1", "mse", 2, 128, 4096, 1, 64, 64, "f32", True, 0, 0, 1, 100, 200),
    "C2": Config("C2", "prod", 3, 128, 16384, 8, 32, 4, "bf16", False, 0, 2, 3, 100, 200),
    "C3": Config("C3", "prod", 3, 128, 65536, 8, 32, 4, "bf16", False, 0, 2, 3, 100, 200),
    "C3b4": Config("C3b4", "prod", 4, 128, 65536, 8, 32, 4, "bf16", False, 0, 2, 3, 100, 200),
    # 2.5 bits per channel: 64 outlier channels at b = 3, 64 at b = 2 (shapes of C2 / C3)
    "C2m": Config("C2m", "prod", 2, 128, 16384, 8, 32, 4, "bf16", False, 0, 2, 3, 100, 200, 64),
    "C3m": Config("C3m", "prod", 2, 128, 65536, 8, 32, 4, "bf16", False, 0, 2, 3, 100, 200, 64),
    # 3.5 bits per channel: 64 outlier channels at b = 4, 64 at b = 3
    "C2h": Config("C2h", "prod", 3, 128, 16384, 8, 32, 4, "bf16", False, 0, 2, 3, 100, 200, 64),
    "C3h": Config("C3h", "prod", 3, 128, 65536, 8, 32, 4, "bf16", False, 0, 2, 3, 100, 200, 64),
    "C4": Config("C4", "mse", 4, 1536, 1000000, 1, 1000, 1000, "f32", True, 10, 4, 5, 101, 201),
    "C5": Config("C5", "prod", 2, 3072, 1000000, 1, 1000, 1000, "f32", True, 10, 6, 7, 102, 202),
    # the same two indexes searched online: four queries at a time instead of a batch of 1000
    "C4q": Config("C4q", "mse", 4, 1536, 1000000, 1, 4, 4, "f32", True, 10, 4, 5, 101, 201),
    "C5q": Config("C5q", "prod", 2, 3072, 1000000, 1, 4, 4, "f32", True, 10, 6, 7, 102, 202),
}


def gaussian_matrix(d: int, seed: int) -> np.ndarray:
    """d x d i.i.d. N(0,1), float64: raw material for the rotation (its QR is
    taken by whoever uses it) and, as is, the sketch matrix S."""
    return np.random.default_rng([seed, 0]).standard_normal((d, d))


def sketch_matrix(d: int, seed: int) -> np.ndarray:
    """S: d x d i.i.d. N(0,1), rounded to float32 once."""
    return gaussian_matrix(d, seed).astype(np.float32)


def unit_gaussian_rows(n: int, d: int, seed: int) -> np.ndarray:
    """n rows i.i.d. N(0, I_d), each scaled to unit L2 norm; float32."""
    x = np.random.default_rng([seed, 1]).standard_normal((n, d))
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    return x.astype(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of float32 to bfloat16 bit patterns
    (uint16).  Inputs here are finite."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def kv_outlier_channels(n_heads: int, d: int, seed: int, n_out: int = 4) -> np.ndarray:
    """For each head, n_out fixed channel numbers taken from a seeded
    permutation."""
    rng = np.random.default_rng([seed, 2])
    return np.stack([rng.permutation(d)[:n_out] for _ in range(n_heads)])


def kv_hi_channels(n_heads: int, d: int, seed: int, d_hi: int) -> np.ndarray:
    """The channel set given more bits when the key cache is split into two
    instances: every head's outlier channels, filled up to d_hi with the
    lowest-numbered remaining channels.  Ascending."""
    out = np.unique(kv_outlier_channels(n_heads, d, seed))[:d_hi]
    rest = np.setdiff1d(np.arange(d), out)[: d_hi - out.size]
    return np.sort(np.concatenate([out, rest]))


def kv_keys_chunk(head: int, start: int, rows: int, d: int, seed: int,
                  outliers: np.ndarray) -> np.ndarray:
    """rows keys of one head, N(0,1) per channel with that head's outlier
    channels multiplied by 20; returned as bfloat16 bit patterns [rows, d].
    start must be a multiple of CHUNK or rows must stay inside one chunk."""
    out = np.empty((rows, d), dtype=np.uint16)
    done = 0
    while done < rows:
        ci, off = divmod(start + done, CHUNK)
        take = min(rows - done, CHUNK - off)
        rng = np.random.default_rng([seed, 3, head, ci])
        blk = rng.standard_normal((CHUNK, d), dtype=np.float32)[off:off + take]
        blk[:, outliers[head]] *= 20.0
        out[done:done + take] = f32_to_bf16_bits(blk)
        done += take
    return out


def kv_keys(n_heads: int, n_tokens: int, d: int, seed: int) -> np.ndarray:
    """[n_heads, n_tokens, d] bfloat16 bit patterns (uint16)."""
    outl = kv_outlier_channels(n_heads, d, seed)
    return np.stack([kv_keys_chunk(h, 0, n_tokens, d, seed, outl) for h in range(n_heads)])


def mixture_centers(d: int, seed: int, n_centers: int = 256) -> np.ndarray:
    return np.random.default_rng([seed, 4]).standard_normal((n_centers, d)).astype(np.float32)


def mixture_chunk(chunk_index: int, rows: int, d: int, seed: int, centers: np.ndarray,
                  sigma: float = 0.3) -> np.ndarray:
    """rows <= CHUNK rows of the Gaussian mixture: a uniformly chosen centre
    plus sigma * N(0, I), scaled to unit norm; float32."""
    rng = np.random.default_rng([seed, 5, chunk_index])
    k = rng.integers(0, centers.shape[0], size=CHUNK)[:rows]
    x = rng.standard_normal((rows, d), dtype=np.float32)
    x *= np.float32(sigma)
    x += centers[k]
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    return x


def mixture_rows(n: int, d: int, seed: int, centers_seed: int, threads: int = 8):
    """Generator of (start_row, float32 block) over all n rows, chunks made
    by a small thread pool (numpy releases the GIL while filling)."""
    centers = mixture_centers(d, centers_seed)
    n_chunks = (n + CHUNK - 1) // CHUNK

    def make(ci):
        rows = min(CHUNK, n - ci * CHUNK)
        return ci * CHUNK, mixture_chunk(ci, rows, d, seed, centers)

    with ThreadPoolExecutor(max_workers=threads) as pool:
        pending = []
        for ci in range(n_chunks):
            pending.append(pool.submit(make, ci))
            if len(pending) >= threads:
                yield pending.pop(0).result()
        for f in pending:
            yield f.result()


def mixture_all(n: int, d: int, seed: int, centers_seed: int) -> np.ndarray:
    out = np.empty((n, d), dtype=np.float32)
    for start, blk in mixture_rows(n, d, seed, centers_seed):
        out[start:start + blk.shape[0]] = blk
    return out


def gaussian_queries(nq: int, d: int, seed: int, unit: bool) -> np.ndarray:
    q = np.random.default_rng([seed, 6]).standard_normal((nq, d))
    if unit:
        q /= np.linalg.norm(q, axis=1, keepdims=True)
    return q.astype(np.float32)
