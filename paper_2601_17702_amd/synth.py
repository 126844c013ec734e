"""Seeded synthetic input streams (keys, queries, SAE weights) for the five workloads.

This module only draws random numbers and rounds them to the storage dtype.  It holds
none of the method's arithmetic (no encoder, no Top-k, no index, no scoring) and is the
only code shared between the CPU oracle's tests and the GPU path's tests/bench.

Every tensor is generated per (workload seed, tensor kind, head, chunk) from a
counter-based Philox stream, so any head or chunk can be regenerated on its own and the
bytes do not depend on generation order or thread count.

Workload shapes stand in for the paper's models (Sec. 4.1 and App. A: Llama-3.1-8B,
Qwen2-7B; d_head = 128, GQA 32:8 and 28:4; App. B.3 Table: chunk 2048, expansion 128).
No dataset, model weight or benchmark item is reproduced: all values are random.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from concurrent.futures import ThreadPoolExecutor
import numpy as np

# tensor kinds (second half of the Philox key)
_T_PARAMS, _T_KEYS, _T_WENC, _T_BENC, _T_QUERY, _T_PERM = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    kv_heads: int
    L: int            # context tokens
    T: int            # streaming chunk size (tokens per encode call)
    d_head: int
    n_feat: int
    k: int
    dtype: str        # "bf16" | "fp32": storage dtype of K/Q and W_enc
    nq: int           # query vectors per KV head (query tokens x Q heads in the GQA group)
    span_len: int
    top_b: int
    seed: int
    recipe: str       # "iso" | "lowrank" | "zipf"
    b_std: float = 0.01

    @property
    def n_heads(self) -> int:
        return self.layers * self.kv_heads

    @property
    def n_chunks(self) -> int:
        return (self.L + self.T - 1) // self.T

    @property
    def token_heads(self) -> int:
        return self.L * self.n_heads


WORKLOADS = {
    # 1 layer x 1 KV head, one 2048-token chunk, fp32, channel-scaled Gaussian keys
    "c1_tiny": Workload("c1_tiny", 1, 1, 2048, 2048, 128, 4096, 16, "fp32", 8, 32, 8, 0, "iso"),
    # Llama-3-8B shape: 32 layers x 8 KV heads, 32K tokens, 64 query tokens x 4 Q heads per KV head
    "c2_llama8b": Workload("c2_llama8b", 32, 8, 32768, 2048, 128, 16384, 32, "bf16", 256, 64, 16, 1, "lowrank"),
    # long stream with Zipf-skewed feature popularity
    "c3_long": Workload("c3_long", 32, 8, 131072, 4096, 128, 16384, 32, "bf16", 256, 64, 16, 2, "zipf"),
    # Qwen2.5-7B shape: 28 layers x 4 KV heads, 128 query tokens x 7 Q heads per KV head
    "c4_qwen7b": Workload("c4_qwen7b", 28, 4, 65536, 2048, 128, 32768, 64, "bf16", 896, 32, 32, 3, "lowrank"),
    # the paper's own SAE setting (App. B.3: expansion 128 -> 16384 features for d_head 128, k = 128) on a
    # Mistral-7B-like shape with four target layers (App. A, layer table): 4 layers x 8 KV heads, chunk 2048,
    # N = 40 centres; 64 query tokens x 4 Q heads per KV head
    "c6_paper_sae": Workload("c6_paper_sae", 4, 8, 32768, 2048, 128, 16384, 128, "bf16", 256, 48, 40, 5, "lowrank"),
    # wide SAE stress
    "c5_wide": Workload("c5_wide", 1, 8, 1048576, 8192, 128, 65536, 64, "bf16", 256, 128, 64, 4, "lowrank", 0.05),
}

# Zipf recipe constants: b_enc[f] = ZIPF_BETA * (-1.1 * ln rank(f)) + ZIPF_C, fixed so that the
# most popular features of c3_long are active in >= 1e5 of the 131072 tokens of a head (measured with the
# oracle on 4096 tokens of head 0: the four most frequent features are in 92 %, 87 %, 86 % and 83 % of the rows,
# about 1100 of the 16384 features are used at all, the 32 most frequent ones hold half of the postings).
ZIPF_BETA = 1.0
ZIPF_C = 9.0


def shrink(w: Workload, **kw) -> Workload:
    """A smaller instance of the same recipe (used by parity tests and samples)."""
    return replace(w, **kw)


def _rng(seed: int, kind: int, head: int, chunk: int = 0) -> np.random.Generator:
    key = np.array([(np.uint64(seed) << np.uint64(32)) | np.uint64(kind),
                    (np.uint64(head) << np.uint64(32)) | np.uint64(chunk)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


# ---------------------------------------------------------------- storage dtypes
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array -> storage array: float32 for "fp32", uint16 bf16 bit patterns for "bf16"."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a if dtype == "fp32" else f32_to_bf16_bits(a)


def storage_to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored values to float64."""
    return (a if dtype == "fp32" else bf16_bits_to_f32(a)).astype(np.float64)


# ---------------------------------------------------------------- per-head distribution parameters
def _head_params(w: Workload, head: int) -> dict:
    g = _rng(w.seed, _T_PARAMS, head)
    d = w.d_head
    p = {"s": np.exp(0.5 * g.standard_normal(d)).astype(np.float32)}  # per-channel variance, log-normal(0, 0.5)
    if w.recipe != "iso":
        p["means"] = g.standard_normal((32, 16)).astype(np.float32)       # 32-component mixture in R^16
        p["A"] = (g.standard_normal((16, d)) / 4.0).astype(np.float32)    # rank-16 map, entries N(0, 1/16)
        p["outliers"] = g.choice(d, size=2, replace=False)                 # 2 outlier channels, x8
    return p


def _draw_vectors(w: Workload, head: int, g: np.random.Generator, n: int) -> np.ndarray:
    p = _head_params(w, head)
    d = w.d_head
    if w.recipe == "iso":
        # K[t, c] = sqrt(s[c]) * N(0, 1)
        return (g.standard_normal((n, d), dtype=np.float32) * np.sqrt(p["s"])[None, :]).astype(np.float32)
    comp = g.integers(0, 32, size=n)
    u = p["means"][comp] + 0.5 * g.standard_normal((n, 16), dtype=np.float32)
    x = u @ p["A"] + 0.5 * np.sqrt(p["s"])[None, :] * g.standard_normal((n, d), dtype=np.float32)
    x[:, p["outliers"]] *= 8.0
    return x.astype(np.float32)


def gen_keys(w: Workload, head: int, chunk: int) -> np.ndarray:
    """Key projections of one chunk of one (layer, KV head): storage array [T_chunk, d_head]."""
    t0 = chunk * w.T
    n = min(w.T, w.L - t0)
    return to_storage(_draw_vectors(w, head, _rng(w.seed, _T_KEYS, head, chunk), n), w.dtype)


def gen_queries(w: Workload, head: int) -> np.ndarray:
    """Query projections mapped to one KV head (all Q heads of its GQA group): [nq, d_head]."""
    return to_storage(_draw_vectors(w, head, _rng(w.seed, _T_QUERY, head), w.nq), w.dtype)


def gen_w_enc(w: Workload, head: int) -> np.ndarray:
    """Encoder matrix, feature-major [n_feat, d_head]; rows unit-norm before rounding to storage."""
    g = _rng(w.seed, _T_WENC, head)
    a = g.standard_normal((w.n_feat, w.d_head), dtype=np.float32)
    a /= np.linalg.norm(a.astype(np.float64), axis=1, keepdims=True).astype(np.float32)
    return to_storage(a, w.dtype)


def gen_b_enc(w: Workload, head: int) -> np.ndarray:
    """Encoder bias [n_feat], float32 (b_dec is taken as zero / already folded in)."""
    g = _rng(w.seed, _T_BENC, head)
    b = (w.b_std * g.standard_normal(w.n_feat)).astype(np.float32)
    if w.recipe == "zipf":
        rank = _rng(w.seed, _T_PERM, head).permutation(w.n_feat).astype(np.float64) + 1.0
        b = b + (ZIPF_BETA * (-1.1 * np.log(rank)) + ZIPF_C).astype(np.float32)
    return b


def gen_many(fn, w: Workload, heads, *args, threads: int = 8) -> list:
    """Generate fn(w, head, *args) for several heads on a thread pool (numpy releases the GIL)."""
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda h: fn(w, h, *args), heads))
