"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws numbers and lays them out; it holds none of the method's
arithmetic (no RoPE, no attention, no gather) so both the HIP path and the CPU
oracle can consume exactly the same bits from it.

Everything comes from numpy.random.Generator(PCG64(SEED_BASE + config number)).
Values are float32 normal draws rounded once to the storage dtype by torch's
conversion (round to nearest even).  Tensors are torch CPU tensors in the storage
dtype with token-major layout [rows, heads, head_dim].

The workloads stand in for the paper's LongBench / batch-scaling inputs (Sec. 4.4,
Table 2, Table 4): the hot path never sees text, only shapes, so the synthetic
inputs take the paper's context/query lengths and the model attention shapes.
Stored keys are drawn directly as N(0,1): a rotation of an isotropic Gaussian
vector has the same distribution, so they are statistically what "keys rotated at
chunk-local positions" look like (tests that need the raw keys build the store
from `raw_chunks`).
"""
from dataclasses import dataclass, field, replace
from typing import List, Optional

import numpy as np
import torch

SEED_BASE = 20241007

POS_COMPOSITE, POS_REORDERED = 0, 1


@dataclass(frozen=True)
class Shape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str          # "f32" | "bf16"
    rope_base: float
    rope_layout: int = 0   # 0: pair m = channels (2m, 2m+1); 1: pair m = channels (m, m + head_dim/2)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads


@dataclass(frozen=True)
class Config:
    number: int
    name: str
    shape: Shape
    store_chunks: int
    chunk_len_lo: int
    chunk_len_hi: int            # inclusive; lo == hi: fixed length
    n_requests: int
    chunks_per_request: int
    n_q_lo: int
    n_q_hi: int                  # inclusive
    pos_modes: tuple             # allowed modes; >1 entries: drawn per request
    id_draw: str                 # "first" | "uniform" | "zipf" | "shuffle_all" | "packed"
    zipf_s: float = 1.1


QWEN2_7B = Shape(28, 4, 128, "bf16", 1.0e6)
LLAMA3_8B = Shape(32, 8, 128, "bf16", 5.0e5)

CONFIGS = {
    1: Config(1, "tiny-fp32", Shape(4, 4, 64, "f32", 1.0e4), 2, 64, 64, 1, 2, 16, 16,
              (POS_COMPOSITE, POS_REORDERED), "first"),
    2: Config(2, "qwen2-7b-8x512-q64", QWEN2_7B, 256, 512, 512, 1, 8, 64, 64, (POS_REORDERED,), "uniform"),
    3: Config(3, "batched-serving-16req", QWEN2_7B, 1000, 256, 1024, 16, 10, 32, 128,
              (POS_COMPOSITE, POS_REORDERED), "zipf"),
    4: Config(4, "llama3-8b-32x1024-q256", LLAMA3_8B, 32, 1024, 1024, 1, 32, 256, 256, (POS_REORDERED,),
              "shuffle_all"),
    5: Config(5, "offline-64x512", LLAMA3_8B, 64, 512, 512, 1, 64, 0, 0, (POS_COMPOSITE,), "packed"),
}


def scaled(cfg: Config, **kw) -> Config:
    """A smaller (or otherwise altered) copy of a configuration, same recipe."""
    return replace(cfg, **kw)


def rng_for(cfg: Config, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([SEED_BASE + cfg.number, stream]))


def normal_tensor(rng: np.random.Generator, shape, torch_dtype) -> torch.Tensor:
    """N(0,1) float32 draws rounded once to the storage dtype."""
    n = int(np.prod(shape))
    out = torch.empty(shape, dtype=torch_dtype)
    flat = out.view(-1)
    step = 1 << 24                     # bounded temporaries for the 1.3 GB store of config 3
    for s in range(0, n, step):
        e = min(n, s + step)
        flat[s:e] = torch.from_numpy(rng.standard_normal(e - s, dtype=np.float32)).to(torch_dtype)
    return out


def as_oracle_array(t: torch.Tensor) -> np.ndarray:
    """Storage-typed view for the CPU oracle: float32 array, or uint16 array of bf16 bits."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.uint16).numpy()
    if t.dtype == torch.float32:
        return t.numpy()
    raise TypeError(t.dtype)


def from_bits(a: np.ndarray, shape: Shape) -> torch.Tensor:
    """Inverse of as_oracle_array."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.view(torch.bfloat16) if shape.dtype == "bf16" else t


@dataclass
class Store:
    k: torch.Tensor              # [rows, n_kv, d] keys rotated at chunk-local positions
    v: torch.Tensor              # [rows, n_kv, d]
    row_start: np.ndarray        # int64 [n_chunks+1]

    @property
    def n_chunks(self):
        return self.row_start.size - 1

    def chunk_len(self, c):
        return int(self.row_start[c + 1] - self.row_start[c])


@dataclass
class Request:
    chunk_ids: np.ndarray        # int32 [k]
    pos_mode: int
    n_q: int
    q: torch.Tensor              # [n_q, n_q_heads, d]  raw (un-rotated) queries
    k_q: torch.Tensor            # [n_q, n_kv, d]       raw keys of the query tokens
    v_q: torch.Tensor            # [n_q, n_kv, d]
    q_pos: np.ndarray            # int32 [n_q] RoPE position ids of the query tokens
    n_doc: int = 0
    chunk_lens: List[int] = field(default_factory=list)


def chunk_lengths(cfg: Config) -> np.ndarray:
    rng = rng_for(cfg, 1)
    if cfg.chunk_len_lo == cfg.chunk_len_hi:
        return np.full(cfg.store_chunks, cfg.chunk_len_lo, np.int64)
    return rng.integers(cfg.chunk_len_lo, cfg.chunk_len_hi + 1, cfg.store_chunks).astype(np.int64)


def make_store(cfg: Config) -> Store:
    lens = chunk_lengths(cfg)
    row_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    rows = int(row_start[-1])
    sh = cfg.shape
    rng = rng_for(cfg, 2)
    k = normal_tensor(rng, (rows, sh.n_kv_heads, sh.head_dim), sh.torch_dtype)
    v = normal_tensor(rng, (rows, sh.n_kv_heads, sh.head_dim), sh.torch_dtype)
    return Store(k, v, row_start)


def raw_chunks(cfg: Config):
    """Raw (un-rotated) keys and values of the store's chunks, for tests that build
    the store themselves: (k_raw, v, row_start)."""
    s = make_store(cfg)
    return s.k, s.v, s.row_start


def _zipf_ids(rng, cfg: Config, k: int) -> np.ndarray:
    """k distinct ids with P(rank r) proportional to r^-s over the bounded support 1..n,
    ranks mapped to ids by a fixed seeded permutation (popular chunks are not id 0,1,2..)."""
    n = cfg.store_chunks
    w = np.arange(1, n + 1, dtype=np.float64) ** (-cfg.zipf_s)
    cdf = np.cumsum(w / w.sum())
    perm = rng_for(cfg, 3).permutation(n)
    picked = []
    while len(picked) < k:
        r = int(np.searchsorted(cdf, rng.random(), side="right"))
        r = min(r, n - 1)
        if perm[r] not in picked:
            picked.append(int(perm[r]))
    return np.asarray(picked, np.int32)


def query_start(pos_mode: int, chunk_lens) -> int:
    """First position id of the query tokens: after the whole context under reordered
    positions; after the longest chunk under composite positions (config 1 fixes 64 for
    two 64-token chunks; the paper's figure with the ids is not available)."""
    if pos_mode == POS_REORDERED:
        return int(sum(chunk_lens))
    return int(max(chunk_lens)) if len(chunk_lens) else 0


def make_requests(cfg: Config, store: Store, pos_mode: Optional[int] = None) -> List[Request]:
    sh = cfg.shape
    rng = rng_for(cfg, 4)
    reqs = []
    for _ in range(cfg.n_requests):
        k = cfg.chunks_per_request
        if cfg.id_draw == "first":
            ids = np.arange(k, dtype=np.int32)
        elif cfg.id_draw == "uniform":
            ids = rng.choice(cfg.store_chunks, size=k, replace=False).astype(np.int32)
        elif cfg.id_draw == "zipf":
            ids = _zipf_ids(rng, cfg, k)
        elif cfg.id_draw == "shuffle_all":
            ids = rng.permutation(cfg.store_chunks)[:k].astype(np.int32)
        else:
            raise ValueError(cfg.id_draw)
        mode = pos_mode if pos_mode is not None else int(cfg.pos_modes[int(rng.integers(len(cfg.pos_modes)))])
        n_q = int(rng.integers(cfg.n_q_lo, cfg.n_q_hi + 1))
        lens = [store.chunk_len(int(c)) for c in ids]
        q = normal_tensor(rng, (n_q, sh.n_q_heads, sh.head_dim), sh.torch_dtype)
        k_q = normal_tensor(rng, (n_q, sh.n_kv_heads, sh.head_dim), sh.torch_dtype)
        v_q = normal_tensor(rng, (n_q, sh.n_kv_heads, sh.head_dim), sh.torch_dtype)
        q_pos = (query_start(mode, lens) + np.arange(n_q)).astype(np.int32)
        reqs.append(Request(ids, mode, n_q, q, k_q, v_q, q_pos, int(sum(lens)), lens))
    return reqs


@dataclass
class PackedChunks:
    q: torch.Tensor              # [T, n_q_heads, d] raw
    k: torch.Tensor              # [T, n_kv, d] raw
    v: torch.Tensor              # [T, n_kv, d]
    cu: np.ndarray               # int32 [n_chunks+1]


def make_packed_chunks(cfg: Config) -> PackedChunks:
    """Offline precompute input (config 5): chunks packed into one token axis."""
    sh = cfg.shape
    lens = chunk_lengths(cfg)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    rng = rng_for(cfg, 5)
    q = normal_tensor(rng, (T, sh.n_q_heads, sh.head_dim), sh.torch_dtype)
    k = normal_tensor(rng, (T, sh.n_kv_heads, sh.head_dim), sh.torch_dtype)
    v = normal_tensor(rng, (T, sh.n_kv_heads, sh.head_dim), sh.torch_dtype)
    return PackedChunks(q, k, v, cu)
