"""Seeded synthetic inputs shaped like the paper's RAG workloads.

This module only draws random numbers and lays them out; it contains none of
the method's arithmetic (no RoPE, no attention, no ranking, no position
allocation), so that the CPU oracle and the HIP library can both be fed from
it without sharing any computation.

The paper evaluates on Natural Questions / TriviaQA with 100-word Wikipedia
passages behind a chat template (a shared system prefix, k retrieved passages
of roughly 100-200 tokens, a short question).  None of that text is available
or reproduced; these generators keep only the *shapes* (head geometry of
LLaMA-2-7B / Qwen2, prefix + k passages + question, length mix) and fill them
with seeded Gaussians.  A few documents per query get a "planted relevance"
component along the query's mean direction so that the ranking has a known
answer.

Conventions handed to both sides:
  * The store holds the shared prefix in tokens [0, P) followed by the documents
    back to back; ``doc_off`` is the CSR offset table in tokens.
  * All tensors are row-major [token, head, head_dim] and already rounded (RNE)
    to the configuration's dtype, returned as float32 (f32/bf16) or float16.
  * Stored keys are *declared* to carry RoPE for positions
    ``doc_stored_start + t`` (documents), ``t`` (prefix), ``t`` (the query's own
    block, local positions); since an isotropic Gaussian is rotation invariant
    the draws need no rotation to have that distribution.
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Geometry:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" | "bf16" | "f16"
    rope_base: float
    max_positions: int

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


@dataclass(frozen=True)
class Config:
    name: str
    index: int                      # 1-based position in the list of configurations
    geometry: Geometry
    prefix_len: int
    n_store_docs: int
    doc_len_range: Tuple[int, int]  # inclusive
    batch: int
    tq: int
    docs_per_query: int
    n_planted: int
    keep: int
    doc_stored_start: int
    n_layers: int = 1
    prune_layers: Tuple[int, ...] = ()     # 0-based layers after which a prune event happens
    keep_frac: float = 0.0                 # fractional keep used by the layer stack
    plant_gain: float = 0.5


LLAMA2_7B = Geometry(32, 32, 128, "bf16", 1.0e4, 4096)
QWEN2_7B = Geometry(28, 4, 128, "bf16", 1.0e6, 32768)
QWEN2_1P5B = Geometry(12, 2, 128, "f16", 1.0e6, 32768)

CONFIGS: Dict[str, Config] = {
    "tiny_f32": Config("tiny_f32", 1, Geometry(4, 4, 64, "f32", 1.0e4, 4096),
                       prefix_len=4, n_store_docs=4, doc_len_range=(32, 32), batch=1, tq=8,
                       docs_per_query=4, n_planted=1, keep=2, doc_stored_start=0),
    "llama2_7b_layer": Config("llama2_7b_layer", 2, LLAMA2_7B,
                              prefix_len=32, n_store_docs=10, doc_len_range=(160, 160), batch=1,
                              tq=48, docs_per_query=10, n_planted=2, keep=5, doc_stored_start=32),
    "qwen2_7b_layer": Config("qwen2_7b_layer", 3, QWEN2_7B,
                             prefix_len=32, n_store_docs=50, doc_len_range=(100, 200), batch=1,
                             tq=64, docs_per_query=50, n_planted=5, keep=20, doc_stored_start=32),
    "llama2_7b_stack": Config("llama2_7b_stack", 4, LLAMA2_7B,
                              prefix_len=32, n_store_docs=30, doc_len_range=(160, 160), batch=1,
                              tq=48, docs_per_query=30, n_planted=3, keep=5, doc_stored_start=32,
                              n_layers=32, prune_layers=(7, 15, 23, 31), keep_frac=0.6),
    "qwen2_1p5b_batch": Config("qwen2_1p5b_batch", 5, QWEN2_1P5B,
                               prefix_len=0, n_store_docs=10000, doc_len_range=(100, 200),
                               batch=64, tq=64, docs_per_query=20, n_planted=3, keep=8,
                               doc_stored_start=0),
}


def scaled(cfg: Config, **changes) -> Config:
    """A copy of a configuration with some fields replaced (for reduced-size tests)."""
    d = dict(cfg.__dict__)
    d.update(changes)
    return Config(**d)


# --------------------------------------------------------------------------- rounding
def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the nearest-even value of ``dtype``; the result is
    float32 (f32, bf16) or float16 (f16) and exactly representable in it."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        bits = x.view(np.uint32)
        lsb = (bits >> np.uint32(16)) & np.uint32(1)
        rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
        return rounded.view(np.float32)
    raise ValueError(dtype)


# --------------------------------------------------------------------------- structure
@dataclass
class Structure:
    """Integer side of a workload: lengths, offsets, which documents each query uses."""
    doc_lens: np.ndarray            # [n_store_docs] int32
    doc_off: np.ndarray             # [n_store_docs + 1] int64, tokens, starts after the prefix
    n_store_tokens: int
    query_docs: np.ndarray          # [batch, docs_per_query] int32 store ids (slot order = retriever rank)
    planted: np.ndarray             # [batch, n_planted] int32 query-local slots
    seed: int


def build_structure(cfg: Config, seed: Optional[int] = None) -> Structure:
    seed = 7000 + cfg.index if seed is None else seed
    rng = np.random.default_rng(seed)
    lo, hi = cfg.doc_len_range
    doc_lens = rng.integers(lo, hi + 1, size=cfg.n_store_docs, dtype=np.int64).astype(np.int32)
    doc_off = np.zeros(cfg.n_store_docs + 1, dtype=np.int64)
    doc_off[0] = cfg.prefix_len
    doc_off[1:] = cfg.prefix_len + np.cumsum(doc_lens.astype(np.int64))
    need = cfg.batch * cfg.docs_per_query
    if need > cfg.n_store_docs:
        raise ValueError("not enough documents in the store for disjoint selections")
    if need == cfg.n_store_docs and cfg.batch == 1:
        sel = np.arange(cfg.n_store_docs)
    else:
        sel = rng.permutation(cfg.n_store_docs)[:need]
    query_docs = sel.reshape(cfg.batch, cfg.docs_per_query).astype(np.int32)
    planted = np.stack([np.sort(rng.permutation(cfg.docs_per_query)[:cfg.n_planted])
                        for _ in range(cfg.batch)]).astype(np.int32)
    return Structure(doc_lens, doc_off, int(doc_off[-1]), query_docs, planted, seed)


# --------------------------------------------------------------------------- tensors
def _normal(rng, shape, dtype):
    if dtype == "f16":
        out = np.empty(shape, dtype=np.float16)
        flat = out.reshape(-1)
        step = 1 << 24
        for i in range(0, flat.size, step):
            n = min(step, flat.size - i)
            flat[i:i + n] = rng.standard_normal(n, dtype=np.float32).astype(np.float16)
        return out
    return round_to_dtype(rng.standard_normal(shape, dtype=np.float32), dtype)


def build_layer(cfg: Config, st: Structure, layer: int = 0, seed: Optional[int] = None) -> dict:
    """Draw one layer's tensors.

    Returns dict(q [batch*tq, Hq, d], k_self, v_self [batch*tq, Hkv, d],
    k_store, v_store [n_store_tokens, Hkv, d]).  Planted documents of query b
    get ``plant_gain * qbar_b[kv head]`` added to every key, where qbar_b is the
    mean of that query's q over its tokens and the heads of the kv group,
    rescaled to unit RMS per component.
    """
    g = cfg.geometry
    seed = 1000 * cfg.index + layer if seed is None else seed
    rng = np.random.default_rng(seed)
    nq = cfg.batch * cfg.tq
    q = _normal(rng, (nq, g.n_q_heads, g.head_dim), g.dtype)
    k_self = _normal(rng, (nq, g.n_kv_heads, g.head_dim), g.dtype)
    v_self = _normal(rng, (nq, g.n_kv_heads, g.head_dim), g.dtype)
    k_store = _normal(rng, (st.n_store_tokens, g.n_kv_heads, g.head_dim), g.dtype)
    v_store = _normal(rng, (st.n_store_tokens, g.n_kv_heads, g.head_dim), g.dtype)
    for b in range(cfg.batch):
        qb = q[b * cfg.tq:(b + 1) * cfg.tq].astype(np.float32)
        qbar = qb.reshape(cfg.tq, g.n_kv_heads, g.group, g.head_dim).mean(axis=(0, 2))
        qbar /= np.sqrt(np.mean(qbar * qbar, axis=-1, keepdims=True))
        for slot in st.planted[b]:
            doc = int(st.query_docs[b, slot])
            a, e = int(st.doc_off[doc]), int(st.doc_off[doc + 1])
            planted = k_store[a:e].astype(np.float32) + cfg.plant_gain * qbar[None, :, :]
            k_store[a:e] = round_to_dtype(planted, g.dtype)
    return dict(q=q, k_self=k_self, v_self=v_self, k_store=k_store, v_store=v_store)


def kv_tokens_per_call(cfg: Config, st: Structure, n_docs: Optional[int] = None) -> int:
    """Key positions attended in one layer call, summed over the batch
    (prefix + selected documents + the query's own block; not times heads)."""
    total = 0
    for b in range(cfg.batch):
        docs = st.query_docs[b][:n_docs] if n_docs is not None else st.query_docs[b]
        total += cfg.prefix_len + int(st.doc_lens[docs].sum()) + cfg.tq
    return total
