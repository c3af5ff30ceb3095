"""GPU-side glue for the parity tests: upload a synthetic workload, run the library through
its C ABI (via the binding), fetch results, and compute the error metrics."""

from __future__ import annotations

import numpy as np
import torch

from oracle import cachefocus_oracle as orc
from paper_2502_11101_amd import binding as cf
from paper_2502_11101_amd import pipeline as pl
from paper_2502_11101_amd import workloads as wl

OUT_TOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 2e-2}
MASS_TOL = {"f32": 1e-5, "bf16": 1e-4, "f16": 1e-4}
# Masses against the rounded-key reference (helpers.rounded_key_reference) on shapes with few rows and short
# documents: 1e-4 for the kernels' own arithmetic plus as much again for key elements that the kernels' fp32
# rotation (hardware sine/cosine) rounds to the other 16-bit neighbour than the reference's fp64 rotation does — a
# few elements in a thousand, each moving one score by a 16-bit step.  (Seen over all such tests: at most 1.2e-4.)
NEAR_MASS_TOL = {"f32": 1e-5, "bf16": 2e-4, "f16": 2e-4}


def rounds_moved_keys(g, pairing, seg_stride) -> bool:
    """Whether a call of this shape takes the 16-bit MFMA kernels, which round a moved key once to the storage
    type (the generic kernel moves keys in fp32 on the fly and rounds nothing)."""
    return g.dtype != "f32" and g.head_dim == 128 and pairing == cf.CF_ROPE_HALF and seg_stride <= 256


# store layouts exercised by the tests: token-major, head-major, head-major with unused rows per head
LAYOUTS = {"token": ("token", 0), "head": ("head", 0), "head_padded": ("head", 5)}


def desc_of(cfg: wl.Config, pairing=cf.CF_ROPE_HALF, layout="token", n_store_tokens=0):
    g = cfg.geometry
    kind, pad = LAYOUTS[layout]
    ts, hs = (0, 0) if layout == "token" else pl.store_strides(n_store_tokens, g.n_kv_heads, g.head_dim, kind, pad)
    return cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions, pairing,
                        store_token_stride=ts, store_head_stride=hs)


def upload_layer(cfg: wl.Config, tensors: dict, layout="token"):
    g = cfg.geometry
    kind, pad = LAYOUTS[layout]
    return {k: (pl.store_to_device(v, g.dtype, kind, pad) if k in ("k_store", "v_store") else pl.to_device(v, g.dtype))
            for k, v in tensors.items()}


def make_batch(cfg: wl.Config, st: wl.Structure, pairing=cf.CF_ROPE_HALF, layout="token") -> pl.PrefillBatch:
    off = st.doc_off[:-1][st.query_docs]                 # [batch, k]
    lens = st.doc_lens[st.query_docs]
    return pl.PrefillBatch(desc_of(cfg, pairing, layout, st.n_store_tokens), off, lens, cfg.tq, cfg.prefix_len,
                           cfg.doc_stored_start, st.n_store_tokens)


def row_error(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max over (row, head) of ||gpu - ref||_inf / ||ref[row, head]||_inf."""
    diff = np.abs(gpu.astype(np.float64) - ref).max(axis=-1)
    norm = np.abs(ref).max(axis=-1)
    return float((diff / norm).max())


def rel_error(gpu: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    return float((np.abs(gpu.astype(np.float64) - ref) / np.maximum(np.abs(ref), 1e-300)).max())


def device_segments(pb: pl.PrefillBatch, b: int):
    """Query b's current segment table as oracle Segment tuples."""
    n = int(pb.n_seg[b].item())
    arr = cf.segments_from_device(pb.segs[b], n)
    return [orc.Segment(int(r["tok_offset"]), int(r["len"]), int(r["stored_start"]), int(r["new_start"]),
                        int(r["kind"]), int(r["doc"])) for r in arr]


def oracle_on_device_segments(cfg: wl.Config, tensors: dict, pb: pl.PrefillBatch, b: int, pairing="half"):
    """Run the oracle for query b on exactly the segment table the device holds."""
    g = cfg.geometry
    segs = device_segments(pb, b)
    q_start = int(pb.q_start[b].item())
    q = np.asarray(tensors["q"][b * cfg.tq:(b + 1) * cfg.tq], dtype=np.float64)
    out, mass = orc.prefill_attention(q, pb.q_stored_start, q_start, tensors["k_store"], tensors["v_store"],
                                      tensors["k_self"], tensors["v_self"], segs, g.n_kv_heads, g.rope_base,
                                      pairing)
    return segs, out, mass
