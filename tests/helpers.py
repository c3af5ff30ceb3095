"""Glue shared by the tests: turn a synthetic workload into the oracle's inputs."""

from __future__ import annotations

import numpy as np

from oracle import cachefocus_oracle as orc
from paper_2502_11101_amd import workloads as wl


def f64(x):
    return np.asarray(x, dtype=np.float64)


def initial_segments(cfg: wl.Config, st: wl.Structure, b: int, docs=None, shift: int = 0):
    """Segment list of query b before any prune: prefix, the query's documents at the
    positions the oracle's allocator gives them (slot 0 nearest the query), own block."""
    g = cfg.geometry
    slots = list(range(cfg.docs_per_query)) if docs is None else list(docs)
    lens = [int(st.doc_lens[st.query_docs[b, s]]) for s in range(cfg.docs_per_query)]
    new_start, q_start, n_reuse = orc.assign_positions(
        lens, slots, cfg.prefix_len, g.max_positions - cfg.tq, orc.STRATEGY_SORT)
    segs = []
    if cfg.prefix_len:
        segs.append(orc.Segment(0, cfg.prefix_len, 0, 0 + shift, orc.KIND_PREFIX, -1))
    for s in slots:
        doc = int(st.query_docs[b, s])
        segs.append(orc.Segment(int(st.doc_off[doc]), lens[s], cfg.doc_stored_start,
                                new_start[s] + shift, orc.KIND_DOC, s))
    segs.append(orc.Segment(b * cfg.tq, cfg.tq, 0, q_start + shift, orc.KIND_SELF, -1))
    return segs, q_start + shift, lens


def oracle_query(cfg: wl.Config, st: wl.Structure, tensors: dict, b: int, segs, q_start,
                 **kw):
    g = cfg.geometry
    q = f64(tensors["q"][b * cfg.tq:(b + 1) * cfg.tq])
    return orc.prefill_attention(q, 0, q_start, tensors["k_store"], tensors["v_store"],
                                 tensors["k_self"], tensors["v_self"], segs,
                                 g.n_kv_heads, g.rope_base, **kw)


def doc_scores(segs, mass, n_slots):
    s = np.zeros(n_slots)
    for seg, m in zip(segs, mass):
        if seg.kind == orc.KIND_DOC:
            s[seg.doc] += m
    return s
