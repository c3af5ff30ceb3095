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


def rounded_key_reference(dtype: str, q_rows, q_stored_start: int, q_new_start: int, k_store, v_store, k_self, v_self,
                          segs, n_kv_heads: int, rope_base: float, pairing: str = "half", scale=None):
    """A second expected value, from oracle calls only, that carries the one rounding a fused kernel applies
    to a re-positioned key.  Scores depend on relative positions only (Eq. 2), so every segment's keys are
    moved by their shift relative to the query (Eq. 5, orc.reposition_keys), rounded once to the storage
    type, and Eq. 1 is then evaluated on a table without any shift and the query rows as stored.  What is
    left between this and a kernel's result is the kernel's own arithmetic (fp32 scores, softmax, sums),
    not the rounding of the moved keys.  Returns (out, mass) like orc.prefill_attention."""
    q_shift = q_new_start - q_stored_start
    store_k, store_v, own_k, own_v, table = [], [], [], [], []
    n_store = n_own = 0
    for seg in segs:
        own = seg.kind == orc.KIND_SELF
        src_k, src_v = (k_self, v_self) if own else (k_store, v_store)
        k = f64(src_k[seg.tok_offset:seg.tok_offset + seg.len])
        rel = seg.new_start - seg.stored_start - q_shift
        moved = orc.reposition_keys(k, [orc.Segment(0, seg.len, 0, rel, seg.kind)], rope_base, pairing)
        moved = wl.round_to_dtype(moved.astype(np.float32), dtype) if rel != 0 else k
        (own_k if own else store_k).append(f64(moved))
        (own_v if own else store_v).append(f64(src_v[seg.tok_offset:seg.tok_offset + seg.len]))
        table.append(orc.Segment(n_own if own else n_store, seg.len, 0, 0, seg.kind, seg.doc))
        if own:
            n_own += seg.len
        else:
            n_store += seg.len
    cat = lambda xs: np.concatenate(xs) if xs else None
    return orc.prefill_attention(f64(q_rows), 0, 0, cat(store_k), cat(store_v), cat(own_k), cat(own_v), table,
                                 n_kv_heads, rope_base, pairing, scale=scale)


def compact_query(segs, k_store, v_store):
    """The store tokens a table touches, gathered into small arrays, and the table re-addressed to them — so that
    the oracle need not convert a store of millions of tokens to evaluate one query.  Own-block entries are kept."""
    ks, vs, table, n = [], [], [], 0
    for seg in segs:
        if seg.kind == orc.KIND_SELF:
            table.append(seg)
            continue
        ks.append(np.asarray(k_store[seg.tok_offset:seg.tok_offset + seg.len]))
        vs.append(np.asarray(v_store[seg.tok_offset:seg.tok_offset + seg.len]))
        table.append(orc.Segment(n, seg.len, seg.stored_start, seg.new_start, seg.kind, seg.doc))
        n += seg.len
    return np.concatenate(ks), np.concatenate(vs), table


def check_cut(kept, ref_score, lens, alive, keep, planted=(), margin=1e-3):
    """The margin rule for a cut taken on 16-bit scores: a candidate whose length-normalised oracle score is more
    than `margin` (relative) above the oracle's keep-th score must be kept, one that far below must not be; where
    the oracle's own gap at the cut is at least `margin` the kept set therefore equals the oracle's.  Planted
    documents must survive.  Returns the oracle's relative gap at the cut."""
    key = {i: float(ref_score[i]) / int(lens[i]) for i in alive}
    ranked = sorted(alive, key=lambda i: (-key[i], i))
    cut = key[ranked[keep - 1]]
    for i in alive:
        if key[i] > cut * (1 + margin):
            assert i in kept, (i, key[i], cut)
        if key[i] < cut * (1 - margin):
            assert i not in kept, (i, key[i], cut)
    gap = (cut - key[ranked[keep]]) / cut if keep < len(ranked) else float("inf")
    if gap >= margin:
        assert sorted(kept) == sorted(ranked[:keep])
    assert set(int(p) for p in planted) <= set(kept)
    return gap
