"""CPU oracle for the CacheFocus re-positioned cached-KV prefill path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, double-precision
definition that the HIP library is checked against.  It is imported by the
tests, by the smoke check and by the benchmark's CPU-baseline leg, and by
nothing on the product path.  It shares no code with the HIP path and does not
import the package.

Everything is NumPy float64 on the dtype-rounded inputs the GPU receives; a
matmul is the only library primitive used as a step.  No blocking, no fusion,
no online softmax: each function is the paper's definition written out.

What each function follows:

* ``rope_theta``, ``rotate``            RoPE rotation matrix, Eq. 2 (Background).
* ``reposition_keys``                   Cache Re-Positioning, Eq. 5 (Sec. 2.3).
* ``assemble_final_cache``              Alg. 2, Phase 2 (Final Re-Positioning): the gathered,
                                        re-positioned cache of one layer; ``decode_attention``
                                        is Eq. 1 over it (Phase 3's attention).
* ``prefill_attention``                 Eq. 1 over prefix + parallel document caches +
                                        the query's own causal block (Alg. 2, the
                                        ``layer_l`` step), and the document-wise
                                        attention score of the footnote in Sec. 2.4.
* ``prune_topk``                        Alg. 2, the ``argsort`` / ``prun`` steps.
* ``keep_schedule``                     the k_prune formula of the set-up appendix.
* ``assign_positions``                  Adaptive Re-Positioning, Eq. 6 (Sec. 2.3.1) and
                                        the "align" / "sort" strategies of Sec. 2.5.
* ``layer_adaptive_prefill``            Alg. 2, Phase 1, as a loop over the above.

Pins (tests/test_oracle_pins.py):
  rotate / reposition_keys   rotation by +D then -D is the identity; both forms
                             of Eq. 5 agree; norm preservation; D = 0 is exact.
  prefill_attention          softmax rows sum to 1; masses sum to Hq*Tq; closed
                             form for Q = 0; equality with torch's
                             scaled_dot_product_attention in the reducible
                             cases (also with a non-default ``scale``, against the
                             library's own scale argument); invariance under a
                             common position shift; brute-force triple loop on the
                             tiny configuration.
  assemble_final_cache       plain attention of an absolutely positioned query over the
                             assembled cache equals prefill_attention on the original
                             store (relative-position invariance); zero shift copies;
                             positions listed match the allocation.
  prune_topk                 brute force by full sort; planted documents survive.
  keep_schedule              the appendix's worked example (28, 4, 40, 5 -> 5).
  assign_positions           exhaustive slot marking; the "k = 20, N_reuse = k/5"
                             example; N_reuse = 1 gives contiguous packing.
Readings of the paper that nothing in it pins ("parity unpinned", fixed by this
build's own reading only): the half-split element pairing of RoPE, what counts
as the positional range L in Eq. 6, l_C for unequal lengths (the maximum),
contiguous-chunk grouping, right-alignment of every group to the query, and
raw-sum aggregation of the attention mass with length normalisation at ranking
time.
"""

from __future__ import annotations

import math
from fractions import Fraction
from typing import Callable, NamedTuple, Optional, Sequence

import numpy as np

KIND_PREFIX = 0
KIND_DOC = 1
KIND_SELF = 2

STRATEGY_KEEP = 0
STRATEGY_ALIGN = 1
STRATEGY_SORT = 2


class Segment(NamedTuple):
    """One run of cached tokens attended by a query.

    ``tok_offset`` indexes the K/V store (PREFIX, DOC) or the query's own K/V
    block (SELF).  Token ``t`` of the segment was cached at position
    ``stored_start + t`` and is attended at position ``new_start + t``.
    ``doc`` is the query-local document slot (retriever rank), or -1.
    """

    tok_offset: int
    len: int
    stored_start: int
    new_start: int
    kind: int
    doc: int = -1


# --------------------------------------------------------------------------- RoPE
def rope_theta(head_dim: int, rope_base: float) -> np.ndarray:
    """Per-pair angular step theta_m = base^(-2m/d), m = 0 .. d/2-1.

    The paper only names "the rotation angle r_i for position i" (Eq. 2); the
    linear schedule r_i = i * theta_m is RoPE's own definition.
    """
    m = np.arange(head_dim // 2, dtype=np.float64)
    return np.float64(rope_base) ** (-2.0 * m / head_dim)


def _pair_index(head_dim: int, pairing: str):
    half = head_dim // 2
    m = np.arange(half)
    if pairing == "half":
        return m, m + half
    if pairing == "interleaved":
        return 2 * m, 2 * m + 1
    raise ValueError(f"unknown pairing {pairing!r}")


def rotate(x, delta, rope_base: float, pairing: str = "half") -> np.ndarray:
    """Apply the 2x2 rotation of Eq. 2 by ``delta`` positions to every pair of x.

    x: [..., d]; delta: integer(s) broadcastable against x.shape[:-1].
    For the pair (a, b) of slice m:  a' = a cos(D th_m) - b sin(D th_m),
                                     b' = a sin(D th_m) + b cos(D th_m).
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    theta = rope_theta(d, rope_base)
    ang = np.asarray(delta, dtype=np.float64)[..., None] * theta
    c, s = np.cos(ang), np.sin(ang)
    ia, ib = _pair_index(d, pairing)
    a, b = x[..., ia], x[..., ib]
    out = np.empty_like(x)
    out[..., ia] = a * c - b * s
    out[..., ib] = a * s + b * c
    return out


def reposition_keys(k_store, segments: Sequence[Segment], rope_base: float,
                    pairing: str = "half") -> np.ndarray:
    """Eq. 5: move every key of every listed segment from its stored position to
    its new one, k_j = R_j R_i^T k_i, i.e. a rotation by (j - i) positions.
    Tokens outside the listed segments are returned unchanged."""
    out = np.array(k_store, dtype=np.float64, copy=True)
    for seg in segments:
        sl = slice(seg.tok_offset, seg.tok_offset + seg.len)
        out[sl] = rotate(out[sl], seg.new_start - seg.stored_start, rope_base, pairing)
    return out


def assemble_final_cache(k_store, v_store, k_self, v_self, segments: Sequence[Segment],
                         tq: int, rope_base: float, pairing: str = "half"):
    """Alg. 2, Phase 2 (Final Re-Positioning) for one layer and one query:
    C_final = concat(repos(C, ids), C_Q).  The listed segments, in table order, are
    gathered into one contiguous cache; every key is moved from its stored position
    to its final one by Eq. 5 (the query's own block like any other segment, from
    the position it was computed at to the final q_start); values are copied.
    Returns (k_final [N, Hkv, d], v_final [N, Hkv, d], pos [N]): pos is the position
    each gathered token now sits at.  Only the first ``tq`` tokens of the own block
    exist."""
    ks, vs, ps = [], [], []
    for seg in segments:
        own = seg.kind == KIND_SELF
        n = min(seg.len, tq) if own else seg.len
        src_k = k_self if own else k_store
        src_v = v_self if own else v_store
        k = np.asarray(src_k[seg.tok_offset:seg.tok_offset + n], dtype=np.float64)
        ks.append(rotate(k, seg.new_start - seg.stored_start, rope_base, pairing))
        vs.append(np.asarray(src_v[seg.tok_offset:seg.tok_offset + n], dtype=np.float64))
        ps.append(seg.new_start + np.arange(n))
    if not ks:
        raise ValueError("no segments")
    return np.concatenate(ks), np.concatenate(vs), np.concatenate(ps)


def decode_attention(q_abs, k_final, v_final, n_kv_heads: int, scale: Optional[float] = None):
    """Eq. 1 for decode-time queries over an assembled cache (Alg. 2, Phase 3): q_abs
    [T, Hq, d] already carries RoPE for its absolute position, the keys of k_final
    theirs; every query sees the whole cache.  Plain softmax(q k^T / sqrt(d)) v."""
    q = np.asarray(q_abs, dtype=np.float64)
    k = np.asarray(k_final, dtype=np.float64)
    v = np.asarray(v_final, dtype=np.float64)
    t, hq, d = q.shape
    g = hq // n_kv_heads
    sc = (1.0 / math.sqrt(d)) if scale is None else scale
    out = np.zeros_like(q)
    for h in range(hq):
        s = sc * (q[:, h, :] @ k[:, h // g, :].T)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, h // g, :]
    return out


# --------------------------------------------------------------------------- attention
def prefill_attention(q, q_stored_start: int, q_new_start: int,
                      k_store, v_store, k_self, v_self,
                      segments: Sequence[Segment], n_kv_heads: int,
                      rope_base: float, pairing: str = "half",
                      scale: Optional[float] = None, return_probs: bool = False):
    """One layer's attention of one query against its segment list.

    q: [Tq, Hq, d], row t rotated for position q_stored_start + t, attended at
    q_new_start + t.  k_store/v_store: [tokens, Hkv, d].  k_self/v_self:
    [Tq, Hkv, d] or None.

    Row (t, h) sees all tokens of PREFIX and DOC segments and tokens 0..t of
    the SELF segment (causal masking, the footnote to Eq. 1), in one softmax
    (Eq. 1) with kv head h // (Hq/Hkv).  Returns (out [Tq, Hq, d],
    mass [n_seg]) where mass[s] is the probability summed over heads, query
    tokens and the tokens of segment s (the document-wise score of Alg. 2).
    """
    q = np.asarray(q, dtype=np.float64)
    tq, hq, d = q.shape
    group = hq // n_kv_heads
    if scale is None:
        scale = 1.0 / math.sqrt(d)

    keys, vals, col_seg, col_tok = [], [], [], []
    for si, seg in enumerate(segments):
        if seg.kind == KIND_SELF:
            ks = np.asarray(k_self, dtype=np.float64)[seg.tok_offset:seg.tok_offset + seg.len]
            vs = np.asarray(v_self, dtype=np.float64)[seg.tok_offset:seg.tok_offset + seg.len]
        else:
            ks = np.asarray(k_store, dtype=np.float64)[seg.tok_offset:seg.tok_offset + seg.len]
            vs = np.asarray(v_store, dtype=np.float64)[seg.tok_offset:seg.tok_offset + seg.len]
        keys.append(rotate(ks, seg.new_start - seg.stored_start, rope_base, pairing))
        vals.append(vs)
        col_seg.append(np.full(seg.len, si))
        col_tok.append(np.arange(seg.len))
    n_seg = len(segments)
    if not keys:
        return np.zeros_like(q), np.zeros(0)
    k_all = np.concatenate(keys, axis=0)            # [N, Hkv, d]
    v_all = np.concatenate(vals, axis=0)
    col_seg = np.concatenate(col_seg)
    col_tok = np.concatenate(col_tok)
    n_tok = k_all.shape[0]

    q_rot = rotate(q, q_new_start - q_stored_start, rope_base, pairing)

    # visibility [Tq, N]
    visible = np.ones((tq, n_tok), dtype=bool)
    for si, seg in enumerate(segments):
        if seg.kind == KIND_SELF:
            cols = np.nonzero(col_seg == si)[0]
            visible[:, cols] = col_tok[cols][None, :] <= np.arange(tq)[:, None]

    out = np.zeros((tq, hq, d))
    mass = np.zeros(n_seg)
    probs = np.zeros((hq, tq, n_tok)) if return_probs else None
    for h in range(hq):
        kv = h // group
        s = scale * (q_rot[:, h, :] @ k_all[:, kv, :].T)     # [Tq, N]
        s = np.where(visible, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        m = np.where(np.isfinite(m), m, 0.0)
        p = np.exp(s - m)
        z = p.sum(axis=1, keepdims=True)
        pn = np.divide(p, z, out=np.zeros_like(p), where=z > 0)
        out[:, h, :] = pn @ v_all[:, kv, :]
        mass += np.bincount(col_seg, weights=pn.sum(axis=0), minlength=n_seg)
        if return_probs:
            probs[h] = pn
    if return_probs:
        return out, mass, probs
    return out, mass


# --------------------------------------------------------------------------- pruning
def prune_topk(score, lens, cand: Sequence[int], keep: int):
    """Alg. 2's argsort + prun: rank the candidate documents and keep the best.

    score[i] is the accumulated attention mass S_i of document slot i.  When
    ``lens`` is given the ranking key is S_i / len_i (equal to ranking by S_i
    for equal lengths, the paper's fixed-length-passage regime), compared
    exactly as S_i * len_j versus S_j * len_i.  Descending; ties go to the lower
    document index.  Returns the kept slots, best first.
    """
    cand = [int(c) for c in cand]
    if keep < 0 or keep > len(cand):
        raise ValueError("keep out of range")
    for c in cand:
        if not math.isfinite(float(score[c])):
            raise ValueError("non-finite score")
    if lens is None:
        key = {c: Fraction(float(score[c])) for c in cand}
    else:
        key = {c: Fraction(float(score[c])) / int(lens[c]) for c in cand}
    ranked = sorted(cand, key=lambda c: (-key[c], c))
    return ranked[:keep]


def keep_schedule(n_layers: int, every: int, k: int, k_finish: int):
    """Documents kept after each prune event of Alg. 2 (events at layers that
    are multiples of ``every``).  The appendix prunes (k - k_finish)/(L/n) per
    event; when that is not an integer the cumulative amount is floored so the
    last event leaves exactly k_finish."""
    events = n_layers // every
    if events == 0:
        return []
    return [k - (j * (k - k_finish)) // events for j in range(1, events + 1)]


def keep_fraction(k_current: int, frac: float) -> int:
    """Fractional form used by the layer-stack configuration: keep
    ceil(frac * k_current), at least one."""
    return max(1, int(math.ceil(frac * k_current - 1e-12)))


# --------------------------------------------------------------------------- position allocation
def assign_positions(lens, ranked: Sequence[int], pos_begin: int, pos_end: int,
                     strategy: int = STRATEGY_SORT, force_n_reuse: int = 0):
    """Adaptive Re-Positioning (Eq. 6) + Adaptive Positional Allocation (Sec. 2.5).

    lens[i]: length of document slot i.  ranked: the survivors, best first.
    Positions available to documents are [pos_begin, pos_end).

    l_C = longest survivor; capacity = floor((pos_end - pos_begin) / l_C);
    N_reuse = ceil(n / capacity) unless forced.  The placement order is
    ``ranked`` for "sort", the survivors by ascending slot index (their original
    retriever order) for "align".  That order is cut into N_reuse contiguous
    chunks of ceil(n / N_reuse); inside a chunk documents sit back to back, the
    first of the chunk ending where the query starts, so every chunk ends at
    q_start and q_start = pos_begin + the longest chunk's span.

    Returns (new_start {slot: position}, q_start, n_reuse).  STRATEGY_KEEP
    leaves positions alone and returns ({}, None, 0).
    """
    if strategy == STRATEGY_KEEP:
        return {}, None, 0
    order = [int(r) for r in ranked]
    n = len(order)
    if strategy == STRATEGY_ALIGN:
        order = sorted(order)
    elif strategy != STRATEGY_SORT:
        raise ValueError("unknown strategy")
    if n == 0:
        return {}, pos_begin, 0
    span_avail = pos_end - pos_begin
    l_c = max(int(lens[i]) for i in order)
    if l_c <= 0:
        raise ValueError("empty document")
    cap = span_avail // l_c
    if cap <= 0:
        raise ValueError("a document is longer than the positional range")
    n_reuse = force_n_reuse if force_n_reuse > 0 else -(-n // cap)
    n_reuse = min(n_reuse, n)
    per_group = -(-n // n_reuse)
    groups = [order[g * per_group:(g + 1) * per_group] for g in range(n_reuse)]
    spans = [sum(int(lens[i]) for i in grp) for grp in groups]
    if max(spans) > span_avail:
        raise ValueError("group does not fit the positional range")
    q_start = pos_begin + max(spans)
    new_start = {}
    for grp in groups:
        end = q_start
        for i in grp:
            end -= int(lens[i])
            new_start[i] = end
    return new_start, q_start, n_reuse


# --------------------------------------------------------------------------- Alg. 2, Phase 1
def layer_adaptive_prefill(n_layers: int, layer_inputs: Callable[[int], dict],
                           doc_lens: Sequence[int], doc_tok_offset: Sequence[int],
                           doc_stored_start: int, prefix_len: int, tq: int,
                           n_kv_heads: int, rope_base: float, max_positions: int,
                           prune_layers: dict, strategy: int = STRATEGY_SORT,
                           pairing: str = "half", normalise_by_len: bool = True):
    """Alg. 2, Phase 1, for one query.

    layer_inputs(l) -> dict(q, k_store, v_store, k_self, v_self) for layer l
    (0-based).  The prefix occupies store tokens [0, prefix_len) at positions
    [0, prefix_len).  prune_layers maps a 0-based layer index to the number of
    documents kept after that layer.  A prune decided after layer l takes
    effect from layer l+1; S is never reset.

    Returns a list with, per layer, dict(out, mass, segments, q_start, ids,
    n_reuse) and the final (ids, S).
    """
    k = len(doc_lens)
    ids = list(range(k))                 # retriever order, slot 0 = best
    score = np.zeros(k)
    pos_begin = prefix_len
    pos_end = max_positions - tq
    new_start, q_start, n_reuse = assign_positions(doc_lens, ids, pos_begin, pos_end,
                                                   STRATEGY_SORT)
    trace = []
    for layer in range(n_layers):
        t = layer_inputs(layer)
        segs = []
        if prefix_len:
            segs.append(Segment(0, prefix_len, 0, 0, KIND_PREFIX, -1))
        for i in ids:
            segs.append(Segment(int(doc_tok_offset[i]), int(doc_lens[i]), doc_stored_start,
                                new_start[i], KIND_DOC, i))
        segs.append(Segment(0, tq, 0, q_start, KIND_SELF, -1))
        out, mass = prefill_attention(t["q"], 0, q_start, t["k_store"], t["v_store"],
                                      t["k_self"], t["v_self"], segs, n_kv_heads,
                                      rope_base, pairing)
        for seg, m in zip(segs, mass):
            if seg.kind == KIND_DOC:
                score[seg.doc] += m
        trace.append(dict(out=out, mass=mass, segments=segs, q_start=q_start,
                          ids=list(ids), n_reuse=n_reuse, score=score.copy()))
        if layer in prune_layers:
            ranked = prune_topk(score, doc_lens if normalise_by_len else None, ids,
                                prune_layers[layer])
            if strategy == STRATEGY_KEEP:
                kept = set(ranked)
                ids = [i for i in ids if i in kept]
            else:
                ns, q_start, n_reuse = assign_positions(doc_lens, ranked, pos_begin, pos_end,
                                                        strategy)
                new_start = {**new_start, **ns}
                ids = sorted(ranked) if strategy == STRATEGY_ALIGN else list(ranked)
    return trace, ids, score
