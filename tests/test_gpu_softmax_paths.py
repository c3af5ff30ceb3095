"""GPU parity of Eq. 1's softmax on inputs built to move the running reference of an online softmax:
scores that rise (or fall) tile after tile, segment after segment and split after split, one late dominant
key, all-equal scores, and a non-default softmax scale.  Every case runs through cf_prefill_attention on
hand-written segment tables and is checked element by element — outputs and per-segment mass — against the
oracle.  The shapes are chosen so that each attention kernel and each kind of launch plan is reached:
few stacked rows / many (the two 16-bit kernels), several splits / one split (partials merged by a second
kernel / rows written by the attention kernel), tables of at most 64 entries / more, and the fp32 kernel.

Only the inputs are adversarial; they are made here, on the generator side, from seeded draws."""

from __future__ import annotations

import math
import sys

import numpy as np
import pytest
import torch

from oracle import cachefocus_oracle as orc
from paper_2502_11101_amd import binding as cf
from paper_2502_11101_amd import pipeline as pl
from paper_2502_11101_amd import workloads as wl
from tests import gpu_harness as G
from tests import helpers as H

pytestmark = pytest.mark.gpu
I32 = dict(dtype=torch.int32, device="cuda")


def _say(msg):
    print(msg, file=sys.stderr, flush=True)


# name -> (geometry, batch, tq, prefix, documents per query, (min, max) document length)
SHAPES = {
    # at most four 16-row blocks per kv head: attn_tile_kernel, several splits, two wavefront groups each
    "few_rows_splits": (wl.Geometry(8, 8, 128, "bf16", 1.0e6, 32768), 1, 48, 32, 6, (160, 160)),
    # the same kernel with one split per (query, head): it normalises and writes the rows itself
    "few_rows_one_split": (wl.Geometry(8, 8, 128, "f16", 1.0e6, 32768), 32, 5, 3, 3, (20, 70)),
    # 28 row blocks per kv head in three row groups: attn_pipe_kernel, several splits
    "many_rows_splits": (wl.Geometry(28, 4, 128, "bf16", 1.0e6, 32768), 1, 64, 32, 8, (100, 200)),
    # 15 row blocks in two row groups, many units: attn_pipe_kernel, one split
    "many_rows_one_split": (wl.Geometry(12, 2, 128, "f16", 1.0e6, 32768), 40, 40, 0, 3, (20, 90)),
    # more than 64 table entries: the segment table lives in LDS instead of registers
    "few_rows_long_table": (wl.Geometry(4, 4, 128, "bf16", 1.0e6, 32768), 1, 16, 2, 70, (1, 9)),
    "many_rows_long_table": (wl.Geometry(14, 2, 128, "bf16", 1.0e6, 32768), 1, 13, 2, 70, (1, 9)),
    # fp32, head_dim 64: the generic kernel
    "f32_generic": (wl.Geometry(4, 2, 64, "f32", 1.0e6, 32768), 2, 8, 4, 4, (20, 40)),
}
# fp16 shapes whose plans have several splits (used by the range test at the end)
FP16_SHAPES = {
    "few_rows_splits_f16": (wl.Geometry(8, 8, 128, "f16", 1.0e6, 32768), 1, 48, 32, 12, (160, 160)),
    "many_rows_splits_f16": (wl.Geometry(28, 4, 128, "f16", 1.0e6, 32768), 1, 64, 32, 16, (100, 200)),
}
PATTERNS = ["rising", "falling", "late_spike", "sawtooth", "equal"]
SPREAD = 4.0            # largest coefficient of the common direction: about 45 nats between first and last key


def _common_direction(d):
    """A vector of squared norm d that lives in the sixteen slowest 2-D slices of the head dimension, which a
    shift of a few thousand positions turns by well under a tenth of a radian at base 1e6: keys that carry it
    stay aligned with queries that carry it whether or not they are re-positioned."""
    u = np.zeros(d, dtype=np.float32)
    half = d // 2
    lo = half - 16
    amp = math.sqrt(d / 32.0)
    u[lo:half] = amp
    u[half + lo:] = amp
    return u


def _build_case(shape, pattern, rotated, seed, shapes=None):
    """Inputs and tables of one case.  Unrotated: every segment sits where it was cached and the query where it
    was computed, so the kernels rotate nothing and their keys equal the oracle's bit for bit.  Rotated: documents
    were cached at the prefix length and are moved to packed positions, the query from 0 to behind them."""
    g, batch, tq, prefix, docs, (lo, hi) = (shapes or SHAPES)[shape]
    rng = np.random.default_rng(seed)
    lens = rng.integers(lo, hi + 1, size=(batch, docs))
    doc_off = prefix + np.concatenate([[0], np.cumsum(lens.reshape(-1))])
    n_store = int(doc_off[-1])
    nq = batch * tq
    u = _common_direction(g.head_dim)
    noise = lambda *s: rng.standard_normal(s, dtype=np.float32)
    q = noise(nq, g.n_q_heads, g.head_dim) + u
    k_store, v_store = noise(n_store, g.n_kv_heads, g.head_dim), noise(n_store, g.n_kv_heads, g.head_dim)
    k_self, v_self = noise(nq, g.n_kv_heads, g.head_dim), noise(nq, g.n_kv_heads, g.head_dim)
    tables, q_pos = [], []
    q_stored = 0 if rotated else prefix + int(lens.sum(axis=1).max())
    for b in range(batch):
        total = int(lens[b].sum())
        qp = prefix + total
        q_pos.append(qp if rotated else q_stored)
        segs = []
        if prefix:
            segs.append(orc.Segment(0, prefix, 0, 0, orc.KIND_PREFIX, -1))
        pos = prefix
        for s in range(docs):
            n = int(lens[b, s])
            segs.append(orc.Segment(int(doc_off[b * docs + s]), n, prefix if rotated else pos, pos, orc.KIND_DOC, s))
            pos += n
        segs.append(orc.Segment(b * tq, tq, q_stored, q_pos[-1], orc.KIND_SELF, -1))
        tables.append(segs)
        # the coefficient of the common direction for every key of the query, in table order
        n_tok = sum(s.len for s in segs)
        idx = 0
        for si, s in enumerate(segs):
            i = idx + np.arange(s.len)
            if pattern == "rising":
                c = SPREAD * i / max(n_tok - 1, 1)
            elif pattern == "falling":
                c = SPREAD * (1.0 - i / max(n_tok - 1, 1))
            elif pattern == "late_spike":
                c = np.where(i == (4 * n_tok) // 5, SPREAD, 0.0)
            elif pattern == "sawtooth":
                c = SPREAD * np.arange(s.len) / max(s.len - 1, 1) * ((si % 3) + 1) / 3.0
            else:
                c = np.zeros(s.len)
            idx += s.len
            if s.kind == orc.KIND_PREFIX and b > 0:
                continue                                   # shared: keeps what the first query gave it
            dst = k_self if s.kind == orc.KIND_SELF else k_store
            dst[s.tok_offset:s.tok_offset + s.len] += c[:, None, None].astype(np.float32) * u
    if pattern == "equal":
        # every key of every query identical: each row's scores are all equal
        one = noise(1, g.n_kv_heads, g.head_dim)
        k_store[:] = one
        k_self[:] = one
    rd = lambda x: wl.round_to_dtype(x, g.dtype)
    t = dict(q=rd(q), k_store=rd(k_store), v_store=rd(v_store), k_self=rd(k_self), v_self=rd(v_self))
    return g, batch, tq, n_store, tables, q_stored, q_pos, t


def _run(g, batch, tq, n_store, tables, q_stored, q_pos, t, layout="token", softmax_scale=0.0):
    kind, pad = G.LAYOUTS[layout]
    ts, hs = (0, 0) if layout == "token" else pl.store_strides(n_store, g.n_kv_heads, g.head_dim, kind, pad)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions,
                        softmax_scale=softmax_scale, store_token_stride=ts, store_head_stride=hs)
    seg_stride = max(len(tb) for tb in tables)
    flat = []
    for tb in tables:
        flat += list(tb) + [orc.Segment(0, 0, 0, 0, orc.KIND_DOC, -1)] * (seg_stride - len(tb))
    segs = cf.segments_to_device(cf.segments_array(flat))
    n_seg = torch.tensor([len(tb) for tb in tables], **I32)
    dev = {k: (pl.store_to_device(v, g.dtype, kind, pad) if k in ("k_store", "v_store") else pl.to_device(v, g.dtype))
           for k, v in t.items()}
    out = torch.full_like(dev["q"], 7.0)
    mass = torch.full((batch, seg_stride), -1.0, dtype=torch.float32, device="cuda")
    max_kv = max(sum(s.len for s in tb) for tb in tables)
    ws_bytes = cf.cf_prefill_workspace_bytes(desc, batch, tq, seg_stride, max_kv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    flag = torch.zeros(1, **I32)
    q_off = torch.arange(0, (batch + 1) * tq, tq, **I32)
    cf.cf_prefill_attention(desc, dev["q"], q_off, q_stored, torch.tensor(q_pos, **I32), dev["k_store"], dev["v_store"], n_store,
                            dev["k_self"], dev["v_self"], segs, n_seg, seg_stride, batch, tq, max_kv, out, mass, None, 1,
                            ws, ws_bytes, flag)
    torch.cuda.synchronize()
    assert flag.item() == 0
    return out.float().cpu().numpy(), mass.cpu().numpy()


def _check(g, batch, tq, tables, q_stored, q_pos, t, got, m, rotated, scale=None, queries=None):
    """Outputs (row-normalised) and every segment's mass (relative): against the plain oracle where no key is
    moved — the kernels' keys are then the oracle's, bit for bit — and against the rounded-key reference where
    keys are moved (with keys this large and softmaxes this sharp, the one rounding of a moved key alone moves an
    output by more than the output tolerance; the reference carries that rounding, so the bound stays the same)."""
    worst_out = worst_mass = 0.0
    for b in (range(batch) if queries is None else queries):
        rows = slice(b * tq, (b + 1) * tq)
        ref_out, ref_mass = orc.prefill_attention(H.f64(t["q"][rows]), q_stored, q_pos[b], t["k_store"], t["v_store"], t["k_self"],
                                                  t["v_self"], tables[b], g.n_kv_heads, g.rope_base, scale=scale)
        if rotated:
            ref_out, ref_mass = H.rounded_key_reference(g.dtype, t["q"][rows], q_stored, q_pos[b], t["k_store"], t["v_store"],
                                                  t["k_self"], t["v_self"], tables[b], g.n_kv_heads, g.rope_base, scale=scale)
        worst_out = max(worst_out, G.row_error(got[rows], ref_out))
        worst_mass = max(worst_mass, G.rel_error(m[b, :len(tables[b])], ref_mass))
        assert m[b, :len(tables[b])].sum() == pytest.approx(g.n_q_heads * tq, rel=1e-5)
    return worst_out, worst_mass


# (all-equal scores exist only in place: moved keys are no longer identical)
@pytest.mark.parametrize("shape,pattern,rotated", [(sh, pa, ro) for sh in SHAPES for pa in PATTERNS for ro in (False, True)
                                                   if not (pa == "equal" and ro)])
def test_reference_moving_score_orders(shape, pattern, rotated):
    _say(f"softmax order {shape} {pattern} {'moved' if rotated else 'in place'}")
    g, batch, tq, n_store, tables, q_stored, q_pos, t = _build_case(shape, pattern, rotated, seed=sum(map(ord, shape + pattern)))
    got, m = _run(g, batch, tq, n_store, tables, q_stored, q_pos, t, layout="head" if rotated else "token")
    queries = None if batch <= 4 else [0, batch // 2, batch - 1]
    worst_out, worst_mass = _check(g, batch, tq, tables, q_stored, q_pos, t, got, m, rotated, queries=queries)
    _say(f"  out err {worst_out:.3e}  mass err {worst_mass:.3e}")
    assert worst_out <= G.OUT_TOL[g.dtype]
    assert worst_mass <= G.MASS_TOL[g.dtype]
    if pattern == "equal":
        # closed form: uniform probabilities over what a row sees
        for b in ([0] if batch > 1 else range(batch)):
            cached = sum(s.len for s in tables[b] if s.kind != orc.KIND_SELF)
            for si, s in enumerate(tables[b]):
                vis = [s.len if s.kind != orc.KIND_SELF else r + 1 for r in range(tq)]
                expect = g.n_q_heads * sum(v / (cached + r + 1) for r, v in enumerate(vis))
                assert m[b, si] == pytest.approx(expect, rel=1e-4)


@pytest.mark.parametrize("factor", [8.0, 0.05])
@pytest.mark.parametrize("shape", ["few_rows_splits", "few_rows_one_split", "many_rows_splits", "many_rows_one_split",
                                   "f32_generic"])
def test_softmax_scale_override(shape, factor):
    """cf_layer_desc.softmax_scale instead of 1/sqrt(d): eight times sharper (row maxima dominate, references move
    often) and twenty times flatter, on plain Gaussian inputs, keys in place and moved."""
    g = SHAPES[shape][0]
    scale = factor / math.sqrt(g.head_dim)
    for rotated in (False, True):
        _say(f"softmax scale {factor}/sqrt(d) {shape} {'moved' if rotated else 'in place'}")
        g, batch, tq, n_store, tables, q_stored, q_pos, t = _build_case(shape, "plain", rotated, seed=400 + int(10 * factor))
        got, m = _run(g, batch, tq, n_store, tables, q_stored, q_pos, t, softmax_scale=scale)
        queries = None if batch <= 4 else [0, batch - 1]
        worst_out, worst_mass = _check(g, batch, tq, tables, q_stored, q_pos, t, got, m, rotated, scale=scale, queries=queries)
        _say(f"  out err {worst_out:.3e}  mass err {worst_mass:.3e}")
        assert worst_out <= G.OUT_TOL[g.dtype]
        # The reference moves keys in fp64, the kernels in fp32: where the two round a key element to different
        # 16-bit neighbours a score differs by one rounding step times the scale, so the sharper softmax is allowed
        # that factor on moved keys.
        assert worst_mass <= G.MASS_TOL[g.dtype] * (max(1.0, factor) if rotated else 1.0)
    # the override is used: the default scale gives something else
    got_default, _ = _run(g, batch, tq, n_store, tables, q_stored, q_pos, t)
    assert G.row_error(got_default, got.astype(np.float64)) > 1e-2


@pytest.mark.parametrize("shape", ["few_rows_splits_f16", "many_rows_splits_f16"])
def test_values_near_the_top_of_fp16_survive_the_split_merge(shape):
    """Several splits per row hand partial rows to the merge in the tensors' 16-bit type.  With values of a few
    ten thousand — the top of fp16 — and thousands of keys, a row's unnormalised accumulator passes fp16's range by
    orders of magnitude; the partial rows are therefore divided by the split's own row sum first and stay bounded by
    the values themselves.  Outputs (Eq. 1) must still match the oracle in the usual metric and none may be
    infinite."""
    _say(f"fp16 range {shape}")
    g, batch, tq, n_store, tables, q_stored, q_pos, t = _build_case(shape, "sawtooth", False, seed=len(shape), shapes=FP16_SHAPES)
    rng = np.random.default_rng(99)
    for name in ("v_store", "v_self"):
        big = rng.uniform(-3.0e4, 3.0e4, size=t[name].shape).astype(np.float32)
        t[name] = wl.round_to_dtype(big, g.dtype)
    got, m = _run(g, batch, tq, n_store, tables, q_stored, q_pos, t)
    assert np.isfinite(got).all()
    worst_out, worst_mass = _check(g, batch, tq, tables, q_stored, q_pos, t, got, m, rotated=False)
    _say(f"  out err {worst_out:.3e}  mass err {worst_mass:.3e}")
    assert worst_out <= G.OUT_TOL[g.dtype]
    assert worst_mass <= G.MASS_TOL[g.dtype]
