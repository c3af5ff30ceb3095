"""GPU tests of what the kernels do with the device-resident tables beyond the plain case: a document listed as
several segments (its score is the sum of their masses, S += s^l of Alg. 2, added in a fixed order), and entries or
queries whose positions leave [0, max_positions) (flagged and skipped, never attended or written)."""

from __future__ import annotations

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


def _inputs(g, n_store, nq, seed):
    rng = np.random.default_rng(seed)
    rnd = lambda *shape: wl.round_to_dtype(rng.standard_normal(shape, dtype=np.float32), g.dtype)
    return dict(q=rnd(nq, g.n_q_heads, g.head_dim), k_self=rnd(nq, g.n_kv_heads, g.head_dim), v_self=rnd(nq, g.n_kv_heads, g.head_dim),
                k_store=rnd(n_store, g.n_kv_heads, g.head_dim), v_store=rnd(n_store, g.n_kv_heads, g.head_dim))


def _attend(g, t, tables, tq, q_stored, q_pos, n_store, n_docs, score0=None):
    """cf_prefill_attention on hand-written tables; returns (out, mass, score, flag)."""
    batch = len(tables)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions)
    seg_stride = max(len(tb) for tb in tables)
    flat = []
    for tb in tables:
        flat += list(tb) + [orc.Segment(0, 0, 0, 0, orc.KIND_DOC, -1)] * (seg_stride - len(tb))
    segs = cf.segments_to_device(cf.segments_array(flat))
    n_seg = torch.tensor([len(tb) for tb in tables], **I32)
    dev = {k: pl.to_device(v, g.dtype) for k, v in t.items()}
    out = torch.full_like(dev["q"], 7.0)
    mass = torch.full((batch, seg_stride), -1.0, dtype=torch.float32, device="cuda")
    score = torch.zeros((batch, n_docs), dtype=torch.float32, device="cuda") if score0 is None else score0.clone()
    max_kv = max(sum(max(s.len, 0) for s in tb) for tb in tables) + 1
    ws_bytes = cf.cf_prefill_workspace_bytes(desc, batch, tq, seg_stride, max_kv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    flag = torch.zeros(1, **I32)
    q_off = torch.arange(0, (batch + 1) * tq, tq, **I32)
    cf.cf_prefill_attention(desc, dev["q"], q_off, q_stored, torch.tensor(q_pos, **I32), dev["k_store"], dev["v_store"], n_store,
                            dev["k_self"], dev["v_self"], segs, n_seg, seg_stride, batch, tq, max_kv, out, mass, score, n_docs,
                            ws, ws_bytes, flag)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), mass.cpu().numpy(), score.cpu().numpy(), int(flag.item())


# geometry, tq, pieces per document: the single-wavefront mass path (at most 64 entries), the block-wide one (more), the
# kernel for many stacked rows, and the fp32 kernel
SPLIT_CASES = {
    "few_rows_small_table": (wl.Geometry(4, 4, 128, "bf16", 1.0e4, 8192), 6, 3),
    "few_rows_long_table": (wl.Geometry(4, 4, 128, "bf16", 1.0e4, 8192), 6, 30),
    "many_rows": (wl.Geometry(14, 2, 128, "f16", 1.0e4, 8192), 13, 4),
    "f32_generic": (wl.Geometry(4, 2, 64, "f32", 1.0e4, 8192), 5, 3),
}


@pytest.mark.parametrize("case", list(SPLIT_CASES))
def test_document_listed_as_several_segments(case):
    """Three documents, each cut into consecutive pieces that are listed as separate table entries feeding the same
    document slot, the pieces of different documents interleaved: every piece's mass matches the oracle, the slot's
    accumulated score is the sum of its pieces on top of what it held, and three runs give the same bits."""
    g, tq, pieces = SPLIT_CASES[case]
    _say(f"split documents {case}")
    prefix, n_docs = 4, 3
    piece_len = [7, 5, 9]
    doc_len = [pieces * n for n in piece_len]
    doc_off = prefix + np.concatenate([[0], np.cumsum(doc_len)])
    n_store = int(doc_off[-1])
    t = _inputs(g, n_store, 2 * tq, seed=61)
    tables, q_pos = [], []
    for b in range(2):
        segs = [orc.Segment(0, prefix, 0, 0, orc.KIND_PREFIX, -1)]
        pos = prefix
        for p in range(pieces):                         # piece p of every document, so a slot's entries are not adjacent
            for d in range(n_docs):
                n = piece_len[d]
                segs.append(orc.Segment(int(doc_off[d]) + p * n, n, prefix + p * n, pos, orc.KIND_DOC, d if b == 0 else n_docs - 1 - d))
                pos += n
        segs.append(orc.Segment(b * tq, tq, 0, pos, orc.KIND_SELF, -1))
        tables.append(segs)
        q_pos.append(pos)
    start = torch.tensor([[0.5, 0.25, 2.0], [1.0, 3.0, 0.125]], dtype=torch.float32, device="cuda")
    runs = [_attend(g, t, tables, tq, 0, q_pos, n_store, n_docs, score0=start) for _ in range(3)]
    out, mass, score, flag = runs[0]
    assert flag == 0
    for other in runs[1:]:
        assert np.array_equal(other[1], mass) and np.array_equal(other[2], score) and np.array_equal(other[0], out)
    for b in range(2):
        rows = slice(b * tq, (b + 1) * tq)
        ref_out, ref_mass = orc.prefill_attention(H.f64(t["q"][rows]), 0, q_pos[b], t["k_store"], t["v_store"], t["k_self"], t["v_self"],
                                                  tables[b], g.n_kv_heads, g.rope_base)
        _, near_mass = H.rounded_key_reference(g.dtype, t["q"][rows], 0, q_pos[b], t["k_store"], t["v_store"], t["k_self"], t["v_self"],
                                               tables[b], g.n_kv_heads, g.rope_base)
        assert G.row_error(out[rows], ref_out) <= G.OUT_TOL[g.dtype]
        tol = G.NEAR_MASS_TOL[g.dtype]
        if not G.rounds_moved_keys(g, cf.CF_ROPE_HALF, len(tables[b])):
            near_mass, tol = ref_mass, G.MASS_TOL[g.dtype]         # the fp32 kernel rounds no moved key
        assert G.rel_error(mass[b, :len(tables[b])], near_mass) <= tol
        expect = start.cpu().numpy()[b].astype(np.float64) + H.doc_scores(tables[b], near_mass, n_docs)
        assert G.rel_error(score[b], expect) <= tol
        # and exactly the sum, in table order, of the masses this call itself reported
        own = start.cpu().numpy()[b].copy()
        for d in range(n_docs):
            s = np.float32(0.0)
            for sg, m in zip(tables[b], mass[b]):
                if sg.kind == orc.KIND_DOC and sg.doc == d:
                    s = np.float32(s + m)
            own[d] = np.float32(own[d] + s)
        assert np.array_equal(score[b], own)


def test_fused_layer_with_split_documents_matches_separate_calls():
    """The fused layer call (epilogue kernel) and the separate calls add a split document's pieces alike."""
    g = wl.Geometry(4, 4, 128, "bf16", 1.0e4, 8192)
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name="split_fused", geometry=g, n_store_docs=6, docs_per_query=6, batch=1,
                    doc_len_range=(24, 24), tq=8, prefix_len=4, doc_stored_start=4, n_planted=1)
    st = wl.build_structure(cfg, seed=7300)
    t = wl.build_layer(cfg, st, seed=73)
    dev = G.upload_layer(cfg, t)
    res = []
    for fused in (False, True):
        pb = G.make_batch(cfg, st)
        pb.allocate_initial()
        torch.cuda.synchronize()
        # cut every document's entry in two halves that feed the same slot: the table grows from 8 to 14 entries
        segs = G.device_segments(pb, 0)
        cut = []
        for s in segs:
            if s.kind == orc.KIND_DOC:
                cut.append(orc.Segment(s.tok_offset, 12, s.stored_start, s.new_start, s.kind, s.doc))
                cut.append(orc.Segment(s.tok_offset + 12, 12, s.stored_start + 12, s.new_start + 12, s.kind, s.doc))
            else:
                cut.append(s)
        wide = pl.PrefillBatch(pb.desc, st.doc_off[:-1][st.query_docs], st.doc_lens[st.query_docs], cfg.tq, cfg.prefix_len,
                               cfg.doc_stored_start, st.n_store_tokens)
        wide.seg_stride = 14
        wide.segs = cf.segments_to_device(cf.segments_array(cut)).reshape(1, 14, 32)
        wide.next_segs = torch.zeros_like(wide.segs)
        wide.n_seg = torch.tensor([14], **I32)
        wide.mass = torch.zeros((1, 14), dtype=torch.float32, device="cuda")
        wide.q_start.copy_(pb.q_start)
        wide.new_start.copy_(pb.new_start)
        wide.ws_bytes = cf.cf_prefill_workspace_bytes(wide.desc, 1, cfg.tq, 14, wide.max_kv_tokens)
        wide.workspace = torch.zeros(wide.ws_bytes, dtype=torch.uint8, device="cuda")
        out = torch.empty_like(dev["q"])
        if fused:
            wide.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, keep=3)
        else:
            wide.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out)
            wide.prune(3)
        torch.cuda.synchronize()
        assert wide.flags() == 0
        res.append(dict(out=out.clone(), mass=wide.mass.clone(), score=wide.score.clone(), keep=wide.keep_idx.clone(),
                        segs=wide.next_segs.clone(), cut=cut, q_start=int(pb.q_start.item())))
    a, b = res
    assert torch.equal(a["out"], b["out"]) and torch.equal(a["mass"], b["mass"]) and torch.equal(a["score"], b["score"])
    assert torch.equal(a["keep"], b["keep"]) and torch.equal(a["segs"][:, :5], b["segs"][:, :5])
    _, ref_mass = H.rounded_key_reference(g.dtype, t["q"][:cfg.tq], 0, a["q_start"], t["k_store"], t["v_store"], t["k_self"], t["v_self"],
                                          a["cut"], g.n_kv_heads, g.rope_base)
    assert G.rel_error(a["score"].cpu().numpy()[0], H.doc_scores(a["cut"], ref_mass, 6)) <= G.NEAR_MASS_TOL[g.dtype]
    lens = [int(x) for x in st.doc_lens[st.query_docs[0]]]
    assert a["keep"][0, :3].tolist() == orc.prune_topk(a["score"].cpu().numpy()[0], lens, list(range(6)), 3)


RANGE_CASES = {
    # geometry, tq, extra empty documents (a table of more than 64 entries lives in LDS)
    "few_rows": (wl.Geometry(4, 4, 128, "bf16", 1.0e4, 1024), 6, 0),
    "few_rows_long_table": (wl.Geometry(4, 4, 128, "bf16", 1.0e4, 1024), 6, 70),
    "many_rows": (wl.Geometry(14, 2, 128, "f16", 1.0e4, 1024), 13, 0),
    "f32_generic": (wl.Geometry(4, 2, 64, "f32", 1.0e4, 1024), 5, 0),
}


@pytest.mark.parametrize("case", list(RANGE_CASES))
def test_attention_flags_positions_outside_the_range(case):
    """Entries whose new or stored positions leave [0, max_positions) raise CF_FLAG_POS_RANGE and are skipped: the
    call gives what the table without them gives (to the last bits: a longer table may cut the tokens into splits
    elsewhere, which changes the order of fp32 sums).  A query placed beyond the range attends nothing (zero rows,
    zero masses); the other query of the batch is unaffected."""
    g, tq, extra = RANGE_CASES[case]
    _say(f"position range {case}")
    mp = g.max_positions
    doc_len = [30, 17, 40, 22]
    doc_off = np.concatenate([[0], np.cumsum(doc_len)])
    n_store = int(doc_off[-1])
    t = _inputs(g, n_store, 2 * tq, seed=67)
    fill = [orc.Segment(0, 0, 0, 0, orc.KIND_DOC, -1)] * extra                 # empty entries, legal
    good = lambda b: fill + [orc.Segment(int(doc_off[0]), 30, 0, 100, orc.KIND_DOC, 0), orc.Segment(int(doc_off[2]), 40, 5, 130, orc.KIND_DOC, 2),
                             orc.Segment(b * tq, tq, 0, 170, orc.KIND_SELF, -1)]
    bad_entries = [orc.Segment(int(doc_off[1]), 17, 0, mp - 16, orc.KIND_DOC, 1),       # last token at max_positions
                   orc.Segment(int(doc_off[3]), 22, 3, -1, orc.KIND_DOC, 3),            # starts before 0
                   orc.Segment(int(doc_off[1]), 17, mp - 5, 40, orc.KIND_DOC, 1)]       # was "stored" beyond the range
    with_bad = lambda b: fill + [good(b)[extra], bad_entries[0], bad_entries[1], good(b)[extra + 1], bad_entries[2], good(b)[extra + 2]]
    ref = _attend(g, t, [good(0), good(1)], tq, 0, [170, 170], n_store, 4)
    assert ref[3] == 0
    got = _attend(g, t, [with_bad(0), with_bad(1)], tq, 0, [170, 170], n_store, 4)
    assert got[3] == cf.CF_FLAG_POS_RANGE
    ulp = 1e-6 if g.dtype == "f32" else 2.0 ** -7
    assert G.row_error(got[0], ref[0].astype(np.float64)) <= ulp
    keep = [extra + 0, extra + 3, extra + 5]
    assert G.rel_error(got[1][:, keep], ref[1][:, extra:extra + 3]) <= 1e-5
    assert np.all(got[1][:, [extra + 1, extra + 2, extra + 4]] == 0.0)
    assert G.rel_error(got[2][:, [0, 2]], ref[2][:, [0, 2]]) <= 1e-5 and np.all(got[2][:, [1, 3]] == 0.0)
    # an entry that ends exactly at max_positions is inside
    edge = [orc.Segment(int(doc_off[1]), 17, 0, mp - 17 - tq, orc.KIND_DOC, 1), orc.Segment(0, tq, 0, mp - tq, orc.KIND_SELF, -1)]
    assert _attend(g, t, [edge, edge], tq, 0, [mp - tq, mp - tq], n_store, 4)[3] == 0
    # query 1 placed so that its last row would sit at max_positions
    out, mass, score, flag = _attend(g, t, [good(0), good(1)], tq, 0, [170, mp - tq + 1], n_store, 4)
    assert flag == cf.CF_FLAG_POS_RANGE
    assert G.row_error(out[:tq], ref[0][:tq].astype(np.float64)) <= ulp and G.rel_error(mass[0, extra:extra + 3], ref[1][0, extra:extra + 3]) <= 1e-5
    assert np.all(out[tq:] == 0.0) and np.all(mass[1, :extra + 3] == 0.0) and np.all(score[1] == 0.0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_reposition_and_assembly_flag_positions_outside_the_range(dtype):
    """cf_reposition_keys leaves an out-of-range entry's tokens untouched; cf_assemble_cache gathers nothing for it."""
    g = wl.Geometry(4, 2, 64, dtype, 1.0e4, 512)
    rng = np.random.default_rng(71)
    n_store, tq = 60, 4
    k = wl.round_to_dtype(rng.standard_normal((n_store, g.n_kv_heads, g.head_dim), dtype=np.float32), g.dtype)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions)
    table = [orc.Segment(0, 20, 0, 100, orc.KIND_DOC, 0), orc.Segment(20, 20, 10, 500, orc.KIND_DOC, 1),
             orc.Segment(40, 20, 0, 492, orc.KIND_DOC, 2)]              # the second ends at 520 > 512, the third at 512
    segs = cf.segments_to_device(cf.segments_array(table))
    k_in = pl.to_device(k, g.dtype)
    k_out = torch.full_like(k_in, 7.0)
    flag = torch.zeros(1, **I32)
    cf.cf_reposition_keys(desc, k_in, k_out, segs, 3, n_store, 20, flag)
    torch.cuda.synchronize()
    assert flag.item() == cf.CF_FLAG_POS_RANGE
    got = k_out.float().cpu().numpy()
    assert np.all(got[20:40] == 7.0)
    ref = orc.reposition_keys(k, [table[0], table[2]], g.rope_base)
    tol = 1e-5 if dtype == "f32" else 2.0 ** -6         # half a bf16 step of the largest magnitudes drawn
    assert np.max(np.abs(got[:20] - ref[:20])) <= tol and np.max(np.abs(got[40:] - ref[40:])) <= tol
    # assembly: the out-of-range entry contributes no tokens
    v_in = pl.to_device(k[::-1].copy(), g.dtype)
    ks = pl.to_device(k[:tq], g.dtype)
    with_self = table + [orc.Segment(0, tq, 0, 200, orc.KIND_SELF, -1)]
    segs = cf.segments_to_device(cf.segments_array(with_self))
    k_f = torch.full((64, g.n_kv_heads, g.head_dim), 7.0, dtype=k_in.dtype, device="cuda")
    v_f = torch.full_like(k_f, 7.0)
    final_len = torch.zeros(1, **I32)
    final_pos = torch.full((64,), -1, **I32)
    flag.zero_()
    cf.cf_assemble_cache(desc, k_in, v_in, n_store, ks, ks, torch.tensor([0, tq], **I32), segs, torch.tensor([4], **I32), 4, 1, tq, 20,
                         torch.zeros(1, dtype=torch.int64, device="cuda"), 64, g.n_kv_heads * g.head_dim, g.head_dim, k_f, v_f,
                         final_len, final_pos, flag)
    torch.cuda.synchronize()
    assert flag.item() == cf.CF_FLAG_POS_RANGE and final_len.item() == 44
    pos = final_pos.cpu().numpy()
    assert pos[:44].tolist() == list(range(100, 120)) + list(range(492, 512)) + list(range(200, 204)) and np.all(pos[44:] == -1)
    assert np.all(k_f.float().cpu().numpy()[44:] == 7.0)
