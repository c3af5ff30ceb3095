"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Integer results (kept indices, positions, segment tables) must be bit-exact;
attention outputs within 1e-4 (fp32) / 2e-2 (16-bit) in the row-normalised max error; masses
within 1e-5 / 1e-4 relative."""

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
    print(msg, flush=True)


# ----------------------------------------------------------------------------- cf_reposition_keys
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("pairing", [cf.CF_ROPE_HALF, cf.CF_ROPE_INTERLEAVED])
@pytest.mark.parametrize("hkv,d,base", [(4, 64, 1.0e4), (2, 128, 1.0e6)])
def test_reposition_keys_matches_oracle(dtype, pairing, hkv, d, base):
    _say(f"reposition dtype={dtype} pairing={pairing} hkv={hkv} d={d}")
    rng = np.random.default_rng(21)
    n_tok = 700
    k = wl.round_to_dtype(rng.standard_normal((n_tok, hkv, d), dtype=np.float32), dtype)
    segs = [orc.Segment(0, 33, 0, 0, 1, 0), orc.Segment(40, 161, 32, 1999, 1, 1),
            orc.Segment(210, 1, 5, 30000 if base > 1e5 else 4000, 1, 2), orc.Segment(300, 0, 0, 9, 1, 3),
            orc.Segment(320, 380, 32, 7, 1, 4)]
    desc = cf.make_desc(hkv, hkv, d, dtype, base, 32768, pairing)
    k_dev = pl.to_device(k, dtype)
    out = torch.empty_like(k_dev)
    out.copy_(k_dev)
    seg_dev = cf.segments_to_device(cf.segments_array(segs))
    flag = torch.zeros(1, **I32)
    cf.cf_reposition_keys(desc, k_dev, out, seg_dev, len(segs), n_tok, 64, flag)
    torch.cuda.synchronize()
    ref = orc.reposition_keys(k, segs, base, "half" if pairing == cf.CF_ROPE_HALF else "interleaved")
    got = out.float().cpu().numpy().astype(np.float64)
    tol = {"f32": 2e-6, "bf16": 2.0 ** -8, "f16": 2.0 ** -10}[dtype]
    assert np.max(np.abs(got - ref)) <= tol * max(1.0, np.abs(ref).max())
    assert flag.item() == 0
    # the zero-shift segment and all unlisted tokens are bit-identical
    same = torch.ones(n_tok, dtype=torch.bool)
    for s in segs[1:]:
        same[s.tok_offset:s.tok_offset + s.len] = False
    assert torch.equal(out.cpu()[same], k_dev.cpu()[same])
    # in place, then back: rotation by +D then -D returns the input to within rounding
    cf.cf_reposition_keys(desc, k_dev, k_dev, seg_dev, len(segs), n_tok, 64, flag)
    assert torch.equal(k_dev, out)
    back = [s._replace(stored_start=s.new_start, new_start=s.stored_start) for s in segs]
    cf.cf_reposition_keys(desc, k_dev, k_dev, cf.segments_to_device(cf.segments_array(back)), len(back), n_tok,
                          64, flag)
    torch.cuda.synchronize()
    assert np.max(np.abs(k_dev.float().cpu().numpy() - k)) <= 2.5 * tol * max(1.0, np.abs(k).max())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_reposition_keys_head_major_store(dtype):
    """The same call on a head-major store [kv head][token + unused rows][head_dim]."""
    _say(f"reposition head-major dtype={dtype}")
    rng = np.random.default_rng(22)
    n_tok, hkv, d, base, pad = 500, 3, 128, 1.0e4, 7
    k = wl.round_to_dtype(rng.standard_normal((n_tok, hkv, d), dtype=np.float32), dtype)
    segs = [orc.Segment(0, 40, 0, 0, 1, 0), orc.Segment(40, 161, 32, 1999, 1, 1), orc.Segment(260, 240, 32, 7, 1, 2)]
    ts, hs = pl.store_strides(n_tok, hkv, d, "head", pad)
    desc = cf.make_desc(hkv, hkv, d, dtype, base, 32768, store_token_stride=ts, store_head_stride=hs)
    k_dev = pl.store_to_device(k, dtype, "head", pad)
    k_dev[:, n_tok:] = 3.0                      # the unused rows must stay untouched
    out = k_dev.clone()
    flag = torch.zeros(1, **I32)
    cf.cf_reposition_keys(desc, k_dev, out, cf.segments_to_device(cf.segments_array(segs)), len(segs), n_tok, 64, flag)
    torch.cuda.synchronize()
    ref = orc.reposition_keys(k, segs, base, "half")
    got = out[:, :n_tok].float().cpu().numpy().astype(np.float64).transpose(1, 0, 2)
    tol = {"f32": 2e-6, "bf16": 2.0 ** -8}[dtype]
    assert np.max(np.abs(got - ref)) <= tol * max(1.0, np.abs(ref).max())
    assert flag.item() == 0 and torch.all(out[:, n_tok:] == 3.0)


def test_reposition_flags_bad_segments_without_touching_memory():
    desc = cf.make_desc(2, 2, 64, "bf16", 1.0e4, 4096)
    k = torch.randn(50, 2, 64, device="cuda").to(torch.bfloat16)
    ref = k.clone()
    segs = [orc.Segment(40, 20, 0, 5, 1, 0), orc.Segment(-3, 5, 0, 5, 1, 1), orc.Segment(0, -1, 0, 5, 1, 2)]
    flag = torch.zeros(1, **I32)
    cf.cf_reposition_keys(desc, k, k, cf.segments_to_device(cf.segments_array(segs)), 3, 50, 32, flag)
    torch.cuda.synchronize()
    assert flag.item() == cf.CF_FLAG_BAD_SEGMENT
    assert torch.equal(k, ref)


# ----------------------------------------------------------------------------- cf_prune_topk
def test_prune_topk_bit_exact_random_and_ties():
    rng = np.random.default_rng(31)
    batch, stride = 37, 50
    score = (rng.integers(0, 12, size=(batch, stride)) / 8.0).astype(np.float32)     # many exact ties
    score[::2] = rng.random((len(score[::2]), stride), dtype=np.float32) * 100
    lens = rng.integers(100, 201, size=(batch, stride)).astype(np.int32)
    n_cand = rng.integers(1, stride + 1, size=batch).astype(np.int32)
    cand = np.stack([rng.permutation(stride) for _ in range(batch)]).astype(np.int32)
    for use_len in (True, False):
        for keep in (0, 1, 7, 50):
            keep_idx = torch.full((batch, stride), -1, **I32)
            n_keep = torch.zeros(batch, **I32)
            flag = torch.zeros(1, **I32)
            cf.cf_prune_topk(torch.from_numpy(score).cuda(), torch.from_numpy(lens).cuda() if use_len else None,
                             torch.from_numpy(cand).cuda(), torch.from_numpy(n_cand).cuda(), keep, batch, stride,
                             keep_idx, n_keep, flag)
            torch.cuda.synchronize()
            assert flag.item() == 0
            ki, nk = keep_idx.cpu().numpy(), n_keep.cpu().numpy()
            for b in range(batch):
                c = cand[b, :n_cand[b]].tolist()
                k = min(keep, len(c))
                ref = orc.prune_topk(score[b], lens[b] if use_len else None, c, k)
                assert nk[b] == k
                assert ki[b, :k].tolist() == ref
                assert np.all(ki[b, k:] == -1)


def test_prune_topk_flags():
    score = torch.tensor([[1.0, float("nan"), 2.0, 0.5]], device="cuda")
    cand = torch.arange(4, **I32).reshape(1, 4)
    n_cand = torch.tensor([4], **I32)
    keep_idx = torch.full((1, 4), -1, **I32)
    n_keep = torch.full((1,), 9, **I32)
    flag = torch.zeros(1, **I32)
    cf.cf_prune_topk(score, None, cand, n_cand, 2, 1, 4, keep_idx, n_keep, flag)
    torch.cuda.synchronize()
    assert flag.item() == cf.CF_FLAG_NONFINITE_SCORE and n_keep.item() == 0
    flag.zero_()
    cand[0, 1] = 77
    cf.cf_prune_topk(torch.ones(1, 4, device="cuda"), None, cand, n_cand, 2, 1, 4, keep_idx, n_keep, flag)
    torch.cuda.synchronize()
    assert flag.item() == cf.CF_FLAG_BAD_INDEX and n_keep.item() == 0


# ----------------------------------------------------------------------------- cf_assign_positions
@pytest.mark.parametrize("strategy", [cf.CF_ALLOC_SORT, cf.CF_ALLOC_ALIGN])
def test_assign_positions_bit_exact(strategy):
    rng = np.random.default_rng(41)
    batch, stride = 64, 40
    lens = rng.integers(1, 201, size=(batch, stride)).astype(np.int32)
    n_ranked = rng.integers(0, stride + 1, size=batch).astype(np.int32)
    ranked = np.stack([rng.permutation(stride) for _ in range(batch)]).astype(np.int32)
    for pos_begin, pos_end, force in [(32, 4048, 0), (0, 32704, 0), (32, 900, 0), (32, 4048, 5), (7, 300, 0),
                                      (0, 150, 0)]:
        new_start = torch.full((batch, stride), -7, **I32)
        q_start = torch.full((batch,), -7, **I32)
        n_reuse = torch.full((batch,), -7, **I32)
        order = torch.full((batch, stride), -7, **I32)
        flag = torch.zeros(1, **I32)
        cf.cf_assign_positions(torch.from_numpy(lens).cuda(), torch.from_numpy(ranked).cuda(),
                               torch.from_numpy(n_ranked).cuda(), batch, stride, pos_begin, pos_end, strategy,
                               force, new_start, q_start, n_reuse, order, flag)
        torch.cuda.synchronize()
        ns, qs, nr, od = (x.cpu().numpy() for x in (new_start, q_start, n_reuse, order))
        expect_flag = 0
        for b in range(batch):
            r = ranked[b, :n_ranked[b]].tolist()
            try:
                ref_ns, ref_q, ref_nr = orc.assign_positions(lens[b], r, pos_begin, pos_end, strategy, force)
            except ValueError as e:
                expect_flag |= cf.CF_FLAG_DOC_TOO_LONG if "longer" in str(e) else cf.CF_FLAG_POS_OVERFLOW
                assert qs[b] == -7 and np.all(ns[b] == -7)          # untouched
                continue
            assert qs[b] == ref_q and nr[b] == ref_nr
            for slot in range(stride):
                assert ns[b, slot] == ref_ns.get(slot, -7)
            ref_order = sorted(r) if strategy == cf.CF_ALLOC_ALIGN else r
            assert od[b, :len(r)].tolist() == ref_order
        assert flag.item() == expect_flag


def test_assign_keep_only_lists_survivors():
    lens = torch.full((1, 6), 10, **I32)
    ranked = torch.tensor([[4, 1, 3, 0, 0, 0]], **I32)
    new_start = torch.full((1, 6), 5, **I32)
    q_start = torch.full((1,), 99, **I32)
    n_reuse = torch.full((1,), 1, **I32)
    order = torch.zeros((1, 6), **I32)
    cf.cf_assign_positions(lens, ranked, torch.tensor([3], **I32), 1, 6, 0, 100, cf.CF_ALLOC_KEEP, 0, new_start,
                           q_start, n_reuse, order)
    torch.cuda.synchronize()
    assert order[0, :3].tolist() == [1, 3, 4]
    assert q_start.item() == 99 and torch.all(new_start == 5)


# ----------------------------------------------------------------------------- generic attention path
def _run_single_layer(cfg, pairing=cf.CF_ROPE_HALF, seed=None, mass_tol=None, layout="token"):
    """Masses are checked twice.  Against the rounded-key reference (the oracle on keys moved by Eq. 5 and
    rounded once to the storage type, as the fused kernels hold them) the bound is always the tight one,
    1e-4 for 16-bit types: what is left there is the kernels' own arithmetic.  Against the plain oracle
    ``mass_tol`` may loosen the bound for shapes with so few rows and tokens that the one rounding of a
    moved key (2^-9 relative per element) is not averaged away."""
    st = wl.build_structure(cfg, seed=None if seed is None else 7000 + seed)
    t = wl.build_layer(cfg, st, seed=seed)
    g = cfg.geometry
    pname = "half" if pairing == cf.CF_ROPE_HALF else "interleaved"
    pb = G.make_batch(cfg, st, pairing, layout)
    dev = G.upload_layer(cfg, t, layout)
    out = torch.empty_like(dev["q"])
    pb.allocate_initial()
    pb.workspace.fill_(0xFF)          # the workspace is scratch: stale contents (here NaN patterns) must not matter
    pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out)
    torch.cuda.synchronize()
    assert pb.flags() == 0
    out_np = out.float().cpu().numpy()
    mass_np = pb.mass.cpu().numpy()
    score_np = pb.score.cpu().numpy()
    worst_out = worst_mass = worst_near = 0.0
    loosened = mass_tol is not None
    mass_tol = G.MASS_TOL[g.dtype] if mass_tol is None else mass_tol
    for b in range(cfg.batch):
        # positions and segment table: bit-exact against the oracle's own allocation
        ref_segs, ref_q, _ = H.initial_segments(cfg, st, b)
        segs = G.device_segments(pb, b)
        assert segs == ref_segs and int(pb.q_start[b].item()) == ref_q
        ref_out, ref_mass = H.oracle_query(cfg, st, t, b, ref_segs, ref_q, pairing=pname)
        worst_out = max(worst_out, G.row_error(out_np[b * cfg.tq:(b + 1) * cfg.tq], ref_out))
        worst_mass = max(worst_mass, G.rel_error(mass_np[b, :len(segs)], ref_mass))
        ref_score = H.doc_scores(ref_segs, ref_mass, cfg.docs_per_query)
        assert G.rel_error(score_np[b], ref_score) <= mass_tol
        assert mass_np[b, :len(segs)].sum() == pytest.approx(g.n_q_heads * cfg.tq, rel=1e-5)
        rows = t["q"][b * cfg.tq:(b + 1) * cfg.tq]
        _, near_mass = H.rounded_key_reference(g.dtype, rows, 0, ref_q, t["k_store"], t["v_store"], t["k_self"], t["v_self"],
                                               ref_segs, g.n_kv_heads, g.rope_base, pname)
        worst_near = max(worst_near, G.rel_error(mass_np[b, :len(segs)], near_mass))
    _say(f"{cfg.name} [{layout}]: out err {worst_out:.3e}  mass err {worst_mass:.3e}  against rounded moved keys {worst_near:.3e}")
    assert worst_out <= G.OUT_TOL[g.dtype]
    if G.rounds_moved_keys(g, pairing, pb.seg_stride):
        assert worst_mass <= mass_tol
        assert worst_near <= (G.NEAR_MASS_TOL if loosened else G.MASS_TOL)[g.dtype]
    else:
        assert worst_mass <= G.MASS_TOL[g.dtype]            # keys moved in fp32, nothing rounded: the plain oracle is the reference
    return cfg, st, t, pb, dev, out


def test_tiny_fp32_configuration_end_to_end():
    """Configuration 1: attention, mass, keep top-2, re-pack after the 4-token prefix."""
    cfg, st, t, pb, dev, out = _run_single_layer(wl.CONFIGS["tiny_f32"])
    # prune with the oracle's own scores fed to the device: indices must match exactly
    ref_segs, ref_q, lens = H.initial_segments(cfg, st, 0)
    _, ref_mass = H.oracle_query(cfg, st, t, 0, ref_segs, ref_q)
    ref_score = H.doc_scores(ref_segs, ref_mass, cfg.docs_per_query).astype(np.float32)
    ref_keep = orc.prune_topk(ref_score, lens, list(range(4)), cfg.keep)
    pb.score.copy_(torch.from_numpy(ref_score).reshape(1, -1))
    pb.prune(cfg.keep, cf.CF_ALLOC_SORT)
    pb.advance()
    torch.cuda.synchronize()
    assert pb.flags() == 0
    assert pb.keep_idx[0, :cfg.keep].tolist() == ref_keep
    assert set(st.planted[0].tolist()) <= set(ref_keep)
    ref_ns, ref_qs, ref_nr = orc.assign_positions(lens, ref_keep, cfg.prefix_len, cfg.geometry.max_positions - cfg.tq)
    assert pb.q_start.item() == ref_qs == 68
    ns = pb.new_start.cpu().numpy()[0]
    for slot, pos in ref_ns.items():
        assert ns[slot] == pos
    assert sorted(ref_ns.values()) == [4, 36]
    segs = G.device_segments(pb, 0)
    assert [s.kind for s in segs] == [cf.CF_SEG_PREFIX, cf.CF_SEG_DOC, cf.CF_SEG_DOC, cf.CF_SEG_SELF]
    assert [s.doc for s in segs[1:3]] == ref_keep
    # second layer on the pruned, re-packed set
    pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, accumulate=False)
    torch.cuda.synchronize()
    _, ref_out, ref_mass2 = G.oracle_on_device_segments(cfg, t, pb, 0)
    assert G.row_error(out.float().cpu().numpy(), ref_out) <= 1e-4
    assert G.rel_error(pb.mass.cpu().numpy()[0, :4], ref_mass2) <= 1e-5


@pytest.mark.parametrize("layout", ["token", "head_padded"])
@pytest.mark.parametrize("dtype,pairing,d,hq,hkv", [("f32", cf.CF_ROPE_INTERLEAVED, 64, 4, 2),
                                                    ("bf16", cf.CF_ROPE_INTERLEAVED, 128, 8, 2),
                                                    ("f16", cf.CF_ROPE_HALF, 64, 6, 3),
                                                    ("f32", cf.CF_ROPE_HALF, 256, 2, 1)])
def test_generic_path_shapes(dtype, pairing, d, hq, hkv, layout):
    base = wl.CONFIGS["tiny_f32"]
    cfg = wl.scaled(base, name=f"generic_{dtype}_{d}", geometry=wl.Geometry(hq, hkv, d, dtype, 1.0e6, 32768),
                    n_store_docs=12, docs_per_query=4, batch=3, doc_len_range=(1, 150), tq=11, prefix_len=5,
                    doc_stored_start=5, n_planted=1)
    _run_single_layer(cfg, pairing, seed=55, layout=layout)


def test_attention_flags_bad_table_entries():
    cfg = wl.CONFIGS["tiny_f32"]
    st = wl.build_structure(cfg)
    t = wl.build_layer(cfg, st)
    pb = G.make_batch(cfg, st)
    dev = G.upload_layer(cfg, t)
    out = torch.empty_like(dev["q"])
    pb.allocate_initial()
    segs = cf.segments_from_device(pb.segs[0], 6)
    segs[2]["tok_offset"] = 10 ** 9          # far outside the store: must be skipped, not read
    segs[3]["len"] = -5
    pb.segs[0].copy_(cf.segments_to_device(segs).reshape(6, 32))
    pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out)
    torch.cuda.synchronize()
    assert pb.flags() & cf.CF_FLAG_BAD_SEGMENT
    mass = pb.mass.cpu().numpy()[0]
    assert mass[2] == 0 and mass[3] == 0
    assert mass[:6].sum() == pytest.approx(cfg.geometry.n_q_heads * cfg.tq, rel=1e-5)


# ----------------------------------------------------------------------------- 16-bit MFMA path
def _cut_against_oracle(cfg, st, t, pb, dev, out):
    """The prune event of a configuration on the scores the device accumulated: exact for those scores, and against
    the cut the oracle takes on its own scores by the margin rule (equal sets where the oracle's gap at the cut is at
    least 1e-3, as for the LLaMA-2-7B layer's seed; with 45 unplanted documents of the Qwen2-7B layer the gap is
    ~1e-4 whatever the seed, and only documents within 1e-3 of the cut may fall either way); planted documents
    kept; the survivors' positions those of the oracle's allocator."""
    g = cfg.geometry
    pb.prune(cfg.keep, cf.CF_ALLOC_SORT)
    torch.cuda.synchronize()
    assert pb.flags() == 0
    for b in range(cfg.batch):
        ref_segs, ref_q, lens = H.initial_segments(cfg, st, b)
        _, ref_mass = H.oracle_query(cfg, st, t, b, ref_segs, ref_q)
        ref_score = H.doc_scores(ref_segs, ref_mass, cfg.docs_per_query)
        alive = list(range(cfg.docs_per_query))
        kept = pb.keep_idx[b, :cfg.keep].tolist()
        assert kept == orc.prune_topk(pb.score.cpu().numpy()[b], lens, alive, cfg.keep)
        gap = H.check_cut(kept, ref_score, lens, alive, cfg.keep, st.planted[b])
        _say(f"  {cfg.name}: oracle gap at the cut {gap:.2e}")
        if cfg.name == "llama2_7b_layer":
            assert gap >= 1e-3 and sorted(kept) == sorted(orc.prune_topk(ref_score, lens, alive, cfg.keep))
        ref_ns, ref_qs, ref_nr = orc.assign_positions(lens, kept, cfg.prefix_len, g.max_positions - cfg.tq)
        assert int(pb.next_q_start[b].item()) == ref_qs and int(pb.n_reuse[b].item()) == ref_nr
        ns = pb.next_new_start.cpu().numpy()[b]
        assert all(int(ns[s]) == p for s, p in ref_ns.items())


@pytest.mark.parametrize("layout", ["token", "head"])
def test_llama2_7b_layer_configuration(layout):
    """Configuration 2 (MHA, bf16, HBM-bound shape) at full size; head-major is the layout bench.py times."""
    _cut_against_oracle(*_run_single_layer(wl.CONFIGS["llama2_7b_layer"], layout=layout))


@pytest.mark.parametrize("layout", ["token", "head"])
def test_qwen2_7b_layer_configuration(layout):
    """Configuration 3 (GQA 28/4, bf16, 50 ragged documents) at full size."""
    _cut_against_oracle(*_run_single_layer(wl.CONFIGS["qwen2_7b_layer"], layout=layout))


def test_qwen2_1p5b_batch_reduced():
    """Configuration 5's shape (fp16 GQA 12/2, ragged documents, batch of queries over a shared
    store) with a smaller store and batch so the oracle finishes in seconds."""
    cfg = wl.scaled(wl.CONFIGS["qwen2_1p5b_batch"], n_store_docs=300, batch=6)
    _run_single_layer(cfg)


@pytest.mark.parametrize("dtype,layout", [("bf16", "token"), ("f16", "token"), ("bf16", "head_padded")])
@pytest.mark.parametrize("hq,hkv,tq,docs,len_range,prefix", [
    (4, 4, 1, 3, (1, 70), 0),          # single query row, no prefix
    (8, 2, 5, 1, (33, 33), 7),         # one document, ragged everything
    (6, 2, 17, 9, (1, 40), 3),         # stacked rows straddle the 64-row tile
    (2, 2, 70, 4, (90, 130), 16),      # more rows than one tile in MHA
    (14, 2, 13, 6, (1, 150), 5),       # GQA, six row blocks: the producer/consumer kernel with idle math wavefronts
    (12, 2, 40, 5, (20, 90), 0),       # GQA, fifteen row blocks: two row groups of unequal size, no prefix
])
def test_mfma_path_edge_shapes(dtype, layout, hq, hkv, tq, docs, len_range, prefix):
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name=f"edge_{dtype}_{hq}_{hkv}_{tq}",
                    geometry=wl.Geometry(hq, hkv, 128, dtype, 1.0e6, 32768), n_store_docs=2 * docs,
                    docs_per_query=docs, batch=2, doc_len_range=len_range, tq=tq, prefix_len=prefix,
                    doc_stored_start=prefix, n_planted=1)
    _run_single_layer(cfg, seed=77, mass_tol=2e-3, layout=layout)


@pytest.mark.parametrize("dtype,layout", [("bf16", "token"), ("f16", "head"), ("bf16", "head_padded")])
@pytest.mark.parametrize("hq,hkv,tq,docs,len_range,prefix,batch", [
    (4, 4, 1, 3, (1, 70), 0, 2),            # one row per kv head, no prefix
    (32, 32, 1, 10, (160, 160), 32, 1),     # a decode step of the LLaMA-2-7B shape: several splits
    (8, 4, 1, 5, (20, 90), 3, 2),           # GQA group of two
    (4, 4, 2, 4, (5, 64), 2, 3),            # two query tokens: the causal own block
    (6, 2, 1, 6, (1, 150), 5, 2),           # group of three: one padding row in the four-row instance
    (2, 2, 4, 3, (33, 33), 7, 2),           # four query tokens
    (4, 2, 2, 7, (1, 100), 0, 2),           # group of two times two tokens
    (4, 4, 1, 2, (10, 40), 4, 70),          # many queries: a single split, rows written by the attention kernel
])
def test_few_rows_outputs_only(dtype, layout, hq, hkv, tq, docs, len_range, prefix, batch):
    """Outputs-only calls (no mass buffer) with at most four stacked rows per kv head, the shape of decode steps:
    checked against the oracle on re-positioned tables (documents moved from where they were cached), and
    against the same call with masses."""
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name=f"fewrow_{dtype}_{hq}_{hkv}_{tq}_{batch}",
                    geometry=wl.Geometry(hq, hkv, 128, dtype, 1.0e4, 8192), n_store_docs=batch * docs,
                    docs_per_query=docs, batch=batch, doc_len_range=len_range, tq=tq, prefix_len=prefix,
                    doc_stored_start=prefix + 11, n_planted=1)
    _say(f"few rows {cfg.name} [{layout}]")
    g = cfg.geometry
    st = wl.build_structure(cfg, seed=7090)
    t = wl.build_layer(cfg, st, seed=91)
    pb = G.make_batch(cfg, st, layout=layout)
    dev = G.upload_layer(cfg, t, layout)
    pb.allocate_initial()
    pb.workspace.fill_(0xFF)
    out = torch.full_like(dev["q"], 7.0)
    cf.cf_prefill_attention(pb.desc, dev["q"], pb.q_off, pb.q_stored_start, pb.q_start, dev["k_store"], dev["v_store"],
                            pb.n_store_tokens, dev["k_self"], dev["v_self"], pb.segs, pb.n_seg, pb.seg_stride, pb.batch, pb.tq,
                            pb.max_kv_tokens, out, None, None, pb.stride, pb.workspace, pb.ws_bytes, pb.dev_flag)
    torch.cuda.synchronize()
    assert pb.flags() == 0
    with_mass = torch.empty_like(out)
    pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], with_mass, accumulate=False)
    torch.cuda.synchronize()
    out_np, other = out.float().cpu().numpy(), with_mass.float().cpu().numpy()
    worst = 0.0
    for b in range(min(cfg.batch, 6)):
        segs, q_start, _ = H.initial_segments(cfg, st, b)
        assert any(sg.new_start != sg.stored_start for sg in segs if sg.kind == cf.CF_SEG_DOC)
        ref_out, _ = H.oracle_query(cfg, st, t, b, segs, q_start)
        worst = max(worst, G.row_error(out_np[b * cfg.tq:(b + 1) * cfg.tq], ref_out))
    _say(f"  out err {worst:.3e}")
    assert worst <= G.OUT_TOL[g.dtype]
    assert G.row_error(out_np, other) <= G.OUT_TOL[g.dtype]


def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        hkv = int(rng.choice([1, 2, 3, 4, 8]))
        group = int(rng.choice([1, 1, 2, 4, 7]))
        tq = int(rng.choice([1, 2, 3, 8, 16, 17, 31, 48, 64, 70]))
        docs = int(rng.integers(1, 13))
        lo = int(rng.integers(1, 60))
        hi = lo + int(rng.integers(0, 120))
        prefix = int(rng.choice([0, 0, 1, 7, 32, 33]))
        batch = int(rng.choice([1, 2, 3, 5]))
        dtype = str(rng.choice(["bf16", "f16"]))
        layout = str(rng.choice(["token", "head", "head_padded"]))
        shapes.append((dtype, layout, hkv * group, hkv, tq, docs, (lo, hi), prefix, batch))
    return shapes


@pytest.mark.parametrize("dtype,layout,hq,hkv,tq,docs,len_range,prefix,batch", _random_shapes(24, 20250211))
def test_mfma_path_seeded_random_shapes(dtype, layout, hq, hkv, tq, docs, len_range, prefix, batch):
    """A seeded sweep over head counts, group sizes, query lengths, document counts and lengths, prefixes, batches,
    dtypes and store layouts: outputs, masses, accumulated scores and tables against the oracle (both 16-bit
    attention kernels, single-split and multi-split plans, ragged tiles, one-token documents)."""
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name=f"rand_{dtype}_{hq}_{hkv}_{tq}_{docs}_{batch}",
                    geometry=wl.Geometry(hq, hkv, 128, dtype, 1.0e6, 32768), n_store_docs=batch * docs + 3,
                    docs_per_query=docs, batch=batch, doc_len_range=len_range, tq=tq, prefix_len=prefix,
                    doc_stored_start=prefix + 5, n_planted=1)
    _run_single_layer(cfg, seed=int(hq * 131 + tq * 17 + docs), mass_tol=4e-3, layout=layout)


@pytest.mark.parametrize("docs,fused", [(254, False), (300, False), (300, True)])
def test_more_segments_than_the_16_bit_kernels_hold(docs, fused):
    """254 documents fill the 256-entry segment table of the 16-bit kernels exactly; 300 do not fit and the call
    takes the generic kernel (and, fused, the stand-alone prune kernels) — same results either way."""
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name=f"segs_{docs}", geometry=wl.Geometry(4, 2, 128, "bf16", 1.0e4, 8192),
                    n_store_docs=docs, docs_per_query=docs, batch=1, doc_len_range=(1, 9), tq=3, prefix_len=2,
                    doc_stored_start=2, n_planted=3)
    if not fused:
        _run_single_layer(cfg, seed=55, mass_tol=4e-3)
        return
    st = wl.build_structure(cfg, seed=7055)
    a, b = _fused_and_separate(cfg, st, wl.build_layer(cfg, st, seed=55), 40, cf.CF_ALLOC_SORT)
    assert a["flags"] == 0 and b["flags"] == 0
    assert torch.equal(a["out"], b["out"]) and torch.equal(a["score"], b["score"])
    assert torch.equal(a["keep"][:, :40], b["keep"][:, :40]) and torch.equal(a["segs"][:, :42], b["segs"][:, :42])
    ref = orc.prune_topk(b["score"][0].cpu().numpy(), st.doc_lens[st.query_docs[0]], list(range(docs)), 40)
    assert b["keep"][0, :40].tolist() == ref


def test_mfma_path_is_deterministic():
    cfg = wl.CONFIGS["llama2_7b_layer"]
    st = wl.build_structure(cfg)
    dev = G.upload_layer(cfg, wl.build_layer(cfg, st))
    pb = G.make_batch(cfg, st)
    pb.allocate_initial()
    outs, masses = [], []
    for _ in range(3):
        out = torch.empty_like(dev["q"])
        pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, accumulate=False)
        torch.cuda.synchronize()
        outs.append(out.clone())
        masses.append(pb.mass.clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    assert torch.equal(masses[0], masses[1]) and torch.equal(masses[0], masses[2])


def test_kernel_timing_aid_counts_launches_and_leaves_results_alone():
    """cf_profile_kernel_events / cf_profile_kernel_ms: one bracketed launch per call of the 16-bit path, a positive
    mean duration, an error when timing is off, and outputs identical to an untimed call."""
    cfg = wl.CONFIGS["llama2_7b_layer"]
    st = wl.build_structure(cfg)
    dev = G.upload_layer(cfg, wl.build_layer(cfg, st))
    pb = G.make_batch(cfg, st)
    pb.allocate_initial()
    ref = torch.empty_like(dev["q"])
    pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], ref, accumulate=False)
    torch.cuda.synchronize()
    with pytest.raises(cf.CacheFocusError):
        cf.cf_profile_kernel_ms()
    cf.cf_profile_kernel_events(True)
    try:
        assert cf.cf_profile_kernel_ms() == (0.0, 0)
        out = torch.empty_like(dev["q"])
        for _ in range(3):
            pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, accumulate=False)
        mean_ms, n = cf.cf_profile_kernel_ms()
        assert n == 3 and 0.0 < mean_ms < 5.0
        assert torch.equal(out, ref)
    finally:
        cf.cf_profile_kernel_events(False)
    with pytest.raises(cf.CacheFocusError):
        cf.cf_profile_kernel_ms()


# ----------------------------------------------------------------------------- fused layer call
@pytest.mark.parametrize("name", ["tiny_f32", "llama2_7b_layer", "qwen2_7b_layer"])
@pytest.mark.parametrize("strategy", [cf.CF_ALLOC_SORT, cf.CF_ALLOC_ALIGN, cf.CF_ALLOC_KEEP])
def test_fused_layer_equals_separate_calls(name, strategy):
    """cf_prefill_layer = cf_prefill_attention + cf_prune_topk + cf_assign_positions + cf_gather_segments."""
    cfg = wl.CONFIGS[name]
    st = wl.build_structure(cfg)
    t = wl.build_layer(cfg, st)
    dev = G.upload_layer(cfg, t)
    g = cfg.geometry
    res = []
    for fused in (False, True):
        pb = G.make_batch(cfg, st)
        out = torch.empty_like(dev["q"])
        pb.allocate_initial()
        if fused:
            pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, keep=cfg.keep,
                     strategy=strategy)
        else:
            pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out)
            pb.prune(cfg.keep, strategy)
        torch.cuda.synchronize()
        assert pb.flags() == 0
        score = pb.score.cpu().numpy()
        lens = st.doc_lens[st.query_docs[0]]
        # the ranking must be exact for the scores this path itself produced
        ref_keep = orc.prune_topk(score[0], lens, list(range(cfg.docs_per_query)), cfg.keep)
        assert pb.keep_idx[0, :cfg.keep].tolist() == ref_keep
        pb.advance()
        res.append(dict(out=out.clone(), mass=pb.mass.cpu().numpy().copy(), score=score,
                        segs=G.device_segments(pb, 0), q_start=int(pb.q_start[0].item()),
                        cand=pb.cand[0, :cfg.keep].tolist()))
    a, b = res
    assert torch.equal(a["out"], b["out"])
    n = cfg.docs_per_query + 2
    assert G.rel_error(b["mass"][0, :n], a["mass"][0, :n]) < 2e-6
    assert a["segs"] == b["segs"] and a["q_start"] == b["q_start"] and a["cand"] == b["cand"]
    if strategy != cf.CF_ALLOC_KEEP:
        lens = [int(x) for x in st.doc_lens[st.query_docs[0]]]
        ref_ns, ref_q, _ = orc.assign_positions(lens, a["cand"] if strategy == cf.CF_ALLOC_SORT else sorted(a["cand"]),
                                                cfg.prefix_len, g.max_positions - cfg.tq, cf.CF_ALLOC_SORT)
        assert b["q_start"] == ref_q
        assert {s.doc: s.new_start for s in b["segs"] if s.kind == cf.CF_SEG_DOC} == ref_ns


def _fused_and_separate(cfg, st, t, keep, strategy, **kw):
    dev = G.upload_layer(cfg, t)
    res = []
    for fused in (False, True):
        pb = G.make_batch(cfg, st)
        out = torch.empty_like(dev["q"])
        pb.allocate_initial()
        for name, val in kw.items():                     # changes that apply to the prune step only
            setattr(pb, name, val)
        if fused:
            pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, keep=keep, strategy=strategy)
        else:
            pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out)
            pb.prune(keep, strategy)
        torch.cuda.synchronize()
        res.append(dict(flags=pb.flags(), out=out.clone(), score=pb.score.clone(), mass=pb.mass.clone(), keep=pb.keep_idx.clone(),
                        n_keep=pb.n_keep.clone(),
                        order=pb.order.clone(), new_start=pb.next_new_start.clone(), q_start=pb.next_q_start.clone(),
                        n_reuse=pb.n_reuse.clone(), segs=pb.next_segs.clone(), n_seg=pb.next_n_seg.clone()))
    return res


@pytest.mark.parametrize("strategy", [cf.CF_ALLOC_SORT, cf.CF_ALLOC_ALIGN])
def test_fused_layer_many_candidates_and_batch(strategy):
    """More than 64 candidates per query (the ranking runs on the whole workgroup) and a batch of queries:
    the fused call and the separate calls leave identical tables."""
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name="many_docs", geometry=wl.Geometry(4, 2, 128, "bf16", 1.0e4, 8192),
                    n_store_docs=220, docs_per_query=70, batch=3, doc_len_range=(5, 40), tq=9, prefix_len=6,
                    doc_stored_start=6, n_planted=2)
    st = wl.build_structure(cfg, seed=7101)
    a, b = _fused_and_separate(cfg, st, wl.build_layer(cfg, st, seed=31), 23, strategy)
    assert a["flags"] == 0 and b["flags"] == 0
    assert torch.equal(a["out"], b["out"]) and torch.equal(a["n_keep"], b["n_keep"]) and a["n_keep"].tolist() == [23] * 3
    for q in range(3):
        assert a["keep"][q, :23].tolist() == b["keep"][q, :23].tolist()
        assert a["order"][q, :23].tolist() == b["order"][q, :23].tolist()
        ref = orc.prune_topk(b["score"][q].cpu().numpy(), st.doc_lens[st.query_docs[q]], list(range(70)), 23)
        assert b["keep"][q, :23].tolist() == ref
    for key in ("new_start", "q_start", "n_reuse", "n_seg"):
        assert torch.equal(a[key], b[key]), key
    n = int(a["n_seg"][0].item())
    assert torch.equal(a["segs"][:, :n], b["segs"][:, :n])


@pytest.mark.parametrize("case", range(12))
def test_fused_layer_seeded_random_prunes(case):
    """A seeded sweep of prune events through cf_prefill_layer: random geometry, candidate count, keep and
    strategy; the cut must be exact for the scores the device accumulated, the allocation and the next table
    bit-exact against the oracle's allocator."""
    rng = np.random.default_rng(4100 + case)
    hkv = int(rng.choice([1, 2, 4, 8]))
    group = int(rng.choice([1, 2, 7]))
    tq = int(rng.choice([1, 5, 16, 48]))
    docs = int(rng.integers(2, 40))
    keep = int(rng.integers(1, docs + 1))
    lo = int(rng.integers(1, 50))
    hi = lo + int(rng.integers(0, 60))
    prefix = int(rng.choice([0, 3, 32]))
    batch = int(rng.choice([1, 2, 4]))
    strategy = int(rng.choice([cf.CF_ALLOC_SORT, cf.CF_ALLOC_ALIGN]))
    dtype = str(rng.choice(["bf16", "f16"]))
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name=f"randprune_{case}", geometry=wl.Geometry(hkv * group, hkv, 128, dtype, 1.0e4, 8192),
                    n_store_docs=batch * docs, docs_per_query=docs, batch=batch, doc_len_range=(lo, hi), tq=tq,
                    prefix_len=prefix, doc_stored_start=prefix, n_planted=1)
    _say(f"random prune {case}: {dtype} {hkv * group}/{hkv} heads, tq {tq}, {docs} documents keep {keep}, batch {batch}, strategy {strategy}")
    g = cfg.geometry
    st = wl.build_structure(cfg, seed=7200 + case)
    t = wl.build_layer(cfg, st, seed=300 + case)
    pb = G.make_batch(cfg, st, layout="head")
    dev = G.upload_layer(cfg, t, "head")
    out = torch.empty_like(dev["q"])
    pb.allocate_initial()
    pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, keep=keep, strategy=strategy)
    torch.cuda.synchronize()
    assert pb.flags() == 0
    score = pb.score.cpu().numpy()
    pb.advance()
    for b in range(batch):
        lens = [int(x) for x in st.doc_lens[st.query_docs[b]]]
        kept = pb.cand[b, :keep].tolist() if strategy == cf.CF_ALLOC_SORT else None
        ranked = orc.prune_topk(score[b], lens, list(range(docs)), keep)
        assert int(pb.n_cand[b].item()) == keep
        assert sorted(pb.cand[b, :keep].tolist()) == sorted(ranked)
        if kept is not None:
            assert kept == ranked
        order = ranked if strategy == cf.CF_ALLOC_SORT else sorted(ranked)
        ref_ns, ref_q, ref_nr = orc.assign_positions(lens, order, cfg.prefix_len, g.max_positions - cfg.tq)
        assert int(pb.q_start[b].item()) == ref_q and int(pb.n_reuse[b].item()) == ref_nr
        assert {sg.doc: sg.new_start for sg in G.device_segments(pb, b) if sg.kind == cf.CF_SEG_DOC} == ref_ns
        segs = G.device_segments(pb, b)
        assert len(segs) == keep + (1 if prefix else 0) + 1 and segs[-1].kind == cf.CF_SEG_SELF and segs[-1].new_start == ref_q


def test_mass_reduction_forms_add_in_the_same_order():
    """Many kv heads: the separate call's mass kernel stages the slot partials through LDS in rounds, the fused
    epilogue's single wavefront reads them all at once; both must add in the same order — masses and accumulated
    scores bit for bit, and so the same survivors."""
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name="many_heads", geometry=wl.Geometry(80, 80, 128, "bf16", 1.0e4, 8192),
                    n_store_docs=100, docs_per_query=50, batch=2, doc_len_range=(5, 30), tq=3, prefix_len=6,
                    doc_stored_start=6, n_planted=2)
    st = wl.build_structure(cfg, seed=7102)
    a, b = _fused_and_separate(cfg, st, wl.build_layer(cfg, st, seed=32), 20, cf.CF_ALLOC_SORT)
    assert a["flags"] == 0 and b["flags"] == 0
    assert torch.equal(a["out"], b["out"]) and torch.equal(a["mass"], b["mass"]) and torch.equal(a["score"], b["score"])
    assert torch.equal(a["keep"][:, :20], b["keep"][:, :20]) and torch.equal(a["segs"][:, :22], b["segs"][:, :22])
    assert float(a["mass"][0, :52].sum()) == pytest.approx(80 * 3, rel=1e-5)


def test_fused_layer_too_large_for_the_epilogue_kernel():
    """128 kv heads times 120 documents: the slot partials of a query do not fit the fused epilogue's LDS, so the
    fused call falls back to the mass kernel and the stand-alone prune kernels; same tables as the separate calls."""
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name="big_epilogue", geometry=wl.Geometry(128, 128, 128, "bf16", 1.0e4, 8192),
                    n_store_docs=120, docs_per_query=120, batch=1, doc_len_range=(2, 12), tq=2, prefix_len=3,
                    doc_stored_start=3, n_planted=2)
    st = wl.build_structure(cfg, seed=7103)
    a, b = _fused_and_separate(cfg, st, wl.build_layer(cfg, st, seed=33), 30, cf.CF_ALLOC_SORT)
    assert a["flags"] == 0 and b["flags"] == 0
    assert torch.equal(a["out"], b["out"]) and torch.equal(a["mass"], b["mass"]) and torch.equal(a["score"], b["score"])
    assert torch.equal(a["keep"][:, :30], b["keep"][:, :30]) and torch.equal(a["segs"][:, :32], b["segs"][:, :32])
    ref = orc.prune_topk(b["score"][0].cpu().numpy(), st.doc_lens[st.query_docs[0]], list(range(120)), 30)
    assert b["keep"][0, :30].tolist() == ref
    assert float(a["mass"][0, :122].sum()) == pytest.approx(128 * 2, rel=1e-5)
    # (44 bytes per document row + 4 bytes per (kv head, slot) partial: 5280 + 4 * 128 * 126 = 69 792 > 60 KB)


def test_fused_layer_flags_like_the_separate_calls():
    """A positional range too short for the longest survivor: both paths raise the same flag and leave the
    positions and the placement order as they were."""
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name="no_room", geometry=wl.Geometry(4, 4, 128, "bf16", 1.0e4, 4096),
                    n_store_docs=14, docs_per_query=6, batch=2, doc_len_range=(40, 60), tq=8, prefix_len=4,
                    doc_stored_start=4, n_planted=1)
    st = wl.build_structure(cfg, seed=7102)
    t = wl.build_layer(cfg, st, seed=32)
    a, b = _fused_and_separate(cfg, st, t, 3, cf.CF_ALLOC_SORT)
    assert a["flags"] == 0 and b["flags"] == 0 and torch.equal(a["segs"], b["segs"])
    # shrink the range handed to the allocator below one document
    a, b = _fused_and_separate(cfg, st, t, 3, cf.CF_ALLOC_SORT, pos_end=4 + 30)
    assert a["flags"] == b["flags"] == cf.CF_FLAG_DOC_TOO_LONG
    for key in ("keep", "n_keep", "new_start", "q_start", "order"):
        assert torch.equal(a[key], b[key]), key


def test_layer_stack_with_pruning_matches_oracle():
    """A reduced layer stack in the LLaMA-2-7B geometry (the full one is 32 layers x 30 documents):
    Alg. 2, Phase 1 on the GPU through cf_prefill_layer, checked against the oracle layer by layer on
    the state the device holds.  Every cut must be exact for the scores the device accumulated, and
    must agree with the oracle's own scores wherever those are not within 1e-3 of the cut (documents
    closer than that to the boundary may legitimately fall either way in 16-bit arithmetic)."""
    base = wl.CONFIGS["llama2_7b_stack"]
    cfg = wl.scaled(base, n_store_docs=12, docs_per_query=12, n_planted=2, n_layers=6, prune_layers=(1, 3, 5))
    g = cfg.geometry
    st = wl.build_structure(cfg, seed=9100)
    lens = [int(x) for x in st.doc_lens]
    keeps, k = {}, cfg.docs_per_query
    for layer in cfg.prune_layers:
        k = orc.keep_fraction(k, cfg.keep_frac)
        keeps[layer] = k
    assert list(keeps.values()) == [8, 5, 3]
    pb = G.make_batch(cfg, st)
    pb.allocate_initial()
    ref_score = np.zeros(cfg.docs_per_query)
    alive = list(range(cfg.docs_per_query))
    for layer in range(cfg.n_layers):
        t = wl.build_layer(cfg, st, layer, seed=910000 + layer)
        dev = G.upload_layer(cfg, t)
        out = torch.empty_like(dev["q"])
        segs, ref_out, ref_mass = G.oracle_on_device_segments(cfg, t, pb, 0)
        assert sorted(s.doc for s in segs if s.kind == cf.CF_SEG_DOC) == sorted(alive)
        pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, keep=keeps.get(layer),
                 strategy=cf.CF_ALLOC_SORT)
        torch.cuda.synchronize()
        assert pb.flags() == 0
        assert G.row_error(out.float().cpu().numpy(), ref_out) <= G.OUT_TOL[g.dtype]
        assert G.rel_error(pb.mass.cpu().numpy()[0, :len(segs)], ref_mass) <= G.MASS_TOL[g.dtype]
        ref_score += H.doc_scores(segs, ref_mass, cfg.docs_per_query)
        dev_score = pb.score.cpu().numpy()[0]
        assert G.rel_error(dev_score[alive], ref_score[alive]) <= G.MASS_TOL[g.dtype]
        if layer in keeps:
            keep = keeps[layer]
            kept = pb.keep_idx[0, :keep].tolist()
            assert int(pb.n_keep[0].item()) == keep
            assert kept == orc.prune_topk(dev_score, lens, alive, keep)            # exact for its own scores
            key = {i: ref_score[i] / lens[i] for i in alive}
            cut = sorted(key.values(), reverse=True)[keep - 1]
            for i in alive:
                if key[i] > cut * (1 + 1e-3):
                    assert i in kept
                if key[i] < cut * (1 - 1e-3):
                    assert i not in kept
            ref_ns, ref_q, _ = orc.assign_positions(lens, kept, cfg.prefix_len, g.max_positions - cfg.tq)
            pb.advance()
            assert int(pb.q_start[0].item()) == ref_q
            assert {s.doc: s.new_start for s in G.device_segments(pb, 0) if s.kind == cf.CF_SEG_DOC} == ref_ns
            alive = kept
    assert set(st.planted[0].tolist()) <= set(alive)


# ----------------------------------------------------------------------------- full sizes, sampled
@pytest.mark.parametrize("deferred", [False, True])
def test_llama2_7b_stack_full_size(deferred):
    """(deferred: as bench.py runs it — the layers between two prune events leave their scores pending and the prune
    layer takes them in; their per-layer masses are then not reported, everything else is checked alike.)
    Configuration 4 at full size (32 layers, 30 documents x 160 tokens, pruning to 60 % after layers
    8/16/24/32), head-major store as bench.py runs it.  Every layer: flags, mass total, accumulated
    scores finite; every prune: the cut exact for the device's scores, the allocation bit-exact.  The
    oracle attends on every layer, on the tables the device holds, and accumulates its own scores: every cut also
    obeys the margin rule against those, and equals the oracle's cut where the oracle's gap is at least 1e-3."""
    cfg = wl.CONFIGS["llama2_7b_stack"]
    g = cfg.geometry
    st = wl.build_structure(cfg)
    lens = [int(x) for x in st.doc_lens]
    keeps, k = {}, cfg.docs_per_query
    for layer in cfg.prune_layers:
        k = orc.keep_fraction(k, cfg.keep_frac)
        keeps[layer] = k
    assert list(keeps.values()) == [18, 11, 7, 5]
    pb = G.make_batch(cfg, st, layout="head")
    pb.allocate_initial()
    assert int(pb.n_reuse[0].item()) == 2                      # 30 x 160 tokens do not fit 4096 positions once
    alive = list(range(cfg.docs_per_query))
    ref_score = np.zeros(cfg.docs_per_query)
    sampled = set(range(cfg.n_layers))
    for layer in range(cfg.n_layers):
        t = wl.build_layer(cfg, st, layer)
        dev = G.upload_layer(cfg, t, "head")
        out = torch.empty_like(dev["q"])
        if layer in sampled:
            segs, ref_out, ref_mass = G.oracle_on_device_segments(cfg, t, pb, 0)
            ref_score += H.doc_scores(segs, ref_mass, cfg.docs_per_query)
        pending = deferred and layer not in keeps
        pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, keep=keeps.get(layer),
                 strategy=cf.CF_ALLOC_SORT, defer=pending)
        torch.cuda.synchronize()
        assert pb.flags() == 0
        n_seg = int(pb.n_seg[0].item())
        assert n_seg == len(alive) + 2
        if layer in sampled:
            _say(f"stack layer {layer}: {len(alive)} documents")
            assert G.row_error(out.float().cpu().numpy(), ref_out) <= G.OUT_TOL[g.dtype]
        if layer in sampled and not pending:
            mass = pb.mass.cpu().numpy()[0, :n_seg]
            assert mass.sum() == pytest.approx(g.n_q_heads * cfg.tq, rel=1e-5)
            assert G.rel_error(mass, ref_mass) <= G.MASS_TOL[g.dtype]
            assert G.rel_error(pb.score.cpu().numpy()[0][alive], ref_score[alive]) <= G.MASS_TOL[g.dtype]
        if layer in keeps:
            keep = keeps[layer]
            dev_score = pb.score.cpu().numpy()[0]
            kept = pb.keep_idx[0, :keep].tolist()
            assert kept == orc.prune_topk(dev_score, lens, alive, keep)
            gap = H.check_cut(kept, ref_score, lens, alive, keep, st.planted[0])
            _say(f"  prune to {keep}: oracle gap at the cut {gap:.2e}")
            ref_ns, ref_q, ref_nr = orc.assign_positions(lens, kept, cfg.prefix_len, g.max_positions - cfg.tq)
            pb.advance()
            assert int(pb.q_start[0].item()) == ref_q and int(pb.n_reuse[0].item()) == ref_nr
            assert {s.doc: s.new_start for s in G.device_segments(pb, 0) if s.kind == cf.CF_SEG_DOC} == ref_ns
            alive = kept
    assert set(st.planted[0].tolist()) <= set(alive)


def test_qwen2_1p5b_batch_full_size_sampled():
    """Configuration 5 at full size (store of 10 000 documents, 64 queries x 20 documents, fp16 GQA 12/2):
    every query against the oracle element by element (outputs, masses), every cut against the oracle's own scores
    by the margin rule, the planted documents' survival."""
    cfg = wl.CONFIGS["qwen2_1p5b_batch"]
    g = cfg.geometry
    st = wl.build_structure(cfg)
    t = wl.build_layer(cfg, st)
    pb = G.make_batch(cfg, st, layout="head")
    dev = G.upload_layer(cfg, t, "head")
    out = torch.empty_like(dev["q"])
    pb.allocate_initial()
    pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, keep=cfg.keep,
             strategy=cf.CF_ALLOC_SORT)
    torch.cuda.synchronize()
    assert pb.flags() == 0
    mass = pb.mass.cpu().numpy()
    score = pb.score.cpu().numpy()
    keep_idx = pb.keep_idx.cpu().numpy()
    out_np = out.float().cpu().numpy()
    for b in range(cfg.batch):
        assert mass[b, :cfg.docs_per_query + 1].sum() == pytest.approx(g.n_q_heads * cfg.tq, rel=1e-5)
        qlens = st.doc_lens[st.query_docs[b]]
        assert keep_idx[b, :cfg.keep].tolist() == orc.prune_topk(score[b], qlens, list(range(cfg.docs_per_query)), cfg.keep)
        assert set(st.planted[b].tolist()) <= set(keep_idx[b, :cfg.keep].tolist())
    worst_out = worst_mass = 0.0
    smallest_gap = float("inf")
    for b in range(cfg.batch):
        ref_segs, ref_q, qlens = H.initial_segments(cfg, st, b)
        k_small, v_small, table = H.compact_query(ref_segs, t["k_store"], t["v_store"])    # the store holds 1.5 M tokens
        ref_out, ref_mass = orc.prefill_attention(H.f64(t["q"][b * cfg.tq:(b + 1) * cfg.tq]), 0, ref_q, k_small, v_small,
                                                  t["k_self"], t["v_self"], table, g.n_kv_heads, g.rope_base)
        worst_out = max(worst_out, G.row_error(out_np[b * cfg.tq:(b + 1) * cfg.tq], ref_out))
        worst_mass = max(worst_mass, G.rel_error(mass[b, :len(ref_segs)], ref_mass))
        ref_score = H.doc_scores(ref_segs, ref_mass, cfg.docs_per_query)
        gap = H.check_cut(keep_idx[b, :cfg.keep].tolist(), ref_score, qlens, list(range(cfg.docs_per_query)), cfg.keep,
                          st.planted[b])
        smallest_gap = min(smallest_gap, gap)
    _say(f"batch of {cfg.batch}: out err {worst_out:.3e}  mass err {worst_mass:.3e}  smallest oracle gap at a cut {smallest_gap:.2e}")
    assert worst_out <= G.OUT_TOL[g.dtype]
    assert worst_mass <= G.MASS_TOL[g.dtype]


# ----------------------------------------------------------------------------- N_reuse ablation modes
@pytest.mark.parametrize("max_positions", [4096, 2048])
def test_n_reuse_ablation_modes(max_positions):
    """The allocator settings of the N_reuse ablation (Sec. 3.3.2): N_reuse = k (every cache its own window),
    1 (no reuse), k/5, a fixed 5, and the adaptive value of Eq. 6, for k = 20 caches of 160 tokens.  Positions
    bit-exact against the oracle, attention on those positions within tolerance; a setting whose groups do not
    fit the positional range (the overflow the paper warns about) raises the flag and allocates nothing."""
    base = wl.CONFIGS["llama2_7b_layer"]
    g = wl.Geometry(8, 8, 128, "bf16", 1.0e4, max_positions)
    cfg = wl.scaled(base, name=f"ablation_{max_positions}", geometry=g, n_store_docs=20, docs_per_query=20, n_planted=2)
    st = wl.build_structure(cfg, seed=7300)
    t = wl.build_layer(cfg, st, seed=73)
    dev = G.upload_layer(cfg, t)
    k = cfg.docs_per_query
    lens = [int(x) for x in st.doc_lens[st.query_docs[0]]]
    pos_begin, pos_end = cfg.prefix_len, max_positions - cfg.tq
    seen = {}
    for name, force in [("k", k), ("one", 1), ("k/5", k // 5), ("five", 5), ("adaptive", 0)]:
        pb = G.make_batch(cfg, st)
        pb.allocate_initial(force_n_reuse=force)
        torch.cuda.synchronize()
        try:
            ref_ns, ref_q, ref_nr = orc.assign_positions(lens, list(range(k)), pos_begin, pos_end, orc.STRATEGY_SORT, force)
        except ValueError:
            # the allocator writes nothing: positions and q_start keep their initial zeros
            assert pb.flags() == cf.CF_FLAG_POS_OVERFLOW
            assert int(pb.q_start[0].item()) == 0 and not pb.new_start.any()
            seen[name] = "overflow"
            continue
        assert pb.flags() == 0
        assert int(pb.q_start[0].item()) == ref_q and int(pb.n_reuse[0].item()) == ref_nr
        assert pb.new_start[0].tolist() == [ref_ns[s] for s in range(k)]
        out = torch.empty_like(dev["q"])
        pb.attention(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out)
        torch.cuda.synchronize()
        segs, ref_out, ref_mass = G.oracle_on_device_segments(cfg, t, pb, 0)
        assert G.row_error(out.float().cpu().numpy(), ref_out) <= G.OUT_TOL["bf16"]
        assert G.rel_error(pb.mass.cpu().numpy()[0, :len(segs)], ref_mass) <= G.MASS_TOL["bf16"]
        seen[name] = ref_nr
    _say(f"N_reuse modes at {max_positions} positions: {seen}")
    if max_positions == 4096:
        assert seen == {"k": 20, "one": 1, "k/5": 4, "five": 5, "adaptive": 1}
    else:
        assert seen == {"k": 20, "one": "overflow", "k/5": 4, "five": 5, "adaptive": 2}


# ----------------------------------------------------------------------------- Alg. 2 Phase 2: cf_assemble_cache
def _assemble(cfg, st, t, pb, layout_in, layout_out, pairing=cf.CF_ROPE_HALF, capacity_pad=3):
    """Run cf_assemble_cache on the tables `pb` holds; returns device outputs and the geometry used."""
    g = cfg.geometry
    dev = G.upload_layer(cfg, t, layout_in)
    lens = st.doc_lens[st.query_docs]
    per_query = int(cfg.prefix_len + lens.sum(axis=1).max() + cfg.tq) + capacity_pad
    capacity = per_query * cfg.batch
    kind, pad = G.LAYOUTS[layout_out]
    ts, hs = pl.store_strides(capacity, g.n_kv_heads, g.head_dim, kind, pad)
    shape = (capacity, g.n_kv_heads, g.head_dim) if kind == "token" else (g.n_kv_heads, capacity + pad, g.head_dim)
    k_final = torch.full(shape, 7.0, dtype=pl.TORCH_DTYPE[g.dtype], device="cuda")
    v_final = torch.full(shape, 7.0, dtype=pl.TORCH_DTYPE[g.dtype], device="cuda")
    final_off = torch.arange(cfg.batch, dtype=torch.int64, device="cuda") * per_query
    final_len = torch.full((cfg.batch,), -1, **I32)
    final_pos = torch.full((capacity,), -1, **I32)
    cf.cf_assemble_cache(pb.desc, dev["k_store"], dev["v_store"], st.n_store_tokens, dev["k_self"], dev["v_self"], pb.q_off,
                         pb.segs, pb.n_seg, pb.seg_stride, cfg.batch, cfg.tq, int(max(lens.max(), cfg.prefix_len, cfg.tq)),
                         final_off, capacity, ts, hs, k_final, v_final, final_len, final_pos, pb.dev_flag)
    torch.cuda.synchronize()
    as_tokens = (lambda x: x) if kind == "token" else (lambda x: x[:, :capacity].permute(1, 0, 2))
    return dict(k=as_tokens(k_final).float().cpu().numpy(), v=as_tokens(v_final).float().cpu().numpy(),
                len=final_len.cpu().numpy(), pos=final_pos.cpu().numpy(), per_query=per_query, dev=dev,
                k_dev=k_final, v_dev=v_final, strides=(ts, hs), capacity=capacity)


@pytest.mark.parametrize("dtype,pairing,layout_in,layout_out", [
    ("bf16", cf.CF_ROPE_HALF, "head", "head"), ("bf16", cf.CF_ROPE_HALF, "token", "head_padded"),
    ("f16", cf.CF_ROPE_INTERLEAVED, "head_padded", "token"), ("f32", cf.CF_ROPE_HALF, "token", "token")])
def test_assemble_cache_matches_oracle(dtype, pairing, layout_in, layout_out):
    """Final Re-Positioning after a prune: gathered keys within one rounding of the oracle's, values and
    unmoved keys bit-exact copies, positions and lengths exact, nothing written outside the runs."""
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name=f"phase2_{dtype}", geometry=wl.Geometry(6, 3, 128, dtype, 1.0e4, 4096),
                    n_store_docs=24, docs_per_query=7, batch=3, doc_len_range=(3, 90), tq=5, prefix_len=9,
                    doc_stored_start=9, n_planted=1)
    _say(f"assemble {dtype} pairing={pairing} {layout_in}->{layout_out}")
    st = wl.build_structure(cfg, seed=7400)
    t = wl.build_layer(cfg, st, seed=74)
    pb = G.make_batch(cfg, st, pairing, layout_in)
    pb.allocate_initial()
    pb.score.copy_(torch.from_numpy(np.random.default_rng(3).random((cfg.batch, cfg.docs_per_query), dtype=np.float32)))
    pb.prune(4, cf.CF_ALLOC_SORT)                            # survivors re-packed: most documents move
    pb.advance()
    r = _assemble(cfg, st, t, pb, layout_in, layout_out, pairing)
    assert pb.flags() == 0
    pname = "half" if pairing == cf.CF_ROPE_HALF else "interleaved"
    tol = {"f32": 2e-6, "bf16": 2.0 ** -8, "f16": 2.0 ** -10}[dtype]
    written = np.zeros(r["capacity"], dtype=bool)
    for b in range(cfg.batch):
        segs = G.device_segments(pb, b)
        k_ref, v_ref, pos_ref = orc.assemble_final_cache(t["k_store"], t["v_store"], t["k_self"][b * cfg.tq:], t["v_self"][b * cfg.tq:],
                                                         [s._replace(tok_offset=0) if s.kind == cf.CF_SEG_SELF else s for s in segs],
                                                         cfg.tq, cfg.geometry.rope_base, pname)
        n = len(pos_ref)
        lo = b * r["per_query"]
        assert r["len"][b] == n and r["pos"][lo:lo + n].tolist() == pos_ref.tolist()
        assert np.max(np.abs(r["k"][lo:lo + n] - k_ref)) <= tol * max(1.0, np.abs(k_ref).max())
        assert np.array_equal(r["v"][lo:lo + n], v_ref)
        # segments that do not move are exact copies
        at = 0
        for s in segs:
            m = min(s.len, cfg.tq) if s.kind == cf.CF_SEG_SELF else s.len
            if s.new_start == s.stored_start:
                assert np.array_equal(r["k"][lo + at:lo + at + m], k_ref[at:at + m])
            at += m
        written[lo:lo + n] = True
    assert np.all(r["k"][~written] == 7.0) and np.all(r["v"][~written] == 7.0) and np.all(r["pos"][~written] == -1)


def test_decode_step_over_assembled_cache():
    """Alg. 2 Phase 3's attention: one new token per query attends over the assembled cache through
    cf_prefill_attention (one zero-shift segment, strides of the decode cache) and matches the oracle."""
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name="decode", geometry=wl.Geometry(8, 8, 128, "bf16", 1.0e4, 4096),
                    n_store_docs=12, docs_per_query=5, batch=2, doc_len_range=(100, 200), tq=48, prefix_len=32,
                    doc_stored_start=32, n_planted=1)
    g = cfg.geometry
    st = wl.build_structure(cfg, seed=7401)
    t = wl.build_layer(cfg, st, seed=75)
    pb = G.make_batch(cfg, st, layout="head")
    pb.allocate_initial()
    r = _assemble(cfg, st, t, pb, "head", "head")
    assert pb.flags() == 0
    rng = np.random.default_rng(76)
    q_raw = wl.round_to_dtype(rng.standard_normal((cfg.batch, g.n_q_heads, g.head_dim), dtype=np.float32), g.dtype)
    ts, hs = r["strides"]
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions,
                        store_token_stride=ts, store_head_stride=hs)
    # the queries arrive with RoPE for their absolute positions (right after each query block), rounded to bf16
    p_new = [int(pb.q_start[b].item()) + cfg.tq for b in range(cfg.batch)]
    q_abs = wl.round_to_dtype(np.stack([orc.rotate(q_raw[b].astype(np.float64), p_new[b], g.rope_base)
                                        for b in range(cfg.batch)]).astype(np.float32), g.dtype)
    segs = cf.segments_array([(b * r["per_query"], int(r["len"][b]), 0, 0, cf.CF_SEG_PREFIX, -1) for b in range(cfg.batch)])
    seg_dev = cf.segments_to_device(segs)
    n_seg = torch.ones(cfg.batch, **I32)
    q_off = torch.arange(cfg.batch + 1, **I32)
    zeros = torch.zeros(cfg.batch, **I32)
    q_dev = pl.to_device(q_abs, g.dtype)
    out = torch.empty_like(q_dev)
    mass = torch.zeros((cfg.batch, 1), dtype=torch.float32, device="cuda")
    max_kv = int(r["len"].max())
    ws_bytes = cf.cf_prefill_workspace_bytes(desc, cfg.batch, 1, 1, max_kv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    flag = torch.zeros(1, **I32)
    cf.cf_prefill_attention(desc, q_dev, q_off, 0, zeros, r["k_dev"], r["v_dev"], r["capacity"], None, None, seg_dev, n_seg, 1,
                            cfg.batch, 1, max_kv, out, mass, None, 1, ws, ws_bytes, flag)
    torch.cuda.synchronize()
    assert flag.item() == 0
    got = out.float().cpu().numpy()
    for b in range(cfg.batch):
        dsegs = G.device_segments(pb, b)
        k_ref, v_ref, _ = orc.assemble_final_cache(t["k_store"], t["v_store"], t["k_self"][b * cfg.tq:], t["v_self"][b * cfg.tq:],
                                                   [s._replace(tok_offset=0) if s.kind == cf.CF_SEG_SELF else s for s in dsegs],
                                                   cfg.tq, g.rope_base)
        ref = orc.decode_attention(q_abs[b:b + 1].astype(np.float64), k_ref, v_ref, g.n_kv_heads)
        assert G.row_error(got[b:b + 1], ref) <= G.OUT_TOL[g.dtype]
        assert mass[b, 0].item() == pytest.approx(g.n_q_heads, rel=1e-5)
    # outputs only (no mass buffer, as a decode loop calls it): the same bar
    out2 = torch.empty_like(out)
    cf.cf_prefill_attention(desc, q_dev, q_off, 0, zeros, r["k_dev"], r["v_dev"], r["capacity"], None, None, seg_dev, n_seg, 1,
                            cfg.batch, 1, max_kv, out2, None, None, 1, ws, ws_bytes, flag)
    torch.cuda.synchronize()
    assert flag.item() == 0 and torch.equal(out2, out)           # the same kernels: the same outputs, bit for bit


def test_assemble_cache_flags():
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], name="phase2_flags", geometry=wl.Geometry(4, 4, 64, "f32", 1.0e4, 4096))
    st = wl.build_structure(cfg)
    t = wl.build_layer(cfg, st)
    pb = G.make_batch(cfg, st)
    pb.allocate_initial()
    r = _assemble(cfg, st, t, pb, "token", "token", capacity_pad=-1)          # one token short
    assert pb.flags() == cf.CF_FLAG_BAD_INDEX and r["len"][0] == 0 and np.all(r["k"] == 7.0)
    pb.dev_flag.zero_()
    segs = cf.segments_from_device(pb.segs[0], 6)
    segs[2]["len"] = -4
    pb.segs[0].copy_(cf.segments_to_device(segs).reshape(6, 32))
    r = _assemble(cfg, st, t, pb, "token", "token")
    assert pb.flags() == cf.CF_FLAG_BAD_SEGMENT and r["len"][0] == 4 + 3 * 32 + 8


# ----------------------------------------------------------------------------- offline cache builder shape
def test_document_encoding_attention_shape():
    """The attention of query-independent parallel document caching (Sec. 2.2): every document attends to the
    shared prefix and causally to itself, never to another document.  Expressed through the same call — each
    document is a "query" with its own length whose table lists the prefix and its own block — and checked
    against the oracle; ragged query lengths in one batch."""
    rng = np.random.default_rng(81)
    g = wl.Geometry(8, 2, 128, "bf16", 1.0e6, 32768)
    prefix = 24
    doc_lens = [100, 200, 137, 64, 1, 163]
    q_off = np.concatenate([[0], np.cumsum(doc_lens)]).astype(np.int32)
    total = int(q_off[-1])
    rnd = lambda *shape: wl.round_to_dtype(rng.standard_normal(shape, dtype=np.float32), g.dtype)
    q, k_self, v_self = rnd(total, g.n_q_heads, g.head_dim), rnd(total, g.n_kv_heads, g.head_dim), rnd(total, g.n_kv_heads, g.head_dim)
    k_store, v_store = rnd(prefix, g.n_kv_heads, g.head_dim), rnd(prefix, g.n_kv_heads, g.head_dim)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions)
    batch, seg_stride, max_tq = len(doc_lens), 2, max(doc_lens)
    # every document is encoded right after the prefix: positions [prefix, prefix + len)
    tables = [[orc.Segment(0, prefix, 0, 0, orc.KIND_PREFIX, -1), orc.Segment(int(q_off[b]), doc_lens[b], prefix, prefix, orc.KIND_SELF, -1)]
              for b in range(batch)]
    segs = cf.segments_to_device(cf.segments_array([s for tb in tables for s in tb]))
    n_seg = torch.full((batch,), 2, **I32)
    q_new = torch.full((batch,), prefix, **I32)
    dev = {name: pl.to_device(x, g.dtype) for name, x in dict(q=q, k_self=k_self, v_self=v_self, k_store=k_store, v_store=v_store).items()}
    out = torch.empty_like(dev["q"])
    mass = torch.zeros((batch, seg_stride), dtype=torch.float32, device="cuda")
    max_kv = prefix + max_tq
    ws_bytes = cf.cf_prefill_workspace_bytes(desc, batch, max_tq, seg_stride, max_kv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    flag = torch.zeros(1, **I32)
    cf.cf_prefill_attention(desc, dev["q"], torch.from_numpy(q_off).cuda(), prefix, q_new, dev["k_store"], dev["v_store"], prefix,
                            dev["k_self"], dev["v_self"], segs, n_seg, seg_stride, batch, max_tq, max_kv, out, mass, None, 1,
                            ws, ws_bytes, flag)
    torch.cuda.synchronize()
    assert flag.item() == 0
    got, m = out.float().cpu().numpy(), mass.cpu().numpy()
    for b in range(batch):
        lo, hi = int(q_off[b]), int(q_off[b + 1])
        ref_out, ref_mass = orc.prefill_attention(q[lo:hi].astype(np.float64), prefix, prefix, k_store, v_store, k_self, v_self,
                                                  tables[b], g.n_kv_heads, g.rope_base)
        assert G.row_error(got[lo:hi], ref_out) <= G.OUT_TOL[g.dtype]
        assert G.rel_error(m[b], ref_mass) <= G.MASS_TOL[g.dtype]           # nothing moves here: the keys are the oracle's


@pytest.mark.parametrize("layout", ["head", "token"])
def test_offline_store_builder_writes_the_cache_store(layout):
    """Sec. 2.2 end to end for one layer: the shared prefix, then the documents, are encoded (attention over
    the prefix and causally over themselves, each from local position 0) and their keys, moved to the positions
    they are cached at (Eq. 5), and values are written into the store; a query then prefills over the store the device built.  The
    store must equal the oracle's rotation of the fresh keys within one rounding (values bit for bit), the
    encoders' outputs and the query's outputs and masses must match the oracle."""
    rng = np.random.default_rng(83)
    g = wl.Geometry(8, 2, 128, "bf16", 1.0e6, 32768)
    prefix = 24
    doc_lens = np.array([100, 200, 137, 64, 1, 163], dtype=np.int32)
    doc_off = np.concatenate([[prefix], prefix + np.cumsum(doc_lens)]).astype(np.int64)
    n_store = int(doc_off[-1])
    _say(f"store builder {layout}: {len(doc_lens)} documents, {n_store} store tokens")
    rnd = lambda *shape: wl.round_to_dtype(rng.standard_normal(shape, dtype=np.float32), g.dtype)
    fresh = {name: (rnd(n, g.n_q_heads, g.head_dim), rnd(n, g.n_kv_heads, g.head_dim), rnd(n, g.n_kv_heads, g.head_dim))
             for name, n in (("prefix", prefix), ("docs", int(doc_lens.sum())))}
    ts, hs = pl.store_strides(n_store, g.n_kv_heads, g.head_dim, layout)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions,
                        store_token_stride=ts, store_head_stride=hs)
    shape = (n_store, g.n_kv_heads, g.head_dim) if layout == "token" else (g.n_kv_heads, n_store, g.head_dim)
    k_store = torch.full(shape, 7.0, dtype=torch.bfloat16, device="cuda")
    v_store = torch.full(shape, 7.0, dtype=torch.bfloat16, device="cuda")
    as_tokens = (lambda x: x) if layout == "token" else (lambda x: x.permute(1, 0, 2))

    # ---- the device builds the store: the prefix at positions [0, prefix), every document at [prefix, prefix + len)
    builders = {"prefix": pl.StoreBuilder(desc, np.array([0]), np.array([prefix]), np.array([0]), 0, n_store),
                "docs": pl.StoreBuilder(desc, doc_off[:-1], doc_lens, np.full(len(doc_lens), prefix), prefix, n_store)}
    outs = {}
    for name in ("prefix", "docs"):
        q, k, v = (pl.to_device(x, g.dtype) for x in fresh[name])
        outs[name] = torch.empty_like(q)
        builders[name].attend(q, k, v, k_store, v_store, outs[name])
        builders[name].write(k, v, k_store, v_store, ts, hs)
        torch.cuda.synchronize()
        assert builders[name].flags() == 0
    assert builders["docs"].final_len.tolist() == doc_lens.tolist()
    k_dev = as_tokens(k_store).float().cpu().numpy()
    v_dev = as_tokens(v_store).float().cpu().numpy()

    # ---- the store the oracle expects
    # (a text's fresh keys carry RoPE for its local positions 0..len-1; the documents move by `prefix`, Eq. 5)
    k_ref = np.concatenate([fresh["prefix"][1].astype(np.float64),
                            orc.rotate(fresh["docs"][1].astype(np.float64), prefix, g.rope_base)])
    assert np.max(np.abs(k_dev - k_ref)) <= 2.0 ** -8 * max(1.0, np.abs(k_ref).max())
    assert np.array_equal(v_dev, np.concatenate([fresh["prefix"][2], fresh["docs"][2]]))
    assert np.array_equal(k_dev[:prefix], fresh["prefix"][1])                  # the prefix does not move: exact copies
    assert not np.array_equal(k_dev[prefix:], fresh["docs"][1])
    # the oracle's own store (moved keys rounded once to the storage type) is what every expected value below is
    # computed on; the device's differs from it by at most one rounding step in a few elements (checked above)
    k_orc = wl.round_to_dtype(k_ref.astype(np.float32), g.dtype)
    v_orc = np.concatenate([fresh["prefix"][2], fresh["docs"][2]])
    assert np.mean(k_dev != k_orc) < 2e-3

    # ---- the encoders' outputs against the oracle
    q_p, k_p, v_p = fresh["prefix"]
    ref, _ = orc.prefill_attention(q_p.astype(np.float64), 0, 0, k_orc, v_orc, k_p, v_p,
                                   [orc.Segment(0, prefix, 0, 0, orc.KIND_SELF, -1)], g.n_kv_heads, g.rope_base)
    assert G.row_error(outs["prefix"].float().cpu().numpy(), ref) <= G.OUT_TOL[g.dtype]
    q_d, k_d, v_d = fresh["docs"]
    got = outs["docs"].float().cpu().numpy()
    q_off = np.concatenate([[0], np.cumsum(doc_lens)])
    for b in range(len(doc_lens)):
        lo, hi = int(q_off[b]), int(q_off[b + 1])
        table = [orc.Segment(0, prefix, 0, 0, orc.KIND_PREFIX, -1), orc.Segment(lo, hi - lo, 0, prefix, orc.KIND_SELF, -1)]
        ref, _ = orc.prefill_attention(q_d[lo:hi].astype(np.float64), 0, prefix, k_orc, v_orc, k_d, v_d, table,
                                       g.n_kv_heads, g.rope_base)
        assert G.row_error(got[lo:hi], ref) <= G.OUT_TOL[g.dtype]

    # ---- a query prefills over the store the device built (every document a candidate, keep 3)
    tq = 16
    pb = pl.PrefillBatch(desc, doc_off[:-1][None, :], doc_lens[None, :], tq, prefix, prefix, n_store)
    pb.allocate_initial()
    q, k_self, v_self = rnd(tq, g.n_q_heads, g.head_dim), rnd(tq, g.n_kv_heads, g.head_dim), rnd(tq, g.n_kv_heads, g.head_dim)
    dq, dk, dv = (pl.to_device(x, g.dtype) for x in (q, k_self, v_self))
    out = torch.empty_like(dq)
    segs = G.device_segments(pb, 0)
    pb.layer(dq, dk, dv, k_store, v_store, out, keep=3)
    torch.cuda.synchronize()
    assert pb.flags() == 0
    q_start = int(pb.q_start[0].item())
    ref_out, ref_mass = orc.prefill_attention(q.astype(np.float64), 0, q_start, k_orc, v_orc, k_self, v_self,
                                              segs, g.n_kv_heads, g.rope_base)
    assert G.row_error(out.float().cpu().numpy(), ref_out) <= G.OUT_TOL[g.dtype]
    mass = pb.mass.cpu().numpy()[0, :len(segs)]
    # loose: the keys were rounded when they entered the store and again when this call moved them, and a one-token
    # document's mass hangs on one such key
    long_ = np.array([sg.len >= 8 for sg in segs])
    assert G.rel_error(mass[long_], ref_mass[long_]) <= 2e-4
    assert G.rel_error(mass[~long_], ref_mass[~long_]) <= 4e-3
    assert pb.keep_idx[0, :3].tolist() == orc.prune_topk(pb.score.cpu().numpy()[0], [int(x) for x in doc_lens], list(range(len(doc_lens))), 3)
    # tight: the same call over the oracle's store, against the oracle on keys moved and rounded as the kernel holds them
    pb2 = pl.PrefillBatch(desc, doc_off[:-1][None, :], doc_lens[None, :], tq, prefix, prefix, n_store)
    pb2.allocate_initial()
    out2 = torch.empty_like(dq)
    pb2.attention(dq, dk, dv, pl.store_to_device(k_orc, g.dtype, layout), pl.store_to_device(v_orc, g.dtype, layout), out2)
    torch.cuda.synchronize()
    assert pb2.flags() == 0
    _, near_mass = H.rounded_key_reference(g.dtype, q, 0, q_start, k_orc, v_orc, k_self, v_self, segs, g.n_kv_heads, g.rope_base)
    assert G.row_error(out2.float().cpu().numpy(), ref_out) <= G.OUT_TOL[g.dtype]
    assert G.rel_error(pb2.mass.cpu().numpy()[0, :len(segs)], near_mass) <= G.NEAR_MASS_TOL[g.dtype]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_batch_with_an_empty_query(dtype):
    """Queries of 5, 0 and 7 rows in one batch (the middle one has no rows at all) over shared documents: the
    non-empty ones match the oracle, the empty one leaves zero masses, nothing is written out of place."""
    rng = np.random.default_rng(97)
    g = wl.Geometry(4, 2, 128 if dtype == "bf16" else 64, dtype, 1.0e4, 4096)
    prefix, doc_lens, tqs = 6, [40, 33, 1], [5, 0, 7]
    doc_off = np.concatenate([[prefix], prefix + np.cumsum(doc_lens)])
    n_store = int(doc_off[-1])
    q_off = np.concatenate([[0], np.cumsum(tqs)]).astype(np.int32)
    total = int(q_off[-1])
    rnd = lambda *shape: wl.round_to_dtype(rng.standard_normal(shape, dtype=np.float32), g.dtype)
    q, k_self, v_self = rnd(total, g.n_q_heads, g.head_dim), rnd(total, g.n_kv_heads, g.head_dim), rnd(total, g.n_kv_heads, g.head_dim)
    k_store, v_store = rnd(n_store, g.n_kv_heads, g.head_dim), rnd(n_store, g.n_kv_heads, g.head_dim)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions)
    batch, seg_stride, max_tq = 3, 5, max(tqs)
    q_pos = [100, 200, 300]
    tables = [[orc.Segment(0, prefix, 0, 0, orc.KIND_PREFIX, -1)] +
              [orc.Segment(int(doc_off[d]), doc_lens[d], prefix, 10 + 50 * d + 3 * b, orc.KIND_DOC, d) for d in range(3)] +
              [orc.Segment(int(q_off[b]), tqs[b], 0, q_pos[b], orc.KIND_SELF, -1)] for b in range(batch)]
    segs = cf.segments_to_device(cf.segments_array([s for tb in tables for s in tb]))
    n_seg = torch.full((batch,), 5, **I32)
    dev = {name: pl.to_device(x, g.dtype) for name, x in dict(q=q, k_self=k_self, v_self=v_self, k_store=k_store, v_store=v_store).items()}
    out = torch.full_like(dev["q"], 7.0)
    mass = torch.full((batch, seg_stride), -1.0, dtype=torch.float32, device="cuda")
    score = torch.zeros((batch, 3), dtype=torch.float32, device="cuda")
    max_kv = prefix + sum(doc_lens) + max_tq
    ws_bytes = cf.cf_prefill_workspace_bytes(desc, batch, max_tq, seg_stride, max_kv)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    flag = torch.zeros(1, **I32)
    cf.cf_prefill_attention(desc, dev["q"], torch.from_numpy(q_off).cuda(), 0, torch.tensor(q_pos, **I32), dev["k_store"], dev["v_store"],
                            n_store, dev["k_self"], dev["v_self"], segs, n_seg, seg_stride, batch, max_tq, max_kv, out, mass, score, 3,
                            ws, ws_bytes, flag)
    torch.cuda.synchronize()
    assert flag.item() == 0
    got, m, sc = out.float().cpu().numpy(), mass.cpu().numpy(), score.cpu().numpy()
    for b in (0, 2):
        lo, hi = int(q_off[b]), int(q_off[b + 1])
        ref_out, ref_mass = orc.prefill_attention(q[lo:hi].astype(np.float64), 0, q_pos[b], k_store, v_store, k_self, v_self,
                                                  tables[b], g.n_kv_heads, g.rope_base)
        assert G.row_error(got[lo:hi], ref_out) <= G.OUT_TOL[g.dtype]
        # few rows, short documents: against the plain oracle the one rounding of a moved key shows
        assert G.rel_error(m[b], ref_mass) <= (4e-3 if dtype == "bf16" else G.MASS_TOL[g.dtype])
        _, near_mass = H.rounded_key_reference(g.dtype, q[lo:hi], 0, q_pos[b], k_store, v_store, k_self, v_self, tables[b],
                                               g.n_kv_heads, g.rope_base)
        assert G.rel_error(m[b], near_mass) <= G.NEAR_MASS_TOL[g.dtype]
        assert G.rel_error(sc[b], near_mass[1:4]) <= G.NEAR_MASS_TOL[g.dtype]
    assert np.all(m[1] == 0.0) and np.all(sc[1] == 0.0)


@pytest.mark.parametrize("base,max_pos", [(1.0e4, 4096), (1.0e6, 32768)])
def test_largest_relative_shifts(base, max_pos):
    """Documents at the start of the positional range and the query at its very end (and the other way round): the
    relative shift of a key reaches the whole range; cos/sin of that many positions times theta must still be
    accurate (angle reduced in fp64)."""
    rng = np.random.default_rng(98)
    g = wl.Geometry(4, 4, 128, "bf16", base, max_pos)
    doc_lens, tq = [70, 45], 6
    doc_off = np.concatenate([[0], np.cumsum(doc_lens)])
    n_store = int(doc_off[-1])
    rnd = lambda *shape: wl.round_to_dtype(rng.standard_normal(shape, dtype=np.float32), g.dtype)
    q, k_self, v_self = rnd(2 * tq, g.n_q_heads, g.head_dim), rnd(2 * tq, g.n_kv_heads, g.head_dim), rnd(2 * tq, g.n_kv_heads, g.head_dim)
    k_store, v_store = rnd(n_store, g.n_kv_heads, g.head_dim), rnd(n_store, g.n_kv_heads, g.head_dim)
    desc = cf.make_desc(g.n_q_heads, g.n_kv_heads, g.head_dim, g.dtype, g.rope_base, g.max_positions)
    q_pos = [max_pos - tq, 0]                        # query 0 at the end of the range, query 1 at its start
    tables = [[orc.Segment(0, 70, max_pos - 70, 0, orc.KIND_DOC, 0), orc.Segment(70, 45, 0, 70, orc.KIND_DOC, 1),
               orc.Segment(0, tq, 0, q_pos[0], orc.KIND_SELF, -1)],
              [orc.Segment(0, 70, 0, max_pos - 200, orc.KIND_DOC, 0), orc.Segment(70, 45, 17, max_pos - 130, orc.KIND_DOC, 1),
               orc.Segment(tq, tq, max_pos - tq, q_pos[1], orc.KIND_SELF, -1)]]
    segs = cf.segments_to_device(cf.segments_array([s for tb in tables for s in tb]))
    n_seg = torch.full((2,), 3, **I32)
    dev = {name: pl.to_device(x, g.dtype) for name, x in dict(q=q, k_self=k_self, v_self=v_self, k_store=k_store, v_store=v_store).items()}
    out = torch.empty_like(dev["q"])
    mass = torch.zeros((2, 3), dtype=torch.float32, device="cuda")
    ws_bytes = cf.cf_prefill_workspace_bytes(desc, 2, tq, 3, n_store + tq)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    flag = torch.zeros(1, **I32)
    # q rows carry RoPE for local positions (q_stored_start 0); the own block of query 1 was stored at the range's end
    cf.cf_prefill_attention(desc, dev["q"], torch.tensor([0, tq, 2 * tq], **I32), 0, torch.tensor(q_pos, **I32), dev["k_store"],
                            dev["v_store"], n_store, dev["k_self"], dev["v_self"], segs, n_seg, 3, 2, tq, n_store + tq, out, mass,
                            None, 1, ws, ws_bytes, flag)
    torch.cuda.synchronize()
    assert flag.item() == 0
    got, m = out.float().cpu().numpy(), mass.cpu().numpy()
    for b in range(2):
        ref_out, ref_mass = orc.prefill_attention(q[b * tq:(b + 1) * tq].astype(np.float64), 0, q_pos[b], k_store, v_store, k_self,
                                                  v_self, tables[b], g.n_kv_heads, g.rope_base)
        assert G.row_error(got[b * tq:(b + 1) * tq], ref_out) <= G.OUT_TOL[g.dtype]
        assert G.rel_error(m[b], ref_mass) <= 4e-3               # six rows: the one rounding of a moved key shows
        _, near_mass = H.rounded_key_reference(g.dtype, q[b * tq:(b + 1) * tq], 0, q_pos[b], k_store, v_store, k_self, v_self,
                                               tables[b], g.n_kv_heads, g.rope_base)
        assert G.rel_error(m[b], near_mass) <= G.NEAR_MASS_TOL[g.dtype]


@pytest.mark.parametrize("deferred", [False, True])
def test_layer_calls_replay_from_a_hip_graph(deferred):
    """The library allocates nothing and clears nothing with memsets, so its calls can be captured: four layer calls
    (a prune event in each — or, deferred, three layers that leave their scores pending and a prune event that takes
    them in) recorded into one HIP graph replay to exactly the eager results, several times, with eager work and
    synchronisations between the replays."""
    cfg = wl.CONFIGS["llama2_7b_layer"]
    st = wl.build_structure(cfg)
    layers = [G.upload_layer(cfg, wl.build_layer(cfg, st, layer), "head") for layer in range(4)]
    pb = G.make_batch(cfg, st, layout="head")
    pb.allocate_initial()
    outs = [torch.empty_like(layers[0]["q"]) for _ in layers]

    def run_all():
        for i, (L, o) in enumerate(zip(layers, outs)):
            last = i == len(layers) - 1
            pb.layer(L["q"], L["k_self"], L["v_self"], L["k_store"], L["v_store"], o,
                     keep=cfg.keep if (last or not deferred) else None, defer=deferred and not last)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        pb.score.zero_()
        run_all()
        torch.cuda.synchronize()
        assert pb.flags() == 0
        eager = dict(outs=[o.clone() for o in outs], score=pb.score.clone(), keep=pb.keep_idx.clone(), segs=pb.next_segs.clone(),
                     mass=pb.mass.clone())
        graph = torch.cuda.CUDAGraph()
        pb.score.zero_()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run_all()
        scratch = torch.zeros(1 << 20, device="cuda")
        for rep in range(3):
            pb.score.zero_()
            pb.mass.fill_(-1.0)
            pb.next_segs.zero_()
            for o in outs:
                o.zero_()
            scratch.add_(1.0)                        # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert pb.flags() == 0
            assert all(torch.equal(a, b) for a, b in zip(outs, eager["outs"])), rep
            assert torch.equal(pb.score, eager["score"]) and torch.equal(pb.keep_idx, eager["keep"]), rep
            assert torch.equal(pb.next_segs, eager["segs"]) and torch.equal(pb.mass, eager["mass"]), rep
