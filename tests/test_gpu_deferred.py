"""Deferred document-wise scores (cf_prefill_layer with defer / n_pending): layers between two prune events leave their
slot partials pending in the workspace and the next call that does not defer takes them in, in layer order.  Alg. 2's
S, every cut and every table must come out bit for bit as when each layer accumulates its own scores."""

from __future__ import annotations

import sys

import numpy as np
import pytest
import torch

from oracle import cachefocus_oracle as orc
from paper_2502_11101_amd import binding as cf
from paper_2502_11101_amd import workloads as wl
from tests import gpu_harness as G
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, file=sys.stderr, flush=True)


def _run_stack(cfg, st, layers, keeps, deferred: bool, layout="head"):
    pb = G.make_batch(cfg, st, layout=layout)
    pb.allocate_initial()
    outs, snap = [], []
    for layer, dev in enumerate(layers):
        out = torch.empty_like(dev["q"])
        keep = keeps.get(layer)
        last = layer == len(layers) - 1
        defer = deferred and keep is None and not last and pb.n_pending < cf.CF_MAX_PENDING
        pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, keep=keep, defer=defer)
        outs.append(out)
        if keep is not None:
            torch.cuda.synchronize()
            snap.append(dict(score=pb.score.clone(), keep=pb.keep_idx.clone(), n_keep=pb.n_keep.clone(), mass=pb.mass.clone(),
                             segs=pb.next_segs.clone(), q_start=pb.next_q_start.clone()))
            pb.advance()
    torch.cuda.synchronize()
    assert pb.flags() == 0 and pb.n_pending == 0
    return dict(outs=outs, snap=snap, score=pb.score.clone(), mass=pb.mass.clone())


CASES = {
    # geometry, docs per query, doc lengths, tq, batch, layers, prune layers -> keep
    "llama_stack": (wl.LLAMA2_7B, 12, (160, 160), 48, 1, 9, {3: 8, 7: 5}),
    "gqa_batch": (wl.Geometry(12, 2, 128, "f16", 1.0e6, 32768), 6, (40, 90), 24, 3, 6, {2: 4, 4: 2}),
    "long_table": (wl.Geometry(4, 4, 128, "bf16", 1.0e4, 8192), 80, (1, 9), 5, 1, 5, {3: 30}),      # more than 64 entries: block-wide reductions
    "no_prune_at_all": (wl.Geometry(8, 8, 128, "bf16", 1.0e4, 4096), 5, (30, 60), 16, 2, 18, {}),   # 15 layers pending, then a flush, then more
}


@pytest.mark.parametrize("case", list(CASES))
def test_deferred_scores_equal_eager_scores(case):
    g, docs, len_range, tq, batch, n_layers, keeps = CASES[case]
    _say(f"deferred scores {case}")
    cfg = wl.scaled(wl.CONFIGS["llama2_7b_stack"], name=case, geometry=g, n_store_docs=batch * docs, docs_per_query=docs,
                    doc_len_range=len_range, tq=tq, batch=batch, n_planted=1, n_layers=n_layers, prefix_len=8, doc_stored_start=8)
    st = wl.build_structure(cfg, seed=7400 + len(case))
    tensors = [wl.build_layer(cfg, st, layer, seed=7450 + layer) for layer in range(n_layers)]
    layers = [G.upload_layer(cfg, t, "head") for t in tensors]
    eager = _run_stack(cfg, st, layers, keeps, deferred=False)
    lazy = _run_stack(cfg, st, layers, keeps, deferred=True)
    assert all(torch.equal(a, b) for a, b in zip(eager["outs"], lazy["outs"]))
    assert torch.equal(eager["score"], lazy["score"]) and torch.equal(eager["mass"], lazy["mass"])
    assert len(eager["snap"]) == len(keeps)
    for a, b in zip(eager["snap"], lazy["snap"]):
        for key in a:
            assert torch.equal(a[key], b[key]), key
    # and the accumulated scores are the oracle's (on keys moved and rounded as the kernels hold them): layer by layer on
    # the tables the device used, up to the first prune event
    first_prune = min(keeps) if keeps else n_layers - 1
    pb = G.make_batch(cfg, st, layout="head")
    pb.allocate_initial()
    torch.cuda.synchronize()
    ref = np.zeros((batch, docs))
    for layer in range(first_prune + 1):
        for b in range(batch):
            segs = G.device_segments(pb, b)
            t = tensors[layer]
            _, mass = H.rounded_key_reference(g.dtype, t["q"][b * tq:(b + 1) * tq], 0, int(pb.q_start[b].item()), t["k_store"],
                                              t["v_store"], t["k_self"], t["v_self"], segs, g.n_kv_heads, g.rope_base)
            ref[b] += H.doc_scores(segs, mass, docs)
    got = (lazy["snap"][0]["score"] if keeps else None)
    if got is not None:
        assert G.rel_error(got.cpu().numpy(), ref) <= G.NEAR_MASS_TOL[g.dtype]


def test_pending_layers_need_a_free_part_and_no_prune_step():
    cfg = wl.scaled(wl.CONFIGS["llama2_7b_layer"], n_store_docs=3, docs_per_query=3, n_planted=1)
    st = wl.build_structure(cfg)
    dev = G.upload_layer(cfg, wl.build_layer(cfg, st))
    pb = G.make_batch(cfg, st)
    pb.allocate_initial()
    out = torch.empty_like(dev["q"])
    with pytest.raises(cf.CacheFocusError):
        pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, keep=2, defer=True)
    pb.n_pending = cf.CF_MAX_PENDING
    with pytest.raises(cf.CacheFocusError):
        pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out, defer=True)
    pb.n_pending = cf.CF_MAX_PENDING + 1
    with pytest.raises(cf.CacheFocusError):
        pb.layer(dev["q"], dev["k_self"], dev["v_self"], dev["k_store"], dev["v_store"], out)
