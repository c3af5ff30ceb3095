"""cf_prefill_attention_static — the entry point for callers that cannot allocate — against cf_prefill_attention:
the same kernels on a library-owned scratch buffer instead of a caller's workspace give bit-identical outputs and
masses.  Two calls in a row, the second on a smaller input (the buffer keeps the first call's contents), then a
shape beyond the buffer, which must be refused before anything is launched."""

from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2502_11101_amd import binding as cf
from paper_2502_11101_amd import workloads as wl
from tests import gpu_harness as G

pytestmark = pytest.mark.gpu


def _both(cfg, seed):
    st = wl.build_structure(cfg, seed=7000 + seed)
    t = wl.build_layer(cfg, st, seed=seed)
    pb = G.make_batch(cfg, st)
    dev = G.upload_layer(cfg, t)
    pb.allocate_initial()
    res = []
    for static in (False, True):
        out = torch.full_like(dev["q"], 7.0)
        mass = torch.full_like(pb.mass, -1.0)
        score = torch.zeros_like(pb.score)
        args = (pb.desc, dev["q"], pb.q_off, pb.q_stored_start, pb.q_start, dev["k_store"], dev["v_store"], pb.n_store_tokens,
                dev["k_self"], dev["v_self"], pb.segs, pb.n_seg, pb.seg_stride, pb.batch, pb.tq, pb.max_kv_tokens, out, mass,
                score, pb.stride)
        if static:
            cf.cf_prefill_attention_static(*args, pb.dev_flag)
        else:
            pb.workspace.fill_(0xFF)
            cf.cf_prefill_attention(*args, pb.workspace, pb.ws_bytes, pb.dev_flag)
        torch.cuda.synchronize()
        assert pb.flags() == 0
        res.append((out, mass, score))
    (o0, m0, s0), (o1, m1, s1) = res
    assert torch.equal(o0, o1) and torch.equal(m0, m1) and torch.equal(s0, s1)
    assert float(m1[0, :int(pb.n_seg[0].item())].sum()) == pytest.approx(cfg.geometry.n_q_heads * cfg.tq, rel=1e-5)
    return pb


def test_static_scratch_entry_point_matches_the_workspace_one():
    big = wl.CONFIGS["llama2_7b_layer"]                                   # several splits: partial outputs go through the scratch
    pb = _both(big, seed=11)
    assert pb.ws_bytes <= cf.CF_STATIC_SCRATCH_BYTES
    small = wl.scaled(big, name="small", n_store_docs=3, docs_per_query=3, n_planted=1, tq=7, doc_len_range=(40, 90))
    _both(small, seed=12)                                                 # smaller, right after: stale contents must not matter
    gqa = wl.scaled(wl.CONFIGS["qwen2_1p5b_batch"], name="gqa_small", n_store_docs=80, batch=3)
    _both(gqa, seed=13)                                                   # the other 16-bit kernel
    _both(wl.CONFIGS["tiny_f32"], seed=14)                                # and the fp32 one


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    cfg = wl.scaled(wl.CONFIGS["qwen2_7b_layer"], name="too_big", batch=64, n_store_docs=3200)      # 61 MiB of partials
    st = wl.build_structure(cfg, seed=7015)
    pb = G.make_batch(cfg, st)
    assert pb.ws_bytes > cf.CF_STATIC_SCRATCH_BYTES
    g = cfg.geometry
    q = torch.zeros((cfg.batch * cfg.tq, g.n_q_heads, g.head_dim), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((cfg.batch * cfg.tq, g.n_kv_heads, g.head_dim), dtype=torch.bfloat16, device="cuda")
    store = torch.zeros((st.n_store_tokens, g.n_kv_heads, g.head_dim), dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, 7.0)
    with pytest.raises(cf.CacheFocusError) as err:
        cf.cf_prefill_attention_static(pb.desc, q, pb.q_off, 0, pb.q_start, store, store, pb.n_store_tokens, kv, kv, pb.segs, pb.n_seg,
                                       pb.seg_stride, pb.batch, pb.tq, pb.max_kv_tokens, out, pb.mass, None, pb.stride, pb.dev_flag)
    assert err.value.status == cf.CF_ERR_WORKSPACE and "library-owned" in err.value.message
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
