"""Pins of the CPU oracle against what the paper and the mathematics fix.

Every check here compares the oracle with something that is not the oracle:
complex multiplication, explicit 2x2 matrices, closed forms, torch's own
attention, triple-loop brute force, exhaustive slot marking, and the worked
examples the paper prints (tests/golden/).
"""

import cmath
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import cachefocus_oracle as orc
from paper_2502_11101_amd import workloads as wl
from tests import helpers as H

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ RoPE, Eq. 2 and Eq. 5
@pytest.mark.parametrize("pairing", ["half", "interleaved"])
@pytest.mark.parametrize("d,base", [(64, 1.0e4), (128, 1.0e6)])
def test_rotate_is_complex_multiplication(pairing, d, base):
    """Eq. 2's matrix acting on (a, b) is multiplication of a + ib by exp(i r)."""
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 3, d))
    delta = np.array([0, 1, -7, 1234, 32767])
    got = orc.rotate(x, delta[:, None], base, pairing)
    half = d // 2
    for t in range(5):
        for h in range(3):
            for m in range(half):
                ia, ib = (m, m + half) if pairing == "half" else (2 * m, 2 * m + 1)
                theta = base ** (-2.0 * m / d)
                z = complex(x[t, h, ia], x[t, h, ib]) * cmath.exp(1j * float(delta[t]) * theta)
                assert abs(got[t, h, ia] - z.real) < 1e-9
                assert abs(got[t, h, ib] - z.imag) < 1e-9


def test_rotation_sign_matches_the_printed_matrix():
    """R = [[cos, -sin], [sin, cos]]: the unit vector (1, 0) turns towards +b."""
    x = np.zeros((1, 4))
    x[0, 0] = 1.0          # pair 0 = (x[0], x[2]) under half-split pairing
    y = orc.rotate(x, 1, 1.0e4, "half")
    assert y[0, 0] == pytest.approx(math.cos(1.0))
    assert y[0, 2] == pytest.approx(math.sin(1.0))
    assert y[0, 1] == 0.0 and y[0, 3] == 0.0


def test_rotate_inverse_and_norm():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((40, 2, 128))
    delta = rng.integers(-4000, 4000, size=(40, 1))
    y = orc.rotate(x, delta, 1.0e4)
    back = orc.rotate(y, -delta, 1.0e4)
    assert np.max(np.abs(back - x)) < 1e-12
    half = 64
    n_in = x[..., :half] ** 2 + x[..., half:] ** 2
    n_out = y[..., :half] ** 2 + y[..., half:] ** 2
    assert np.max(np.abs(n_in - n_out)) < 1e-12


def test_zero_delta_is_bit_exact():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((7, 2, 64))
    assert np.array_equal(orc.rotate(x, 0, 1.0e6), x)


def test_eq5_both_forms_with_explicit_matrices():
    """k_j = R_j R_i^T k_i = R_j k_0 with R built as explicit 2x2 blocks."""
    d, base = 64, 1.0e4
    rng = np.random.default_rng(4)
    k0 = rng.standard_normal(d)
    half = d // 2

    def big_r(pos):
        r = np.zeros((d, d))
        for m in range(half):
            a = pos * base ** (-2.0 * m / d)
            r[m, m], r[m, m + half] = math.cos(a), -math.sin(a)
            r[m + half, m], r[m + half, m + half] = math.sin(a), math.cos(a)
        return r

    i, j = 37, 911
    k_i = big_r(i) @ k0
    direct = big_r(j) @ k0
    via = big_r(j) @ big_r(i).T @ k_i
    assert np.max(np.abs(direct - via)) < 1e-12
    seg = orc.Segment(0, 1, i, j, orc.KIND_DOC, 0)
    got = orc.reposition_keys(k_i.reshape(1, 1, d), [seg], base)[0, 0]
    assert np.max(np.abs(got - direct)) < 1e-12
    # a segment of several tokens keeps each token's own offset
    ks = np.stack([big_r(i + t) @ k0 for t in range(5)]).reshape(5, 1, d)
    seg = orc.Segment(0, 5, i, j, orc.KIND_DOC, 0)
    got = orc.reposition_keys(ks, [seg], base)
    for t in range(5):
        assert np.max(np.abs(got[t, 0] - big_r(j + t) @ k0)) < 1e-11


def test_reposition_leaves_unlisted_tokens_alone():
    rng = np.random.default_rng(5)
    k = rng.standard_normal((10, 2, 64))
    out = orc.reposition_keys(k, [orc.Segment(3, 4, 0, 9, orc.KIND_DOC, 0)], 1.0e4)
    assert np.array_equal(out[:3], k[:3]) and np.array_equal(out[7:], k[7:])
    assert not np.allclose(out[3:7], k[3:7])


# ------------------------------------------------------------------ attention, Eq. 1
def _tiny():
    cfg = wl.CONFIGS["tiny_f32"]
    st = wl.build_structure(cfg)
    t = wl.build_layer(cfg, st)
    segs, q_start, lens = H.initial_segments(cfg, st, 0)
    return cfg, st, t, segs, q_start, lens


def test_rows_sum_to_one_and_mass_totals():
    cfg, st, t, segs, q_start, _ = _tiny()
    out, mass, probs = H.oracle_query(cfg, st, t, 0, segs, q_start, return_probs=True)
    assert np.max(np.abs(probs.sum(axis=2) - 1.0)) < 1e-12
    g = cfg.geometry
    assert mass.sum() == pytest.approx(g.n_q_heads * cfg.tq, abs=1e-9)
    assert len(mass) == len(segs)
    # causal block: row t puts nothing on own-block tokens after t
    self_cols = probs[:, :, -cfg.tq:]
    for tt in range(cfg.tq):
        assert np.all(self_cols[:, tt, tt + 1:] == 0.0)
        assert np.all(self_cols[:, tt, :tt + 1] > 0.0)


def test_brute_force_tiny_configuration():
    """Triple loop with libm on the tiny configuration, written apart from the oracle."""
    cfg, st, t, segs, q_start, _ = _tiny()
    g = cfg.geometry
    d, half = g.head_dim, g.head_dim // 2
    out, mass = H.oracle_query(cfg, st, t, 0, segs, q_start)

    def rope(vec, delta):
        res = [0.0] * d
        for m in range(half):
            ang = delta * g.rope_base ** (-2.0 * m / d)
            a, b = float(vec[m]), float(vec[m + half])
            res[m] = a * math.cos(ang) - b * math.sin(ang)
            res[m + half] = a * math.sin(ang) + b * math.cos(ang)
        return res

    bf_out = np.zeros_like(out)
    bf_mass = np.zeros(len(segs))
    for h in range(g.n_q_heads):
        kv = h // g.group
        for tt in range(cfg.tq):
            qv = rope(t["q"][tt, h], q_start - 0)
            scores, vals, owner = [], [], []
            for si, seg in enumerate(segs):
                src_k = t["k_self"] if seg.kind == orc.KIND_SELF else t["k_store"]
                src_v = t["v_self"] if seg.kind == orc.KIND_SELF else t["v_store"]
                for n in range(seg.len):
                    if seg.kind == orc.KIND_SELF and n > tt:
                        continue
                    kvec = rope(src_k[seg.tok_offset + n, kv], seg.new_start - seg.stored_start)
                    scores.append(sum(a * b for a, b in zip(qv, kvec)) / math.sqrt(d))
                    vals.append(src_v[seg.tok_offset + n, kv])
                    owner.append(si)
            mx = max(scores)
            e = [math.exp(s - mx) for s in scores]
            z = sum(e)
            for p, v, o in zip(e, vals, owner):
                bf_out[tt, h] += (p / z) * v.astype(np.float64)
                bf_mass[o] += p / z
    assert np.max(np.abs(bf_out - out)) < 1e-10
    assert np.max(np.abs(bf_mass - mass)) < 1e-10


def test_uniform_closed_form_when_q_is_zero():
    cfg, st, t, segs, q_start, _ = _tiny()
    g = cfg.geometry
    t = dict(t)
    t["q"] = np.zeros_like(t["q"])
    out, mass = H.oracle_query(cfg, st, t, 0, segs, q_start)
    n_cached = sum(s.len for s in segs if s.kind != orc.KIND_SELF)
    expect_mass = np.zeros(len(segs))
    for tt in range(cfg.tq):
        n_vis = n_cached + tt + 1
        for si, seg in enumerate(segs):
            vis = seg.len if seg.kind != orc.KIND_SELF else tt + 1
            expect_mass[si] += g.n_q_heads * vis / n_vis
    assert np.max(np.abs(mass - expect_mass)) < 1e-10
    # out = mean of visible V
    v_cached = np.concatenate([H.f64(t["v_store"][s.tok_offset:s.tok_offset + s.len])
                               for s in segs if s.kind != orc.KIND_SELF])
    for tt in range(cfg.tq):
        vis_v = np.concatenate([v_cached, H.f64(t["v_self"][:tt + 1])])
        mean_v = vis_v.mean(axis=0)          # [Hkv, d]
        for h in range(g.n_q_heads):
            assert np.max(np.abs(out[tt, h] - mean_v[h // g.group])) < 1e-12


@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2)])
def test_reduces_to_library_sdpa(hq, hkv):
    """One document at its stored position and no own block is plain attention;
    the own block alone is causal attention (kv heads repeated for GQA)."""
    rng = np.random.default_rng(8)
    tq, n, d = 6, 19, 64
    q = rng.standard_normal((tq, hq, d))
    k = rng.standard_normal((n, hkv, d))
    v = rng.standard_normal((n, hkv, d))
    seg = [orc.Segment(0, n, 5, 5, orc.KIND_DOC, 0)]
    out, mass = orc.prefill_attention(q, 0, 0, k, v, None, None, seg, hkv, 1.0e4)
    rep = hq // hkv
    tq_, tk, tv = (torch.from_numpy(q).permute(1, 0, 2),
                   torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(rep, dim=0),
                   torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(rep, dim=0))
    ref = torch.nn.functional.scaled_dot_product_attention(tq_, tk, tv).permute(1, 0, 2).numpy()
    assert np.max(np.abs(out - ref)) < 1e-12
    assert mass[0] == pytest.approx(hq * tq)

    ks = rng.standard_normal((tq, hkv, d))
    vs = rng.standard_normal((tq, hkv, d))
    seg = [orc.Segment(0, tq, 0, 0, orc.KIND_SELF, -1)]
    out, _ = orc.prefill_attention(q, 0, 0, None, None, ks, vs, seg, hkv, 1.0e4)
    tk = torch.from_numpy(ks).permute(1, 0, 2).repeat_interleave(rep, dim=0)
    tv = torch.from_numpy(vs).permute(1, 0, 2).repeat_interleave(rep, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(tq_, tk, tv, is_causal=True)
    assert np.max(np.abs(out - ref.permute(1, 0, 2).numpy())) < 1e-12


@pytest.mark.parametrize("factor", [8.0, 0.05, 1.7])
def test_scale_argument_against_library_sdpa(factor):
    """Eq. 1's scale when it is not the default 1/sqrt(d): the ``scale`` argument of prefill_attention and of
    decode_attention against torch's scaled_dot_product_attention(scale=...) — cached document, causal own
    block (GQA, kv heads repeated), and the document-wise mass against probabilities formed from torch's
    softmax of the scaled scores."""
    rng = np.random.default_rng(81)
    tq, n, d, hq, hkv = 5, 23, 64, 6, 2
    scale = factor / np.sqrt(d)
    q = rng.standard_normal((tq, hq, d))
    k = rng.standard_normal((n, hkv, d))
    v = rng.standard_normal((n, hkv, d))
    ks = rng.standard_normal((tq, hkv, d))
    vs = rng.standard_normal((tq, hkv, d))
    rep = hq // hkv
    heads_first = lambda x, r=1: torch.from_numpy(x).permute(1, 0, 2).repeat_interleave(r, dim=0)
    sdpa = torch.nn.functional.scaled_dot_product_attention
    # one cached document at its stored position
    out, mass = orc.prefill_attention(q, 0, 0, k, v, None, None, [orc.Segment(0, n, 5, 5, orc.KIND_DOC, 0)], hkv, 1.0e4,
                                      scale=scale)
    ref = sdpa(heads_first(q), heads_first(k, rep), heads_first(v, rep), scale=scale).permute(1, 0, 2).numpy()
    assert np.max(np.abs(out - ref)) < 1e-12
    # the default differs from it (the argument is not ignored)
    plain, _ = orc.prefill_attention(q, 0, 0, k, v, None, None, [orc.Segment(0, n, 5, 5, orc.KIND_DOC, 0)], hkv, 1.0e4)
    assert np.max(np.abs(out - plain)) > 1e-3
    # the own block alone, causal
    out, _ = orc.prefill_attention(q, 0, 0, None, None, ks, vs, [orc.Segment(0, tq, 0, 0, orc.KIND_SELF, -1)], hkv, 1.0e4,
                                   scale=scale)
    ref = sdpa(heads_first(q), heads_first(ks, rep), heads_first(vs, rep), is_causal=True, scale=scale)
    assert np.max(np.abs(out - ref.permute(1, 0, 2).numpy())) < 1e-12
    # two documents: per-document mass from torch's softmax of the scaled scores
    segs = [orc.Segment(0, 9, 2, 2, orc.KIND_DOC, 0), orc.Segment(9, n - 9, 2, 2, orc.KIND_DOC, 1)]
    _, mass = orc.prefill_attention(q, 0, 0, k, v, None, None, segs, hkv, 1.0e4, scale=scale)
    probs = torch.softmax(scale * torch.einsum("htd,hnd->htn", heads_first(q), heads_first(k, rep)), dim=-1).numpy()
    assert mass[0] == pytest.approx(probs[:, :, :9].sum(), rel=1e-12)
    assert mass[1] == pytest.approx(probs[:, :, 9:].sum(), rel=1e-12)
    # decode-time attention over an assembled cache
    got = orc.decode_attention(q, k, v, hkv, scale=scale)
    ref = sdpa(heads_first(q), heads_first(k, rep), heads_first(v, rep), scale=scale).permute(1, 0, 2).numpy()
    assert np.max(np.abs(got - ref)) < 1e-12


def test_repositioned_attention_equals_attention_on_directly_roped_keys():
    """Keys cached at one position and moved by Eq. 5 give the same attention as
    keys that were given RoPE for the new position in the first place (torch SDPA
    on explicitly rotated tensors)."""
    rng = np.random.default_rng(9)
    tq, n, d, h = 4, 11, 64, 2
    base = 1.0e4
    q0 = rng.standard_normal((tq, h, d))
    k0 = rng.standard_normal((n, h, d))
    v = rng.standard_normal((n, h, d))
    stored, new, q_new = 3, 40, 77
    half = d // 2

    def rope_np(x, pos):      # complex form, separate from the oracle
        theta = base ** (-2.0 * np.arange(half) / d)
        z = (x[..., :half] + 1j * x[..., half:]) * np.exp(1j * pos[:, None, None] * theta)
        return np.concatenate([z.real, z.imag], axis=-1)

    k_stored = rope_np(k0, stored + np.arange(n))
    q_local = rope_np(q0, np.arange(tq))
    seg = [orc.Segment(0, n, stored, new, orc.KIND_DOC, 0)]
    out, _ = orc.prefill_attention(q_local, 0, q_new, k_stored, v, None, None, seg, h, base)
    k_direct = rope_np(k0, new + np.arange(n))
    q_direct = rope_np(q0, q_new + np.arange(tq))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q_direct).permute(1, 0, 2), torch.from_numpy(k_direct).permute(1, 0, 2),
        torch.from_numpy(v).permute(1, 0, 2)).permute(1, 0, 2).numpy()
    assert np.max(np.abs(out - ref)) < 1e-11


def test_common_position_shift_changes_nothing():
    """q_j^T k_i depends on j - i only: moving every new position and the query by
    the same amount leaves outputs and masses unchanged."""
    cfg, st, t, segs, q_start, _ = _tiny()
    out0, mass0 = H.oracle_query(cfg, st, t, 0, segs, q_start)
    segs1, q_start1, _ = H.initial_segments(cfg, st, 0, shift=1000)
    out1, mass1 = H.oracle_query(cfg, st, t, 0, segs1, q_start1)
    assert np.max(np.abs(out0 - out1)) < 1e-10
    assert np.max(np.abs(mass0 - mass1)) < 1e-10
    # ...whereas moving only the documents does change the result
    segs2 = [s._replace(new_start=s.new_start + 7) if s.kind == orc.KIND_DOC else s for s in segs]
    out2, _ = H.oracle_query(cfg, st, t, 0, segs2, q_start)
    assert np.max(np.abs(out0 - out2)) > 1e-6


# ------------------------------------------------------------------ pruning
def test_prune_topk_against_full_sort():
    rng = np.random.default_rng(10)
    for _ in range(50):
        n = int(rng.integers(1, 12))
        score = rng.integers(0, 5, size=n).astype(np.float32) / 4.0   # many ties
        lens = rng.integers(1, 4, size=n)
        cand = sorted(rng.permutation(n)[:int(rng.integers(1, n + 1))].tolist())
        keep = int(rng.integers(0, len(cand) + 1))
        got = orc.prune_topk(score, lens, cand, keep)
        # brute force: every permutation-free definition — pick the best repeatedly
        rest, ref = list(cand), []
        for _k in range(keep):
            best = rest[0]
            for c in rest[1:]:
                a = float(score[c]) * float(lens[best])
                b = float(score[best]) * float(lens[c])
                if a > b or (a == b and c < best):
                    best = c
            ref.append(best)
            rest.remove(best)
        assert got == ref


def test_equal_lengths_raw_and_normalised_rank_alike():
    rng = np.random.default_rng(11)
    score = rng.random(30).astype(np.float32)
    lens = np.full(30, 160)
    cand = list(range(30))
    assert orc.prune_topk(score, lens, cand, 12) == orc.prune_topk(score, None, cand, 12)


def test_prune_rejects_nan_and_bad_keep():
    with pytest.raises(ValueError):
        orc.prune_topk(np.array([1.0, np.nan]), None, [0, 1], 1)
    with pytest.raises(ValueError):
        orc.prune_topk(np.array([1.0, 2.0]), None, [0, 1], 3)


def test_keep_schedule_worked_example():
    with open(os.path.join(GOLDEN, "keep_schedule_example.json")) as f:
        ex = json.load(f)
    sched = orc.keep_schedule(ex["n_layers"], ex["prune_every"], ex["k"], ex["k_finish"])
    assert sched == ex["kept_after_each_event"]
    assert len(sched) == ex["events"]
    drops = [ex["k"] - sched[0]] + [a - b for a, b in zip(sched, sched[1:])]
    assert drops == [ex["k_prune_per_event"]] * ex["events"]
    # non-integer case still ends exactly at k_finish and never grows
    s = orc.keep_schedule(32, 4, 30, 5)
    assert s[-1] == 5 and all(a >= b for a, b in zip(s, s[1:]))


def test_fractional_keep_of_the_layer_stack():
    k, got = 30, []
    for _ in range(4):
        k = orc.keep_fraction(k, 0.6)
        got.append(k)
    assert got == [18, 11, 7, 5]


@pytest.mark.parametrize("name", ["tiny_f32", "llama2_7b_layer", "qwen2_7b_layer"])
def test_planted_documents_survive(name):
    cfg = wl.CONFIGS[name]
    st = wl.build_structure(cfg)
    t = wl.build_layer(cfg, st)
    segs, q_start, lens = H.initial_segments(cfg, st, 0)
    _, mass = H.oracle_query(cfg, st, t, 0, segs, q_start)
    score = H.doc_scores(segs, mass, cfg.docs_per_query)
    kept = orc.prune_topk(score, lens, list(range(cfg.docs_per_query)), cfg.keep)
    assert set(st.planted[0].tolist()) <= set(kept)
    g = cfg.geometry
    assert mass.sum() == pytest.approx(g.n_q_heads * cfg.tq, rel=1e-9)


# ------------------------------------------------------------------ position allocation, Eq. 6
def _check_allocation(lens, order, pos_begin, pos_end, new_start, q_start, n_reuse, per_group):
    """Exhaustive slot marking: inside a group no position is used twice, groups are
    back to back and end at the query, nothing leaves [pos_begin, q_start)."""
    groups = [order[i:i + per_group] for i in range(0, len(order), per_group)]
    assert len(groups) <= n_reuse
    longest = 0
    for grp in groups:
        used = set()
        for i in grp:
            rng_ = range(new_start[i], new_start[i] + lens[i])
            assert not (used & set(rng_))
            used |= set(rng_)
        assert max(used) == q_start - 1
        assert used == set(range(min(used), q_start))      # no holes
        assert min(used) >= pos_begin
        longest = max(longest, len(used))
        # first of the group is adjacent to the query
        assert new_start[grp[0]] + lens[grp[0]] == q_start
    assert q_start == pos_begin + longest
    assert q_start <= pos_end


def test_allocator_invariants_random():
    rng = np.random.default_rng(12)
    for _ in range(200):
        n = int(rng.integers(1, 40))
        lens = rng.integers(1, 50, size=n).tolist()
        order = rng.permutation(n).tolist()
        pos_begin = int(rng.integers(0, 20))
        l_c = max(lens)
        pos_end = pos_begin + int(rng.integers(l_c, l_c * n + 10))
        ns, q_start, n_reuse = orc.assign_positions(lens, order, pos_begin, pos_end)
        cap = (pos_end - pos_begin) // l_c
        assert n_reuse == -(-n // cap)                        # Eq. 6, minimal
        _check_allocation(lens, order, pos_begin, pos_end, ns, q_start, n_reuse, -(-n // n_reuse))
        # "align" places the same survivors in ascending slot order
        ns_a, q_a, _ = orc.assign_positions(lens, order, pos_begin, pos_end, orc.STRATEGY_ALIGN)
        _check_allocation(lens, sorted(order), pos_begin, pos_end, ns_a, q_a, n_reuse,
                          -(-n // n_reuse))


def test_allocator_paper_examples():
    with open(os.path.join(GOLDEN, "n_reuse_examples.json")) as f:
        ex = json.load(f)
    e = ex["k20_reuse_k_over_5"]
    lens = [160] * e["k"]
    ns, q_start, n_reuse = orc.assign_positions(lens, list(range(e["k"])), 32, 4096 - 48,
                                                force_n_reuse=e["n_reuse"])
    assert n_reuse == e["n_reuse"]
    starts = sorted(set(ns.values()))
    assert len(starts) == e["windows_with_continuous_positions"]     # 5 distinct windows ...
    for s in starts:
        assert sum(1 for v in ns.values() if v == s) == e["n_reuse"]  # ... each used 4 times
    assert q_start == 32 + 5 * 160
    # Qwen2's 32K range: 50 documents of at most 200 tokens need no reuse
    e = ex["qwen2_32k"]
    lens = [200] * 50
    ns, q_start, n_reuse = orc.assign_positions(lens, list(range(50)), 32,
                                                e["max_positions"] - 64)
    assert n_reuse == e["n_reuse"]
    assert sorted(ns.values()) == [32 + 200 * i for i in range(50)]   # contiguous packing
    assert q_start == 32 + 50 * 200
    # LLaMA-2's 4K range with 30 x 160 tokens needs two groups
    _, _, n_reuse = orc.assign_positions([160] * 30, list(range(30)), 32, 4096 - 48)
    assert n_reuse == 2


def test_allocator_tiny_configuration_contiguous_after_prefix():
    ns, q_start, n_reuse = orc.assign_positions([32] * 4, [2, 0], 4, 4096 - 8)
    assert n_reuse == 1 and q_start == 68
    assert ns == {2: 36, 0: 4}            # best document right before the query
    ns, q_start, _ = orc.assign_positions([32] * 4, [2, 0], 4, 4096 - 8, orc.STRATEGY_ALIGN)
    assert ns == {0: 36, 2: 4} and q_start == 68


def test_allocator_errors():
    with pytest.raises(ValueError):
        orc.assign_positions([100], [0], 0, 50)                     # longer than the range
    with pytest.raises(ValueError):
        orc.assign_positions([10] * 10, list(range(10)), 0, 50, force_n_reuse=1)   # overflow


# ------------------------------------------------------------------ Alg. 2 driver
def _small_stack(strategy):
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], n_store_docs=6, docs_per_query=6, n_planted=2,
                    n_layers=6)
    st = wl.build_structure(cfg, seed=77)
    g = cfg.geometry
    lens = [int(x) for x in st.doc_lens]

    def layer_inputs(layer):
        return wl.build_layer(cfg, st, layer, seed=500 + layer)

    return cfg, st, orc.layer_adaptive_prefill(
        cfg.n_layers, layer_inputs, lens, st.doc_off[:-1], cfg.doc_stored_start, cfg.prefix_len,
        cfg.tq, g.n_kv_heads, g.rope_base, g.max_positions, {1: 4, 3: 2}, strategy)


def test_strategies_agree_until_first_prune_takes_effect():
    """Rows of the re-ranking table at the first listed layer are identical for
    pruning alone, "align" and "sort": nothing can differ before a prune acts."""
    runs = {s: _small_stack(s)[2] for s in (orc.STRATEGY_KEEP, orc.STRATEGY_ALIGN,
                                            orc.STRATEGY_SORT)}
    ref = runs[orc.STRATEGY_KEEP][0]
    for s, (trace, ids, score) in runs.items():
        for layer in (0, 1):
            assert np.array_equal(trace[layer]["out"], ref[layer]["out"])
            assert trace[layer]["segments"] == ref[layer]["segments"]
    # afterwards the strategies do place documents differently
    a = runs[orc.STRATEGY_KEEP][0][2]["segments"]
    b = runs[orc.STRATEGY_SORT][0][2]["segments"]
    assert a != b


def test_driver_invariants():
    cfg, st, (trace, ids, score) = _small_stack(orc.STRATEGY_SORT)
    prev_ids, prev_score = None, np.zeros(6)
    for layer, rec in enumerate(trace):
        assert np.all(rec["score"] >= prev_score)                 # S only grows
        prev_score = rec["score"]
        if prev_ids is not None:
            assert set(rec["ids"]) <= set(prev_ids)               # ids only shrink
            if layer - 1 not in (1, 3):
                assert rec["ids"] == prev_ids                     # and only at prune layers
        prev_ids = rec["ids"]
        g = cfg.geometry
        assert rec["mass"].sum() == pytest.approx(g.n_q_heads * cfg.tq, rel=1e-9)
    assert [len(r["ids"]) for r in trace] == [6, 6, 4, 4, 2, 2]
    assert len(ids) == 2


# ------------------------------------------------------------------ Alg. 2 Phase 2: the assembled cache
def _phase2_case(seed=5):
    rng = np.random.default_rng(seed)
    hq, hkv, d, base, tq = 4, 2, 64, 1.0e4, 3
    n_store = 90
    k_store = rng.standard_normal((n_store, hkv, d))
    v_store = rng.standard_normal((n_store, hkv, d))
    k_self = rng.standard_normal((tq, hkv, d))
    v_self = rng.standard_normal((tq, hkv, d))
    # keys as stored: RoPE at the stored positions applied to "raw" keys, so that direct RoPE at the
    # final position is available as an independent reference
    segs = [orc.Segment(0, 6, 0, 0, orc.KIND_PREFIX, -1), orc.Segment(40, 17, 6, 31, orc.KIND_DOC, 1),
            orc.Segment(10, 25, 6, 6, orc.KIND_DOC, 0), orc.Segment(0, tq, 0, 48, orc.KIND_SELF, -1)]
    return hq, hkv, d, base, tq, k_store, v_store, k_self, v_self, segs


def test_assembled_cache_layout_positions_and_zero_shift():
    hq, hkv, d, base, tq, k_store, v_store, k_self, v_self, segs = _phase2_case()
    k_f, v_f, pos = orc.assemble_final_cache(k_store, v_store, k_self, v_self, segs, tq, base)
    assert k_f.shape == v_f.shape == (6 + 17 + 25 + tq, hkv, d)
    assert pos.tolist() == list(range(0, 6)) + list(range(31, 48)) + list(range(6, 31)) + list(range(48, 48 + tq))
    np.testing.assert_array_equal(k_f[:6], k_store[:6])                       # zero shift: an exact copy
    np.testing.assert_array_equal(k_f[23:48], k_store[10:35])                 # stored at 6, stays at 6
    np.testing.assert_array_equal(v_f[6:23], v_store[40:57])                  # values are copied, never rotated
    np.testing.assert_array_equal(v_f[48:], v_self[:tq])
    # a moved key is RoPE applied directly at the final position to the un-rotated key (Eq. 5, both forms)
    raw = orc.rotate(k_store[40:57], -(6 + np.arange(17))[:, None], base)
    direct = orc.rotate(raw, (31 + np.arange(17))[:, None], base)
    np.testing.assert_allclose(k_f[6:23], direct, atol=1e-12)
    np.testing.assert_allclose(np.linalg.norm(k_f, axis=-1), np.linalg.norm(
        np.concatenate([k_store[:6], k_store[40:57], k_store[10:35], k_self[:tq]]), axis=-1), rtol=1e-12)


def test_decode_over_assembled_cache_equals_prefill_on_the_store():
    """Plain attention of an absolutely positioned query over C_final gives what the prefill path gives on
    the original store with the same segment table: scores depend on relative positions only (Eq. 2)."""
    hq, hkv, d, base, tq, k_store, v_store, k_self, v_self, segs = _phase2_case(6)
    rng = np.random.default_rng(60)
    k_f, v_f, pos = orc.assemble_final_cache(k_store, v_store, k_self, v_self, segs, tq, base)
    q_raw = rng.standard_normal((1, hq, d))                 # a decode-step query before RoPE
    p_new = 48 + tq                                         # it sits right after the query block
    q_abs = orc.rotate(q_raw, p_new, base)
    got = orc.decode_attention(q_abs, k_f, v_f, hkv)
    # the same through the prefill definition: the new token as a one-row query stored at position 0 and
    # placed at p_new; the earlier query block is now an ordinary, fully visible cached segment
    segs_dec = [s if s.kind != orc.KIND_SELF else orc.Segment(n_store_off, s.len, s.stored_start, s.new_start, orc.KIND_DOC, -1)
                for s, n_store_off in ((s, 90) for s in segs)]
    store_k = np.concatenate([k_store, k_self])
    store_v = np.concatenate([v_store, v_self])
    ref, _ = orc.prefill_attention(q_raw, 0, p_new, store_k, store_v, None, None, segs_dec, hkv, base)
    np.testing.assert_allclose(got, ref, atol=1e-12)
    # and against torch's attention on the assembled cache
    qt = torch.from_numpy(q_abs).permute(1, 0, 2)[None]
    kt = torch.from_numpy(np.repeat(k_f, hq // hkv, axis=1)).permute(1, 0, 2)[None]
    vt = torch.from_numpy(np.repeat(v_f, hq // hkv, axis=1)).permute(1, 0, 2)[None]
    sdpa = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, sdpa, atol=1e-12)
