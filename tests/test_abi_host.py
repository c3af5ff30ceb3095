"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, and rejects bad host arguments before touching the device."""

import ctypes as C
import os
import re

import pytest

from paper_2502_11101_amd import binding as cf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "cachefocus.h")


def _declared():
    text = open(HEADER).read()
    return sorted(set(re.findall(r"CF_API[^;(]*?\b(cf_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = cf.load()
    names = _declared()
    assert set(names) == set(cf.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert cf.cf_version() >= 100


def test_struct_layouts_match_the_header():
    assert C.sizeof(cf.cf_layer_desc) == 56
    assert cf.SEGMENT_DTYPE.itemsize == 32
    assert cf.SEGMENT_DTYPE.fields["len"][1] == 8 and cf.SEGMENT_DTYPE.fields["doc"][1] == 24


def _desc(**kw):
    args = dict(n_q_heads=8, n_kv_heads=2, head_dim=128, dtype="bf16", rope_base=1.0e4, max_positions=4096)
    args.update(kw)
    return cf.make_desc(**args)


def _status(fn, *a, **k):
    with pytest.raises(cf.CacheFocusError) as e:
        fn(*a, **k)
    return e.value.status, e.value.message


FAKE = 0x1000  # never dereferenced: validation fails first


def test_descriptor_validation():
    for bad, code in [(_desc(n_q_heads=7), cf.CF_ERR_INVALID_ARG), (_desc(head_dim=100), cf.CF_ERR_UNSUPPORTED),
                      (_desc(head_dim=512), cf.CF_ERR_UNSUPPORTED), (_desc(dtype=9), cf.CF_ERR_INVALID_ARG),
                      (_desc(rope_base=0.5), cf.CF_ERR_INVALID_ARG), (_desc(max_positions=0), cf.CF_ERR_INVALID_ARG),
                      (_desc(rope_pairing=5), cf.CF_ERR_INVALID_ARG),
                      (_desc(store_token_stride=128), cf.CF_ERR_INVALID_ARG),          # one stride without the other
                      (_desc(store_token_stride=128, store_head_stride=64), cf.CF_ERR_INVALID_ARG),   # below head_dim
                      (_desc(store_token_stride=132, store_head_stride=1280), cf.CF_ERR_INVALID_ARG),  # not 16-byte rows
                      (_desc(store_token_stride=1 << 25, store_head_stride=128), cf.CF_ERR_UNSUPPORTED)]:
        st, msg = _status(cf.cf_reposition_keys, bad, FAKE, FAKE, FAKE, 1, 10, 1, stream=0)
        assert st == code and msg
        assert cf.cf_prefill_workspace_bytes(bad, 1, 8, 4, 100) == 0
    assert cf.cf_prefill_workspace_bytes(_desc(), 1, 8, 4, 100) > 0
    assert cf.cf_prefill_workspace_bytes(_desc(store_token_stride=128, store_head_stride=128 * 1000), 1, 8, 4, 100) > 0
    assert cf.cf_prefill_workspace_bytes(_desc(), 1, 8, 4, 100) % 256 == 0


def test_reposition_argument_checks():
    d = _desc()
    assert _status(cf.cf_reposition_keys, d, None, FAKE, FAKE, 1, 10, 1, stream=0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.cf_reposition_keys, d, FAKE + 4, FAKE, FAKE, 1, 10, 1, stream=0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.cf_reposition_keys, d, FAKE, FAKE, FAKE, -1, 10, 1, stream=0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.cf_reposition_keys, d, FAKE, FAKE, FAKE, 1, 10, 0, stream=0)[0] == cf.CF_ERR_INVALID_ARG
    cf.cf_reposition_keys(d, None, None, None, 0, 0, 1, stream=0)      # empty table: nothing to do


def test_prefill_argument_checks():
    d = _desc()

    def call(**kw):
        a = dict(desc=d, q=FAKE, q_off=FAKE, q_stored_start=0, q_new_start=FAKE, k_store=FAKE, v_store=FAKE,
                 n_store_tokens=100, k_self=FAKE, v_self=FAKE, segs=FAKE, n_seg=FAKE, seg_stride=4, batch=1,
                 max_tq=8, max_kv_tokens=100, out=FAKE, mass=FAKE, score_accum=None, score_stride=0,
                 workspace=0x10000, workspace_bytes=1 << 30, stream=0)
        a.update(kw)
        return _status(cf.cf_prefill_attention, **a)

    assert call(q=None)[0] == cf.CF_ERR_INVALID_ARG
    assert call(v_self=None)[0] == cf.CF_ERR_INVALID_ARG
    assert call(k_store=None, v_store=None)[0] == cf.CF_ERR_INVALID_ARG
    assert call(out=FAKE + 2)[0] == cf.CF_ERR_INVALID_ARG
    assert call(max_tq=0)[0] == cf.CF_ERR_INVALID_ARG
    assert call(seg_stride=0)[0] == cf.CF_ERR_INVALID_ARG
    assert call(score_accum=FAKE, score_stride=0)[0] == cf.CF_ERR_INVALID_ARG
    assert call(mass=None, score_accum=FAKE, score_stride=4)[0] == cf.CF_ERR_INVALID_ARG     # scores need the masses
    assert call(mass=None, workspace=None)[0] == cf.CF_ERR_WORKSPACE                          # outputs only: accepted so far
    assert call(q_stored_start=4096)[0] == cf.CF_ERR_RANGE
    assert call(workspace=None)[0] == cf.CF_ERR_WORKSPACE
    assert call(workspace_bytes=16)[0] == cf.CF_ERR_WORKSPACE
    assert call(workspace=0x10010)[0] == cf.CF_ERR_WORKSPACE
    st, msg = call(workspace_bytes=16)
    assert "workspace" in msg
    # more queries than a grid dimension holds: refused before any launch
    big = cf.cf_prefill_workspace_bytes(d, 70000, 8, 4, 100)
    st, msg = call(batch=70000, workspace_bytes=big)
    assert st == cf.CF_ERR_UNSUPPORTED and "65535" in msg
    # the kernel timing aid: nothing to report while it is off, switching it off twice is fine (no GPU needed)
    assert _status(cf.cf_profile_kernel_ms)[0] == cf.CF_ERR_INVALID_ARG
    cf.cf_profile_kernel_events(False)
    # an empty batch is a no-op and needs no GPU
    cf.cf_prefill_attention(d, None, None, 0, None, None, None, 0, None, None, None, None, 4, 0, 8, 0, None, None,
                            None, 0, None, 0, stream=0)


def test_deferred_score_and_static_scratch_argument_checks():
    """cf_prefill_layer's n_pending / defer and cf_prefill_attention_static's size limit are checked on the host, before
    any HIP call."""
    d = _desc()
    layer = dict(desc=d, q=FAKE, q_off=FAKE, q_stored_start=0, q_new_start=FAKE, k_store=FAKE, v_store=FAKE, n_store_tokens=100,
                 k_self=FAKE, v_self=FAKE, segs=FAKE, n_seg=FAKE, seg_stride=4, batch=1, max_tq=8, max_kv_tokens=100, out=FAKE,
                 mass=FAKE, score_accum=FAKE, score_stride=2, workspace=None, workspace_bytes=0, stream=0)
    assert _status(cf.cf_prefill_layer, **layer)[0] == cf.CF_ERR_WORKSPACE                    # everything else is accepted
    assert _status(cf.cf_prefill_layer, **dict(layer, n_pending=-1))[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.cf_prefill_layer, **dict(layer, n_pending=cf.CF_MAX_PENDING + 1))[0] == cf.CF_ERR_INVALID_ARG
    st, msg = _status(cf.cf_prefill_layer, **dict(layer, n_pending=cf.CF_MAX_PENDING, defer=True))
    assert st == cf.CF_ERR_INVALID_ARG and "flush" in msg
    assert _status(cf.cf_prefill_layer, **dict(layer, n_pending=cf.CF_MAX_PENDING))[0] == cf.CF_ERR_WORKSPACE
    assert _status(cf.cf_prefill_layer, **dict(layer, score_accum=None))[0] == cf.CF_ERR_INVALID_ARG
    # the library-owned scratch: a shape whose workspace exceeds it is refused with the sizes in the message
    big = _desc()
    big.n_q_heads, big.n_kv_heads = 28, 4
    need = cf.cf_prefill_workspace_bytes(big, 64, 64, 52, 8000)
    assert need > cf.CF_STATIC_SCRATCH_BYTES
    static = {k: v for k, v in layer.items() if k not in ("workspace", "workspace_bytes")}
    st, msg = _status(cf.cf_prefill_attention_static, **dict(static, desc=big, batch=64, max_tq=64, seg_stride=52, max_kv_tokens=8000))
    assert st == cf.CF_ERR_WORKSPACE and str(need) in msg and "library-owned" in msg
    # calibration kernels: bad arguments
    assert _status(cf.cf_calibrate, cf.CF_CALIB_READ, None, None, 1024, 16, 0, FAKE, stream=0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.cf_calibrate, cf.CF_CALIB_COPY, FAKE, FAKE, 1024, 16, 0, FAKE, stream=0)[0] == cf.CF_ERR_INVALID_ARG   # dst == src
    assert _status(cf.cf_calibrate, 9, FAKE, FAKE + 4096, 1024, 16, 0, FAKE, stream=0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.cf_calibrate, cf.CF_CALIB_MFMA_BF16, None, None, 0, 16, 0, FAKE, stream=0)[0] == cf.CF_ERR_INVALID_ARG     # iters 0


def test_prune_and_assign_argument_checks():
    assert _status(cf.cf_prune_topk, FAKE, None, FAKE, FAKE, 5, 1, 4, FAKE + 64, FAKE, stream=0)[0] == cf.CF_ERR_INVALID_ARG  # keep > stride
    assert _status(cf.cf_prune_topk, FAKE, None, FAKE, FAKE, -1, 1, 4, FAKE + 64, FAKE, stream=0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.cf_prune_topk, None, None, FAKE, FAKE, 1, 1, 4, FAKE + 64, FAKE, stream=0)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.cf_prune_topk, FAKE, None, FAKE, FAKE, 1, 1, 4, FAKE, FAKE, stream=0)[0] == cf.CF_ERR_INVALID_ARG       # alias
    assert _status(cf.cf_prune_topk, FAKE, None, FAKE, FAKE, 1, 1, 100000, FAKE + 64, FAKE, stream=0)[0] == cf.CF_ERR_INVALID_ARG

    def assign(**kw):
        a = dict(len_=FAKE, ranked=FAKE, n_ranked=FAKE, batch=1, stride=4, pos_begin=4, pos_end=100,
                 strategy=cf.CF_ALLOC_SORT, force_n_reuse=0, new_start=FAKE, q_start=FAKE, n_reuse=FAKE,
                 order=FAKE + 64, stream=0)
        a.update(kw)
        return _status(cf.cf_assign_positions, **a)

    assert assign(pos_end=4)[0] == cf.CF_ERR_RANGE
    assert assign(pos_begin=-1)[0] == cf.CF_ERR_RANGE
    assert assign(strategy=7)[0] == cf.CF_ERR_INVALID_ARG
    assert assign(force_n_reuse=-2)[0] == cf.CF_ERR_INVALID_ARG
    assert assign(new_start=None)[0] == cf.CF_ERR_INVALID_ARG
    assert assign(order=FAKE)[0] == cf.CF_ERR_INVALID_ARG
    assert _status(cf.cf_gather_segments, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 4, 0, 0, 0, FAKE, FAKE, 1,
                   stream=0)[0] == cf.CF_ERR_INVALID_ARG


def test_last_error_is_set():
    _status(cf.cf_prune_topk, FAKE, None, FAKE, FAKE, 9, 1, 4, FAKE + 64, FAKE, stream=0)
    assert "keep" in cf.cf_last_error()


def test_assemble_argument_checks():
    d = _desc()

    def call(**kw):
        a = dict(desc=d, k_store=FAKE, v_store=FAKE + 0x100, n_store_tokens=100, k_self=FAKE + 0x200, v_self=FAKE + 0x300,
                 q_off=FAKE, segs=FAKE, n_seg=FAKE, seg_stride=4, batch=1, max_tq=8, max_seg_len=64, final_off=FAKE,
                 final_capacity=500, final_token_stride=256, final_head_stride=128, k_final=FAKE + 0x400,
                 v_final=FAKE + 0x500, final_len=FAKE, stream=0)
        a.update(kw)
        return _status(cf.cf_assemble_cache, **a)

    assert call(k_final=None)[0] == cf.CF_ERR_INVALID_ARG
    assert call(final_len=None)[0] == cf.CF_ERR_INVALID_ARG
    assert call(v_self=None)[0] == cf.CF_ERR_INVALID_ARG                    # k_self without v_self
    assert call(final_token_stride=100)[0] == cf.CF_ERR_INVALID_ARG        # below head_dim
    assert call(final_head_stride=132)[0] == cf.CF_ERR_INVALID_ARG         # rows not 16-byte aligned
    assert call(k_final=FAKE)[0] == cf.CF_ERR_INVALID_ARG                  # aliases k_store
    assert call(v_final=FAKE + 0x400)[0] == cf.CF_ERR_INVALID_ARG          # aliases k_final
    assert call(k_final=FAKE + 0x404)[0] == cf.CF_ERR_INVALID_ARG          # misaligned
    assert call(max_seg_len=0)[0] == cf.CF_ERR_INVALID_ARG
    assert call(final_capacity=-1)[0] == cf.CF_ERR_INVALID_ARG
    # the kernel timing aid: nothing to report while it is off, switching it off twice is fine (no GPU needed)
    assert _status(cf.cf_profile_kernel_ms)[0] == cf.CF_ERR_INVALID_ARG
    cf.cf_profile_kernel_events(False)
    # an empty batch is a no-op and needs no GPU
    cf.cf_assemble_cache(d, None, None, 0, None, None, None, None, None, 4, 0, 8, 64, None, 0, 256, 128, None, None, None,
                         stream=0)


def test_hot_path_kernels_keep_everything_in_registers():
    """The build records what the compiler reports per kernel; the kernels of the hot path must not spill
    to scratch memory (the build itself refuses that, this keeps the record and the refusal in place)."""
    import json

    from paper_2502_11101_amd import build as cfbuild

    assert os.path.exists(cfbuild.RESOURCES), "run python -m paper_2502_11101_amd.build"
    usage = json.load(open(cfbuild.RESOURCES))
    for name in cfbuild.NO_SCRATCH:
        hits = {k: u for k, u in usage.items() if name in k}
        assert hits, name
        for k, u in hits.items():
            assert u["scratch_bytes"] == 0, (k, u)
    # both attention kernels are sized for one workgroup per CU: two wavefronts per SIMD
    for k, u in usage.items():
        if "attn_tile_kernel" in k or "attn_pipe_kernel" in k:
            assert u["waves_per_simd"] == 2 and u["vgprs"] + u["agprs"] <= 256, (k, u)


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py says so and exits without touching a device."""
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
