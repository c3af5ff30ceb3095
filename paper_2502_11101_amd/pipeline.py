"""Sequencing of the cf_* calls for Alg. 2, Phase 1 (per-layer prefill with pruning).

Nothing is computed here: this module owns the device-resident tables of a batch of
queries (candidate lists, accumulated scores S, positions, segment tables, workspace) and
issues the library calls in the order of Alg. 2.  All state lives in torch CUDA tensors;
nothing returns to the host between layers.
"""

from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as cf

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def to_device(x: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """Upload values that are already exactly representable in ``dtype``."""
    t = torch.from_numpy(np.ascontiguousarray(x))
    return t.to(device=device, dtype=TORCH_DTYPE[dtype])


def store_strides(n_store_tokens: int, n_kv_heads: int, head_dim: int, layout: str, pad_tokens: int = 0):
    """(store_token_stride, store_head_stride) in elements for a cache store laid out "token"-major
    [token][kv head][head_dim] or "head"-major [kv head][token (+ pad_tokens unused rows)][head_dim]."""
    if layout == "token":
        return n_kv_heads * head_dim, head_dim
    if layout == "head":
        return head_dim, (n_store_tokens + pad_tokens) * head_dim
    raise ValueError(f"unknown store layout {layout!r}")


def store_to_device(x: np.ndarray, dtype: str, layout: str, pad_tokens: int = 0, device="cuda") -> torch.Tensor:
    """Upload a [token][kv head][head_dim] array of the cache store in the given layout."""
    if layout == "token":
        return to_device(x, dtype, device)
    t = to_device(np.ascontiguousarray(x.transpose(1, 0, 2)), dtype, device)
    if pad_tokens:
        padded = torch.zeros((t.shape[0], t.shape[1] + pad_tokens, t.shape[2]), dtype=t.dtype, device=device)
        padded[:, :t.shape[1]].copy_(t)
        return padded
    return t


class PrefillBatch:
    """Device tables of ``batch`` queries, each with up to ``stride`` candidate documents.

    doc_tok_offset / doc_len: [batch, stride] host arrays (slot order = retriever rank).
    All queries have ``tq`` rows.  Positions for documents are [prefix_len, max_positions - tq).
    """

    def __init__(self, desc: cf.cf_layer_desc, doc_tok_offset: np.ndarray, doc_len: np.ndarray, tq: int,
                 prefix_len: int, doc_stored_start: int, n_store_tokens: int, q_stored_start: int = 0,
                 device="cuda"):
        self.desc = desc
        self.device = device
        self.batch, self.stride = doc_len.shape
        self.tq = tq
        self.prefix_len = prefix_len
        self.doc_stored_start = doc_stored_start
        self.q_stored_start = q_stored_start
        self.n_store_tokens = n_store_tokens
        self.seg_stride = self.stride + 2
        self.pos_begin = prefix_len
        self.pos_end = desc.max_positions - tq
        i32 = dict(dtype=torch.int32, device=device)
        self.doc_tok_offset = torch.from_numpy(np.ascontiguousarray(doc_tok_offset, dtype=np.int64)).to(device)
        self.doc_len = torch.from_numpy(np.ascontiguousarray(doc_len, dtype=np.int32)).to(device)
        self.q_off = torch.arange(0, (self.batch + 1) * tq, tq, **i32)
        self.cand = torch.arange(self.stride, **i32).repeat(self.batch, 1).contiguous()
        self.n_cand = torch.full((self.batch,), self.stride, **i32)
        self.keep_idx = torch.zeros((self.batch, self.stride), **i32)
        self.n_keep = torch.zeros((self.batch,), **i32)
        self.order = torch.zeros((self.batch, self.stride), **i32)
        self.new_start = torch.zeros((self.batch, self.stride), **i32)
        self.q_start = torch.zeros((self.batch,), **i32)
        self.n_reuse = torch.zeros((self.batch,), **i32)
        self.score = torch.zeros((self.batch, self.stride), dtype=torch.float32, device=device)
        self.mass = torch.zeros((self.batch, self.seg_stride), dtype=torch.float32, device=device)
        self.segs = torch.zeros((self.batch, self.seg_stride, 32), dtype=torch.uint8, device=device)
        self.n_seg = torch.zeros((self.batch,), **i32)
        # tables of the next layer, written by prune() and made current by advance()
        self.next_segs = torch.zeros_like(self.segs)
        self.next_n_seg = torch.zeros_like(self.n_seg)
        self.next_new_start = torch.zeros_like(self.new_start)
        self.next_q_start = torch.zeros_like(self.q_start)
        self.dev_flag = torch.zeros((1,), **i32)
        self.max_kv_tokens = int(prefix_len + doc_len.sum(axis=1).max() + tq)
        self.ws_bytes = cf.cf_prefill_workspace_bytes(desc, self.batch, tq, self.seg_stride, self.max_kv_tokens)
        self.workspace = torch.zeros(self.ws_bytes, dtype=torch.uint8, device=device)   # contents are scratch
        self.n_alive = self.stride
        self.n_pending = 0          # layers whose scores are still pending in the workspace (layer(defer=True))
        self._cache = None          # device addresses and the prune-step struct of the current tables (layer())

    # -- Alg. 2 init: every document is a candidate, placement order = retriever order
    def allocate_initial(self, force_n_reuse: int = 0) -> None:
        cf.cf_assign_positions(self.doc_len, self.cand, self.n_cand, self.batch, self.stride, self.pos_begin,
                               self.pos_end, cf.CF_ALLOC_SORT, force_n_reuse, self.new_start, self.q_start,
                               self.n_reuse, self.order, self.dev_flag)
        cf.cf_gather_segments(self.doc_tok_offset, self.doc_len, self.order, self.n_cand, self.new_start,
                              self.q_start, self.q_off, self.batch, self.stride, self.prefix_len,
                              self.doc_stored_start, self.q_stored_start, self.segs, self.n_seg, self.seg_stride,
                              self.dev_flag)

    # -- Alg. 2: layer_l on the re-positioned caches, S += s^l
    def attention(self, q, k_self, v_self, k_store, v_store, out, accumulate: bool = True) -> None:
        cf.cf_prefill_attention(self.desc, q, self.q_off, self.q_stored_start, self.q_start, k_store, v_store,
                                self.n_store_tokens, k_self, v_self, self.segs, self.n_seg, self.seg_stride,
                                self.batch, self.tq, self.max_kv_tokens, out, self.mass,
                                self.score if accumulate else None, self.stride, self.workspace, self.ws_bytes,
                                self.dev_flag)

    # -- Alg. 2: ids_sort = argsort(S); ids = prun(ids_sort); then Sec. 2.5 re-allocation.
    # Writes the next layer's tables; the current ones stay valid until advance().
    def prune(self, keep: int, strategy: int = cf.CF_ALLOC_SORT, normalise_by_len: bool = True,
              force_n_reuse: int = 0) -> None:
        cf.cf_prune_topk(self.score, self.doc_len if normalise_by_len else None, self.cand, self.n_cand, keep,
                         self.batch, self.stride, self.keep_idx, self.n_keep, self.dev_flag)
        if strategy == cf.CF_ALLOC_KEEP:
            self.next_new_start.copy_(self.new_start)
            self.next_q_start.copy_(self.q_start)
        cf.cf_assign_positions(self.doc_len, self.keep_idx, self.n_keep, self.batch, self.stride, self.pos_begin,
                               self.pos_end, strategy, force_n_reuse, self.next_new_start, self.next_q_start,
                               self.n_reuse, self.order, self.dev_flag)
        cf.cf_gather_segments(self.doc_tok_offset, self.doc_len, self.order, self.n_keep, self.next_new_start,
                              self.next_q_start, self.q_off, self.batch, self.stride, self.prefix_len,
                              self.doc_stored_start, self.q_stored_start, self.next_segs, self.next_n_seg,
                              self.seg_stride, self.dev_flag)
        self._pending_keep = keep

    # -- Alg. 2, one whole layer in one call: attention, S += s^l and, with `keep` given, the prune event
    # With `defer` (no prune event in this layer) the layer's scores stay pending in the workspace and are taken in, in
    # layer order, by the next call that does not defer — Alg. 2 reads S only at the prune events.
    def layer(self, q, k_self, v_self, k_store, v_store, out, keep: Optional[int] = None,
              strategy: int = cf.CF_ALLOC_SORT, normalise_by_len: bool = True, force_n_reuse: int = 0,
              defer: bool = False) -> None:
        # the tables' addresses only change in advance(): marshal them once, not per call
        c = self._cache
        if c is None:
            c = self._cache = dict(
                steps={}, q_off=self.q_off.data_ptr(), q_start=self.q_start.data_ptr(), segs=self.segs.data_ptr(),
                n_seg=self.n_seg.data_ptr(), mass=self.mass.data_ptr(), score=self.score.data_ptr(),
                workspace=self.workspace.data_ptr(), dev_flag=self.dev_flag.data_ptr())
        step = None
        if keep is not None:
            if strategy == cf.CF_ALLOC_KEEP:
                self.next_new_start.copy_(self.new_start)
                self.next_q_start.copy_(self.q_start)
            key = (keep, strategy, force_n_reuse, normalise_by_len, self.pos_begin, self.pos_end)
            step = c["steps"].get(key)
            if step is None:
                step = c["steps"][key] = cf.make_prune_step(
                    keep, strategy, force_n_reuse, normalise_by_len, self.stride, self.pos_begin, self.pos_end,
                    self.prefix_len, self.doc_stored_start, self.doc_tok_offset, self.doc_len, self.cand, self.n_cand,
                    self.keep_idx, self.n_keep, self.next_new_start, self.next_q_start, self.n_reuse, self.order,
                    self.next_segs, self.next_n_seg)
            self._pending_keep = keep
        cf.cf_prefill_layer(self.desc, q.data_ptr(), c["q_off"], self.q_stored_start, c["q_start"], k_store.data_ptr(),
                            v_store.data_ptr(), self.n_store_tokens, k_self.data_ptr(), v_self.data_ptr(), c["segs"],
                            c["n_seg"], self.seg_stride, self.batch, self.tq, self.max_kv_tokens, out.data_ptr(),
                            c["mass"], c["score"], self.stride, c["workspace"], self.ws_bytes, step, c["dev_flag"],
                            None, self.n_pending, defer)
        self.n_pending = self.n_pending + 1 if defer else 0

    # -- the survivors, in placement order, become the candidates of the following layers
    def advance(self) -> None:
        assert self.n_pending == 0, "scores cannot be pending across a change of the tables"
        self.cand, self.order = self.order, self.cand
        self.n_cand, self.n_keep = self.n_keep, self.n_cand
        self.segs, self.next_segs = self.next_segs, self.segs
        self.n_seg, self.next_n_seg = self.next_n_seg, self.n_seg
        self.new_start, self.next_new_start = self.next_new_start, self.new_start
        self.q_start, self.next_q_start = self.next_q_start, self.q_start
        self.n_alive = min(self._pending_keep, self.n_alive)
        self._cache = None

    def flags(self) -> int:
        return int(self.dev_flag.item())


class StoreBuilder:
    """Query-independent parallel document caching (Sec. 2.2, Alg. 2 "offline") for one layer.

    Every text of a batch (the shared prefix on its own, or the documents) attends to the first
    ``prefix_len`` tokens of the store and causally to itself at positions
    [position, position + len); its keys, moved to those positions, and its values are then
    written to the Context KV Cache Store at ``store_off``.  Sequencing only: the attention is
    cf_prefill_attention with each text as a "query" whose table lists the prefix and its own block, the
    write is cf_assemble_cache with the store as the target (Eq. 5 from the local position to the cached one).

    store_off / lens / positions: host arrays [n]; the fresh q / k / v of the texts are packed back to back,
    [sum lens][heads][head_dim], row t of a text carrying RoPE for its local position t.
    """

    def __init__(self, desc: cf.cf_layer_desc, store_off: np.ndarray, lens: np.ndarray, positions: np.ndarray,
                 prefix_len: int, n_store_tokens: int, device="cuda"):
        self.desc = desc
        self.n = len(lens)
        self.prefix_len = int(prefix_len)
        self.n_store_tokens = int(n_store_tokens)
        self.max_len = int(np.max(lens))
        q_off = np.zeros(self.n + 1, dtype=np.int64)
        q_off[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
        self.total = int(q_off[-1])
        i32 = dict(dtype=torch.int32, device=device)
        self.q_off = torch.from_numpy(q_off.astype(np.int32)).to(device)
        self.q_new = torch.from_numpy(np.asarray(positions, dtype=np.int32)).to(device)
        own = [(int(q_off[b]), int(lens[b]), 0, int(positions[b]), cf.CF_SEG_SELF, -1) for b in range(self.n)]
        pre = (0, self.prefix_len, 0, 0, cf.CF_SEG_PREFIX, -1)
        self.seg_stride = 2 if self.prefix_len else 1
        attend = [s for o in own for s in (([pre] if self.prefix_len else []) + [o])]
        self.attend_segs = cf.segments_to_device(cf.segments_array(attend), device)
        self.attend_n = torch.full((self.n,), self.seg_stride, **i32)
        self.write_segs = cf.segments_to_device(cf.segments_array(own), device)
        self.write_n = torch.ones((self.n,), **i32)
        self.final_off = torch.from_numpy(np.asarray(store_off, dtype=np.int64)).to(device)
        self.final_len = torch.zeros((self.n,), **i32)
        self.dev_flag = torch.zeros((1,), **i32)
        self.max_kv_tokens = self.prefix_len + self.max_len
        self.ws_bytes = cf.cf_prefill_workspace_bytes(desc, self.n, self.max_len, self.seg_stride, self.max_kv_tokens)
        self.workspace = torch.zeros(self.ws_bytes, dtype=torch.uint8, device=device)

    def attend(self, q, k, v, k_store, v_store, out) -> None:
        """out = attention of every text over the prefix (read from the store) and causally over itself."""
        cf.cf_prefill_attention(self.desc, q, self.q_off, 0, self.q_new, k_store if self.prefix_len else None,
                                v_store if self.prefix_len else None, self.n_store_tokens if self.prefix_len else 0, k, v,
                                self.attend_segs, self.attend_n, self.seg_stride, self.n, self.max_len, self.max_kv_tokens,
                                out, None, None, 1, self.workspace, self.ws_bytes, self.dev_flag)

    def write(self, k, v, k_store, v_store, store_token_stride: int, store_head_stride: int) -> None:
        """The texts' keys, rotated to their cached positions, and values go to their place in the store."""
        cf.cf_assemble_cache(self.desc, None, None, 0, k, v, self.q_off, self.write_segs, self.write_n, 1, self.n,
                             self.max_len, self.max_len, self.final_off, self.n_store_tokens, store_token_stride,
                             store_head_stride, k_store, v_store, self.final_len, None, self.dev_flag)

    def flags(self) -> int:
        return int(self.dev_flag.item())
