/*
 * cachefocus.h — C ABI of the MI355X (gfx950) library for the CacheFocus
 * query pre-fill over a Context KV Cache Store.
 *
 * One transformer layer at a time, a query attends a shared-prefix cache, a set of
 * independently cached document KV blocks and its own causal block.  Before the
 * attention the cached keys are moved from the positions they were cached at to
 * newly allocated positions by re-rotating their RoPE phase (Cache Re-Positioning,
 * Sec. 2.3, Eq. 5).  The same attention yields a per-document attention mass
 * (footnote of Sec. 2.4) that is accumulated over layers and drives Layer-Adaptive
 * Cache Pruning (Alg. 2) and the position allocation of the survivors (Eq. 6,
 * Sec. 2.5).
 *
 * Conventions for every call
 *   - "device" pointers are HIP device memory owned by the caller; "host" values are
 *     passed by value or as host pointers.  The library allocates no device memory and
 *     never frees or retains caller memory.  What it keeps between calls: the thread-local
 *     text of cf_last_error(), the per-device address of the buffer behind
 *     cf_prefill_attention_static, and — only while the measurement aids at the end of
 *     this header are switched on — their events.  None of it changes a call's results.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue work and return; outputs are valid once the stream reaches that point.
 *   - Host arguments are validated before any HIP call; a failed validation returns a
 *     negative cf_status and launches nothing.  Device-resident tables cannot be
 *     checked on the host: kernels guard them (no out-of-range access is made on the
 *     strength of a table entry beyond the bounds the host arguments state) and
 *     report through the optional `dev_flag` word (device int32, OR-ed with
 *     cf_dev_flag bits, never cleared by the library).
 *   - Tensors are row-major [token, head, head_dim]; base pointers 16-byte aligned.
 *   - cf_last_error() returns a thread-local message for the last non-OK status.
 */
#ifndef CACHEFOCUS_H
#define CACHEFOCUS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CF_API __attribute__((visibility("default")))

typedef enum cf_status {
    CF_OK = 0,
    CF_ERR_INVALID_ARG = -1,  /* null pointer, negative size, misaligned base, keep > stride ...   */
    CF_ERR_UNSUPPORTED = -2,  /* head_dim / dtype / pairing combination no kernel exists for, or a size past a kernel's limit */
    CF_ERR_RANGE = -3,        /* positions outside [0, max_positions), range too small              */
    CF_ERR_WORKSPACE = -4,    /* workspace missing or smaller than cf_prefill_workspace_bytes()     */
    CF_ERR_DEVICE = -5        /* a HIP runtime call failed; see cf_last_error()                     */
} cf_status;

typedef enum cf_dtype { CF_F32 = 0, CF_BF16 = 1, CF_F16 = 2 } cf_dtype;

/* Which two elements of a head vector form the 2-D slice m of Eq. 2. */
typedef enum cf_rope_pairing {
    CF_ROPE_HALF = 0,        /* (m, m + head_dim/2) */
    CF_ROPE_INTERLEAVED = 1  /* (2m, 2m + 1)        */
} cf_rope_pairing;

typedef enum cf_seg_kind {
    CF_SEG_PREFIX = 0,  /* shared prefix cache: visible to every query row, never pruned          */
    CF_SEG_DOC = 1,     /* one cached document: visible to every query row                        */
    CF_SEG_SELF = 2     /* the query's own block: row t sees tokens 0..t (causal, footnote Eq. 1) */
} cf_seg_kind;

typedef enum cf_alloc_strategy {
    CF_ALLOC_KEEP = 0,   /* survivors keep their old positions (pruning alone)                     */
    CF_ALLOC_ALIGN = 1,  /* Dynamic Positional Allocation: survivors re-packed in retriever order  */
    CF_ALLOC_SORT = 2    /* Attention-Guided Allocation: survivors re-packed by accumulated score  */
} cf_alloc_strategy;

/* Bits OR-ed into *dev_flag by kernels that find a bad device-resident table entry. */
typedef enum cf_dev_flag {
    CF_FLAG_BAD_SEGMENT = 1,    /* negative length/offset, unknown kind, more segments than stride */
    CF_FLAG_NONFINITE_SCORE = 2,/* NaN/Inf in the score array handed to cf_prune_topk              */
    CF_FLAG_DOC_TOO_LONG = 4,   /* a document longer than the positional range                     */
    CF_FLAG_POS_OVERFLOW = 8,   /* an allocation that does not fit [pos_begin, pos_end)            */
    CF_FLAG_BAD_INDEX = 16,     /* candidate / ranked index outside [0, stride)                    */
    CF_FLAG_POS_RANGE = 32      /* a segment or query whose stored or new positions leave [0, max_positions) */
} cf_dev_flag;

/* Geometry of one attention layer (host struct, passed by pointer, read during the call). */
typedef struct cf_layer_desc {
    int32_t n_q_heads;
    int32_t n_kv_heads;      /* divides n_q_heads; q head h uses kv head h / (n_q_heads/n_kv_heads) */
    int32_t head_dim;        /* multiple of 16, <= 256 (the 16-bit MFMA kernels serve 128)         */
    int32_t dtype;           /* cf_dtype of q, k, v and out                                         */
    int32_t rope_pairing;    /* cf_rope_pairing                                                     */
    int32_t max_positions;   /* positions are valid in [0, max_positions)                           */
    double  rope_base;       /* theta_m = rope_base^(-2m/head_dim)                                  */
    float   softmax_scale;   /* 0 => 1/sqrt(head_dim) (Eq. 1)                                       */
    int32_t reserved;        /* must be 0                                                           */
    /* Layout of the cache store (k_store, v_store; k_in, k_out of cf_reposition_keys), in elements:
     * channel c of kv head h of token t sits at t*store_token_stride + h*store_head_stride + c.
     * Both 0: token-major [token][n_kv_heads][head_dim].  Head-major [n_kv_heads][tokens][head_dim]
     * (token stride head_dim, head stride tokens*head_dim) makes every (head, document) run
     * contiguous, which is what the streaming kernels read fastest.  Both must be multiples of 8 and
     * at least head_dim.  q, out, k_self and v_self are always token-major. */
    int64_t store_token_stride;
    int64_t store_head_stride;
} cf_layer_desc;

/* One run of cached tokens attended by a query (device-resident table entry, 32 bytes).
 * Token t of the segment was cached with RoPE for position stored_start + t and is attended
 * at position new_start + t: its key is rotated by (new_start - stored_start) positions. */
typedef struct cf_segment {
    int64_t tok_offset;    /* first token: into k_store/v_store (PREFIX, DOC) or k_self/v_self (SELF) */
    int32_t len;           /* tokens, >= 0                                                            */
    int32_t stored_start;
    int32_t new_start;
    int32_t kind;          /* cf_seg_kind                                                             */
    int32_t doc;           /* query-local document slot whose score this segment feeds, or -1         */
    int32_t reserved;
} cf_segment;

/* ---------------------------------------------------------------------------------------------
 * Cache Re-Positioning, materialised (Sec. 2.3, Eq. 5: k_j = R_j R_i^T k_i).
 * For every listed segment, every token t, every kv head: rotate the key by
 * (new_start - stored_start) positions and write it to k_out at the same token offset.
 *   k_in, k_out  device [tokens, n_kv_heads, head_dim] of desc->dtype; k_out may alias k_in.
 *                Tokens outside the listed segments are not touched.
 *   segs         device [n_seg]; kind is ignored, all offsets index k_in/k_out.
 *   n_store_tokens  host: number of tokens in k_in/k_out; entries reaching beyond it are
 *                skipped and flagged CF_FLAG_BAD_SEGMENT.
 *   max_seg_len  host: launch-sizing hint (>= 1); longer segments are still processed fully.
 * A rotation by 0 positions copies bit-exactly.  Rotation arithmetic is fp32 with the angle
 * reduced in fp64; the result is rounded once (RNE) to desc->dtype.
 */
CF_API cf_status cf_reposition_keys(const cf_layer_desc* desc, const void* k_in, void* k_out,
                             const cf_segment* segs, int32_t n_seg, int64_t n_store_tokens,
                             int32_t max_seg_len, int32_t* dev_flag, void* stream);

/* Bytes of device workspace cf_prefill_attention needs for these bounds (host only, no HIP
 * call).  Returns 0 for an invalid/unsupported descriptor. */
CF_API size_t cf_prefill_workspace_bytes(const cf_layer_desc* desc, int32_t batch, int32_t max_tq,
                                  int32_t seg_stride, int64_t max_kv_tokens);

/* ---------------------------------------------------------------------------------------------
 * One layer's query pre-fill attention (Eq. 1; the layer_l step of Alg. 2) with the cached keys
 * re-positioned on the fly (Eq. 5) and the document-wise attention score as a by-product.
 *
 * For query b (rows q_off[b] .. q_off[b+1]-1), row t, q head h (kv head h/G):
 *   scores over every token of every PREFIX/DOC segment of the query and tokens 0..t of its
 *   SELF segment, each key taken at position new_start + token and the query row at position
 *   q_new_start[b] + t; one softmax over all of them; out = sum p * v.
 *   mass[b*seg_stride + s] = sum over q heads, rows and tokens of segment s of p   (overwritten)
 *   score_accum[b*score_stride + segs[s].doc] += mass of s   for segments with doc >= 0 (S += s^l)
 *
 * Only relative positions enter a RoPE score, so the kernels leave q as it is and rotate each
 * key by (new_start - stored_start) - (q_new_start[b] - q_stored_start); rotated keys live in
 * on-chip memory only and are never written back.
 *
 *   q            device [q_off[batch], n_q_heads, head_dim]; row t of query b carries RoPE for
 *                position q_stored_start + t (0 = local positions)
 *   q_off        device int32 [batch+1], ascending; query lengths <= max_tq
 *   q_new_start  device int32 [batch]: position at which row 0 of each query is attended
 *                (the q_start written by cf_assign_positions)
 *   k_store, v_store  device [n_store_tokens, n_kv_heads, head_dim]: the Context KV Cache Store
 *   k_self, v_self    device [q_off[batch], n_kv_heads, head_dim] (may be NULL if no SELF segment)
 *   segs         device [batch*seg_stride]; query b uses entries b*seg_stride .. + n_seg[b]-1
 *   n_seg        device int32 [batch], each <= seg_stride
 *   max_kv_tokens host: upper bound on the tokens one query attends (sizing only)
 *   out          device [q_off[batch], n_q_heads, head_dim], desc->dtype
 *   mass         device float [batch*seg_stride]; may be NULL when score_accum is NULL too (outputs only, as
 *                in a decode step, Alg. 2 Phase 3: no mass is reduced)
 *   score_accum  device float [batch*score_stride] or NULL
 *   workspace    device, >= cf_prefill_workspace_bytes(desc, batch, max_tq, seg_stride, max_kv_tokens),
 *                256-byte aligned; contents are scratch
 * Reductions run in a fixed order: the same inputs give bit-identical outputs.
 * Limits of the 16-bit kernels (CF_ERR_UNSUPPORTED beyond them): batch <= 65535 and
 * n_kv_heads * ceil(n_q_heads / n_kv_heads * max_tq / 192) <= 65535 (grid dimensions).
 */
CF_API cf_status cf_prefill_attention(const cf_layer_desc* desc,
                               const void* q, const int32_t* q_off, int32_t q_stored_start,
                               const int32_t* q_new_start,
                               const void* k_store, const void* v_store, int64_t n_store_tokens,
                               const void* k_self, const void* v_self,
                               const cf_segment* segs, const int32_t* n_seg, int32_t seg_stride,
                               int32_t batch, int32_t max_tq, int64_t max_kv_tokens,
                               void* out, float* mass, float* score_accum, int32_t score_stride,
                               void* workspace, size_t workspace_bytes,
                               int32_t* dev_flag, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cf_prefill_attention for callers that cannot allocate device memory or hand in a workspace: code that
 * runs under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments,
 * same kernels and bit-identical results, but the partial results of the splits live in a buffer the
 * library owns: a file-scope device array of CF_STATIC_SCRATCH_BYTES that every GPU the library runs on
 * holds until the process ends.  The call itself allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine).
 *   - Shapes whose workspace (cf_prefill_workspace_bytes) exceeds CF_STATIC_SCRATCH_BYTES are
 *     rejected with CF_ERR_WORKSPACE before anything is launched.
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress, once per device,
 *     with that device current); make that call outside stream capture.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *     streams or threads) race and must be serialised by the caller.  The array keeps the last call's
 *     contents; nothing in it needs clearing between calls.
 */
#define CF_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
CF_API cf_status cf_prefill_attention_static(const cf_layer_desc* desc,
                               const void* q, const int32_t* q_off, int32_t q_stored_start,
                               const int32_t* q_new_start,
                               const void* k_store, const void* v_store, int64_t n_store_tokens,
                               const void* k_self, const void* v_self,
                               const cf_segment* segs, const int32_t* n_seg, int32_t seg_stride,
                               int32_t batch, int32_t max_tq, int64_t max_kv_tokens,
                               void* out, float* mass, float* score_accum, int32_t score_stride,
                               int32_t* dev_flag, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Layer-Adaptive Cache Pruning, the ranking step (Alg. 2: ids_sort = argsort(S); ids = prun(ids_sort)).
 * Per query b: rank the candidate slots cand[b*stride .. + n_cand[b]) by accumulated score,
 * descending, ties to the lower slot index, and write the best min(keep, n_cand[b]) to
 * keep_idx[b*stride ..], best first; n_keep[b] receives their number.
 * With `len` given the ranking key is score/len (the same order as the raw score when all
 * lengths are equal, the paper's fixed-length passages), compared exactly as
 * score_i*len_j vs score_j*len_i in fp64.
 *   score     device float [batch*stride]   (slot-indexed)
 *   len       device int32 [batch*stride] or NULL
 *   cand      device int32 [batch*stride], n_cand device int32 [batch]
 *   keep      host, 0 <= keep <= stride
 *   keep_idx  device int32 [batch*stride] (must not alias cand), n_keep device int32 [batch]
 * Integer results are exact: the same score array always yields the same indices.
 */
CF_API cf_status cf_prune_topk(const float* score, const int32_t* len, const int32_t* cand,
                        const int32_t* n_cand, int32_t keep, int32_t batch, int32_t stride,
                        int32_t* keep_idx, int32_t* n_keep, int32_t* dev_flag, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Adaptive Re-Positioning (Eq. 6) with the allocation strategies of Sec. 2.5.
 * Per query b with survivors ranked[b*stride .. + n_ranked[b]) (best first):
 *   l_C = longest survivor, capacity = floor((pos_end - pos_begin)/l_C),
 *   N_reuse = ceil(n/capacity) (or force_n_reuse > 0), placement order = ranked (SORT) or the
 *   survivors by ascending slot (ALIGN), cut into N_reuse contiguous chunks of ceil(n/N_reuse);
 *   inside a chunk documents sit back to back and the first ends where the query starts, so
 *   q_start = pos_begin + longest chunk span and every chunk ends at q_start.
 * Outputs (device): new_start[b*stride + slot] for survivors (others untouched), q_start[b],
 * n_reuse[b], order[b*stride ..] = the placement order (first = nearest the query).
 * CF_ALLOC_KEEP writes only `order` (= the survivors by ascending slot); positions and q_start
 * stay as they are.  A document longer than the range or a forced N_reuse that does not fit
 * sets CF_FLAG_DOC_TOO_LONG / CF_FLAG_POS_OVERFLOW and leaves that query's outputs untouched.
 *   len       device int32 [batch*stride]
 *   ranked    device int32 [batch*stride], n_ranked device int32 [batch]
 *   pos_begin, pos_end  host: documents may occupy [pos_begin, pos_end); 0 <= pos_begin < pos_end
 */
CF_API cf_status cf_assign_positions(const int32_t* len, const int32_t* ranked, const int32_t* n_ranked,
                              int32_t batch, int32_t stride, int32_t pos_begin, int32_t pos_end,
                              int32_t strategy, int32_t force_n_reuse,
                              int32_t* new_start, int32_t* q_start, int32_t* n_reuse,
                              int32_t* order, int32_t* dev_flag, void* stream);

/* ---------------------------------------------------------------------------------------------
 * The logical concat of Alg. 2 (C_pre = concat(prefix, {C_di : i in ids})): writes each query's
 * segment table — prefix, the surviving documents in placement order, the query's own block —
 * without copying any K/V bytes.
 *   doc_tok_offset device int64 [batch*stride]: first store token of the document in each slot
 *   len            device int32 [batch*stride]
 *   order, n_order device: the slots to include (from cf_assign_positions)
 *   new_start      device int32 [batch*stride]; q_start device int32 [batch]
 *   q_off          device int32 [batch+1]
 *   prefix_len     host: tokens [0, prefix_len) of the store at positions [0, prefix_len); 0 = none
 *   doc_stored_start host: position the first token of every document was cached at
 *   q_stored_start host: position the first row of q / k_self was rotated for
 *   segs           device [batch*seg_stride], n_seg device int32 [batch]; seg_stride >= stride + 2
 */
CF_API cf_status cf_gather_segments(const int64_t* doc_tok_offset, const int32_t* len,
                             const int32_t* order, const int32_t* n_order,
                             const int32_t* new_start, const int32_t* q_start,
                             const int32_t* q_off, int32_t batch, int32_t stride,
                             int32_t prefix_len, int32_t doc_stored_start, int32_t q_stored_start,
                             cf_segment* segs, int32_t* n_seg, int32_t seg_stride,
                             int32_t* dev_flag, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Alg. 2, Phase 2 (Final Re-Positioning) for one layer: C_final = concat(repos(C, ids), C_Q).
 * Every query's listed segments are gathered, in table order, into one contiguous run of the
 * decode cache k_final / v_final; each key is moved from its stored position to its final one
 * (Eq. 5: rotation by new_start - stored_start; the query's own block like any other segment),
 * values are copied.  Streaming: K and V are read once and written once.
 *   desc           host; its store strides describe k_store / v_store
 *   k_store,v_store device, read; k_self,v_self device [sum tq][n_kv_heads][head_dim] (may be NULL
 *                  if no table lists an own block); q_off device int32 [batch+1]
 *   segs, n_seg, seg_stride  device tables as for cf_prefill_attention (segments of kind SELF take
 *                  min(len, tq) tokens, tq = min(q_off[b+1]-q_off[b], max_tq))
 *   max_seg_len    host: upper bound of any segment's length (sizes the launch)
 *   final_off      device int64 [batch]: token index in k_final / v_final where query b's run starts
 *   final_capacity host: tokens k_final / v_final can hold; a run that would pass it is not written
 *                  and raises CF_FLAG_BAD_INDEX
 *   final_token_stride, final_head_stride  host: element strides of k_final / v_final (multiples
 *                  of 8, at least head_dim): channel c of kv head h of token t at
 *                  t*token_stride + h*head_stride + c
 *   k_final,v_final device, written; must not overlap the inputs
 *   final_len      device int32 [batch], written: tokens in query b's run
 *   final_pos      device int32 [final_capacity] or NULL: position of every gathered token
 * Bad table entries are skipped (zero tokens) and raise CF_FLAG_BAD_SEGMENT.
 */
CF_API cf_status cf_assemble_cache(const cf_layer_desc* desc, const void* k_store, const void* v_store,
                            int64_t n_store_tokens, const void* k_self, const void* v_self,
                            const int32_t* q_off, const cf_segment* segs, const int32_t* n_seg,
                            int32_t seg_stride, int32_t batch, int32_t max_tq, int32_t max_seg_len,
                            const int64_t* final_off, int64_t final_capacity,
                            int64_t final_token_stride, int64_t final_head_stride,
                            void* k_final, void* v_final, int32_t* final_len, int32_t* final_pos,
                            int32_t* dev_flag, void* stream);

/* ---------------------------------------------------------------------------------------------
 * One whole layer of Alg. 2, Phase 1, in one call: the attention of cf_prefill_attention (with
 * S += s^l into score_accum, which must be given) followed — when `prune` is not NULL — by the
 * prune event of that layer: cf_prune_topk on the accumulated scores, cf_assign_positions for the
 * survivors and cf_gather_segments into the NEXT layer's table.  Results are identical to the
 * four separate calls; on the 16-bit path the mass reduction, ranking, allocation and table rebuild
 * run in one kernel, so a layer costs three launches instead of six.
 * The current table (segs / n_seg / q_new_start) is only read; the prune step writes next_segs,
 * next_n_seg, new_start, q_start, which therefore must not alias the current ones.
 * All pointers in cf_prune_step are device memory with the shapes given at the stand-alone calls
 * (stride = document slots per query; next_segs has the same seg_stride as segs).
 * With strategy CF_ALLOC_KEEP new_start / q_start are not written: hand in arrays that already
 * hold the current positions.
 *
 * Deferred scores.  Alg. 2 reads the accumulated scores S only at a prune event (every n-th layer), so the layers
 * in between need not bring S up to date themselves.  A call with `defer` = 1 (and no prune step) runs the attention
 * and leaves the layer's per-slot partial masses in the workspace instead of reducing them: neither `mass` nor
 * `score_accum` is touched and the call is one launch shorter.  The next call with `defer` = 0 — with or without a
 * prune step — is told in `n_pending` how many such layers precede it and adds their masses to S first, oldest first,
 * then its own: S, `mass` (the last layer's) and every later result are bit-identical to those of calls that never
 * deferred.  Rules: every call passes the number of layers pending before it (0 after a call that did not defer); at
 * most CF_MAX_PENDING layers may be pending; the pending layers and the call that takes them in must use the same
 * workspace, descriptor, batch, max_tq, seg_stride and max_kv_tokens, and the same, unchanged segs / n_seg / q_off /
 * q_new_start (a prune step changes the tables, so scores cannot be pending across one).  Shapes served by the generic
 * kernel do not defer: there a `defer` call accumulates at once and `n_pending` is ignored, with the same results.
 */
#define CF_MAX_PENDING 15
typedef struct cf_prune_step {
    int32_t keep;              /* documents kept per query, 0 <= keep <= stride                    */
    int32_t strategy;          /* cf_alloc_strategy                                                */
    int32_t force_n_reuse;     /* 0 = Eq. 6                                                        */
    int32_t normalise_by_len;  /* non-zero: rank by score/len                                      */
    int32_t stride;
    int32_t pos_begin, pos_end;
    int32_t prefix_len, doc_stored_start;
    int32_t reserved;          /* must be 0                                                        */
    const int64_t* doc_tok_offset;  /* [batch*stride] */
    const int32_t* doc_len;         /* [batch*stride] */
    const int32_t* cand;            /* [batch*stride] current candidates                           */
    const int32_t* n_cand;          /* [batch]                                                     */
    int32_t* keep_idx;              /* [batch*stride] out: survivors, best first                   */
    int32_t* n_keep;                /* [batch] out                                                 */
    int32_t* new_start;             /* [batch*stride] out (survivors' entries)                     */
    int32_t* q_start;               /* [batch] out                                                 */
    int32_t* n_reuse;               /* [batch] out                                                 */
    int32_t* order;                 /* [batch*stride] out: placement order = next candidates       */
    cf_segment* next_segs;          /* [batch*seg_stride] out                                      */
    int32_t* next_n_seg;            /* [batch] out                                                 */
} cf_prune_step;

CF_API cf_status cf_prefill_layer(const cf_layer_desc* desc,
                                  const void* q, const int32_t* q_off, int32_t q_stored_start,
                                  const int32_t* q_new_start,
                                  const void* k_store, const void* v_store, int64_t n_store_tokens,
                                  const void* k_self, const void* v_self,
                                  const cf_segment* segs, const int32_t* n_seg, int32_t seg_stride,
                                  int32_t batch, int32_t max_tq, int64_t max_kv_tokens,
                                  void* out, float* mass, float* score_accum, int32_t score_stride,
                                  void* workspace, size_t workspace_bytes,
                                  const cf_prune_step* prune, int32_t n_pending, int32_t defer,
                                  int32_t* dev_flag, void* stream);

/* Thread-local text for the last non-OK status returned on this thread (static storage). */
CF_API const char* cf_last_error(void);

/* Library version as major*10000 + minor*100 + patch. */
CF_API int32_t cf_version(void);

/* =============================================================================================
 * Measurement aids.  Not part of the method; none of them changes what the calls above compute.
 * ============================================================================================= */

/* While enabled (nonzero), every launch of the attention kernel proper
 * by cf_prefill_attention / cf_prefill_layer on this thread's 16-bit path carries a start and a stop event that
 * take the time at which that dispatch begins and ends on the GPU; the events of the last 1024 launches are kept.  Enabling creates the events (host memory
 * only) and forgets earlier launches; disabling destroys them.  Host call, not to be issued during stream capture.
 * Returns CF_OK or CF_ERR_DEVICE. */
CF_API cf_status cf_profile_kernel_events(int32_t enable);

/* Waits for the bracketed launches to finish and reports their number (at most 1024) and the mean of their
 * event-to-event durations in milliseconds (0 when there are none).  Both pointers are host memory, non-NULL.
 * CF_ERR_INVALID_ARG when timing is not enabled or a pointer is NULL, CF_ERR_DEVICE on a runtime error. */
CF_API cf_status cf_profile_kernel_ms(double* mean_ms, int32_t* launches);

/* Calibration kernels of known size, for pricing measurements against what this GPU sustains rather than
 * against its nominal peaks.  Each call enqueues ONE kernel on `stream` and returns; time it with events.
 *   CF_CALIB_READ   reads `bytes` bytes of `src` once (16-byte loads, every workgroup a contiguous share)
 *   CF_CALIB_COPY   reads `bytes` bytes of `src` and writes them to `dst`
 *   CF_CALIB_MFMA_BF16 / _F16   no memory traffic: every wavefront of `workgroups` workgroups of 256 threads issues
 *                   iters * 64 dense v_mfma_f32_32x32x16 (32 768 flops each) on eight independent accumulators;
 *                   *flops receives the launch's flop count
 * src, dst: device, 16-byte aligned, `bytes` a multiple of 16 (dst may be NULL except for COPY); sink: device,
 * at least 16 bytes, receives nothing meaningful (it keeps the loads alive); flops: host, may be NULL. */
typedef enum cf_calib_kind { CF_CALIB_READ = 0, CF_CALIB_COPY = 1, CF_CALIB_MFMA_BF16 = 2, CF_CALIB_MFMA_F16 = 3 } cf_calib_kind;
CF_API cf_status cf_calibrate(int32_t kind, const void* src, void* dst, size_t bytes, int32_t workgroups, int32_t iters,
                              void* sink, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CACHEFOCUS_H */
