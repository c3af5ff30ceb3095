// Device-side building blocks of the integer side of Layer-Adaptive Cache Pruning: ranking
// (Alg. 2, argsort + prun), position allocation (Eq. 6, Sec. 2.5) and the segment-table rebuild
// (the logical concat of Alg. 2), each executed by one workgroup for one query.  They are used
// by the stand-alone kernels behind cf_prune_topk / cf_assign_positions / cf_gather_segments and
// by the fused layer epilogue.  Candidate sets are small (tens to a few hundred documents), so
// ranking is by counting with exact comparisons: results do not depend on thread order.
#pragma once

#include "cf_common.h"

namespace cf {

// true when candidate (score sa, len la, slot ia, list position pa) ranks before (sb, lb, ib, pb):
// higher score/len first, compared as sa*lb vs sb*la in fp64 (exact: 24-bit significand times an
// integer below 2^24 fits 53 bits), then lower slot, then earlier list position.
__device__ __forceinline__ bool ranks_before(float sa, int la, int ia, int pa, float sb, int lb, int ib, int pb) {
    const double x = (double)sa * (double)lb;
    const double y = (double)sb * (double)la;
    if (x != y) return x > y;
    if (ia != ib) return ia < ib;
    return pa < pb;
}

// smem: 3*stride 32-bit words.  All threads of the workgroup must call; returns the number kept
// (0 after a flagged error).  score/len/cand/keep_idx point at this query's rows.
__device__ inline int prune_topk_block(const float* score, const int32_t* len, const int32_t* cand, int n, int keep,
                                       int stride, int32_t* keep_idx, int32_t* dev_flag, unsigned char* smem,
                                       int* s_bad) {
    float* s_score = reinterpret_cast<float*>(smem);
    int32_t* s_len = reinterpret_cast<int32_t*>(s_score + stride);
    int32_t* s_idx = s_len + stride;
    const int tid = threadIdx.x, nthr = blockDim.x;
    if (tid == 0) *s_bad = 0;
    __syncthreads();
    if (n < 0 || n > stride) {
        if (tid == 0) raise_flag(dev_flag, CF_FLAG_BAD_INDEX);
        return 0;
    }
    for (int i = tid; i < n; i += nthr) {
        const int c = cand[i];
        int flag = 0;
        float sc = 0.f;
        int ln = 1;
        if (c < 0 || c >= stride) {
            flag = CF_FLAG_BAD_INDEX;
        } else {
            sc = score[c];
            ln = len ? len[c] : 1;
            if (!isfinite(sc)) flag = CF_FLAG_NONFINITE_SCORE;
            if (ln <= 0 || ln >= (1 << 24)) flag |= CF_FLAG_BAD_SEGMENT;
        }
        if (flag) atomicOr(s_bad, flag);
        s_score[i] = sc;
        s_len[i] = ln;
        s_idx[i] = c;
    }
    __syncthreads();
    if (*s_bad) {
        if (tid == 0) raise_flag(dev_flag, *s_bad);
        return 0;
    }
    const int k = min(keep, n);
    for (int i = tid; i < n; i += nthr) {
        const float si = s_score[i];
        const int li = s_len[i], ci = s_idx[i];
        int rank = 0;
        for (int j = 0; j < n; ++j)
            rank += (j != i) && ranks_before(s_score[j], s_len[j], s_idx[j], j, si, li, ci, i);
        if (rank < k) keep_idx[rank] = ci;
    }
    return k;
}

// smem: 3*stride 32-bit words; s_int: 3 ints of LDS.  All threads must call.  Pointers are this
// query's rows; q_start / n_reuse point at this query's entries.  Returns false (outputs
// untouched) after a flagged error.
__device__ inline bool assign_positions_block(const int32_t* len, const int32_t* ranked, int n, int stride, int pos_begin,
                                              int pos_end, int strategy, int force_n_reuse, int32_t* new_start,
                                              int32_t* q_start, int32_t* n_reuse, int32_t* order, int32_t* dev_flag,
                                              unsigned char* smem, int* s_int) {
    int32_t* s_ord = reinterpret_cast<int32_t*>(smem);   // placement order (slots)
    int32_t* s_len = s_ord + stride;                      // length per placement rank
    int32_t* s_cum = s_len + stride;                      // distance from the query to the start
    int &bad = s_int[0], &lmax = s_int[1], &span_max = s_int[2];
    const int tid = threadIdx.x, nthr = blockDim.x;
    __syncthreads();
    if (tid == 0) { bad = 0; lmax = 0; span_max = 0; }
    __syncthreads();
    if (n < 0 || n > stride) {
        if (tid == 0) raise_flag(dev_flag, CF_FLAG_BAD_INDEX);
        return false;
    }
    // placement order: as ranked ("sort") or by ascending slot ("align", and the listing order of "keep")
    for (int i = tid; i < n; i += nthr) {
        const int c = ranked[i];
        if (c < 0 || c >= stride) atomicOr(&bad, CF_FLAG_BAD_INDEX);
        s_cum[i] = c;
    }
    __syncthreads();
    if (bad) {
        if (tid == 0) raise_flag(dev_flag, bad);
        return false;
    }
    for (int i = tid; i < n; i += nthr) {
        const int c = s_cum[i];
        int r = i;
        if (strategy != CF_ALLOC_SORT) {
            r = 0;
            for (int j = 0; j < n; ++j) {
                const int cj = s_cum[j];
                r += (cj < c) || (cj == c && j < i);
            }
        }
        s_ord[r] = c;
    }
    __syncthreads();
    for (int i = tid; i < n; i += nthr) {
        const int l = len[s_ord[i]];
        s_len[i] = l;
        if (l <= 0) atomicOr(&bad, CF_FLAG_BAD_SEGMENT);
        atomicMax(&lmax, l);
    }
    __syncthreads();
    if (bad) {
        if (tid == 0) raise_flag(dev_flag, bad);
        return false;
    }
    if (strategy == CF_ALLOC_KEEP || n == 0) {
        for (int i = tid; i < n; i += nthr) order[i] = s_ord[i];
        if (n == 0 && strategy != CF_ALLOC_KEEP && tid == 0) { *q_start = pos_begin; *n_reuse = 0; }
        return true;
    }
    const int avail = pos_end - pos_begin;
    const int cap = avail / lmax;
    if (cap <= 0) {
        if (tid == 0) raise_flag(dev_flag, CF_FLAG_DOC_TOO_LONG);
        return false;
    }
    int groups = force_n_reuse > 0 ? force_n_reuse : (n + cap - 1) / cap;
    groups = min(groups, n);
    const int per_group = (n + groups - 1) / groups;
    for (int i = tid; i < n; i += nthr) {
        const int first = (i / per_group) * per_group;
        int cum = 0;
        for (int j = first; j <= i; ++j) cum += s_len[j];
        s_cum[i] = cum;
        const bool last = (i == n - 1) || ((i + 1) % per_group == 0);
        if (last) atomicMax(&span_max, cum);
    }
    __syncthreads();
    if (span_max > avail) {
        if (tid == 0) raise_flag(dev_flag, CF_FLAG_POS_OVERFLOW);
        return false;
    }
    const int qs = pos_begin + span_max;
    for (int i = tid; i < n; i += nthr) {
        new_start[s_ord[i]] = qs - s_cum[i];
        order[i] = s_ord[i];
    }
    if (tid == 0) { *q_start = qs; *n_reuse = groups; }
    return true;
}

// All threads must call.  doc_tok_offset/len/order/new_start point at this query's rows, out at
// this query's segment-table row.  q_lo/q_hi: this query's rows in q.
__device__ inline void gather_segments_block(const int64_t* doc_tok_offset, const int32_t* len, const int32_t* order, int n,
                                             const int32_t* new_start, int q_start, int q_lo, int q_hi, int stride,
                                             int prefix_len, int doc_stored_start, int q_stored_start, cf_segment* out,
                                             int32_t* n_seg, int seg_stride, int32_t* dev_flag) {
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int has_prefix = prefix_len > 0 ? 1 : 0;
    if (n < 0 || n > stride || n + has_prefix + 1 > seg_stride) {
        if (tid == 0) { raise_flag(dev_flag, CF_FLAG_BAD_INDEX); *n_seg = 0; }
        return;
    }
    if (tid == 0) {
        if (has_prefix) {
            cf_segment p;
            p.tok_offset = 0; p.len = prefix_len; p.stored_start = 0; p.new_start = 0;
            p.kind = CF_SEG_PREFIX; p.doc = -1; p.reserved = 0;
            out[0] = p;
        }
        cf_segment q;
        q.tok_offset = q_lo; q.len = q_hi - q_lo; q.stored_start = q_stored_start;
        q.new_start = q_start; q.kind = CF_SEG_SELF; q.doc = -1; q.reserved = 0;
        out[has_prefix + n] = q;
        *n_seg = has_prefix + n + 1;
    }
    for (int i = tid; i < n; i += nthr) {
        const int c = order[i];
        cf_segment sgm;
        if (c < 0 || c >= stride) {
            raise_flag(dev_flag, CF_FLAG_BAD_INDEX);
            sgm.tok_offset = 0; sgm.len = 0; sgm.stored_start = 0; sgm.new_start = 0;
            sgm.kind = CF_SEG_DOC; sgm.doc = -1; sgm.reserved = 0;
        } else {
            sgm.tok_offset = doc_tok_offset[c]; sgm.len = len[c];
            sgm.stored_start = doc_stored_start; sgm.new_start = new_start[c];
            sgm.kind = CF_SEG_DOC; sgm.doc = c; sgm.reserved = 0;
        }
        out[has_prefix + i] = sgm;
    }
}

}  // namespace cf
