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

// The three functions below are called by the first `nthr` threads of a workgroup, all of them, and by
// no others; when the workgroup's other wavefronts have exited, nthr is one wavefront and the barriers
// inside cost nothing.
//
// smem: 3*stride 32-bit words.  Returns the number kept (0 after a flagged error).
// score/len/cand/keep_idx point at this query's rows.
__device__ inline int prune_topk_block(const float* score, const int32_t* len, const int32_t* cand, int n, int keep,
                                       int stride, int32_t* keep_idx, int32_t* dev_flag, unsigned char* smem,
                                       int* s_bad, int nthr) {
    float* s_score = reinterpret_cast<float*>(smem);
    int32_t* s_len = reinterpret_cast<int32_t*>(s_score + stride);
    int32_t* s_idx = s_len + stride;
    const int tid = threadIdx.x;
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

// smem: 3*stride 32-bit words; s_int: 3 ints of LDS.  Pointers are this query's rows; q_start /
// n_reuse point at this query's entries.  Returns false (outputs untouched) after a flagged error.
__device__ inline bool assign_positions_block(const int32_t* len, const int32_t* ranked, int n, int stride, int pos_begin,
                                              int pos_end, int strategy, int force_n_reuse, int32_t* new_start,
                                              int32_t* q_start, int32_t* n_reuse, int32_t* order, int32_t* dev_flag,
                                              unsigned char* smem, int* s_int, int nthr) {
    int32_t* s_ord = reinterpret_cast<int32_t*>(smem);   // placement order (slots)
    int32_t* s_len = s_ord + stride;                      // length per placement rank
    int32_t* s_cum = s_len + stride;                      // distance from the query to the start
    int &bad = s_int[0], &lmax = s_int[1], &span_max = s_int[2];
    const int tid = threadIdx.x;
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

// doc_tok_offset/len/order/new_start point at this query's rows, out at this query's segment-table
// row.  q_lo/q_hi: this query's rows in q.
__device__ inline void gather_segments_block(const int64_t* doc_tok_offset, const int32_t* len, const int32_t* order, int n,
                                             const int32_t* new_start, int q_start, int q_lo, int q_hi, int stride,
                                             int prefix_len, int doc_stored_start, int q_stored_start, cf_segment* out,
                                             int32_t* n_seg, int seg_stride, int32_t* dev_flag, int nthr) {
    const int tid = threadIdx.x;
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

// ---------------------------------------------------------------------------------------------
// The same three stages for at most 64 candidates, executed by one wavefront with every list in
// registers (lane i = list position i): ranks by comparing against broadcast lanes, lists turned
// into one another through small LDS scatters, sums and maxima by wavefront scans.  No barriers, no
// atomics.  Results are those of the block functions; on any condition they would flag (bad
// index, non-finite score, bad length, document too long, overflow, table too small) nothing is
// written and false is returned, so that the caller runs the block functions, which raise the flag.
// All pointers are this query's rows and may live in LDS; keep_idx also serves as scratch (entries
// below the candidate count); *q_start / *n_reuse are written like the block function does.
struct SelectWaveArgs {
    const float* score; const int32_t* len; const int32_t* cand; const int64_t* tok;
    int32_t* keep_idx; int32_t* new_start; int32_t* order;
    uint4* bcast;                                   // LDS, 64 entries: the ranking keys, read back as broadcasts
    int n, keep, stride, normalise_by_len, strategy, force_n_reuse, pos_begin, pos_end;
    int prefix_len, doc_stored_start, q_stored_start, q_lo, q_hi, seg_stride;
};

// In-register reductions over the 64 lanes of a wavefront with DPP (row shifts, then the two row broadcasts,
// lane 63 ends up with the result): an inclusive prefix sum, and a maximum handed to every lane.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ int wave_max_i32(int v) {
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x111, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x112, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x114, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x118, 0xf, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x142, 0xa, 0xf, false));
    v = max(v, __builtin_amdgcn_update_dpp(v, v, 0x143, 0xc, 0xf, false));
    return __builtin_amdgcn_readlane(v, 63);
}

__device__ inline bool select_wave64(const SelectWaveArgs& s, int* n_keep_out, int* q_start, int* n_reuse, cf_segment* out,
                                     int32_t* n_seg_out) {
    const int lane = threadIdx.x & 63;
    const int n = s.n;
    if (n < 0 || n > 64 || n > s.stride) return false;
    // ---- ranking (Alg. 2: argsort of the accumulated scores, then the cut)
    const bool have = lane < n;
    const int c = have ? s.cand[lane] : 0;
    const bool c_ok = c >= 0 && c < s.stride;
    const float sc = have && c_ok ? s.score[c] : 0.f;
    const int ln_rank = have && c_ok && s.normalise_by_len ? s.len[c] : 1;
    const bool bad = have && (!c_ok || !isfinite(sc) || ln_rank <= 0 || ln_rank >= (1 << 24));
    if (__any(bad)) return false;
    int rank = 0;
    if (s.stride <= (1 << 26) && __all(!have || ln_rank == __builtin_amdgcn_readlane(ln_rank, 0))) {
        // equal lengths (the paper's regime, or no normalisation): the products of ranks_before compare as the
        // scores themselves do
        // as one unsigned key per lane: score (order-preserving bits, -0 as +0), then lower slot, then earlier position
        uint32_t u = __float_as_uint(sc + 0.f);
        u ^= (u >> 31) ? 0xffffffffu : 0x80000000u;
        const uint32_t low = ((uint32_t)(s.stride - 1 - c) << 6) | (uint32_t)(63 - lane);     // stride <= 2^26
        const uint64_t key = ((uint64_t)u << 32) | low;
        // every lane's key goes to LDS once; candidate j's key is then one broadcast read (the same address in every
        // lane), eight requested at a time
        // (lanes past n publish the smallest key: read, never counted)
        s.bcast[lane] = have ? make_uint4(low, u, 0u, 0u) : make_uint4(0u, 0u, 0u, 0u);
        __builtin_amdgcn_wave_barrier();
        for (int j0 = 0; j0 < n; j0 += 8) {
            uint2 e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = *reinterpret_cast<const uint2*>(&s.bcast[(j0 + i) & 63]);
#pragma unroll
            for (int i = 0; i < 8; ++i) rank += ((((uint64_t)e[i].y << 32) | e[i].x) > key) ? 1 : 0;
        }
    } else {
        // Unequal lengths: the quotient score/len in fp64 orders exactly as the cross products of ranks_before do —
        // two different cross products (a 24-bit significand times an integer below 2^24 each) make quotients
        // that differ by more than 2^-48 of their size, far above the quotient's rounding, and equal ones give
        // the same quotient — so every lane divides once and the loop compares, without branches.
        const double q = (double)sc / (double)ln_rank;
        const int q_lo = (int)(uint32_t)__builtin_bit_cast(uint64_t, q), q_hi = (int)(uint32_t)(__builtin_bit_cast(uint64_t, q) >> 32);
        const uint32_t low = ((uint32_t)(s.stride - 1 - c) << 6) | (uint32_t)(63 - lane);   // lower slot, then earlier position
        auto lane_quotient = [&](int j) {
            const uint64_t bits = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(q_hi, j) << 32) |
                                  (uint32_t)__builtin_amdgcn_readlane(q_lo, j);
            return __builtin_bit_cast(double, bits);
        };
        if (s.stride <= (1 << 26)) {
            // as above: (quotient, tie-break word) of every lane in LDS, broadcast reads, eight at a time
            // (lanes past n publish minus infinity: read, never counted; the selects keep the predicate in vector
            // registers instead of wavefront masks worked on by the scalar unit)
            const uint64_t never = __builtin_bit_cast(uint64_t, -__builtin_inf());
            s.bcast[lane] = have ? make_uint4((uint32_t)q_lo, (uint32_t)q_hi, low, 0u) : make_uint4((uint32_t)never, (uint32_t)(never >> 32), 0u, 0u);
            __builtin_amdgcn_wave_barrier();
            for (int j0 = 0; j0 < n; j0 += 8) {
                uint4 e[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) e[i] = s.bcast[(j0 + i) & 63];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const double qj = __builtin_bit_cast(double, ((uint64_t)e[i].y << 32) | e[i].x);
                    const int tie = e[i].z > low ? 1 : 0;
                    const int eq = qj == q ? tie : 0;
                    rank += qj > q ? 1 : eq;
                }
            }
        } else {                                     // `low` would not hold the slot
            for (int j = 0; j < n; ++j) {
                const double qj = lane_quotient(j);
                const int cj = __builtin_amdgcn_readlane(c, j);
                rank += (int)((qj > q) | ((qj == q) & (cj != c ? cj < c : j < lane)));
            }
        }
    }
    const int k = min(s.keep, n);
    const int has_prefix = s.prefix_len > 0 ? 1 : 0;
    if (k + has_prefix + 1 > s.seg_stride) return false;
    // ranked list: lane r gets the candidate of rank r
    if (have && rank < k) s.keep_idx[rank] = c;
    __builtin_amdgcn_wave_barrier();
    const bool in = lane < k;
    const int rc = in ? s.keep_idx[lane] : 0x7fffffff;
    __builtin_amdgcn_wave_barrier();
    // ---- placement order (Sec. 2.5): as ranked ("sort") or by ascending slot ("align"; listing order of "keep")
    int place = lane;
    if (s.strategy != CF_ALLOC_SORT) {
        place = 0;
        for (int j = 0; j < k; ++j) {
            const int cj = __builtin_amdgcn_readlane(rc, j);
            place += (cj < rc) || (cj == rc && j < lane);
        }
    }
    if (in) s.keep_idx[place] = rc;                       // scratch use; the ranked list is written back below
    __builtin_amdgcn_wave_barrier();
    const int oc = in ? s.keep_idx[lane] : 0;             // slot at placement rank `lane`
    __builtin_amdgcn_wave_barrier();
    const int pl = in ? s.len[oc] : 0;
    if (__any(in && pl <= 0)) return false;
    int qs = *q_start, groups = *n_reuse;
    int my_start = in ? s.new_start[oc] : 0;
    bool write_pos = false;
    if (s.strategy != CF_ALLOC_KEEP && k > 0) {
        // ---- allocation (Eq. 6): capacity by the longest survivor, balanced contiguous groups, every group
        // ends at the query
        const int lmax = wave_max_i32(pl);
        const int avail = s.pos_end - s.pos_begin;
        const int cap = (int)div_exact((unsigned)max(avail, 0), (unsigned)lmax);      // lmax >= 1: every kept length is positive
        if (cap <= 0) return false;
        groups = s.force_n_reuse > 0 ? s.force_n_reuse : (cap >= k ? 1 : (int)div_exact((unsigned)(k + cap - 1), (unsigned)cap));
        groups = min(groups, k);
        const int per_group = (int)div_exact((unsigned)(k + groups - 1), (unsigned)groups);
        const int incl = wave_inclusive_scan(pl);         // inclusive prefix over placement ranks
        const int first = (int)div_exact((unsigned)lane, (unsigned)per_group) * per_group;
        const int before = __shfl(incl, max(first - 1, 0));
        const int cum = incl - (first > 0 ? before : 0);
        const bool last = in && ((lane == k - 1) || (lane + 1 == first + per_group));
        const int span_max = wave_max_i32(last ? cum : 0);
        if (span_max > avail) return false;
        qs = s.pos_begin + span_max;
        my_start = qs - cum;
        write_pos = true;
    } else if (s.strategy != CF_ALLOC_KEEP) {             // nothing survives
        qs = s.pos_begin;
        groups = 0;
    }
    // ---- everything checked: write the lists and the next segment table (Alg. 2, the logical concat)
    if (in) {
        s.keep_idx[lane] = rc;
        s.order[lane] = oc;
        if (write_pos) s.new_start[oc] = my_start;
    }
    if (lane == 0) {
        *n_keep_out = k;
        if (s.strategy != CF_ALLOC_KEEP) { *q_start = qs; *n_reuse = groups; }
        if (has_prefix) {
            cf_segment p;
            p.tok_offset = 0; p.len = s.prefix_len; p.stored_start = 0; p.new_start = 0;
            p.kind = CF_SEG_PREFIX; p.doc = -1; p.reserved = 0;
            out[0] = p;
        }
        cf_segment q;
        q.tok_offset = s.q_lo; q.len = s.q_hi - s.q_lo; q.stored_start = s.q_stored_start;
        q.new_start = qs; q.kind = CF_SEG_SELF; q.doc = -1; q.reserved = 0;
        out[has_prefix + k] = q;
        *n_seg_out = has_prefix + k + 1;
    }
    if (in) {
        cf_segment sg;
        sg.tok_offset = s.tok[oc]; sg.len = pl; sg.stored_start = s.doc_stored_start; sg.new_start = my_start;
        sg.kind = CF_SEG_DOC; sg.doc = oc; sg.reserved = 0;
        out[has_prefix + lane] = sg;
    }
    return true;
}

}  // namespace cf
