// Integer side of Layer-Adaptive Cache Pruning: ranking (Alg. 2, argsort + prun), position
// allocation (Eq. 6, Sec. 2.5) and the segment-table rebuild (the logical concat of Alg. 2).
// The candidate sets are small (tens to a few hundred documents per query), so each query is
// one workgroup that ranks by counting; every comparison is exact, so results do not depend on
// thread order.
#include "cf_common.h"

namespace cf {
namespace {

constexpr int kThreads = 256;

// true when candidate (score sa, len la, slot ia, list position pa) ranks before (sb, lb, ib, pb):
// higher score/len first, compared as sa*lb vs sb*la in fp64 (exact: 24-bit significand times an
// integer below 2^24 fits 53 bits), then lower slot, then earlier list position.
__device__ __forceinline__ bool ranks_before(float sa, int la, int ia, int pa, float sb, int lb, int ib,
                                             int pb) {
    const double x = (double)sa * (double)lb;
    const double y = (double)sb * (double)la;
    if (x != y) return x > y;
    if (ia != ib) return ia < ib;
    return pa < pb;
}

__global__ __launch_bounds__(kThreads) void prune_topk_kernel(
    const float* __restrict__ score, const int32_t* __restrict__ len, const int32_t* __restrict__ cand,
    const int32_t* __restrict__ n_cand, int keep, int stride, int32_t* __restrict__ keep_idx,
    int32_t* __restrict__ n_keep, int32_t* dev_flag) {
    extern __shared__ unsigned char smem[];
    float* s_score = reinterpret_cast<float*>(smem);
    int32_t* s_len = reinterpret_cast<int32_t*>(s_score + stride);
    int32_t* s_idx = s_len + stride;
    __shared__ int bad;
    const int b = blockIdx.x;
    const int64_t off = (int64_t)b * stride;
    int n = n_cand[b];
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    if (n < 0 || n > stride) {
        if (threadIdx.x == 0) { raise_flag(dev_flag, CF_FLAG_BAD_INDEX); n_keep[b] = 0; }
        return;
    }
    for (int i = threadIdx.x; i < n; i += kThreads) {
        const int c = cand[off + i];
        int flag = 0;
        float sc = 0.f;
        int ln = 1;
        if (c < 0 || c >= stride) {
            flag = CF_FLAG_BAD_INDEX;
        } else {
            sc = score[off + c];
            ln = len ? len[off + c] : 1;
            if (!isfinite(sc)) flag = CF_FLAG_NONFINITE_SCORE;
            if (ln <= 0 || ln >= (1 << 24)) flag |= CF_FLAG_BAD_SEGMENT;
        }
        if (flag) atomicOr(&bad, flag);
        s_score[i] = sc;
        s_len[i] = ln;
        s_idx[i] = c;
    }
    __syncthreads();
    if (bad) {
        if (threadIdx.x == 0) { raise_flag(dev_flag, bad); n_keep[b] = 0; }
        return;
    }
    const int k = min(keep, n);
    for (int i = threadIdx.x; i < n; i += kThreads) {
        const float si = s_score[i];
        const int li = s_len[i], ci = s_idx[i];
        int rank = 0;
        for (int j = 0; j < n; ++j)
            rank += (j != i) && ranks_before(s_score[j], s_len[j], s_idx[j], j, si, li, ci, i);
        if (rank < k) keep_idx[off + rank] = ci;
    }
    if (threadIdx.x == 0) n_keep[b] = k;
}

__global__ __launch_bounds__(kThreads) void assign_positions_kernel(
    const int32_t* __restrict__ len, const int32_t* __restrict__ ranked, const int32_t* __restrict__ n_ranked,
    int stride, int pos_begin, int pos_end, int strategy, int force_n_reuse, int32_t* __restrict__ new_start,
    int32_t* __restrict__ q_start, int32_t* __restrict__ n_reuse, int32_t* __restrict__ order,
    int32_t* dev_flag) {
    extern __shared__ unsigned char smem[];
    int32_t* s_ord = reinterpret_cast<int32_t*>(smem);   // placement order (slots)
    int32_t* s_len = s_ord + stride;                      // length per placement rank
    int32_t* s_cum = s_len + stride;                      // distance from the query to the start
    __shared__ int bad, lmax, span_max;
    const int b = blockIdx.x;
    const int64_t off = (int64_t)b * stride;
    const int n = n_ranked[b];
    if (threadIdx.x == 0) { bad = 0; lmax = 0; span_max = 0; }
    __syncthreads();
    if (n < 0 || n > stride) {
        if (threadIdx.x == 0) raise_flag(dev_flag, CF_FLAG_BAD_INDEX);
        return;
    }
    // placement order: as ranked ("sort") or by ascending slot ("align", and the listing order
    // of "keep")
    for (int i = threadIdx.x; i < n; i += kThreads) {
        const int c = ranked[off + i];
        if (c < 0 || c >= stride) atomicOr(&bad, CF_FLAG_BAD_INDEX);
        s_cum[i] = c;
    }
    __syncthreads();
    if (bad) {
        if (threadIdx.x == 0) raise_flag(dev_flag, bad);
        return;
    }
    for (int i = threadIdx.x; i < n; i += kThreads) {
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
    for (int i = threadIdx.x; i < n; i += kThreads) {
        const int l = len[off + s_ord[i]];
        s_len[i] = l;
        if (l <= 0) atomicOr(&bad, CF_FLAG_BAD_SEGMENT);
        atomicMax(&lmax, l);
    }
    __syncthreads();
    if (bad) {
        if (threadIdx.x == 0) raise_flag(dev_flag, bad);
        return;
    }
    if (strategy == CF_ALLOC_KEEP || n == 0) {
        for (int i = threadIdx.x; i < n; i += kThreads) order[off + i] = s_ord[i];
        if (n == 0 && strategy != CF_ALLOC_KEEP && threadIdx.x == 0) { q_start[b] = pos_begin; n_reuse[b] = 0; }
        return;
    }
    const int avail = pos_end - pos_begin;
    const int cap = avail / lmax;
    if (cap <= 0) {
        if (threadIdx.x == 0) raise_flag(dev_flag, CF_FLAG_DOC_TOO_LONG);
        return;
    }
    int groups = force_n_reuse > 0 ? force_n_reuse : (n + cap - 1) / cap;
    groups = min(groups, n);
    const int per_group = (n + groups - 1) / groups;
    for (int i = threadIdx.x; i < n; i += kThreads) {
        const int first = (i / per_group) * per_group;
        int cum = 0;
        for (int j = first; j <= i; ++j) cum += s_len[j];
        s_cum[i] = cum;
        const bool last = (i == n - 1) || ((i + 1) % per_group == 0);
        if (last) atomicMax(&span_max, cum);
    }
    __syncthreads();
    if (span_max > avail) {
        if (threadIdx.x == 0) raise_flag(dev_flag, CF_FLAG_POS_OVERFLOW);
        return;
    }
    const int qs = pos_begin + span_max;
    for (int i = threadIdx.x; i < n; i += kThreads) {
        new_start[off + s_ord[i]] = qs - s_cum[i];
        order[off + i] = s_ord[i];
    }
    if (threadIdx.x == 0) { q_start[b] = qs; n_reuse[b] = groups; }
}

__global__ __launch_bounds__(kThreads) void gather_segments_kernel(
    const int64_t* __restrict__ doc_tok_offset, const int32_t* __restrict__ len,
    const int32_t* __restrict__ order, const int32_t* __restrict__ n_order,
    const int32_t* __restrict__ new_start, const int32_t* __restrict__ q_start,
    const int32_t* __restrict__ q_off, int stride, int prefix_len, int doc_stored_start, int q_stored_start,
    cf_segment* __restrict__ segs, int32_t* __restrict__ n_seg, int seg_stride, int32_t* dev_flag) {
    const int b = blockIdx.x;
    const int64_t off = (int64_t)b * stride;
    cf_segment* out = segs + (int64_t)b * seg_stride;
    const int n = n_order[b];
    const int has_prefix = prefix_len > 0 ? 1 : 0;
    if (n < 0 || n > stride || n + has_prefix + 1 > seg_stride) {
        if (threadIdx.x == 0) { raise_flag(dev_flag, CF_FLAG_BAD_INDEX); n_seg[b] = 0; }
        return;
    }
    if (threadIdx.x == 0) {
        if (has_prefix) {
            cf_segment p;
            p.tok_offset = 0; p.len = prefix_len; p.stored_start = 0; p.new_start = 0;
            p.kind = CF_SEG_PREFIX; p.doc = -1; p.reserved = 0;
            out[0] = p;
        }
        cf_segment q;
        q.tok_offset = q_off[b]; q.len = q_off[b + 1] - q_off[b]; q.stored_start = q_stored_start;
        q.new_start = q_start[b]; q.kind = CF_SEG_SELF; q.doc = -1; q.reserved = 0;
        out[has_prefix + n] = q;
        n_seg[b] = has_prefix + n + 1;
    }
    for (int i = threadIdx.x; i < n; i += kThreads) {
        const int c = order[off + i];
        cf_segment sgm;
        if (c < 0 || c >= stride) {
            raise_flag(dev_flag, CF_FLAG_BAD_INDEX);
            sgm.tok_offset = 0; sgm.len = 0; sgm.stored_start = 0; sgm.new_start = 0;
            sgm.kind = CF_SEG_DOC; sgm.doc = -1; sgm.reserved = 0;
        } else {
            sgm.tok_offset = doc_tok_offset[off + c]; sgm.len = len[off + c];
            sgm.stored_start = doc_stored_start; sgm.new_start = new_start[off + c];
            sgm.kind = CF_SEG_DOC; sgm.doc = c; sgm.reserved = 0;
        }
        out[has_prefix + i] = sgm;
    }
}

}  // namespace

cf_status launch_prune(const float* score, const int32_t* len, const int32_t* cand, const int32_t* n_cand,
                       int32_t keep, int32_t batch, int32_t stride, int32_t* keep_idx, int32_t* n_keep,
                       int32_t* dev_flag, hipStream_t s) {
    const size_t shm = (size_t)stride * 12;
    hipLaunchKernelGGL(prune_topk_kernel, dim3(batch), dim3(kThreads), shm, s, score, len, cand, n_cand, keep,
                       stride, keep_idx, n_keep, dev_flag);
    CF_HIP(hipGetLastError());
    return CF_OK;
}

cf_status launch_assign(const int32_t* len, const int32_t* ranked, const int32_t* n_ranked, int32_t batch,
                        int32_t stride, int32_t pos_begin, int32_t pos_end, int32_t strategy,
                        int32_t force_n_reuse, int32_t* new_start, int32_t* q_start, int32_t* n_reuse,
                        int32_t* order, int32_t* dev_flag, hipStream_t s) {
    const size_t shm = (size_t)stride * 12;
    hipLaunchKernelGGL(assign_positions_kernel, dim3(batch), dim3(kThreads), shm, s, len, ranked, n_ranked,
                       stride, pos_begin, pos_end, strategy, force_n_reuse, new_start, q_start, n_reuse, order,
                       dev_flag);
    CF_HIP(hipGetLastError());
    return CF_OK;
}

cf_status launch_gather(const int64_t* doc_tok_offset, const int32_t* len, const int32_t* order,
                        const int32_t* n_order, const int32_t* new_start, const int32_t* q_start,
                        const int32_t* q_off, int32_t batch, int32_t stride, int32_t prefix_len,
                        int32_t doc_stored_start, int32_t q_stored_start, cf_segment* segs, int32_t* n_seg,
                        int32_t seg_stride, int32_t* dev_flag, hipStream_t s) {
    hipLaunchKernelGGL(gather_segments_kernel, dim3(batch), dim3(kThreads), 0, s, doc_tok_offset, len, order,
                       n_order, new_start, q_start, q_off, stride, prefix_len, doc_stored_start, q_stored_start,
                       segs, n_seg, seg_stride, dev_flag);
    CF_HIP(hipGetLastError());
    return CF_OK;
}

}  // namespace cf
