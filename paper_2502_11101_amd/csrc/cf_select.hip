// Integer side of Layer-Adaptive Cache Pruning: ranking (Alg. 2, argsort + prun), position
// allocation (Eq. 6, Sec. 2.5) and the segment-table rebuild (the logical concat of Alg. 2).
// The candidate sets are small (tens to a few hundred documents per query), so each query is
// one workgroup that ranks by counting; every comparison is exact, so results do not depend on
// thread order.
#include "cf_common.h"
#include "cf_select_dev.h"

namespace cf {
namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void prune_topk_kernel(
    const float* __restrict__ score, const int32_t* __restrict__ len, const int32_t* __restrict__ cand,
    const int32_t* __restrict__ n_cand, int keep, int stride, int32_t* __restrict__ keep_idx,
    int32_t* __restrict__ n_keep, int32_t* dev_flag) {
    extern __shared__ unsigned char smem[];
    __shared__ int s_bad;
    const int b = blockIdx.x;
    const int64_t off = (int64_t)b * stride;
    const int k = prune_topk_block(score + off, len ? len + off : nullptr, cand + off, n_cand[b], keep, stride,
                                   keep_idx + off, dev_flag, smem, &s_bad, kThreads);
    if (threadIdx.x == 0) n_keep[b] = k;
}

__global__ __launch_bounds__(kThreads) void assign_positions_kernel(
    const int32_t* __restrict__ len, const int32_t* __restrict__ ranked, const int32_t* __restrict__ n_ranked,
    int stride, int pos_begin, int pos_end, int strategy, int force_n_reuse, int32_t* __restrict__ new_start,
    int32_t* __restrict__ q_start, int32_t* __restrict__ n_reuse, int32_t* __restrict__ order,
    int32_t* dev_flag) {
    extern __shared__ unsigned char smem[];
    __shared__ int s_int[3];
    const int b = blockIdx.x;
    const int64_t off = (int64_t)b * stride;
    assign_positions_block(len + off, ranked + off, n_ranked[b], stride, pos_begin, pos_end, strategy, force_n_reuse,
                           new_start ? new_start + off : nullptr, q_start ? q_start + b : nullptr,
                           n_reuse ? n_reuse + b : nullptr, order + off, dev_flag, smem, s_int, kThreads);
}

__global__ __launch_bounds__(kThreads) void gather_segments_kernel(
    const int64_t* __restrict__ doc_tok_offset, const int32_t* __restrict__ len,
    const int32_t* __restrict__ order, const int32_t* __restrict__ n_order,
    const int32_t* __restrict__ new_start, const int32_t* __restrict__ q_start,
    const int32_t* __restrict__ q_off, int stride, int prefix_len, int doc_stored_start, int q_stored_start,
    cf_segment* __restrict__ segs, int32_t* __restrict__ n_seg, int seg_stride, int32_t* dev_flag) {
    const int b = blockIdx.x;
    const int64_t off = (int64_t)b * stride;
    gather_segments_block(doc_tok_offset + off, len + off, order + off, n_order[b], new_start + off, q_start[b], q_off[b],
                          q_off[b + 1], stride, prefix_len, doc_stored_start, q_stored_start,
                          segs + (int64_t)b * seg_stride, n_seg + b, seg_stride, dev_flag, kThreads);
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
