// Cache Re-Positioning, materialised (Sec. 2.3, Eq. 5): every key of every listed segment is
// rotated from the position it was cached at to its new position.  Pure streaming kernel:
// 16-byte loads and stores, one read and one write of K, bound by HBM bandwidth.
#include "cf_common.h"

namespace cf {
namespace {

constexpr int kThreads = 256;
constexpr int kTokPerBlock = 16;   // tokens one block handles per sweep of the segment

// Eight consecutive elements held as floats.
template <int DT> struct Vec8;
template <> struct Vec8<CF_F32> {
    static __device__ __forceinline__ void load(const void* base, int64_t idx, float (&v)[8]) {
        const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + idx);
        float4 a = p[0], b = p[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    static __device__ __forceinline__ void store(void* base, int64_t idx, const float (&v)[8]) {
        float4* p = reinterpret_cast<float4*>(static_cast<float*>(base) + idx);
        p[0] = make_float4(v[0], v[1], v[2], v[3]);
        p[1] = make_float4(v[4], v[5], v[6], v[7]);
    }
};
template <int DT> struct Vec8Half {
    static __device__ __forceinline__ void load(const void* base, int64_t idx, float (&v)[8]) {
        uint4 r = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + idx);
        uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (DT == CF_BF16) {
                v[2 * i] = bf16_bits_to_float(w[i] & 0xffffu);
                v[2 * i + 1] = bf16_bits_to_float(w[i] >> 16);
            } else {
                v[2 * i] = f16_bits_to_float(w[i] & 0xffffu);
                v[2 * i + 1] = f16_bits_to_float(w[i] >> 16);
            }
        }
    }
    static __device__ __forceinline__ void store(void* base, int64_t idx, const float (&v)[8]) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (DT == CF_BF16)
                w[i] = float_to_bf16_bits(v[2 * i]) | (float_to_bf16_bits(v[2 * i + 1]) << 16);
            else
                w[i] = float_to_f16_bits(v[2 * i]) | (float_to_f16_bits(v[2 * i + 1]) << 16);
        }
        *reinterpret_cast<uint4*>(static_cast<uint16_t*>(base) + idx) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};
template <> struct Vec8<CF_BF16> : Vec8Half<CF_BF16> {};
template <> struct Vec8<CF_F16> : Vec8Half<CF_F16> {};

// grid = (n_seg, sweeps); block = 256 threads.  A work item is 8 pairs of one (token, kv head):
// under half-split pairing the 8 first elements [8j, 8j+8) and their partners [d/2+8j, ...);
// under interleaved pairing 16 consecutive elements.  Consecutive threads take consecutive
// items, so each load instruction covers contiguous 128-byte (or longer) runs of a token row.
template <int DT, int PAIRING>
__global__ __launch_bounds__(kThreads) void reposition_kernel(
    const void* k_in, void* k_out, const cf_segment* __restrict__ segs,
    int64_t n_store_tokens, int n_kv_heads, int head_dim, int64_t tok_stride, int64_t head_stride, RopeFreq freq,
    int32_t* dev_flag, int tok_per_block, int max_positions) {
    __shared__ float2 cs[kMaxHalf];
    const cf_segment seg = segs[blockIdx.x];
    const int half = head_dim >> 1;
    if (seg.len < 0 || seg.tok_offset < 0 || seg.tok_offset + seg.len > n_store_tokens) {
        if (threadIdx.x == 0 && blockIdx.y == 0) raise_flag(dev_flag, CF_FLAG_BAD_SEGMENT);
        return;
    }
    if (!positions_ok(seg.stored_start, seg.len, max_positions) || !positions_ok(seg.new_start, seg.len, max_positions)) {
        if (threadIdx.x == 0 && blockIdx.y == 0) raise_flag(dev_flag, CF_FLAG_POS_RANGE);
        return;
    }
    const int delta = seg.new_start - seg.stored_start;
    for (int m = threadIdx.x; m < half; m += kThreads) cs[m] = rope_cos_sin(delta, freq.rev[m]);
    __syncthreads();

    const int items_per_head = half / 8;                 // head_dim % 16 == 0 checked on the host
    const int items_per_tok = n_kv_heads * items_per_head;
    for (int tok0 = blockIdx.y * tok_per_block; tok0 < seg.len; tok0 += gridDim.y * tok_per_block) {
        const int ntok = min(tok_per_block, seg.len - tok0);
        const int n_items = ntok * items_per_tok;
        for (int it = threadIdx.x; it < n_items; it += kThreads) {
            const int tok = (int)div_exact((unsigned)it, (unsigned)items_per_tok);
            const int r = it - tok * items_per_tok;
            const int head = (int)div_exact((unsigned)r, (unsigned)items_per_head);
            const int j = r - head * items_per_head;
            const int64_t base = (seg.tok_offset + tok0 + tok) * tok_stride + (int64_t)head * head_stride;
            float a[8], b[8];
            if (PAIRING == CF_ROPE_HALF) {
                Vec8<DT>::load(k_in, base + 8 * j, a);
                Vec8<DT>::load(k_in, base + half + 8 * j, b);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float2 w = cs[8 * j + e];
                    const float na = a[e] * w.x - b[e] * w.y;
                    const float nb = a[e] * w.y + b[e] * w.x;
                    a[e] = na;
                    b[e] = nb;
                }
                Vec8<DT>::store(k_out, base + 8 * j, a);
                Vec8<DT>::store(k_out, base + half + 8 * j, b);
            } else {
                Vec8<DT>::load(k_in, base + 16 * j, a);
                Vec8<DT>::load(k_in, base + 16 * j + 8, b);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float2 w0 = cs[8 * j + e];
                    const float x0 = a[2 * e] * w0.x - a[2 * e + 1] * w0.y;
                    const float y0 = a[2 * e] * w0.y + a[2 * e + 1] * w0.x;
                    a[2 * e] = x0;
                    a[2 * e + 1] = y0;
                    const float2 w1 = cs[8 * j + 4 + e];
                    const float x1 = b[2 * e] * w1.x - b[2 * e + 1] * w1.y;
                    const float y1 = b[2 * e] * w1.y + b[2 * e + 1] * w1.x;
                    b[2 * e] = x1;
                    b[2 * e + 1] = y1;
                }
                Vec8<DT>::store(k_out, base + 16 * j, a);
                Vec8<DT>::store(k_out, base + 16 * j + 8, b);
            }
        }
    }
}

template <int DT>
cf_status launch_dt(const cf_layer_desc* d, const RopeFreq& f, const void* k_in, void* k_out,
                    const cf_segment* segs, int32_t n_seg, int64_t n_store_tokens, int32_t max_seg_len,
                    int32_t* dev_flag, hipStream_t s) {
    // tokens per block and sweep: few enough that even a short table fills the chip several times over
    int64_t tpb = (int64_t)n_seg * max_seg_len / (256 * 8);
    tpb = tpb < 2 ? 2 : (tpb > kTokPerBlock ? kTokPerBlock : tpb);
    int sweeps = (int)((max_seg_len + tpb - 1) / tpb);
    // enough blocks to cover the chip a few times over, no more
    const int64_t want = 256 * 8;
    int64_t cap = (want + n_seg - 1) / n_seg;
    if (cap < 1) cap = 1;
    if (sweeps > cap) sweeps = (int)cap;
    if (sweeps < 1) sweeps = 1;
    if (sweeps > 65535) sweeps = 65535;
    dim3 grid(n_seg, sweeps);
    if (d->rope_pairing == CF_ROPE_HALF)
        hipLaunchKernelGGL((reposition_kernel<DT, CF_ROPE_HALF>), grid, dim3(kThreads), 0, s, k_in, k_out,
                           segs, n_store_tokens, d->n_kv_heads, d->head_dim, store_token_stride(d), store_head_stride(d), f,
                           dev_flag, (int)tpb, d->max_positions);
    else
        hipLaunchKernelGGL((reposition_kernel<DT, CF_ROPE_INTERLEAVED>), grid, dim3(kThreads), 0, s, k_in,
                           k_out, segs, n_store_tokens, d->n_kv_heads, d->head_dim, store_token_stride(d),
                           store_head_stride(d), f, dev_flag, (int)tpb, d->max_positions);
    CF_HIP(hipGetLastError());
    return CF_OK;
}

// Final Re-Positioning (Alg. 2, Phase 2): gather + rotate.  grid = (batch * seg_stride, sweeps); block
// (b, s) owns segment s of query b.  It first adds up the visible lengths of the query's segments (its own
// output offset is the sum over the segments before it), then streams its tokens: per (token, kv head,
// 8-pair item) two 16-byte K chunks are rotated and two V chunks copied, from the store's (or the own
// block's) layout to the decode cache's.
template <int DT, int PAIRING>
__global__ __launch_bounds__(kThreads) void assemble_kernel(AssembleArgs a, RopeFreq freq, int tok_per_block) {
    __shared__ float2 cs[kMaxHalf];
    __shared__ int s_before, s_total, s_bad, s_off_range;
    const int b = blockIdx.x / a.seg_stride, s = blockIdx.x - b * a.seg_stride;
    const int tid = threadIdx.x;
    int n = a.n_seg[b];
    if (n < 0 || n > a.seg_stride) {
        if (tid == 0 && s == 0 && blockIdx.y == 0) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        n = n < 0 ? 0 : a.seg_stride;
    }
    if (s >= n && s != 0) return;
    const int q0 = a.q_off[b];
    const int tq = min(a.q_off[b + 1] - q0, a.max_tq);
    const int64_t q_total = a.q_off[a.batch];
    if (tid == 0) { s_before = 0; s_total = 0; s_bad = 0; s_off_range = 0; }
    __syncthreads();
    // visible tokens of an entry: 0 for a rejected one (bad: malformed; *bad == 2: positions outside the
    // range), min(len, tq) for the own block
    auto visible = [&](const cf_segment& g, int* bad) {
        const bool self = g.kind == CF_SEG_SELF;
        const int64_t limit = self ? q_total : a.n_store_tokens;
        *bad = g.kind < 0 || g.kind > CF_SEG_SELF || g.len < 0 || g.tok_offset < 0 || g.tok_offset + g.len > limit ||
               (self && (a.k_self == nullptr || a.v_self == nullptr));
        if (*bad) return 0;
        const int vis = self ? min(g.len, tq) : g.len;
        if (!positions_ok(g.stored_start, vis, a.max_positions) || !positions_ok(g.new_start, vis, a.max_positions)) *bad = 2;
        return *bad ? 0 : vis;
    };
    for (int t = tid; t < n; t += kThreads) {
        int bad;
        const int vis = visible(a.segs[(int64_t)b * a.seg_stride + t], &bad);
        if (bad == 1) atomicOr(&s_bad, 1);
        if (bad == 2) atomicOr(&s_off_range, 1);
        atomicAdd(&s_total, vis);
        if (t < s) atomicAdd(&s_before, vis);
    }
    __syncthreads();
    const int64_t run0 = a.final_off[b];
    const bool fits = run0 >= 0 && run0 + s_total <= a.final_capacity;
    if (s == 0 && blockIdx.y == 0 && tid == 0) {
        if (s_bad) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        if (s_off_range) raise_flag(a.dev_flag, CF_FLAG_POS_RANGE);
        if (!fits) raise_flag(a.dev_flag, CF_FLAG_BAD_INDEX);
        a.final_len[b] = fits ? s_total : 0;
    }
    if (s >= n || !fits) return;
    const cf_segment seg = a.segs[(int64_t)b * a.seg_stride + s];
    int bad;
    const int vis = visible(seg, &bad);
    if (vis == 0) return;
    const bool self = seg.kind == CF_SEG_SELF;
    const int half = a.head_dim >> 1;
    const int delta = seg.new_start - seg.stored_start;
    for (int m = tid; m < half; m += kThreads) cs[m] = rope_cos_sin(delta, freq.rev[m]);
    __syncthreads();

    const void* k_in = self ? a.k_self : a.k_store;
    const void* v_in = self ? a.v_self : a.v_store;
    const int64_t in_ts = self ? (int64_t)a.n_kv_heads * a.head_dim : a.store_ts;
    const int64_t in_hs = self ? a.head_dim : a.store_hs;
    const int64_t out0 = run0 + s_before;
    const int items_per_head = half / 8;                 // head_dim % 16 == 0 checked on the host
    const int items_per_tok = a.n_kv_heads * items_per_head;
    for (int tok0 = blockIdx.y * tok_per_block; tok0 < vis; tok0 += gridDim.y * tok_per_block) {
        const int ntok = min(tok_per_block, vis - tok0);
        const int n_items = ntok * items_per_tok;
        for (int it = tid; it < n_items; it += kThreads) {
            const int tok = (int)div_exact((unsigned)it, (unsigned)items_per_tok);
            const int r = it - tok * items_per_tok;
            const int head = (int)div_exact((unsigned)r, (unsigned)items_per_head);
            const int j = r - head * items_per_head;
            const int64_t src = (seg.tok_offset + tok0 + tok) * in_ts + (int64_t)head * in_hs;
            const int64_t dst = (out0 + tok0 + tok) * a.final_ts + (int64_t)head * a.final_hs;
            const int o0 = PAIRING == CF_ROPE_HALF ? 8 * j : 16 * j;
            const int o1 = PAIRING == CF_ROPE_HALF ? half + 8 * j : 16 * j + 8;
            float x[8], y[8], va[8], vb[8];
            Vec8<DT>::load(k_in, src + o0, x);
            Vec8<DT>::load(k_in, src + o1, y);
            Vec8<DT>::load(v_in, src + o0, va);
            Vec8<DT>::load(v_in, src + o1, vb);
            if (delta != 0) {
                if (PAIRING == CF_ROPE_HALF) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float2 w = cs[8 * j + e];
                        const float nx = x[e] * w.x - y[e] * w.y;
                        const float ny = x[e] * w.y + y[e] * w.x;
                        x[e] = nx;
                        y[e] = ny;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float2 w0 = cs[8 * j + e];
                        const float x0 = x[2 * e] * w0.x - x[2 * e + 1] * w0.y;
                        const float y0 = x[2 * e] * w0.y + x[2 * e + 1] * w0.x;
                        x[2 * e] = x0;
                        x[2 * e + 1] = y0;
                        const float2 w1 = cs[8 * j + 4 + e];
                        const float x1 = y[2 * e] * w1.x - y[2 * e + 1] * w1.y;
                        const float y1 = y[2 * e] * w1.y + y[2 * e + 1] * w1.x;
                        y[2 * e] = x1;
                        y[2 * e + 1] = y1;
                    }
                }
            }
            Vec8<DT>::store(a.k_final, dst + o0, x);
            Vec8<DT>::store(a.k_final, dst + o1, y);
            Vec8<DT>::store(a.v_final, dst + o0, va);
            Vec8<DT>::store(a.v_final, dst + o1, vb);
            if (a.final_pos && r == 0) a.final_pos[out0 + tok0 + tok] = seg.new_start + tok0 + tok;
        }
    }
}

template <int DT>
cf_status launch_assemble_dt(const cf_layer_desc* d, const RopeFreq& f, const AssembleArgs& a, int32_t max_seg_len,
                             hipStream_t s) {
    // tokens per block and sweep: few enough that even a short table fills the chip several times over
    const int64_t blocks = (int64_t)a.batch * a.seg_stride;
    int64_t tpb = blocks * max_seg_len / (256 * 8);
    tpb = tpb < 2 ? 2 : (tpb > kTokPerBlock ? kTokPerBlock : tpb);
    int64_t sweeps = (max_seg_len + tpb - 1) / tpb;
    if (sweeps > 65535) sweeps = 65535;
    dim3 grid((unsigned)blocks, (unsigned)sweeps);
    if (d->rope_pairing == CF_ROPE_HALF)
        hipLaunchKernelGGL((assemble_kernel<DT, CF_ROPE_HALF>), grid, dim3(kThreads), 0, s, a, f, (int)tpb);
    else
        hipLaunchKernelGGL((assemble_kernel<DT, CF_ROPE_INTERLEAVED>), grid, dim3(kThreads), 0, s, a, f, (int)tpb);
    CF_HIP(hipGetLastError());
    return CF_OK;
}

}  // namespace

cf_status launch_assemble(const cf_layer_desc* d, const RopeFreq& f, const AssembleArgs& a, int32_t max_seg_len,
                          hipStream_t s) {
    switch (d->dtype) {
        case CF_F32: return launch_assemble_dt<CF_F32>(d, f, a, max_seg_len, s);
        case CF_BF16: return launch_assemble_dt<CF_BF16>(d, f, a, max_seg_len, s);
        default: return launch_assemble_dt<CF_F16>(d, f, a, max_seg_len, s);
    }
}

cf_status launch_reposition(const cf_layer_desc* d, const RopeFreq& f, const void* k_in, void* k_out,
                            const cf_segment* segs, int32_t n_seg, int64_t n_store_tokens,
                            int32_t max_seg_len, int32_t* dev_flag, hipStream_t s) {
    switch (d->dtype) {
        case CF_F32: return launch_dt<CF_F32>(d, f, k_in, k_out, segs, n_seg, n_store_tokens, max_seg_len, dev_flag, s);
        case CF_BF16: return launch_dt<CF_BF16>(d, f, k_in, k_out, segs, n_seg, n_store_tokens, max_seg_len, dev_flag, s);
        default: return launch_dt<CF_F16>(d, f, k_in, k_out, segs, n_seg, n_store_tokens, max_seg_len, dev_flag, s);
    }
}

}  // namespace cf
