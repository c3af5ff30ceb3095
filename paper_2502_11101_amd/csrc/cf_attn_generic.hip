// Generic prefill attention: any dtype, head_dim (multiple of 16, <= 256) and RoPE pairing.
// One wavefront per (query, row, q head) walks the query's segments with an online softmax
// (Eq. 1), rotating each key on the fly by its relative position shift (Eq. 5) in fp32.
// It serves the fp32 configurations and every 16-bit shape the MFMA kernels do not cover.
//
// Per row it leaves, for every segment, the pair (running max at the end of the segment,
// sum of exp2(score - that max) over the segment's visible tokens) and the row's final
// (max, normaliser); a second kernel turns those into per-segment attention mass (the
// document-wise score of Alg. 2) with a fixed-order reduction over rows and heads.
#include "cf_common.h"

namespace cf {
namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / kWave;

template <int DT>
__device__ __forceinline__ void load8(const void* base, int64_t idx, float (&v)[8]) {
    if (DT == CF_F32) {
        const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + idx);
        const float4 a = p[0], b = p[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
        const uint4 r = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + idx);
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
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
}

// workspace layout: rowstat[rows*Hq] float2 (M, Z) | rowseg[rows*Hq*seg_stride] float2 (m, l)
template <int DT, int PAIRING>
__global__ __launch_bounds__(kThreads) void attn_rows_kernel(AttnArgs a, RopeFreq freq, float2* rowstat,
                                                             float2* rowseg) {
    using E = Elem<DT>;
    using T = typename E::type;
    __shared__ float q_lds[kWavesPerBlock][kMaxHeadDim];
    __shared__ float2 cs_lds[kWavesPerBlock][kMaxHalf];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t gw = (int64_t)blockIdx.x * kWavesPerBlock + wave;
    const int hq = a.n_q_heads, d = a.head_dim, half = d >> 1;
    const int64_t per_query = (int64_t)a.max_tq * hq;
    const int b = (int)(gw / per_query);
    if (b >= a.batch) return;
    const int rem = (int)(gw - (int64_t)b * per_query);
    const int t = rem / hq;
    const int h = rem - t * hq;
    const int q0 = a.q_off[b];
    const int tq = a.q_off[b + 1] - q0;
    if (t >= tq) return;
    const int64_t q_total = a.q_off[a.batch];
    const int64_t row = (int64_t)q0 + t;
    const int kvh = h / (hq / a.n_kv_heads);
    const int64_t kv_row = (int64_t)a.n_kv_heads * d;

    float* qv = q_lds[wave];
    float2* cs = cs_lds[wave];
    const T* qp = static_cast<const T*>(a.q) + (row * hq + h) * d;
    for (int c = lane; c < d; c += kWave) qv[c] = E::load(qp + c);

    int nseg = a.n_seg[b];
    if (nseg > a.seg_stride || nseg < 0) {
        if (lane == 0) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        nseg = nseg < 0 ? 0 : a.seg_stride;
    }
    const int q_new = a.q_new_start[b];
    const int qdelta = q_new - a.q_stored_start;
    const int64_t rs_base = (row * hq + h) * (int64_t)a.seg_stride;
    // a query placed (or stored) outside the positional range attends nothing
    const int tq_vis = min(tq, a.max_tq);
    const bool q_ok = positions_ok(q_new, tq_vis, a.max_positions) && positions_ok(a.q_stored_start, tq_vis, a.max_positions);
    if (!q_ok && lane == 0) raise_flag(a.dev_flag, CF_FLAG_POS_RANGE);

    float m_run = -INFINITY, l_run = 0.f;
    float o[4] = {0.f, 0.f, 0.f, 0.f};

    for (int s = 0; s < nseg; ++s) {
        const cf_segment seg = a.segs[(int64_t)b * a.seg_stride + s];
        const bool self = seg.kind == CF_SEG_SELF;
        const int64_t limit = self ? q_total : a.n_store_tokens;
        const bool bad = seg.kind < 0 || seg.kind > CF_SEG_SELF || seg.len < 0 || seg.tok_offset < 0 ||
                         seg.tok_offset + seg.len > limit || (self && a.k_self == nullptr);
        float seg_l = 0.f;
        const int len_vis = bad ? 0 : (self ? min(seg.len, tq_vis) : seg.len);
        const bool off_range = !(positions_ok(seg.new_start, len_vis, a.max_positions) &&
                                 positions_ok(seg.stored_start, len_vis, a.max_positions));
        if (bad) {
            if (lane == 0) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        } else if (off_range || !q_ok) {
            if (off_range && lane == 0) raise_flag(a.dev_flag, CF_FLAG_POS_RANGE);
        } else {
            const int vis = self ? min(seg.len, t + 1) : seg.len;
            const int delta = seg.new_start - seg.stored_start - qdelta;
            __builtin_amdgcn_wave_barrier();
            for (int m = lane; m < half; m += kWave) cs[m] = rope_cos_sin(delta, freq.rev[m]);
            __builtin_amdgcn_wave_barrier();
            const T* kb = static_cast<const T*>(self ? a.k_self : a.k_store);
            const T* vb = static_cast<const T*>(self ? a.v_self : a.v_store);
            const int64_t tok_stride = self ? kv_row : a.store_ts;       // the own block is always token-major
            const int64_t head_off = (int64_t)kvh * (self ? d : a.store_hs);
            for (int tok0 = 0; tok0 < vis; tok0 += kWave) {
                const int tok = tok0 + lane;
                const bool valid = tok < vis;
                float sc = -INFINITY;
                if (valid) {
                    const int64_t kbase = (seg.tok_offset + tok) * tok_stride + head_off;
                    float acc = 0.f;
                    for (int j = 0; j < half / 8; ++j) {
                        float x[8], y[8];
                        if (PAIRING == CF_ROPE_HALF) {
                            load8<DT>(kb, kbase + 8 * j, x);
                            load8<DT>(kb, kbase + half + 8 * j, y);
#pragma unroll
                            for (int e = 0; e < 8; ++e) {
                                const int m = 8 * j + e;
                                const float2 w = cs[m];
                                const float ka = x[e] * w.x - y[e] * w.y;
                                const float kc = x[e] * w.y + y[e] * w.x;
                                acc += qv[m] * ka + qv[m + half] * kc;
                            }
                        } else {
                            load8<DT>(kb, kbase + 16 * j, x);
                            load8<DT>(kb, kbase + 16 * j + 8, y);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const int m0 = 8 * j + e, m1 = 8 * j + 4 + e;
                                const float2 w0 = cs[m0], w1 = cs[m1];
                                const float a0 = x[2 * e] * w0.x - x[2 * e + 1] * w0.y;
                                const float b0 = x[2 * e] * w0.y + x[2 * e + 1] * w0.x;
                                const float a1 = y[2 * e] * w1.x - y[2 * e + 1] * w1.y;
                                const float b1 = y[2 * e] * w1.y + y[2 * e + 1] * w1.x;
                                acc += qv[2 * m0] * a0 + qv[2 * m0 + 1] * b0 + qv[2 * m1] * a1 + qv[2 * m1 + 1] * b1;
                            }
                        }
                    }
                    sc = acc * a.scale_log2e;
                }
                const float m_new = fmaxf(m_run, wave_max(sc));   // finite: lane 0 is always valid
                const float alpha = exp2f(m_run - m_new);          // exp2(-inf) = 0 on the first block
                const float p = valid ? exp2f(sc - m_new) : 0.f;
                const float bs = wave_sum(p);
                l_run = l_run * alpha + bs;
                seg_l = seg_l * alpha + bs;
                m_run = m_new;
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] *= alpha;
                const int cnt = min(kWave, vis - tok0);
                for (int jj = 0; jj < cnt; ++jj) {
                    const float pj = __shfl(p, jj);
                    const T* vp = vb + (seg.tok_offset + tok0 + jj) * tok_stride + head_off;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int c = lane + kWave * i;
                        if (c < d) o[i] += pj * E::load(vp + c);
                    }
                }
            }
        }
        if (lane == 0) rowseg[rs_base + s] = make_float2(m_run, seg_l);
    }
    if (lane == 0) rowstat[row * hq + h] = make_float2(m_run, l_run);
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
    T* op = static_cast<T*>(a.out) + (row * hq + h) * d;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = lane + kWave * i;
        if (c < d) E::store(op + c, o[i] * inv);
    }
}

// mass[b, s] = sum over rows t and q heads h of l[t,h,s] * exp2(m[t,h,s] - M[t,h]) / Z[t,h],
// accumulated in double with a fixed partition and a fixed tree, then S += mass.
__global__ __launch_bounds__(kThreads) void mass_reduce_kernel(AttnArgs a, const float2* rowstat,
                                                               const float2* rowseg) {
    __shared__ double part[kThreads];
    const int b = blockIdx.y, s = blockIdx.x;
    const int nseg = min(max(a.n_seg[b], 0), a.seg_stride);
    if (s >= nseg) return;
    const int q0 = a.q_off[b];
    const int tq = min(a.q_off[b + 1] - q0, a.max_tq);
    const int hq = a.n_q_heads;
    const int n = tq * hq;
    double acc = 0.0;
    for (int i = threadIdx.x; i < n; i += kThreads) {
        const int64_t rh = (int64_t)q0 * hq + i;
        const float2 st = rowstat[rh];
        const float2 ml = rowseg[rh * a.seg_stride + s];
        if (ml.y > 0.f && st.y > 0.f) acc += (double)(ml.y * exp2f(ml.x - st.x)) / (double)st.y;
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) a.mass[(int64_t)b * a.seg_stride + s] = (float)part[0];
}

// S += s^l (Alg. 2): one thread per (query, document slot) adds the masses of the segments that feed its
// slot, in table order — no atomics, so the result does not depend on timing even when a document is
// listed as several segments.
__global__ __launch_bounds__(kThreads) void score_add_kernel(AttnArgs a) {
    const int b = blockIdx.y;
    const int doc = blockIdx.x * kThreads + threadIdx.x;
    if (doc >= a.score_stride) return;
    const int nseg = min(max(a.n_seg[b], 0), a.seg_stride);
    float sum = 0.f;
    bool any = false;
    for (int s = 0; s < nseg; ++s)
        if (a.segs[(int64_t)b * a.seg_stride + s].doc == doc) { sum += a.mass[(int64_t)b * a.seg_stride + s]; any = true; }
    if (any) a.score_accum[(int64_t)b * a.score_stride + doc] += sum;
}

}  // namespace

size_t generic_workspace_bytes(const cf_layer_desc* d, int32_t batch, int32_t max_tq, int32_t seg_stride) {
    const size_t rows = (size_t)batch * max_tq * d->n_q_heads;
    return rows * sizeof(float2) * (1 + (size_t)seg_stride);
}

cf_status launch_attention_generic(const AttnArgs& a, const RopeFreq& f, hipStream_t s) {
    const size_t rows = (size_t)a.batch * a.max_tq * a.n_q_heads;
    float2* rowstat = static_cast<float2*>(a.workspace);
    float2* rowseg = rowstat + rows;
    const int64_t waves = (int64_t)a.batch * a.max_tq * a.n_q_heads;
    const unsigned blocks = (unsigned)((waves + kWavesPerBlock - 1) / kWavesPerBlock);
#define CF_LAUNCH_ROWS(DT, PR) \
    hipLaunchKernelGGL((attn_rows_kernel<DT, PR>), dim3(blocks), dim3(kThreads), 0, s, a, f, rowstat, rowseg)
    const bool halfp = a.pairing == CF_ROPE_HALF;
    if (a.dtype == CF_F32) { if (halfp) CF_LAUNCH_ROWS(CF_F32, CF_ROPE_HALF); else CF_LAUNCH_ROWS(CF_F32, CF_ROPE_INTERLEAVED); }
    else if (a.dtype == CF_BF16) { if (halfp) CF_LAUNCH_ROWS(CF_BF16, CF_ROPE_HALF); else CF_LAUNCH_ROWS(CF_BF16, CF_ROPE_INTERLEAVED); }
    else { if (halfp) CF_LAUNCH_ROWS(CF_F16, CF_ROPE_HALF); else CF_LAUNCH_ROWS(CF_F16, CF_ROPE_INTERLEAVED); }
#undef CF_LAUNCH_ROWS
    CF_HIP(hipGetLastError());
    if (a.mass == nullptr) return CF_OK;             // outputs only
    hipLaunchKernelGGL(mass_reduce_kernel, dim3(a.seg_stride, a.batch), dim3(kThreads), 0, s, a, rowstat, rowseg);
    CF_HIP(hipGetLastError());
    if (a.score_accum == nullptr) return CF_OK;
    hipLaunchKernelGGL(score_add_kernel, dim3((a.score_stride + kThreads - 1) / kThreads, a.batch), dim3(kThreads), 0, s, a);
    CF_HIP(hipGetLastError());
    return CF_OK;
}

}  // namespace cf
