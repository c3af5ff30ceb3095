// 16-bit MFMA prefill attention for gfx950 (head_dim 128, half-split RoPE pairing).
//
// Work decomposition.  For one (query b, kv head, tile of 64 stacked query rows) — a "unit" —
// the attended tokens are cut into blocks of 32 tokens that never straddle a segment.  The
// block list of a unit is divided evenly over `nsplit` workgroups and, inside a workgroup,
// over its 4 wavefronts; a wavefront is therefore an independent flash-attention worker over a
// contiguous run of blocks ("sub-split") for all 64 rows of the tile:
//   * K/V blocks are fetched with coalesced 16-byte loads into registers one block ahead,
//   * the key block is rotated in registers by the segment's relative position shift (Eq. 5;
//     cos/sin of the shift per 2-D slice, angle reduced in fp64) and rounded once to the storage
//     type while it is staged into LDS — rotated keys never return to memory,
//   * S^T = K Q^T and O^T += V^T P^T run on v_mfma_f32_32x32x16 (Q fragments live in registers;
//     the transposed forms keep one query row per lane, so softmax statistics need one cross-lane
//     exchange and rescaling needs none),
//   * softmax is online in fp32 in the exp2 domain.
// Per segment a wavefront leaves (running max, sum of exp2) per row; a second kernel merges the
// partial outputs of the splits and turns those pairs into per-segment attention mass (the
// document-wise score of Alg. 2) with fixed-order reductions.
#include <cstdlib>

#include "cf_common.h"

namespace cf {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kD = 128;
constexpr int kHalf = 64;
constexpr int kBlk = 32;        // tokens per block
constexpr int kRowTile = 64;    // stacked query rows per unit
constexpr int kSK = 136;        // LDS row stride of a staged K block, elements (272 B)
constexpr int kSV = 40;         // LDS row stride of a staged V^T block, elements (80 B)
constexpr int kKBytes = kBlk * kSK * 2;
constexpr int kVBytes = kD * kSV * 2;
constexpr int kStageBytes = kKBytes + kVBytes;          // per wavefront
constexpr int kMaxSegs = 512;
constexpr int kORegs = 128;                             // fp32 accumulator registers per lane

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct Plan {
    int rowtiles, units_per_b, units, nsplit, nsub, slots;
    size_t off_counters, off_ml, off_opart, off_massml, off_massunit, total;
};

Plan make_plan(int n_q_heads, int n_kv_heads, int batch, int max_tq, int seg_stride, int64_t max_kv_tokens) {
    Plan p;
    const int group = n_q_heads / n_kv_heads;
    p.rowtiles = (group * max_tq + kRowTile - 1) / kRowTile;
    p.units_per_b = n_kv_heads * p.rowtiles;
    p.units = batch * p.units_per_b;
    const int64_t est_blocks = max_kv_tokens / kBlk + seg_stride;
    int64_t ns = (256 + p.units - 1) / p.units;
    const int64_t cap = est_blocks / kWaves > 1 ? est_blocks / kWaves : 1;
    if (ns > cap) ns = cap;
    if (ns > 64) ns = 64;
    if (ns < 1) ns = 1;
    p.nsplit = (int)ns;
    p.nsub = p.nsplit * kWaves;
    p.slots = seg_stride + p.nsub;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
    p.off_counters = take((size_t)batch * 4);
    p.off_ml = take((size_t)p.units * p.nsplit * kRowTile * sizeof(float2));
    p.off_opart = take((size_t)p.units * p.nsplit * kORegs * kWave * sizeof(float));
    p.off_massml = take((size_t)p.units * p.slots * kRowTile * sizeof(float2));
    p.off_massunit = take((size_t)p.units * seg_stride * sizeof(float));
    p.total = off;
    return p;
}

// Per-query segment table in LDS, with the block prefix that defines the partition.
struct SegTable {
    int64_t tok[kMaxSegs];     // first token in its tensor
    int32_t vis[kMaxSegs];     // visible tokens (0 for a rejected entry)
    int32_t delta[kMaxSegs];   // relative shift: (new - stored) - (q_new - q_stored)
    int32_t self[kMaxSegs];    // 1 for the causal own block
    int32_t blk0[kMaxSegs + 1];// exclusive prefix of 32-token block counts
    int32_t n;
};

// Every workgroup that works on query b builds the same table (both kernels use this).
__device__ void build_table(const AttnArgs& a, int b, SegTable* t) {
    int n = a.n_seg[b];
    if (n < 0 || n > a.seg_stride) {
        if (threadIdx.x == 0) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        n = n < 0 ? 0 : a.seg_stride;
    }
    const int q0 = a.q_off[b];
    const int tq = min(a.q_off[b + 1] - q0, a.max_tq);
    const int64_t q_total = a.q_off[a.batch];
    const int qdelta = a.q_new_start[b] - a.q_stored_start;
    for (int s = threadIdx.x; s < n; s += kThreads) {
        const cf_segment seg = a.segs[(int64_t)b * a.seg_stride + s];
        const bool self = seg.kind == CF_SEG_SELF;
        const int64_t limit = self ? q_total : a.n_store_tokens;
        const bool bad = seg.kind < 0 || seg.kind > CF_SEG_SELF || seg.len < 0 || seg.tok_offset < 0 ||
                         seg.tok_offset + seg.len > limit || (self && a.k_self == nullptr);
        if (bad) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        const int vis = bad ? 0 : (self ? min(seg.len, tq) : seg.len);
        t->tok[s] = seg.tok_offset;
        t->vis[s] = vis;
        t->delta[s] = seg.new_start - seg.stored_start - qdelta;
        t->self[s] = self ? 1 : 0;
        t->blk0[s + 1] = (vis + kBlk - 1) / kBlk;
    }
    if (threadIdx.x == 0) { t->n = n; t->blk0[0] = 0; }
    __syncthreads();
    if (threadIdx.x < kWave) {                       // inclusive scan by the first wavefront
        int carry = 0;
        for (int c0 = 0; c0 < n; c0 += kWave) {
            const int s = c0 + threadIdx.x;
            int v = s < n ? t->blk0[s + 1] : 0;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int u = __shfl_up(v, o);
                if ((int)threadIdx.x >= o) v += u;
            }
            if (s < n) t->blk0[s + 1] = v + carry;
            carry += __shfl(v, kWave - 1);
        }
    }
    __syncthreads();
}

// sub-split ss of a unit owns blocks [lo, hi) of its `total` blocks
__device__ __forceinline__ void sub_range(int total, int nsplit, int ss, int* lo, int* hi) {
    const int split = ss / kWaves, w = ss % kWaves;
    const int b0 = (int)(((int64_t)total * split) / nsplit);
    const int b1 = (int)(((int64_t)total * (split + 1)) / nsplit);
    const int n = b1 - b0;
    *lo = b0 + (n * w) / kWaves;
    *hi = b0 + (n * (w + 1)) / kWaves;
}

template <int DT> struct Mma;
template <> struct Mma<CF_BF16> {
    static __device__ __forceinline__ f32x16 run(uint4 a, uint4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_f(uint32_t bits) { return bf16_bits_to_float(bits); }
    static __device__ __forceinline__ uint32_t from_f(float f) { return float_to_bf16_bits(f); }
};
template <> struct Mma<CF_F16> {
    static __device__ __forceinline__ f32x16 run(uint4 a, uint4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float to_f(uint32_t bits) { return f16_bits_to_float(bits); }
    static __device__ __forceinline__ uint32_t from_f(float f) { return float_to_f16_bits(f); }
};

template <int DT>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    return Mma<DT>::from_f(lo) | (Mma<DT>::from_f(hi) << 16);
}

struct BlockDesc {
    int seg;       // segment index
    int tok0;      // first token of the block inside the segment
    int ntok;      // valid tokens (1..32)
};

template <int DT>
__global__ __launch_bounds__(kThreads) void attn_mfma_kernel(AttnArgs a, RopeFreq freq, Plan p) {
    __shared__ SegTable tbl;
    __shared__ __attribute__((aligned(16))) unsigned char stage_all[kWaves * kStageBytes];
    __shared__ float2 ml_w[kWaves][kRowTile];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int li = lane & 31, lg = lane >> 5;

    const int bid = blockIdx.x;
    const int split = bid % p.nsplit;
    const int unit = bid / p.nsplit;
    const int rowtile = unit % p.rowtiles;
    const int hkv = (unit / p.rowtiles) % a.n_kv_heads;
    const int b = unit / p.units_per_b;

    if (bid == 0) {
        int32_t* counters = reinterpret_cast<int32_t*>(static_cast<char*>(a.workspace) + p.off_counters);
        for (int i = threadIdx.x; i < a.batch; i += kThreads) counters[i] = 0;
    }

    const int hq = a.n_q_heads;
    const int group = hq / a.n_kv_heads;
    const int q0 = a.q_off[b];
    const int tq = min(a.q_off[b + 1] - q0, a.max_tq);
    const int n_rows = group * tq;                 // stacked rows of this (b, kv head)

    // ---- Q fragments: row m = g*tq + t of the stack is q[q0 + t][hkv*group + g]
    uint4 qf[2][8];
    int trow[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int m = rowtile * kRowTile + rb * 32 + li;
        const bool valid = m < n_rows;
        const int gi = valid ? m / tq : 0;
        const int t = valid ? m - gi * tq : 0;
        trow[rb] = valid ? t : 0x7fffffff;        // padding rows: nothing to mask, results unused
        const uint16_t* qp = static_cast<const uint16_t*>(a.q) + (((int64_t)q0 + t) * hq + hkv * group + gi) * kD + 8 * lg;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            qf[rb][kk] = valid ? *reinterpret_cast<const uint4*>(qp + 16 * kk) : make_uint4(0, 0, 0, 0);
    }

    build_table(a, b, &tbl);

    const int total = tbl.blk0[tbl.n];
    int wb0, wb1;
    sub_range(total, p.nsplit, split * kWaves + wave, &wb0, &wb1);

    unsigned char* stage = stage_all + wave * kStageBytes;
    uint16_t* k_lds = reinterpret_cast<uint16_t*>(stage);
    uint16_t* v_lds = reinterpret_cast<uint16_t*>(stage + kKBytes);

    f32x16 acc[4][2];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][rb][r] = 0.f;
    float m_run[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};
    float seg_l[2] = {0.f, 0.f};

    const int64_t kv_row = (int64_t)a.n_kv_heads * kD;
    float2* massml = reinterpret_cast<float2*>(static_cast<char*>(a.workspace) + p.off_massml) +
                     (int64_t)unit * p.slots * kRowTile;
    const int ss = split * kWaves + wave;

    // staging registers (one block ahead)
    uint4 kreg_a[4], kreg_b[4], vreg[2][4];
    const int kj = lane & 7, ktr = lane >> 3;       // K: 8 lanes per token, 8 tokens per load
    const int vj = lane & 15, vtg = lane >> 4;      // V: 16 lanes per token, 4 tokens per load

    auto describe = [&](int blk, int s) {
        BlockDesc d;
        d.seg = s;
        d.tok0 = (blk - tbl.blk0[s]) * kBlk;
        d.ntok = min(kBlk, tbl.vis[s] - d.tok0);
        return d;
    };
    auto locate = [&](int blk, int s) {             // first segment at or after s whose blocks reach past blk
        while (tbl.blk0[s + 1] <= blk) ++s;
        return s;
    };
    auto issue_loads = [&](const BlockDesc& d) {
        const bool self = tbl.self[d.seg] != 0;
        const uint16_t* kb = static_cast<const uint16_t*>(self ? a.k_self : a.k_store);
        const uint16_t* vb = static_cast<const uint16_t*>(self ? a.v_self : a.v_store);
        const int64_t base = (tbl.tok[d.seg] + d.tok0) * kv_row + (int64_t)hkv * kD;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int tok = 8 * it + ktr;
            if (tok < d.ntok) {
                const uint16_t* pk = kb + base + tok * kv_row + 8 * kj;
                kreg_a[it] = *reinterpret_cast<const uint4*>(pk);
                kreg_b[it] = *reinterpret_cast<const uint4*>(pk + kHalf);
            } else {
                kreg_a[it] = make_uint4(0, 0, 0, 0);
                kreg_b[it] = make_uint4(0, 0, 0, 0);
            }
        }
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int tok = 16 * it + 4 * vtg + r;
                vreg[it][r] = tok < d.ntok ? *reinterpret_cast<const uint4*>(vb + base + tok * kv_row + 8 * vj)
                                           : make_uint4(0, 0, 0, 0);
            }
    };
    auto emit = [&](int s) {                        // (running max, segment sum) per row for segment s
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const float tot = seg_l[rb] + __shfl_xor(seg_l[rb], 32);
            if (lg == 0) massml[(int64_t)(s + ss) * kRowTile + rb * 32 + li] = make_float2(m_run[rb], tot);
        }
    };

    if (wb0 < wb1) {
        int s_next = locate(wb0, 0);
        BlockDesc nd = describe(wb0, s_next);
        issue_loads(nd);
        int cur_seg = -1;
        int cur_delta = 0;
        float cs_c[8], cs_s[8];
        for (int blk = wb0; blk < wb1; ++blk) {
            const BlockDesc cd = nd;
            if (cd.seg != cur_seg) {
                if (cur_seg >= 0) emit(cur_seg);
                cur_seg = cd.seg;
                seg_l[0] = seg_l[1] = 0.f;
                cur_delta = tbl.delta[cur_seg];
                if (cur_delta != 0) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float2 w = rope_cos_sin(cur_delta, freq.rev[8 * kj + e]);
                        cs_c[e] = w.x;
                        cs_s[e] = w.y;
                    }
                }
            }
            // ---- stage K: rotate pairs (c, c + 64), round once, write [token][c]
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                uint4 ra = kreg_a[it], rb4 = kreg_b[it];
                if (cur_delta != 0) {
                    uint32_t wa[4] = {ra.x, ra.y, ra.z, ra.w}, wb[4] = {rb4.x, rb4.y, rb4.z, rb4.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float a0 = Mma<DT>::to_f(wa[i] & 0xffffu), a1 = Mma<DT>::to_f(wa[i] >> 16);
                        const float b0 = Mma<DT>::to_f(wb[i] & 0xffffu), b1 = Mma<DT>::to_f(wb[i] >> 16);
                        const float c0 = cs_c[2 * i], s0 = cs_s[2 * i], c1 = cs_c[2 * i + 1], s1 = cs_s[2 * i + 1];
                        wa[i] = pack2<DT>(a0 * c0 - b0 * s0, a1 * c1 - b1 * s1);
                        wb[i] = pack2<DT>(a0 * s0 + b0 * c0, a1 * s1 + b1 * c1);
                    }
                    ra = make_uint4(wa[0], wa[1], wa[2], wa[3]);
                    rb4 = make_uint4(wb[0], wb[1], wb[2], wb[3]);
                }
                uint16_t* dst = k_lds + (8 * it + ktr) * kSK + 8 * kj;
                *reinterpret_cast<uint4*>(dst) = ra;
                *reinterpret_cast<uint4*>(dst + kHalf) = rb4;
            }
            // ---- stage V transposed: [dv][token], tokens ordered so that each MFMA k-group is contiguous
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const uint32_t x0[4] = {vreg[it][0].x, vreg[it][0].y, vreg[it][0].z, vreg[it][0].w};
                const uint32_t x1[4] = {vreg[it][1].x, vreg[it][1].y, vreg[it][1].z, vreg[it][1].w};
                const uint32_t x2[4] = {vreg[it][2].x, vreg[it][2].y, vreg[it][2].z, vreg[it][2].w};
                const uint32_t x3[4] = {vreg[it][3].x, vreg[it][3].y, vreg[it][3].z, vreg[it][3].w};
                // quad (4 consecutive tokens) index in the block: 4*it + vtg; its slot in the row
                const int pos = (2 * it + (vtg & 1)) * 8 + (vtg >> 1) * 4;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint2 lo, hi;
                    lo.x = __builtin_amdgcn_perm(x1[i], x0[i], 0x05040100u);
                    lo.y = __builtin_amdgcn_perm(x3[i], x2[i], 0x05040100u);
                    hi.x = __builtin_amdgcn_perm(x1[i], x0[i], 0x07060302u);
                    hi.y = __builtin_amdgcn_perm(x3[i], x2[i], 0x07060302u);
                    *reinterpret_cast<uint2*>(v_lds + (8 * vj + 2 * i) * kSV + pos) = lo;
                    *reinterpret_cast<uint2*>(v_lds + (8 * vj + 2 * i + 1) * kSV + pos) = hi;
                }
            }
            // ---- next block's loads fly during this block's math
            if (blk + 1 < wb1) {
                s_next = locate(blk + 1, s_next);
                nd = describe(blk + 1, s_next);
                issue_loads(nd);
            }
            __builtin_amdgcn_wave_barrier();

            // ---- S^T = K Q^T : lane (li, lg) gets, for query row li, tokens 8*(r>>2) + 4*lg + (r&3)
            f32x16 sc[2];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) sc[rb][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const uint4 ka = *reinterpret_cast<const uint4*>(k_lds + li * kSK + 16 * kk + 8 * lg);
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) sc[rb] = Mma<DT>::run(ka, qf[rb][kk], sc[rb]);
            }
            // ---- online softmax (exp2 domain), fp32
            const bool causal = tbl.self[cd.seg] != 0;
            uint4 pfrag[2][2];
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                float x[16];
                float mloc = -INFINITY;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int tk = 8 * (r >> 2) + 4 * lg + (r & 3);
                    const bool ok = tk < cd.ntok && (!causal || cd.tok0 + tk <= trow[rb]);
                    x[r] = ok ? sc[rb][r] * a.scale_log2e : -INFINITY;
                    mloc = fmaxf(mloc, x[r]);
                }
                mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
                const float m_new = fmaxf(m_run[rb], mloc);
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = exp2f(m_run[rb] - m_safe);
                float lsum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    x[r] = exp2f(x[r] - m_safe);
                    lsum += x[r];
                }
                l_run[rb] = l_run[rb] * alpha + lsum;
                seg_l[rb] = seg_l[rb] * alpha + lsum;
                m_run[rb] = m_new;
                if (__any(alpha != 1.f)) {
#pragma unroll
                    for (int db = 0; db < 4; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[db][rb][r] *= alpha;
                }
                pfrag[rb][0] = make_uint4(pack2<DT>(x[0], x[1]), pack2<DT>(x[2], x[3]), pack2<DT>(x[4], x[5]), pack2<DT>(x[6], x[7]));
                pfrag[rb][1] = make_uint4(pack2<DT>(x[8], x[9]), pack2<DT>(x[10], x[11]), pack2<DT>(x[12], x[13]), pack2<DT>(x[14], x[15]));
            }
            // ---- O^T += V^T P^T
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const uint4 va = *reinterpret_cast<const uint4*>(v_lds + (32 * db + li) * kSV + (2 * h + lg) * 8);
#pragma unroll
                    for (int rb = 0; rb < 2; ++rb) acc[db][rb] = Mma<DT>::run(va, pfrag[rb][h], acc[db][rb]);
                }
            __builtin_amdgcn_wave_barrier();
        }
        emit(cur_seg);
    }

    // ---- merge the 4 sub-splits of this workgroup (same rows, different tokens)
    float l_tot[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        l_tot[rb] = l_run[rb] + __shfl_xor(l_run[rb], 32);
        if (lg == 0) ml_w[wave][rb * 32 + li] = make_float2(m_run[rb], l_tot[rb]);
    }
    __syncthreads();
    float mx[2], zz[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int row = rb * 32 + li;
        float m = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) m = fmaxf(m, ml_w[w][row].x);
        const float ms = m == -INFINITY ? 0.f : m;
        float z = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) z += ml_w[w][row].y * exp2f(ml_w[w][row].x - ms);
        mx[rb] = m;
        zz[rb] = z;
        const float f = exp2f(m_run[rb] - ms);
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][rb][r] *= f;
    }
    float* red = reinterpret_cast<float*>(stage_all);           // 2 slots of kORegs*64 floats (64 KB)
    auto put = [&](int slot) {
        float* dst = red + slot * kORegs * kWave + lane;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) dst[((db * 2 + rb) * 16 + r) * kWave] = acc[db][rb][r];
    };
    auto add = [&](int slot) {
        const float* src = red + slot * kORegs * kWave + lane;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[db][rb][r] += src[((db * 2 + rb) * 16 + r) * kWave];
    };
    if (wave >= 2) put(wave - 2);
    __syncthreads();
    if (wave < 2) add(wave);
    __syncthreads();
    if (wave == 1) put(0);
    __syncthreads();
    if (wave == 0) {
        add(0);
        float* opart = reinterpret_cast<float*>(static_cast<char*>(a.workspace) + p.off_opart) +
                       ((int64_t)unit * p.nsplit + split) * kORegs * kWave + lane;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) opart[((db * 2 + rb) * 16 + r) * kWave] = acc[db][rb][r];
        float2* ml = reinterpret_cast<float2*>(static_cast<char*>(a.workspace) + p.off_ml) +
                     ((int64_t)unit * p.nsplit + split) * kRowTile;
        if (lg == 0) {
            ml[li] = make_float2(mx[0], zz[0]);
            ml[32 + li] = make_float2(mx[1], zz[1]);
        }
    }
}

// One workgroup per unit: merges the splits' partial outputs, writes the output tile, reduces the
// per-segment (max, sum) pairs over the tile's rows; the last unit of a query to finish adds the
// units' masses in a fixed order.
template <int DT>
__global__ __launch_bounds__(kThreads) void attn_combine_kernel(AttnArgs a, Plan p) {
    __shared__ SegTable tbl;
    __shared__ float wgt[64][kRowTile];          // per split: exp2(m_split - M) / Z
    __shared__ float row_m[kRowTile], row_iz[kRowTile];
    __shared__ __attribute__((aligned(16))) uint16_t otile[kRowTile][kD + 8];
    __shared__ int is_last;

    const int unit = blockIdx.x;
    const int rowtile = unit % p.rowtiles;
    const int hkv = (unit / p.rowtiles) % a.n_kv_heads;
    const int b = unit / p.units_per_b;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int hq = a.n_q_heads, group = hq / a.n_kv_heads;
    const int q0 = a.q_off[b];
    const int tq = min(a.q_off[b + 1] - q0, a.max_tq);
    const int n_rows = group * tq;

    build_table(a, b, &tbl);

    const float2* ml = reinterpret_cast<const float2*>(static_cast<const char*>(a.workspace) + p.off_ml) +
                       (int64_t)unit * p.nsplit * kRowTile;
    if (threadIdx.x < kRowTile) {
        const int row = threadIdx.x;
        float m = -INFINITY;
        for (int s = 0; s < p.nsplit; ++s) m = fmaxf(m, ml[s * kRowTile + row].x);
        const float ms = m == -INFINITY ? 0.f : m;
        float z = 0.f;
        for (int s = 0; s < p.nsplit; ++s) z += ml[s * kRowTile + row].y * exp2f(ml[s * kRowTile + row].x - ms);
        const float iz = z > 0.f ? 1.f / z : 0.f;
        for (int s = 0; s < p.nsplit; ++s) wgt[s][row] = exp2f(ml[s * kRowTile + row].x - ms) * iz;
        row_m[row] = ms;
        row_iz[row] = iz;
    }
    __syncthreads();

    // ---- output tile: element (reg, lane) of a partial is O^T[dv][row] of the MFMA layout
    const float* opart = reinterpret_cast<const float*>(static_cast<const char*>(a.workspace) + p.off_opart) +
                         (int64_t)unit * p.nsplit * kORegs * kWave;
    for (int idx = threadIdx.x; idx < kORegs * kWave; idx += kThreads) {
        const int reg = idx >> 6, ln = idx & 63;
        const int db = reg >> 5, rb = (reg >> 4) & 1, r = reg & 15;
        const int row = rb * 32 + (ln & 31);
        const int dv = 32 * db + 8 * (r >> 2) + 4 * (ln >> 5) + (r & 3);
        float v = 0.f;
        for (int s = 0; s < p.nsplit; ++s) v += wgt[s][row] * opart[(int64_t)s * kORegs * kWave + idx];
        otile[row][dv] = (uint16_t)Mma<DT>::from_f(v);
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < kRowTile * (kD / 8); idx += kThreads) {
        const int row = idx / (kD / 8), c = idx % (kD / 8);
        const int m = rowtile * kRowTile + row;
        if (m < n_rows) {
            const int gi = m / tq, t = m - gi * tq;
            uint16_t* op = static_cast<uint16_t*>(a.out) + (((int64_t)q0 + t) * hq + hkv * group + gi) * kD + 8 * c;
            *reinterpret_cast<uint4*>(op) = *reinterpret_cast<const uint4*>(&otile[row][8 * c]);
        }
    }

    // ---- per-segment mass of this unit: wavefront w owns segments s = w, w+4, ...; lane = row
    const float2* massml = reinterpret_cast<const float2*>(static_cast<const char*>(a.workspace) + p.off_massml) +
                           (int64_t)unit * p.slots * kRowTile;
    float* massunit = reinterpret_cast<float*>(static_cast<char*>(a.workspace) + p.off_massunit);
    const int total = tbl.blk0[tbl.n];
    const int row_valid = (rowtile * kRowTile + lane) < n_rows;
    for (int s = wave; s < tbl.n; s += kWaves) {
        const int bs = tbl.blk0[s], be = tbl.blk0[s + 1];
        float accm = 0.f;
        if (be > bs) {
            for (int ss = 0; ss < p.nsub; ++ss) {
                int lo, hi;
                sub_range(total, p.nsplit, ss, &lo, &hi);
                if (lo < be && hi > bs && lo < hi) {
                    const float2 v = massml[(int64_t)(s + ss) * kRowTile + lane];
                    const float c = row_valid ? v.y * exp2f(v.x - row_m[lane]) * row_iz[lane] : 0.f;
                    accm += wave_sum(c);
                }
            }
        }
        if (lane == 0) massunit[((int64_t)b * p.units_per_b + (unit % p.units_per_b)) * a.seg_stride + s] = accm;
    }

    // ---- last unit of query b sums the units in order
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t* counters = reinterpret_cast<int32_t*>(static_cast<char*>(a.workspace) + p.off_counters);
        is_last = atomicAdd(&counters[b], 1) == p.units_per_b - 1;
    }
    __syncthreads();
    if (is_last) {
        __threadfence();
        for (int s = threadIdx.x; s < tbl.n; s += kThreads) {
            float tot = 0.f;
            for (int u = 0; u < p.units_per_b; ++u)
                tot += __builtin_nontemporal_load(&massunit[((int64_t)b * p.units_per_b + u) * a.seg_stride + s]);
            a.mass[(int64_t)b * a.seg_stride + s] = tot;
            const int doc = a.segs[(int64_t)b * a.seg_stride + s].doc;
            if (a.score_accum && doc >= 0 && doc < a.score_stride)
                atomicAdd(&a.score_accum[(int64_t)b * a.score_stride + doc], tot);
        }
    }
}

}  // namespace

bool mfma_path_supported(const cf_layer_desc* d) {
    return (d->dtype == CF_BF16 || d->dtype == CF_F16) && d->head_dim == kD && d->rope_pairing == CF_ROPE_HALF;
}

static bool mfma_shape_ok(int seg_stride) { return seg_stride <= kMaxSegs; }

size_t mfma_workspace_bytes(const cf_layer_desc* d, int32_t batch, int32_t max_tq, int32_t seg_stride,
                            int64_t max_kv_tokens) {
    const size_t gen = generic_workspace_bytes(d, batch, max_tq, seg_stride);
    if (!mfma_shape_ok(seg_stride)) return gen;
    const Plan p = make_plan(d->n_q_heads, d->n_kv_heads, batch, max_tq, seg_stride, max_kv_tokens);
    return p.total;
}

cf_status launch_attention_mfma(const AttnArgs& a, const RopeFreq& f, hipStream_t s) {
    if (!mfma_shape_ok(a.seg_stride)) return launch_attention_generic(a, f, s);
    const Plan p = make_plan(a.n_q_heads, a.n_kv_heads, a.batch, a.max_tq, a.seg_stride, a.max_kv_tokens);
    const unsigned grid = (unsigned)(p.units * p.nsplit);
    if (a.dtype == CF_BF16) {
        hipLaunchKernelGGL((attn_mfma_kernel<CF_BF16>), dim3(grid), dim3(kThreads), 0, s, a, f, p);
        CF_HIP(hipGetLastError());
        hipLaunchKernelGGL((attn_combine_kernel<CF_BF16>), dim3(p.units), dim3(kThreads), 0, s, a, p);
    } else {
        hipLaunchKernelGGL((attn_mfma_kernel<CF_F16>), dim3(grid), dim3(kThreads), 0, s, a, f, p);
        CF_HIP(hipGetLastError());
        hipLaunchKernelGGL((attn_combine_kernel<CF_F16>), dim3(p.units), dim3(kThreads), 0, s, a, p);
    }
    CF_HIP(hipGetLastError());
    return CF_OK;
}

}  // namespace cf
