// Device helpers of the 16-bit attention kernels: where a tile comes from, the rotation of a key chunk pair
// (Eq. 5), the staged K tile, a wavefront's running softmax state, the math of one staged tile, and what a
// wavefront leaves behind for the kernels that merge the splits.
#pragma once

#include "cf_attn_plan.h"

namespace cf {
namespace attn {

// The softmax reference of a row is a stale maximum: it only moves when the eight probabilities a lane
// has just formed against it add up to more than this (so none of them is larger), which is rare after a
// row's first tiles; the common path has no maximum and no cross-lane exchange.
constexpr float kProbLimit = 256.f;

typedef short short4v __attribute__((ext_vector_type(4)));

// cos/sin of delta*theta from the hardware sine/cosine (argument in revolutions, reduced in fp64):
// their absolute error is far below the rounding step of the 16-bit keys this feeds.
__device__ __forceinline__ float2 rope_cos_sin_fast(int delta, double theta_rev) {
    const double x = (double)delta * theta_rev;
    const float fr = (float)(x - rint(x));
    return make_float2(__builtin_amdgcn_cosf(fr), __builtin_amdgcn_sinf(fr));
}

// Where a tile's keys and values start for kv head `hkv`, and the distance between its tokens.
// Without a tile: the first bytes of the workspace, so that a fetch always has something to read.
struct TileSource { const char *k, *v; uint32_t row_bytes; int last; };

__device__ __forceinline__ TileSource tile_source(const AttnArgs& a, const Tile& d, int64_t seg_tok, int hkv) {
    TileSource t;
    t.k = t.v = static_cast<const char*>(a.workspace);
    t.row_bytes = 0;
    t.last = -1;
    if (d.ntok > 0) {
        // the own block is always token-major; the store has its own strides
        const int64_t tok_stride = d.self ? (int64_t)a.n_kv_heads * kD : a.store_ts;
        const int64_t base = ((seg_tok + d.tok0) * tok_stride + (int64_t)hkv * (d.self ? kD : a.store_hs)) * 2;
        t.k = static_cast<const char*>(d.self ? a.k_self : a.k_store) + base;
        t.v = static_cast<const char*>(d.self ? a.v_self : a.v_store) + base;
        t.row_bytes = (uint32_t)tok_stride * 2;
        t.last = d.ntok - 1;
    }
    return t;
}

// The (cos, sin) pairs of a thread's eight 2-D slices (chunk kj: slices 8*kj .. 8*kj + 7), two pairs per
// float4, read from the segment's LDS table once per tile.
struct ChunkAngles { float4 cs[4]; };
__device__ __forceinline__ ChunkAngles load_chunk_angles(const float2* cs8) {
    ChunkAngles c;
    const float4* p = reinterpret_cast<const float4*>(cs8);
#pragma unroll
    for (int i = 0; i < 4; ++i) c.cs[i] = p[i];
    return c;
}

// Rotates the pair of 16-byte key chunks (channels c..c+7 and c+64..c+71) by the chunk's angles (Eq. 5),
// in fp32, and rounds once to the storage type.
template <int DT>
__device__ __forceinline__ void rotate_chunk_pair(uint4& ra, uint4& rb4, const ChunkAngles& ang) {
    uint32_t wa[4] = {ra.x, ra.y, ra.z, ra.w}, wb[4] = {rb4.x, rb4.y, rb4.z, rb4.w};
    const float4 (&cs)[4] = ang.cs;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float4 w = cs[i];          // (cos, sin) of slices 2i, 2i + 1 of the chunk
        const float a0 = Mma<DT>::lo(wa[i]), a1 = Mma<DT>::hi(wa[i]);
        const float b0 = Mma<DT>::lo(wb[i]), b1 = Mma<DT>::hi(wb[i]);
        wa[i] = Mma<DT>::pack(a0 * w.x - b0 * w.y, a1 * w.z - b1 * w.w);
        wb[i] = Mma<DT>::pack(a0 * w.y + b0 * w.x, a1 * w.w + b1 * w.z);
    }
    ra = make_uint4(wa[0], wa[1], wa[2], wa[3]);
    rb4 = make_uint4(wb[0], wb[1], wb[2], wb[3]);
}

// Staged K tile: [token][kKRow bytes], 128 channels and 16 bytes of padding per token, so that the
// fragment reads of the 16 lanes that share a channel group fall into different banks.  (Measured on this part: a
// 16-byte LDS read runs at half the byte rate of an 8-byte one, but splitting the fragment into two 8-byte reads,
// in either a two-plane or an in-row layout, made the kernels slower, not faster.)
__device__ __forceinline__ void k_tile_write(unsigned char* k_lds, int t, int j, uint4 v) {
    *reinterpret_cast<uint4*>(k_lds + t * kKRow + 16 * j) = v;
}
// the MFMA operand of a lane for token t, channels 8*slot .. 8*slot + 7
__device__ __forceinline__ uint4 k_tile_fragment(const unsigned char* k_lds, int t, int slot) {
    return *reinterpret_cast<const uint4*>(k_lds + t * kKRow + 16 * slot);
}

// Running state of a wavefront's NRB 16-row blocks: lane (li, lg) holds, for query row li of each
// block, the output channels 16*db + 4*lg + r, the reference maximum, and the sums of exp2 over the
// tokens this lane has seen (whole call and current segment).
template <int NRB>
struct RowState {
    f32x4 acc[NRB][8];
    float m_run[NRB], l_run[NRB], seg_l[NRB];
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
            for (int db = 0; db < 8; ++db) acc[rb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
            m_run[rb] = -INFINITY; l_run[rb] = 0.f; seg_l[rb] = 0.f;
        }
    }
};

// The math of one staged tile for one wavefront: S^T = K Q^T from LDS key fragments and the register-resident
// Q fragments, online softmax against a stale maximum, O^T += V^T P^T with V^T fragments from
// transposing LDS reads.  K tile: see k_tile_write; V tile: row-major [token][256 bytes], chunk c of
// row t at chunk c ^ 2*(t & 7).  `trow`: query position of the lane's row inside the own block
// (causal mask), `tr_base`/`tr_x`: the lane's transposing-read offsets.
template <int DT, int NRB, int TILE>
__device__ __forceinline__ void tile_math(const Tile& cd, const unsigned char* k_lds, const unsigned char* v_lds,
                                          const uint4 (&qf)[NRB][4], const int (&trow)[NRB], RowState<NRB>& st,
                                          float scale_log2e, int li, int lg, uint32_t tr_base, uint32_t tr_x) {
    const bool causal = cd.self != 0;
    // ---- S^T = K Q^T of 32-token half h2: lane (li, lg) gets, for query row li, tokens 32*h2 + 16*tb + 4*lg + r
    auto scores = [&](int h2, f32x4 (&sc)[NRB][2]) {
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) { sc[rb][0] = f32x4{0.f, 0.f, 0.f, 0.f}; sc[rb][1] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        uint4 kf[2][4];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                kf[tb][kk] = k_tile_fragment(k_lds, 32 * h2 + 16 * tb + li, 4 * kk + lg);
        __builtin_amdgcn_sched_barrier(0);       // all eight reads are out before the first MFMA waits
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb) sc[rb][tb] = Mma<DT>::run(kf[tb][kk], qf[rb][kk], sc[rb][tb]);
    };
    // ---- softmax of half h2 and O^T += V^T P^T
    auto weigh = [&](int h2, f32x4 (&sc)[NRB][2]) {
        const int nt = cd.ntok - 32 * h2;      // valid tokens of this half
        // V^T fragments, requested before the softmax arithmetic that hides their latency
        short4v vlo[8], vhi[8];
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const unsigned char* src = v_lds + h2 * 32 * 256 + tr_base + ((uint32_t)(32 * db) ^ tr_x);
            vlo[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(src));
            vhi[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(src + 16 * 256));
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- online softmax (exp2 domain), fp32, against a stale row maximum (see kProbLimit)
        const bool need_mask = causal || nt < 32;
        uint4 pfrag[NRB];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            float xv[8];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int e = 0; e < 4; ++e) xv[4 * tb + e] = sc[rb][tb][e];
            if (need_mask) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int tk = 16 * (e >> 2) + 4 * lg + (e & 3);
                    const bool ok = tk < nt && (!causal || cd.tok0 + 32 * h2 + tk <= trow[rb]);
                    xv[e] = ok ? xv[e] : -INFINITY;
                }
            }
            // Probabilities against the reference as it stands; their sum tells whether one of them left the
            // range the reference allows (or no reference exists yet) — only then is the maximum worked out,
            // the reference moved, everything accumulated so far rescaled, and the probabilities redone.
            float pv[8];
            float lsum = 0.f;
            auto probabilities = [&](float m_ref) {
                const float m_safe = m_ref == -INFINITY ? 0.f : m_ref;
                lsum = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    pv[e] = __builtin_amdgcn_exp2f(fmaf(xv[e], scale_log2e, -m_safe));
                    lsum += pv[e];
                }
            };
            probabilities(st.m_run[rb]);
            if (__any(!(lsum <= kProbLimit) || st.m_run[rb] == -INFINITY)) {
                float mloc = fmaxf(fmaxf(fmaxf(xv[0], xv[1]), fmaxf(xv[2], xv[3])), fmaxf(fmaxf(xv[4], xv[5]), fmaxf(xv[6], xv[7])));
                mloc *= scale_log2e;                     // scale > 0: max commutes with it
                mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
                mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
                const float m_old = st.m_run[rb];
                const float m_new = fmaxf(m_old, mloc);
                const float alpha = __builtin_amdgcn_exp2f(m_old - (m_new == -INFINITY ? 0.f : m_new));
                st.l_run[rb] *= alpha;
                st.seg_l[rb] *= alpha;
                st.m_run[rb] = m_new;
                if (__any(alpha != 1.f && m_old != -INFINITY)) {     // nothing accumulated yet: nothing to rescale
#pragma unroll
                    for (int db = 0; db < 8; ++db) st.acc[rb][db] *= alpha;
                }
                probabilities(m_new);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) xv[e] = pv[e];
            st.l_run[rb] += lsum;
            st.seg_l[rb] += lsum;
            pfrag[rb] = make_uint4(Mma<DT>::pack(xv[0], xv[1]), Mma<DT>::pack(xv[2], xv[3]),
                                   Mma<DT>::pack(xv[4], xv[5]), Mma<DT>::pack(xv[6], xv[7]));
        }
        // ---- O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const uint2 l2 = __builtin_bit_cast(uint2, vlo[db]), h2v = __builtin_bit_cast(uint2, vhi[db]);
            const uint4 va = make_uint4(l2.x, l2.y, h2v.x, h2v.y);
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) st.acc[rb][db] = Mma<DT>::run(va, pfrag[rb], st.acc[rb][db]);
        }
    };
    // The scores of the second half are requested before the first half is weighed: their MFMAs run
    // beside the first half's softmax arithmetic.  A ragged tile of at most 32 tokens has no second half.
    f32x4 sc0[NRB][2];
    scores(0, sc0);
    if (TILE == 64) {
        f32x4 sc1[NRB][2];
        const bool two = cd.ntok > 32;
        if (two) scores(1, sc1);
        weigh(0, sc0);
        if (two) weigh(1, sc1);
    } else {
        weigh(0, sc0);
    }
}

// Q fragments of a wavefront's row blocks [first_blk, first_blk + NRB) of the stacked rows of kv head
// `hkv`: row m = g*tq + t is q[q0 + t][hkv*group + g].  Rows at or past `row_limit` are padding (zero
// fragments, nothing to mask, results unused).
template <int NRB>
__device__ __forceinline__ void load_q_fragments(const AttnArgs& a, int q0, int tq, int hkv, int group, int first_blk,
                                                 int row_base, int row_limit, int li, int lg, uint4 (&qf)[NRB][4],
                                                 int (&trow)[NRB]) {
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int m = row_base + (first_blk + rb) * 16 + li;
        const bool valid = m < row_limit;
        const int gi = valid ? (int)div_exact((unsigned)m, (unsigned)tq) : 0;
        const int t = valid ? m - gi * tq : 0;
        trow[rb] = valid ? t : 0x7fffffff;
        const uint16_t* qp = static_cast<const uint16_t*>(a.q) + (((int64_t)q0 + t) * a.n_q_heads + hkv * group + gi) * kD + 8 * lg;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            qf[rb][kk] = valid ? *reinterpret_cast<const uint4*>(qp + 32 * kk) : make_uint4(0, 0, 0, 0);
    }
}

// (running reference, segment sum) per row of the wavefront's row blocks for slot `slot`
template <int NRB>
__device__ __forceinline__ void emit_segment(const RowState<NRB>& st, float2* massml, int slot, int rows_wg, int first_blk,
                                             int li, int lg) {
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        float tot = st.seg_l[rb] + __shfl_xor(st.seg_l[rb], 16);
        tot += __shfl_xor(tot, 32);
        if (lg == 0) massml[(int64_t)slot * rows_wg + (first_blk + rb) * 16 + li] = make_float2(st.m_run[rb], tot);
    }
}

// Results of a split.  Several splits: partial O^T in MFMA layout (four 16-bit values per lane, row block and
// channel block, each row divided by the split's own row sum) for the merge kernel.  One split: nothing to merge, the rows are normalised and written to
// `out` here (row m = g*tq + t of the stacked rows is out[q0 + t][hkv*group + g]).  Either way (reference,
// row sum) per row, which the mass reduction needs.
template <int DT, int NRB>
__device__ __forceinline__ void store_partials(const AttnArgs& a, const Plan& p, int unit, int split, int first_blk,
                                               const RowState<NRB>& st, const float (&l_row)[NRB], int lane, int q0, int tq,
                                               int hkv, int group, int row_base, int row_limit) {
    char* ws = static_cast<char*>(a.workspace);
    float2* ml = reinterpret_cast<float2*>(ws + p.off_ml) + ((int64_t)unit * p.nsplit + split) * p.rows_wg;
    if (p.direct_out) {
        const int li = lane & 15, lg = lane >> 4;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            const int m = row_base + (first_blk + rb) * 16 + li;
            if (lg == 0) ml[(first_blk + rb) * 16 + li] = make_float2(st.m_run[rb], l_row[rb]);
            if (m >= row_limit) continue;
            const int gi = (int)div_exact((unsigned)m, (unsigned)tq), t = m - gi * tq;
            const float inv = l_row[rb] > 0.f ? 1.f / l_row[rb] : 0.f;
            uint16_t* op = static_cast<uint16_t*>(a.out) + (((int64_t)q0 + t) * a.n_q_heads + hkv * group + gi) * kD + 4 * lg;
#pragma unroll
            for (int db = 0; db < 8; ++db) {
                const f32x4 o = st.acc[rb][db] * inv;
                uint2 pk;
                pk.x = Mma<DT>::pack(o[0], o[1]);
                pk.y = Mma<DT>::pack(o[2], o[3]);
                *reinterpret_cast<uint2*>(op + 16 * db) = pk;
            }
        }
        return;
    }
    // the split's rows leave normalised by their own sums, in the tensors' 16-bit type: bounded by the values
    // themselves whatever the sums are, and half the bytes of the accumulators
    uint2* opart = reinterpret_cast<uint2*>(ws + p.off_opart) +
                   (((int64_t)unit * p.nsplit + split) * p.rows_wg / 16 + first_blk) * 8 * kWave + lane;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const float inv = l_row[rb] > 0.f ? 1.f / l_row[rb] : 0.f;
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const f32x4 o = st.acc[rb][db] * inv;
            opart[(rb * 8 + db) * kWave] = make_uint2(Mma<DT>::pack(o[0], o[1]), Mma<DT>::pack(o[2], o[3]));
        }
        if ((lane >> 4) == 0) ml[(first_blk + rb) * 16 + (lane & 15)] = make_float2(st.m_run[rb], l_row[rb]);
    }
}

}  // namespace attn
}  // namespace cf
