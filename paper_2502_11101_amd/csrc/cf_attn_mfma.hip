// 16-bit MFMA prefill attention for gfx950 (head_dim 128, half-split RoPE pairing).
//
// Work decomposition.  The query rows that share a kv head (all rows of the G = Hq/Hkv heads of
// the group, stacked: row m = g*tq + t) are cut into 16-row blocks; a workgroup owns a run of such blocks of one
// (query, kv head) and a contiguous run of the attended tokens.  Tokens are counted in tiles that never
// straddle a segment; the tile list of a (query, kv head) is divided evenly over `nsplit` workgroups.
//   * At most 4 row blocks (MHA, short queries: HBM- and latency-bound): attn_tile_kernel, 32-token tiles,
//     one row block per wavefront, every wavefront loads, stages and computes; two groups of four wavefronts
//     per workgroup stream disjoint runs of tiles.
//   * More (GQA groups, long queries: MFMA-bound): attn_pc_kernel, 64-token tiles, two wavefronts load, rotate
//     and stage while six do the math of the previous tile, two row blocks each (up to 192 rows per workgroup).
// Per tile, in both:
//   * the tile two ahead is in flight in registers (coalesced 16-byte loads),
//   * the key tile is rotated in registers by its segment's relative position shift (Eq. 5;
//     cos/sin per 2-D slice from an fp64-reduced angle), rounded once to the storage type and
//     staged into LDS — rotated keys never return to memory; V is staged as loaded,
//   * S^T = K Q^T and O^T += V^T P^T run on v_mfma_f32_16x16x32 with the Q fragments resident
//     in registers and the V^T fragments read with transposing LDS reads; the transposed forms keep
//     one query row per lane, so the online softmax (fp32, exp2 domain) needs no cross-lane exchange
//     except when its reference maximum moves.
// At the end of each segment a wavefront leaves (reference maximum, sum of exp2) per row.
//
// A second kernel merges the splits' partial outputs and writes the output rows; a third reduces
// the (max, sum) pairs to per-segment attention mass (the document-wise score of Alg. 2) in a
// fixed order and adds it to the accumulated scores.  Results cross between the kernels at the
// kernel boundaries: no fences, no atomics on the data path, bit-identical reruns.
#include <type_traits>

#include <hip/hip_ext.h>

#include "cf_attn_tile.h"

namespace cf {
using namespace attn;
namespace {

// ---------------------------------------------------------------------------------------------
// The attention kernel for few stacked rows: the four wavefronts of a group stream the same TILE-token
// tiles and own different query rows (wavefront w the 16-row blocks [w*NRB, (w+1)*NRB)), so there is
// nothing to merge inside a group.  Per tile:
//   * every thread's K/V loads for the tile two ahead are in flight in registers (a fixed number of
//     loads per step, so the wait for one tile never covers a later one);
//   * staging: a thread rotates the pairs (c, c + 64) of its 16-byte key chunks (Eq. 5) and writes
//     them [token][channel] to one of two LDS tile buffers; V chunks are copied as loaded, row-major
//     with a 32-byte XOR swizzle; one workgroup barrier per tile;
//   * the tile's math (tile_math).
// With GROUPS == 2 two such groups share a workgroup, stream disjoint runs of tiles and merge at the end.
template <int DT, int NRB, int TILE, int GROUPS, bool REG_TABLE>
__global__ __launch_bounds__(kThreads * GROUPS, 2) void attn_tile_kernel(AttnArgs a, RopeFreq freq, Plan p) {
    static_assert(GROUPS == 1 || (GROUPS == 2 && NRB == 1), "two groups: one row block per wavefront");
    constexpr int kKTile = TILE * kKRow;             // bytes
    constexpr int kVTile = TILE * kD * 2;
    constexpr int kKItems = TILE / 32;               // (row, chunk pair) items per thread
    constexpr int kVItems = TILE / 16;               // (row, chunk) items per thread
    __shared__ SegTable tbl;
    __shared__ __attribute__((aligned(16))) unsigned char k_buf[GROUPS][2][kKTile];
    __shared__ __attribute__((aligned(16))) unsigned char v_buf[GROUPS][2][kVTile];
    __shared__ __attribute__((aligned(16))) float2 cs_lds[GROUPS][2][kHalf];

    const int tid = threadIdx.x & (kThreads - 1);    // thread, wavefront: inside the group of four wavefronts
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int grp = GROUPS == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x / kThreads);
    const int li = lane & 15, lg = lane >> 4;
    {
        const void *p0 = a.q, *p1 = a.q_off, *p2 = a.q_new_start, *p3 = a.k_store, *p4 = a.v_store, *p5 = a.k_self,
                   *p6 = a.v_self, *p7 = a.segs, *p8 = a.n_seg, *p9 = a.workspace;
        asm volatile("" ::"s"(p0), "s"(p1), "s"(p2), "s"(p3), "s"(p4), "s"(p5), "s"(p6), "s"(p7), "s"(p8), "s"(p9),
                     "s"(a.n_store_tokens), "s"(a.seg_stride), "s"(a.batch), "s"(a.max_tq), "s"(a.n_q_heads),
                     "s"(a.n_kv_heads), "s"(a.scale_log2e), "s"(a.q_stored_start), "s"(p.nsplit), "s"(p.slots),
                     "s"(p.off_ml), "s"(p.off_opart), "s"(p.off_massml));
    }

    // grid (split, kv head, query): nothing to divide; one row group (at most four row blocks)
    const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
    constexpr int rg = 0;
    const int unit = b * a.n_kv_heads + hkv;
    const int group = p.group;
    const QueryHead qh = load_query_head(a, b, REG_TABLE ? lane : (int)threadIdx.x);
    const double my_freq = freq.rev[tid & (kHalf - 1)];
    const int tq = min(qh.tq_raw, a.max_tq);

    // ---- Q fragments first (loads return in order)
    uint4 qf[NRB][4];
    int trow[NRB];
    const int row_base = rg * p.blocks_rg * 16;
    const int row_limit = min(group * tq, row_base + p.blocks_rg * 16);
    const bool has_rows = row_base + wave * NRB * 16 < row_limit;        // wavefront-uniform
    load_q_fragments<NRB>(a, qh.q0, tq, hkv, group, wave * NRB, row_base, row_limit, li, lg, qf, trow);

    // at most 64 table entries: every wavefront keeps the table in registers; more: one table in LDS
    RegSegTable rtbl;
    unsigned total;
    if constexpr (REG_TABLE) {
        rtbl = build_reg_table(a, qh, lane, TILE);
        total = (unsigned)rtbl.total;
    } else {
        build_table(a, qh, &tbl, TILE);
        total = (unsigned)tbl.tile0[tbl.n];
    }
    // a group streams a contiguous run of the workgroup's tiles of its own (sub-split `ss`)
    const unsigned nsub = (unsigned)(p.nsplit * GROUPS);
    const int ss = split * GROUPS + grp;

    // staging items: K (row kr + 32*it, chunks kj and kj + 8), V (row vr + 16*it, chunk vc)
    const int kr = tid >> 3, kj = tid & 7;
    const int vr = tid >> 4, vc = tid & 15;
    struct StageRegs { uint4 ka[kKItems], kb[kKItems], v[kVItems]; };
    StageRegs regs0, regs1;

    TileWalk<TILE> walk(split_begin(total, nsub, ss), split_begin(total, nsub, ss + 1));
    // Every call issues the same loads whether or not a tile is left, so the number of loads in flight
    // at any point of the loop is fixed.  Rows past the end of a ragged tile re-read its last row (in
    // bounds; their scores are masked).
    auto fetch = [&](Tile& d, StageRegs& r) {
        if constexpr (REG_TABLE) d = walk.next(rtbl, lane);
        else d = walk.next(tbl, lane);
        const TileSource src = tile_source(a, d, walk.c_tok, hkv);
#pragma unroll
        for (int it = 0; it < kKItems; ++it) {
            const uint32_t off = src.last < 0 ? 0u : (uint32_t)min(kr + 32 * it, src.last) * src.row_bytes + 16 * kj;
            r.ka[it] = *reinterpret_cast<const uint4*>(src.k + off);
            r.kb[it] = *reinterpret_cast<const uint4*>(src.k + off + (src.last < 0 ? 0 : 128));
        }
#pragma unroll
        for (int it = 0; it < kVItems; ++it) {
            const uint32_t off = src.last < 0 ? 0u : (uint32_t)min(vr + 16 * it, src.last) * src.row_bytes + 16 * vc;
            r.v[it] = *reinterpret_cast<const uint4*>(src.v + off);
        }
    };
    Tile d0, d1;
    fetch(d0, regs0);
    fetch(d1, regs1);
    // workgroup-uniform: the longest run among the groups (not needed before the loop, so worked out once the
    // first loads are out)
    int most_tiles = 0;
#pragma unroll
    for (int g = 0; g < GROUPS; ++g)
        most_tiles = max(most_tiles, split_begin(total, nsub, split * GROUPS + g + 1) - split_begin(total, nsub, split * GROUPS + g));

    RowState<NRB> st;
    st.clear();
    char* ws = static_cast<char*>(a.workspace);
    float2* massml = reinterpret_cast<float2*>(ws + p.off_massml) + (int64_t)unit * p.slots * p.rows_wg;

    // V staging offsets and the transposing reads: lane 16*lg + s addresses row 4*lg + s/4 (+16), 8 bytes at
    // channel 16*db + 4*(s&3)
    const uint32_t vw_off = (uint32_t)vr * 256 + 16 * (vc ^ (2 * (vr & 7)));    // rows vr + 16*it keep (t & 7)
    const int tr_row = 4 * lg + (li >> 2);
    const uint32_t tr_base = (uint32_t)tr_row * 256 + 8 * (li & 3);
    const uint32_t tr_x = (uint32_t)(tr_row & 7) * 32;

    int cs_slot = 0;
    int cur_seg = -1;
    if (d0.ntok > 0 && d0.delta != 0 && tid < kHalf) cs_lds[grp][0][tid] = rope_cos_sin_fast(d0.delta, my_freq);
    __syncthreads();

    // Stage tile `cur` from its registers into buffer `buf`, refill the registers with the tile after
    // `nxt`, prepare the cos/sin table of `nxt`; after the barrier, the math of `cur`.
    auto step = [&](Tile& cur, StageRegs& r, const Tile& nxt, int buf) {
        const Tile cd = cur;
        const bool live = cd.ntok > 0;
        unsigned char* k_lds = k_buf[grp][buf];
        unsigned char* v_lds = v_buf[grp][buf];
        if (live) {
            ChunkAngles ang;
            if (cd.delta != 0) ang = load_chunk_angles(cs_lds[grp][cs_slot] + 8 * kj);
#pragma unroll
            for (int it = 0; it < kKItems; ++it) {
                uint4 ra = r.ka[it], rb4 = r.kb[it];
                if (cd.delta != 0) rotate_chunk_pair<DT>(ra, rb4, ang);
                k_tile_write(k_lds, kr + 32 * it, kj, ra);
                k_tile_write(k_lds, kr + 32 * it, kj + 8, rb4);
            }
#pragma unroll
            for (int it = 0; it < kVItems; ++it) *reinterpret_cast<uint4*>(v_lds + it * 16 * 256 + vw_off) = r.v[it];
        }
        fetch(cur, r);                               // the registers are free again
        if (nxt.ntok > 0 && nxt.seg != cd.seg && nxt.delta != 0) {
            cs_slot ^= 1;
            if (tid < kHalf) cs_lds[grp][cs_slot][tid] = rope_cos_sin_fast(nxt.delta, my_freq);
        }
        __syncthreads();            // tile `cur` is staged; every wavefront is done with the other buffer
        if (!live || !has_rows) return;
        if (cd.seg != cur_seg) {
            if (cur_seg >= 0) emit_segment<NRB>(st, massml, cur_seg + ss, p.rows_wg, wave * NRB, li, lg);
            cur_seg = cd.seg;
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) st.seg_l[rb] = 0.f;
        }
        tile_math<DT, NRB, TILE>(cd, k_lds, v_lds, qf, trow, st, a.scale_log2e, li, lg, tr_base, tr_x);
    };
    // Steps come in pairs and the trip count is the workgroup's: every path round the loop issues the
    // same loads and meets the same barriers.  A group with fewer tiles runs steps without one.
    for (int it = 0; it < most_tiles; it += 2) {
        step(d0, regs0, d1, 0);
        step(d1, regs1, d0, 1);
    }
    if (cur_seg >= 0) emit_segment<NRB>(st, massml, cur_seg + ss, p.rows_wg, wave * NRB, li, lg);

    float l_row[NRB];                                // row sums (each lane holds those of its own tokens so far)
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        l_row[rb] = st.l_run[rb] + __shfl_xor(st.l_run[rb], 16);
        l_row[rb] += __shfl_xor(l_row[rb], 32);
    }
    if (GROUPS == 2) {
        // the second group hands its rows' results (same rows, other tokens) to the first through the tile
        // buffers, which nobody reads any more
        f32x4* red = reinterpret_cast<f32x4*>(&k_buf[0][0][0]);                    // 4 wavefronts x 8 x 64 lanes
        float2* red_ml = reinterpret_cast<float2*>(&v_buf[0][0][0]);               // 4 wavefronts x 16 rows
        __syncthreads();
        if (grp == 1) {
#pragma unroll
            for (int db = 0; db < 8; ++db) red[(wave * 8 + db) * kWave + lane] = st.acc[0][db];
            if (lg == 0) red_ml[wave * 16 + li] = make_float2(st.m_run[0], l_row[0]);
        }
        __syncthreads();
        if (grp == 1) return;
        const float2 o = red_ml[wave * 16 + li];
        const float m = fmaxf(st.m_run[0], o.x);
        const float ms = m == -INFINITY ? 0.f : m;
        const float f0 = __builtin_amdgcn_exp2f(st.m_run[0] - ms), f1 = __builtin_amdgcn_exp2f(o.x - ms);
#pragma unroll
        for (int db = 0; db < 8; ++db) st.acc[0][db] = st.acc[0][db] * f0 + red[(wave * 8 + db) * kWave + lane] * f1;
        l_row[0] = l_row[0] * f0 + o.y * f1;
        st.m_run[0] = m;
    }
    // a wavefront whose rows are all padding leaves nothing
    if (!has_rows) return;
    store_partials<DT, NRB>(a, p, unit, split, wave * NRB, st, l_row, lane, qh.q0, tq, hkv, group, row_base, row_limit);
}

// ---------------------------------------------------------------------------------------------
// The attention kernel for many stacked rows (GQA groups, long queries), where staging a tile costs
// as much issue time as its math: eight wavefronts, of which the first kProducers only load, rotate
// (Eq. 5) and stage tiles, and the others only do the math, two 16-row blocks each — so the rotation
// and the LDS writes of tile j + 1 run beside the MFMAs and the softmax of tile j instead of before
// them, and one staged tile serves 32*(8 - kProducers) rows.  One workgroup barrier per tile:
//   producers:  B0; for j: { stage tile j into buffer j & 1; B }
//   the others: B0; for j: { B; math of tile j }
// so tile j is staged before the barrier that its math follows, and its buffer is written again (tile
// j + 2) only after the next barrier, which the math of tile j precedes.  Only the producers walk the segment
// table; the others take each tile's description from a small ring in LDS.
constexpr int kPcTile = 64;

template <int DT, int kProducers, bool REG_TABLE>
__global__ __launch_bounds__(kPcWaves * kWave, 2) void attn_pc_kernel(AttnArgs a, RopeFreq freq, Plan p) {
    constexpr int TILE = kPcTile, NRB = kPcNrb;
    constexpr int kPT = kProducers * kWave;          // producer threads
    constexpr int kKTile = TILE * kKRow, kVTile = TILE * kD * 2;
    constexpr int kKItems = TILE * 8 / kPT;          // (row, chunk pair) items per producer thread
    constexpr int kVItems = TILE * 16 / kPT;         // (row, chunk) items per producer thread
    __shared__ SegTable tbl;
    __shared__ __attribute__((aligned(16))) unsigned char k_buf[2][kKTile];
    __shared__ __attribute__((aligned(16))) unsigned char v_buf[2][kVTile];
    __shared__ __attribute__((aligned(16))) float2 cs_lds[2][kHalf];
    // (segment, first token, tokens, own block) of tile j in entry j & 3, written by the producers when they
    // fetch the tile, two steps before its math: the math wavefronts do not walk the table themselves
    __shared__ int4 tile_ring[4];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int li = lane & 15, lg = lane >> 4;

    // (plain scalar divisions here: this kernel has no registers to spare for the vector form)
    const int bid = blockIdx.x;
    const int rg = bid / p.x_count;
    const int x = bid - rg * p.x_count;
    const int split = x % p.nsplit;
    const int hkv = (x / p.nsplit) % a.n_kv_heads;
    const int b = __builtin_amdgcn_readfirstlane(x / (p.nsplit * a.n_kv_heads));
    const int unit = (b * a.n_kv_heads + hkv) * p.n_rg + rg;
    const int group = p.group;
    const QueryHead qh = load_query_head<false>(a, b, REG_TABLE ? lane : (int)threadIdx.x);
    const int tq = min(qh.tq_raw, a.max_tq);
    const int row_base = rg * p.blocks_rg * 16;
    const int row_limit = min(group * tq, row_base + p.blocks_rg * 16);
    const int cw = wave - kProducers;                // index among the wavefronts that do the math
    const bool has_rows = cw >= 0 && row_base + cw * NRB * 16 < row_limit;       // wavefront-uniform
    uint4 qf[NRB][4];
    int trow[NRB];
    if (cw >= 0) load_q_fragments<NRB>(a, qh.q0, tq, hkv, group, cw * NRB, row_base, row_limit, li, lg, qf, trow);
    RegSegTable rtbl;
    unsigned total;
    if constexpr (REG_TABLE) {
        rtbl = build_reg_table(a, qh, lane, TILE);
        total = (unsigned)rtbl.total;
    } else {
        build_table(a, qh, &tbl, TILE);
        total = (unsigned)tbl.tile0[tbl.n];
    }
    const int t_begin = split_begin(total, (unsigned)p.nsplit, split), t_end = split_begin(total, (unsigned)p.nsplit, split + 1);
    const int n_tiles = t_end - t_begin;

    if (wave < kProducers) {
        // ------------------------------------------------------------------ producers
        const double my_freq = freq.rev[tid & (kHalf - 1)];
        // staging items: K (row kr + (kPT/8)*it, chunks kj and kj + 8), V (row vr + (kPT/16)*it, chunk vc)
        const int kr = tid >> 3, kj = tid & 7;
        const int vr = tid >> 4, vc = tid & 15;
        struct StageRegs { uint4 ka[kKItems], kb[kKItems], v[kVItems]; };
        StageRegs regs0, regs1;
        TileWalk<TILE> walk(t_begin, t_end);
        int n_fetched = 0;
        auto fetch = [&](Tile& d, StageRegs& r) {    // a fixed number of loads, as in attn_tile_kernel
            if constexpr (REG_TABLE) d = walk.next(rtbl, lane);
            else d = walk.next(tbl, lane);
            if (tid == 0) tile_ring[n_fetched & 3] = make_int4(d.seg, d.tok0, d.ntok, d.self);
            ++n_fetched;
            const TileSource src = tile_source(a, d, walk.c_tok, hkv);
#pragma unroll
            for (int it = 0; it < kKItems; ++it) {
                const uint32_t off = src.last < 0 ? 0u : (uint32_t)min(kr + (kPT / 8) * it, src.last) * src.row_bytes + 16 * kj;
                r.ka[it] = *reinterpret_cast<const uint4*>(src.k + off);
                r.kb[it] = *reinterpret_cast<const uint4*>(src.k + off + (src.last < 0 ? 0 : 128));
            }
#pragma unroll
            for (int it = 0; it < kVItems; ++it) {
                const uint32_t off = src.last < 0 ? 0u : (uint32_t)min(vr + (kPT / 16) * it, src.last) * src.row_bytes + 16 * vc;
                r.v[it] = *reinterpret_cast<const uint4*>(src.v + off);
            }
        };
        Tile d0, d1;
        fetch(d0, regs0);
        fetch(d1, regs1);
        int cs_slot = 0;
        if (d0.ntok > 0 && d0.delta != 0 && tid < kHalf) cs_lds[0][tid] = rope_cos_sin_fast(d0.delta, my_freq);
        __syncthreads();                             // B0
        auto stage = [&](Tile& cur, StageRegs& r, const Tile& nxt, int buf) {
            const Tile cd = cur;
            unsigned char* k_lds = k_buf[buf];
            unsigned char* v_lds = v_buf[buf];
            if (cd.ntok > 0) {
                ChunkAngles ang;
                if (cd.delta != 0) ang = load_chunk_angles(cs_lds[cs_slot] + 8 * kj);
#pragma unroll
                for (int it = 0; it < kKItems; ++it) {
                    uint4 ra = r.ka[it], rb4 = r.kb[it];
                    if (cd.delta != 0) rotate_chunk_pair<DT>(ra, rb4, ang);
                    k_tile_write(k_lds, kr + (kPT / 8) * it, kj, ra);
                    k_tile_write(k_lds, kr + (kPT / 8) * it, kj + 8, rb4);
                }
#pragma unroll
                for (int it = 0; it < kVItems; ++it) {
                    const int t = vr + (kPT / 16) * it;
                    *reinterpret_cast<uint4*>(v_lds + t * 256 + 16 * (vc ^ (2 * (t & 7)))) = r.v[it];
                }
            }
            fetch(cur, r);
            if (nxt.ntok > 0 && nxt.seg != cd.seg && nxt.delta != 0) {
                cs_slot ^= 1;
                if (tid < kHalf) cs_lds[cs_slot][tid] = rope_cos_sin_fast(nxt.delta, my_freq);
            }
            __syncthreads();
        };
        for (int it = 0; it < n_tiles; it += 2) {
            stage(d0, regs0, d1, 0);
            stage(d1, regs1, d0, 1);
        }
        return;
    }

    // ---------------------------------------------------------------------- the others: math
    RowState<NRB> st;
    st.clear();
    float2* massml = reinterpret_cast<float2*>(static_cast<char*>(a.workspace) + p.off_massml) + (int64_t)unit * p.slots * p.rows_wg;
    const int tr_row = 4 * lg + (li >> 2);
    const uint32_t tr_base = (uint32_t)tr_row * 256 + 8 * (li & 3);
    const uint32_t tr_x = (uint32_t)(tr_row & 7) * 32;
    int cur_seg = -1;
    __syncthreads();                                 // B0
    // the tile to do next, in scalars; its successor's ring entry is read while the tile's math runs
    auto ring_tile = [&](int j) {
        const int4 e = tile_ring[j & 3];
        Tile t;
        t.seg = __builtin_amdgcn_readfirstlane(e.x);
        t.tok0 = __builtin_amdgcn_readfirstlane(e.y);
        t.ntok = __builtin_amdgcn_readfirstlane(e.z);
        t.self = __builtin_amdgcn_readfirstlane(e.w);
        t.delta = 0;                                 // the staged keys are rotated already
        return t;
    };
    Tile upcoming = ring_tile(0);
    int n_done = 0;
    auto math = [&](int buf) {
        __syncthreads();                             // the tile is staged
        const Tile cd = upcoming;
        const int4 next_entry = tile_ring[(n_done + 1) & 3];     // written before the barrier just passed
        ++n_done;
        auto take_next = [&]() {
            upcoming.seg = __builtin_amdgcn_readfirstlane(next_entry.x);
            upcoming.tok0 = __builtin_amdgcn_readfirstlane(next_entry.y);
            upcoming.ntok = __builtin_amdgcn_readfirstlane(next_entry.z);
            upcoming.self = __builtin_amdgcn_readfirstlane(next_entry.w);
        };
        if (cd.ntok <= 0 || !has_rows) { take_next(); return; }
        if (cd.seg != cur_seg) {
            if (cur_seg >= 0) emit_segment<NRB>(st, massml, cur_seg + split, p.rows_wg, cw * NRB, li, lg);
            cur_seg = cd.seg;
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) st.seg_l[rb] = 0.f;
        }
        tile_math<DT, NRB, TILE>(cd, k_buf[buf], v_buf[buf], qf, trow, st, a.scale_log2e, li, lg, tr_base, tr_x);
        take_next();
    };
    for (int it = 0; it < n_tiles; it += 2) {
        math(0);
        math(1);
    }
    if (!has_rows) return;
    if (cur_seg >= 0) emit_segment<NRB>(st, massml, cur_seg + split, p.rows_wg, cw * NRB, li, lg);
    float l_row[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        l_row[rb] = st.l_run[rb] + __shfl_xor(st.l_run[rb], 16);
        l_row[rb] += __shfl_xor(l_row[rb], 32);
    }
    store_partials<DT, NRB>(a, p, unit, split, cw * NRB, st, l_row, lane, qh.q0, tq, hkv, group, row_base, row_limit);
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

cf_status launch_attention_mfma(const AttnArgs& a, const RopeFreq& f, hipStream_t s, const cf_prune_step* prune) {
    if (!mfma_shape_ok(a.seg_stride)) {
        cf_status st = launch_attention_generic(a, f, s);
        return st != CF_OK || !prune ? st : launch_prune_step(a, prune, s);
    }
    const Plan p = make_plan(a.n_q_heads, a.n_kv_heads, a.batch, a.max_tq, a.seg_stride, a.max_kv_tokens);
    const dim3 grid((unsigned)(p.x_count * p.n_rg));
    const dim3 grid3((unsigned)p.nsplit, (unsigned)a.n_kv_heads, (unsigned)a.batch);     // attn_tile_kernel's
    if (a.batch > 65535 || (int64_t)a.n_kv_heads * p.n_rg > 65535) {          // grid dimensions of this path's kernels
        set_error("batch and n_kv_heads * row groups must not exceed 65535 on this path");
        return CF_ERR_UNSUPPORTED;
    }
    const bool reg_table = a.seg_stride <= kWave;    // the attention kernels keep a table this small in registers
    // the attention kernel's launch carries the profiling aid's start/stop events (null when it is off)
    hipEvent_t ev_start = nullptr, ev_stop = nullptr;
    profile_kernel_pair(&ev_start, &ev_stop);
#define CF_LAUNCH_TIMED(KERNEL, GRID, BLOCK) hipExtLaunchKernelGGL(KERNEL, GRID, BLOCK, 0, s, ev_start, ev_stop, 0, a, f, p)
#define CF_LAUNCH_DT(DT)                                                                                                       \
    if (p.producers == 0) {                                                                                                    \
        if (reg_table) CF_LAUNCH_TIMED((attn_tile_kernel<DT, 1, 32, 2, true>), grid3, dim3(2 * kThreads));                            \
        else CF_LAUNCH_TIMED((attn_tile_kernel<DT, 1, 32, 2, false>), grid3, dim3(2 * kThreads));                                     \
    } else {                                                                                                                   \
        if (reg_table) CF_LAUNCH_TIMED((attn_pc_kernel<DT, kPcProducers, true>), grid, dim3(kPcWaves * kWave));                      \
        else CF_LAUNCH_TIMED((attn_pc_kernel<DT, kPcProducers, false>), grid, dim3(kPcWaves * kWave));                               \
    }                                                                                                                          \
    CF_HIP(hipGetLastError());
    if (a.dtype == CF_BF16) { CF_LAUNCH_DT(CF_BF16) } else { CF_LAUNCH_DT(CF_F16) }
#undef CF_LAUNCH_DT
#undef CF_LAUNCH_TIMED
    if (!(p.direct_out && a.mass == nullptr)) launch_combine(a, p, s);    // else nothing left to merge or reduce
    CF_HIP(hipGetLastError());
    if (prune) {
        if (epilogue_fits(p, prune)) {
            launch_epilogue(a, p, prune, s);
        } else {
            launch_mass(a, p, s);
            CF_HIP(hipGetLastError());
            return launch_prune_step(a, prune, s);
        }
    } else if (a.mass != nullptr) {
        launch_mass(a, p, s);
    }
    CF_HIP(hipGetLastError());
    return CF_OK;
}

}  // namespace cf
