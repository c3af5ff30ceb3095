// 16-bit MFMA prefill attention for gfx950 (head_dim 128, half-split RoPE pairing).
//
// Work decomposition.  The query rows that share a kv head (all rows of the G = Hq/Hkv heads of
// the group, stacked: row m = g*tq + t) are cut into 16-row blocks; a workgroup owns a run of such blocks of one
// (query, kv head) and a contiguous run of the attended tokens.  Tokens are counted in tiles that never
// straddle a segment; the tile list of a (query, kv head) is divided evenly over `nsplit` workgroups.
//   * At most 4 row blocks (MHA, short queries: HBM- and latency-bound): attn_tile_kernel, 32-token tiles,
//     one row block per wavefront, every wavefront loads, stages and computes; two groups of four wavefronts
//     per workgroup stream disjoint runs of tiles.
//   * More (GQA groups, long queries: MFMA-bound): attn_pipe_kernel, 32-token units, two wavefronts load, rotate
//     and stage while six do the math, two row blocks each (up to 192 rows per workgroup), software-pipelined
//     over three units.
// Per tile, in both:
//   * the tiles two steps ahead are in flight in registers (coalesced 16-byte loads),
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
// The attention kernel for many stacked rows (GQA groups, long queries), where staging costs as much issue time as
// the math: eight wavefronts, of which the first two only load, rotate (Eq. 5) and stage, and six only do the math,
// two 16-row blocks each (up to 192 rows per workgroup) — so the rotation and the LDS writes run beside the MFMAs and
// the softmax instead of before them.  The unit of work is 32 tokens, and a math wavefront keeps three units in flight, so that its MFMAs and its softmax arithmetic — which depend on each other
// inside a unit — come from different units and run side by side:
//   iteration i:   S^T(i+1) = K(i+1) Q^T      16 MFMAs  \  interleaved in one basic block
//                  softmax of S^T(i) -> P(i)   VALU      |  (scheduling groups), no branch inside
//                  O^T += V^T(i-1) P^T(i-1)    16 MFMAs  /
//   with the K fragments of unit i+2 and the V^T fragments of unit i requested from LDS inside the block, for the
//   next iteration.  The softmax reference is the stale maximum of tile_math (kProbLimit); the rare iteration in which
//   a reference has to move is repaired after the block: maximum, rescale of everything accumulated (which by then
//   includes unit i-1), probabilities redone.
// Staging: units are staged in pairs into a ring of eight unit slots; one workgroup barrier per pair.  With the barrier
// of step s passed, pair s is staged; the math of units 2k and 2k+1 touches pairs k-1 and k (V) and k+1 (K) and runs
// after the barrier of step k+1, while the producers stage pair k+2 over pair k-2, which no one reads any more.
constexpr int kPipeUnit = 32;                        // tokens per unit
constexpr int kPipeSlots = 8;                        // unit slots in LDS: four pairs
constexpr int kPipeKUnit = kPipeUnit * kKRow;        // bytes
constexpr int kPipeVUnit = kPipeUnit * kD * 2;
constexpr int kPipeDesc = 16;                        // unit descriptors kept for the math wavefronts
constexpr int kPipeCs = 4;                           // cos/sin tables: the pair being staged and the next may use two each

template <int DT, bool REG_TABLE>
__global__ __launch_bounds__(kPcWaves * kWave, 2) void attn_pipe_kernel(AttnArgs a, RopeFreq freq, Plan p) {
    constexpr int NRB = kPcNrb;
    constexpr int kPT = kPcProducers * kWave;        // producer threads: 128
    constexpr int kKItems = kPipeUnit * 8 / kPT;     // (row, chunk pair) items per producer thread and unit: 2
    constexpr int kVItems = kPipeUnit * 16 / kPT;    // (row, chunk) items: 4
    __shared__ SegTable tbl;
    __shared__ __attribute__((aligned(16))) unsigned char k_ring[kPipeSlots][kPipeKUnit];
    __shared__ __attribute__((aligned(16))) unsigned char v_ring[kPipeSlots][kPipeVUnit];
    __shared__ __attribute__((aligned(16))) float2 cs_lds[kPipeCs][kHalf];
    __shared__ int4 desc_ring[kPipeDesc];            // (segment, first token, tokens, own block) of unit u in entry u & 15

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int li = lane & 15, lg = lane >> 4;

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
    const int cw = wave - kPcProducers;              // index among the wavefronts that do the math
    const bool has_rows = cw >= 0 && row_base + cw * NRB * 16 < row_limit;       // wavefront-uniform
    uint4 qf[NRB][4];
    int trow[NRB];
    if (cw >= 0) load_q_fragments<NRB>(a, qh.q0, tq, hkv, group, cw * NRB, row_base, row_limit, li, lg, qf, trow);
    RegSegTable rtbl;
    unsigned total;
    if constexpr (REG_TABLE) {
        rtbl = build_reg_table(a, qh, lane, kPipeUnit);
        total = (unsigned)rtbl.total;
    } else {
        build_table(a, qh, &tbl, kPipeUnit);
        total = (unsigned)tbl.tile0[tbl.n];
    }
    const int t_begin = split_begin(total, (unsigned)p.nsplit, split), t_end = split_begin(total, (unsigned)p.nsplit, split + 1);
    const int n_units = t_end - t_begin;
    const int n_pairs = (n_units + 1) >> 1;
    const int n_steps = (n_pairs + 2) & ~1;          // producer steps (pairs 0 .. n_pairs and, to make it even, one more)

    if (wave < kPcProducers) {
        // ------------------------------------------------------------------ producers
        const double my_freq = freq.rev[tid & (kHalf - 1)];
        // K items: row kr + 16*it, chunks kj and kj + 8.  The two rows that the sixteen lanes of one LDS write pass
        // cover lie eight apart: their 16-byte chunks then fall into disjoint halves of the banks (rows are 272 bytes).
        const int kr = ((tid >> 3) & 1) * 8 + (tid >> 4), kj = tid & 7;
        const int vr = tid >> 4, vc = tid & 15;      // V items: row vr + 8*it, chunk vc
        struct UnitRegs { uint4 ka[kKItems], kb[kKItems], v[kVItems]; };
        struct Unit { Tile d; int cs; };
        TileWalk<kPipeUnit> walk(t_begin, t_end);
        int n_fetched = 0, n_tables = 0, last_seg = -1;
        // Loads go through buffer descriptors whose base is the unit's first key / value (wavefront-uniform, worked
        // out on the scalar unit); a thread's offsets inside a unit depend only on the distance between tokens and
        // are kept: rows past the end of a ragged unit re-read its last row.
        uint32_t row_bytes = 0, koff[kKItems], voff[kVItems];
        auto fetch = [&](Unit& u, UnitRegs& r) {     // a fixed number of loads, as in attn_tile_kernel
            if constexpr (REG_TABLE) u.d = walk.next(rtbl, lane);
            else u.d = walk.next(tbl, lane);
            if (tid == kWave) desc_ring[n_fetched & (kPipeDesc - 1)] = make_int4(u.d.seg, u.d.tok0, u.d.ntok, u.d.self);
            ++n_fetched;
            const TileSource src = tile_source(a, u.d, walk.c_tok, hkv);
            if (src.row_bytes != row_bytes && src.last >= 0) {           // the store's and the own block's rows differ
                row_bytes = src.row_bytes;
#pragma unroll
                for (int it = 0; it < kKItems; ++it) koff[it] = (uint32_t)(kr + (kPT / 8) * it) * row_bytes + 16 * kj;
#pragma unroll
                for (int it = 0; it < kVItems; ++it) voff[it] = (uint32_t)(vr + (kPT / 16) * it) * row_bytes + 16 * vc;
            }
            const int last = src.last;               // -1: no unit left, everything reads the first bytes of the workspace
            const uint32_t last_row = last < 0 ? 0u : (uint32_t)last * row_bytes;
            const uint32_t klast = last < 0 ? 0u : last_row + 16 * kj, vlast = last < 0 ? 0u : last_row + 16 * vc;
            const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(src.k), 0, 0x7fffffff, 0x00020000);
            const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(src.v), 0, 0x7fffffff, 0x00020000);
            const int hi = last < 0 ? 0 : 128;       // the second chunk of a pair sits 64 channels on
#pragma unroll
            for (int it = 0; it < kKItems; ++it) {
                const uint32_t off = kr + (kPT / 8) * it > last ? klast : koff[it];
                r.ka[it] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rk, off, 0, 0));
                r.kb[it] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rk, off, hi, 0));
            }
#pragma unroll
            for (int it = 0; it < kVItems; ++it) {
                const uint32_t off = vr + (kPT / 16) * it > last ? vlast : voff[it];
                r.v[it] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rv, off, 0, 0));
            }
        };
        // the cos/sin table of a unit that starts a segment with a shift; units of one segment share theirs
        // (made by the second producer wavefront, which also writes the unit descriptors)
        auto table_for = [&](Unit& u) {
            if (u.d.ntok > 0 && u.d.delta != 0 && u.d.seg != last_seg) {
                ++n_tables;
                if (tid >= kWave) cs_lds[n_tables & (kPipeCs - 1)][tid - kWave] = rope_cos_sin_fast(u.d.delta, my_freq);
            }
            if (u.d.ntok > 0) last_seg = u.d.seg;
            u.cs = n_tables & (kPipeCs - 1);
        };
        auto stage = [&](const Unit& u, const UnitRegs& r, int slot) {
            if (u.d.ntok <= 0) return;
            unsigned char* k_lds = k_ring[slot];
            unsigned char* v_lds = v_ring[slot];
            ChunkAngles ang;
            if (u.d.delta != 0) ang = load_chunk_angles(cs_lds[u.cs] + 8 * kj);
#pragma unroll
            for (int it = 0; it < kKItems; ++it) {
                uint4 ra = r.ka[it], rb4 = r.kb[it];
                if (u.d.delta != 0) rotate_chunk_pair<DT>(ra, rb4, ang);
                k_tile_write(k_lds, kr + (kPT / 8) * it, kj, ra);
                k_tile_write(k_lds, kr + (kPT / 8) * it, kj + 8, rb4);
            }
#pragma unroll
            for (int it = 0; it < kVItems; ++it) {
                const int t = vr + (kPT / 16) * it;
                *reinterpret_cast<uint4*>(v_lds + t * 256 + 16 * (vc ^ (2 * (t & 7)))) = r.v[it];
            }
        };
        Unit a0, a1, b0, b1;
        UnitRegs ra0, ra1, rb0, rb1;
        fetch(a0, ra0); fetch(a1, ra1); fetch(b0, rb0); fetch(b1, rb1);
        table_for(a0); table_for(a1);
        __syncthreads();                             // the tables of pair 0 are published
        int slot = 0;                                // the slot pair s goes to: 2 * (s % 4)
        // step s: stage pair s, refill its registers with pair s + 2, make the tables of pair s + 1
        auto step = [&](Unit& x0, Unit& x1, UnitRegs& r0, UnitRegs& r1, Unit& y0, Unit& y1) {
            stage(x0, r0, slot);
            stage(x1, r1, slot + 1);
            slot = (slot + 2) & (kPipeSlots - 1);
            fetch(x0, r0);
            fetch(x1, r1);
            table_for(y0);
            table_for(y1);
            __syncthreads();
        };
        for (int s = 0; s < n_steps; s += 2) {
            step(a0, a1, ra0, ra1, b0, b1);
            step(b0, b1, rb0, rb1, a0, a1);
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
    const float scale_log2e = a.scale_log2e;
    int cur_seg = -1;

    // fragments and results in flight (see the head of the kernel)
    uint4 kf[2][4];                                  // K fragments of the unit whose scores come next
    short4v vlo[8], vhi[8];                          // V^T fragments of the unit whose O^T update comes next
    f32x4 sc[NRB][2];                                // S^T of the unit whose softmax comes next
    uint4 pfrag[NRB];                                // P^T of the unit whose O^T update comes next
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) pfrag[rb] = make_uint4(0, 0, 0, 0);

    // slot: the unit's index modulo kPipeSlots, kept by the caller (no division inside the scheduled blocks)
    auto read_k = [&](int slot) {
        const unsigned char* k_lds = k_ring[slot];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) kf[tb][kk] = k_tile_fragment(k_lds, 16 * tb + li, 4 * kk + lg);
    };
    auto read_v = [&](int slot) {
        const unsigned char* v_lds = v_ring[slot];
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const unsigned char* src = v_lds + tr_base + ((uint32_t)(32 * db) ^ tr_x);
            vlo[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(src));
            vhi[db] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(src + 16 * 256));
        }
    };
    auto scores_into = [&](f32x4 (&out)[NRB][2]) {
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) { out[rb][0] = f32x4{0.f, 0.f, 0.f, 0.f}; out[rb][1] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb) out[rb][tb] = Mma<DT>::run(kf[tb][kk], qf[rb][kk], out[rb][tb]);
    };
    auto weigh_prev = [&]() {                        // O^T += V^T P^T of the previous unit
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const uint2 l2 = __builtin_bit_cast(uint2, vlo[db]), h2v = __builtin_bit_cast(uint2, vhi[db]);
            const uint4 va = make_uint4(l2.x, l2.y, h2v.x, h2v.y);
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) st.acc[rb][db] = Mma<DT>::run(va, pfrag[rb], st.acc[rb][db]);
        }
    };
    auto desc_of = [&](int u) {
        const int4 e = desc_ring[u & (kPipeDesc - 1)];
        Tile t;
        t.seg = __builtin_amdgcn_readfirstlane(e.x);
        t.tok0 = __builtin_amdgcn_readfirstlane(e.y);
        t.ntok = __builtin_amdgcn_readfirstlane(e.z);
        t.self = __builtin_amdgcn_readfirstlane(e.w);
        t.delta = 0;                                 // the staged keys are rotated already
        return t;
    };

    // One iteration (see the head of the kernel).  MASKED: unit i is ragged or the causal own block; FIRST: i == 0,
    // nothing to weigh yet.  The K and the V^T fragments share their time in registers: the V^T fragments of unit
    // i - 1 are requested while the scores consume the K fragments of unit i + 1, the K fragments of unit i + 2 while
    // the O^T update consumes the V^T fragments.
    int slot_i = 0;                                  // unit i modulo kPipeSlots
    auto iterate = [&](const Tile& cd, auto masked_tag, auto first_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr bool FIRST = decltype(first_tag)::value;
        if (cd.seg != cur_seg) {
            if (cur_seg >= 0) emit_segment<NRB>(st, massml, cur_seg + split, p.rows_wg, cw * NRB, li, lg);
            cur_seg = cd.seg;
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) st.seg_l[rb] = 0.f;
        }
        const bool causal = cd.self != 0;
        f32x4 sn[NRB][2];
        float lsum[NRB];
        uint4 pnew[NRB];
        // probabilities of row block rb against the reference as it stands
        auto probabilities = [&](int rb) {
            float xv[8], pv[8];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int e = 0; e < 4; ++e) xv[4 * tb + e] = sc[rb][tb][e];
            if constexpr (MASKED) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int tk = 16 * (e >> 2) + 4 * lg + (e & 3);
                    const bool ok = tk < cd.ntok && (!causal || cd.tok0 + tk <= trow[rb]);
                    xv[e] = ok ? xv[e] : -INFINITY;
                    sc[rb][e >> 2][e & 3] = xv[e];   // the repair path works on the masked scores
                }
            }
            const float m_safe = st.m_run[rb] == -INFINITY ? 0.f : st.m_run[rb];
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pv[e] = __builtin_amdgcn_exp2f(fmaf(xv[e], scale_log2e, -m_safe));
                s += pv[e];
            }
            lsum[rb] = s;
            pnew[rb] = make_uint4(Mma<DT>::pack(pv[0], pv[1]), Mma<DT>::pack(pv[2], pv[3]), Mma<DT>::pack(pv[4], pv[5]),
                                  Mma<DT>::pack(pv[6], pv[7]));
        };
        const int slot_prev = slot_i == 0 ? kPipeSlots - 1 : slot_i - 1;
        const int slot_next2 = slot_i + 2 >= kPipeSlots ? slot_i + 2 - kPipeSlots : slot_i + 2;
        __builtin_amdgcn_sched_barrier(0);
        // ---- first half: the scores of unit i + 1 beside the softmax of the first row block of unit i
        scores_into(sn);
        probabilities(0);
        if constexpr (!FIRST) read_v(slot_prev);
        // (a V^T read only once four MFMAs have released the K fragments whose registers it takes over)
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, MASKED ? 3 : 2, 0);       // a few VALU
            if (!FIRST && (n & 3) == 3) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);     // four LDS reads
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- second half: O^T of unit i - 1 beside the softmax of the second row block of unit i
        if constexpr (!FIRST) weigh_prev();
        probabilities(1);
        read_k(slot_next2);
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            if (!FIRST) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, MASKED ? 3 : 2, 0);
            if (n & 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- did a reference have to move?  (rare after a row's first units)
        bool off[NRB];
        bool any_off = false;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            off[rb] = !(lsum[rb] <= kProbLimit) || st.m_run[rb] == -INFINITY;
            any_off = any_off || off[rb];
        }
        if (__any(any_off)) {
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) {
                if (!__any(off[rb])) continue;
                float xv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) xv[e] = sc[rb][e >> 2][e & 3];
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
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                float pv[8];
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    pv[e] = __builtin_amdgcn_exp2f(fmaf(xv[e], scale_log2e, -m_safe));
                    s += pv[e];
                }
                lsum[rb] = s;
                pnew[rb] = make_uint4(Mma<DT>::pack(pv[0], pv[1]), Mma<DT>::pack(pv[2], pv[3]), Mma<DT>::pack(pv[4], pv[5]),
                                      Mma<DT>::pack(pv[6], pv[7]));
            }
        }
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            st.l_run[rb] += lsum[rb];
            st.seg_l[rb] += lsum[rb];
            pfrag[rb] = pnew[rb];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb) sc[rb][tb] = sn[rb][tb];
        }
        slot_i = slot_i + 1 == kPipeSlots ? 0 : slot_i + 1;
    };

    __syncthreads();                                 // the tables of pair 0
    __syncthreads();                                 // step 0: pair 0 is staged
    Tile upcoming = desc_of(0);
    if (has_rows && n_units > 0) {
        read_k(0);
        scores_into(sc);
        read_k(1);
    }
    auto run_unit = [&](int i, auto first_tag) {
        if (i >= n_units) return;
        const Tile cd = upcoming;
        upcoming = desc_of(i + 1);
        if (cd.ntok < kPipeUnit || cd.self != 0) iterate(cd, std::true_type{}, first_tag);
        else iterate(cd, std::false_type{}, first_tag);
    };
    __syncthreads();                                 // step 1: pair 1 is staged
    if (has_rows) {
        run_unit(0, std::true_type{});
        run_unit(1, std::false_type{});
    }
    for (int k = 1; k < n_steps - 1; ++k) {
        __syncthreads();                             // step k + 1: pair k + 1 is staged; the loads in flight have landed
        if (!has_rows) continue;
        run_unit(2 * k, std::false_type{});
        run_unit(2 * k + 1, std::false_type{});
    }
    if (!has_rows) return;
    if (n_units > 0) {                               // the last unit's O^T update
        read_v(slot_i == 0 ? kPipeSlots - 1 : slot_i - 1);
        weigh_prev();
    }
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
    // grid dimensions of this path's kernels (the merge kernel's may carry one more row, for pending score parts)
    if (a.batch > 65535 || (int64_t)a.n_kv_heads * p.n_rg + 1 > 65535) {
        set_error("batch must not exceed 65535 and n_kv_heads * row groups 65534 on this path");
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
        if (reg_table) CF_LAUNCH_TIMED((attn_pipe_kernel<DT, true>), grid, dim3(kPcWaves * kWave));                                  \
        else CF_LAUNCH_TIMED((attn_pipe_kernel<DT, false>), grid, dim3(kPcWaves * kWave));                                           \
    }                                                                                                                          \
    CF_HIP(hipGetLastError());
    if (a.dtype == CF_BF16) { CF_LAUNCH_DT(CF_BF16) } else { CF_LAUNCH_DT(CF_F16) }
#undef CF_LAUNCH_DT
#undef CF_LAUNCH_TIMED
    const bool combine = !(p.direct_out && a.mass == nullptr);            // else nothing left to merge or reduce
    // before a fused epilogue the pending score parts are taken in by one more row of the combine kernel's grid
    const bool pending_beside = combine && !a.defer && prune && a.n_pending > 0 && epilogue_fits(p, prune) && pending_fit_combine(a, p);
    if (combine) launch_combine(a, p, pending_beside, s);
    CF_HIP(hipGetLastError());
    if (a.defer) return CF_OK;                       // the slot partials stay in the ledger for a later call
    if (prune) {
        if (epilogue_fits(p, prune)) {
            if (a.n_pending > 0 && !pending_beside) launch_pending_masses(a, p, s);
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
