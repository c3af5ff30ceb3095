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

#include "cf_common.h"
#include "cf_select_dev.h"

namespace cf {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kD = 128;
constexpr int kHalf = 64;
constexpr int kKRow = 272;      // bytes per token of a staged K tile
constexpr int kMaxSegs = 256;
constexpr int kMaxSplit = 32;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

struct Plan {
    int row_blocks;     // 16-row blocks of the stacked rows of one kv head
    int producers;      // 0: attn_tile_kernel (few rows); else attn_pc_kernel with that many loading wavefronts
    int nrb;            // 64-row passes of a workgroup's rows (what the combine kernel handles at a time)
    int rows_wg;        // rows a workgroup has room for: 64 * nrb
    int n_rg;           // row groups per (query, kv head)
    int blocks_rg;      // 16-row blocks per row group
    int units_per_b, units, nsplit, slots, x_count;
    int tile;           // tokens per tile: 32 or 64
    int groups;         // groups of four wavefronts per workgroup (each streams its own run of tiles): 1 or 2
    size_t off_ml, off_opart, off_massml, off_masspart, total;
};

constexpr int kPcWaves = 8;         // wavefronts of an attn_pc_kernel workgroup
constexpr int kPcProducers = 2;     // of which load and stage
constexpr int kPcNrb = 2;           // 16-row blocks per math wavefront

Plan make_plan(int n_q_heads, int n_kv_heads, int batch, int max_tq, int seg_stride, int64_t max_kv_tokens) {
    Plan p;
    const int group = n_q_heads / n_kv_heads;
    const int row_blocks = (group * max_tq + 15) / 16;
    p.row_blocks = row_blocks;
    if (row_blocks <= 4) {
        // Few stacked rows (MHA-like, HBM-bound): one row block per wavefront, small tiles, so that ragged
        // segment ends waste little and a split still holds several tiles; two groups of four wavefronts per
        // workgroup run two tiles at a time on one CU and hide each other's LDS and barrier waits.
        p.producers = 0;
        p.n_rg = 1;
        p.nrb = 1;
        p.tile = 32;
        p.groups = 2;
    } else {
        // Many rows (GQA, long queries): 64-token tiles, two row blocks per math wavefront.
        const int blocks_wg = kPcNrb * (kPcWaves - kPcProducers);
        p.producers = kPcProducers;
        p.n_rg = (row_blocks + blocks_wg - 1) / blocks_wg;
        p.nrb = blocks_wg / 4;
        p.tile = 64;
        p.groups = 1;
    }
    p.blocks_rg = (row_blocks + p.n_rg - 1) / p.n_rg;
    p.rows_wg = 64 * p.nrb;
    p.units_per_b = n_kv_heads * p.n_rg;
    p.units = batch * p.units_per_b;
    const int64_t est_tiles = max_kv_tokens / p.tile + seg_stride;
    // One workgroup per CU and launch wave.  A CU holds one attn_pc_kernel workgroup at a time, so there the
    // count stays within the 256 CUs; two of the small kernel's fit, and a few more than 256 do no harm.
    int64_t ns = p.producers ? 256 / p.units : (256 + p.units - 1) / p.units;
    const int64_t cap = est_tiles / (2 * p.groups) > 1 ? est_tiles / (2 * p.groups) : 1;
    if (ns > cap) ns = cap;
    if (ns > kMaxSplit) ns = kMaxSplit;
    if (ns < 1) ns = 1;
    p.nsplit = (int)ns;
    p.slots = seg_stride + p.nsplit * p.groups;
    p.x_count = batch * n_kv_heads * p.nsplit;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
    p.off_ml = take((size_t)p.units * p.nsplit * p.rows_wg * sizeof(float2));
    p.off_opart = take((size_t)p.units * p.nsplit * p.rows_wg * kD * sizeof(float));
    p.off_massml = take((size_t)p.units * p.slots * p.rows_wg * sizeof(float2));
    p.off_masspart = take((size_t)p.units * p.nrb * p.slots * sizeof(float));
    p.total = off;
    return p;
}


// Per-query segment table in LDS with the tile prefix that defines the partition.
struct SegTable {
    int64_t tok[kMaxSegs];      // first token in its tensor
    int32_t vis[kMaxSegs];      // visible tokens (0 for a rejected entry)
    int32_t delta[kMaxSegs];    // relative shift: (new - stored) - (q_new - q_stored)
    int32_t self[kMaxSegs];     // 1 for the causal own block
    int32_t doc[kMaxSegs];      // document slot of the entry (-1: none)
    int32_t tile0[kMaxSegs + 1];// exclusive prefix of tile counts
    int32_t n;
};

// Per-query scalars and this thread's segment-table entry, fetched in one batch: the entry is
// read for the whole stride so that its load does not wait for the segment count.
struct QueryHead {
    int q0, tq_raw, n_seg, qdelta;
    int64_t q_total;
    cf_segment seg;
};

// `entry`: which table entry this thread takes (its index in the workgroup for the LDS table, its lane
// for the register table).
__device__ __forceinline__ QueryHead load_query_head(const AttnArgs& a, int b, int entry) {   // b: wave-uniform
    QueryHead h;
    if (entry < a.seg_stride) h.seg = a.segs[(int64_t)b * a.seg_stride + entry];   // seg_stride <= kMaxSegs == kThreads
    const int q0 = a.q_off[b], q1 = a.q_off[b + 1], qt = a.q_off[a.batch], n = a.n_seg[b], qn = a.q_new_start[b];
    asm volatile("" ::"s"(q0), "s"(q1), "s"(qt), "s"(n), "s"(qn));    // all five scalar loads are out before any is used
    h.q0 = q0;
    h.tq_raw = q1 - q0;
    h.q_total = qt;
    h.n_seg = n;
    h.qdelta = qn - a.q_stored_start;
    return h;
}

// All threads of a workgroup call this; every workgroup of query b builds the same table.
__device__ __forceinline__ void build_table(const AttnArgs& a, const QueryHead& h, SegTable* t, int tile_tokens) {
    const int tid = threadIdx.x;
    const cf_segment& seg = h.seg;
    int n = h.n_seg;
    if (n < 0 || n > a.seg_stride) {
        if (tid == 0) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        n = n < 0 ? 0 : a.seg_stride;
    }
    const int tq = min(h.tq_raw, a.max_tq);
    if (tid < n) {
        const bool self = seg.kind == CF_SEG_SELF;
        const int64_t limit = self ? h.q_total : a.n_store_tokens;
        const bool bad = seg.kind < 0 || seg.kind > CF_SEG_SELF || seg.len < 0 || seg.tok_offset < 0 ||
                         seg.tok_offset + seg.len > limit || (self && a.k_self == nullptr);
        if (bad) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        const int vis = bad ? 0 : (self ? min(seg.len, tq) : seg.len);
        t->tok[tid] = seg.tok_offset;
        t->vis[tid] = vis;
        t->delta[tid] = seg.new_start - seg.stored_start - h.qdelta;
        t->self[tid] = self ? 1 : 0;
        t->doc[tid] = seg.doc;
        t->tile0[tid + 1] = (vis + tile_tokens - 1) / tile_tokens;
    }
    if (tid == 0) { t->n = n; t->tile0[0] = 0; }
    __syncthreads();
    if (tid < kWave) {                               // inclusive scan by the first wavefront
        int carry = 0;
        for (int c0 = 0; c0 < n; c0 += kWave) {
            const int s = c0 + tid;
            int v = s < n ? t->tile0[s + 1] : 0;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int u = __shfl_up(v, o);
                if (tid >= o) v += u;
            }
            if (s < n) t->tile0[s + 1] = v + carry;
            carry += __shfl(v, kWave - 1);
        }
    }
    __syncthreads();
}

// split i of a list of `total` tiles owns [total*i/nsplit, total*(i+1)/nsplit)
__device__ __forceinline__ int split_begin(unsigned total, unsigned nsplit, unsigned i) { return (int)div_exact(total * i, nsplit); }
// the split that owns tile x
__device__ __forceinline__ int split_of(unsigned total, unsigned nsplit, unsigned x) { return (int)div_exact((x + 1) * nsplit - 1, total); }

template <int DT> struct Mma;
template <> struct Mma<CF_BF16> {
    static __device__ __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
    static __device__ __forceinline__ uint32_t pack(float x, float y) {
        f32x2 v = {x, y};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    }
};
template <> struct Mma<CF_F16> {
    static __device__ __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float lo(uint32_t w) { return (float)__builtin_bit_cast(f16x2, w)[0]; }
    static __device__ __forceinline__ float hi(uint32_t w) { return (float)__builtin_bit_cast(f16x2, w)[1]; }
    static __device__ __forceinline__ uint32_t pack(float x, float y) {
        f32x2 v = {x, y};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
    }
};

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

// One tile of the walk over a split's tiles; ntok == 0 marks "no tile left".
struct Tile { int seg, tok0, ntok, delta, self; };

// The same table for at most 64 segments, held in registers: lane s of every wavefront describes segment s.
// Built by each wavefront for itself — no LDS, no barrier — and searched with a ballot and lane reads.
struct RegSegTable {
    int64_t tok;                // this lane's segment, as in SegTable
    int32_t vis, delta, self;
    int32_t t0, t1;             // its tiles [t0, t1)
    int32_t n, total;           // wavefront-uniform: segments, tiles
};

// `h.seg` is entry `lane`; seg_stride <= 64.
__device__ __forceinline__ RegSegTable build_reg_table(const AttnArgs& a, const QueryHead& h, int lane, int tile_tokens) {
    RegSegTable t;
    const cf_segment& seg = h.seg;
    int n = h.n_seg;
    if (n < 0 || n > a.seg_stride) {
        if (lane == 0) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        n = n < 0 ? 0 : a.seg_stride;
    }
    const int tq = min(h.tq_raw, a.max_tq);
    int vis = 0;
    t.tok = 0; t.delta = 0; t.self = 0;
    if (lane < n) {
        const bool self = seg.kind == CF_SEG_SELF;
        const int64_t limit = self ? h.q_total : a.n_store_tokens;
        const bool bad = seg.kind < 0 || seg.kind > CF_SEG_SELF || seg.len < 0 || seg.tok_offset < 0 ||
                         seg.tok_offset + seg.len > limit || (self && a.k_self == nullptr);
        if (bad) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        vis = bad ? 0 : (self ? min(seg.len, tq) : seg.len);
        t.tok = seg.tok_offset;
        t.delta = seg.new_start - seg.stored_start - h.qdelta;
        t.self = self ? 1 : 0;
    }
    t.vis = vis;
    const int tiles = (vis + tile_tokens - 1) / tile_tokens;
    t.t1 = wave_inclusive_scan(tiles);
    t.t0 = t.t1 - tiles;
    t.n = n;
    t.total = __builtin_amdgcn_readlane(t.t1, kWave - 1);
    return t;
}

// The segment that owns tile x (x < total) and its fields, in scalars.  `prev`: the segment found last (-1: none).
struct FoundSegment { int seg, first, end, vis, delta, self; int64_t tok; };

__device__ __forceinline__ FoundSegment find_segment(const SegTable& tbl, int x, int lane, int prev) {
    // the first segment whose tiles reach past x: every lane tests one entry per round
    int s = 0;
    for (int s0 = prev < 0 ? 0 : (prev & ~(kWave - 1));; s0 += kWave) {
        const int idx = s0 + lane;
        const unsigned long long hit = __ballot(idx < tbl.n && tbl.tile0[idx + 1] > x);
        if (hit) { s = s0 + __builtin_ctzll(hit); break; }
    }
    FoundSegment f;
    f.seg = s;
    f.first = tbl.tile0[s];
    f.end = tbl.tile0[s + 1];
    f.vis = tbl.vis[s];
    f.delta = tbl.delta[s];
    f.self = tbl.self[s];
    f.tok = tbl.tok[s];
    return f;
}

__device__ __forceinline__ FoundSegment find_segment(const RegSegTable& t, int x, int lane, int) {
    const unsigned long long hit = __ballot(lane < t.n && t.t1 > x);
    const int s = hit ? __builtin_ctzll(hit) : 0;       // x < total: some lane always answers
    FoundSegment f;
    f.seg = s;
    f.first = __builtin_amdgcn_readlane(t.t0, s);
    f.end = __builtin_amdgcn_readlane(t.t1, s);
    f.vis = __builtin_amdgcn_readlane(t.vis, s);
    f.delta = __builtin_amdgcn_readlane(t.delta, s);
    f.self = __builtin_amdgcn_readlane(t.self, s);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)t.tok, s);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)t.tok >> 32), s);
    f.tok = (int64_t)(((uint64_t)hi << 32) | lo);
    return f;
}

// Walks the tiles [next_tile, t_end) of the segment table in order.  All state is wavefront-uniform;
// the segment of the tile handed out last is cached, since most tiles continue their predecessor's.
template <int TILE>
struct TileWalk {
    int next_tile, t_end;
    int c_seg = -1, c_first = 0, c_end = 0, c_vis = 0, c_delta = 0, c_self = 0;
    int64_t c_tok = 0;          // first token of the cached segment in its tensor

    __device__ __forceinline__ TileWalk(int begin, int end) : next_tile(begin), t_end(end) {}

    // The next tile, or a tile with ntok == 0 when none is left.
    template <class Table>
    __device__ __forceinline__ Tile next(const Table& tbl, int lane) {
        Tile d;
        if (next_tile < t_end) {
            if (next_tile >= c_end) {
                const FoundSegment f = find_segment(tbl, next_tile, lane, c_seg);
                c_seg = f.seg;
                c_first = f.first;
                c_end = f.end;
                c_vis = f.vis;
                c_delta = f.delta;
                c_self = f.self;
                c_tok = f.tok;
            }
            d.seg = c_seg;
            d.tok0 = (next_tile - c_first) * TILE;
            d.ntok = max(0, min(TILE, c_vis - d.tok0));
            d.delta = c_delta;
            d.self = c_self;
            ++next_tile;
        } else {
            d.seg = 0; d.tok0 = 0; d.ntok = 0; d.delta = 0; d.self = 0;
        }
        return d;
    }
};

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
        const int gi = valid ? m / tq : 0;
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

// Partial results of a split: O^T in MFMA layout (one float4 per lane, row block and channel block)
// and (reference, row sum) per row.
template <int NRB>
__device__ __forceinline__ void store_partials(const AttnArgs& a, const Plan& p, int unit, int split, int first_blk,
                                               const RowState<NRB>& st, const float (&l_row)[NRB], int lane) {
    char* ws = static_cast<char*>(a.workspace);
    f32x4* opart = reinterpret_cast<f32x4*>(ws + p.off_opart) +
                   (((int64_t)unit * p.nsplit + split) * p.rows_wg / 16 + first_blk) * 8 * kWave + lane;
    float2* ml = reinterpret_cast<float2*>(ws + p.off_ml) + ((int64_t)unit * p.nsplit + split) * p.rows_wg;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
        for (int db = 0; db < 8; ++db) opart[(rb * 8 + db) * kWave] = st.acc[rb][db];
        if ((lane >> 4) == 0) ml[(first_blk + rb) * 16 + (lane & 15)] = make_float2(st.m_run[rb], l_row[rb]);
    }
}

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

    // block -> (row group, query, kv head, split); workgroups that read the same K/V tiles differ
    // by a multiple of x_count
    const int bid = blockIdx.x;
    const int rg = bid / p.x_count;
    const int x = bid - rg * p.x_count;
    const int split = x % p.nsplit;
    const int hkv = (x / p.nsplit) % a.n_kv_heads;
    const int b = __builtin_amdgcn_readfirstlane(x / (p.nsplit * a.n_kv_heads));
    const int unit = (b * a.n_kv_heads + hkv) * p.n_rg + rg;

    const int group = a.n_q_heads / a.n_kv_heads;
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
    int most_tiles = 0;                              // workgroup-uniform: the longest run among the groups
#pragma unroll
    for (int g = 0; g < GROUPS; ++g)
        most_tiles = max(most_tiles, split_begin(total, nsub, split * GROUPS + g + 1) - split_begin(total, nsub, split * GROUPS + g));

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
    store_partials<NRB>(a, p, unit, split, wave * NRB, st, l_row, lane);
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

    const int bid = blockIdx.x;
    const int rg = bid / p.x_count;
    const int x = bid - rg * p.x_count;
    const int split = x % p.nsplit;
    const int hkv = (x / p.nsplit) % a.n_kv_heads;
    const int b = __builtin_amdgcn_readfirstlane(x / (p.nsplit * a.n_kv_heads));
    const int unit = (b * a.n_kv_heads + hkv) * p.n_rg + rg;
    const int group = a.n_q_heads / a.n_kv_heads;
    const QueryHead qh = load_query_head(a, b, REG_TABLE ? lane : (int)threadIdx.x);
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
    store_partials<NRB>(a, p, unit, split, cw * NRB, st, l_row, lane);
}

// Second kernel: one workgroup per (unit, 64-row pass, eighth of the output channels) merges the
// splits' partial outputs and writes its output rows; the eight workgroups of a (unit, pass) also share
// the reduction, over the pass's 64 rows, of every (segment, split) slot's (max, sum) pairs to
// sum * exp2(max - row max) / row sum, which the mass kernel then only has to add up.
template <int DT>
__global__ __launch_bounds__(kThreads) void attn_combine_kernel(AttnArgs a, Plan p) {
    __shared__ float2 mlw[kMaxSplit * 64];       // (m, l) per split and row, then the split's weight in .x
    __shared__ float2 rstat[64];                 // (max, 1/sum) per row of this pass
    constexpr int kPre = 8;                      // splits whose partial outputs are fetched before the statistics are ready

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int li = lane & 15, lg = lane >> 4;
    char* ws = static_cast<char*>(a.workspace);
    const int hq = a.n_q_heads, group = hq / a.n_kv_heads;
    const int dbq = blockIdx.x & 7;
    const int pass = (blockIdx.x >> 3) % p.nrb;
    const int unit = blockIdx.x / (8 * p.nrb);
    const int rg = unit % p.n_rg;
    const int hkv = (unit / p.n_rg) % a.n_kv_heads;
    const int b = unit / p.units_per_b;
    const int q0 = a.q_off[b], q1 = a.q_off[b + 1];
    const float2* ml = reinterpret_cast<const float2*>(ws + p.off_ml) + (int64_t)unit * p.nsplit * p.rows_wg + pass * 64;
    const f32x4* opart = reinterpret_cast<const f32x4*>(ws + p.off_opart) + (int64_t)unit * p.nsplit * p.rows_wg * (kD / 4);
    const int blk = pass * kWaves + wave;                      // row block inside the workgroup tile
    const f32x4* src = opart + ((int64_t)blk * 8 + dbq) * kWave + lane;
    const int64_t split_stride = (int64_t)p.rows_wg / 16 * 8 * kWave;
    const float2* massml = reinterpret_cast<const float2*>(ws + p.off_massml) + (int64_t)unit * p.slots * p.rows_wg + pass * 64 + lane;
    const int k_first = dbq * kWaves + wave, k_step = 8 * kWaves;

    // Everything this workgroup reads is requested up front — row statistics, partial outputs of the
    // first splits, the first slot statistics — so the three round trips to memory overlap.
    for (int idx = tid; idx < p.nsplit * 64; idx += kThreads) mlw[idx] = ml[(idx >> 6) * p.rows_wg + (idx & 63)];
    // (a wavefront whose 16 rows are all padding reads what an earlier call left there: in bounds, never stored;
    // not waiting for the query's length here saves a round trip)
    f32x4 pre[kPre];
#pragma unroll
    for (int s = 0; s < kPre; ++s) pre[s] = s < p.nsplit ? src[s * split_stride] : f32x4{0.f, 0.f, 0.f, 0.f};
    float2 sv[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int k = k_first + j * k_step;
        sv[j] = k < p.slots ? massml[(int64_t)k * p.rows_wg] : make_float2(0.f, 0.f);
    }
    const int tq = min(q1 - q0, a.max_tq);
    const int n_rows = group * tq;
    const int row_base = rg * p.blocks_rg * 16;
    const int rows_here = min(p.blocks_rg * 16, n_rows - row_base);
    const bool blk_has_rows = pass * 64 + wave * 16 < rows_here;
    __syncthreads();
    if (tid < 64) {
        float m = -INFINITY;
        for (int s = 0; s < p.nsplit; ++s) m = fmaxf(m, mlw[s * 64 + tid].x);
        const float ms = m == -INFINITY ? 0.f : m;
        float z = 0.f;
        for (int s = 0; s < p.nsplit; ++s) z += mlw[s * 64 + tid].y * exp2f(mlw[s * 64 + tid].x - ms);
        const float iz = z > 0.f ? 1.f / z : 0.f;
        for (int s = 0; s < p.nsplit; ++s) mlw[s * 64 + tid].x = exp2f(mlw[s * 64 + tid].x - ms) * iz;
        rstat[tid] = make_float2(ms, pass * 64 + tid < rows_here ? iz : 0.f);    // padding rows carry no mass
    }
    __syncthreads();
    f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < kPre; ++s)
        if (s < p.nsplit) o += pre[s] * mlw[s * 64 + wave * 16 + li].x;
    if (blk_has_rows)
        for (int s0 = kPre; s0 < p.nsplit; s0 += kPre) {         // further splits, eight loads at a time
            f32x4 more[kPre];
#pragma unroll
            for (int i = 0; i < kPre; ++i) more[i] = s0 + i < p.nsplit ? src[(s0 + i) * split_stride] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < kPre; ++i)
                if (s0 + i < p.nsplit) o += more[i] * mlw[(s0 + i) * 64 + wave * 16 + li].x;
        }
    const int lrow = pass * 64 + wave * 16 + li;
    if (lrow < rows_here) {
        const int m2 = row_base + lrow;
        const int gi = m2 / tq, t = m2 - gi * tq;
        uint16_t* op = static_cast<uint16_t*>(a.out) + (((int64_t)q0 + t) * hq + hkv * group + gi) * kD + 16 * dbq + 4 * lg;
        uint2 pk;
        pk.x = Mma<DT>::pack(o[0], o[1]);
        pk.y = Mma<DT>::pack(o[2], o[3]);
        *reinterpret_cast<uint2*>(op) = pk;
    }
    // slot partials: slot k = segment + split; slots no split wrote this call hold stale pairs and
    // give meaningless numbers that the mass kernel never reads
    if (a.mass != nullptr) {
        float* masspart = reinterpret_cast<float*>(ws + p.off_masspart) + ((int64_t)unit * p.nrb + pass) * p.slots;
        const float2 st = rstat[lane];
        auto reduce = [&](int k, float2 v) {
            const float c = wave_sum_dpp(st.y > 0.f ? v.y * exp2f(v.x - st.x) * st.y : 0.f);
            if (lane == 0 && k < p.slots) masspart[k] = c;
        };
#pragma unroll
        for (int j = 0; j < 2; ++j) reduce(k_first + j * k_step, sv[j]);
        for (int k = k_first + 2 * k_step; k < p.slots; k += k_step) reduce(k, massml[(int64_t)k * p.rows_wg]);
    }
}

// Per-segment attention mass of one query, by the whole workgroup, in a fixed order: first every
// slot's partials are added over the (unit, pass) parts, then a segment adds the slots of the
// splits that hold its tiles.  A split between a segment's first and last may own no tile at
// all (fewer tiles than splits): its slot was not written by this call and is skipped.
// `parts`: [nparts][slots] floats, in LDS (stage == nullptr; overwritten) or in memory (stage: kMassStage floats
// of LDS).  `on_mass(s, m)` is called once per segment.  Both forms add in the same order: the parts of a
// column in groups of eight, each group from zero, then the group sums from zero.
// Sum of n <= 8 values `pitch` floats apart, added in order from zero.  A full group's loads all go out
// before the first add (a loop with a run-time bound would wait for each in turn).
__device__ __forceinline__ float group_sum(const float* x, int pitch, int n) {
    float gs = 0.f;
    if (n == 8) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = x[i * pitch];
#pragma unroll
        for (int i = 0; i < 8; ++i) gs += v[i];
    } else {
        for (int i = 0; i < n; ++i) gs += x[i * pitch];
    }
    return gs;
}

struct MassScratch {
    float colsum[kMaxSegs + 2 * kMaxSplit];
    int32_t sub_begin[2 * kMaxSplit + 1];
};
constexpr int kMassStage = 4096;            // floats of partials staged per round by the stand-alone mass kernel

template <class F>
__device__ __forceinline__ void segment_masses_block(const Plan& p, const SegTable& tbl, float* parts, float* stage,
                                                     MassScratch* ms, F on_mass) {
    const int tid = threadIdx.x, nthr = blockDim.x;
    const unsigned total = (unsigned)tbl.tile0[tbl.n];
    const unsigned nsub = (unsigned)(p.nsplit * p.groups);
    const int nparts = p.units_per_b * p.nrb;
    constexpr int kGroup = 8;
    if (stage == nullptr) {                          // partials already in LDS: one thread per (group, column), in place
        const int ngroups = (nparts + kGroup - 1) / kGroup;
        for (int idx = tid; idx < ngroups * p.slots; idx += nthr) {
            const int g = idx / p.slots, k = idx - g * p.slots;
            const float gs = group_sum(parts + g * kGroup * p.slots + k, p.slots, min(kGroup, nparts - g * kGroup));
            parts[g * kGroup * p.slots + k] = gs;
        }
        __syncthreads();
        for (int k = tid; k < p.slots; k += nthr) {
            float c = 0.f;
            for (int g = 0; g < ngroups; ++g) c += parts[g * kGroup * p.slots + k];
            ms->colsum[k] = c;
        }
    } else {                                         // partials in memory: whole rows through LDS, many loads in flight
        const int rows = kMassStage / p.slots / kGroup * kGroup;   // slots <= kMassStage / kGroup: whole groups per round
        float c[2] = {0.f, 0.f};                     // this thread's columns tid, tid + nthr (slots <= 2 * nthr)
        for (int r0 = 0; r0 < nparts; r0 += rows) {
            const int nr = min(rows, nparts - r0);
            __syncthreads();
            for (int i = tid; i < nr * p.slots; i += nthr) stage[i] = parts[(int64_t)r0 * p.slots + i];
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int k = tid + j * nthr;
                if (k < p.slots)
                    for (int g0 = 0; g0 < nr; g0 += kGroup) c[j] += group_sum(stage + g0 * p.slots + k, p.slots, min(kGroup, nr - g0));
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (tid + j * nthr < p.slots) ms->colsum[tid + j * nthr] = c[j];
    }
    for (int sp = tid; sp <= (int)nsub; sp += nthr) ms->sub_begin[sp] = split_begin(total, nsub, sp);
    __syncthreads();
    for (int s = tid; s < tbl.n; s += nthr) {
        const int ts = tbl.tile0[s], te = tbl.tile0[s + 1];
        float m = 0.f;
        if (te > ts) {
            const int s0 = split_of(total, nsub, ts), s1 = split_of(total, nsub, te - 1);
            for (int sp = s0; sp <= s1; ++sp)
                if (ms->sub_begin[sp] < ms->sub_begin[sp + 1]) m += ms->colsum[s + sp];
        }
        on_mass(s, m);
    }
}

// The same for one wavefront on its own, for a query with at most 128 slots and a register table: lane k adds
// up columns k and k + 64, lane s then collects segment s's slots — the same sums in the same order, no barrier.
template <class F>
__device__ __forceinline__ void segment_masses_wave(const Plan& p, const RegSegTable& t, const float* parts, int lane, F on_mass) {
    const unsigned total = (unsigned)t.total;
    const unsigned nsub = (unsigned)(p.nsplit * p.groups);
    const int nparts = p.units_per_b * p.nrb;
    constexpr int kGroup = 8;
    float c[2] = {0.f, 0.f};                         // columns lane, lane + 64
#pragma unroll
    for (int j = 0; j < 2; ++j)
        if (lane + 64 * j < p.slots)
            for (int g0 = 0; g0 < nparts; g0 += kGroup)
                c[j] += group_sum(parts + g0 * p.slots + lane + 64 * j, p.slots, min(kGroup, nparts - g0));
    // sub-splits that own at least one tile (a split between a segment's first and last may own none)
    const bool owns = lane < (int)nsub && split_begin(total, nsub, lane) < split_begin(total, nsub, lane + 1);
    const unsigned long long owns_mask = __ballot(owns);
    const bool has_tiles = lane < t.n && t.t1 > t.t0;
    int s0 = 0, s1 = -1;
    if (has_tiles) { s0 = split_of(total, nsub, t.t0); s1 = split_of(total, nsub, t.t1 - 1); }
    const int span = wave_max_i32(s1 - s0);
    float m = 0.f;
    for (int d = 0; d <= span; ++d) {
        const int sp = s0 + d;
        const int slot = lane + sp;                                  // slot = segment + sub-split, < 128
        const float c_lo = __shfl(c[0], slot & (kWave - 1)), c_hi = __shfl(c[1], slot & (kWave - 1));
        if (has_tiles && sp <= s1 && ((owns_mask >> sp) & 1)) m += slot < kWave ? c_lo : c_hi;
    }
    if (lane < t.n) on_mass(lane, m);
}

// Third kernel: per-segment attention mass, one workgroup per query; then S += mass.
__global__ __launch_bounds__(kThreads) void attn_mass_kernel(AttnArgs a, Plan p) {
    __shared__ SegTable tbl;
    __shared__ MassScratch ms;
    __shared__ float stage[kMassStage];
    const char* ws = static_cast<const char*>(a.workspace);
    const int b = __builtin_amdgcn_readfirstlane(blockIdx.x);
    const QueryHead qh = load_query_head(a, b, (int)threadIdx.x);
    build_table(a, qh, &tbl, p.tile);
    const float* mp_b = reinterpret_cast<const float*>(ws + p.off_masspart) + (int64_t)b * p.units_per_b * p.nrb * p.slots;
    segment_masses_block(p, tbl, const_cast<float*>(mp_b), stage, &ms, [&](int s, float m) {
        a.mass[(int64_t)b * a.seg_stride + s] = m;
        const int doc = tbl.doc[s];
        if (a.score_accum && doc >= 0 && doc < a.score_stride) atomicAdd(&a.score_accum[(int64_t)b * a.score_stride + doc], m);
    });
}

// Fused layer epilogue (third kernel of cf_prefill_layer): one workgroup per query computes the
// attention mass of every segment (fixed summation order), adds it to the accumulated scores, and — when a prune step is attached —
// ranks the candidates, allocates the survivors' positions and writes the next layer's segment
// table, i.e. Alg. 2's "S += s; ids_sort = argsort(S); ids = prun(ids_sort)" followed by the
// allocation of Sec. 2.5, without leaving the GPU.
constexpr int kEpiThreads = 1024;

struct PruneArgs {
    int32_t enabled, keep, strategy, force_n_reuse, normalise_by_len, stride, pos_begin, pos_end, prefix_len,
        doc_stored_start;
    const int64_t* doc_tok_offset;
    const int32_t* doc_len;
    const int32_t* cand;
    const int32_t* n_cand;
    int32_t* keep_idx;
    int32_t* n_keep;
    int32_t* new_start;
    int32_t* q_start;
    int32_t* n_reuse;
    int32_t* order;
    cf_segment* next_segs;
    int32_t* next_n_seg;
};

// Every per-document row of the query (scores, lengths, candidates, offsets, positions) and the slot
// partial masses are fetched into LDS in one batch at the start: the ranking, the allocation and the
// table rebuild then run out of LDS with workgroup barriers between them instead of a round trip
// through memory per stage, and the results are written back at the end.
// Dynamic LDS: 44*stride + 4*parts*slots bytes; larger problems take the stand-alone kernels.
__global__ __launch_bounds__(kEpiThreads) void layer_epilogue_kernel(AttnArgs a, Plan p, PruneArgs pr) {
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    __shared__ SegTable tbl;
    __shared__ MassScratch ms;
    __shared__ int s_int[6];

    const int tid = threadIdx.x;
    const int stride = pr.stride;
    int64_t* l_tok = reinterpret_cast<int64_t*>(dyn_smem);
    unsigned char* scratch = dyn_smem + (size_t)8 * stride;            // 3*stride words for ranking / allocation
    float* l_score = reinterpret_cast<float*>(scratch + (size_t)12 * stride);
    int32_t* l_len = reinterpret_cast<int32_t*>(l_score + stride);
    int32_t* l_cand = l_len + stride;
    int32_t* l_keep = l_cand + stride;
    int32_t* l_start = l_keep + stride;
    int32_t* l_order = l_start + stride;
    float* l_part = reinterpret_cast<float*>(l_order + stride);

    const char* ws = static_cast<const char*>(a.workspace);
    const int b = __builtin_amdgcn_readfirstlane(blockIdx.x);
    const int64_t off = (int64_t)b * stride;
    const int nparts = p.units_per_b * p.nrb;
    const float* mp_b = reinterpret_cast<const float*>(ws + p.off_masspart) + (int64_t)b * nparts * p.slots;
    // The first batch of row loads and slot partials goes out before anything waits for the query's scalars.
    const bool row0 = tid < stride;
    int64_t r_tok = 0;
    int32_t r_len = 0, r_cand = 0, r_start = 0, r_order = 0;
    float r_score = 0.f, r_part = 0.f;
    if (row0) {
        r_tok = pr.doc_tok_offset[off + tid];
        r_len = pr.doc_len[off + tid];
        r_cand = pr.cand[off + tid];
        r_score = a.score_accum[off + tid];
        r_start = pr.new_start[off + tid];
        r_order = pr.order[off + tid];
    }
    if (tid < nparts * p.slots) r_part = mp_b[tid];
    const QueryHead qh = load_query_head(a, b, (int)threadIdx.x);
    const int n_cand = pr.n_cand[b];
    if (tid == 0) { s_int[4] = pr.q_start[b]; s_int[5] = pr.n_reuse[b]; }
    if (row0) {
        l_tok[tid] = r_tok; l_len[tid] = r_len; l_cand[tid] = r_cand; l_score[tid] = r_score; l_start[tid] = r_start;
        l_order[tid] = r_order;
    }
    for (int i = tid + kEpiThreads; i < stride; i += kEpiThreads) {
        l_tok[i] = pr.doc_tok_offset[off + i];
        l_len[i] = pr.doc_len[off + i];
        l_cand[i] = pr.cand[off + i];
        l_score[i] = a.score_accum[off + i];
        l_start[i] = pr.new_start[off + i];
        l_order[i] = pr.order[off + i];
    }
    if (tid < nparts * p.slots) l_part[tid] = r_part;
    for (int i = tid + kEpiThreads; i < nparts * p.slots; i += kEpiThreads) l_part[i] = mp_b[i];
    // With few candidates one wavefront finishes alone: the others leave, and the barriers of the stages
    // below (which only wait for wavefronts that are still running) cost nothing.
    const int nthr = n_cand <= 2 * kWave ? kWave : kEpiThreads;
    if (nthr == kWave && p.slots <= 2 * kWave && a.seg_stride <= kWave) {
        // small query: the first wavefront also does the masses, from a table in its registers
        __syncthreads();                             // publishes the rows above
        if (tid >= kWave) return;
        const RegSegTable rtbl = build_reg_table(a, qh, tid, p.tile);
        segment_masses_wave(p, rtbl, l_part, tid, [&](int s, float m) {
            a.mass[(int64_t)b * a.seg_stride + s] = m;
            const int doc = qh.seg.doc;              // this lane's entry
            if (doc >= 0 && doc < stride) atomicAdd(&l_score[doc], m);
        });
        __syncthreads();
    } else {
        build_table(a, qh, &tbl, p.tile);            // its barriers also publish the rows above
        segment_masses_block(p, tbl, l_part, nullptr, &ms, [&](int s, float m) {
            a.mass[(int64_t)b * a.seg_stride + s] = m;
            const int doc = tbl.doc[s];
            if (doc >= 0 && doc < stride) atomicAdd(&l_score[doc], m);
        });
        __syncthreads();
    }
    if (tid >= nthr) return;
    for (int i = tid; i < stride; i += nthr) a.score_accum[off + i] = l_score[i];
    int k = min(pr.keep, n_cand);
    bool done = false;
    if (n_cand <= kWave) {                               // the usual case: everything in one wavefront's registers
        SelectWaveArgs sw;
        sw.score = l_score; sw.len = l_len; sw.cand = l_cand; sw.tok = l_tok; sw.keep_idx = l_keep; sw.new_start = l_start;
        sw.order = l_order; sw.n = n_cand; sw.keep = pr.keep; sw.stride = stride; sw.normalise_by_len = pr.normalise_by_len;
        sw.strategy = pr.strategy; sw.force_n_reuse = pr.force_n_reuse; sw.pos_begin = pr.pos_begin; sw.pos_end = pr.pos_end;
        sw.prefix_len = pr.prefix_len; sw.doc_stored_start = pr.doc_stored_start; sw.q_stored_start = a.q_stored_start;
        sw.q_lo = qh.q0; sw.q_hi = qh.q0 + qh.tq_raw; sw.seg_stride = a.seg_stride;
        done = select_wave64(sw, pr.n_keep + b, &s_int[4], &s_int[5], pr.next_segs + (int64_t)b * a.seg_stride,
                             pr.next_n_seg + b);
        __builtin_amdgcn_wave_barrier();
    }
    if (!done) {
        k = prune_topk_block(l_score, pr.normalise_by_len ? l_len : nullptr, l_cand, n_cand, pr.keep, stride, l_keep,
                             a.dev_flag, scratch, &s_int[3], nthr);
        if (tid == 0) pr.n_keep[b] = k;
        __syncthreads();
        assign_positions_block(l_len, l_keep, k, stride, pr.pos_begin, pr.pos_end, pr.strategy, pr.force_n_reuse, l_start,
                               &s_int[4], &s_int[5], l_order, a.dev_flag, scratch, s_int, nthr);
        __syncthreads();
        gather_segments_block(l_tok, l_len, l_order, k, l_start, s_int[4], qh.q0, qh.q0 + qh.tq_raw, stride, pr.prefix_len,
                              pr.doc_stored_start, a.q_stored_start, pr.next_segs + (int64_t)b * a.seg_stride,
                              pr.next_n_seg + b, a.seg_stride, a.dev_flag, nthr);
    }
    for (int i = tid; i < stride; i += nthr) {
        if (i < k) pr.keep_idx[off + i] = l_keep[i];
        pr.new_start[off + i] = l_start[i];
        pr.order[off + i] = l_order[i];
    }
    if (tid == 0) { pr.q_start[b] = s_int[4]; pr.n_reuse[b] = s_int[5]; }
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
    const int phases = profile_phases();
    const Plan p = make_plan(a.n_q_heads, a.n_kv_heads, a.batch, a.max_tq, a.seg_stride, a.max_kv_tokens);
    const dim3 grid((unsigned)(p.x_count * p.n_rg)), block(kThreads);
    const dim3 grid2((unsigned)(p.units * p.nrb * 8)), grid3((unsigned)a.batch);
    const bool reg_table = a.seg_stride <= kWave;    // the attention kernels keep a table this small in registers
    // the attention kernel's launch carries the profiling aid's start/stop events (null when it is off)
    hipEvent_t ev_start = nullptr, ev_stop = nullptr;
    if (phases & 1) profile_kernel_pair(&ev_start, &ev_stop);
#define CF_LAUNCH_TIMED(KERNEL, BLOCK) hipExtLaunchKernelGGL(KERNEL, grid, BLOCK, 0, s, ev_start, ev_stop, 0, a, f, p)
#define CF_LAUNCH_DT(DT)                                                                                                       \
    if (!(phases & 1)) {                                                                                                       \
    } else if (p.producers == 0) {                                                                                             \
        if (reg_table) CF_LAUNCH_TIMED((attn_tile_kernel<DT, 1, 32, 2, true>), dim3(2 * kThreads));                            \
        else CF_LAUNCH_TIMED((attn_tile_kernel<DT, 1, 32, 2, false>), dim3(2 * kThreads));                                     \
    } else {                                                                                                                   \
        if (reg_table) CF_LAUNCH_TIMED((attn_pc_kernel<DT, kPcProducers, true>), dim3(kPcWaves * kWave));                      \
        else CF_LAUNCH_TIMED((attn_pc_kernel<DT, kPcProducers, false>), dim3(kPcWaves * kWave));                               \
    }                                                                                                                          \
    CF_HIP(hipGetLastError());                                                                                                 \
    if (phases & 2) hipLaunchKernelGGL((attn_combine_kernel<DT>), grid2, block, 0, s, a, p);
    if (a.dtype == CF_BF16) { CF_LAUNCH_DT(CF_BF16) } else { CF_LAUNCH_DT(CF_F16) }
#undef CF_LAUNCH_DT
#undef CF_LAUNCH_TIMED
    CF_HIP(hipGetLastError());
    if (prune) {
        PruneArgs pr;
        pr.enabled = 1; pr.keep = prune->keep; pr.strategy = prune->strategy; pr.force_n_reuse = prune->force_n_reuse;
        pr.normalise_by_len = prune->normalise_by_len; pr.stride = prune->stride; pr.pos_begin = prune->pos_begin;
        pr.pos_end = prune->pos_end; pr.prefix_len = prune->prefix_len; pr.doc_stored_start = prune->doc_stored_start;
        pr.doc_tok_offset = prune->doc_tok_offset; pr.doc_len = prune->doc_len; pr.cand = prune->cand;
        pr.n_cand = prune->n_cand; pr.keep_idx = prune->keep_idx; pr.n_keep = prune->n_keep;
        pr.new_start = prune->new_start; pr.q_start = prune->q_start; pr.n_reuse = prune->n_reuse;
        pr.order = prune->order; pr.next_segs = prune->next_segs; pr.next_n_seg = prune->next_n_seg;
        const size_t lds_rows = (size_t)44 * prune->stride + (size_t)4 * p.units_per_b * p.nrb * p.slots;
        if (!(phases & 4)) {
        } else if (lds_rows <= 60 * 1024) {          // every per-document row and the slot partials fit LDS
            hipLaunchKernelGGL(layer_epilogue_kernel, dim3(a.batch), dim3(kEpiThreads), lds_rows, s, a, p, pr);
        } else {
            hipLaunchKernelGGL(attn_mass_kernel, grid3, block, 0, s, a, p);
            CF_HIP(hipGetLastError());
            return launch_prune_step(a, prune, s);
        }
    } else if ((phases & 4) && a.mass != nullptr) {
        hipLaunchKernelGGL(attn_mass_kernel, grid3, block, 0, s, a, p);
    }
    CF_HIP(hipGetLastError());
    return CF_OK;
}

}  // namespace cf
