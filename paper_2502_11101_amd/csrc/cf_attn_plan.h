// Shared by the 16-bit attention kernels and the kernels that reduce their partial results: the launch plan
// (how rows, tokens and splits map to workgroups and where the partials live in the workspace), the per-query
// segment table in its two forms (LDS, registers) with the tile walk over it, and the MFMA wrappers.
#pragma once

#include "cf_common.h"
#include "cf_select_dev.h"

namespace cf {
namespace attn {

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
    int group;          // query heads per kv head
    int row_blocks;     // 16-row blocks of the stacked rows of one kv head
    int producers;      // 0: attn_tile_kernel (few rows); else attn_pipe_kernel with that many loading wavefronts
    int nrb;            // 64-row passes of a workgroup's rows (what the combine kernel handles at a time)
    int rows_wg;        // rows a workgroup has room for: 64 * nrb
    int n_rg;           // row groups per (query, kv head)
    int blocks_rg;      // 16-row blocks per row group
    int units_per_b, units, nsplit, slots, x_count;
    int tile;           // tokens per tile: 32 or 64
    int groups;         // groups of four wavefronts per workgroup (each streams its own run of tiles): 1 or 2
    int direct_out;     // one split: the attention kernel writes the output rows itself, nothing to merge
    size_t off_ml, off_opart, off_massml, off_masspart, total;
    size_t masspart_bytes;      // one layer's slot partials (the ledger holds kMaxPending + 1 such parts)
};

constexpr int kPcWaves = 8;         // wavefronts of an attn_pipe_kernel workgroup
constexpr int kPcProducers = 2;     // of which load and stage
constexpr int kPcNrb = 2;           // 16-row blocks per math wavefront

inline Plan make_plan(int n_q_heads, int n_kv_heads, int batch, int max_tq, int seg_stride, int64_t max_kv_tokens) {
    Plan p;
    const int group = n_q_heads / n_kv_heads;
    const int row_blocks = (group * max_tq + 15) / 16;
    p.group = group;
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
        // Many rows (GQA, long queries): 32-token units, two row blocks per math wavefront.
        const int blocks_wg = kPcNrb * (kPcWaves - kPcProducers);
        p.producers = kPcProducers;
        p.n_rg = (row_blocks + blocks_wg - 1) / blocks_wg;
        p.nrb = blocks_wg / 4;
        p.tile = 32;
        p.groups = 1;
    }
    p.blocks_rg = (row_blocks + p.n_rg - 1) / p.n_rg;
    p.rows_wg = 64 * p.nrb;
    p.units_per_b = n_kv_heads * p.n_rg;
    p.units = batch * p.units_per_b;
    const int64_t est_tiles = max_kv_tokens / p.tile + seg_stride;
    // One workgroup per CU and launch wave.  A CU holds one attn_pipe_kernel workgroup at a time, so there the
    // count stays within the 256 CUs; two of the small kernel's fit, and a few more than 256 do no harm.
    int64_t ns = p.producers ? 256 / p.units : (256 + p.units - 1) / p.units;
    const int64_t cap = est_tiles / (2 * p.groups) > 1 ? est_tiles / (2 * p.groups) : 1;
    if (ns > cap) ns = cap;
    if (ns > kMaxSplit) ns = kMaxSplit;
    if (ns < 1) ns = 1;
    p.nsplit = (int)ns;
    p.direct_out = p.nsplit == 1;
    p.slots = seg_stride + p.nsplit * p.groups;
    p.x_count = batch * n_kv_heads * p.nsplit;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
    p.off_ml = take((size_t)p.units * p.nsplit * p.rows_wg * sizeof(float2));
    p.off_opart = take(p.direct_out ? 0 : (size_t)p.units * p.nsplit * p.rows_wg * kD * sizeof(uint16_t));
    p.off_massml = take((size_t)p.units * p.slots * p.rows_wg * sizeof(float2));
    p.masspart_bytes = ((size_t)p.units * p.nrb * p.slots * sizeof(float) + 255) & ~(size_t)255;
    p.off_masspart = take(p.masspart_bytes * (kMaxPending + 1));
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
    int q0, tq_raw, n_seg, qdelta, q_new;
    int64_t q_total;
    cf_segment seg;
};

// `entry`: which table entry this thread takes (its index in the workgroup for the LDS table, its lane
// for the register table).
// kAlways: threads past the stride re-read the last entry instead of skipping the load — a conditional load makes
// the compiler wait for it inside the branch, before the scalar loads below are even issued (a whole round trip).
// (The producer/consumer attention kernel keeps the conditional form: it has no register to spare and runs long.)
template <bool kAlways = true>
__device__ __forceinline__ QueryHead load_query_head(const AttnArgs& a, int b, int entry) {   // b: wave-uniform
    QueryHead h;
    if constexpr (kAlways) {
        h.seg = a.segs[(int64_t)b * a.seg_stride + min(entry, a.seg_stride - 1)];   // seg_stride >= 1; callers test entry < n
    } else {
        if (entry < a.seg_stride) h.seg = a.segs[(int64_t)b * a.seg_stride + entry];   // seg_stride <= kMaxSegs
    }
    const int q0 = a.q_off[b], q1 = a.q_off[b + 1], qt = a.q_off[a.batch], n = a.n_seg[b], qn = a.q_new_start[b];
    asm volatile("" ::"s"(q0), "s"(q1), "s"(qt), "s"(n), "s"(qn));    // all five scalar loads are out before any is used
    h.q0 = q0;
    h.tq_raw = q1 - q0;
    h.q_total = qt;
    h.n_seg = n;
    h.qdelta = qn - a.q_stored_start;
    h.q_new = qn;
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
    // a query placed (or stored) outside the positional range attends nothing: every entry counts as empty
    const bool q_ok = positions_ok(h.q_new, tq, a.max_positions) && positions_ok(a.q_stored_start, tq, a.max_positions);
    if (!q_ok && tid == 0) raise_flag(a.dev_flag, CF_FLAG_POS_RANGE);
    if (tid < n) {
        const bool self = seg.kind == CF_SEG_SELF;
        const int64_t limit = self ? h.q_total : a.n_store_tokens;
        const bool bad = seg.kind < 0 || seg.kind > CF_SEG_SELF || seg.len < 0 || seg.tok_offset < 0 ||
                         seg.tok_offset + seg.len > limit || (self && a.k_self == nullptr);
        if (bad) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        const int len_vis = bad ? 0 : (self ? min(seg.len, tq) : seg.len);
        const bool off_range = !(positions_ok(seg.new_start, len_vis, a.max_positions) &&
                                 positions_ok(seg.stored_start, len_vis, a.max_positions));
        if (off_range && !bad) raise_flag(a.dev_flag, CF_FLAG_POS_RANGE);
        const int vis = off_range || !q_ok ? 0 : len_vis;
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
    // a query placed (or stored) outside the positional range attends nothing: every entry counts as empty
    const bool q_ok = positions_ok(h.q_new, tq, a.max_positions) && positions_ok(a.q_stored_start, tq, a.max_positions);
    if (!q_ok && lane == 0) raise_flag(a.dev_flag, CF_FLAG_POS_RANGE);
    int vis = 0;
    t.tok = 0; t.delta = 0; t.self = 0;
    if (lane < n) {
        const bool self = seg.kind == CF_SEG_SELF;
        const int64_t limit = self ? h.q_total : a.n_store_tokens;
        const bool bad = seg.kind < 0 || seg.kind > CF_SEG_SELF || seg.len < 0 || seg.tok_offset < 0 ||
                         seg.tok_offset + seg.len > limit || (self && a.k_self == nullptr);
        if (bad) raise_flag(a.dev_flag, CF_FLAG_BAD_SEGMENT);
        const int len_vis = bad ? 0 : (self ? min(seg.len, tq) : seg.len);
        const bool off_range = !(positions_ok(seg.new_start, len_vis, a.max_positions) &&
                                 positions_ok(seg.stored_start, len_vis, a.max_positions));
        if (off_range && !bad) raise_flag(a.dev_flag, CF_FLAG_POS_RANGE);
        vis = off_range || !q_ok ? 0 : len_vis;
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
    // (the values are the same in every lane; taking them from the first one tells the compiler so, which keeps
    // everything derived from them — tile descriptions, base addresses — on the scalar unit)
    FoundSegment f;
    f.seg = s;
    f.first = __builtin_amdgcn_readfirstlane(tbl.tile0[s]);
    f.end = __builtin_amdgcn_readfirstlane(tbl.tile0[s + 1]);
    f.vis = __builtin_amdgcn_readfirstlane(tbl.vis[s]);
    f.delta = __builtin_amdgcn_readfirstlane(tbl.delta[s]);
    f.self = __builtin_amdgcn_readfirstlane(tbl.self[s]);
    const int64_t tok = tbl.tok[s];
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)tok);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)tok >> 32));
    f.tok = (int64_t)(((uint64_t)hi << 32) | lo);
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

}  // namespace attn

// The kernels that follow the attention kernel of a call (defined with them; `a.dtype` selects the instance).
void launch_combine(const AttnArgs& a, const attn::Plan& p, bool take_pending, hipStream_t s);
bool pending_fit_combine(const AttnArgs& a, const attn::Plan& p);
void launch_mass(const AttnArgs& a, const attn::Plan& p, hipStream_t s);
// S += the masses of the layers whose scores are pending in the ledger (not the current call's): ahead of the fused epilogue
void launch_pending_masses(const AttnArgs& a, const attn::Plan& p, hipStream_t s);
// The fused epilogue keeps every per-document row and the slot partials of a query in LDS: whether they fit.
bool epilogue_fits(const attn::Plan& p, const cf_prune_step* prune);
void launch_epilogue(const AttnArgs& a, const attn::Plan& p, const cf_prune_step* prune, hipStream_t s);

}  // namespace cf
