// What follows the attention kernel of a call on the 16-bit path: the merge of the splits' partial outputs
// (with the slot partial masses as a by-product), the per-segment mass reduction, and the fused layer epilogue
// (masses, S += mass, ranking, allocation, next segment table).
#include "cf_attn_plan.h"

namespace cf {
using namespace attn;
namespace {

// Second kernel: one workgroup per (unit = (query, kv head, row group), 64-row pass, eighth of the output channels) merges the
// splits' partial outputs and writes its output rows; the eight workgroups of a (unit, pass) also share
// the reduction, over the pass's 64 rows, of every (segment, split) slot's (max, sum) pairs to
// sum * exp2(max - row max) / row sum, which the mass kernel then only has to add up.
__device__ __forceinline__ void pending_masses_block(const AttnArgs& a, const Plan& p, int b, int n_parts, int write_mass,
                                                     float (*m_all)[kWave]);

// With take_pending the grid has one more row of workgroups (the last blockIdx.y); the first of them, per query, takes
// the ledger's pending score parts in beside the merge (pending_masses_block), the others leave at once.
template <int DT>
__global__ __launch_bounds__(kThreads) void attn_combine_kernel(AttnArgs a, Plan p, int take_pending) {
    __shared__ float2 mlw[kMaxSplit * 64];       // (m, l) per split and row, then the split's weight l * exp2(m - row maximum) in .x
    static_assert(sizeof(float2) * kMaxSplit * 64 >= sizeof(float) * (kMaxPending + 1) * kWave, "the parts' masses reuse mlw");
    const int units_y = (int)gridDim.y - take_pending;
    if (take_pending && (int)blockIdx.y == units_y) {
        if (blockIdx.x == 0)
            pending_masses_block(a, p, __builtin_amdgcn_readfirstlane(blockIdx.z), a.n_pending, 0, reinterpret_cast<float (*)[kWave]>(mlw));
        return;
    }
    __shared__ float part_stat[kWaves][64], part_sum[kWaves][64];   // per wavefront: its splits' maximum and sum, per row
    constexpr int kPre = 8;                      // splits whose partial outputs are fetched before the statistics are ready

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int li = lane & 15, lg = lane >> 4;
    char* ws = static_cast<char*>(a.workspace);
    // grid (channel block + 8 * pass — or just the pass when there is nothing to merge —, kv head * row groups + row group, query)
    const int hq = a.n_q_heads, group = p.group;
    const int x_shift = p.direct_out ? 0 : 3;        // nothing to merge: one workgroup per (unit, pass) reduces every slot
    const int dbq = blockIdx.x & ((1 << x_shift) - 1);
    const int pass = (int)(blockIdx.x >> x_shift);
    const int b = blockIdx.z;
    const int hkv = p.n_rg == 1 ? (int)blockIdx.y : (int)div_exact(blockIdx.y, (unsigned)p.n_rg);
    const int rg = (int)blockIdx.y - hkv * p.n_rg;
    const int unit = b * units_y + (int)blockIdx.y;
    const int q0 = a.q_off[b], q1 = a.q_off[b + 1];
    const float2* ml = reinterpret_cast<const float2*>(ws + p.off_ml) + (int64_t)unit * p.nsplit * p.rows_wg + pass * 64;
    const uint2* opart = reinterpret_cast<const uint2*>(ws + p.off_opart) + (int64_t)unit * p.nsplit * p.rows_wg * (kD / 4);
    const int blk = pass * kWaves + wave;                      // row block inside the workgroup tile
    const uint2* src = opart + ((int64_t)blk * 8 + dbq) * kWave + lane;
    auto widen = [](uint2 w) { return f32x4{Mma<DT>::lo(w.x), Mma<DT>::hi(w.x), Mma<DT>::lo(w.y), Mma<DT>::hi(w.y)}; };
    const int64_t split_stride = (int64_t)p.rows_wg / 16 * 8 * kWave;
    const float2* massml = reinterpret_cast<const float2*>(ws + p.off_massml) + (int64_t)unit * p.slots * p.rows_wg + pass * 64 + lane;
    const int k_first = dbq * kWaves + wave, k_step = kWaves << x_shift;
    constexpr int kSv = 8;                           // slot statistics fetched up front per wavefront

    // Everything this workgroup reads is requested up front — row statistics, partial outputs of the first splits,
    // the first slot statistics — so the round trips to memory overlap.  Every load is unconditional (a clamped,
    // in-bounds address; what lies past the end is dropped afterwards): a load inside a branch makes the compiler
    // wait for it before the branch ends, which would put the round trips one behind the other.
    // (A wavefront whose 16 rows are all padding reads what an earlier call left there: never stored; not waiting for
    // the query's length here saves a round trip.  With one split the attention kernel wrote the output rows itself:
    // nothing to merge, the partial outputs' area does not exist and a harmless address is read instead.)
    const bool merge = !p.direct_out;
    constexpr int kMl = kMaxSplit * 64 / kThreads;   // (m, l) pairs per thread
    const int n_ml = p.nsplit * 64;
    float2 ml_regs[kMl];
#pragma unroll
    for (int i = 0; i < kMl; ++i) {
        const int idx = min(tid + i * kThreads, n_ml - 1);
        ml_regs[i] = ml[(idx >> 6) * p.rows_wg + (idx & 63)];
    }
    const uint2* src_safe = merge ? src : reinterpret_cast<const uint2*>(ws + p.off_ml) + (lane & 31);
    const int64_t stride_safe = merge ? split_stride : 0;
    uint2 pre[kPre];
#pragma unroll
    for (int s = 0; s < kPre; ++s) pre[s] = src_safe[min(s, p.nsplit - 1) * stride_safe];
    float2 sv[kSv];
#pragma unroll
    for (int j = 0; j < kSv; ++j) sv[j] = massml[(int64_t)min(k_first + j * k_step, p.slots - 1) * p.rows_wg];
#pragma unroll
    for (int i = 0; i < kMl; ++i)
        if (tid + i * kThreads < n_ml) mlw[tid + i * kThreads] = ml_regs[i];
    const int tq = min(q1 - q0, a.max_tq);
    const int n_rows = group * tq;
    const int row_base = rg * p.blocks_rg * 16;
    const int rows_here = min(p.blocks_rg * 16, n_rows - row_base);
    const bool blk_has_rows = pass * 64 + wave * 16 < rows_here;
    __syncthreads();
    // Row statistics by the whole workgroup: wavefront w takes the splits w, w + 4, ... of every row, the four
    // partial maxima and then the four partial sums (added in a fixed order) meet in LDS.  A split's weight stays
    // unnormalised in LDS; the rows are divided by their sum once at the end.
    {
        float m = -INFINITY;
        for (int s = wave; s < p.nsplit; s += kWaves) m = fmaxf(m, mlw[s * 64 + lane].x);
        part_stat[wave][lane] = m;
    }
    __syncthreads();
    auto row_max = [&](int row) {
        const float m = fmaxf(fmaxf(part_stat[0][row], part_stat[1][row]), fmaxf(part_stat[2][row], part_stat[3][row]));
        return m == -INFINITY ? 0.f : m;
    };
    {
        const float ms = row_max(lane);
        float z = 0.f;
        for (int s = wave; s < p.nsplit; s += kWaves) {
            const float2 v = mlw[s * 64 + lane];
            const float e = exp2f(v.x - ms);
            z += v.y * e;
            mlw[s * 64 + lane].x = v.y * e;          // the split's rows arrive divided by their own sum
        }
        part_sum[wave][lane] = z;
    }
    __syncthreads();
    auto row_inv_sum = [&](int row) {
        const float z = ((part_sum[0][row] + part_sum[1][row]) + part_sum[2][row]) + part_sum[3][row];
        return z > 0.f ? 1.f / z : 0.f;
    };
    f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < kPre; ++s)
        if (s < p.nsplit) o += widen(pre[s]) * mlw[s * 64 + wave * 16 + li].x;
    if (merge && blk_has_rows)
        for (int s0 = kPre; s0 < p.nsplit; s0 += kPre) {         // further splits, eight loads at a time
            uint2 more[kPre];
#pragma unroll
            for (int i = 0; i < kPre; ++i) more[i] = src[min(s0 + i, p.nsplit - 1) * split_stride];      // unconditional, as above
#pragma unroll
            for (int i = 0; i < kPre; ++i)
                if (s0 + i < p.nsplit) o += widen(more[i]) * mlw[(s0 + i) * 64 + wave * 16 + li].x;
        }
    const int lrow = pass * 64 + wave * 16 + li;
    o *= row_inv_sum(wave * 16 + li);
    if (merge && lrow < rows_here) {
        const int m2 = row_base + lrow;
        const int gi = (int)div_exact((unsigned)m2, (unsigned)tq), t = m2 - gi * tq;
        uint16_t* op = static_cast<uint16_t*>(a.out) + (((int64_t)q0 + t) * hq + hkv * group + gi) * kD + 16 * dbq + 4 * lg;
        uint2 pk;
        pk.x = Mma<DT>::pack(o[0], o[1]);
        pk.y = Mma<DT>::pack(o[2], o[3]);
        *reinterpret_cast<uint2*>(op) = pk;
    }
    // slot partials: slot k = segment + split; slots no split wrote this call hold stale pairs and
    // give meaningless numbers that the mass kernel never reads
    if (a.mass != nullptr) {
        float* masspart = reinterpret_cast<float*>(ws + p.off_masspart + (size_t)a.n_pending * p.masspart_bytes) + ((int64_t)unit * p.nrb + pass) * p.slots;
        const float2 st = make_float2(row_max(lane), pass * 64 + lane < rows_here ? row_inv_sum(lane) : 0.f);   // padding rows carry no mass
        auto reduce = [&](int k, float2 v) {
            const float c = wave_sum_dpp(st.y > 0.f ? v.y * exp2f(v.x - st.x) * st.y : 0.f);
            if (lane == 0 && k < p.slots) masspart[k] = c;
        };
#pragma unroll
        for (int j = 0; j < kSv; ++j)
            if (k_first + j * k_step < p.slots) reduce(k_first + j * k_step, sv[j]);
        for (int k = k_first + kSv * k_step; k < p.slots; k += k_step) reduce(k, massml[(int64_t)k * p.rows_wg]);
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
    float seg_mass[kMaxSegs];               // every entry's mass, for the per-document sums
};

// S += s^l (Alg. 2) without atomics, so that the sum does not depend on timing when a document slot is fed by
// several table entries: the first entry of a slot adds up the masses of all entries of that slot in table
// order and is the only one that touches the slot's score.
// Block form: `doc` and `seg_mass` of the n entries in LDS; `score` has `stride` slots (LDS or memory).
__device__ __forceinline__ void add_doc_scores_block(const int32_t* doc, const float* seg_mass, int n, float* score, int stride) {
    for (int s = threadIdx.x; s < n; s += blockDim.x) {
        const int d = doc[s];
        if (d < 0 || d >= stride) continue;
        bool first = true;
        float sum = seg_mass[s];
        for (int j = 0; j < n; ++j) {
            if (doc[j] != d) continue;
            if (j < s) first = false;
            else if (j > s) sum += seg_mass[j];
        }
        if (first) score[d] += sum;
    }
}
// Bitwise OR over the 64 lanes of a wavefront, handed to every lane (DPP row shifts, then the two row broadcasts).
__device__ __forceinline__ uint32_t wave_or_u32(uint32_t x) {
    int v = (int)x;
    v |= __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v |= __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v |= __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v |= __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v |= __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v |= __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane(v, 63);
}
// Wavefront form: lane s < n holds entry s's slot and mass.  With at most 64 document slots a bit mask tells whether
// every slot is fed by one entry only — the usual table — and then every entry adds its own mass (the same single
// addend as below); otherwise the loop runs once per table entry.
__device__ __forceinline__ void add_doc_scores_wave(int doc, float m, int n, int lane, float* score, int stride) {
    const bool valid = lane < n && doc >= 0 && doc < stride;
    const int d = valid ? doc : -1;
    if (stride <= kWave) {
        const unsigned long long bit = valid ? 1ull << d : 0ull;
        const int slots_fed = __builtin_popcount(wave_or_u32((uint32_t)bit)) + __builtin_popcount(wave_or_u32((uint32_t)(bit >> 32)));
        if (slots_fed == __builtin_popcountll(__ballot(valid))) {
            if (valid) score[d] += m;
            return;
        }
    }
    bool first = valid;
    float sum = m;
    for (int j = 0; j < n; ++j) {
        const int dj = __builtin_amdgcn_readlane(d, j);
        const float mj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, m), j));
        if (dj == d) {
            if (j < lane) first = false;
            else if (j > lane) sum += mj;
        }
    }
    if (first) score[d] += sum;
}
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
            const int g = (int)div_exact((unsigned)idx, (unsigned)p.slots), k = idx - g * p.slots;
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
// Returns lane s's segment mass (0 for lanes past the table).
// BATCHED: a column of at most 40 parts is requested in one batch (clamped, unconditional loads) before the first
// add, instead of a round trip — to memory or to LDS — per group of eight.
template <bool BATCHED = false>
__device__ __forceinline__ float segment_masses_wave(const Plan& p, const RegSegTable& t, const float* parts, int lane) {
    const unsigned total = (unsigned)t.total;
    const unsigned nsub = (unsigned)(p.nsplit * p.groups);
    const int nparts = p.units_per_b * p.nrb;
    constexpr int kGroup = 8;
    float c[2] = {0.f, 0.f};                         // columns lane, lane + 64
    int first_looped = 0;
    if constexpr (BATCHED) {
        constexpr int kBatch = 40;
        if (nparts <= kBatch) {
            float v[kBatch];
            const float* col = parts + min(lane, p.slots - 1);
#pragma unroll
            for (int i = 0; i < kBatch; ++i) v[i] = col[min(i, nparts - 1) * p.slots];
            if (lane < p.slots) {
#pragma unroll
                for (int g0 = 0; g0 < kBatch; g0 += kGroup) {
                    float gs = 0.f;                  // the same sums in the same order as group_sum
#pragma unroll
                    for (int i = 0; i < kGroup; ++i)
                        if (g0 + i < nparts) gs += v[g0 + i];
                    if (g0 < nparts) c[0] += gs;
                }
            }
            first_looped = 1;
        }
    }
    for (int j = first_looped; j < 2; ++j)
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
    return lane < t.n ? m : 0.f;
}

// Third kernel: per-segment attention mass, one workgroup per query; then S += mass.
// Takes parts 0 .. n_parts - 1 of the ledger in order; the last one's masses go to `mass` when `write_mass` is set
// (it is not when only layers that deferred their scores are taken in, ahead of the fused epilogue).
__global__ __launch_bounds__(kThreads) void attn_mass_kernel(AttnArgs a, Plan p, int n_parts, int write_mass) {
    __shared__ SegTable tbl;
    __shared__ MassScratch ms;
    __shared__ float stage[kMassStage];
    const char* ws = static_cast<const char*>(a.workspace);
    const int b = __builtin_amdgcn_readfirstlane(blockIdx.x);
    const int tid = threadIdx.x;
    const int n_part_floats = p.units_per_b * p.nrb * p.slots;
    // part j of the ledger: the slot partials of the j-th layer still pending (the last one is this call's)
    auto part = [&](int j) { return reinterpret_cast<const float*>(ws + p.off_masspart + (size_t)j * p.masspart_bytes) + (int64_t)b * n_part_floats; };
    if (p.slots <= 2 * kWave && a.seg_stride <= kWave && n_part_floats <= kMassStage) {
        // small query: the partials go to LDS in one batch (requested before the query's scalars are waited for),
        // then one wavefront finishes alone from a table in its registers — the same sums in the same order
        float r_part[kMassStage / kThreads];
        const float* mp0 = part(0);
#pragma unroll
        for (int i = 0; i < kMassStage / kThreads; ++i) r_part[i] = mp0[min(tid + i * kThreads, n_part_floats - 1)];   // unconditional
        const QueryHead qh = load_query_head(a, b, tid & (kWave - 1));
#pragma unroll
        for (int i = 0; i < kMassStage / kThreads; ++i)
            if (tid + i * kThreads < n_part_floats) stage[tid + i * kThreads] = r_part[i];
        __syncthreads();
        if (n_parts == 1 && tid >= kWave) return;    // the other wavefronts only help to fetch further parts
        const RegSegTable rtbl = build_reg_table(a, qh, tid & (kWave - 1), p.tile);
        for (int j = 0; j < n_parts; ++j) {
            if (j > 0) {
                __syncthreads();                     // the staged part has been read
                const float* mp = part(j);
                for (int i = tid; i < n_part_floats; i += kThreads) stage[i] = mp[i];
                __syncthreads();
            }
            if (tid < kWave) {
                const float m = segment_masses_wave(p, rtbl, stage, tid);
                if (write_mass && j == n_parts - 1 && tid < rtbl.n) a.mass[(int64_t)b * a.seg_stride + tid] = m;
                if (a.score_accum)                   // qh.seg is this lane's entry
                    add_doc_scores_wave(qh.seg.doc, m, rtbl.n, tid, a.score_accum + (int64_t)b * a.score_stride, a.score_stride);
            }
        }
        return;
    }
    const QueryHead qh = load_query_head(a, b, (int)threadIdx.x);
    build_table(a, qh, &tbl, p.tile);
    for (int j = 0; j < n_parts; ++j) {
        const bool last = write_mass && j == n_parts - 1;
        segment_masses_block(p, tbl, const_cast<float*>(part(j)), stage, &ms, [&](int s, float m) {
            if (last) a.mass[(int64_t)b * a.seg_stride + s] = m;
            ms.seg_mass[s] = m;
        });
        if (a.score_accum == nullptr) continue;
        __syncthreads();
        add_doc_scores_block(tbl.doc, ms.seg_mass, tbl.n, a.score_accum + (int64_t)b * a.score_stride, a.score_stride);
        __syncthreads();
    }
}

// The same for a small query with several parts to take in (layers that deferred their scores): one wavefront per
// part works out that layer's masses straight from the ledger, all parts at once; the first wavefront then adds them
// to the scores part by part — S += s^l in layer order, each document slot by the lane of its first table entry, so
// the sums are those of the one-part-after-the-other form above, bit for bit.  Any whole number of wavefronts per block;
// with fewer wavefronts than parts a wavefront takes several parts, one after the other.
__device__ __forceinline__ void pending_masses_block(const AttnArgs& a, const Plan& p, int b, int n_parts, int write_mass,
                                                     float (*m_all)[kWave]) {
    const char* ws = static_cast<const char*>(a.workspace);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
    const int n_waves = (int)blockDim.x / kWave;
    const int n_part_floats = p.units_per_b * p.nrb * p.slots;
    const QueryHead qh = load_query_head(a, b, lane);
    const RegSegTable rtbl = build_reg_table(a, qh, lane, p.tile);
    for (int part = wave; part < n_parts; part += n_waves) {
        const float* mp = reinterpret_cast<const float*>(ws + p.off_masspart + (size_t)part * p.masspart_bytes) + (int64_t)b * n_part_floats;
        const float m = segment_masses_wave<true>(p, rtbl, mp, lane);
        m_all[part][lane] = m;
        if (write_mass && part == n_parts - 1 && lane < rtbl.n) a.mass[(int64_t)b * a.seg_stride + lane] = m;
    }
    __syncthreads();
    if (wave != 0 || a.score_accum == nullptr) return;
    // which entries feed this lane's document slot, and whether this lane is the slot's first entry: as in
    // add_doc_scores_wave, with the table walked once for all parts
    const int doc = qh.seg.doc;
    const bool valid = lane < rtbl.n && doc >= 0 && doc < a.score_stride;
    const int d = valid ? doc : -1;
    bool first = valid;
    unsigned long long later = 0;                    // entries after this one that feed the same slot
    for (int j = 0; j < rtbl.n; ++j) {
        const int dj = __builtin_amdgcn_readlane(d, j);
        if (dj == d) {
            if (j < lane) first = false;
            else if (j > lane) later |= 1ull << j;
        }
    }
    if (!first) return;
    float* slot = a.score_accum + (int64_t)b * a.score_stride + d;
    float s = *slot;
    for (int part = 0; part < n_parts; ++part) {
        float sum = m_all[part][lane];
        for (unsigned long long rest = later; rest; rest &= rest - 1) sum += m_all[part][__builtin_ctzll(rest)];
        s += sum;
    }
    *slot = s;
}

__global__ __launch_bounds__(kWave * (kMaxPending + 1)) void pending_masses_kernel(AttnArgs a, Plan p, int n_parts, int write_mass) {
    __shared__ float m_all[kMaxPending + 1][kWave];
    pending_masses_block(a, p, __builtin_amdgcn_readfirstlane(blockIdx.x), n_parts, write_mass, m_all);
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
    __shared__ uint4 s_bcast[kWave];

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
    // this call's own slot partials are part n_pending of the ledger (earlier parts, of layers that deferred their
    // scores, have been taken in by the mass kernel before this one)
    const float* mp_b = reinterpret_cast<const float*>(ws + p.off_masspart + (size_t)a.n_pending * p.masspart_bytes) + (int64_t)b * nparts * p.slots;
    // The first batch of row loads, the slot partials and the query's scalars all go out before anything is waited
    // for; every load is unconditional (a clamped, in-bounds index: threads past the end re-read the last element and
    // drop it), since a load inside a branch is waited for before the branch ends.
    const bool row0 = tid < stride;
    const int row_i = min(tid, stride - 1);
    const int64_t r_tok = pr.doc_tok_offset[off + row_i];
    const int32_t r_len = pr.doc_len[off + row_i], r_cand = pr.cand[off + row_i];
    const float r_score = a.score_accum[off + row_i];
    const int32_t r_start = pr.new_start[off + row_i], r_order = pr.order[off + row_i];
    constexpr int kPartRegs = 4;                     // slot partials per thread fetched with the first batch
    const int n_part_floats = nparts * p.slots;
    float r_part[kPartRegs];
#pragma unroll
    for (int i = 0; i < kPartRegs; ++i) r_part[i] = mp_b[min(tid + i * kEpiThreads, n_part_floats - 1)];
    const int n_cand = pr.n_cand[b];
    const int r_q_start = pr.q_start[b], r_n_reuse = pr.n_reuse[b];
    const QueryHead qh = load_query_head(a, b, (int)threadIdx.x);
    if (tid == 0) { s_int[4] = r_q_start; s_int[5] = r_n_reuse; }
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
    // With few candidates one wavefront finishes alone: the others leave, and the barriers of the stages
    // below (which only wait for wavefronts that are still running) cost nothing.
    const int nthr = n_cand <= 2 * kWave ? kWave : kEpiThreads;
    const bool small = nthr == kWave && p.slots <= 2 * kWave && a.seg_stride <= kWave;
#pragma unroll
    for (int i = 0; i < kPartRegs; ++i)
        if (tid + i * kEpiThreads < n_part_floats) l_part[tid + i * kEpiThreads] = r_part[i];
    for (int i = tid + kPartRegs * kEpiThreads; i < n_part_floats; i += kEpiThreads) l_part[i] = mp_b[i];
    if (small) {
        // small query: the first wavefront also does the masses, from a table in its registers
        __syncthreads();                             // publishes the rows above
        if (tid >= kWave) return;
        const RegSegTable rtbl = build_reg_table(a, qh, tid, p.tile);
        const float m = segment_masses_wave(p, rtbl, l_part, tid);
        if (tid < rtbl.n) a.mass[(int64_t)b * a.seg_stride + tid] = m;
        add_doc_scores_wave(qh.seg.doc, m, rtbl.n, tid, l_score, stride);       // qh.seg is this lane's entry
        __syncthreads();
    } else {
        build_table(a, qh, &tbl, p.tile);            // its barriers also publish the rows above
        segment_masses_block(p, tbl, l_part, nullptr, &ms, [&](int s, float m) {
            a.mass[(int64_t)b * a.seg_stride + s] = m;
            ms.seg_mass[s] = m;
        });
        __syncthreads();
        add_doc_scores_block(tbl.doc, ms.seg_mass, tbl.n, l_score, stride);
        __syncthreads();
    }
    if (tid >= nthr) return;
    for (int i = tid; i < stride; i += nthr) a.score_accum[off + i] = l_score[i];
    int k = min(pr.keep, n_cand);
    bool done = false;
    if (n_cand <= kWave) {                               // the usual case: everything in one wavefront's registers
        SelectWaveArgs sw;
        sw.score = l_score; sw.len = l_len; sw.cand = l_cand; sw.tok = l_tok; sw.keep_idx = l_keep; sw.new_start = l_start;
        sw.order = l_order; sw.bcast = s_bcast; sw.n = n_cand; sw.keep = pr.keep; sw.stride = stride; sw.normalise_by_len = pr.normalise_by_len;
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

bool pending_fit_combine(const AttnArgs& a, const Plan& p) { return p.slots <= 2 * kWave && a.seg_stride <= kWave; }

void launch_combine(const AttnArgs& a, const Plan& p, bool take_pending, hipStream_t s) {
    const int extra = take_pending ? 1 : 0;
    const dim3 grid((unsigned)((p.direct_out ? 1 : 8) * p.nrb), (unsigned)(a.n_kv_heads * p.n_rg + extra), (unsigned)a.batch), block(kThreads);
    if (a.dtype == CF_BF16) hipLaunchKernelGGL((attn_combine_kernel<CF_BF16>), grid, block, 0, s, a, p, extra);
    else hipLaunchKernelGGL((attn_combine_kernel<CF_F16>), grid, block, 0, s, a, p, extra);
}

// several parts of a small query: one wavefront per part (see pending_masses_kernel); else one part after the other
static void launch_masses(const AttnArgs& a, const Plan& p, int n_parts, int write_mass, hipStream_t s) {
    if (n_parts > 1 && pending_fit_combine(a, p))
        hipLaunchKernelGGL(pending_masses_kernel, dim3((unsigned)a.batch), dim3(kWave * n_parts), 0, s, a, p, n_parts, write_mass);
    else
        hipLaunchKernelGGL(attn_mass_kernel, dim3((unsigned)a.batch), dim3(kThreads), 0, s, a, p, n_parts, write_mass);
}

void launch_mass(const AttnArgs& a, const Plan& p, hipStream_t s) { launch_masses(a, p, a.n_pending + 1, 1, s); }

void launch_pending_masses(const AttnArgs& a, const Plan& p, hipStream_t s) { launch_masses(a, p, a.n_pending, 0, s); }

static size_t epilogue_lds_bytes(const Plan& p, const cf_prune_step* prune) {
    return (size_t)44 * prune->stride + (size_t)4 * p.units_per_b * p.nrb * p.slots;
}

bool epilogue_fits(const Plan& p, const cf_prune_step* prune) { return epilogue_lds_bytes(p, prune) <= 60 * 1024; }

void launch_epilogue(const AttnArgs& a, const Plan& p, const cf_prune_step* prune, hipStream_t s) {
    PruneArgs pr;
    pr.enabled = 1; pr.keep = prune->keep; pr.strategy = prune->strategy; pr.force_n_reuse = prune->force_n_reuse;
    pr.normalise_by_len = prune->normalise_by_len; pr.stride = prune->stride; pr.pos_begin = prune->pos_begin;
    pr.pos_end = prune->pos_end; pr.prefix_len = prune->prefix_len; pr.doc_stored_start = prune->doc_stored_start;
    pr.doc_tok_offset = prune->doc_tok_offset; pr.doc_len = prune->doc_len; pr.cand = prune->cand;
    pr.n_cand = prune->n_cand; pr.keep_idx = prune->keep_idx; pr.n_keep = prune->n_keep;
    pr.new_start = prune->new_start; pr.q_start = prune->q_start; pr.n_reuse = prune->n_reuse;
    pr.order = prune->order; pr.next_segs = prune->next_segs; pr.next_n_seg = prune->next_n_seg;
    hipLaunchKernelGGL(layer_epilogue_kernel, dim3(a.batch), dim3(kEpiThreads), epilogue_lds_bytes(p, prune), s, a, p, pr);
}

}  // namespace cf
