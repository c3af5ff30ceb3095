// Internal helpers shared by the HIP translation units of libcachefocus (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <type_traits>
#include <stdint.h>

#include "cachefocus.h"

namespace cf {

constexpr int kWave = 64;

// a / b for unsigned a and b >= 1, exactly: below 2^21 through the float reciprocal and two corrections
// (the estimate is off by less than one), else the long way.  A fraction of the instructions of the compiler's
// general 32-bit division, which the short latency-bound kernels here would otherwise run several times.
__device__ __forceinline__ unsigned div_exact(unsigned a, unsigned b) {
    if (a >= (1u << 21) || b >= (1u << 21)) return a / b;
    int q = (int)((float)a * __builtin_amdgcn_rcpf((float)b));
    int r = (int)a - q * (int)b;
    if (r < 0) { --q; r += (int)b; }
    if (r >= (int)b) ++q;
    return (unsigned)q;
}
constexpr int kMaxHeadDim = 256;
constexpr int kMaxHalf = kMaxHeadDim / 2;

// theta_m / (2 pi) in double for every 2-D slice m (Eq. 2 with the RoPE schedule
// theta_m = base^(-2m/d)); computed on the host, passed to kernels by value.
struct RopeFreq {
    double rev[kMaxHalf];
};

void set_error(const char* fmt, ...);
// the start/stop events of the attention kernel's next launch while cf_profile_kernel_events is on (else both null)
void profile_kernel_pair(hipEvent_t* start, hipEvent_t* stop);
cf_status check_desc(const cf_layer_desc* d);
void fill_rope_freq(const cf_layer_desc* d, RopeFreq* f);
size_t elem_size(int32_t dtype);

#define CF_REQUIRE(cond, status, ...)      \
    do {                                   \
        if (!(cond)) {                     \
            ::cf::set_error(__VA_ARGS__);  \
            return (status);               \
        }                                  \
    } while (0)

#define CF_HIP(call)                                                                  \
    do {                                                                              \
        hipError_t e_ = (call);                                                       \
        if (e_ != hipSuccess) {                                                       \
            ::cf::set_error("%s failed: %s", #call, hipGetErrorString(e_));           \
            return CF_ERR_DEVICE;                                                     \
        }                                                                             \
    } while (0)

// ---------------------------------------------------------------------------------- device side
// cos/sin of delta * theta_m.  The product is formed in fp64 in units of revolutions and
// reduced to [-0.5, 0.5] there, so |delta| up to 2^31 loses nothing; the reduced angle goes
// through the fp32 sincospi.  delta = 0 gives exactly (1, 0).
__device__ __forceinline__ float2 rope_cos_sin(int delta, double theta_rev) {
    double x = (double)delta * theta_rev;
    double fr = x - rint(x);
    float s, c;
    sincospif(2.0f * (float)fr, &s, &c);
    return make_float2(c, s);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even float -> bf16 bits (NaN stays NaN)
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ float f16_bits_to_float(uint32_t b) {
    union { uint16_t u; _Float16 h; } x;
    x.u = (uint16_t)b;
    return (float)x.h;
}

__device__ __forceinline__ uint32_t float_to_f16_bits(float f) {
    union { uint16_t u; _Float16 h; } x;
    x.h = (_Float16)f;   // v_cvt_f16_f32, round to nearest even
    return x.u;
}

template <int DT> struct Elem;
template <> struct Elem<CF_F32> {
    using type = float;
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<CF_BF16> {
    using type = uint16_t;
    static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = (uint16_t)float_to_bf16_bits(v); }
};
template <> struct Elem<CF_F16> {
    using type = uint16_t;
    static __device__ __forceinline__ float load(const uint16_t* p) { return f16_bits_to_float(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = (uint16_t)float_to_f16_bits(v); }
};

__device__ __forceinline__ void raise_flag(int32_t* dev_flag, int bits) {
    if (dev_flag) atomicOr(dev_flag, bits);
}

// whether `len` tokens starting at position `start` all sit inside [0, max_positions)
__device__ __forceinline__ bool positions_ok(int start, int len, int max_positions) {
    return start >= 0 && (int64_t)start + len <= (int64_t)max_positions;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
// the sum over the 64 lanes, in registers (DPP row shifts and row broadcasts; a fixed order of its own), in every lane
__device__ __forceinline__ float wave_sum_dpp(float v) {
    auto step = [](float x, auto ctrl, auto rows) {
        return x + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, decltype(rows)::value, 0xf, false));
    };
    v = step(v, std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xf>{});   // row_shr:1
    v = step(v, std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xf>{});   // row_shr:2
    v = step(v, std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xf>{});   // row_shr:4
    v = step(v, std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xf>{});   // row_shr:8
    v = step(v, std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});   // row_bcast:15 into rows 1 and 3
    v = step(v, std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xc>{});   // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// ---------------------------------------------------------------------------------- launchers
struct AssembleArgs {
    const void *k_store, *v_store, *k_self, *v_self;
    void *k_final, *v_final;
    const int32_t* q_off;
    const cf_segment* segs;
    const int32_t* n_seg;
    const int64_t* final_off;
    int32_t *final_len, *final_pos, *dev_flag;
    int64_t n_store_tokens, final_capacity, store_ts, store_hs, final_ts, final_hs;
    int32_t seg_stride, batch, max_tq, n_kv_heads, head_dim, max_positions;
};
cf_status launch_assemble(const cf_layer_desc* d, const RopeFreq& f, const AssembleArgs& a, int32_t max_seg_len,
                          hipStream_t s);

cf_status launch_reposition(const cf_layer_desc* d, const RopeFreq& f, const void* k_in, void* k_out,
                            const cf_segment* segs, int32_t n_seg, int64_t n_store_tokens,
                            int32_t max_seg_len, int32_t* dev_flag, hipStream_t s);

struct AttnArgs {
    const void* q;
    const int32_t* q_off;
    int32_t q_stored_start;
    const int32_t* q_new_start;
    const void* k_store;
    const void* v_store;
    int64_t n_store_tokens;
    const void* k_self;
    const void* v_self;
    const cf_segment* segs;
    const int32_t* n_seg;
    int32_t seg_stride;
    int32_t batch;
    int32_t max_tq;
    int64_t max_kv_tokens;
    void* out;
    float* mass;
    float* score_accum;
    int32_t score_stride;
    void* workspace;
    size_t workspace_bytes;
    int32_t* dev_flag;
    int32_t n_q_heads, n_kv_heads, head_dim, dtype, pairing;
    float scale_log2e;   // softmax scale times log2(e)
    int64_t store_ts, store_hs;   // element strides of the cache store between tokens / kv heads
    int32_t max_positions;        // positions are valid in [0, max_positions)
    // Deferred document-wise scores (cf_prefill_layer): this call's slot partials go to part `n_pending` of the
    // workspace's ledger; with `defer` set nothing reduces them yet, otherwise the reduction takes parts 0 .. n_pending
    // in order (S += s^l layer by layer, Alg. 2).
    int32_t n_pending, defer;
};
constexpr int kMaxPending = 15;   // layers whose scores may be pending in a workspace

inline int64_t store_token_stride(const cf_layer_desc* d) {
    return d->store_token_stride ? d->store_token_stride : (int64_t)d->n_kv_heads * d->head_dim;
}
inline int64_t store_head_stride(const cf_layer_desc* d) { return d->store_head_stride ? d->store_head_stride : d->head_dim; }

size_t generic_workspace_bytes(const cf_layer_desc* d, int32_t batch, int32_t max_tq, int32_t seg_stride);
cf_status launch_attention_generic(const AttnArgs& a, const RopeFreq& f, hipStream_t s);

bool mfma_path_supported(const cf_layer_desc* d);
size_t mfma_workspace_bytes(const cf_layer_desc* d, int32_t batch, int32_t max_tq, int32_t seg_stride,
                            int64_t max_kv_tokens);
cf_status launch_attention_mfma(const AttnArgs& a, const RopeFreq& f, hipStream_t s, const cf_prune_step* prune);
// the three stand-alone launches of a prune step (ranking, allocation, table rebuild)
cf_status launch_prune_step(const AttnArgs& a, const cf_prune_step* prune, hipStream_t s);

cf_status launch_prune(const float* score, const int32_t* len, const int32_t* cand, const int32_t* n_cand,
                       int32_t keep, int32_t batch, int32_t stride, int32_t* keep_idx, int32_t* n_keep,
                       int32_t* dev_flag, hipStream_t s);
cf_status launch_assign(const int32_t* len, const int32_t* ranked, const int32_t* n_ranked, int32_t batch,
                        int32_t stride, int32_t pos_begin, int32_t pos_end, int32_t strategy,
                        int32_t force_n_reuse, int32_t* new_start, int32_t* q_start, int32_t* n_reuse,
                        int32_t* order, int32_t* dev_flag, hipStream_t s);
cf_status launch_gather(const int64_t* doc_tok_offset, const int32_t* len, const int32_t* order,
                        const int32_t* n_order, const int32_t* new_start, const int32_t* q_start,
                        const int32_t* q_off, int32_t batch, int32_t stride, int32_t prefix_len,
                        int32_t doc_stored_start, int32_t q_stored_start, cf_segment* segs, int32_t* n_seg,
                        int32_t seg_stride, int32_t* dev_flag, hipStream_t s);

constexpr int kMaxSelectStride = 4096;   // documents per query the ranking kernels hold in LDS

}  // namespace cf
