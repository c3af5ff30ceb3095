// C-ABI entry points of libcachefocus: host-side validation and launch planning.
// Every argument that lives on the host is checked here, before any HIP call, so the error
// paths can be exercised without a GPU.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "cf_common.h"

namespace cf {

namespace {
thread_local char g_err[512] = "";
}

namespace {
constexpr int kTimerPairs = 1024;
struct KernelTimer {
    bool on = false;
    long long launches = 0;
    hipEvent_t begin[kTimerPairs], end[kTimerPairs];
};
thread_local KernelTimer g_timer;
}  // namespace

void profile_kernel_pair(hipEvent_t* start, hipEvent_t* stop) {
    *start = *stop = nullptr;
    if (!g_timer.on) return;
    *start = g_timer.begin[g_timer.launches % kTimerPairs];
    *stop = g_timer.end[g_timer.launches % kTimerPairs];
    ++g_timer.launches;
}

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

size_t elem_size(int32_t dtype) { return dtype == CF_F32 ? 4 : 2; }

cf_status check_desc(const cf_layer_desc* d) {
    CF_REQUIRE(d != nullptr, CF_ERR_INVALID_ARG, "desc is NULL");
    CF_REQUIRE(d->n_q_heads > 0 && d->n_kv_heads > 0, CF_ERR_INVALID_ARG, "head counts must be positive");
    CF_REQUIRE(d->n_q_heads % d->n_kv_heads == 0, CF_ERR_INVALID_ARG,
               "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", d->n_q_heads, d->n_kv_heads);
    CF_REQUIRE(d->dtype == CF_F32 || d->dtype == CF_BF16 || d->dtype == CF_F16, CF_ERR_INVALID_ARG,
               "unknown dtype %d", d->dtype);
    CF_REQUIRE(d->rope_pairing == CF_ROPE_HALF || d->rope_pairing == CF_ROPE_INTERLEAVED, CF_ERR_INVALID_ARG,
               "unknown rope_pairing %d", d->rope_pairing);
    CF_REQUIRE(d->head_dim > 0, CF_ERR_INVALID_ARG, "head_dim must be positive");
    CF_REQUIRE(d->head_dim % 16 == 0 && d->head_dim <= kMaxHeadDim, CF_ERR_UNSUPPORTED,
               "head_dim %d unsupported (multiple of 16, at most %d)", d->head_dim, kMaxHeadDim);
    CF_REQUIRE(std::isfinite(d->rope_base) && d->rope_base > 1.0, CF_ERR_INVALID_ARG, "rope_base must be > 1");
    CF_REQUIRE(d->max_positions > 0, CF_ERR_INVALID_ARG, "max_positions must be positive");
    CF_REQUIRE(std::isfinite(d->softmax_scale) && d->softmax_scale >= 0.f, CF_ERR_INVALID_ARG,
               "softmax_scale must be >= 0");
    CF_REQUIRE(d->reserved == 0, CF_ERR_INVALID_ARG, "desc.reserved must be 0");
    if (d->store_token_stride != 0 || d->store_head_stride != 0) {
        CF_REQUIRE(d->store_token_stride >= d->head_dim && d->store_head_stride >= d->head_dim, CF_ERR_INVALID_ARG,
                   "store strides must both be 0 or both at least head_dim");
        CF_REQUIRE(d->store_token_stride % 8 == 0 && d->store_head_stride % 8 == 0, CF_ERR_INVALID_ARG,
                   "store strides must be multiples of 8 elements");
        CF_REQUIRE(d->store_token_stride <= (1 << 24), CF_ERR_UNSUPPORTED, "store_token_stride above 2^24 elements");
    }
    return CF_OK;
}

void fill_rope_freq(const cf_layer_desc* d, RopeFreq* f) {
    const int half = d->head_dim / 2;
    const double two_pi = 6.283185307179586476925286766559;
    for (int m = 0; m < kMaxHalf; ++m)
        f->rev[m] = m < half ? std::pow(d->rope_base, -2.0 * m / d->head_dim) / two_pi : 0.0;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

cf_status launch_prune_step(const AttnArgs& a, const cf_prune_step* pr, hipStream_t s) {
    cf_status st = launch_prune(a.score_accum, pr->normalise_by_len ? pr->doc_len : nullptr, pr->cand, pr->n_cand, pr->keep,
                                a.batch, pr->stride, pr->keep_idx, pr->n_keep, a.dev_flag, s);
    if (st != CF_OK) return st;
    st = launch_assign(pr->doc_len, pr->keep_idx, pr->n_keep, a.batch, pr->stride, pr->pos_begin, pr->pos_end,
                       pr->strategy, pr->force_n_reuse, pr->new_start, pr->q_start, pr->n_reuse, pr->order, a.dev_flag, s);
    if (st != CF_OK) return st;
    return launch_gather(pr->doc_tok_offset, pr->doc_len, pr->order, pr->n_keep, pr->new_start, pr->q_start, a.q_off,
                         a.batch, pr->stride, pr->prefix_len, pr->doc_stored_start, a.q_stored_start, pr->next_segs,
                         pr->next_n_seg, a.seg_stride, a.dev_flag, s);
}

}  // namespace cf

using namespace cf;

extern "C" {

const char* cf_last_error(void) { return g_err; }

int32_t cf_version(void) { return 100; }

cf_status cf_profile_kernel_events(int32_t enable) {
    if (g_timer.on) {
        for (int i = 0; i < kTimerPairs; ++i) { (void)hipEventDestroy(g_timer.begin[i]); (void)hipEventDestroy(g_timer.end[i]); }
        g_timer.on = false;
    }
    g_timer.launches = 0;
    if (!enable) return CF_OK;
    for (int i = 0; i < kTimerPairs; ++i) {
        hipError_t e = hipEventCreate(&g_timer.begin[i]);
        if (e == hipSuccess) e = hipEventCreate(&g_timer.end[i]);
        if (e != hipSuccess) {
            // destroy what exists (a failed begin[i] leaves end[i] uncreated)
            for (int j = 0; j < i; ++j) { (void)hipEventDestroy(g_timer.begin[j]); (void)hipEventDestroy(g_timer.end[j]); }
            set_error("hipEventCreate: %s", hipGetErrorString(e));
            return CF_ERR_DEVICE;
        }
    }
    g_timer.on = true;
    return CF_OK;
}

cf_status cf_profile_kernel_ms(double* mean_ms, int32_t* launches) {
    CF_REQUIRE(mean_ms && launches, CF_ERR_INVALID_ARG, "mean_ms and launches must not be NULL");
    CF_REQUIRE(g_timer.on, CF_ERR_INVALID_ARG, "kernel timing is not enabled");
    const int n = (int)(g_timer.launches < kTimerPairs ? g_timer.launches : kTimerPairs);
    double total = 0.0;
    for (int i = 0; i < n; ++i) {
        CF_HIP(hipEventSynchronize(g_timer.end[i]));
        float ms = 0.f;
        CF_HIP(hipEventElapsedTime(&ms, g_timer.begin[i], g_timer.end[i]));
        total += ms;
    }
    *mean_ms = n ? total / n : 0.0;
    *launches = n;
    return CF_OK;
}

cf_status cf_reposition_keys(const cf_layer_desc* desc, const void* k_in, void* k_out, const cf_segment* segs,
                             int32_t n_seg, int64_t n_store_tokens, int32_t max_seg_len, int32_t* dev_flag,
                             void* stream) {
    cf_status st = check_desc(desc);
    if (st != CF_OK) return st;
    CF_REQUIRE(n_seg >= 0, CF_ERR_INVALID_ARG, "n_seg is negative");
    CF_REQUIRE(n_store_tokens >= 0, CF_ERR_INVALID_ARG, "n_store_tokens is negative");
    CF_REQUIRE(max_seg_len >= 1, CF_ERR_INVALID_ARG, "max_seg_len must be >= 1");
    if (n_seg == 0) return CF_OK;
    CF_REQUIRE(k_in && k_out && segs, CF_ERR_INVALID_ARG, "k_in, k_out and segs must not be NULL");
    CF_REQUIRE(aligned16(k_in) && aligned16(k_out), CF_ERR_INVALID_ARG, "k_in/k_out must be 16-byte aligned");
    RopeFreq f;
    fill_rope_freq(desc, &f);
    return launch_reposition(desc, f, k_in, k_out, segs, n_seg, n_store_tokens, max_seg_len, dev_flag,
                             static_cast<hipStream_t>(stream));
}

size_t cf_prefill_workspace_bytes(const cf_layer_desc* desc, int32_t batch, int32_t max_tq, int32_t seg_stride,
                                  int64_t max_kv_tokens) {
    if (check_desc(desc) != CF_OK) return 0;
    if (batch <= 0 || max_tq <= 0 || seg_stride <= 0 || max_kv_tokens < 0) return 0;
    size_t n = mfma_path_supported(desc) ? mfma_workspace_bytes(desc, batch, max_tq, seg_stride, max_kv_tokens)
                                         : generic_workspace_bytes(desc, batch, max_tq, seg_stride);
    return (n + 255) & ~(size_t)255;
}

static cf_status check_prune_step(const cf_prune_step* pr, int32_t seg_stride, const float* score_accum,
                                  int32_t score_stride, const cf_segment* segs, const int32_t* n_seg,
                                  const int32_t* q_new_start) {
    CF_REQUIRE(score_accum != nullptr, CF_ERR_INVALID_ARG, "a prune step needs score_accum");
    CF_REQUIRE(pr->stride >= 1 && pr->stride <= kMaxSelectStride, CF_ERR_INVALID_ARG, "stride must be in [1, %d]",
               kMaxSelectStride);
    CF_REQUIRE(score_stride == pr->stride, CF_ERR_INVALID_ARG, "score_stride must equal the prune step's stride");
    CF_REQUIRE(pr->keep >= 0 && pr->keep <= pr->stride, CF_ERR_INVALID_ARG, "keep (%d) must be in [0, stride = %d]",
               pr->keep, pr->stride);
    CF_REQUIRE(pr->strategy == CF_ALLOC_KEEP || pr->strategy == CF_ALLOC_ALIGN || pr->strategy == CF_ALLOC_SORT,
               CF_ERR_INVALID_ARG, "unknown strategy %d", pr->strategy);
    CF_REQUIRE(pr->force_n_reuse >= 0 && pr->reserved == 0, CF_ERR_INVALID_ARG, "bad force_n_reuse / reserved");
    CF_REQUIRE(pr->pos_begin >= 0 && pr->pos_end > pr->pos_begin, CF_ERR_RANGE,
               "need 0 <= pos_begin < pos_end (got %d, %d)", pr->pos_begin, pr->pos_end);
    CF_REQUIRE(pr->prefix_len >= 0 && pr->doc_stored_start >= 0, CF_ERR_RANGE, "negative prefix_len / doc_stored_start");
    CF_REQUIRE(seg_stride >= 2, CF_ERR_INVALID_ARG, "seg_stride must be >= 2");
    CF_REQUIRE(pr->doc_tok_offset && pr->doc_len && pr->cand && pr->n_cand && pr->keep_idx && pr->n_keep &&
                   pr->new_start && pr->q_start && pr->n_reuse && pr->order && pr->next_segs && pr->next_n_seg,
               CF_ERR_INVALID_ARG, "NULL pointer in the prune step");
    CF_REQUIRE(pr->keep_idx != pr->cand && pr->order != pr->keep_idx && pr->order != pr->cand, CF_ERR_INVALID_ARG,
               "keep_idx, order and cand must be distinct arrays");
    CF_REQUIRE(pr->next_segs != segs && pr->next_n_seg != n_seg && pr->q_start != q_new_start, CF_ERR_INVALID_ARG,
               "the next layer's tables must not alias the current ones");
    return CF_OK;
}

static cf_status prefill_impl(const cf_layer_desc* desc, const void* q, const int32_t* q_off,
                               int32_t q_stored_start, const int32_t* q_new_start, const void* k_store,
                               const void* v_store, int64_t n_store_tokens, const void* k_self,
                               const void* v_self, const cf_segment* segs, const int32_t* n_seg,
                               int32_t seg_stride, int32_t batch, int32_t max_tq, int64_t max_kv_tokens,
                               void* out, float* mass, float* score_accum, int32_t score_stride,
                               void* workspace, size_t workspace_bytes, const cf_prune_step* prune,
                               int32_t n_pending, int32_t defer, int32_t* dev_flag, void* stream) {
    cf_status st = check_desc(desc);
    if (st != CF_OK) return st;
    CF_REQUIRE(batch >= 0, CF_ERR_INVALID_ARG, "batch is negative");
    CF_REQUIRE(n_pending >= 0 && n_pending <= kMaxPending && (defer == 0 || defer == 1), CF_ERR_INVALID_ARG,
               "n_pending must be in [0, %d] and defer 0 or 1", kMaxPending);
    CF_REQUIRE(!(defer && prune), CF_ERR_INVALID_ARG, "a call with a prune step cannot defer its scores");
    CF_REQUIRE(!(defer && n_pending == kMaxPending), CF_ERR_INVALID_ARG, "%d layers are pending already: flush first", kMaxPending);
    CF_REQUIRE(max_tq >= 1, CF_ERR_INVALID_ARG, "max_tq must be >= 1");
    CF_REQUIRE(seg_stride >= 1, CF_ERR_INVALID_ARG, "seg_stride must be >= 1");
    CF_REQUIRE(n_store_tokens >= 0 && max_kv_tokens >= 0, CF_ERR_INVALID_ARG, "negative token count");
    CF_REQUIRE(score_accum == nullptr || score_stride >= 1, CF_ERR_INVALID_ARG,
               "score_stride must be >= 1 when score_accum is given");
    if (prune) {
        st = check_prune_step(prune, seg_stride, score_accum, score_stride, segs, n_seg, q_new_start);
        if (st != CF_OK) return st;
    }
    if (batch == 0) return CF_OK;
    CF_REQUIRE(q && q_off && q_new_start && segs && n_seg && out, CF_ERR_INVALID_ARG,
               "q, q_off, q_new_start, segs, n_seg and out must not be NULL");
    CF_REQUIRE(mass != nullptr || (score_accum == nullptr && prune == nullptr), CF_ERR_INVALID_ARG,
               "mass may be NULL only when neither scores nor a prune step are asked for");
    CF_REQUIRE((k_self == nullptr) == (v_self == nullptr), CF_ERR_INVALID_ARG,
               "k_self and v_self must be given together");
    CF_REQUIRE(n_store_tokens == 0 || (k_store && v_store), CF_ERR_INVALID_ARG,
               "k_store/v_store are NULL but n_store_tokens > 0");
    CF_REQUIRE(aligned16(q) && aligned16(k_store) && aligned16(v_store) && aligned16(k_self) &&
                   aligned16(v_self) && aligned16(out),
               CF_ERR_INVALID_ARG, "tensor base pointers must be 16-byte aligned");
    CF_REQUIRE(q_stored_start >= 0 && q_stored_start < desc->max_positions, CF_ERR_RANGE,
               "q_stored_start outside [0, max_positions)");
    const size_t need = cf_prefill_workspace_bytes(desc, batch, max_tq, seg_stride, max_kv_tokens);
    CF_REQUIRE(workspace != nullptr && workspace_bytes >= need, CF_ERR_WORKSPACE,
               "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
    CF_REQUIRE((reinterpret_cast<uintptr_t>(workspace) & 255u) == 0, CF_ERR_WORKSPACE,
               "workspace must be 256-byte aligned");

    AttnArgs a;
    std::memset(&a, 0, sizeof(a));
    a.q = q; a.q_off = q_off; a.q_stored_start = q_stored_start; a.q_new_start = q_new_start;
    a.k_store = k_store; a.v_store = v_store; a.n_store_tokens = n_store_tokens;
    a.k_self = k_self; a.v_self = v_self; a.segs = segs; a.n_seg = n_seg; a.seg_stride = seg_stride;
    a.batch = batch; a.max_tq = max_tq; a.max_kv_tokens = max_kv_tokens; a.out = out; a.mass = mass;
    a.score_accum = score_accum; a.score_stride = score_stride; a.workspace = workspace;
    a.workspace_bytes = workspace_bytes; a.dev_flag = dev_flag;
    a.n_q_heads = desc->n_q_heads; a.n_kv_heads = desc->n_kv_heads; a.head_dim = desc->head_dim;
    a.dtype = desc->dtype; a.pairing = desc->rope_pairing;
    const double scale = desc->softmax_scale > 0.f ? (double)desc->softmax_scale : 1.0 / std::sqrt((double)desc->head_dim);
    a.scale_log2e = (float)(scale * 1.4426950408889634073599246810019);
    a.store_ts = store_token_stride(desc);
    a.store_hs = store_head_stride(desc);
    a.max_positions = desc->max_positions;
    a.n_pending = n_pending;
    a.defer = defer;
    RopeFreq f;
    fill_rope_freq(desc, &f);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (mfma_path_supported(desc)) return launch_attention_mfma(a, f, s, prune);
    st = launch_attention_generic(a, f, s);
    if (st != CF_OK || !prune) return st;
    return launch_prune_step(a, prune, s);
}

cf_status cf_prefill_attention(const cf_layer_desc* desc, const void* q, const int32_t* q_off,
                               int32_t q_stored_start, const int32_t* q_new_start, const void* k_store,
                               const void* v_store, int64_t n_store_tokens, const void* k_self,
                               const void* v_self, const cf_segment* segs, const int32_t* n_seg,
                               int32_t seg_stride, int32_t batch, int32_t max_tq, int64_t max_kv_tokens,
                               void* out, float* mass, float* score_accum, int32_t score_stride,
                               void* workspace, size_t workspace_bytes, int32_t* dev_flag, void* stream) {
    return prefill_impl(desc, q, q_off, q_stored_start, q_new_start, k_store, v_store, n_store_tokens, k_self, v_self,
                        segs, n_seg, seg_stride, batch, max_tq, max_kv_tokens, out, mass, score_accum, score_stride,
                        workspace, workspace_bytes, nullptr, 0, 0, dev_flag, stream);
}

// The library-owned scratch of cf_prefill_attention_static: one copy per GPU, at an address of its own on each.
// In host code the array's name is only a handle for the symbol lookup; kernels and copies use the looked-up
// device address.
static __device__ __attribute__((used)) __align__(256) unsigned char g_static_scratch[CF_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxScratchDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_addr[kMaxScratchDevices] = {};

// the array's address on the current device, looked up once per device
cf_status static_scratch(void** addr) {
    int dev = -1;
    CF_HIP(hipGetDevice(&dev));
    CF_REQUIRE(dev >= 0 && dev < kMaxScratchDevices, CF_ERR_UNSUPPORTED, "device ordinal %d beyond %d", dev, kMaxScratchDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_addr[dev] == nullptr) {
        void* p = nullptr;
        CF_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)));
        CF_REQUIRE(p != nullptr && (reinterpret_cast<uintptr_t>(p) & 255u) == 0, CF_ERR_DEVICE, "static scratch at a bad address");
        g_scratch_addr[dev] = p;
    }
    *addr = g_scratch_addr[dev];
    return CF_OK;
}
}  // namespace

cf_status cf_prefill_attention_static(const cf_layer_desc* desc, const void* q, const int32_t* q_off,
                                      int32_t q_stored_start, const int32_t* q_new_start, const void* k_store,
                                      const void* v_store, int64_t n_store_tokens, const void* k_self,
                                      const void* v_self, const cf_segment* segs, const int32_t* n_seg,
                                      int32_t seg_stride, int32_t batch, int32_t max_tq, int64_t max_kv_tokens,
                                      void* out, float* mass, float* score_accum, int32_t score_stride,
                                      int32_t* dev_flag, void* stream) {
    cf_status st = check_desc(desc);
    if (st != CF_OK) return st;
    CF_REQUIRE(batch >= 0 && max_tq >= 1 && seg_stride >= 1 && max_kv_tokens >= 0, CF_ERR_INVALID_ARG,
               "batch, max_tq, seg_stride or max_kv_tokens out of range");
    if (batch == 0) return CF_OK;
    const size_t need = cf_prefill_workspace_bytes(desc, batch, max_tq, seg_stride, max_kv_tokens);
    CF_REQUIRE(need <= CF_STATIC_SCRATCH_BYTES, CF_ERR_WORKSPACE,
               "this shape needs %zu bytes of scratch, the library-owned buffer holds %zu: use cf_prefill_attention with a workspace",
               need, (size_t)CF_STATIC_SCRATCH_BYTES);
    void* scratch = nullptr;
    st = static_scratch(&scratch);
    if (st != CF_OK) return st;
    return prefill_impl(desc, q, q_off, q_stored_start, q_new_start, k_store, v_store, n_store_tokens, k_self, v_self,
                        segs, n_seg, seg_stride, batch, max_tq, max_kv_tokens, out, mass, score_accum, score_stride,
                        scratch, CF_STATIC_SCRATCH_BYTES, nullptr, 0, 0, dev_flag, stream);
}

cf_status cf_prefill_layer(const cf_layer_desc* desc, const void* q, const int32_t* q_off, int32_t q_stored_start,
                           const int32_t* q_new_start, const void* k_store, const void* v_store,
                           int64_t n_store_tokens, const void* k_self, const void* v_self, const cf_segment* segs,
                           const int32_t* n_seg, int32_t seg_stride, int32_t batch, int32_t max_tq,
                           int64_t max_kv_tokens, void* out, float* mass, float* score_accum, int32_t score_stride,
                           void* workspace, size_t workspace_bytes, const cf_prune_step* prune, int32_t n_pending,
                           int32_t defer, int32_t* dev_flag, void* stream) {
    CF_REQUIRE(score_accum != nullptr, CF_ERR_INVALID_ARG, "cf_prefill_layer needs score_accum");
    return prefill_impl(desc, q, q_off, q_stored_start, q_new_start, k_store, v_store, n_store_tokens, k_self, v_self,
                        segs, n_seg, seg_stride, batch, max_tq, max_kv_tokens, out, mass, score_accum, score_stride,
                        workspace, workspace_bytes, prune, n_pending, defer, dev_flag, stream);
}

cf_status cf_prune_topk(const float* score, const int32_t* len, const int32_t* cand, const int32_t* n_cand,
                        int32_t keep, int32_t batch, int32_t stride, int32_t* keep_idx, int32_t* n_keep,
                        int32_t* dev_flag, void* stream) {
    CF_REQUIRE(batch >= 0, CF_ERR_INVALID_ARG, "batch is negative");
    CF_REQUIRE(stride >= 1 && stride <= kMaxSelectStride, CF_ERR_INVALID_ARG, "stride must be in [1, %d]",
               kMaxSelectStride);
    CF_REQUIRE(keep >= 0 && keep <= stride, CF_ERR_INVALID_ARG, "keep (%d) must be in [0, stride = %d]", keep,
               stride);
    if (batch == 0) return CF_OK;
    CF_REQUIRE(score && cand && n_cand && keep_idx && n_keep, CF_ERR_INVALID_ARG,
               "score, cand, n_cand, keep_idx and n_keep must not be NULL");
    CF_REQUIRE(keep_idx != cand, CF_ERR_INVALID_ARG, "keep_idx must not alias cand");
    return launch_prune(score, len, cand, n_cand, keep, batch, stride, keep_idx, n_keep, dev_flag,
                        static_cast<hipStream_t>(stream));
}

cf_status cf_assign_positions(const int32_t* len, const int32_t* ranked, const int32_t* n_ranked, int32_t batch,
                              int32_t stride, int32_t pos_begin, int32_t pos_end, int32_t strategy,
                              int32_t force_n_reuse, int32_t* new_start, int32_t* q_start, int32_t* n_reuse,
                              int32_t* order, int32_t* dev_flag, void* stream) {
    CF_REQUIRE(batch >= 0, CF_ERR_INVALID_ARG, "batch is negative");
    CF_REQUIRE(stride >= 1 && stride <= kMaxSelectStride, CF_ERR_INVALID_ARG, "stride must be in [1, %d]",
               kMaxSelectStride);
    CF_REQUIRE(strategy == CF_ALLOC_KEEP || strategy == CF_ALLOC_ALIGN || strategy == CF_ALLOC_SORT,
               CF_ERR_INVALID_ARG, "unknown strategy %d", strategy);
    CF_REQUIRE(force_n_reuse >= 0, CF_ERR_INVALID_ARG, "force_n_reuse is negative");
    CF_REQUIRE(pos_begin >= 0 && pos_end > pos_begin, CF_ERR_RANGE, "need 0 <= pos_begin < pos_end (got %d, %d)",
               pos_begin, pos_end);
    if (batch == 0) return CF_OK;
    CF_REQUIRE(len && ranked && n_ranked && order, CF_ERR_INVALID_ARG,
               "len, ranked, n_ranked and order must not be NULL");
    CF_REQUIRE(order != ranked, CF_ERR_INVALID_ARG, "order must not alias ranked");
    CF_REQUIRE(strategy == CF_ALLOC_KEEP || (new_start && q_start && n_reuse), CF_ERR_INVALID_ARG,
               "new_start, q_start and n_reuse must not be NULL");
    return launch_assign(len, ranked, n_ranked, batch, stride, pos_begin, pos_end, strategy, force_n_reuse,
                         new_start, q_start, n_reuse, order, dev_flag, static_cast<hipStream_t>(stream));
}

cf_status cf_gather_segments(const int64_t* doc_tok_offset, const int32_t* len, const int32_t* order,
                             const int32_t* n_order, const int32_t* new_start, const int32_t* q_start,
                             const int32_t* q_off, int32_t batch, int32_t stride, int32_t prefix_len,
                             int32_t doc_stored_start, int32_t q_stored_start, cf_segment* segs, int32_t* n_seg,
                             int32_t seg_stride, int32_t* dev_flag, void* stream) {
    CF_REQUIRE(batch >= 0, CF_ERR_INVALID_ARG, "batch is negative");
    CF_REQUIRE(stride >= 1, CF_ERR_INVALID_ARG, "stride must be >= 1");
    CF_REQUIRE(prefix_len >= 0, CF_ERR_INVALID_ARG, "prefix_len is negative");
    CF_REQUIRE(doc_stored_start >= 0 && q_stored_start >= 0, CF_ERR_RANGE, "stored positions are negative");
    CF_REQUIRE(seg_stride >= 2, CF_ERR_INVALID_ARG, "seg_stride must be >= 2");
    if (batch == 0) return CF_OK;
    CF_REQUIRE(doc_tok_offset && len && order && n_order && new_start && q_start && q_off && segs && n_seg,
               CF_ERR_INVALID_ARG, "NULL table pointer");
    return launch_gather(doc_tok_offset, len, order, n_order, new_start, q_start, q_off, batch, stride,
                         prefix_len, doc_stored_start, q_stored_start, segs, n_seg, seg_stride, dev_flag,
                         static_cast<hipStream_t>(stream));
}

cf_status cf_assemble_cache(const cf_layer_desc* desc, const void* k_store, const void* v_store, int64_t n_store_tokens,
                            const void* k_self, const void* v_self, const int32_t* q_off, const cf_segment* segs,
                            const int32_t* n_seg, int32_t seg_stride, int32_t batch, int32_t max_tq, int32_t max_seg_len,
                            const int64_t* final_off, int64_t final_capacity, int64_t final_token_stride,
                            int64_t final_head_stride, void* k_final, void* v_final, int32_t* final_len,
                            int32_t* final_pos, int32_t* dev_flag, void* stream) {
    cf_status st = check_desc(desc);
    if (st != CF_OK) return st;
    CF_REQUIRE(batch >= 0, CF_ERR_INVALID_ARG, "batch is negative");
    CF_REQUIRE(seg_stride >= 1 && max_tq >= 1 && max_seg_len >= 1, CF_ERR_INVALID_ARG,
               "seg_stride, max_tq and max_seg_len must be >= 1");
    CF_REQUIRE(n_store_tokens >= 0 && final_capacity >= 0, CF_ERR_INVALID_ARG, "negative token count");
    CF_REQUIRE(final_token_stride >= desc->head_dim && final_head_stride >= desc->head_dim &&
                   final_token_stride % 8 == 0 && final_head_stride % 8 == 0,
               CF_ERR_INVALID_ARG, "final strides must be multiples of 8 and at least head_dim");
    if (batch == 0) return CF_OK;
    CF_REQUIRE((int64_t)batch * seg_stride <= 0x7fffffff, CF_ERR_UNSUPPORTED, "batch * seg_stride too large");
    CF_REQUIRE(q_off && segs && n_seg && final_off && k_final && v_final && final_len, CF_ERR_INVALID_ARG,
               "q_off, segs, n_seg, final_off, k_final, v_final and final_len must not be NULL");
    CF_REQUIRE((k_self == nullptr) == (v_self == nullptr), CF_ERR_INVALID_ARG, "k_self and v_self must be given together");
    CF_REQUIRE(n_store_tokens == 0 || (k_store && v_store), CF_ERR_INVALID_ARG,
               "k_store/v_store are NULL but n_store_tokens > 0");
    CF_REQUIRE(aligned16(k_store) && aligned16(v_store) && aligned16(k_self) && aligned16(v_self) && aligned16(k_final) &&
                   aligned16(v_final),
               CF_ERR_INVALID_ARG, "tensor base pointers must be 16-byte aligned");
    CF_REQUIRE(k_final != k_store && k_final != k_self && v_final != v_store && v_final != v_self && k_final != v_final,
               CF_ERR_INVALID_ARG, "k_final / v_final must not alias the inputs or each other");
    AssembleArgs a;
    std::memset(&a, 0, sizeof(a));
    a.k_store = k_store; a.v_store = v_store; a.k_self = k_self; a.v_self = v_self; a.k_final = k_final; a.v_final = v_final;
    a.q_off = q_off; a.segs = segs; a.n_seg = n_seg; a.final_off = final_off; a.final_len = final_len; a.final_pos = final_pos;
    a.dev_flag = dev_flag; a.n_store_tokens = n_store_tokens; a.final_capacity = final_capacity;
    a.store_ts = store_token_stride(desc); a.store_hs = store_head_stride(desc);
    a.final_ts = final_token_stride; a.final_hs = final_head_stride;
    a.seg_stride = seg_stride; a.batch = batch; a.max_tq = max_tq; a.n_kv_heads = desc->n_kv_heads; a.head_dim = desc->head_dim;
    a.max_positions = desc->max_positions;
    RopeFreq f;
    fill_rope_freq(desc, &f);
    return launch_assemble(desc, f, a, max_seg_len, static_cast<hipStream_t>(stream));
}

}  // extern "C"
