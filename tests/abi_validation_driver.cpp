// Host-side exercise of the C ABI for a build of the library's host code under AddressSanitizer and
// UndefinedBehaviorSanitizer (tests/test_abi_host_sanitized.py builds and runs it; no GPU is touched).
// Every call below must be settled by the host-side validation — a status code, a message, nothing launched —
// or by host arithmetic alone (the launch plans behind cf_prefill_workspace_bytes).  Pointers that must be non-null
// are fakes that validation never dereferences.  Exit status 0: every expectation held and no sanitizer report.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <initializer_list>

#include "cachefocus.h"

static int g_failures = 0;
static int g_checks = 0;

#define EXPECT(cond)                                                                           \
    do {                                                                                       \
        ++g_checks;                                                                            \
        if (!(cond)) { ++g_failures; std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); } \
    } while (0)

template <typename T>
static T* fake(uintptr_t off = 0) { return reinterpret_cast<T*>(uintptr_t{0x10000} + off); }

static cf_layer_desc desc(int hq = 8, int hkv = 2, int d = 128, int dtype = CF_BF16) {
    cf_layer_desc x;
    std::memset(&x, 0, sizeof x);
    x.n_q_heads = hq; x.n_kv_heads = hkv; x.head_dim = d; x.dtype = dtype; x.rope_pairing = CF_ROPE_HALF;
    x.max_positions = 4096; x.rope_base = 1.0e4;
    return x;
}

static cf_status reposition(const cf_layer_desc& d) {
    return cf_reposition_keys(&d, fake<void>(), fake<void>(), fake<cf_segment>(), 1, 10, 1, nullptr, nullptr);
}

struct PrefillArgs {
    cf_layer_desc d = desc();
    const void* q = fake<void>();
    int32_t q_stored_start = 0;
    const void *k_store = fake<void>(), *v_store = fake<void>(), *k_self = fake<void>(), *v_self = fake<void>();
    int32_t seg_stride = 4, batch = 1, max_tq = 8;
    int64_t max_kv = 100;
    void* out = fake<void>();
    float *mass = fake<float>(), *score = nullptr;
    int32_t score_stride = 0;
    void* ws = fake<void>(0x100);
    size_t ws_bytes = size_t{1} << 30;
    int32_t n_pending = 0, defer = 0;
};

static cf_status attention(const PrefillArgs& a) {
    return cf_prefill_attention(&a.d, a.q, fake<int32_t>(), a.q_stored_start, fake<int32_t>(), a.k_store, a.v_store, 100, a.k_self,
                                a.v_self, fake<cf_segment>(), fake<int32_t>(), a.seg_stride, a.batch, a.max_tq, a.max_kv, a.out,
                                a.mass, a.score, a.score_stride, a.ws, a.ws_bytes, nullptr, nullptr);
}

static cf_status layer(const PrefillArgs& a) {
    return cf_prefill_layer(&a.d, a.q, fake<int32_t>(), a.q_stored_start, fake<int32_t>(), a.k_store, a.v_store, 100, a.k_self,
                            a.v_self, fake<cf_segment>(), fake<int32_t>(), a.seg_stride, a.batch, a.max_tq, a.max_kv, a.out, a.mass,
                            a.score, a.score_stride, a.ws, a.ws_bytes, nullptr, a.n_pending, a.defer, nullptr, nullptr);
}

static void descriptors() {
    cf_layer_desc d;
    d = desc(7, 2); EXPECT(reposition(d) == CF_ERR_INVALID_ARG);
    d = desc(8, 2, 100); EXPECT(reposition(d) == CF_ERR_UNSUPPORTED);
    d = desc(8, 2, 512); EXPECT(reposition(d) == CF_ERR_UNSUPPORTED);
    d = desc(8, 2, 128, 9); EXPECT(reposition(d) == CF_ERR_INVALID_ARG);
    d = desc(); d.rope_base = 0.5; EXPECT(reposition(d) == CF_ERR_INVALID_ARG);
    d = desc(); d.max_positions = 0; EXPECT(reposition(d) == CF_ERR_INVALID_ARG);
    d = desc(); d.rope_pairing = 5; EXPECT(reposition(d) == CF_ERR_INVALID_ARG);
    d = desc(); d.reserved = 1; EXPECT(reposition(d) == CF_ERR_INVALID_ARG);
    d = desc(); d.store_token_stride = 128; EXPECT(reposition(d) == CF_ERR_INVALID_ARG);
    d = desc(); d.store_token_stride = 132; d.store_head_stride = 1280; EXPECT(reposition(d) == CF_ERR_INVALID_ARG);
    d = desc(); d.store_token_stride = int64_t{1} << 25; d.store_head_stride = 128; EXPECT(reposition(d) == CF_ERR_UNSUPPORTED);
    EXPECT(std::strlen(cf_last_error()) > 0);
    EXPECT(cf_reposition_keys(nullptr, fake<void>(), fake<void>(), fake<cf_segment>(), 1, 10, 1, nullptr, nullptr) == CF_ERR_INVALID_ARG);
    d = desc();
    EXPECT(cf_reposition_keys(&d, nullptr, fake<void>(), fake<cf_segment>(), 1, 10, 1, nullptr, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_reposition_keys(&d, fake<void>(4), fake<void>(), fake<cf_segment>(), 1, 10, 1, nullptr, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_reposition_keys(&d, fake<void>(), fake<void>(), fake<cf_segment>(), -1, 10, 1, nullptr, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_reposition_keys(&d, fake<void>(), fake<void>(), fake<cf_segment>(), 1, 10, 0, nullptr, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_reposition_keys(&d, nullptr, nullptr, nullptr, 0, 0, 1, nullptr, nullptr) == CF_OK);      // empty table
}

// The launch plans are host arithmetic: sizes must be positive multiples of 256 and survive extreme (but accepted)
// arguments without overflow.
static void workspace_plans() {
    const int heads[][2] = {{32, 32}, {28, 4}, {12, 2}, {8, 1}, {4, 4}, {64, 8}};
    const int tqs[] = {1, 5, 16, 48, 64, 200, 1024};
    const int strides[] = {1, 3, 12, 52, 64, 65, 256, 300, 4096};
    const int64_t kvs[] = {0, 1, 31, 32, 33, 1680, 7596, 200000, int64_t{1} << 31};
    for (auto& h : heads)
        for (int dt : {CF_BF16, CF_F16, CF_F32})
            for (int tq : tqs)
                for (int st : strides)
                    for (int64_t kv : kvs) {
                        cf_layer_desc d = desc(h[0], h[1], 128, dt);
                        const size_t one = cf_prefill_workspace_bytes(&d, 1, tq, st, kv);
                        const size_t many = cf_prefill_workspace_bytes(&d, 64, tq, st, kv);
                        EXPECT(one > 0 && one % 256 == 0);
                        EXPECT(many > 0 && many % 256 == 0);      // (not monotonic: a batch may need no split partials)
                    }
    cf_layer_desc d = desc();
    EXPECT(cf_prefill_workspace_bytes(&d, 0, 8, 4, 100) == 0);
    EXPECT(cf_prefill_workspace_bytes(&d, 1, 0, 4, 100) == 0);
    EXPECT(cf_prefill_workspace_bytes(&d, 1, 8, 0, 100) == 0);
    EXPECT(cf_prefill_workspace_bytes(&d, 1, 8, 4, -1) == 0);
    EXPECT(cf_prefill_workspace_bytes(nullptr, 1, 8, 4, 100) == 0);
    d.head_dim = 100;
    EXPECT(cf_prefill_workspace_bytes(&d, 1, 8, 4, 100) == 0);
}

static void prefill() {
    PrefillArgs a;
    { PrefillArgs b = a; b.q = nullptr; EXPECT(attention(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = a; b.v_self = nullptr; EXPECT(attention(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = a; b.k_store = b.v_store = nullptr; EXPECT(attention(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = a; b.out = fake<void>(2); EXPECT(attention(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = a; b.max_tq = 0; EXPECT(attention(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = a; b.seg_stride = 0; EXPECT(attention(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = a; b.score = fake<float>(); EXPECT(attention(b) == CF_ERR_INVALID_ARG); }             // score_stride 0
    { PrefillArgs b = a; b.mass = nullptr; b.score = fake<float>(); b.score_stride = 4; EXPECT(attention(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = a; b.q_stored_start = 4096; EXPECT(attention(b) == CF_ERR_RANGE); }
    { PrefillArgs b = a; b.ws = nullptr; EXPECT(attention(b) == CF_ERR_WORKSPACE); }
    { PrefillArgs b = a; b.ws_bytes = 16; EXPECT(attention(b) == CF_ERR_WORKSPACE); EXPECT(std::strstr(cf_last_error(), "workspace") != nullptr); }
    { PrefillArgs b = a; b.ws = fake<void>(0x110); EXPECT(attention(b) == CF_ERR_WORKSPACE); }
    { PrefillArgs b = a; b.batch = 70000; b.ws_bytes = cf_prefill_workspace_bytes(&b.d, 70000, 8, 4, 100);
      EXPECT(attention(b) == CF_ERR_UNSUPPORTED); EXPECT(std::strstr(cf_last_error(), "65535") != nullptr); }
    { PrefillArgs b = a; b.batch = 0; b.q = nullptr; EXPECT(attention(b) == CF_OK); }                         // empty batch
    // one layer in one call: the deferred-score arguments
    PrefillArgs l = a;
    l.score = fake<float>(); l.score_stride = 2; l.ws = nullptr; l.ws_bytes = 0;
    EXPECT(layer(l) == CF_ERR_WORKSPACE);                                                                      // all else accepted
    { PrefillArgs b = l; b.n_pending = -1; EXPECT(layer(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = l; b.n_pending = CF_MAX_PENDING + 1; EXPECT(layer(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = l; b.n_pending = CF_MAX_PENDING; b.defer = 1; EXPECT(layer(b) == CF_ERR_INVALID_ARG); }
    { PrefillArgs b = l; b.n_pending = CF_MAX_PENDING; EXPECT(layer(b) == CF_ERR_WORKSPACE); }
    { PrefillArgs b = l; b.score = nullptr; EXPECT(layer(b) == CF_ERR_INVALID_ARG); }
    // the library-owned scratch has a stated size
    cf_layer_desc big = desc(28, 4);
    const size_t need = cf_prefill_workspace_bytes(&big, 64, 64, 52, 8000);
    EXPECT(need > CF_STATIC_SCRATCH_BYTES);
    EXPECT(cf_prefill_attention_static(&big, fake<void>(), fake<int32_t>(), 0, fake<int32_t>(), fake<void>(), fake<void>(), 100,
                                       fake<void>(), fake<void>(), fake<cf_segment>(), fake<int32_t>(), 52, 64, 64, 8000, fake<void>(),
                                       fake<float>(), nullptr, 0, nullptr, nullptr) == CF_ERR_WORKSPACE);
    EXPECT(std::strstr(cf_last_error(), "library-owned") != nullptr);
}

static void selection() {
    float* s = fake<float>();
    int32_t* i = fake<int32_t>();
    EXPECT(cf_prune_topk(s, nullptr, i, i, 5, 1, 4, fake<int32_t>(64), i, nullptr, nullptr) == CF_ERR_INVALID_ARG);       // keep > stride
    EXPECT(std::strstr(cf_last_error(), "keep") != nullptr);
    EXPECT(cf_prune_topk(s, nullptr, i, i, -1, 1, 4, fake<int32_t>(64), i, nullptr, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_prune_topk(nullptr, nullptr, i, i, 1, 1, 4, fake<int32_t>(64), i, nullptr, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_prune_topk(s, nullptr, i, i, 1, 1, 4, i, i, nullptr, nullptr) == CF_ERR_INVALID_ARG);                       // alias
    EXPECT(cf_prune_topk(s, nullptr, i, i, 1, 1, 100000, fake<int32_t>(64), i, nullptr, nullptr) == CF_ERR_INVALID_ARG);
    auto assign = [&](int pos_begin, int pos_end, int strategy, int force, int32_t* new_start, int32_t* order) {
        return cf_assign_positions(i, i, i, 1, 4, pos_begin, pos_end, strategy, force, new_start, i, i, order, nullptr, nullptr);
    };
    EXPECT(assign(4, 4, CF_ALLOC_SORT, 0, i, fake<int32_t>(64)) == CF_ERR_RANGE);
    EXPECT(assign(-1, 100, CF_ALLOC_SORT, 0, i, fake<int32_t>(64)) == CF_ERR_RANGE);
    EXPECT(assign(4, 100, 7, 0, i, fake<int32_t>(64)) == CF_ERR_INVALID_ARG);
    EXPECT(assign(4, 100, CF_ALLOC_SORT, -2, i, fake<int32_t>(64)) == CF_ERR_INVALID_ARG);
    EXPECT(assign(4, 100, CF_ALLOC_SORT, 0, nullptr, fake<int32_t>(64)) == CF_ERR_INVALID_ARG);
    EXPECT(assign(4, 100, CF_ALLOC_SORT, 0, i, i) == CF_ERR_INVALID_ARG);                                                  // order aliases
    EXPECT(cf_gather_segments(fake<int64_t>(), i, i, i, i, i, i, 1, 4, 0, 0, 0, fake<cf_segment>(), i, 1, nullptr, nullptr) ==
           CF_ERR_INVALID_ARG);                                                                                            // seg_stride too small
}

static void assembly_and_aids() {
    cf_layer_desc d = desc();
    auto call = [&](void* k_final, void* v_final, int32_t* final_len, const void* v_self, int64_t ts, int64_t hs, int32_t max_seg_len,
                    int64_t capacity) {
        return cf_assemble_cache(&d, fake<void>(), fake<void>(0x100), 100, fake<void>(0x200), v_self, fake<int32_t>(), fake<cf_segment>(),
                                 fake<int32_t>(), 4, 1, 8, max_seg_len, fake<int64_t>(), capacity, ts, hs, k_final, v_final, final_len,
                                 nullptr, nullptr, nullptr);
    };
    void *kf = fake<void>(0x400), *vf = fake<void>(0x500);
    int32_t* fl = fake<int32_t>();
    const void* vs = fake<void>(0x300);
    EXPECT(call(nullptr, vf, fl, vs, 256, 128, 64, 500) == CF_ERR_INVALID_ARG);
    EXPECT(call(kf, vf, nullptr, vs, 256, 128, 64, 500) == CF_ERR_INVALID_ARG);
    EXPECT(call(kf, vf, fl, nullptr, 256, 128, 64, 500) == CF_ERR_INVALID_ARG);
    EXPECT(call(kf, vf, fl, vs, 100, 128, 64, 500) == CF_ERR_INVALID_ARG);
    EXPECT(call(kf, vf, fl, vs, 256, 132, 64, 500) == CF_ERR_INVALID_ARG);
    EXPECT(call(fake<void>(), vf, fl, vs, 256, 128, 64, 500) == CF_ERR_INVALID_ARG);          // aliases k_store
    EXPECT(call(kf, kf, fl, vs, 256, 128, 64, 500) == CF_ERR_INVALID_ARG);
    EXPECT(call(fake<void>(0x404), vf, fl, vs, 256, 128, 64, 500) == CF_ERR_INVALID_ARG);
    EXPECT(call(kf, vf, fl, vs, 256, 128, 0, 500) == CF_ERR_INVALID_ARG);
    EXPECT(call(kf, vf, fl, vs, 256, 128, 64, -1) == CF_ERR_INVALID_ARG);
    // measurement aids
    double ms = 0.0;
    int32_t n = 0;
    EXPECT(cf_profile_kernel_ms(&ms, &n) == CF_ERR_INVALID_ARG);                              // switched off
    EXPECT(cf_profile_kernel_ms(nullptr, &n) == CF_ERR_INVALID_ARG);
    EXPECT(cf_profile_kernel_events(0) == CF_OK);
    double flops = 1.0;
    EXPECT(cf_calibrate(CF_CALIB_READ, nullptr, nullptr, 1024, 16, 0, fake<void>(), &flops, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_calibrate(CF_CALIB_COPY, fake<void>(), fake<void>(), 1024, 16, 0, fake<void>(), &flops, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_calibrate(9, fake<void>(), fake<void>(0x1000), 1024, 16, 0, fake<void>(), &flops, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_calibrate(CF_CALIB_MFMA_BF16, nullptr, nullptr, 0, 16, 0, fake<void>(), &flops, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(cf_calibrate(CF_CALIB_READ, fake<void>(), nullptr, 1024, 0, 0, fake<void>(), &flops, nullptr) == CF_ERR_INVALID_ARG);
    EXPECT(flops == 0.0);
    EXPECT(cf_version() >= 100);
}

int main() {
    descriptors();
    workspace_plans();
    prefill();
    selection();
    assembly_and_aids();
    std::printf("%d checks, %d failed\n", g_checks, g_failures);
    return g_failures ? 1 : 0;
}
