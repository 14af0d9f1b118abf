// Runs the library's host code (scheduler, transfer engine, training step) against the host-only
// HIP stand-in of this directory.  Built and run by tests/test_engine_mock.py, plain and under
// the address/undefined and thread sanitizers.  Prints one line per check; exit code 0 = all
// passed.  `--control-race` runs a deliberately unfenced copy/compute pair instead, which the
// thread sanitizer must report (the control that shows the detector sees this kind of bug).
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <string>
#include <vector>

#include "../../include/superpipe.h"

static int g_failed = 0;
#define CHECK(cond, ...)                                             \
    do {                                                             \
        if (!(cond)) {                                               \
            printf("FAIL %s:%d: %s -- ", __FILE__, __LINE__, #cond); \
            printf(__VA_ARGS__);                                     \
            printf("\n");                                            \
            ++g_failed;                                              \
        }                                                            \
    } while (0)

// the stand-in kernels write arbitrary bit patterns (NaNs among them): compare bytes, not floats
static bool same(const std::vector<float>& a, const std::vector<float>& b) {
    return a.size() == b.size() && (a.empty() || !memcmp(a.data(), b.data(), a.size() * sizeof(float)));
}

struct Rig {
    sp_stack_desc desc;
    int L;
    size_t blob_bytes, grad_bytes;
    std::vector<void*> blobs, grads;
    hipStream_t compute, h2d, d2h;
    std::vector<float> x, t;

    Rig(int arch, int n_layers, int B, int S) {
        memset(&desc, 0, sizeof(desc));
        desc.struct_size = sizeof(desc);
        desc.n_layers = L = n_layers;
        desc.d_model = 64;
        desc.n_q_heads = 2;
        desc.n_kv_heads = 1;
        desc.head_dim = 64;
        desc.d_ffn = 128;
        desc.arch = arch;
        desc.causal = arch == SP_DECODER_SWIGLU_RMS;
        desc.norm_eps = 1e-5f;
        desc.max_batch = B;
        desc.max_seq = S;
        blob_bytes = sp_layer_blob_bytes(&desc);
        grad_bytes = sp_layer_grad_bytes(&desc);
        for (int l = 0; l < L; ++l) {
            unsigned char* b = static_cast<unsigned char*>(mock_pinned_alloc(blob_bytes));
            for (size_t i = 0; i < blob_bytes; ++i) b[i] = (unsigned char)((i * 131 + l * 17 + (i >> 9)) & 0xFF);
            blobs.push_back(b);
            grads.push_back(mock_pinned_alloc(grad_bytes));
        }
        compute = mock_stream_create();
        h2d = mock_stream_create();
        d2h = mock_stream_create();
        x.resize((size_t)B * S * 64);
        t.resize(x.size());
        for (size_t i = 0; i < x.size(); ++i) { x[i] = (float)(i % 97) * 0.01f; t[i] = (float)(i % 89) * 0.02f; }
    }
    ~Rig() {
        for (void* b : blobs) mock_pinned_free(b);
        for (void* g : grads) mock_pinned_free(g);
        mock_stream_destroy(compute);
        mock_stream_destroy(h2d);
        mock_stream_destroy(d2h);
    }
    void sync() {
        hipStreamSynchronize(compute);
        hipStreamSynchronize(h2d);
        hipStreamSynchronize(d2h);
    }
};

struct Handle {
    sp_handle h = nullptr;
    void* arena_raw = nullptr;
    unsigned char* arena = nullptr;
    uint64_t budget = 0;
    int rc = SP_OK;
    Handle(Rig& r, int k, int p, uint32_t flags, int budget_layers = 0, int pinned = 0, int units = 0, int frozen = 0) {
        const int mode = (flags & SP_FLAG_TRAINING) ? ((flags & SP_FLAG_KEEP_ACTIVATIONS) ? 2 : 1) : 0;
        const uint64_t slot = (r.blob_bytes + 4095) / 4096 * 4096;
        int nl = budget_layers ? budget_layers : k + p + (pinned > 0 ? pinned : 0);
        if (nl > r.L) nl = r.L;
        budget = sp_workspace_bytes(&r.desc, mode) + (uint64_t)nl * slot;
        arena_raw = malloc(budget + 4096);
        arena = reinterpret_cast<unsigned char*>(((uintptr_t)arena_raw + 4095) & ~(uintptr_t)4095);
        memset(arena, 0xEE, budget);
        sp_config cfg;
        memset(&cfg, 0, sizeof(cfg));
        cfg.struct_size = sizeof(cfg);
        cfg.resident_window_k = k;
        cfg.prefetch_depth_p = p;
        cfg.gpu_budget_bytes = budget;
        cfg.device_arena = arena;
        cfg.compute_stream = r.compute;
        cfg.h2d_stream = r.h2d;
        cfg.d2h_stream = (flags & SP_FLAG_TRAINING) ? r.d2h : nullptr;
        cfg.flags = flags;
        cfg.frozen_layers = frozen;
        cfg.pinned_layers = pinned;
        cfg.units_per_layer = units;
        cfg.delay_us = 300;
        rc = sp_create(&h, &r.desc, r.blobs.data(), &cfg);
    }
    ~Handle() {
        if (h) sp_destroy(h);
        free(arena_raw);
    }
};

static std::vector<float> forward(Rig& r, int k, int p, uint32_t flags, int B, int S, int calls = 1, int budget_layers = 0,
                                  int pinned = 0, int units = 0, sp_stats* st_out = nullptr) {
    Handle H(r, k, p, flags, budget_layers, pinned, units);
    std::vector<float> y((size_t)B * S * 64, -1.f);
    CHECK(H.rc == SP_OK, "sp_create: %s", sp_last_error(nullptr));
    if (H.rc != SP_OK) return y;
    for (int c = 0; c < calls; ++c) {
        int rc = sp_forward(H.h, r.x.data(), y.data(), B, S);
        CHECK(rc == SP_OK, "sp_forward: %s", sp_last_error(H.h));
        r.sync();
    }
    if (st_out) {
        st_out->struct_size = sizeof(*st_out);
        CHECK(sp_get_stats(H.h, st_out) == SP_OK, "stats");
    }
    return y;
}

static void test_forward_windows(int arch) {
    const int B = 2, S = 8;
    Rig r(arch, 6, B, S);
    const std::vector<float> base = forward(r, 8, 8, 0, B, S);
    struct { int k, p; uint32_t flags; int bl, pinned, units, calls; } cases[] = {
        {1, 1, 0, 0, 0, 0, 1},          {2, 1, SP_FLAG_POISON, 0, 0, 0, 2},        {1, 2, SP_FLAG_WRAP_PREFETCH, 0, 0, 0, 3},
        {2, 2, SP_FLAG_NO_OVERLAP, 0, 0, 0, 2}, {1, 1, 0, 1, 0, 0, 2},             {1, 1, SP_FLAG_WRAP_PREFETCH, 0, 2, 0, 3},
        {1, 1, SP_FLAG_WRAP_PREFETCH | SP_FLAG_POISON, 0, 4, 3, 3},              {1, 1, SP_FLAG_TIMING, 0, 0, 3, 2},
        {1, 1, SP_FLAG_DELAY | SP_FLAG_POISON | SP_FLAG_WRAP_PREFETCH, 0, 1, 0, 3}, {2, 1, SP_FLAG_DELAY, 0, 0, 3, 2},
    };
    for (auto& c : cases) {
        sp_stats st;
        const std::vector<float> y = forward(r, c.k, c.p, c.flags, B, S, c.calls, c.bl, c.pinned, c.units, &st);
        CHECK(same(y, base), "arch %d window (%d,%d) flags %u pinned %d units %d differs from the resident run", arch, c.k,
              c.p, c.flags, c.pinned, c.units);
        CHECK(st.calls == (uint64_t)c.calls, "calls");
        if (c.flags & SP_FLAG_TIMING) CHECK(st.n_ops == 6 * (c.units ? c.units : 1) && st.wall_ms >= 0.f, "trace");
    }
    // smaller batch / sequence than the workspace was made for; out-of-range shapes are refused
    {
        Handle H(r, 1, 1, 0);
        std::vector<float> y(1 * 5 * 64);
        CHECK(sp_forward(H.h, r.x.data(), y.data(), 1, 5) == SP_OK, "ragged");
        r.sync();
        CHECK(sp_forward(H.h, r.x.data(), y.data(), 3, 5) == SP_ERR_SHAPE, "B too large");
        CHECK(sp_forward(H.h, nullptr, y.data(), 1, 5) == SP_ERR_INVALID_ARG, "NULL x");
        CHECK(sp_forward(H.h, r.x.data(), y.data(), 1, 5) == SP_OK, "argument errors must leave the handle usable");
        r.sync();
        CHECK(sp_weights_updated(H.h, 2) == SP_OK && sp_weights_updated(H.h, 6) == SP_ERR_INVALID_ARG, "weights_updated");
        CHECK(sp_forward(H.h, r.x.data(), y.data(), 1, 5) == SP_OK, "after weights_updated");
        r.sync();
    }
    printf("ok forward windows arch %d\n", arch);
}

struct StepOut {
    std::vector<float> y, dx;
    float loss = 0;
    std::vector<std::vector<unsigned char>> grads;
    bool operator==(const StepOut& o) const {
        return same(y, o.y) && same(dx, o.dx) && !memcmp(&loss, &o.loss, sizeof(loss)) && grads == o.grads;
    }
};

static StepOut train(Rig& r, int k, int p, uint32_t flags, int B, int S, int calls, int budget_layers = 0, int pinned = 0,
                     int frozen = 0, bool want_dx = true) {
    StepOut o;
    Handle H(r, k, p, SP_FLAG_TRAINING | flags, budget_layers, pinned, 0, frozen);
    CHECK(H.rc == SP_OK, "sp_create(training): %s", sp_last_error(nullptr));
    if (H.rc != SP_OK) return o;
    o.y.assign((size_t)B * S * 64, -1.f);
    o.dx.assign(o.y.size(), -1.f);
    for (int c = 0; c < calls; ++c) {
        for (void* g : r.grads) memset(g, 0xFF, r.grad_bytes);
        int rc = sp_forward_backward(H.h, r.x.data(), r.t.data(), o.y.data(), &o.loss, want_dx ? o.dx.data() : nullptr,
                                     r.grads.data(), B, S);
        CHECK(rc == SP_OK, "sp_forward_backward: %s", sp_last_error(H.h));
        for (int l = r.L - 1; l >= frozen; --l) CHECK(sp_wait_gradient(H.h, l) == SP_OK, "wait_gradient %d", l);
        r.sync();
    }
    for (void* g : r.grads) o.grads.emplace_back(static_cast<unsigned char*>(g), static_cast<unsigned char*>(g) + r.grad_bytes);
    return o;
}

static void test_training(int arch) {
    const int B = 2, S = 9;       // 18 tokens: the weight-gradient contractions pad to 64
    Rig r(arch, 5, B, S);
    const StepOut base = train(r, 8, 8, 0, B, S, 1);
    CHECK(train(r, 1, 1, 0, B, S, 2) == base, "training (1,1) x2 differs");
    CHECK(train(r, 2, 1, SP_FLAG_POISON, B, S, 2) == base, "training (2,1) poison differs");
    CHECK(train(r, 1, 1, 0, B, S, 2, 1) == base, "training one slot differs");
    CHECK(train(r, 1, 1, 0, B, S, 3, 0, 2) == base, "training pinned differs");
    CHECK(train(r, 1, 2, SP_FLAG_KEEP_ACTIVATIONS, B, S, 2) == base, "training kept activations differs");
    CHECK(train(r, 1, 1, SP_FLAG_DELAY | SP_FLAG_POISON, B, S, 2) == base, "training with delays differs");
    const StepOut fr = train(r, 1, 1, 0, B, S, 2, 0, 0, 2, false);
    CHECK(!memcmp(&fr.loss, &base.loss, 4) && same(fr.y, base.y), "frozen: loss / y differ");
    for (int l = 0; l < r.L; ++l) {
        if (l >= 2) CHECK(fr.grads[l] == base.grads[l], "frozen: layer %d gradient differs", l);
        else CHECK(fr.grads[l] == std::vector<unsigned char>(r.grad_bytes, 0xFF), "frozen layer %d was written", l);
    }
    {
        Handle H(r, 1, 1, SP_FLAG_TRAINING);
        float loss;
        void* pageable = malloc(r.grad_bytes);
        std::vector<void*> g = r.grads;
        g[3] = pageable;
        CHECK(sp_forward_backward(H.h, r.x.data(), r.t.data(), nullptr, &loss, nullptr, g.data(), B, S) == SP_ERR_NOT_PINNED,
              "pageable gradient blob accepted");
        CHECK(sp_wait_gradient(H.h, 0) == SP_ERR_STATE, "wait_gradient before any step");
        CHECK(sp_forward_backward(H.h, r.x.data(), r.t.data(), nullptr, &loss, nullptr, r.grads.data(), B, S) == SP_OK, "step");
        r.sync();
        free(pageable);
    }
    printf("ok training arch %d\n", arch);
}

static void test_decode() {
    const int B = 2, S0 = 6, steps = 4, max_len = 16;
    Rig r(SP_DECODER_SWIGLU_RMS, 4, B, S0);
    std::vector<std::vector<float>> outs;
    for (int variant = 0; variant < 3; ++variant) {
        Handle H(r, variant == 0 ? 8 : 1, variant == 0 ? 8 : 1, variant == 2 ? (SP_FLAG_WRAP_PREFETCH | SP_FLAG_POISON) : 0, 0,
                 variant == 2 ? 1 : 0);
        const size_t cb = sp_kv_cache_bytes(&r.desc, B, max_len);
        std::vector<unsigned char> cache(cb, 0xFF);
        std::vector<float> y((size_t)B * S0 * 64), y1((size_t)B * 64), all;
        CHECK(sp_prefill(H.h, r.x.data(), y.data(), cache.data(), B, S0, max_len) == SP_OK, "prefill");
        r.sync();
        all = y;
        for (int s = 0; s < steps; ++s) {
            CHECK(sp_decode(H.h, r.x.data() + s * 64, y1.data(), cache.data(), B, S0 + s, max_len) == SP_OK, "decode");
            r.sync();
            all.insert(all.end(), y1.begin(), y1.end());
        }
        CHECK(sp_decode(H.h, r.x.data(), y1.data(), cache.data(), B, max_len, max_len) == SP_ERR_SHAPE, "pos beyond the cache");
        outs.push_back(all);
    }
    CHECK(same(outs[0], outs[1]) && same(outs[0], outs[2]), "decode outputs differ between windows");
    printf("ok decode\n");
}

// Fails the n-th call of `api` inside a pass, for n = 1, 2, ... until a pass gets through:
// every failing pass must return SP_ERR_HIP with a text naming the call, leave the handle FAILED
// (SP_ERR_STATE from then on) and destroyable; nothing may leak or be touched after free.
static void test_injected_failures(bool training) {
    const int B = 1, S = 8;
    Rig r(SP_DECODER_SWIGLU_RMS, 4, B, S);
    const char* apis[] = {"hipMemcpyAsync", "launch", "hipEventRecord", "hipStreamWaitEvent"};
    for (const char* api : apis) {
        int failures = 0;
        for (int n = 1; n < 4000; ++n) {
            Handle H(r, 1, 1, training ? SP_FLAG_TRAINING : SP_FLAG_WRAP_PREFETCH);
            CHECK(H.rc == SP_OK, "create");
            std::vector<float> y((size_t)B * S * 64), dx(y.size());
            float loss;
            mock_fail_nth(api, n);
            int rc = training ? sp_forward_backward(H.h, r.x.data(), r.t.data(), y.data(), &loss, dx.data(), r.grads.data(), B, S)
                              : sp_forward(H.h, r.x.data(), y.data(), B, S);
            mock_fail_nth(api, 0);
            r.sync();
            if (rc == SP_OK) break;          // n is beyond the calls one pass makes
            ++failures;
            CHECK(rc == SP_ERR_HIP, "%s #%d: rc %d", api, n, rc);
            const std::string msg = sp_last_error(H.h);
            CHECK(msg.find("FAILED") != std::string::npos && msg.find("failed:") != std::string::npos, "%s #%d: text '%s'", api, n,
                  msg.c_str());
            int rc2 = training ? sp_forward_backward(H.h, r.x.data(), r.t.data(), y.data(), &loss, dx.data(), r.grads.data(), B, S)
                               : sp_forward(H.h, r.x.data(), y.data(), B, S);
            CHECK(rc2 == SP_ERR_STATE, "%s #%d: a FAILED handle accepted another pass (rc %d)", api, n, rc2);
            CHECK(std::string(sp_last_error(H.h)) == msg, "the first failure's text must stay");
            sp_stats st;
            CHECK(sp_get_stats(H.h, &st) == SP_OK, "stats on a FAILED handle");
            CHECK(sp_weights_updated(H.h, 0) == SP_ERR_STATE, "weights_updated on a FAILED handle");
            sp_handle h = H.h;
            H.h = nullptr;
            CHECK(sp_destroy(h) == SP_OK, "%s #%d: destroy of a FAILED handle", api, n);
            CHECK(sp_destroy(h) == SP_ERR_STATE, "double destroy");
        }
        CHECK(failures >= 4, "%s: only %d failing positions exercised", api, failures);
        printf("ok injected %s failures (%s): %d positions\n", api, training ? "training step" : "forward", failures);
    }
    // event creation failing inside sp_create: no handle, nothing leaked
    int created = 0, positions = 0;
    for (int n = 1; n < 20000; n += 1 + n / 2, ++positions) {
        mock_fail_nth("hipEventCreateWithFlags", n);
        Handle H(r, 1, 1, training ? SP_FLAG_TRAINING | SP_FLAG_TIMING : SP_FLAG_TIMING);
        mock_fail_nth("hipEventCreateWithFlags", 0);
        if (H.rc == SP_OK) { created = n; break; }
        CHECK(H.rc == SP_ERR_HIP && H.h == nullptr, "create with failing event #%d: rc %d", n, H.rc);
        CHECK(strstr(sp_last_error(nullptr), "hipEventCreate") != nullptr, "text: %s", sp_last_error(nullptr));
    }
    CHECK(created > 10 && positions > 8, "event-creation failures exercised: %d up to call %d", positions, created);
    printf("ok injected event-creation failures: %d positions up to call %d\n", positions, created);
}

static void test_create_errors() {
    Rig r(SP_DECODER_SWIGLU_RMS, 3, 1, 8);
    void* pageable = malloc(r.blob_bytes);
    void* saved = r.blobs[1];
    r.blobs[1] = pageable;
    { Handle H(r, 1, 1, 0); CHECK(H.rc == SP_ERR_NOT_PINNED && !H.h, "pageable weight blob accepted"); }
    r.blobs[1] = saved;
    free(pageable);
    { Handle H(r, 1, 1, 0, 0, 0, 2); CHECK(H.rc == SP_ERR_INVALID_ARG, "units = 2 accepted"); }
    { Handle H(r, 1, 1, SP_FLAG_TRAINING, 0, 0, 3); CHECK(H.rc == SP_ERR_INVALID_ARG, "units with training accepted"); }
    printf("ok create errors\n");
}

// The control: a copy into a buffer on one stream and a kernel reading it on another, with no
// event between them.  Under the thread sanitizer this must be reported as a data race.
static void control_race() {
    hipStream_t a = mock_stream_create(), b = mock_stream_create();
    std::vector<uint32_t> src(1 << 16, 7u), dst(1 << 16, 0u), sink(1 << 16);
    for (int i = 0; i < 50; ++i) {
        hipMemcpyAsync(dst.data(), src.data(), dst.size() * 4, hipMemcpyHostToDevice, a);
        hipMemcpyAsync(sink.data(), dst.data(), dst.size() * 4, hipMemcpyDeviceToHost, b);   // reads dst unfenced
    }
    hipStreamSynchronize(a);
    hipStreamSynchronize(b);
    mock_stream_destroy(a);
    mock_stream_destroy(b);
    printf("control done\n");
}

int main(int argc, char** argv) {
    setvbuf(stdout, nullptr, _IOLBF, 0);
    if (argc > 1 && !strcmp(argv[1], "--control-race")) {
        control_race();
        return 0;
    }
    test_create_errors();
    test_forward_windows(SP_DECODER_SWIGLU_RMS);
    test_forward_windows(SP_ENCODER_GELU_LN);
    test_training(SP_DECODER_SWIGLU_RMS);
    test_training(SP_ENCODER_GELU_LN);
    test_decode();
    test_injected_failures(false);
    test_injected_failures(true);
    printf(g_failed ? "FAILED: %d checks\n" : "all checks passed\n", g_failed);
    return g_failed ? 1 : 0;
}
