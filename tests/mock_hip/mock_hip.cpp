// Host-only stand-in for the HIP runtime and for the library's kernel launchers (see
// hip/hip_runtime.h in this directory).  TEST INFRASTRUCTURE, built only by
// tests/test_engine_mock.py.
//
// Every stream is a thread with an in-order queue; an event completes when its stream reaches
// the record; hipStreamWaitEvent makes a stream wait for the record that was the event's latest
// one when the wait was enqueued -- the HIP semantics the engine relies on.  A "kernel" reads
// every byte of its input operands and overwrites its output operands with values derived from
// them, so (1) results depend on the weights that were in the slot when the kernel ran: a stack
// output is only reproducible across window settings if every layer computed on the right bytes;
// (2) under ThreadSanitizer an unfenced overlap of a layer copy with a layer compute is a data
// race on the slot's bytes; (3) under AddressSanitizer an operand extent beyond the arena or a
// host blob is an out-of-bounds access.
#include <hip/hip_runtime.h>
#include <stdlib.h>
#include <string.h>
#include <unistd.h>

#include <chrono>
#include <condition_variable>
#include <deque>
#include <functional>
#include <map>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "sp_kernels.h"

struct mockEvent {
    std::mutex mu;
    std::condition_variable cv;
    uint64_t recorded = 0;   // records enqueued (host order)
    uint64_t done = 0;       // latest record the stream has reached
    std::chrono::steady_clock::time_point when;
};

struct mockStream {
    std::mutex mu;
    std::condition_variable cv, idle_cv;
    std::deque<std::function<void()>> q;
    bool stop = false, busy = false;
    std::thread th;
    mockStream() : th([this] { run(); }) {}
    ~mockStream() {
        {
            std::lock_guard<std::mutex> lk(mu);
            stop = true;
        }
        cv.notify_all();
        th.join();
    }
    void run() {
        for (;;) {
            std::function<void()> f;
            {
                std::unique_lock<std::mutex> lk(mu);
                cv.wait(lk, [&] { return stop || !q.empty(); });
                if (q.empty()) return;
                f = std::move(q.front());
                q.pop_front();
                busy = true;
            }
            f();
            {
                std::lock_guard<std::mutex> lk(mu);
                busy = false;
            }
            idle_cv.notify_all();
        }
    }
    void push(std::function<void()> f) {
        {
            std::lock_guard<std::mutex> lk(mu);
            q.push_back(std::move(f));
        }
        cv.notify_one();
    }
    void drain() {
        std::unique_lock<std::mutex> lk(mu);
        idle_cv.wait(lk, [&] { return q.empty() && !busy; });
    }
};

namespace {

std::mutex g_mu;
std::map<std::string, int> g_fail;       // api -> calls left until the failing one
std::map<std::string, long> g_count;
std::map<const char*, size_t> g_pinned;  // base -> bytes
mockStream* g_default = nullptr;

bool inject(const char* api) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_count[api]++;
    auto it = g_fail.find(api);
    if (it == g_fail.end() || it->second <= 0) return false;
    if (--it->second == 0) {
        g_fail.erase(it);
        return true;
    }
    return false;
}

mockStream* S(hipStream_t st) {
    if (st) return st;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_default) g_default = new mockStream();
    return g_default;
}

}  // namespace

hipStream_t mock_stream_create(void) { return new mockStream(); }
void mock_stream_destroy(hipStream_t st) { delete st; }

void* mock_pinned_alloc(size_t bytes) {
    char* p = static_cast<char*>(malloc(bytes ? bytes : 1));
    std::lock_guard<std::mutex> lk(g_mu);
    g_pinned[p] = bytes;
    return p;
}
void mock_pinned_free(void* p) {
    {
        std::lock_guard<std::mutex> lk(g_mu);
        g_pinned.erase(static_cast<const char*>(p));
    }
    free(p);
}
void mock_fail_nth(const char* api, int n) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (n > 0) g_fail[api] = n; else g_fail.erase(api);
}
long mock_count(const char* api) {
    std::lock_guard<std::mutex> lk(g_mu);
    return g_count[api];
}
void mock_count_reset(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_count.clear();
}

hipError_t hipEventCreateWithFlags(hipEvent_t* ev, unsigned) {
    if (inject("hipEventCreateWithFlags")) return hipErrorOutOfMemory;
    *ev = new mockEvent();
    return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t* ev) { return hipEventCreateWithFlags(ev, 0); }
hipError_t hipEventDestroy(hipEvent_t ev) {
    delete ev;
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t ev, hipStream_t st) {
    if (inject("hipEventRecord")) return hipErrorUnknown;
    uint64_t seq;
    {
        std::lock_guard<std::mutex> lk(ev->mu);
        seq = ++ev->recorded;
    }
    S(st)->push([ev, seq] {
        {
            std::lock_guard<std::mutex> lk(ev->mu);
            if (seq > ev->done) {
                ev->done = seq;
                ev->when = std::chrono::steady_clock::now();
            }
        }
        ev->cv.notify_all();
    });
    return hipSuccess;
}
hipError_t hipEventSynchronize(hipEvent_t ev) {
    std::unique_lock<std::mutex> lk(ev->mu);
    const uint64_t target = ev->recorded;
    ev->cv.wait(lk, [&] { return ev->done >= target; });
    return hipSuccess;
}
hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b) {
    std::chrono::steady_clock::time_point ta, tb;
    {
        std::lock_guard<std::mutex> lk(a->mu);
        ta = a->when;
    }
    {
        std::lock_guard<std::mutex> lk(b->mu);
        tb = b->when;
    }
    *ms = std::chrono::duration<float, std::milli>(tb - ta).count();
    return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t st, hipEvent_t ev, unsigned) {
    if (inject("hipStreamWaitEvent")) return hipErrorUnknown;
    uint64_t target;
    {
        std::lock_guard<std::mutex> lk(ev->mu);
        target = ev->recorded;     // the latest record at the time of this call; 0 = never recorded: no wait
    }
    S(st)->push([ev, target] {
        std::unique_lock<std::mutex> lk(ev->mu);
        ev->cv.wait(lk, [&] { return ev->done >= target; });
    });
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t st) {
    S(st)->drain();
    return hipSuccess;
}
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t st) {
    if (inject("hipMemcpyAsync")) return hipErrorUnknown;
    S(st)->push([=] { memcpy(dst, src, n); });
    return hipSuccess;
}
hipError_t hipPointerGetAttributes(hipPointerAttribute_t* at, const void* p) {
    std::lock_guard<std::mutex> lk(g_mu);
    const char* c = static_cast<const char*>(p);
    for (auto& kv : g_pinned)
        if (c >= kv.first && c < kv.first + kv.second) {
            at->type = hipMemoryTypeHost;
            return hipSuccess;
        }
    at->type = hipMemoryTypeUnregistered;
    return hipErrorInvalidValue;
}
hipError_t hipFuncSetAttribute(const void*, hipFuncAttribute, int) { return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
const char* hipGetErrorString(hipError_t e) {
    switch (e) {
        case hipSuccess: return "no error";
        case hipErrorInvalidValue: return "invalid argument";
        case hipErrorOutOfMemory: return "out of memory";
        default: return "injected failure";
    }
}

// ---- kernel stand-ins ------------------------------------------------------------------
namespace {

struct Span { const void* p; size_t n; };
struct MSpan { void* p; size_t n; };

// 64-bit FNV-1a over every byte of the inputs, then the outputs are filled from a generator
// seeded with it.  rw spans are read before anything is written.
hipError_t launch(hipStream_t st, uint64_t salt, std::vector<Span> in, std::vector<MSpan> out) {
    if (inject("launch")) return hipErrorUnknown;
    S(st)->push([salt, in, out] {
        uint64_t h = 1469598103934665603ull ^ salt;
        for (const Span& s : in) {
            const unsigned char* b = static_cast<const unsigned char*>(s.p);
            for (size_t i = 0; i < s.n; ++i) h = (h ^ b[i]) * 1099511628211ull;
        }
        for (const MSpan& s : out) {
            unsigned char* b = static_cast<unsigned char*>(s.p);
            for (size_t i = 0; i < s.n; ++i) {
                h = h * 6364136223846793005ull + 1442695040888963407ull;
                b[i] = (unsigned char)(h >> 56);
            }
        }
    });
    return hipSuccess;
}

size_t operand_bytes(int rows, int ld, int form, int K) {
    // KMAJOR: element (r, k) at r * ld + k;  RMAJOR: at k * ld + r
    const size_t last = form == OP_KMAJOR ? (size_t)(rows - 1) * ld + K : (size_t)(K - 1) * ld + rows;
    return last * 2;
}

}  // namespace

hipError_t spk_launch_gemm(hipStream_t st, int epi, const GemmArgs& g) {
    if (g.M <= 0) return hipSuccess;
    if (g.K % 64 || g.N % 8) return hipErrorInvalidValue;
    const int wrows = epi == EPI_SWIGLU_BF16 ? 2 * g.N : g.N;
    const size_t csz = (epi == EPI_RESID_F32 || epi == EPI_F32) ? 4 : 2;
    std::vector<Span> in = {{g.A, operand_bytes(g.M, g.lda, g.a_form, g.K)}, {g.W, operand_bytes(wrows, g.ldw, g.w_form, g.K)}};
    if (g.bias) in.push_back({g.bias, (size_t)g.N * 2});
    if (epi == EPI_RESID_F32) in.push_back({g.R, ((size_t)(g.M - 1) * g.ldr + g.N) * 4});
    // a strided output is written row by row (the gaps belong to other tensors)
    std::vector<MSpan> out;
    for (int m = 0; m < g.M; ++m) out.push_back({static_cast<char*>(g.C) + (size_t)m * g.ldc * csz, (size_t)g.N * csz});
    return launch(st, 1, in, out);
}
hipError_t spk_launch_gemm_skinny(hipStream_t st, int epi, const GemmArgs& g) { return spk_launch_gemm(st, epi, g); }
GemmPlan spk_gemm_plan_host(int, int, int, int M, int) { return GemmPlan{1, M, 0}; }

hipError_t spk_launch_norm(hipStream_t st, const float* h, const bf16_t* gain, const bf16_t* bias, bf16_t* out, int T,
                           int d, float) {
    if (T <= 0) return hipSuccess;
    std::vector<Span> in = {{h, (size_t)T * d * 4}, {gain, (size_t)d * 2}};
    if (bias) in.push_back({bias, (size_t)d * 2});
    return launch(st, 2, in, {{out, (size_t)T * d * 2}});
}
hipError_t spk_launch_swiglu(hipStream_t st, const bf16_t* gu, bf16_t* z, int T, int f) {
    return launch(st, 3, {{gu, (size_t)T * 2 * f * 2}}, {{z, (size_t)T * f * 2}});
}
hipError_t spk_launch_attention(hipStream_t st, const bf16_t* qkv, bf16_t* o, float* lse, const AttnShape& a) {
    const size_t T = (size_t)a.B * a.S;
    std::vector<MSpan> out = {{o, T * a.Hq * a.hd * 2}};
    if (lse) out.push_back({lse, T * a.Hq * 4});
    return launch(st, 4, {{qkv, T * a.ld_qkv * 2}}, out);
}
hipError_t spk_launch_kv_append(hipStream_t st, const bf16_t* qkv, int ld_qkv, bf16_t* kt, bf16_t* v, int B, int S, int pos0,
                                int, int Hkv, int hd, int max_len) {
    if (pos0 < 0 || pos0 + S > max_len) return hipErrorInvalidValue;
    // the stored positions only: [b][h][e][pos] for the keys, [b][h][pos][e] for the values
    std::vector<MSpan> out;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            for (int e = 0; e < hd; ++e) out.push_back({kt + (((size_t)b * Hkv + h) * hd + e) * max_len + pos0, (size_t)S * 2});
            out.push_back({v + (((size_t)b * Hkv + h) * max_len + pos0) * hd, (size_t)S * hd * 2});
        }
    return launch(st, 5, {{qkv, (size_t)B * S * ld_qkv * 2}}, out);
}
hipError_t spk_launch_decode_attention(hipStream_t st, const bf16_t* qkv, int ld_qkv, const bf16_t* kt, const bf16_t* v,
                                       bf16_t* o, int ld_o, int B, int n, int max_len, int, int Hkv, int hd) {
    std::vector<Span> in = {{qkv, (size_t)B * ld_qkv * 2}};
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            for (int e = 0; e < hd; ++e) in.push_back({kt + (((size_t)b * Hkv + h) * hd + e) * max_len, (size_t)n * 2});
            in.push_back({v + ((size_t)b * Hkv + h) * max_len * hd, (size_t)n * hd * 2});
        }
    return launch(st, 6, in, {{o, (size_t)B * ld_o * 2}});
}
hipError_t spk_launch_copy_f32(hipStream_t st, const float* src, float* dst, size_t n) {
    if (n == 0 || src == dst) return hipSuccess;
    if (inject("launch")) return hipErrorUnknown;
    S(st)->push([=] { memmove(dst, src, n * 4); });
    return hipSuccess;
}
hipError_t spk_launch_fill_u32(hipStream_t st, uint32_t* dst, uint32_t v, size_t n) {
    if (n == 0) return hipSuccess;
    if (inject("launch")) return hipErrorUnknown;
    S(st)->push([=] { for (size_t i = 0; i < n; ++i) dst[i] = v; });
    return hipSuccess;
}
hipError_t spk_launch_spin(hipStream_t st, int micros) {
    if (micros <= 0) return hipSuccess;
    if (inject("launch")) return hipErrorUnknown;
    S(st)->push([=] { usleep((useconds_t)std::min(micros, 2000)); });
    return hipSuccess;
}
hipError_t spk_launch_mse(hipStream_t st, const float* y, const float* t, float* dy, bf16_t* dyb, float* part, float* loss,
                          size_t n) {
    // y may alias dy (the loss turns the stream buffer into its gradient in place)
    return launch(st, 7, {{y, n * 4}, {t, n * 4}}, {{dy, n * 4}, {dyb, n * 2}, {part, (size_t)SPK_MSE_PARTS * 4}, {loss, 4}});
}
hipError_t spk_launch_swiglu_bwd(hipStream_t st, const bf16_t* dz, bf16_t* gu, int T, int f) {
    return launch(st, 8, {{dz, (size_t)T * f * 2}, {gu, (size_t)T * 2 * f * 2}}, {{gu, (size_t)T * 2 * f * 2}});
}
hipError_t spk_launch_rmsnorm_bwd(hipStream_t st, const float* da, const float* h, const bf16_t* gain, float* dh_io,
                                  bf16_t* dhb, float* part, float* dgain, int T, int d, float) {
    const size_t n = (size_t)T * d;
    return launch(st, 9, {{da, n * 4}, {h, n * 4}, {gain, (size_t)d * 2}, {dh_io, n * 4}},
                  {{dh_io, n * 4}, {dhb, n * 2}, {part, (size_t)SPK_NORM_BWD_BLOCKS * d * 4}, {dgain, (size_t)d * 4}});
}
hipError_t spk_launch_layernorm_bwd(hipStream_t st, const float* da, const float* h, const bf16_t* gain, float* dh_io,
                                    bf16_t* dhb, float* part, float* dgain, float* dbias, int T, int d, float) {
    const size_t n = (size_t)T * d;
    return launch(st, 10, {{da, n * 4}, {h, n * 4}, {gain, (size_t)d * 2}, {dh_io, n * 4}},
                  {{dh_io, n * 4}, {dhb, n * 2}, {part, (size_t)SPK_NORM_BWD_BLOCKS * 2 * d * 4}, {dgain, (size_t)d * 4},
                   {dbias, (size_t)d * 4}});
}
hipError_t spk_launch_gelu(hipStream_t st, const bf16_t* u, bf16_t* z, size_t n) {
    return launch(st, 11, {{u, n * 2}}, {{z, n * 2}});
}
hipError_t spk_launch_gelu_bwd(hipStream_t st, const bf16_t* dz, bf16_t* u, size_t n) {
    return launch(st, 12, {{dz, n * 2}, {u, n * 2}}, {{u, n * 2}});
}
hipError_t spk_launch_colsum_bf16(hipStream_t st, const bf16_t* src, int ld, int T, int n, float* part, float* out) {
    return launch(st, 13, {{src, ((size_t)(T - 1) * ld + n) * 2}},
                  {{part, (size_t)SPK_NORM_BWD_BLOCKS * n * 4}, {out, (size_t)n * 4}});
}
hipError_t spk_launch_f32_to_bf16(hipStream_t st, const float* src, bf16_t* dst, size_t n) {
    return launch(st, 14, {{src, n * 4}}, {{dst, n * 2}});
}
hipError_t spk_launch_attn_delta(hipStream_t st, const bf16_t* dO, const bf16_t* O, float* delta, int B, int S, int Hq, int hd) {
    const size_t n = (size_t)B * S * Hq * hd;
    return launch(st, 15, {{dO, n * 2}, {O, n * 2}}, {{delta, (size_t)B * S * Hq * 4}});
}
hipError_t spk_launch_attention_bwd(hipStream_t st, const AttnBwdArgs& g, const AttnShape& a) {
    const size_t T = (size_t)a.B * a.S;
    return launch(st, 16, {{g.qkv, T * a.ld_qkv * 2}, {g.dO, T * a.Hq * a.hd * 2}, {g.lse, T * a.Hq * 4}, {g.delta, T * a.Hq * 4}},
                  {{g.dqkv, T * a.ld_qkv * 2}});
}
