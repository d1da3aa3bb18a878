// Host-side cost of the C ABI measured from C++, with no Python in the loop: wall-clock per call with a
// synchronisation after every call, pure enqueue rate, and the throughput of independent steps issued
// round-robin on several HIP streams (default priority), each with its own buffers.
//
//   ragged_call_cost [B] [keep_percent] [steps]        (defaults: 32 20 20000; N=197, H=12, D=64, fp16)
//
// Inputs are synthetic (a 64-bit LCG): the keep mask keeps token 0 of every image and every other token
// with the given probability; features and Q/K/V are small fp16 values.  Nothing is checked here --
// parity lives in the test-suite; this program only times calls.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "ragged.h"

namespace {

#define HIP_OK(call)                                                                              \
    do {                                                                                          \
        hipError_t e_ = (call);                                                                   \
        if (e_ != hipSuccess) {                                                                   \
            std::fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));                \
            std::exit(1);                                                                         \
        }                                                                                         \
    } while (0)
#define RAGGED_OKAY(call)                                                                         \
    do {                                                                                          \
        int s_ = (call);                                                                          \
        if (s_ != RAGGED_OK) {                                                                    \
            std::fprintf(stderr, "%s failed: %s\n", #call, ragged_status_string(s_));             \
            std::exit(1);                                                                         \
        }                                                                                         \
    } while (0)

struct Lcg {
    uint64_t s;
    uint32_t next() { s = s * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(s >> 33); }
};

// fp16 bit pattern of a value in [-1, 1) with 10 random mantissa bits
uint16_t small_half(Lcg& r) {
    const uint32_t u = r.next();
    return (uint16_t)(((u & 1u) << 15) | (14u << 10) | ((u >> 1) & 0x3ffu));   // +-[0.5, 1)
}

struct Buffers {
    void *x, *q, *k, *v, *packed, *o, *out;
    uint8_t* keep;
    int32_t *cu, *gidx;
};

template <typename T>
T* device_copy(const std::vector<T>& h) {
    T* d = nullptr;
    HIP_OK(hipMalloc(&d, h.size() * sizeof(T)));
    HIP_OK(hipMemcpy(d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
    return d;
}

double seconds_since(std::chrono::steady_clock::time_point t0) {
    return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
}

}  // namespace

int main(int argc, char** argv) {
    const int B = argc > 1 ? std::atoi(argv[1]) : 32;
    const int keep_percent = argc > 2 ? std::atoi(argv[2]) : 20;
    const int steps = argc > 3 ? std::atoi(argv[3]) : 20000;
    const int N = 197, H = 12, D = 64, C = H * D;
    if (B < 1 || B > 4096 || keep_percent < 0 || keep_percent > 100 || steps < 1) {
        std::fprintf(stderr, "usage: ragged_call_cost [B 1..4096] [keep_percent 0..100] [steps]\n");
        return 2;
    }
    const int64_t cap = (int64_t)B * N;
    const int kSets = 4;
    Lcg rng{12345};
    std::vector<uint8_t> keep((size_t)cap);
    int T = 0;
    for (int i = 0; i < B; ++i)
        for (int t = 0; t < N; ++t) {
            const bool kp = t == 0 || (int)(rng.next() % 100u) < keep_percent;
            keep[(size_t)i * N + t] = kp ? 1 : 0;
            T += kp;
        }
    std::vector<uint16_t> feat((size_t)cap * C), qkv((size_t)cap * C);
    for (auto& e : feat) e = small_half(rng);
    for (auto& e : qkv) e = small_half(rng);

    std::vector<Buffers> sets(kSets);
    std::vector<hipStream_t> streams(kSets);
    for (int s = 0; s < kSets; ++s) {
        Buffers& b = sets[s];
        b.x = device_copy(feat);
        b.q = device_copy(qkv);
        b.k = device_copy(qkv);
        b.v = device_copy(qkv);
        b.keep = device_copy(keep);
        HIP_OK(hipMalloc(&b.packed, (size_t)cap * C * 2));
        HIP_OK(hipMalloc(&b.o, (size_t)cap * C * 2));
        HIP_OK(hipMalloc(&b.out, (size_t)cap * C * 2));
        HIP_OK(hipMalloc(&b.cu, (size_t)(B + 1) * 4));
        HIP_OK(hipMalloc(&b.gidx, (size_t)cap * 4));
        HIP_OK(hipStreamCreateWithFlags(&streams[s], hipStreamNonBlocking));
    }
    auto step = [&](int s) {
        const Buffers& b = sets[s];
        RAGGED_OKAY(ragged_pack_attn_unpack(b.x, b.keep, b.q, b.k, b.v, B, N, H, D, 0.125f, RAGGED_F16, b.packed, cap, b.cu,
                                            b.gidx, b.o, b.out, 0, streams[s]));
    };
    auto three = [&](int s) {
        const Buffers& b = sets[s];
        RAGGED_OKAY(ragged_pack(b.x, b.keep, B, N, C, RAGGED_F16, b.packed, cap, b.cu, b.gidx, streams[s]));
        RAGGED_OKAY(ragged_attn(b.q, b.k, b.v, b.o, b.cu, B, N, H, D, 0.125f, RAGGED_F16, RAGGED_F16, streams[s]));
        RAGGED_OKAY(ragged_unpack(b.o, b.keep, b.cu, b.gidx, B, N, C, RAGGED_F16, b.out, 0, streams[s]));
    };
    for (int s = 0; s < kSets; ++s) { step(s); three(s); }
    HIP_OK(hipDeviceSynchronize());
    std::printf("{\"B\": %d, \"N\": %d, \"H\": %d, \"D\": %d, \"keep_percent\": %d, \"T\": %d, \"steps\": %d", B, N, H, D,
                keep_percent, T, steps);

    // 1. one call + synchronisation, per call
    {
        const int reps = steps < 2000 ? steps : 2000;
        auto t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < reps; ++i) { RAGGED_OKAY(ragged_noop(B * H * 4, streams[0])); HIP_OK(hipStreamSynchronize(streams[0])); }
        std::printf(", \"noop_call_and_sync_us\": %.3f", seconds_since(t0) / reps * 1e6);
        t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < reps; ++i) { step(0); HIP_OK(hipStreamSynchronize(streams[0])); }
        std::printf(", \"step_call_and_sync_us\": %.3f", seconds_since(t0) / reps * 1e6);
    }
    // 2. back-to-back calls on one stream, one synchronisation at the end
    {
        auto t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < steps; ++i) RAGGED_OKAY(ragged_noop(B * H * 4, streams[0]));
        HIP_OK(hipStreamSynchronize(streams[0]));
        std::printf(", \"noop_back_to_back_us\": %.3f", seconds_since(t0) / steps * 1e6);
        t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < steps; ++i) step(0);
        HIP_OK(hipStreamSynchronize(streams[0]));
        const double one = seconds_since(t0) / steps;
        std::printf(", \"step_one_launch_us\": %.3f, \"step_one_launch_tokens_per_s\": %.0f", one * 1e6, T / one);
        t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < steps; ++i) three(0);
        HIP_OK(hipStreamSynchronize(streams[0]));
        std::printf(", \"step_three_launches_us\": %.3f", seconds_since(t0) / steps * 1e6);
    }
    // 3. independent steps round-robin on 2, 3, 4 streams
    for (int ns = 2; ns <= kSets; ++ns) {
        HIP_OK(hipDeviceSynchronize());
        auto t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < steps; ++i) step(i % ns);
        HIP_OK(hipDeviceSynchronize());
        const double per = seconds_since(t0) / steps;
        std::printf(", \"step_on_%d_streams_us\": %.3f, \"step_on_%d_streams_tokens_per_s\": %.0f", ns, per * 1e6, ns, T / per);
    }
    std::printf("}\n");
    return 0;
}
