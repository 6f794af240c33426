// Exercises the host side of libsom (argument checks, error reporting, workspace and event bookkeeping, the chunked
// loaders with their reader threads) in a build whose HOST code carries AddressSanitizer and
// UndefinedBehaviorSanitizer instrumentation; device code is built as usual.  Test infrastructure: built by
// paper_2604_26555_amd/build.py (build_host_checked) against the instrumented library, run by
// tests/test_host_sanitizers.py.  Exit status 0 = every expectation held and no sanitizer report.
//
//   host_shell_check            calls that need no GPU: error strings, null contexts, creation on a missing device
//   host_shell_check --device   the same, then one context on device 0: streamed epochs from memory and from a file
//                               (several chunks, reader threads), the short-file and bad-argument paths, a resident
//                               epoch, repeated create / destroy
#include <hip/hip_runtime_api.h>

#include <fcntl.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <unistd.h>

#include <vector>

#include "som.h"

static int failures = 0;

#define EXPECT(cond)                                                            \
    do {                                                                        \
        if (!(cond)) {                                                          \
            fprintf(stderr, "line %d: expectation failed: %s\n", __LINE__, #cond); \
            ++failures;                                                         \
        }                                                                       \
    } while (0)

#define HIP_OK(call)                                                            \
    do {                                                                        \
        hipError_t e_ = (call);                                                 \
        if (e_ != hipSuccess) {                                                 \
            fprintf(stderr, "line %d: %s: %s\n", __LINE__, #call, hipGetErrorString(e_)); \
            return 1;                                                           \
        }                                                                       \
    } while (0)

static void without_a_context()
{
    for (int code = 1; code >= -8; --code) EXPECT(som_strerror(code) != nullptr && som_strerror(code)[0] != 0);
    EXPECT(som_last_error(nullptr) != nullptr);
    EXPECT(som_create(nullptr, 0, nullptr) == SOM_EINVAL);
    som_ctx* ctx = (som_ctx*)0x1;
    EXPECT(som_create(&ctx, -1, nullptr) < 0 && ctx == nullptr);
    EXPECT(som_create(&ctx, 1 << 20, nullptr) < 0 && ctx == nullptr);
    som_destroy(nullptr);
    float x = 0.f;
    int32_t b = 0;
    EXPECT(som_sync(nullptr) < 0);
    EXPECT(som_set_search(nullptr, SOM_SEARCH_AUTO) < 0);
    EXPECT(som_set_reproducible(nullptr, 1) < 0);
    EXPECT(som_set_safeguard(nullptr, SOM_SAFEGUARD_THRESHOLD) < 0);
    EXPECT(som_set_update_rule(nullptr, 1.0, 0.0, nullptr) < 0);
    EXPECT(som_profile(nullptr, 1) < 0);
    EXPECT(som_bmu(nullptr, &x, 1, 1, 1, nullptr, 1, &x, 1, &b, nullptr, nullptr) < 0);
    EXPECT(som_epoch(nullptr, &x, 1, 1, 1, nullptr, 1, &x, 1, &x, 1.0, SOM_KERNEL_GAUSSIAN, 0.0, nullptr) < 0);
    EXPECT(som_epoch_host(nullptr, &x, 1, 1, 1, 0, &x, 1, &x, 1.0, SOM_KERNEL_GAUSSIAN, 0.0, nullptr) < 0);
    EXPECT(som_epoch_file(nullptr, 0, 0, 1, 1, 1, &x, 1, &x, 1.0, SOM_KERNEL_GAUSSIAN, 0.0, nullptr) < 0);
    EXPECT(som_topology(nullptr, &x, 1, 1, SOM_TOPOLOGY_MST, &x) < 0);
}

// uniform in [0, 1): a 64-bit linear congruential step, top 24 bits
static float next_uniform(unsigned long long& s)
{
    s = s * 6364136223846793005ull + 1442695040888963407ull;
    return (float)(s >> 40) * (1.0f / 16777216.0f);
}

static int with_a_device()
{
    const int64_t N = 700000;              // 22.4 MB: chunks of 300000 rows are read by several threads each
    const int32_t D = 8, K = 64, side = 8;
    const int64_t chunk = 300000;
    std::vector<float> X((size_t)N * D), W0((size_t)K * D), G((size_t)K * K);
    unsigned long long seed = 12345;
    for (float& v : X) v = next_uniform(seed);
    for (int k = 0; k < K; ++k) memcpy(&W0[(size_t)k * D], &X[(size_t)(k * 977) * D], D * sizeof(float));
    for (int p = 0; p < K; ++p)
        for (int q = 0; q < K; ++q)
            G[(size_t)p * K + q] = hypotf((float)(p % side - q % side), (float)(p / side - q / side));

    char path[] = "/tmp/som_host_shell_XXXXXX";
    const int fd = mkstemp(path);
    EXPECT(fd >= 0);
    if (fd < 0) return 1;
    const size_t bytes = X.size() * sizeof(float);
    size_t done = 0;
    while (done < bytes) {
        const ssize_t w = write(fd, (const char*)X.data() + done, bytes - done);
        if (w <= 0) break;
        done += (size_t)w;
    }
    EXPECT(done == bytes);

    float *Wd = nullptr, *Gd = nullptr, *Xd = nullptr;
    HIP_OK(hipMalloc((void**)&Wd, W0.size() * sizeof(float)));
    HIP_OK(hipMalloc((void**)&Gd, G.size() * sizeof(float)));
    HIP_OK(hipMalloc((void**)&Xd, bytes));
    HIP_OK(hipMemcpy(Gd, G.data(), G.size() * sizeof(float), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(Xd, X.data(), bytes, hipMemcpyHostToDevice));

    std::vector<float> W_file(W0.size()), W_host(W0.size()), W_res(W0.size()), W_after(W0.size());
    for (int round = 0; round < 2; ++round) {          // a context is created, used and destroyed twice
        som_ctx* ctx = nullptr;
        EXPECT(som_create(&ctx, 0, nullptr) == SOM_OK && ctx != nullptr);
        if (!ctx) return 1;
        som_stats st;

        HIP_OK(hipMemcpy(Wd, W0.data(), W0.size() * sizeof(float), hipMemcpyHostToDevice));
        EXPECT(som_epoch_file(ctx, fd, 0, N, D, chunk, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_OK);
        EXPECT(st.m == N);
        HIP_OK(hipMemcpy(W_file.data(), Wd, W0.size() * sizeof(float), hipMemcpyDeviceToHost));

        HIP_OK(hipMemcpy(Wd, W0.data(), W0.size() * sizeof(float), hipMemcpyHostToDevice));
        EXPECT(som_epoch_host(ctx, X.data(), N, D, chunk, 0, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_OK);
        HIP_OK(hipMemcpy(W_host.data(), Wd, W0.size() * sizeof(float), hipMemcpyDeviceToHost));

        HIP_OK(hipMemcpy(Wd, W0.data(), W0.size() * sizeof(float), hipMemcpyHostToDevice));
        EXPECT(som_epoch(ctx, Xd, N, D, D, nullptr, N, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_OK);
        HIP_OK(hipMemcpy(W_res.data(), Wd, W0.size() * sizeof(float), hipMemcpyDeviceToHost));
        for (size_t e = 0; e < W0.size(); ++e) {
            EXPECT(fabsf(W_file[e] - W_res[e]) <= 1e-5f && fabsf(W_host[e] - W_res[e]) <= 1e-5f);
            if (failures) break;
        }

        // refused calls leave the weights alone: a file that ends early (checked up front), an offset that makes it
        // end early, bad arguments
        EXPECT(som_epoch_file(ctx, fd, 0, N + 1, D, chunk, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_EIO);
        EXPECT(strlen(som_last_error(ctx)) > 0);
        EXPECT(som_epoch_file(ctx, fd, 64, N, D, chunk, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_EIO);
        EXPECT(som_epoch_file(ctx, -1, 0, N, D, chunk, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_EINVAL);
        EXPECT(som_epoch_host(ctx, X.data(), N, D, 0, 0, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_EINVAL);
        EXPECT(som_epoch_host(ctx, X.data(), N, D, chunk, 0, Wd, K, Gd, -1.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_EINVAL);
        EXPECT(som_epoch(ctx, Xd, N, D, D - 1, nullptr, N, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_EINVAL);
        EXPECT(som_sync(ctx) == SOM_OK);
        HIP_OK(hipMemcpy(W_after.data(), Wd, W0.size() * sizeof(float), hipMemcpyDeviceToHost));
        EXPECT(memcmp(W_after.data(), W_res.data(), W0.size() * sizeof(float)) == 0);

        // many short chunks: the pool of copy events grows and is reused
        HIP_OK(hipMemcpy(Wd, W0.data(), W0.size() * sizeof(float), hipMemcpyHostToDevice));
        EXPECT(som_epoch_file(ctx, fd, 0, 50000, D, 777, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_OK);
        EXPECT(st.m == 50000);
        EXPECT(som_epoch_host(ctx, X.data(), 0, D, chunk, 0, Wd, K, Gd, 2.0, SOM_KERNEL_GAUSSIAN, 0.0, &st) == SOM_OK);
        EXPECT(st.m == 0 && st.n_empty == K);
        som_destroy(ctx);
    }
    HIP_OK(hipFree(Xd));
    HIP_OK(hipFree(Gd));
    HIP_OK(hipFree(Wd));
    close(fd);
    unlink(path);
    return 0;
}

int main(int argc, char** argv)
{
    without_a_context();
    if (argc > 1 && strcmp(argv[1], "--device") == 0) {
        if (with_a_device() != 0) ++failures;
    }
    if (failures) {
        fprintf(stderr, "host_shell_check: %d failure(s)\n", failures);
        return 1;
    }
    printf("host_shell_check: ok\n");
    return 0;
}
