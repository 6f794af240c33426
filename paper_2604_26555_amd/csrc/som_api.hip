// C ABI of libsom: context, argument checking, and the epoch drivers that chain the kernels.
#include "som_internal.hpp"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <errno.h>
#include <sys/stat.h>
#include <sys/types.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <thread>
#include <vector>

namespace som {

int fail(som_ctx* ctx, int code, const char* fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

int check_hip(som_ctx* ctx, hipError_t e, const char* what)
{
    if (e == hipSuccess) return SOM_OK;
    (void)hipGetLastError();
    return fail(ctx, SOM_EHIP, "%s: %s", what, hipGetErrorString(e));
}

static bool device_readable(const void* p)
{
    hipPointerAttribute_t at;
    if (hipPointerGetAttributes(&at, p) != hipSuccess) {
        (void)hipGetLastError();
        return false; // plain host memory is not known to the runtime
    }
    return at.type == hipMemoryTypeDevice || at.type == hipMemoryTypeManaged || at.type == hipMemoryTypeHost;
}

template <class T>
static int grow(som_ctx* ctx, T** p, size_t* have, size_t want, const char* what)
{
    if (want <= *have) return SOM_OK;
    if (*p) {
        if (int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "sync before workspace growth")) return rc;
        (void)hipFree(*p);
        *p = nullptr;
        *have = 0;
    }
    if (hipMalloc((void**)p, want * sizeof(T)) != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, SOM_ENOMEM, "cannot allocate %zu bytes for %s", want * sizeof(T), what);
    }
    *have = want;
    return SOM_OK;
}

static int common_checks(som_ctx* ctx, const void* X, int64_t N, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
                         const void* W, int32_t K)
{
    if (!ctx) return SOM_EINVAL;
    if (!W || (!X && N != 0)) return fail(ctx, SOM_EINVAL, "null X or W");
    if (K < 1 || D < 1) return fail(ctx, SOM_EINVAL, "K and D must be positive (K=%d, D=%d)", K, D);
    if (N < 0 || m < 0) return fail(ctx, SOM_EINVAL, "negative N or m");
    if (ldx < D) return fail(ctx, SOM_EINVAL, "ldx (%lld) is smaller than D (%d)", (long long)ldx, D);
    if (!idx && m != N) return fail(ctx, SOM_EINVAL, "without an index list m (%lld) must equal N (%lld)", (long long)m, (long long)N);
    if (idx && m > 0 && N < 1) return fail(ctx, SOM_EINVAL, "index list given for an empty X");
    if (m > 0x7fffffffLL) return fail(ctx, SOM_EINVAL, "m above 2^31-1 per call; present the data in chunks");
    if (N > 0xffffffffLL + 1 && idx) return fail(ctx, SOM_EINVAL, "row numbers of an index list are 32-bit");
    if ((int64_t)K * D > (int64_t)1 << 28) return fail(ctx, SOM_EINVAL, "K*D too large");
    return SOM_OK;
}

} // namespace som

using namespace som;

extern "C" {

const char* som_strerror(int code)
{
    switch (code) {
    case SOM_OK: return "ok";
    case SOM_EINVAL: return "invalid argument";
    case SOM_ENOMEM: return "out of memory";
    case SOM_EHIP: return "HIP runtime error";
    case SOM_EIO: return "input/output error";
    case SOM_ESTATE: return "context unusable";
    }
    return "unknown error code";
}

const char* som_last_error(const som_ctx* ctx) { return ctx ? ctx->err : "null context"; }

int som_create(som_ctx** out, int device, void* hip_stream)
{
    if (!out) return SOM_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) {
        (void)hipGetLastError();
        return SOM_ESTATE;
    }
    if (device >= kMaxDevices) return SOM_EINVAL;         // per-device tables of the launchers
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return SOM_ESTATE;
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return SOM_ESTATE; // kernels are built for gfx950 only
    if (hipSetDevice(device) != hipSuccess) return SOM_ESTATE;
    som_ctx* c = new (std::nothrow) som_ctx;
    if (!c) return SOM_ENOMEM;
    c->device = device;
    c->stream = (hipStream_t)hip_stream; // NULL is HIP's default stream, which is what torch uses by default
    bool ok = hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->qe, 2 * sizeof(double)) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->small, 64) == hipSuccess;
    ok = ok && hipMalloc((void**)&c->qe_part, kQeSlots * 2 * sizeof(double)) == hipSuccess;
    ok = ok && hipMemset(c->qe_part, 0, kQeSlots * 2 * sizeof(double)) == hipSuccess;
    ok = ok && hipHostMalloc(&c->host_small, 256, hipHostMallocDefault) == hipSuccess;
    for (int i = 0; i < 2 && ok; ++i) {
        ok = ok && hipEventCreateWithFlags(&c->ev_copied[i], hipEventDisableTiming) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&c->ev_consumed[i], hipEventDisableTiming) == hipSuccess;
    }
    for (int i = 0; i < 4 && ok; ++i) ok = ok && hipEventCreate(&c->ev_t[i]) == hipSuccess;
    ok = ok && update_static_init(c) == SOM_OK;
    if (!ok) {
        (void)hipGetLastError();
        som_destroy(c);
        return SOM_EHIP;
    }
    *out = c;
    return SOM_OK;
}

void som_destroy(som_ctx* c)
{
    if (!c) return;
    (void)hipSetDevice(c->device);
    if (c->stream) (void)hipStreamSynchronize(c->stream);
    if (c->copy_stream) {
        (void)hipStreamSynchronize(c->copy_stream);
        (void)hipStreamDestroy(c->copy_stream);
    }
    for (int i = 0; i < 2; ++i) {
        if (c->ev_copied[i]) (void)hipEventDestroy(c->ev_copied[i]);
        if (c->ev_consumed[i]) (void)hipEventDestroy(c->ev_consumed[i]);
        if (c->pinned[i]) (void)hipHostFree(c->pinned[i]);
        if (c->dchunk[i]) (void)hipFree(c->dchunk[i]);
    }
    for (int i = 0; i < 4; ++i)
        if (c->ev_t[i]) (void)hipEventDestroy(c->ev_t[i]);
    if (c->prep_blob) (void)hipFree(c->prep_blob);
    if (c->recheck) (void)hipFree(c->recheck);
    if (c->bmu_ws) (void)hipFree(c->bmu_ws);
    if (c->acc_blob) (void)hipFree(c->acc_blob);
    if (c->parts_blob) (void)hipFree(c->parts_blob);
    if (c->upd_blob) (void)hipFree(c->upd_blob);
    if (c->topo_blob) (void)hipFree(c->topo_blob);
    if (c->S) (void)hipFree(c->S);
    if (c->n) (void)hipFree(c->n);
    if (c->qe) (void)hipFree(c->qe);
    if (c->small) (void)hipFree(c->small);
    if (c->qe_part) (void)hipFree(c->qe_part);
    if (c->host_small) (void)hipHostFree(c->host_small);
    for (hipEvent_t e : c->h2d_events) (void)hipEventDestroy(e);
    for (auto& pr : c->prof_events) {
        (void)hipEventDestroy(pr.first);
        (void)hipEventDestroy(pr.second);
    }
    delete c;
}

int som_sync(som_ctx* ctx)
{
    if (!ctx) return SOM_EINVAL;
    return check_hip(ctx, hipStreamSynchronize(ctx->stream), "stream synchronize");
}

int som_set_reproducible(som_ctx* ctx, int on)
{
    if (!ctx) return SOM_EINVAL;
    ctx->reproducible = on ? 1 : 0;
    return SOM_OK;
}

int som_set_search(som_ctx* ctx, int mode)
{
    if (!ctx) return SOM_EINVAL;
    if (mode != SOM_SEARCH_AUTO && mode != SOM_SEARCH_FLOAT32) return fail(ctx, SOM_EINVAL, "unknown search mode %d", mode);
    ctx->search = mode;
    return SOM_OK;
}

int som_set_safeguard(som_ctx* ctx, int mode)
{
    if (!ctx) return SOM_EINVAL;
    if (mode != SOM_SAFEGUARD_THRESHOLD && mode != SOM_SAFEGUARD_SHIFT) return fail(ctx, SOM_EINVAL, "unknown safeguard mode %d", mode);
    ctx->safeguard = mode;
    return SOM_OK;
}

int som_set_update_rule(som_ctx* ctx, double eta, double mu, float* velocity)
{
    if (!ctx) return SOM_EINVAL;
    if (!(eta > 0.0 && eta <= 1.0)) return fail(ctx, SOM_EINVAL, "eta must be in (0, 1]");
    if (!(mu >= 0.0 && mu < 1.0)) return fail(ctx, SOM_EINVAL, "mu must be in [0, 1)");
    if (mu != 0.0 && !velocity) return fail(ctx, SOM_EINVAL, "momentum needs a velocity buffer");
    if (velocity && !device_readable(velocity)) return fail(ctx, SOM_EINVAL, "velocity must be device-accessible memory");
    ctx->eta = eta;
    ctx->mu = mu;
    ctx->velocity = velocity;
    return SOM_OK;
}

int som_profile(som_ctx* ctx, int enable)
{
    if (!ctx) return SOM_EINVAL;
    ctx->profiling = enable != 0;
    ctx->prof_used = 0;
    return SOM_OK;
}

int som_profile_read(som_ctx* ctx, float* ms, int32_t capacity, int32_t* count)
{
    if (!ctx || !count || capacity < 0 || (capacity > 0 && !ms)) return ctx ? fail(ctx, SOM_EINVAL, "bad profile buffer") : SOM_EINVAL;
    if (int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "stream synchronize")) return rc;
    int32_t n = 0;
    for (size_t i = 0; i < ctx->prof_used && n < capacity; ++i, ++n)
        if (int rc = check_hip(ctx, hipEventElapsedTime(&ms[n], ctx->prof_events[i].first, ctx->prof_events[i].second), "event timing")) return rc;
    *count = (int32_t)ctx->prof_used;
    ctx->prof_used = 0;
    return SOM_OK;
}

int som_bmu(som_ctx* ctx, const float* X, int64_t N, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
            const float* W, int32_t K, int32_t* bmu, float* d2, double* qe)
{
    if (int rc = common_checks(ctx, X, N, D, ldx, idx, m, W, K)) return rc;
    if (!bmu && m > 0) return fail(ctx, SOM_EINVAL, "null bmu output");
    if ((N > 0 && !device_readable(X)) || !device_readable(W) || (m > 0 && !device_readable(bmu)))
        return fail(ctx, SOM_EINVAL, "X, W and bmu must be device-accessible memory");
    if (int rc = check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice")) return rc;
    if (m == 0) return qe ? launch_fill_zero(ctx, qe, 2 * sizeof(double)) : SOM_OK;
    BmuPrep prep;
    if (int rc = bmu_prepare(ctx, W, K, D, &prep, qe, nullptr)) return rc;
    BmuArgs a{};
    a.X = X;
    a.ldx = ldx;
    a.idx = idx;
    a.m = m;
    a.D = D;
    a.K = K;
    a.W = W;
    a.bmu = bmu;
    a.d2 = d2;
    a.qe = qe;
    return bmu_run(ctx, prep, a);
}

int som_accumulate(som_ctx* ctx, const float* X, int64_t N, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m,
                   const int32_t* bmu, int32_t K, double* S, uint64_t* n, int zero_first)
{
    if (int rc = common_checks(ctx, X, N, D, ldx, idx, m, S, K)) return rc;
    if (!S || !n || (!bmu && m > 0)) return fail(ctx, SOM_EINVAL, "null S, n or bmu");
    if ((N > 0 && !device_readable(X)) || !device_readable(S) || !device_readable(n) || (m > 0 && !device_readable(bmu)))
        return fail(ctx, SOM_EINVAL, "X, bmu, S and n must be device-accessible memory");
    if (int rc = check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice")) return rc;
    return accumulate_run(ctx, X, D, ldx, idx, m, bmu, K, S, (unsigned long long*)n, zero_first != 0);
}

static int update_checks(som_ctx* ctx, const void* G, int32_t K, int32_t D, double sigma, int kernel)
{
    if (!G) return fail(ctx, SOM_EINVAL, "null G");
    if (K < 1 || D < 1) return fail(ctx, SOM_EINVAL, "K and D must be positive");
    if (!(sigma > 0.0) || !isfinite(sigma)) return fail(ctx, SOM_EINVAL, "sigma must be positive and finite");
    if (kernel != SOM_KERNEL_GAUSSIAN) return fail(ctx, SOM_EINVAL, "unknown neighbourhood kernel %d", kernel);
    return SOM_OK;
}

int som_neighborhood_update(som_ctx* ctx, const double* S, const uint64_t* n, const float* G, int32_t K, int32_t D,
                            double sigma, int kernel, double eps_h, float* W, int32_t* n_guarded)
{
    if (!ctx) return SOM_EINVAL;
    if (!S || !n || !W) return fail(ctx, SOM_EINVAL, "null S, n or W");
    if (int rc = update_checks(ctx, G, K, D, sigma, kernel)) return rc;
    if (!device_readable(S) || !device_readable(n) || !device_readable(G) || !device_readable(W))
        return fail(ctx, SOM_EINVAL, "S, n, G and W must be device-accessible memory");
    if (int rc = check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice")) return rc;
    if (eps_h <= 0.0) eps_h = 1e-30;
    if (int rc = launch_fill_zero(ctx, ctx->small, 64)) return rc;
    if (int rc = update_run(ctx, S, (const unsigned long long*)n, G, K, D, sigma, eps_h, W, ctx->small)) return rc;
    if (n_guarded)
        return check_hip(ctx, hipMemcpyAsync(n_guarded, ctx->small, sizeof(int32_t), hipMemcpyDeviceToDevice, ctx->stream),
                         "copying the guarded-node count");
    return SOM_OK;
}

int som_neighborhood_update_static(som_ctx* ctx, const double* S, const uint64_t* n, const float* G, int32_t K, int32_t D,
                                   double sigma, int kernel, double eps_h, float* W, int32_t* n_guarded)
{
    if (!ctx) return SOM_EINVAL;
    if (!S || !n || !W) return fail(ctx, SOM_EINVAL, "null S, n or W");
    if (int rc = update_checks(ctx, G, K, D, sigma, kernel)) return rc;
    if (!device_readable(S) || !device_readable(n) || !device_readable(G) || !device_readable(W))
        return fail(ctx, SOM_EINVAL, "S, n, G and W must be device-accessible memory");
    if (int rc = check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice")) return rc;
    if (eps_h <= 0.0) eps_h = 1e-30;
    if (int rc = launch_fill_zero(ctx, ctx->small, 64)) return rc;
    if (int rc = update_static_run(ctx, S, (const unsigned long long*)n, G, K, D, sigma, eps_h, W, ctx->small)) return rc;
    if (n_guarded)
        return check_hip(ctx, hipMemcpyAsync(n_guarded, ctx->small, sizeof(int32_t), hipMemcpyDeviceToDevice, ctx->stream),
                         "copying the guarded-node count");
    return SOM_OK;
}

// host mirror of the small device-side results
struct HostSmall {
    double qe[2];
    int32_t small[4];
    unsigned int scal[4];
};

static int begin_epoch(som_ctx* ctx, int32_t K, int32_t D, int64_t chunk_rows)
{
    if (int rc = grow(ctx, &ctx->bmu_ws, &ctx->bmu_elems, (size_t)chunk_rows, "the BMU indices")) return rc;
    if (int rc = grow(ctx, &ctx->S, &ctx->S_elems, (size_t)K * D, "the per-node sums")) return rc;
    if (int rc = grow(ctx, &ctx->n, &ctx->n_elems, (size_t)K, "the per-node counts")) return rc;
    return SOM_OK;   // qe and the small counters are cleared by the weight-preparation kernel
}

static int finish_stats(som_ctx* ctx, int64_t m, int64_t n_recheck, som_stats* stats, bool timed, float ms_h2d)
{
    HostSmall* h = (HostSmall*)ctx->host_small;
    if (int rc = check_hip(ctx, hipMemcpyAsync(h->qe, ctx->qe, sizeof(h->qe), hipMemcpyDeviceToHost, ctx->stream), "reading statistics")) return rc;
    if (int rc = check_hip(ctx, hipMemcpyAsync(h->small, ctx->small, sizeof(h->small), hipMemcpyDeviceToHost, ctx->stream), "reading statistics")) return rc;
    if (int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "waiting for the epoch")) return rc;
    stats->sum_dist = h->qe[0];
    stats->sum_dist2 = h->qe[1];
    stats->m = m;
    stats->n_recheck = n_recheck;
    stats->n_guarded = h->small[0];
    stats->n_empty = h->small[1];
    stats->ms_bmu_acc = stats->ms_update = 0.f;
    stats->ms_h2d = ms_h2d;
    if (timed) {
        (void)hipEventElapsedTime(&stats->ms_bmu_acc, ctx->ev_t[0], ctx->ev_t[1]);
        (void)hipEventElapsedTime(&stats->ms_update, ctx->ev_t[1], ctx->ev_t[2]);
    }
    return SOM_OK;
}

int som_epoch(som_ctx* ctx, const float* X, int64_t N, int32_t D, int64_t ldx, const uint32_t* idx, int64_t m, float* W,
              int32_t K, const float* G, double sigma, int kernel, double eps_h, som_stats* stats)
{
    if (int rc = common_checks(ctx, X, N, D, ldx, idx, m, W, K)) return rc;
    if (int rc = update_checks(ctx, G, K, D, sigma, kernel)) return rc;
    if ((N > 0 && !device_readable(X)) || !device_readable(W) || !device_readable(G))
        return fail(ctx, SOM_EINVAL, "X, W and G must be device-accessible memory");
    if (int rc = check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice")) return rc;
    if (eps_h <= 0.0) eps_h = 1e-30;
    if (m == 0) {
        if (stats) {
            memset(stats, 0, sizeof(*stats));
            stats->n_empty = K;
            stats->n_guarded = K;
        }
        return SOM_OK;
    }
    if (int rc = begin_epoch(ctx, K, D, m)) return rc;
    BmuPrep prep;
    if (stats) (void)hipEventRecord(ctx->ev_t[0], ctx->stream);
    if (int rc = bmu_prepare(ctx, W, K, D, &prep, ctx->qe, ctx->small)) return rc;
    BmuArgs a{};
    a.X = X;
    a.ldx = ldx;
    a.idx = idx;
    a.m = m;
    a.D = D;
    a.K = K;
    a.W = W;
    a.qe = stats ? ctx->qe : nullptr;       // no statistics asked for: the search forms no distances
    a.bmu = ctx->bmu_ws;
    if (int rc = bmu_run(ctx, prep, a)) return rc;
    if (int rc = accumulate_run(ctx, X, D, ldx, idx, m, ctx->bmu_ws, K, ctx->S, ctx->n, true)) return rc;
    HostSmall* h = (HostSmall*)ctx->host_small;
    if (stats) {
        (void)hipEventRecord(ctx->ev_t[1], ctx->stream);
        if (int rc = check_hip(ctx, hipMemcpyAsync(h->scal, prep.scal, sizeof(h->scal), hipMemcpyDeviceToHost, ctx->stream), "reading statistics")) return rc;
    }
    if (int rc = update_run(ctx, ctx->S, ctx->n, G, K, D, sigma, eps_h, W, ctx->small)) return rc;
    if (stats) {
        (void)hipEventRecord(ctx->ev_t[2], ctx->stream);
        if (int rc = finish_stats(ctx, m, 0, stats, true, 0.f)) return rc;
        stats->n_recheck = h->scal[3];
    }
    return SOM_OK;
}

// copies [src, src + bytes) with several host threads (page-cache or anonymous memory -> pinned staging buffer)
static void parallel_copy(void* dst, const void* src, size_t bytes)
{
    unsigned hw = std::thread::hardware_concurrency();
    unsigned nt = std::min<unsigned>(hw ? hw : 4, 16);
    if (bytes < ((size_t)8 << 20)) nt = 1;
    if (nt <= 1) {
        memcpy(dst, src, bytes);
        return;
    }
    std::vector<std::thread> th;
    const size_t per = ((bytes / nt) + 4095) & ~(size_t)4095;
    for (unsigned t = 0; t < nt; ++t) {
        const size_t lo = (size_t)t * per;
        if (lo >= bytes) break;
        const size_t len = std::min(per, bytes - lo);
        th.emplace_back([=] { memcpy((char*)dst + lo, (const char*)src + lo, len); });
    }
    for (auto& t : th) t.join();
}

// reads [offset, offset + bytes) of a file into dst with several host threads; 0, or an errno value (EIO for a file
// that ends early)
static int parallel_pread(int fd, void* dst, int64_t offset, size_t bytes)
{
    unsigned hw = std::thread::hardware_concurrency();
    unsigned nt = std::min<unsigned>(hw ? hw : 4, 16);
    if (bytes < ((size_t)8 << 20)) nt = 1;
    const size_t per = ((bytes / nt) + 4095) & ~(size_t)4095;
    std::atomic<int> err{0};
    auto work = [&](size_t lo, size_t len) {
        size_t done = 0;
        while (done < len && err.load(std::memory_order_relaxed) == 0) {
            const ssize_t r = pread(fd, (char*)dst + lo + done, std::min(len - done, (size_t)1 << 30), (off_t)(offset + lo + done));
            if (r < 0) {
                if (errno == EINTR) continue;
                err.store(errno ? errno : EIO);
                return;
            }
            if (r == 0) {           // end of file inside the range the caller promised
                err.store(EIO);
                return;
            }
            done += (size_t)r;
        }
    };
    if (nt <= 1) {
        work(0, bytes);
        return err.load();
    }
    std::vector<std::thread> th;
    for (unsigned t = 0; t < nt; ++t) {
        const size_t lo = (size_t)t * per;
        if (lo >= bytes) break;
        th.emplace_back(work, lo, std::min(per, bytes - lo));
    }
    for (auto& t : th) t.join();
    return err.load();
}

// where the chunks of a streamed epoch come from
struct ChunkSource {
    const float* host = nullptr; // host memory (pageable, mapped or pinned), or
    int pinned = 0;              // ... caller-pinned memory, copied from directly
    int fd = -1;                 // a file descriptor read with pread
    int64_t offset = 0;          // byte offset of row 0 in the file
};

// the chunk loop shared by som_epoch_host and som_epoch_file (Section 3.3.2): stage chunk c + 1 into a pinned buffer and
// copy it to the device on the copy stream while chunk c is searched and accumulated on the compute stream
static int stream_epoch(som_ctx* ctx, const ChunkSource& src, int64_t N, int32_t D, int64_t chunk_rows, float* W, int32_t K,
                        const float* G, double sigma, double eps_h, som_stats* stats)
{
    if (chunk_rows > N) chunk_rows = N;
    const bool staged = !(src.host && src.pinned);
    const size_t chunk_elems = (size_t)chunk_rows * D;
    if (chunk_elems > ctx->chunk_elems || (staged && !ctx->pinned[0])) {
        if (int rc = check_hip(ctx, hipDeviceSynchronize(), "sync before buffer growth")) return rc;
        for (int i = 0; i < 2; ++i) {
            if (ctx->dchunk[i]) (void)hipFree(ctx->dchunk[i]);
            if (ctx->pinned[i]) (void)hipHostFree(ctx->pinned[i]);
            ctx->dchunk[i] = ctx->pinned[i] = nullptr;
        }
        const size_t want = std::max(chunk_elems, ctx->chunk_elems);
        ctx->chunk_elems = 0;
        for (int i = 0; i < 2; ++i) {
            if (hipMalloc((void**)&ctx->dchunk[i], want * sizeof(float)) != hipSuccess ||
                (staged && hipHostMalloc((void**)&ctx->pinned[i], want * sizeof(float), hipHostMallocDefault) != hipSuccess)) {
                (void)hipGetLastError();
                return fail(ctx, SOM_ENOMEM, "cannot allocate the chunk buffers (%zu bytes each)", want * sizeof(float));
            }
        }
        ctx->chunk_elems = want;
    }
    if (int rc = begin_epoch(ctx, K, D, chunk_rows)) return rc;
    const int64_t nchunks = (N + chunk_rows - 1) / chunk_rows;
    // timing events of the copies: a pool owned by the context, grown on demand and reused by every epoch
    const bool timed = stats != nullptr;
    while (timed && ctx->h2d_events.size() < (size_t)(2 * nchunks)) {
        hipEvent_t e;
        if (int rc = check_hip(ctx, hipEventCreate(&e), "event creation")) return rc;
        ctx->h2d_events.push_back(e);
    }
    BmuPrep prep;
    (void)hipEventRecord(ctx->ev_t[0], ctx->stream);
    if (int rc = bmu_prepare(ctx, W, K, D, &prep, ctx->qe, ctx->small)) return rc;

    // After a failure inside the loop both streams are drained before the call returns: nothing of this epoch is
    // still in flight into the chunk buffers when the caller uses the context again.
    auto bail = [&](int rc) {
        (void)hipStreamSynchronize(ctx->copy_stream);
        (void)hipStreamSynchronize(ctx->stream);
        (void)hipGetLastError();
        return rc;
    };
    HostSmall* h = (HostSmall*)ctx->host_small;
    for (int64_t c = 0; c < nchunks; ++c) {
        const int b = (int)(c & 1);
        const int64_t lo = c * chunk_rows;
        const int64_t rows = std::min(chunk_rows, N - lo);
        const size_t bytes = (size_t)rows * D * sizeof(float);
        const float* from = src.host ? src.host + (size_t)lo * D : nullptr;
        if (staged) {
            // the staging buffer is free once its previous copy to the device has finished
            if (c >= 2)
                if (int rc = check_hip(ctx, hipEventSynchronize(ctx->ev_copied[b]), "waiting for a staging buffer")) return bail(rc);
            if (src.host) {
                parallel_copy(ctx->pinned[b], from, bytes);
            } else if (int e = parallel_pread(src.fd, ctx->pinned[b], src.offset + (int64_t)((size_t)lo * D * sizeof(float)), bytes)) {
                return bail(fail(ctx, SOM_EIO, "reading rows %lld..%lld of the sample file: %s", (long long)lo,
                                 (long long)(lo + rows - 1), strerror(e)));
            }
            from = ctx->pinned[b];
        }
        // the device buffer is free once the compute of two chunks ago has consumed it
        if (c >= 2)
            if (int rc = check_hip(ctx, hipStreamWaitEvent(ctx->copy_stream, ctx->ev_consumed[b], 0), "stream wait")) return bail(rc);
        if (timed) (void)hipEventRecord(ctx->h2d_events[2 * c], ctx->copy_stream);
        if (int rc = check_hip(ctx, hipMemcpyAsync(ctx->dchunk[b], from, bytes, hipMemcpyHostToDevice, ctx->copy_stream), "host-to-device copy"))
            return bail(rc);
        if (timed) (void)hipEventRecord(ctx->h2d_events[2 * c + 1], ctx->copy_stream);
        (void)hipEventRecord(ctx->ev_copied[b], ctx->copy_stream);
        if (int rc = check_hip(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev_copied[b], 0), "stream wait")) return bail(rc);
        BmuArgs a{};
        a.X = ctx->dchunk[b];
        a.ldx = D;
        a.idx = nullptr;
        a.m = rows;
        a.D = D;
        a.K = K;
        a.W = W;
        a.qe = stats ? ctx->qe : nullptr;
        a.bmu = ctx->bmu_ws;
        if (int rc = bmu_run(ctx, prep, a)) return bail(rc);
        if (int rc = accumulate_run(ctx, ctx->dchunk[b], D, D, nullptr, rows, ctx->bmu_ws, K, ctx->S, ctx->n, c == 0)) return bail(rc);
        (void)hipEventRecord(ctx->ev_consumed[b], ctx->stream);
    }
    (void)hipEventRecord(ctx->ev_t[1], ctx->stream);
    if (int rc = check_hip(ctx, hipMemcpyAsync(h->scal, prep.scal, sizeof(h->scal), hipMemcpyDeviceToHost, ctx->stream), "reading statistics"))
        return bail(rc);
    if (int rc = update_run(ctx, ctx->S, ctx->n, G, K, D, sigma, eps_h, W, ctx->small)) return bail(rc);
    (void)hipEventRecord(ctx->ev_t[2], ctx->stream);
    int rc = check_hip(ctx, hipStreamSynchronize(ctx->stream), "waiting for the epoch");
    if (!rc) rc = check_hip(ctx, hipStreamSynchronize(ctx->copy_stream), "waiting for the copy stream");
    if (rc) return bail(rc);
    float ms_h2d = 0.f;
    for (int64_t c = 0; timed && c < nchunks; ++c) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ctx->h2d_events[2 * c], ctx->h2d_events[2 * c + 1]) == hipSuccess) ms_h2d += ms;
    }
    if (stats) return finish_stats(ctx, N, (int64_t)h->scal[3], stats, true, ms_h2d);
    return SOM_OK;
}

static int stream_checks(som_ctx* ctx, const void* X, int64_t N, int32_t D, int64_t chunk_rows, const float* W, int32_t K,
                         const float* G, double sigma, int kernel)
{
    if (int rc = common_checks(ctx, X, N, D, D, nullptr, N, W, K)) return rc;
    if (int rc = update_checks(ctx, G, K, D, sigma, kernel)) return rc;
    if (chunk_rows < 1) return fail(ctx, SOM_EINVAL, "chunk_rows must be positive");
    if (chunk_rows > 0x7fffffffLL) return fail(ctx, SOM_EINVAL, "chunk_rows above 2^31-1");
    if (!device_readable(W) || !device_readable(G)) return fail(ctx, SOM_EINVAL, "W and G must be device-accessible memory");
    return check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice");
}

static int empty_epoch(int32_t K, som_stats* stats)
{
    if (stats) {
        memset(stats, 0, sizeof(*stats));
        stats->n_empty = K;
        stats->n_guarded = K;
    }
    return SOM_OK;
}

int som_epoch_host(som_ctx* ctx, const float* Xhost, int64_t N, int32_t D, int64_t chunk_rows, int pinned, float* W,
                   int32_t K, const float* G, double sigma, int kernel, double eps_h, som_stats* stats)
{
    if (int rc = stream_checks(ctx, Xhost, N, D, chunk_rows, W, K, G, sigma, kernel)) return rc;
    if (N == 0) return empty_epoch(K, stats);
    ChunkSource src;
    src.host = Xhost;
    src.pinned = pinned;
    return stream_epoch(ctx, src, N, D, chunk_rows, W, K, G, sigma, eps_h <= 0.0 ? 1e-30 : eps_h, stats);
}

int som_epoch_file(som_ctx* ctx, int fd, int64_t offset, int64_t N, int32_t D, int64_t chunk_rows, float* W, int32_t K,
                   const float* G, double sigma, int kernel, double eps_h, som_stats* stats)
{
    // (the shared checks want a non-null sample pointer for N > 0: the file stands in for it)
    if (int rc = stream_checks(ctx, N > 0 ? (const void*)W : nullptr, N, D, chunk_rows, W, K, G, sigma, kernel)) return rc;
    if (fd < 0 || offset < 0) return fail(ctx, SOM_EINVAL, "bad file descriptor or negative offset");
    struct stat st;
    if (fstat(fd, &st) != 0) return fail(ctx, SOM_EIO, "fstat on the sample file: %s", strerror(errno));
    const int64_t need = offset + (int64_t)((size_t)N * D * sizeof(float));
    if (S_ISREG(st.st_mode) && (int64_t)st.st_size < need)
        return fail(ctx, SOM_EIO, "the sample file holds %lld bytes, %lld rows of %d floats from offset %lld need %lld",
                    (long long)st.st_size, (long long)N, D, (long long)offset, (long long)need);
    if (N == 0) return empty_epoch(K, stats);
    ChunkSource src;
    src.fd = fd;
    src.offset = offset;
    return stream_epoch(ctx, src, N, D, chunk_rows, W, K, G, sigma, eps_h <= 0.0 ? 1e-30 : eps_h, stats);
}

} // extern "C"
