// Host-only part of the library: error text, scratch arena, digest comparison.
#include <cstring>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

#include "sentry_internal.h"

namespace sentry {

int merkle_reserve(uint64_t max_len, uint64_t leaf_bytes, hipStream_t s);   // sha256_merkle.hip
int lthash_reserve(uint64_t max_records, hipStream_t s);                     // blake2_lthash.hip

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

void clear_error() { g_err[0] = '\0'; }

struct StreamCtx {
    void *region[R_COUNT] = {};
    size_t cap[R_COUNT] = {};
    void *tab_host[TABLE_SLOTS] = {};      // pinned
    size_t tab_cap[TABLE_SLOTS] = {};
    hipEvent_t tab_event[TABLE_SLOTS] = {};
    bool tab_pending[TABLE_SLOTS] = {};
    CopyPipe pipe = {};
    bool pipe_ready = false;
    bool hash_streams_ready = false;
};

static std::mutex g_mu;
static std::map<std::pair<int, hipStream_t>, StreamCtx> g_ctx;

static int ctx_for(hipStream_t stream, StreamCtx **out)
{
    int dev = 0;
    SENTRY_HIP_CHECK(hipGetDevice(&dev));
    *out = &g_ctx[std::make_pair(dev, stream)];
    return SENTRY_OK;
}

int scratch_get(hipStream_t stream, Region r, size_t bytes, void **out)
{
    bool fresh;
    return scratch_get_fresh(stream, r, bytes, out, &fresh);
}

size_t scratch_capacity(hipStream_t stream, Region r)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    auto it = g_ctx.find(std::make_pair(dev, stream));
    return it == g_ctx.end() ? 0 : it->second.cap[r];
}

int scratch_get_fresh(hipStream_t stream, Region r, size_t bytes, void **out, bool *fresh)
{
    std::lock_guard<std::mutex> lock(g_mu);
    *fresh = false;
    StreamCtx *c;
    int rc = ctx_for(stream, &c);
    if (rc) return rc;
    if (bytes == 0) bytes = 256;
    if (c->cap[r] < bytes) {
        if (c->region[r]) {
            // work that still uses the old allocation may be in flight on the stream
            SENTRY_HIP_CHECK(hipStreamSynchronize(stream));
            SENTRY_HIP_CHECK(hipFree(c->region[r]));
            c->region[r] = nullptr;
            c->cap[r] = 0;
        }
        size_t want = (bytes + 4095) & ~(size_t)4095;
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, want);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            set_error("scratch allocation of %zu bytes failed: %s", want, hipGetErrorString(e));
            return SENTRY_ERR_NOMEM;
        }
        c->region[r] = p;
        c->cap[r] = want;
        *fresh = true;
    }
    *out = c->region[r];
    return SENTRY_OK;
}

int table_staging_get(hipStream_t stream, size_t bytes, void **host_ptr, int slot)
{
    std::lock_guard<std::mutex> lock(g_mu);
    StreamCtx *c;
    int rc = ctx_for(stream, &c);
    if (rc) return rc;
    if (c->tab_pending[slot]) {   // the previous upload must have left the pinned memory
        SENTRY_HIP_CHECK(hipEventSynchronize(c->tab_event[slot]));
        c->tab_pending[slot] = false;
    }
    if (c->tab_cap[slot] < bytes) {
        if (c->tab_host[slot]) SENTRY_HIP_CHECK(hipHostFree(c->tab_host[slot]));
        c->tab_host[slot] = nullptr;
        c->tab_cap[slot] = 0;
        size_t want = (bytes + 4095) & ~(size_t)4095;
        void *p = nullptr;
        hipError_t e = hipHostMalloc(&p, want, hipHostMallocDefault);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            set_error("pinned table allocation of %zu bytes failed: %s", want, hipGetErrorString(e));
            return SENTRY_ERR_NOMEM;
        }
        c->tab_host[slot] = p;
        c->tab_cap[slot] = want;
    }
    if (!c->tab_event[slot]) SENTRY_HIP_CHECK(hipEventCreateWithFlags(&c->tab_event[slot], hipEventDisableTiming));
    *host_ptr = c->tab_host[slot];
    return SENTRY_OK;
}

int table_staging_mark(hipStream_t stream, int slot)
{
    std::lock_guard<std::mutex> lock(g_mu);
    StreamCtx *c;
    int rc = ctx_for(stream, &c);
    if (rc) return rc;
    SENTRY_HIP_CHECK(hipEventRecord(c->tab_event[slot], stream));
    c->tab_pending[slot] = true;
    return SENTRY_OK;
}

int copy_pipe_get(hipStream_t stream, bool with_hash_streams, CopyPipe **out)
{
    std::lock_guard<std::mutex> lock(g_mu);
    StreamCtx *c;
    int rc = ctx_for(stream, &c);
    if (rc) return rc;
    if (!c->pipe_ready) {
        // default priority on purpose: mixed stream priorities are not used anywhere
        SENTRY_HIP_CHECK(hipStreamCreateWithFlags(&c->pipe.copy_stream, hipStreamNonBlocking));
        SENTRY_HIP_CHECK(hipEventCreateWithFlags(&c->pipe.start, hipEventDisableTiming));
        for (int i = 0; i < PIPE_SLOTS; i++) {
            SENTRY_HIP_CHECK(hipEventCreateWithFlags(&c->pipe.copied[i], hipEventDisableTiming));
            SENTRY_HIP_CHECK(hipEventCreateWithFlags(&c->pipe.consumed[i], hipEventDisableTiming));
        }
        c->pipe_ready = true;
    }
    if (with_hash_streams && !c->hash_streams_ready) {
        for (int i = 0; i < PIPE_SLOTS - 1; i++)
            SENTRY_HIP_CHECK(hipStreamCreateWithFlags(&c->pipe.hash_stream[i], hipStreamNonBlocking));
        c->hash_streams_ready = true;
    }
    *out = &c->pipe;
    return SENTRY_OK;
}

void copy_pipe_drain(CopyPipe *pipe, bool with_hash_streams)
{
    if (!pipe) return;
    (void)hipStreamSynchronize(pipe->copy_stream);
    if (with_hash_streams)
        for (int i = 0; i < PIPE_SLOTS - 1; i++)
            if (pipe->hash_stream[i]) (void)hipStreamSynchronize(pipe->hash_stream[i]);
    (void)hipGetLastError();
}

struct Retired {
    void *ptr;
    hipEvent_t done;
};
static std::vector<Retired> g_retired;

int retire_device_memory(void *dev_ptr, hipStream_t stream)
{
    std::lock_guard<std::mutex> lock(g_mu);
    Retired r = {dev_ptr, nullptr};
    SENTRY_HIP_CHECK(hipEventCreateWithFlags(&r.done, hipEventDisableTiming));
    SENTRY_HIP_CHECK(hipEventRecord(r.done, stream));
    g_retired.push_back(r);
    return SENTRY_OK;
}

static int sweep_retired_locked()
{
    for (size_t i = 0; i < g_retired.size();) {
        hipError_t q = hipEventQuery(g_retired[i].done);
        if (q == hipErrorNotReady) { i++; continue; }
        SENTRY_HIP_CHECK(q);
        SENTRY_HIP_CHECK(hipFree(g_retired[i].ptr));
        SENTRY_HIP_CHECK(hipEventDestroy(g_retired[i].done));
        g_retired[i] = g_retired.back();
        g_retired.pop_back();
    }
    return SENTRY_OK;
}

int sweep_retired()
{
    std::lock_guard<std::mutex> lock(g_mu);
    return sweep_retired_locked();
}

// Bytes the library holds for (current device, stream): scratch regions, and pinned table staging.
int scratch_bytes(hipStream_t stream, size_t *device_bytes, size_t *pinned_bytes)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int dev = 0;
    SENTRY_HIP_CHECK(hipGetDevice(&dev));
    size_t d = 0, h = 0;
    auto it = g_ctx.find(std::make_pair(dev, stream));
    if (it != g_ctx.end()) {
        for (int r = 0; r < R_COUNT; r++) d += it->second.cap[r];
        for (int t = 0; t < TABLE_SLOTS; t++) h += it->second.tab_cap[t];
    }
    *device_bytes = d;
    *pinned_bytes = h;
    return SENTRY_OK;
}

int release_all_scratch()
{
    std::lock_guard<std::mutex> lock(g_mu);
    int dev = 0;
    SENTRY_HIP_CHECK(hipGetDevice(&dev));
    SENTRY_HIP_CHECK(hipDeviceSynchronize());
    {
        int rc = sweep_retired_locked();
        if (rc) return rc;
    }
    for (auto it = g_ctx.begin(); it != g_ctx.end();) {
        if (it->first.first != dev) { ++it; continue; }
        StreamCtx &c = it->second;
        for (int r = 0; r < R_COUNT; r++)
            if (c.region[r]) SENTRY_HIP_CHECK(hipFree(c.region[r]));
        for (int t = 0; t < TABLE_SLOTS; t++) {
            if (c.tab_host[t]) SENTRY_HIP_CHECK(hipHostFree(c.tab_host[t]));
            if (c.tab_event[t]) SENTRY_HIP_CHECK(hipEventDestroy(c.tab_event[t]));
        }
        if (c.pipe_ready) {
            SENTRY_HIP_CHECK(hipStreamDestroy(c.pipe.copy_stream));
            SENTRY_HIP_CHECK(hipEventDestroy(c.pipe.start));
            if (c.hash_streams_ready)
                for (int i = 0; i < PIPE_SLOTS - 1; i++) SENTRY_HIP_CHECK(hipStreamDestroy(c.pipe.hash_stream[i]));
            for (int i = 0; i < PIPE_SLOTS; i++) {
                SENTRY_HIP_CHECK(hipEventDestroy(c.pipe.copied[i]));
                SENTRY_HIP_CHECK(hipEventDestroy(c.pipe.consumed[i]));
            }
        }
        it = g_ctx.erase(it);
    }
    return SENTRY_OK;
}

}  // namespace sentry

extern "C" {

const char *sentry_last_error(void) { return sentry::g_err; }

int sentry_scratch_bytes(void *stream, size_t *out_device_bytes, size_t *out_pinned_bytes)
{
    sentry::clear_error();
    SENTRY_REQUIRE(out_device_bytes != nullptr || out_pinned_bytes != nullptr, "sentry_scratch_bytes: NULL outputs");
    size_t d = 0, h = 0;
    const int rc = sentry::scratch_bytes(static_cast<hipStream_t>(stream), &d, &h);
    if (rc) return rc;
    if (out_device_bytes) *out_device_bytes = d;
    if (out_pinned_bytes) *out_pinned_bytes = h;
    return SENTRY_OK;
}

int sentry_release_scratch(void)
{
    sentry::clear_error();
    return sentry::release_all_scratch();
}

int sentry_reserve_scratch(size_t merkle_max_len, size_t merkle_leaf_bytes, size_t lthash_max_records, void *stream)
{
    sentry::clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    SENTRY_REQUIRE(merkle_leaf_bytes == 0 || merkle_leaf_bytes % 64 == 0,
                   "sentry_reserve_scratch: merkle_leaf_bytes must be 0 or a multiple of 64 (got %zu)", merkle_leaf_bytes);
    SENTRY_REQUIRE(lthash_max_records <= 0xffffffffull / 4 - 64, "sentry_reserve_scratch: too many records");
    int rc;
    if (merkle_leaf_bytes && (rc = sentry::merkle_reserve(merkle_max_len, merkle_leaf_bytes, s))) return rc;
    if (lthash_max_records && (rc = sentry::lthash_reserve(lthash_max_records, s))) return rc;
    return SENTRY_OK;
}

int sentry_verify(const uint8_t *root, const uint8_t *expected)
{
    sentry::clear_error();
    SENTRY_REQUIRE(root && expected, "sentry_verify: NULL digest");
    unsigned diff = 0;   // no early exit: the time does not depend on where they differ
    for (int i = 0; i < SENTRY_DIGEST_BYTES; i++) diff |= (unsigned)(root[i] ^ expected[i]);
    return diff ? SENTRY_MISMATCH : SENTRY_OK;
}

}  // extern "C"
