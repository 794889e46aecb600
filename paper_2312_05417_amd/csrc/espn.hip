// C-ABI of the re-ranking library (declarations and contracts: include/espn.h).
// Host side only validates arguments and enqueues kernels; every step of the path runs in the
// kernels of maxsim_kernels.h / topk_kernels.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <condition_variable>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "../../include/espn.h"
#include "maxsim_kernels.h"
#include "order_kernels.h"
#include "staging_kernels.h"
#include "topk_kernels.h"

#define ESPN_API extern "C" __attribute__((visibility("default")))

namespace {

thread_local char g_err[512] = "";

int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}

#define HIP_TRY(call)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (call);                                                            \
        if (e_ != hipSuccess)                                                              \
            return fail(e_ == hipErrorOutOfMemory ? ESPN_ERR_NOMEM : ESPN_ERR_HIP,         \
                        "%s failed: %s", #call, hipGetErrorString(e_));                    \
    } while (0)

// Restores the caller's current device on scope exit.
struct DeviceScope {
    int prev = -1;
    bool ok = false;
    explicit DeviceScope(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
    }
    ~DeviceScope()
    {
        int cur = -1;
        if (prev >= 0 && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

constexpr size_t kAlign = 256;
// Most devices a process is expected to see (the per-device address of the static scratch is kept in a table).
constexpr int kMaxDevices = 64;
// Workgroups of the host-to-HBM copy kernel: 32 x 4 waves x 8 KiB = 1 MiB of reads in flight.  PCIe needs
// about 64 GB/s x 5 us = 0.3 MiB to stay busy (measured: 8 workgroups reach 45 GB/s, 16 and more 56-57 GB/s),
// and every host read that waits in the memory system's queues delays the HBM reads of the scoring kernel
// running beside it (measured: with 256 workgroups a 2.7 ms scoring launch took 45 ms on average, with 32: 3.1 ms).
constexpr unsigned kGatherBlocks = 32;
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

// Scratch of espn_rerank_noalloc: the scores of one batch, up to ESPN_NOALLOC_MAX_PAIRS of them, in an array
// that is part of the code object, so that the call has nothing to allocate.  Every device the library runs on
// holds a copy of its own at an address of its own; in host code the name below is only a handle for
// hipGetSymbolAddress, never an address to pass to a kernel.
static __device__ __align__(256) unsigned char scratch[sizeof(float) * (size_t)ESPN_NOALLOC_MAX_PAIRS];

namespace {
std::mutex g_scratch_mutex;
void *g_scratch_of_device[kMaxDevices] = {};

// Address of `scratch` on `device`, which must be the current device; asked for once per device.
int scratch_address(int device, void **out)
{
    if (device < 0 || device >= kMaxDevices) return fail(ESPN_ERR_UNSUPPORTED, "device %d is beyond the %d this build tracks", device, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_of_device[device]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(ESPN_ERR_HIP, "hipGetSymbolAddress gave no address for the static scratch on device %d", device);
        g_scratch_of_device[device] = p;
    }
    *out = g_scratch_of_device[device];
    return ESPN_OK;
}
}  // namespace

// One HBM staging slot of a host-resident table (all device memory, owned by the table).
struct StagingSlot {
    void *rows = nullptr;                  // [capacity_rows, dim] in the table's row format
    int64_t *row_map = nullptr;            // [n_docs] first staged row of a document (valid if its bit is set)
    unsigned *bits = nullptr;              // [ceil(n_docs / 32)] documents held by the slot
    int64_t *uniq = nullptr;               // [capacity_docs] distinct documents of the batch
    int64_t *other_row = nullptr;          // [capacity_docs] where each one's rows come from: a row of another slot, or -1 (host)
    int64_t *handed = nullptr;             // [capacity_docs] the same for the packing engine (which keeps slot rows in other_row)
    unsigned long long *counters = nullptr;  // [4]: distinct documents, rows reserved, rows taken from other slots
    uint64_t filled_at = 0;                // sequence number of the last prefetch into the slot (0: never)
    hipEvent_t ready = nullptr;            // recorded when a prefetch into the slot has been enqueued
    hipEvent_t consumed = nullptr;         // recorded when a re-rank reading the slot has been enqueued
};

// Worker threads of the packing prefetch engine: run(n, f) calls f(0) .. f(n-1), f(0) on the calling thread.
class PackPool {
public:
    ~PackPool()
    {
        {
            std::lock_guard<std::mutex> lock(m_);
            stop_ = true;
        }
        go_.notify_all();
        for (std::thread &t : workers_) t.join();
    }
    // may throw (std::system_error, std::bad_alloc): call it inside a try block
    void start(int n_workers)
    {
        for (int x = 0; x < n_workers; ++x) workers_.emplace_back([this, x] { loop(x + 1); });
    }
    int parts() const { return (int)workers_.size() + 1; }
    template <typename F>
    void run(int n, const F &f)
    {
        struct Call { static void thunk(const void *ctx, int x) { (*static_cast<const F *>(ctx))(x); } };
        {
            std::lock_guard<std::mutex> lock(m_);
            job_ = &Call::thunk;
            ctx_ = &f;
            n_ = n;
            pending_ = std::min(n, parts()) - 1;
            ++generation_;
        }
        go_.notify_all();
        f(0);
        std::unique_lock<std::mutex> lock(m_);
        done_.wait(lock, [this] { return pending_ == 0; });
    }

private:
    void loop(int x)
    {
        uint64_t seen = 0;
        while (true) {
            void (*job)(const void *, int);
            const void *ctx;
            {
                std::unique_lock<std::mutex> lock(m_);
                go_.wait(lock, [&] { return stop_ || generation_ != seen; });
                if (stop_) return;
                seen = generation_;
                if (x >= n_) continue;
                job = job_;
                ctx = ctx_;
            }
            job(ctx, x);
            std::lock_guard<std::mutex> lock(m_);
            if (--pending_ == 0) done_.notify_one();
        }
    }
    std::vector<std::thread> workers_;
    std::mutex m_;
    std::condition_variable go_, done_;
    void (*job_)(const void *, int) = nullptr;
    const void *ctx_ = nullptr;
    int n_ = 0, pending_ = 0;
    uint64_t generation_ = 0;
    bool stop_ = false;
};

// Host side of the packing prefetch engine (espn_prefetch_packed), made on its first call.
struct PackState {
    void *buf[2] = {nullptr, nullptr};          // pinned, kPackBytes each: rows on their way to a slot
    hipEvent_t sent[2] = {nullptr, nullptr};    // recorded after the copy out of buf[i] has been enqueued
    bool in_flight[2] = {false, false};
    int64_t *uniq = nullptr;                    // pinned, [capacity_docs]: distinct documents of the batch
    int64_t *row0 = nullptr;                    // pinned, [capacity_docs]: first slot row of each
    int64_t *from = nullptr;                    // pinned, [capacity_docs]: slot << OTHER_SHIFT | row it can be taken from, or -1
    // Which slot holds a document since the newest packed prefetch that brought it (slot << OTHER_SHIFT | first row
    // there; -1: none), and that slot's prefetch number then: the entry holds while the slot has not been refilled.
    std::vector<int64_t> where;
    std::vector<uint32_t> where_gen;
    std::vector<int64_t> scratch;               // [3 * capacity_docs]: the lists while they are put in order
    std::vector<int64_t> found;                 // [2 * pairs of the largest batch so far]: (id, length) as the threads find them
    hipEvent_t lists_sent = nullptr;            // the copies out of uniq / row0 have been enqueued
    bool lists_in_flight = false;
    std::vector<uint64_t> seen;                 // one bit per document of the table
    PackPool pool;
};

struct espn_table {
    const void *emb = nullptr;       // borrowed; the device-visible address if the table is in host memory
    const uint8_t *emb_host = nullptr;   // borrowed; the host address of a host-resident table
    int64_t *off_host = nullptr;     // owned copy of the offsets of a host-resident table, [n_docs + 1]
    PackState *pack = nullptr;       // owned
    float *scale_dev = nullptr;      // owned, [n_docs] document scales of an E4M3 table, else nullptr
    int32_t elem_bytes = 2;          // 2: binary16 rows, 1: E4M3 codes
    int64_t *off_dev = nullptr;      // owned, [n_docs + 1]
    unsigned *err_dev = nullptr;     // owned, one flag word
    void *static_scratch = nullptr;  // this device's copy of the file-scope scratch array (espn_rerank_noalloc)
    int n_cu = 256;                  // compute units of the device
    int64_t n_docs = 0;
    int64_t total_rows = 0;
    int32_t dim = 0;
    int32_t residency = 0;
    int32_t device = 0;
    int32_t fetch = ESPN_FETCH_AUTO;   // how rows of 128 bytes and more are fetched
    float *share_host = nullptr;       // owned, pinned: where espn_table_sample's kernel leaves its result
    float *share_dev = nullptr;        // the same word as the device sees it
    float overlap = -1.f;              // the last espn_table_sample result (-1: none yet); read by plan_slices
    unsigned *popular_dev = nullptr;   // owned, one bit per document: listed by many queries of the sampled batch
    bool popular_valid = false;        // the last sample found overlapping lists and filled popular_dev
    hipStream_t lane[ESPN_BATCH_LANES] = {};      // owned: the streams espn_rerank_batches spreads its batches over
    hipEvent_t fork = nullptr;                    // owned: the caller's stream has reached the call
    hipEvent_t joined[ESPN_BATCH_LANES] = {};     // owned: a lane has finished the call's batches
    StagingSlot slot[espn::MAX_SLOTS];
    int n_slots = 0;
    uint64_t prefetches = 0;         // prefetches enqueued so far
    int64_t capacity_rows = 0;
    int64_t capacity_docs = 0;
    bool has_staging = false;
};

ESPN_API const char *espn_status_string(int status)
{
    switch (status) {
        case ESPN_OK: return "ok";
        case ESPN_ERR_ARG: return "bad argument";
        case ESPN_ERR_SHAPE: return "inconsistent sizes";
        case ESPN_ERR_OFFSETS: return "malformed offsets";
        case ESPN_ERR_ID_RANGE: return "candidate id out of range";
        case ESPN_ERR_NOMEM: return "out of memory";
        case ESPN_ERR_HIP: return "HIP runtime error";
        case ESPN_ERR_UNSUPPORTED: return "unsupported shape";
        default: return "unknown status";
    }
}

ESPN_API const char *espn_last_error(void) { return g_err; }

namespace {
int load_table(const void *emb, const float *doc_scale_host, const int64_t *offsets_host, int64_t n_docs, int32_t dim,
               int32_t residency, int32_t device, espn_table **out);

void destroy_lanes(espn_table *t)
{
    for (int l = 0; l < ESPN_BATCH_LANES; ++l) {
        if (t->lane[l]) (void)hipStreamDestroy(t->lane[l]);
        if (t->joined[l]) (void)hipEventDestroy(t->joined[l]);
        t->lane[l] = nullptr;
        t->joined[l] = nullptr;
    }
    if (t->fork) (void)hipEventDestroy(t->fork);
    t->fork = nullptr;
}
}

ESPN_API int espn_table_load(const void *emb, const int64_t *offsets_host, int64_t n_docs, int32_t dim,
                             int32_t residency, int32_t device, espn_table **out)
{
    return load_table(emb, nullptr, offsets_host, n_docs, dim, residency, device, out);
}

ESPN_API int espn_table_load_e4m3(const void *codes, const float *doc_scale_host, const int64_t *offsets_host,
                                  int64_t n_docs, int32_t dim, int32_t residency, int32_t device, espn_table **out)
{
    if (out) *out = nullptr;
    if (!doc_scale_host) return fail(ESPN_ERR_ARG, "doc_scale_host is NULL");
    if (dim != 32 && dim != 128) return fail(ESPN_ERR_UNSUPPORTED, "E4M3 tables need dim 32 or 128, got %d", dim);
    for (int64_t i = 0; i < n_docs; ++i)
        if (!(doc_scale_host[i] > 0.f) || !(doc_scale_host[i] < __builtin_inff()))
            return fail(ESPN_ERR_ARG, "scale of document %lld is not positive and finite", (long long)i);
    return load_table(codes, doc_scale_host, offsets_host, n_docs, dim, residency, device, out);
}

namespace {
int load_table(const void *emb, const float *doc_scale_host, const int64_t *offsets_host, int64_t n_docs, int32_t dim,
               int32_t residency, int32_t device, espn_table **out)
{
    if (!out) return fail(ESPN_ERR_ARG, "out is NULL");
    *out = nullptr;
    if (!offsets_host) return fail(ESPN_ERR_ARG, "offsets_host is NULL");
    if (n_docs < 0) return fail(ESPN_ERR_ARG, "n_docs = %lld is negative", (long long)n_docs);
    if (dim <= 0 || dim % 8 != 0) return fail(ESPN_ERR_ARG, "dim = %d is not a positive multiple of 8", dim);
    if (residency != ESPN_RESIDENT_HBM && residency != ESPN_RESIDENT_HOST_PINNED && residency != ESPN_RESIDENT_HOST)
        return fail(ESPN_ERR_ARG, "residency = %d is not a known value", residency);
    if (offsets_host[0] != 0) return fail(ESPN_ERR_OFFSETS, "offsets[0] = %lld, expected 0", (long long)offsets_host[0]);
    for (int64_t i = 0; i < n_docs; ++i)
        if (offsets_host[i + 1] < offsets_host[i])
            return fail(ESPN_ERR_OFFSETS, "offsets decrease at document %lld", (long long)i);
    const int64_t total = offsets_host[n_docs];
    if (total > 0 && !emb) return fail(ESPN_ERR_ARG, "emb is NULL");
    if (!aligned16(emb)) return fail(ESPN_ERR_ARG, "emb is not 16-byte aligned");
    int ndev = 0;
    HIP_TRY(hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) return fail(ESPN_ERR_ARG, "device %d of %d", device, ndev);

    DeviceScope scope(device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", device);
    espn_table *t = new (std::nothrow) espn_table;
    if (!t) return fail(ESPN_ERR_NOMEM, "host allocation failed");
    t->emb = emb;
    t->elem_bytes = doc_scale_host ? 1 : 2;
    if (residency == ESPN_RESIDENT_HOST_PINNED && total > 0) {
        void *dev_view = nullptr;
        hipError_t he = hipHostGetDevicePointer(&dev_view, const_cast<void *>(emb), 0);
        if (he != hipSuccess || !dev_view) {
            (void)hipGetLastError();
            delete t;
            return fail(ESPN_ERR_ARG, "emb is not pinned host memory the device can address (%s)",
                        hipGetErrorString(he));
        }
        t->emb = dev_view;
        t->emb_host = static_cast<const uint8_t *>(emb);
    }
    if (residency == ESPN_RESIDENT_HOST) {       // ordinary host memory: only the host ever reads it
        t->emb = nullptr;
        t->emb_host = static_cast<const uint8_t *>(emb);
    }
    if (residency != ESPN_RESIDENT_HBM) {
        t->off_host = new (std::nothrow) int64_t[(size_t)n_docs + 1];
        if (!t->off_host) {
            delete t;
            return fail(ESPN_ERR_NOMEM, "host allocation failed");
        }
        std::memcpy(t->off_host, offsets_host, sizeof(int64_t) * ((size_t)n_docs + 1));
    }
    t->n_docs = n_docs;
    t->total_rows = total;
    t->dim = dim;
    t->residency = residency;
    t->device = device;
    const size_t off_bytes = sizeof(int64_t) * (size_t)(n_docs + 1);
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&t->off_dev), off_bytes);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&t->err_dev), kAlign);
    if (e == hipSuccess) e = hipMemcpy(t->off_dev, offsets_host, off_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(t->err_dev, 0, kAlign);
    if (e == hipSuccess) {
        int n_cu = 0;
        e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device);
        if (e == hipSuccess && n_cu > 0) t->n_cu = n_cu;
    }
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void **>(&t->share_host), kAlign, hipHostMallocDefault);
    if (e == hipSuccess) {
        *t->share_host = -1.f;
        e = hipHostGetDevicePointer(reinterpret_cast<void **>(&t->share_dev), t->share_host, 0);
    }
    // the streams of espn_rerank_batches (default priority, not synchronising with the null stream) and its events
    for (int l = 0; l < ESPN_BATCH_LANES && e == hipSuccess; ++l) {
        e = hipStreamCreateWithFlags(&t->lane[l], hipStreamNonBlocking);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&t->joined[l], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&t->fork, hipEventDisableTiming);
    if (e == hipSuccess && doc_scale_host) {
        e = hipMalloc(reinterpret_cast<void **>(&t->scale_dev), sizeof(float) * (size_t)(n_docs + 1));
        if (e == hipSuccess && n_docs > 0)
            e = hipMemcpy(t->scale_dev, doc_scale_host, sizeof(float) * (size_t)n_docs, hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    int scratch_rc = ESPN_OK;
    if (e == hipSuccess) scratch_rc = scratch_address(device, &t->static_scratch);      // `device` is current here
    if (e != hipSuccess || scratch_rc != ESPN_OK) {
        (void)hipFree(t->off_dev);
        (void)hipFree(t->err_dev);
        (void)hipFree(t->scale_dev);
        if (t->share_host) (void)hipHostFree(t->share_host);
        destroy_lanes(t);
        delete[] t->off_host;
        delete t;
        if (e == hipSuccess) return scratch_rc;           // the message is already set
        return fail(e == hipErrorOutOfMemory ? ESPN_ERR_NOMEM : ESPN_ERR_HIP, "table set-up failed: %s",
                    hipGetErrorString(e));
    }
    *out = t;
    return ESPN_OK;
}
}  // namespace

namespace {
void free_pack_state(espn_table *t)
{
    PackState *p = t->pack;
    if (!p) return;
    for (int i = 0; i < 2; ++i) {
        if (p->buf[i]) (void)hipHostFree(p->buf[i]);
        if (p->sent[i]) (void)hipEventDestroy(p->sent[i]);
    }
    if (p->uniq) (void)hipHostFree(p->uniq);
    if (p->row0) (void)hipHostFree(p->row0);
    if (p->from) (void)hipHostFree(p->from);
    if (p->lists_sent) (void)hipEventDestroy(p->lists_sent);
    delete p;
    t->pack = nullptr;
}

void free_staging(espn_table *t)
{
    free_pack_state(t);                 // its lists are sized by the slots' capacity
    for (StagingSlot &s : t->slot) {
        (void)hipFree(s.rows);
        (void)hipFree(s.row_map);
        (void)hipFree(s.bits);
        (void)hipFree(s.uniq);
        (void)hipFree(s.other_row);
        (void)hipFree(s.handed);
        (void)hipFree(s.counters);
        if (s.ready) (void)hipEventDestroy(s.ready);
        if (s.consumed) (void)hipEventDestroy(s.consumed);
        s = StagingSlot();
    }
    t->n_slots = 0;
    t->has_staging = false;
}
}  // namespace

ESPN_API int espn_table_free(espn_table *table)
{
    if (!table) return ESPN_OK;
    DeviceScope scope(table->device);
    (void)hipDeviceSynchronize();
    free_staging(table);
    (void)hipFree(table->off_dev);
    (void)hipFree(table->err_dev);
    (void)hipFree(table->scale_dev);
    if (table->share_host) (void)hipHostFree(table->share_host);
    (void)hipFree(table->popular_dev);
    destroy_lanes(table);
    delete[] table->off_host;
    delete table;
    return ESPN_OK;
}

namespace {
// Lists of a batch are taken to share documents if more than this fraction of a sample of 4096 pairs repeats a
// document of the sample (uniform lists over 2 M documents: 0.002; Zipf(1.1) lists: above 0.5)
constexpr float kShareThreshold = 0.05f;
// ... and a document is popular (fetched through the caches by launches that stream the rest) if at least this many
// of the sampled batch's lists name it, and at least one list in kPopularShare.  (2048 Zipf(1.1) lists of 1000 over
// 2 M documents, the 3 000 to 30 000 most listed documents marked: the same speed to within 2 %; 100 000: 3 % slower.)
constexpr int kPopularListings = 2;
constexpr int kPopularShare = 256;
// Launches of at least this many workgroups per compute unit take lists that overlap in id order (the ordering pass
// is a launch of its own, of about 1 % of a long scoring launch).  One call per batch, Zipf lists of 1000 over 2 M
// documents, 256-byte rows: 128 queries (768 workgroups) 294 against 307 us, 192 queries (768) 411 against 448, 2048
// queries 3.80 against 4.66 ms; 64 queries (256 workgroups) 172 against 165, 32 queries 113 against 92.
constexpr int kOrderFrom = 3;
}  // namespace

ESPN_API int espn_table_set_fetch(espn_table *table, int32_t mode)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (mode != ESPN_FETCH_AUTO && mode != ESPN_FETCH_STREAMING && mode != ESPN_FETCH_CACHED)
        return fail(ESPN_ERR_ARG, "fetch mode %d is not a known value", mode);
    table->fetch = mode;
    return ESPN_OK;
}

ESPN_API int espn_table_sharing_estimate(const espn_table *table, float *estimate)
{
    if (!table || !estimate) return fail(ESPN_ERR_ARG, "NULL pointer");
    *estimate = table->overlap;
    return ESPN_OK;
}

ESPN_API int espn_table_sample(espn_table *table, const int64_t *cand, int32_t B, int32_t K, void *stream)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (B < 0 || K < 0) return fail(ESPN_ERR_ARG, "B = %d, K = %d: negative size", B, K);
    if (B > 0 && K > 0 && !cand) return fail(ESPN_ERR_ARG, "cand is NULL");
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    *table->share_host = 0.f;
    if (B > 0 && K > 0) {
        hipLaunchKernelGGL(espn::sharing_probe_kernel, dim3(1), dim3(1024), 0, st, cand, (int64_t)B * K, K, K,
                           table->share_dev);
        HIP_TRY(hipGetLastError());
    }
    HIP_TRY(hipStreamSynchronize(st));
    table->overlap = *static_cast<volatile const float *>(table->share_host);
    // overlapping lists: which documents they keep coming back to
    table->popular_valid = false;
    if (table->overlap >= kShareThreshold && table->residency == ESPN_RESIDENT_HBM && table->dim != 32) {
        const int64_t words = (table->n_docs + 31) / 32;
        if (!table->popular_dev) HIP_TRY(hipMalloc(&table->popular_dev, sizeof(unsigned) * (size_t)words));
        unsigned *counts = nullptr;
        HIP_TRY(hipMalloc(&counts, sizeof(unsigned) * (size_t)table->n_docs));
        const int64_t n_pairs = (int64_t)B * K;
        const unsigned at_least = (unsigned)std::max(kPopularListings, B / kPopularShare);
        hipError_t e = hipMemsetAsync(counts, 0, sizeof(unsigned) * (size_t)table->n_docs, st);
        if (e == hipSuccess) {
            hipLaunchKernelGGL(espn::listings_kernel, dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, st, cand,
                               n_pairs, K, K, table->n_docs, counts);
            hipLaunchKernelGGL(espn::popular_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, counts,
                               table->n_docs, at_least, table->popular_dev);
            e = hipGetLastError();
        }
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        (void)hipFree(counts);
        HIP_TRY(e);
        table->popular_valid = true;
    }
    return ESPN_OK;
}

ESPN_API int espn_table_info(const espn_table *table, int64_t *n_docs, int64_t *total_rows, int32_t *dim,
                             int32_t *residency, int32_t *device)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (n_docs) *n_docs = table->n_docs;
    if (total_rows) *total_rows = table->total_rows;
    if (dim) *dim = table->dim;
    if (residency) *residency = table->residency;
    if (device) *device = table->device;
    return ESPN_OK;
}

namespace {

int check_batch(const espn_table *table, const void *q, const int64_t *cand, int32_t B, int32_t Q, int32_t K)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (B < 0 || K < 0) return fail(ESPN_ERR_ARG, "B = %d, K = %d: negative size", B, K);
    if (Q < 1) return fail(ESPN_ERR_ARG, "Q = %d: a query needs at least one row", Q);
    // one workgroup per candidate at most (the generic kernel: four candidates per workgroup), in a
    // one-dimensional grid
    if ((int64_t)B * std::max(K, 1) > (int64_t)0x7fffffff)
        return fail(ESPN_ERR_UNSUPPORTED, "B * K = %lld exceeds 2^31 - 1 pairs per call", (long long)B * K);
    if (B > 0 && K > 0 && (!q || !cand)) return fail(ESPN_ERR_ARG, "q or cand is NULL");
    if (!aligned16(q)) return fail(ESPN_ERR_ARG, "q is not 16-byte aligned");
    return ESPN_OK;
}

// Waves per workgroup of the matrix-core kernel: two workgroups fit a compute unit for the paper's two
// row lengths (32: 40 VGPRs x 16 waves, 128: 112 VGPRs x 8 waves); longer rows hold more registers per wave.
constexpr int waves_per_workgroup(int dim) { return dim == 32 ? 16 : dim <= 128 ? 8 : 4; }
// 64-byte rows, launches of at least four workgroups per compute unit: the same 32 waves per compute
// unit come as four workgroups of 8 waves, which start and retire in smaller steps (measured 5-10 %
// faster from 1024 workgroups on, slower below).
constexpr int kNarrowWaves = 8;
// 256-byte binary16 rows, at least eight workgroups per compute unit: four workgroups of 4 waves per
// compute unit instead of two of 8 (measured: c3 764 -> 760 us, c4 4.80 -> 4.68 ms; E4M3 rows of the
// same length lose 4 % with it and keep 8 waves).
constexpr int kNarrowWaves128 = 4;

// The planner's numbers, all per compute unit (n_cu comes from the device) or per workgroup:
constexpr int kResidentPerCu = 2;        // workgroups of the scoring kernel a compute unit holds at once (32 waves: 2 x 16 or 2 x 8 + registers)
constexpr int kThreePerCu = 3;           // the cut that gives three workgroups per compute unit (171-192 queries)
constexpr int kFewestFitted = 4;         // 193-255 queries: slice counts tried for the best fit to whole rounds of
constexpr int kMostFitted = 12;          //   one workgroup per compute unit ...
constexpr double kPerSlicePenalty = 0.02;    // ... fewer slices preferred: a slice more must fill 2 % more of its last round
constexpr int kLongestCutSlice = 256;    // a cut that fills the device once may make slices of up to this many candidates
constexpr int kFixedSlice32 = 125;       // slice of launches beyond one round: candidates of 64-byte rows (2.5 KB each)
constexpr int kFixedSlice128 = 63;       //   and of 256-byte rows (18 KB each); +/- a factor 2 costs 1-2 %
constexpr int kNarrowFrom = 4;           // workgroups per compute unit from which 64-byte rows run in workgroups of kNarrowWaves
constexpr int kNarrowFrom128 = 8;        //   and 256-byte binary16 rows in workgroups of kNarrowWaves128

// How a batch is cut into workgroup slices, and whether the scoring kernel ranks as well.
struct SlicePlan {
    int slice = 0;          // candidates per workgroup
    int slices = 0;         // workgroups per query
    int waves = 0;          // waves per workgroup
    bool rank = false;      // the scoring kernel writes the top-k itself
    bool linear = false;    // non-temporal row loads (rows longer than 64 bytes: lane-linear, tiles transposed through LDS)
};

// Slices per query.  A launch small enough to be resident at once (two workgroups per compute unit)
// is cut so that it fills the device exactly once: nothing is left to start late, and the waves of
// a workgroup share its documents one by one, so all workgroups end together.  Larger launches use
// slices of a fixed size that the dispatcher hands out as workgroups retire (measured on MI355X:
// 125 candidates of 2.5 KB and 63 of 18 KB are the best sizes, +/- a factor 2 costs 1-2 %).
// The kernel ranks as well when that leaves one slice of at most RANK_MAX candidates per query.
//
// Refinements, all measured over batches of 1 to 768 queries with lists of 16 to 1000 candidates (two here, two
// more where plan_slices applies them):
// - the cut rounds down (floor(slots / B) slices, not ceil): a few workgroups more than the device holds
//   run after the others, alone, and the launch takes as long as two rounds (136 queries of 256
//   candidates, 64-byte rows: 25.8 us with 3 slices, 28.0 with 4; 192 queries: 2 slices beat 3 for every
//   list length and both row lengths, by 2-8 %).  More than half the slots' worth of queries: 2 slices.
// - a list short enough that the waves of one workgroup finish it in a few documents each is not cut at
//   all: the scoring kernel then ranks it, and the second launch (a 4.5-5 us kernel) costs more than the
//   documents a wave takes one after the other.  How many documents per wave that may be depends on what the
//   cut would buy (uncut_rounds): with few queries it spreads them over compute units that would idle, from
//   half a workgroup per compute unit on there is little left to spread to.  64 candidates of 64-byte rows:
//   9.7 against 12.3 us per batch of 1 to 64 queries, 12.3 against 15.8 at 192 queries.
// Documents per wave up to which a rankable list stays uncut, by queries per compute unit (n_cu = 256 here;
// whole path, us per batch, uncut against cut the way plan_slices cuts; "narrow" = 64-byte rows in workgroups of
// 16 waves, "wide" = longer rows in workgroups of 8, "codes" = 32-byte rows of E4M3 codes in workgroups of 16, for
// which the cut list is cheaper than for binary16 rows: 80 candidates at 100 queries 13.5 uncut against 12.0 cut,
// 96 candidates at 192 queries 16.4 against 15.2, but 64 candidates 9.2-12.4 against 11.7-13.7 at 16 to 256 queries):
// "wide, cached" = the longer rows when the lists of a batch share documents and the rows are fetched with ordinary
// loads (each lane its own part of a row): a document costs more there while the launch is short, so lists of few
// queries are cut sooner (Zipf lists, 16 queries of 16 candidates: 16.6 uncut against 12.5 cut, 100 queries of 32:
// 26.2 against 21.7, 150 queries of 64: 43.6 against 41.0; from 171 queries on uncut wins as before, 192 queries of
// 128 candidates: 76.9 against 84.3).  64-byte rows keep their limits under such lists (64 candidates: 9.6-14.5
// against 12.0-17.0 at 16 to 400 queries; 112 candidates at 256 queries: 18.2 against 17.0).
struct UncutBand {
    int num, den;           // the band ends at B = num / den * n_cu
    int narrow, wide, codes, wide_cached;
};
constexpr UncutBand kUncutBands[] = {
    // few queries: narrow, 80 candidates (5 per wave) 11.4 against 11.8 at 16 queries, 12.4 against 12.9 at 64;
    // 100 candidates 14.4 against 12.4 at 64.  Wide, 16 candidates (2 per wave) 12.4 against 12.8 at 16 queries;
    // 24 candidates 15.5 against 13.4
    {3, 8, 5, 2, 4, 1},
    // 100-128 queries: wide, 32 candidates (4 per wave) 20.6 against 23.4; 64 candidates 33.5 against 29.6
    {1, 2, 5, 4, 4, 2},
    // 129-170: narrow, 80 candidates 13.7 against 15.5, 112 candidates (7 per wave) 18.4 against 17.5;
    // wide, 64 candidates (8 per wave) 36.9 against 39.9
    {2, 3, 6, 8, 5, 4},
    // up to one workgroup per compute unit: narrow, 192 queries, 64 candidates 12.3 against 15.8, 100 candidates
    // 17.8 against 19.4, 128 a tie; wide, 32 candidates 24.8 against 31.7, 64 candidates 41.6 against 49.0, 128
    // candidates (16 per wave) 77.7 against 83.2 (at 256 queries: 98.6 against 99.5)
    {1, 1, 7, 16, 5, 16},
    // some compute units get two workgroups and others one: narrow, 320 queries, 80 candidates 21.4 against 23.0
    // but 112 candidates 28.0 against 27.1; wide, 32 candidates 42.9 against 44.3 but 64 candidates 75.6 against 72.1
    {11, 8, 5, 4, 5, 4},
};
// ... and beyond (up to two per compute unit; from there on nothing is cut anyway): narrow, 400 queries, 112
// candidates 30.3 against 32.5, 100 candidates 26.8 against 30.5; wide, 64 candidates 80.5 against 90.0
constexpr UncutBand kUncutBeyond = {0, 1, 7, 8, 6, 8};

int uncut_rounds(int dim, int elem_bytes, bool streaming, int B, int n_cu)
{
    const UncutBand *band = &kUncutBeyond;
    for (const UncutBand &b : kUncutBands)
        if ((int64_t)B * b.den <= (int64_t)b.num * n_cu) {
            band = &b;
            break;
        }
    if (dim != 32) return streaming ? band->wide : band->wide_cached;
    return elem_bytes == 1 ? band->codes : band->narrow;
}

SlicePlan plan_slices(const espn_table *t, int B, int K, int k)
{
    // Rows of 128 bytes and more can be fetched in two ways.  Each lane loading its own D/2 contiguous bytes
    // needs no transpose, but its four instructions come back to every cache line, so the lines have to stay
    // cached: ordinary loads.  Lane-linear loads take whole lines with one instruction each and can be
    // non-temporal, which this machine streams 13 % faster (c3 761 -> 673 us before the transpose is paid
    // for), but a document that several queries of the batch list is then fetched from memory every time.
    // So, unless the caller has said which it wants: non-temporal when the batch cannot repeat documents much
    // (pairs <= half the documents of the table).  That is right for lists drawn uniformly and wrong for small
    // batches of lists that share popular documents (Zipf: cached loads win from 64 queries on).
    // ... unless the caller has had a batch's lists sampled (espn_table_sample) and so shown how much they overlap
    bool streaming = 2 * (int64_t)B * K <= t->n_docs;
    const float overlap = t->overlap;
    if (overlap >= 0.f) streaming = overlap < kShareThreshold;
    // 64-byte rows are fetched lane-linearly either way, so only the hint is at stake: non-temporal unless a
    // sample has shown overlapping lists (uniform lists, 1024 queries: 1.9 % faster; Zipf lists: 27-36 % slower)
    if (t->dim == 32) streaming = !(overlap >= kShareThreshold);
    // (a host-resident table is scored from a staging slot, which holds each document once for all the queries that
    // list it: ordinary loads)
    const bool linear = t->residency == ESPN_RESIDENT_HBM &&
                        (t->fetch == ESPN_FETCH_STREAMING || (t->fetch == ESPN_FETCH_AUTO && streaming));

    const int waves = waves_per_workgroup(t->dim);
    const int slots = kResidentPerCu * t->n_cu;       // workgroups the device holds at once
    // Rows longer than 64 bytes: the cut aims at ONE workgroup per compute unit, and it may leave half the waves of
    // a workgroup without a document.  Every slice count timed for batches of 8 to 256 queries, 256-byte rows: the
    // best is floor(n_cu / B) throughout, with a cliff right behind it (20 queries of 128 candidates: 17.9 us with
    // 12 slices = 240 workgroups, 21.8 with 13 = 260; 64 queries: 32.9 us with 4 slices, 34.7 with 8; 100
    // queries: 45.8 with 2, 47.5 with 5; 8 queries: 13.0 with 32 slices of 4, 14.1 with 16 of 8).  More than half
    // a compute unit's worth of queries cannot have that and fill the two slots per compute unit instead (136-170
    // queries: 3 slices beat 1, 2 and 4 by 2-25 %).  171 to 192 queries, for which that would be 2 slices, take 4,
    // three workgroups per compute unit (192 queries of 300 candidates: 165.7 us against 175.7; under Zipf lists 144.4
    // against 174.0; as E4M3 codes 93.0 against 98.2), and 193 to 256 queries no longer fit a whole number of
    // workgroups per compute unit with so few slices (200 queries of 500 candidates: 296 us with 3 slices, 276 with
    // 5; Zipf lists 284 against 244; E4M3 165 against 151; from 224 queries on all counts are within a few per cent).  64-byte rows gain 1-8 % from the
    // one-per-compute-unit rule at 20 to 48 queries and nothing elsewhere, and keep two workgroups per compute unit.
    const bool wide = t->dim != 32;
    int one_round = (wide ? t->n_cu : slots) / std::max(B, 1);
    if (one_round < 2) one_round = slots / std::max(B, 1);
    bool fixed = false;
    if (one_round == 2 && B <= t->n_cu && (wide || kThreePerCu * t->n_cu / B >= kFewestFitted)) {
        // (171 to 192 queries: 4 slices for 64-byte rows too: 1000 candidates 83.7-90.1 us against 86.6-91.2 with
        // the fixed slices, 300 candidates 33.3-35.4 against 36.5-37.3 with 2; under Zipf lists 67.5-69.0 against
        // 72.4-72.5 and 27.0-27.5 against 29.4-30.0; as E4M3 codes 58.5-61.7 against 59.2-60.8 and 26.3-26.9
        // against 27.3-27.5.  From 193 queries on no count is better for them in all three settings.)
        one_round = kThreePerCu * t->n_cu / B;
        if (one_round < kFewestFitted) {
            // the count of 4 to 12 slices whose workgroups come closest, from below, to a whole number per compute
            // unit, fewer slices preferred (196-200 queries: 5, 980-1000 workgroups; 210: 6; 240: 4); a full device's
            // worth of queries keeps the fixed slices
            fixed = B == t->n_cu;
            double best = -1.;
            for (int s = kFewestFitted; s <= kMostFitted && !fixed; ++s) {
                const int64_t groups = (int64_t)B * s, rounds = (groups + t->n_cu - 1) / t->n_cu;
                const double score = (double)groups / (double)(rounds * t->n_cu) - kPerSlicePenalty * s;
                if (score > best) {
                    best = score;
                    one_round = s;
                }
            }
        }
    }
    if (one_round < 2) one_round = B < slots ? 2 : 1;
    const int most_slices = std::max(1, wide ? 2 * K / waves : K / waves);     // slices a list can usefully have
    const bool uncut = k >= 1 && K <= espn::RANK_MAX && (K + waves - 1) / waves <= uncut_rounds(t->dim, t->elem_bytes, linear, B, t->n_cu);
    int slices;
    if (uncut) slices = 1;
    else if (!fixed && (K + one_round - 1) / one_round <= kLongestCutSlice) slices = std::min(one_round, most_slices);
    else {
        // fixed slices: 125 candidates of 64-byte rows, 63 of 256-byte rows, in between by row bytes
        const int per_slice = t->dim == 32 ? kFixedSlice32 : std::max(16, kFixedSlice128 * 128 / t->dim);
        slices = (K + per_slice - 1) / per_slice;
    }
    slices = std::max(slices, (K + espn::MAX_SLICE - 1) / espn::MAX_SLICE);
    SlicePlan p;
    p.slice = (K + slices - 1) / slices;
    p.slices = (K + p.slice - 1) / p.slice;
    p.rank = p.slices == 1 && K <= espn::RANK_MAX && k >= 1;
    const int64_t workgroups = (int64_t)B * p.slices;
    p.waves = waves;
    if (t->dim == 32 && workgroups >= kNarrowFrom * (int64_t)t->n_cu) p.waves = kNarrowWaves;
    if (t->dim == 128 && t->elem_bytes == 2 && workgroups >= kNarrowFrom128 * (int64_t)t->n_cu) p.waves = kNarrowWaves128;     // Q <= 32 only
    p.linear = linear;
    return p;
}

// Waves per workgroup a launch runs with (the kernel's WAVES argument), for QG groups of 16 query rows in registers.
// 64 query rows of 192 or 256 bytes take 122-154 VGPRs per lane: in workgroups of 4 waves three of them share a
// compute unit, in workgroups of 8 only one would fit.
int launched_waves(int D, int EB, int QG, const SlicePlan &plan)
{
    if (D == 128 && EB == 2 && QG == 2 && plan.waves == kNarrowWaves128) return kNarrowWaves128;
    if (D == 32 && plan.waves == kNarrowWaves) return kNarrowWaves;
    return (QG == 4 && D > 64) ? 4 : waves_per_workgroup(D);
}
constexpr int kPipeline = 4;                     // register pipeline depth in 16-row tiles (the kernel's P argument)

// QG = groups of 16 query rows the kernel holds in registers: 2 (Q <= 32) or 4 (Q <= 64, rows up to 256 bytes)
template <int D, int EB, bool RANK, int QG, bool LINEAR>
void launch_slices(const espn::DocSource &src, const espn::Batch &bt, const espn::BatchSet &set, const SlicePlan &plan,
                   unsigned *err, const espn::RankOut &ro, hipStream_t st)
{
    constexpr int WAVES = (QG == 4 && D > 64) ? 4 : waves_per_workgroup(D);
    constexpr int P = kPipeline;
    const dim3 grid((unsigned)plan.slices * (unsigned)set.n * (unsigned)set.B);
    const int waves = launched_waves(D, EB, QG, plan);
    if constexpr (D == 128 && EB == 2 && QG == 2) {
        if (waves == kNarrowWaves128) {
            hipLaunchKernelGGL((espn::maxsim_slice_kernel<D, kNarrowWaves128, P, EB, RANK, QG, LINEAR>), grid,
                               dim3(kNarrowWaves128 * 64), 0, st, src, bt, set, err, plan.slice, ro);
            return;
        }
    }
    if constexpr (D == 32) {
        if (waves == kNarrowWaves) {
            hipLaunchKernelGGL((espn::maxsim_slice_kernel<D, kNarrowWaves, P, EB, RANK, QG, LINEAR>), grid,
                               dim3(kNarrowWaves * 64), 0, st, src, bt, set, err, plan.slice, ro);
            return;
        }
    }
    hipLaunchKernelGGL((espn::maxsim_slice_kernel<D, WAVES, P, EB, RANK, QG, LINEAR>), grid, dim3(WAVES * 64), 0, st,
                       src, bt, set, err, plan.slice, ro);
}

template <int D, int EB, bool RANK, int QG>
void launch_slices(const espn::DocSource &src, const espn::Batch &bt, const espn::BatchSet &set, const SlicePlan &plan,
                   unsigned *err, const espn::RankOut &ro, hipStream_t st)
{
    if (plan.linear) launch_slices<D, EB, RANK, QG, true>(src, bt, set, plan, err, ro, st);
    else launch_slices<D, EB, RANK, QG, false>(src, bt, set, plan, err, ro, st);
}

// rows longer than 256 bytes are held for 32 query rows only (their fragments would not fit the registers)
constexpr bool takes_long_queries(int D) { return D <= 128; }

template <int D, int EB>
void launch_slices(const espn::DocSource &src, const espn::Batch &bt, const espn::BatchSet &set, const SlicePlan &plan,
                   unsigned *err, const espn::RankOut &ro, hipStream_t st)
{
    if constexpr (takes_long_queries(D)) {
        if (bt.Q > 32) {
            if (plan.rank) launch_slices<D, EB, true, 4>(src, bt, set, plan, err, ro, st);
            else launch_slices<D, EB, false, 4>(src, bt, set, plan, err, ro, st);
            return;
        }
    }
    if (plan.rank) launch_slices<D, EB, true, 2>(src, bt, set, plan, err, ro, st);
    else launch_slices<D, EB, false, 2>(src, bt, set, plan, err, ro, st);
}

// 16-row query groups in registers: up to 32 query rows for every row length that is a multiple of 32
// up to 256 components, up to 64 for rows of up to 128 components
bool on_matrix_cores(const espn_table *t, int Q)
{
    return t->dim % 32 == 0 && t->dim <= 256 && (Q <= 32 || (Q <= 64 && takes_long_queries(t->dim)));
}

// One batch as the set a launch scores.
espn::BatchSet one_batch(const espn::Batch &bt, int B, float *scores, int64_t *out_ids = nullptr, float *out_scores = nullptr)
{
    espn::BatchSet set{};
    set.n = 1;
    set.B = B;
    set.q[0] = bt.q;
    set.cand[0] = bt.cand;
    set.prior[0] = bt.prior;
    set.scores[0] = scores;
    set.out_ids[0] = out_ids;
    set.out_scores[0] = out_scores;
    return set;
}

// Enqueue the scoring kernel for documents found through `src` (the table itself or a staging slot): the batches
// of `set`, all of the shape `bt` gives, in one launch of set.n * set.B queries that `plan` was made for.
// plan.rank: the kernel also writes the ranked top-k, rows of the shape `ro`.
int enqueue_score(const espn_table *t, const espn::DocSource &src, const espn::Batch &bt, const espn::BatchSet &set,
                  const SlicePlan &plan, const espn::RankOut &ro, hipStream_t st)
{
    using namespace espn;
    if (set.n == 0 || set.B == 0 || bt.K == 0) return ESPN_OK;
    if (t->elem_bytes == 1 && bt.Q > 64)
        return fail(ESPN_ERR_UNSUPPORTED, "E4M3 tables take at most 64 query rows, got %d", bt.Q);
    if (on_matrix_cores(t, bt.Q)) {
        if (t->elem_bytes == 1) {
            if (t->dim == 32) launch_slices<32, 1>(src, bt, set, plan, t->err_dev, ro, st);
            else launch_slices<128, 1>(src, bt, set, plan, t->err_dev, ro, st);
        } else {
            switch (t->dim) {
                case 32: launch_slices<32, 2>(src, bt, set, plan, t->err_dev, ro, st); break;
                case 64: launch_slices<64, 2>(src, bt, set, plan, t->err_dev, ro, st); break;
                case 96: launch_slices<96, 2>(src, bt, set, plan, t->err_dev, ro, st); break;
                case 128: launch_slices<128, 2>(src, bt, set, plan, t->err_dev, ro, st); break;
                case 160: launch_slices<160, 2>(src, bt, set, plan, t->err_dev, ro, st); break;
                case 192: launch_slices<192, 2>(src, bt, set, plan, t->err_dev, ro, st); break;
                case 224: launch_slices<224, 2>(src, bt, set, plan, t->err_dev, ro, st); break;
                default: launch_slices<256, 2>(src, bt, set, plan, t->err_dev, ro, st); break;
            }
        }
    } else {
        const size_t lds = (size_t)bt.Q * t->dim * 2;
        if (lds > 64 * 1024)
            return fail(ESPN_ERR_UNSUPPORTED, "Q * dim * 2 = %zu bytes exceeds the 64 KiB the generic kernel holds", lds);
        const dim3 grid((unsigned)((bt.K + 3) / 4) * set.B), block(256);
        for (int i = 0; i < set.n; ++i) {       // the plain kernel takes one batch per launch
            Batch one = bt;
            one.q = set.q[i];
            one.cand = set.cand[i];
            one.prior = set.prior[i];
            hipLaunchKernelGGL(maxsim_generic_kernel, grid, block, lds, st, src, t->dim, one, set.scores[i], t->err_dev);
        }
    }
    HIP_TRY(hipGetLastError());
    return ESPN_OK;
}

// A batch whose lists are scored whole, without a prior.
espn::Batch plain_batch(const void *q, const int64_t *cand, int Q, int K)
{
    return espn::Batch{static_cast<const uint16_t *>(q), cand, nullptr, 0.f, K, Q, K, 0};
}

espn::DocSource hbm_source(const espn_table *t)
{
    // (64-byte rows gain nothing from telling popular documents from the others: Zipf lists, 64 to 4096 queries per
    // batch, within 1.5 % either way, and 16 % slower in fused launches of 64-query batches)
    return espn::DocSource{t->emb, t->off_dev, nullptr, nullptr, t->n_docs, t->scale_dev,
                           t->popular_valid && t->dim != 32 ? t->popular_dev : nullptr};
}

// Whole-list sort of n <= kSortMax entries per query (one list, or two taken together).
constexpr int kSortMax = 4096;
template <typename Lists>
void launch_sort(const Lists &lists, int B, int n, int k, int ldo, int64_t *out_ids, float *out_scores, hipStream_t st)
{
    using namespace espn;
    if (n <= 256)
        hipLaunchKernelGGL((topk_sort_kernel<256, 64, Lists>), dim3(B), dim3(64), 0, st, lists, k, ldo, out_ids,
                           out_scores);
    else if (n <= 1024)
        hipLaunchKernelGGL((topk_sort_kernel<1024, 256, Lists>), dim3(B), dim3(256), 0, st, lists, k, ldo, out_ids,
                           out_scores);
    else if (n <= 2048)
        hipLaunchKernelGGL((topk_sort_kernel<2048, 512, Lists>), dim3(B), dim3(512), 0, st, lists, k, ldo, out_ids,
                           out_scores);
    else
        hipLaunchKernelGGL((topk_sort_kernel<4096, 512, Lists>), dim3(B), dim3(512), 0, st, lists, k, ldo, out_ids,
                           out_scores);
}

// Which stand-alone kernel ranks lists of K entries for k ranks.
// Few ranks: one wave per query keeps the list in registers and ranks the handful of entries
// that can reach the top k (5 us for 64 lists of 1000, k = 10; its cost grows with k and it
// falls back to k selection rounds once more than 64 entries survive its threshold).
// More ranks: the whole list is sorted, at a cost independent of k (11 us for the same lists).
// Lists beyond 4096 entries: k selection rounds over the list.
enum class RankKernel { Wave4, Wave16, Wave32, Sort256, Sort1024, Sort2048, Sort4096, Rounds };
RankKernel rank_kernel(int K, int k)
{
    if (k <= 32 && K <= 64 * 4) return RankKernel::Wave4;
    if (k <= 32 && K <= 64 * 16) return RankKernel::Wave16;
    if (k <= 32 && K <= 64 * 32) return RankKernel::Wave32;
    if (K <= 256) return RankKernel::Sort256;
    if (K <= 1024) return RankKernel::Sort1024;
    if (K <= 2048) return RankKernel::Sort2048;
    if (K <= kSortMax) return RankKernel::Sort4096;
    return RankKernel::Rounds;
}
const char *rank_kernel_name(RankKernel r)
{
    switch (r) {
        case RankKernel::Wave4: return "espn::topk_wave_kernel<4>";
        case RankKernel::Wave16: return "espn::topk_wave_kernel<16>";
        case RankKernel::Wave32: return "espn::topk_wave_kernel<32>";
        case RankKernel::Sort256: return "espn::topk_sort_kernel<256, 64, espn::OneList>";
        case RankKernel::Sort1024: return "espn::topk_sort_kernel<1024, 256, espn::OneList>";
        case RankKernel::Sort2048: return "espn::topk_sort_kernel<2048, 512, espn::OneList>";
        case RankKernel::Sort4096: return "espn::topk_sort_kernel<4096, 512, espn::OneList>";
        default: return "espn::topk_rounds_kernel<16>";
    }
}

// Ranks the first k of K scored candidates per query; cand rows have leading dimension ldc, output rows ldo.
int enqueue_topk(const float *scores, const int64_t *cand, int ldc, int B, int K, int k, int ldo, int64_t *out_ids,
                 float *out_scores, hipStream_t st)
{
    using namespace espn;
    if (B == 0 || k == 0) return ESPN_OK;
    switch (rank_kernel(K, k)) {
        case RankKernel::Wave4:
            hipLaunchKernelGGL((topk_wave_kernel<4>), dim3(B), dim3(64), 0, st, scores, cand, ldc, K, k, ldo, out_ids,
                               out_scores);
            break;
        case RankKernel::Wave16:
            hipLaunchKernelGGL((topk_wave_kernel<16>), dim3(B), dim3(64), 0, st, scores, cand, ldc, K, k, ldo, out_ids,
                               out_scores);
            break;
        case RankKernel::Wave32:
            hipLaunchKernelGGL((topk_wave_kernel<32>), dim3(B), dim3(64), 0, st, scores, cand, ldc, K, k, ldo, out_ids,
                               out_scores);
            break;
        case RankKernel::Rounds:
            hipLaunchKernelGGL((topk_rounds_kernel<16>), dim3(B), dim3(256), 0, st, scores, cand, ldc, K, k, ldo, out_ids,
                               out_scores);
            break;
        default:
            launch_sort(OneList{scores, cand, ldc, K}, B, K, k, ldo, out_ids, out_scores, st);
    }
    HIP_TRY(hipGetLastError());
    return ESPN_OK;
}

}  // namespace

ESPN_API int espn_score(espn_table *table, const void *q, const int64_t *cand, int32_t B, int32_t Q, int32_t K,
                        float *scores, void *stream)
{
    if (int rc = check_batch(table, q, cand, B, Q, K)) return rc;
    if (B > 0 && K > 0 && !scores) return fail(ESPN_ERR_ARG, "scores is NULL");
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    if (table->residency != ESPN_RESIDENT_HBM)
        return fail(ESPN_ERR_UNSUPPORTED, "table is host-resident: use espn_prefetch + espn_rerank_staged");
    const espn::Batch bt = plain_batch(q, cand, Q, K);
    return enqueue_score(table, hbm_source(table), bt, one_batch(bt, B, scores), plan_slices(table, B, K, 0),
                         espn::RankOut{}, static_cast<hipStream_t>(stream));
}

ESPN_API int espn_topk(const float *scores, const int64_t *cand, int32_t B, int32_t K, int32_t k, int64_t *out_ids,
                       float *out_scores, void *stream)
{
    if (B < 0 || K < 0 || k < 0) return fail(ESPN_ERR_ARG, "B = %d, K = %d, k = %d: negative size", B, K, k);
    if (k > K) return fail(ESPN_ERR_SHAPE, "k = %d exceeds K = %d", k, K);
    if (B > 0 && k > 0 && (!scores || !cand || !out_ids || !out_scores)) return fail(ESPN_ERR_ARG, "NULL pointer");
    return enqueue_topk(scores, cand, K, B, K, k, k, out_ids, out_scores, static_cast<hipStream_t>(stream));
}

namespace {
// the two parts of a batch's workspace: its scores [B, K], then its lists in id order [B, K] (8 bytes per entry)
size_t score_bytes(int32_t B, int32_t K)
{
    if (B <= 0 || K <= 0) return kAlign;
    const size_t bytes = sizeof(float) * (size_t)B * (size_t)K;
    return (bytes + kAlign - 1) / kAlign * kAlign;
}
size_t order_bytes(int32_t B, int32_t K)
{
    if (B <= 0 || K <= 0) return 0;
    const size_t bytes = sizeof(int64_t) * (size_t)B * (size_t)K;
    return (bytes + kAlign - 1) / kAlign * kAlign;
}
}  // namespace

ESPN_API size_t espn_workspace_bytes(int32_t B, int32_t K) { return score_bytes(B, K) + order_bytes(B, K); }

namespace {
int check_rerank_outputs(int32_t B, int32_t K, int32_t k, const int64_t *out_ids, const float *out_scores,
                         const void *workspace, size_t workspace_bytes, bool scores_only = false)
{
    const size_t needed = scores_only ? score_bytes(B, K) : espn_workspace_bytes(B, K);
    if (k < 0) return fail(ESPN_ERR_ARG, "k = %d is negative", k);
    if (k > K) return fail(ESPN_ERR_SHAPE, "k = %d exceeds K = %d", k, K);
    if (B > 0 && k > 0 && (!out_ids || !out_scores)) return fail(ESPN_ERR_ARG, "output pointer is NULL");
    if (B > 0 && K > 0) {
        if (!workspace) return fail(ESPN_ERR_ARG, "workspace is NULL");
        if ((reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0)
            return fail(ESPN_ERR_ARG, "workspace is not %zu-byte aligned", kAlign);
        if (workspace_bytes < needed)
            return fail(ESPN_ERR_SHAPE, "workspace holds %zu bytes, %zu needed", workspace_bytes, needed);
    }
    return ESPN_OK;
}
}  // namespace

namespace {

// Whether a batch of whole lists, planned as `plan`, is scored in id order (an ordering launch first): the table
// is in HBM with rows of 128 bytes or more, a sample has shown lists that overlap (and named the popular documents),
// and the scoring launch is long - many workgroups per compute unit, taken slice by slice.
bool scored_in_id_order(const espn_table *t, const SlicePlan &plan, int B, int Q, int K)
{
    return t->popular_valid && t->dim != 32 && t->residency == ESPN_RESIDENT_HBM && on_matrix_cores(t, Q) && !plan.linear && !plan.rank &&
           plan.slices > 1 && K <= kSortMax && (int64_t)B * plan.slices >= (int64_t)kOrderFrom * t->n_cu &&
           t->n_docs < ((int64_t)1 << (63 - espn::SLOT_BITS));
}

int enqueue_order(const espn::OrderSet &set, int K, int64_t n_docs, hipStream_t st)
{
    using namespace espn;
    const dim3 grid((unsigned)set.n * (unsigned)set.B);
    if (K <= 256) hipLaunchKernelGGL((order_lists_kernel<256, 64>), grid, dim3(64), 0, st, set, K, K, n_docs);
    else if (K <= 1024) hipLaunchKernelGGL((order_lists_kernel<1024, 256>), grid, dim3(256), 0, st, set, K, K, n_docs);
    else if (K <= 2048) hipLaunchKernelGGL((order_lists_kernel<2048, 512>), grid, dim3(512), 0, st, set, K, K, n_docs);
    else hipLaunchKernelGGL((order_lists_kernel<4096, 512>), grid, dim3(512), 0, st, set, K, K, n_docs);
    HIP_TRY(hipGetLastError());
    return ESPN_OK;
}
const char *order_kernel_name(int K)
{
    return K <= 256 ? "espn::order_lists_kernel<256, 64>" : K <= 1024 ? "espn::order_lists_kernel<1024, 256>" :
           K <= 2048 ? "espn::order_lists_kernel<2048, 512>" : "espn::order_lists_kernel<4096, 512>";
}

// Score bt.K candidates per query into the workspace and write the first k of their ranking to
// rows of leading dimension ldo: in one launch where the scoring kernel can rank, else in two.
// `ordered`: room for the batch's lists in id order ([B, K] entries of 8 bytes), or nullptr: scored as they come.
int enqueue_rerank(espn_table *t, const espn::DocSource &src, const espn::Batch &bt, int B, int k, int ldo,
                   int64_t *out_ids, float *out_scores, void *workspace, int64_t *ordered, hipStream_t st)
{
    if (B == 0 || bt.K == 0) return ESPN_OK;
    float *scores = static_cast<float *>(workspace);
    SlicePlan plan = plan_slices(t, B, bt.K, k);
    if (!on_matrix_cores(t, bt.Q)) plan.rank = false;
    if (src.row_map) plan.linear = false;    // a staging slot holds each document once for all the queries that list it
    const espn::RankOut ro{k, ldo};
    espn::Batch scored = bt;
    if (ordered && !src.row_map && !bt.prior && bt.ldc == bt.K && scored_in_id_order(t, plan, B, bt.Q, bt.K)) {
        espn::OrderSet lists{};
        lists.n = 1;
        lists.B = B;
        lists.cand[0] = bt.cand;
        lists.ordered[0] = ordered;
        if (int rc = enqueue_order(lists, bt.K, t->n_docs, st)) return rc;
        scored.cand = ordered;
        scored.order = espn::ORDER_BY_ID;
    }
    if (int rc = enqueue_score(t, src, scored, one_batch(scored, B, scores, out_ids, out_scores), plan, ro, st)) return rc;
    if (plan.rank) return ESPN_OK;
    return enqueue_topk(scores, bt.cand, bt.ldc, B, bt.K, k, ldo, out_ids, out_scores, st);
}

}  // namespace

ESPN_API int espn_rerank_plan(const espn_table *table, int32_t B, int32_t Q, int32_t K, int32_t k, int32_t *slices,
                              int32_t *slice, int32_t *launches)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (B < 0 || K < 0 || k < 0 || Q < 1) return fail(ESPN_ERR_ARG, "B = %d, Q = %d, K = %d, k = %d", B, Q, K, k);
    if (k > K) return fail(ESPN_ERR_SHAPE, "k = %d exceeds K = %d", k, K);
    SlicePlan plan;
    int n = 0;
    if (B > 0 && K > 0) {
        if (on_matrix_cores(table, Q)) {
            plan = plan_slices(table, B, K, k);
        } else {
            plan.slices = K;                 // the generic kernel: one wave per candidate, never ranks
            plan.slice = 1;
        }
        n = 1 + ((k > 0 && !plan.rank) ? 1 : 0) + (scored_in_id_order(table, plan, B, Q, K) ? 1 : 0);
    }
    if (slices) *slices = plan.slices;
    if (slice) *slice = plan.slice;
    if (launches) *launches = n;
    return ESPN_OK;
}

namespace {
// Profiler names of the kernels one launch pair of the path runs for `queries` queries in one launch (a batch, or a
// fused chunk of a queue: `fused` then names the ranking kernel that takes a set of batches).  text: 256 bytes.
void kernel_names(const espn_table *table, int queries, int Q, int K, int k, bool fused, char *text, size_t len)
{
    bool ranked = false;
    if (on_matrix_cores(table, Q)) {
        const SlicePlan plan = plan_slices(table, queries, K, k);
        const int QG = Q > 32 ? 4 : 2;
        ranked = plan.rank;
        snprintf(text, len, "espn::maxsim_slice_kernel<%d, %d, %d, %d, %s, %d, %s>", table->dim,
                 launched_waves(table->dim, table->elem_bytes, QG, plan), kPipeline, table->elem_bytes,
                 plan.rank ? "true" : "false", QG, plan.linear ? "true" : "false");
    } else {
        snprintf(text, len, "espn::maxsim_generic_kernel");
    }
    if (on_matrix_cores(table, Q) && scored_in_id_order(table, plan_slices(table, queries, K, k), queries, Q, K)) {
        const size_t at = std::strlen(text);
        snprintf(text + at, len - at, ";%s", order_kernel_name(K));
    }
    if (k > 0 && !ranked) {
        const size_t at = std::strlen(text);
        const RankKernel r = rank_kernel(K, k);
        if (fused) snprintf(text + at, len - at, ";espn::topk_wave_set_kernel<%d>", r == RankKernel::Wave4 ? 4 : r == RankKernel::Wave16 ? 16 : 32);
        else snprintf(text + at, len - at, ";%s", rank_kernel_name(r));
    }
}

int copy_out(const char *text, char *buf, size_t buf_len)
{
    if (std::strlen(text) + 1 > buf_len) return fail(ESPN_ERR_SHAPE, "buf holds %zu bytes, %zu needed", buf_len, std::strlen(text) + 1);
    std::memcpy(buf, text, std::strlen(text) + 1);
    return ESPN_OK;
}
}  // namespace

ESPN_API int espn_rerank_plan_kernels(const espn_table *table, int32_t B, int32_t Q, int32_t K, int32_t k, char *buf,
                                      size_t buf_len)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (!buf || buf_len == 0) return fail(ESPN_ERR_ARG, "buf is NULL or empty");
    if (B < 0 || K < 0 || k < 0 || Q < 1) return fail(ESPN_ERR_ARG, "B = %d, Q = %d, K = %d, k = %d", B, Q, K, k);
    if (k > K) return fail(ESPN_ERR_SHAPE, "k = %d exceeds K = %d", k, K);
    buf[0] = 0;
    if (B == 0 || K == 0) return ESPN_OK;
    char text[256];
    kernel_names(table, B, Q, K, k, false, text, sizeof(text));
    return copy_out(text, buf, buf_len);
}

ESPN_API int espn_rerank(espn_table *table, const void *q, const int64_t *cand, int32_t B, int32_t Q, int32_t K,
                         int32_t k, int64_t *out_ids, float *out_scores, void *workspace, size_t workspace_bytes,
                         void *stream)
{
    if (int rc = check_batch(table, q, cand, B, Q, K)) return rc;
    if (int rc = check_rerank_outputs(B, K, k, out_ids, out_scores, workspace, workspace_bytes)) return rc;
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    if (table->residency != ESPN_RESIDENT_HBM)
        return fail(ESPN_ERR_UNSUPPORTED, "table is host-resident: use espn_prefetch + espn_rerank_staged");
    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t *ordered = reinterpret_cast<int64_t *>(static_cast<uint8_t *>(workspace) + score_bytes(B, K));
    return enqueue_rerank(table, hbm_source(table), plain_batch(q, cand, Q, K), B, k, k, out_ids, out_scores, workspace,
                          ordered, st);
}

namespace {
// How espn_rerank_batches runs a queue of n batches of B queries.  Batches whose scoring launch would be short (few
// workgroups: 64 queries x 8 slices = 512, a 30 us launch of which the launch gap and the dependent look-ups
// at its start are a sixth) are scored `fuse` at a time by ONE launch and ranked by one more, which streams
// like one batch of fuse * B queries; the chunks of `fuse` batches are dealt to the lanes in turn, so that one
// chunk's ranking and the start of the next chunk's scoring overlap with the streaming of the chunk before.
// Batches that fill the device many times over on their own (fuse = 1) are dealt to the lanes one by one.
constexpr int64_t kFusedWorkgroups = 8192;      // aim of a fused launch: 16 batches of 512 workgroups
struct QueuePlan {
    int fuse = 1;           // batches per launch at most
    int chunks = 0;         // launches of the scoring kernel
    int lanes = 0;          // streams used (1: the caller's own)
};
QueuePlan plan_queue(const espn_table *t, int n_batches, int B, int Q, int K, int k)
{
    QueuePlan qp;
    if (n_batches <= 0) return qp;
    if (B > 0 && K > 0 && on_matrix_cores(t, Q)) {
        const SlicePlan one = plan_slices(t, B, K, k);
        const bool rank_fuses = k == 0 || one.rank || rank_kernel(K, k) <= RankKernel::Wave32;
        const int64_t per_batch = (int64_t)B * one.slices;
        if (rank_fuses && (int64_t)B * espn::MAX_FUSED * std::max(K, 1) <= (int64_t)0x7fffffff)
            qp.fuse = (int)std::max<int64_t>(1, std::min<int64_t>(espn::MAX_FUSED, kFusedWorkgroups / per_batch));
    }
    qp.chunks = (n_batches + qp.fuse - 1) / qp.fuse;
    qp.lanes = std::min(qp.chunks, (int)ESPN_BATCH_LANES);
    return qp;
}
}  // namespace

ESPN_API size_t espn_batches_workspace_bytes(const espn_table *table, int32_t n_batches, int32_t B, int32_t Q,
                                             int32_t K, int32_t k)
{
    if (!table || n_batches <= 0 || Q < 1) return espn_workspace_bytes(B, K);
    const QueuePlan qp = plan_queue(table, n_batches, B, Q, K, std::max(k, 0));
    return (size_t)qp.lanes * (size_t)std::min(qp.fuse, n_batches) * espn_workspace_bytes(B, K);
}

ESPN_API int espn_batches_plan(const espn_table *table, int32_t n_batches, int32_t B, int32_t Q, int32_t K, int32_t k,
                               int32_t *fuse, int32_t *launches, int32_t *streams, char *kernels, size_t kernels_len)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (n_batches < 0 || B < 0 || K < 0 || k < 0 || Q < 1)
        return fail(ESPN_ERR_ARG, "n_batches = %d, B = %d, Q = %d, K = %d, k = %d", n_batches, B, Q, K, k);
    if (k > K) return fail(ESPN_ERR_SHAPE, "k = %d exceeds K = %d", k, K);
    const bool nothing = n_batches == 0 || B == 0 || K == 0;
    const QueuePlan qp = nothing ? QueuePlan{} : plan_queue(table, n_batches, B, Q, K, k);
    const int per_launch = nothing ? 0 : (n_batches + qp.chunks - 1) / qp.chunks;       // the larger of the two chunk sizes
    if (fuse) *fuse = per_launch;
    if (launches) *launches = qp.chunks;
    if (streams) *streams = qp.lanes;
    if (kernels && kernels_len > 0) {
        kernels[0] = 0;
        if (!nothing) {
            char text[256];
            kernel_names(table, per_launch * B, Q, K, k, per_launch > 1, text, sizeof(text));
            return copy_out(text, kernels, kernels_len);
        }
    }
    return ESPN_OK;
}

ESPN_API int espn_rerank_batches(espn_table *table, int32_t n_batches, const void *const *q, const int64_t *const *cand,
                                 int32_t B, int32_t Q, int32_t K, int32_t k, int64_t *const *out_ids,
                                 float *const *out_scores, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (n_batches < 0) return fail(ESPN_ERR_ARG, "n_batches = %d is negative", n_batches);
    if (n_batches == 0) return ESPN_OK;
    if (!q || !cand) return fail(ESPN_ERR_ARG, "q or cand (the pointer lists) is NULL");
    const bool ranked = k > 0 && B > 0;
    if (ranked && (!out_ids || !out_scores)) return fail(ESPN_ERR_ARG, "out_ids or out_scores (the pointer lists) is NULL");
    if (Q < 1) return fail(ESPN_ERR_ARG, "Q = %d: a query needs at least one row", Q);
    const size_t per_batch = espn_workspace_bytes(B, K);
    const size_t needed = espn_batches_workspace_bytes(table, n_batches, B, Q, K, k);
    if (B > 0 && K > 0 && workspace_bytes < needed)
        return fail(ESPN_ERR_SHAPE, "workspace holds %zu bytes, %zu needed (espn_batches_workspace_bytes)", workspace_bytes, needed);
    // everything is checked before anything is enqueued
    for (int i = 0; i < n_batches; ++i) {
        if (int rc = check_batch(table, q[i], cand[i], B, Q, K)) return rc;
        if (int rc = check_rerank_outputs(B, K, k, ranked ? out_ids[i] : nullptr, ranked ? out_scores[i] : nullptr, workspace, per_batch))
            return rc;
    }
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    if (table->residency != ESPN_RESIDENT_HBM)
        return fail(ESPN_ERR_UNSUPPORTED, "table is host-resident: use espn_prefetch + espn_rerank_staged");
    if (B == 0 || K == 0) return ESPN_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const espn::DocSource src = hbm_source(table);
    const QueuePlan qp = plan_queue(table, n_batches, B, Q, K, k);
    const size_t per_lane = (size_t)std::min(qp.fuse, n_batches) * per_batch;

    // chunk c: batches [first, first + count), scored by one launch into the lane's part of the workspace, then ranked
    auto run_chunk = [&](int first, int count, uint8_t *ws, hipStream_t on) -> int {
        if (count == 1)
            return enqueue_rerank(table, src, plain_batch(q[first], cand[first], Q, K), B, k, k, ranked ? out_ids[first] : nullptr,
                                  ranked ? out_scores[first] : nullptr, ws, reinterpret_cast<int64_t *>(ws + score_bytes(B, K)), on);
        espn::Batch shape = plain_batch(nullptr, nullptr, Q, K);
        espn::BatchSet set{};
        espn::TopkSet lists{};
        set.n = lists.n = count;
        set.B = lists.B = B;
        for (int x = 0; x < count; ++x) {
            set.q[x] = static_cast<const uint16_t *>(q[first + x]);
            set.cand[x] = lists.cand[x] = cand[first + x];
            set.scores[x] = reinterpret_cast<float *>(ws + (size_t)x * per_batch);
            lists.scores[x] = set.scores[x];
            set.out_ids[x] = lists.out_ids[x] = ranked ? out_ids[first + x] : nullptr;
            set.out_scores[x] = lists.out_scores[x] = ranked ? out_scores[first + x] : nullptr;
        }
        // the launch is planned as what it is: one batch of count * B queries
        const SlicePlan plan = plan_slices(table, count * B, K, k);
        if (scored_in_id_order(table, plan, count * B, Q, K)) {
            espn::OrderSet order{};
            order.n = count;
            order.B = B;
            for (int x = 0; x < count; ++x) {
                order.cand[x] = cand[first + x];
                order.ordered[x] = reinterpret_cast<int64_t *>(ws + (size_t)x * per_batch + score_bytes(B, K));
                set.cand[x] = order.ordered[x];
            }
            if (int rc = enqueue_order(order, K, table->n_docs, on)) return rc;
            shape.order = espn::ORDER_BY_ID;
        }
        if (int rc = enqueue_score(table, src, shape, set, plan, espn::RankOut{k, k}, on)) return rc;
        if (k == 0 || plan.rank) return ESPN_OK;
        const dim3 grid((unsigned)count * B);
        switch (rank_kernel(K, k)) {
            case RankKernel::Wave4: hipLaunchKernelGGL((espn::topk_wave_set_kernel<4>), grid, dim3(64), 0, on, lists, K, K, k, k); break;
            case RankKernel::Wave16: hipLaunchKernelGGL((espn::topk_wave_set_kernel<16>), grid, dim3(64), 0, on, lists, K, K, k, k); break;
            default: hipLaunchKernelGGL((espn::topk_wave_set_kernel<32>), grid, dim3(64), 0, on, lists, K, K, k, k); break;
        }
        HIP_TRY(hipGetLastError());
        return ESPN_OK;
    };
    // chunks of equal size (to within one batch)
    auto chunk_first = [&](int c) { return (int)((int64_t)n_batches * c / qp.chunks); };

    if (qp.lanes == 1)      // one launch (or one batch): the caller's stream itself
        return run_chunk(0, n_batches, static_cast<uint8_t *>(workspace), st);
    // The lanes are streams of the library's own, created together, so that each has a hardware queue to itself
    // (a process has few of those, and the caller's stream may share one with a lane: taking it as one of the lanes
    // was measured at 32 us per batch instead of 27).  They start where the caller's stream is now - nothing to
    // wait for if it is idle, which one query tells (an event record and a wait per lane cost about 5 us each on the
    // host, at the start of the call, with the device idle) - and the caller's stream goes on when they are through
    // (those records and waits are enqueued behind the call's own work).
    // (a stream that is being captured into a graph may not be queried: there the dependency is always recorded,
    // which is also what pulls the library's streams into the capture; the join below brings them back)
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &capturing) != hipSuccess) {
        (void)hipGetLastError();
        capturing = hipStreamCaptureStatusNone;
    }
    const bool idle = capturing == hipStreamCaptureStatusNone && hipStreamQuery(st) == hipSuccess;
    if (!idle) {
        (void)hipGetLastError();                     // hipErrorNotReady is the expected answer, not an error
        HIP_TRY(hipEventRecord(table->fork, st));
        for (int l = 0; l < qp.lanes; ++l) HIP_TRY(hipStreamWaitEvent(table->lane[l], table->fork, 0));
    }
    int status = ESPN_OK;
    for (int c = 0; c < qp.chunks && status == ESPN_OK; ++c) {
        const int l = c % qp.lanes;
        status = run_chunk(chunk_first(c), chunk_first(c + 1) - chunk_first(c),
                           static_cast<uint8_t *>(workspace) + (size_t)l * per_lane, table->lane[l]);
    }
    // joined even after a failure, so that the caller's stream never runs ahead of work already enqueued
    for (int l = 0; l < qp.lanes; ++l) {
        const hipError_t e1 = hipEventRecord(table->joined[l], table->lane[l]);
        const hipError_t e2 = e1 == hipSuccess ? hipStreamWaitEvent(st, table->joined[l], 0) : e1;
        if (e2 != hipSuccess && status == ESPN_OK)
            status = fail(ESPN_ERR_HIP, "joining lane %d failed: %s", l, hipGetErrorString(e2));
    }
    return status;
}

ESPN_API int espn_rerank_noalloc(espn_table *table, const void *q, const int64_t *cand, int32_t B, int32_t Q,
                                 int32_t K, int32_t k, int64_t *out_ids, float *out_scores, void *stream)
{
    if (int rc = check_batch(table, q, cand, B, Q, K)) return rc;
    if ((int64_t)B * K > (int64_t)ESPN_NOALLOC_MAX_PAIRS)
        return fail(ESPN_ERR_SHAPE, "B * K = %lld pairs exceed the %lld the static scratch holds", (long long)B * K,
                    (long long)ESPN_NOALLOC_MAX_PAIRS);
    void *ws = table->static_scratch;
    if (int rc = check_rerank_outputs(B, K, k, out_ids, out_scores, ws, sizeof(float) * (size_t)ESPN_NOALLOC_MAX_PAIRS, true))
        return rc;
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    if (table->residency != ESPN_RESIDENT_HBM)
        return fail(ESPN_ERR_UNSUPPORTED, "table is host-resident: use espn_prefetch + espn_rerank_staged");
    return enqueue_rerank(table, hbm_source(table), plain_batch(q, cand, Q, K), B, k, k, out_ids, out_scores, ws, nullptr,
                          static_cast<hipStream_t>(stream));
}

ESPN_API int espn_rerank_partial(espn_table *table, const void *q, const int64_t *cand, int32_t B, int32_t Q,
                                 int32_t K, int32_t R, int32_t k, int64_t *out_ids, float *out_scores,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (int rc = check_batch(table, q, cand, B, Q, K)) return rc;
    if (R < 0 || R > K) return fail(ESPN_ERR_SHAPE, "R = %d outside [0, K = %d]", R, K);
    if (int rc = check_rerank_outputs(B, R, std::min(k, R), out_ids, out_scores, workspace, workspace_bytes))
        return rc;
    if (k < 0) return fail(ESPN_ERR_ARG, "k = %d is negative", k);
    if (k > K) return fail(ESPN_ERR_SHAPE, "k = %d exceeds K = %d", k, K);
    if (B > 0 && k > 0 && (!out_ids || !out_scores)) return fail(ESPN_ERR_ARG, "output pointer is NULL");
    if (table->residency != ESPN_RESIDENT_HBM)
        return fail(ESPN_ERR_UNSUPPORTED, "table is host-resident: use espn_prefetch + espn_rerank_staged");
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const espn::Batch bt{static_cast<const uint16_t *>(q), cand, nullptr, 0.f, K, Q, R, 0};
    if (int rc = enqueue_rerank(table, hbm_source(table), bt, B, std::min(k, R), k, out_ids, out_scores, workspace, nullptr, st))
        return rc;
    if (B > 0 && k > R) {
        hipLaunchKernelGGL(espn::append_unranked_kernel, dim3(B, (k - R + 255) / 256), dim3(256), 0, st, cand, K, R, k,
                           out_ids, out_scores);
        HIP_TRY(hipGetLastError());
    }
    return ESPN_OK;
}

ESPN_API int espn_rerank_prior(espn_table *table, const void *q, const int64_t *cand, const float *prior,
                               float alpha, int32_t B, int32_t Q, int32_t K, int32_t k, int64_t *out_ids,
                               float *out_scores, void *workspace, size_t workspace_bytes, void *stream)
{
    if (int rc = check_batch(table, q, cand, B, Q, K)) return rc;
    if (int rc = check_rerank_outputs(B, K, k, out_ids, out_scores, workspace, workspace_bytes)) return rc;
    if (B > 0 && K > 0 && !prior) return fail(ESPN_ERR_ARG, "prior is NULL");
    if (table->residency != ESPN_RESIDENT_HBM)
        return fail(ESPN_ERR_UNSUPPORTED, "table is host-resident: use espn_prefetch + espn_rerank_staged");
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const espn::Batch bt{static_cast<const uint16_t *>(q), cand, prior, alpha, K, Q, K, 0};
    return enqueue_rerank(table, hbm_source(table), bt, B, k, k, out_ids, out_scores, workspace, nullptr, st);
}

ESPN_API int espn_merge_topk(const int64_t *ids_a, const float *scores_a, int32_t ka, const int64_t *ids_b,
                             const float *scores_b, int32_t kb, int32_t B, int32_t k, int64_t *out_ids,
                             float *out_scores, void *stream)
{
    if (B < 0 || ka < 0 || kb < 0 || k < 0) return fail(ESPN_ERR_ARG, "negative size");
    if ((int64_t)k > (int64_t)ka + kb) return fail(ESPN_ERR_SHAPE, "k = %d exceeds ka + kb = %d", k, ka + kb);
    if (B == 0 || k == 0) return ESPN_OK;
    if ((ka > 0 && (!ids_a || !scores_a)) || (kb > 0 && (!ids_b || !scores_b)) || !out_ids || !out_scores)
        return fail(ESPN_ERR_ARG, "NULL pointer");
    // up to 4096 entries per query: sorted as one list (cost independent of k); beyond: k selection rounds
    if ((int64_t)ka + kb <= kSortMax)
        launch_sort(espn::TwoLists{ids_a, scores_a, ka, ids_b, scores_b, kb}, B, ka + kb, k, k, out_ids, out_scores,
                    static_cast<hipStream_t>(stream));
    else
        hipLaunchKernelGGL(espn::merge_topk_kernel, dim3(B), dim3(64), 0, static_cast<hipStream_t>(stream), ids_a,
                           scores_a, ka, ids_b, scores_b, kb, k, out_ids, out_scores);
    HIP_TRY(hipGetLastError());
    return ESPN_OK;
}

ESPN_API double espn_batch_threshold(double bandwidth_bytes_per_s, double budget_s, double bytes_per_query)
{
    if (!(bytes_per_query > 0.0)) return 0.0;
    return bandwidth_bytes_per_s * budget_s / bytes_per_query;
}

ESPN_API int espn_table_check(espn_table *table, void *stream)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned flags = 0;
    HIP_TRY(hipMemcpyAsync(&flags, table->err_dev, sizeof(flags), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (flags) {
        HIP_TRY(hipMemsetAsync(table->err_dev, 0, sizeof(unsigned), st));
        HIP_TRY(hipStreamSynchronize(st));
    }
    if (flags & espn::ERR_ID_RANGE) return fail(ESPN_ERR_ID_RANGE, "a candidate id was outside [0, %lld)",
                                                (long long)table->n_docs);
    if (flags & espn::ERR_STAGING_FULL)
        return fail(ESPN_ERR_NOMEM, "a prefetch needed more than the %lld rows / %lld documents a staging slot holds",
                    (long long)table->capacity_rows, (long long)table->capacity_docs);
    if (flags & espn::ERR_NOT_STAGED)
        return fail(ESPN_ERR_SHAPE, "a staged re-rank named a document its slot does not hold "
                                    "(candidates differ from the prefetched ones, or the slot overflowed)");
    return ESPN_OK;
}

ESPN_API int espn_staging_create(espn_table *table, int64_t capacity_rows, int64_t capacity_docs)
{
    return espn_staging_create_ring(table, 2, capacity_rows, capacity_docs);
}

ESPN_API int espn_staging_create_ring(espn_table *table, int32_t n_slots, int64_t capacity_rows, int64_t capacity_docs)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (n_slots < 2 || n_slots > espn::MAX_SLOTS)
        return fail(ESPN_ERR_ARG, "n_slots = %d outside [2, %d]", n_slots, espn::MAX_SLOTS);
    if (capacity_rows < 1 || capacity_docs < 1) return fail(ESPN_ERR_ARG, "capacities must be positive");
    if (capacity_rows >= (int64_t)1 << espn::OTHER_SHIFT)
        return fail(ESPN_ERR_UNSUPPORTED, "capacity_rows = %lld is beyond 2^%d", (long long)capacity_rows, espn::OTHER_SHIFT);
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    (void)hipDeviceSynchronize();
    free_staging(table);
    const size_t n_words = (size_t)(table->n_docs + 31) / 32 + 1;
    hipError_t e = hipSuccess;
    for (int i = 0; i < n_slots; ++i) {
        StagingSlot &s = table->slot[i];
        if (e == hipSuccess) e = hipMalloc(&s.rows, (size_t)capacity_rows * table->dim * table->elem_bytes);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s.row_map), sizeof(int64_t) * (size_t)(table->n_docs + 1));
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s.bits), sizeof(unsigned) * n_words);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s.uniq), sizeof(int64_t) * (size_t)capacity_docs);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s.other_row), sizeof(int64_t) * (size_t)capacity_docs);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s.handed), sizeof(int64_t) * (size_t)capacity_docs);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s.counters), kAlign);
        if (e == hipSuccess) e = hipMemset(s.bits, 0, sizeof(unsigned) * n_words);
        if (e == hipSuccess) e = hipMemset(s.counters, 0, kAlign);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&s.ready, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&s.consumed, hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        free_staging(table);
        (void)hipGetLastError();
        return fail(e == hipErrorOutOfMemory ? ESPN_ERR_NOMEM : ESPN_ERR_HIP, "staging set-up failed: %s",
                    hipGetErrorString(e));
    }
    table->capacity_rows = capacity_rows;
    table->capacity_docs = capacity_docs;
    table->n_slots = n_slots;
    table->prefetches = 0;
    table->has_staging = true;
    return ESPN_OK;
}

namespace {
int check_slot(const espn_table *table, int32_t slot)
{
    if (!table) return fail(ESPN_ERR_ARG, "table is NULL");
    if (!table->has_staging) return fail(ESPN_ERR_ARG, "espn_staging_create has not been called for this table");
    if (slot < 0 || slot >= table->n_slots)
        return fail(ESPN_ERR_ARG, "slot = %d outside [0, %d)", slot, table->n_slots);
    return ESPN_OK;
}
}  // namespace

ESPN_API int espn_prefetch(espn_table *table, const int64_t *cand, int32_t B, int32_t K, int32_t slot,
                           void *side_stream)
{
    if (int rc = check_slot(table, slot)) return rc;
    if (B < 0 || K < 0) return fail(ESPN_ERR_ARG, "B = %d, K = %d: negative size", B, K);
    if (B > 0 && K > 0 && !cand) return fail(ESPN_ERR_ARG, "cand is NULL");
    if (table->residency == ESPN_RESIDENT_HOST)
        return fail(ESPN_ERR_UNSUPPORTED, "the table is in host memory the device cannot read (not pinned): use espn_prefetch_packed");
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    hipStream_t st = static_cast<hipStream_t>(side_stream);
    StagingSlot &s = table->slot[slot];
    // The slot may still be read by the re-rank that used it last.  The other slots, whose documents
    // this prefetch may take over, must have been filled, and none of them may be refilled before
    // this prefetch is through with it: every prefetch waits for the last prefetch into every other
    // slot, which puts all prefetches of a table in one order (a no-op if they share a stream).
    HIP_TRY(hipStreamWaitEvent(st, s.consumed, 0));
    espn::OtherSlots others{};
    {
        int order[espn::MAX_SLOTS];
        int n = 0;
        for (int i = 0; i < table->n_slots; ++i)
            if (i != slot) {
                HIP_TRY(hipStreamWaitEvent(st, table->slot[i].ready, 0));
                if (table->slot[i].filled_at) order[n++] = i;
            }
        std::sort(order, order + n, [&](int a, int b) { return table->slot[a].filled_at > table->slot[b].filled_at; });
        others.n = n;
        for (int x = 0; x < n; ++x) {
            const StagingSlot &o = table->slot[order[x]];
            others.bits[x] = o.bits;
            others.row_map[x] = o.row_map;
            others.rows[x] = static_cast<const uint4 *>(o.rows);
        }
    }
    s.filled_at = ++table->prefetches;
    const int64_t n_words = (table->n_docs + 31) / 32 + 1;
    const int64_t n_pairs = (int64_t)B * K;
    hipLaunchKernelGGL(espn::staging_clear_kernel, dim3((unsigned)std::min<int64_t>((n_words + 255) / 256, 1024)),
                       dim3(256), 0, st, s.bits, n_words, s.counters);
    if (n_pairs > 0) {
        hipLaunchKernelGGL(espn::staging_mark_kernel, dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, st, cand,
                           n_pairs, table->off_dev, table->n_docs, s.bits, s.row_map, s.uniq, s.other_row, others,
                           s.counters, table->capacity_rows, table->capacity_docs, table->err_dev);
        hipLaunchKernelGGL(espn::staging_gather_kernel, dim3(kGatherBlocks), dim3(256), 0, st,
                           static_cast<const uint4 *>(table->emb), others, table->off_dev, s.uniq, s.other_row,
                           s.row_map, s.counters, table->capacity_docs,
                           static_cast<uint4 *>(s.rows), table->dim * table->elem_bytes / 16);
    }
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(s.ready, st));
    return ESPN_OK;
}

namespace {
constexpr size_t kPackBytes = (size_t)64 << 20;     // one pinned pack buffer
constexpr int kPackThreads = 16;

int make_pack_state(espn_table *t)
{
    if (t->pack) return ESPN_OK;
    PackState *p = new (std::nothrow) PackState;
    if (!p) return fail(ESPN_ERR_NOMEM, "host allocation failed");
    t->pack = p;                        // freed with the staging slots whatever happens below
    hipError_t e = hipSuccess;
    for (int i = 0; i < 2 && e == hipSuccess; ++i) {
        e = hipHostMalloc(&p->buf[i], kPackBytes, hipHostMallocDefault);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&p->sent[i], hipEventDisableTiming);
    }
    const size_t list_bytes = sizeof(int64_t) * (size_t)t->capacity_docs;
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void **>(&p->uniq), list_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void **>(&p->row0), list_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void **>(&p->from), list_bytes, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p->lists_sent, hipEventDisableTiming);
    if (e != hipSuccess) {
        free_pack_state(t);
        (void)hipGetLastError();
        return fail(e == hipErrorOutOfMemory ? ESPN_ERR_NOMEM : ESPN_ERR_HIP, "pack buffers: %s", hipGetErrorString(e));
    }
    try {
        p->seen.assign(((size_t)t->n_docs + 63) / 64, 0);
        p->where.assign((size_t)t->n_docs, -1);
        p->where_gen.assign((size_t)t->n_docs, 0);
        p->scratch.resize(3 * (size_t)t->capacity_docs);
        p->pool.start(kPackThreads - 1);
    } catch (...) {                     // bad_alloc, or no more threads to be had
        free_pack_state(t);
        return fail(ESPN_ERR_NOMEM, "host allocation or thread creation failed");
    }
    return ESPN_OK;
}

// `bytes` from src to dst with stores that do not first read the destination's cache lines (the pack buffer is
// written once and then read by the copy engine, never by this core again).  dst 32-byte aligned, bytes a
// multiple of 32; anything else goes through memcpy.
__attribute__((target("avx2"))) void copy_streaming_avx2(uint8_t *dst, const uint8_t *src, size_t bytes)
{
    typedef long long v4di __attribute__((vector_size(32), aligned(32)));
    typedef long long v4di_u __attribute__((vector_size(32), aligned(1)));
    for (size_t x = 0; x < bytes; x += 32)
        __builtin_nontemporal_store(*reinterpret_cast<const v4di_u *>(src + x), reinterpret_cast<v4di *>(dst + x));
}

void copy_document(uint8_t *dst, const uint8_t *src, size_t bytes, bool avx2)
{
    if (avx2 && (reinterpret_cast<uintptr_t>(dst) & 31u) == 0 && bytes % 32 == 0) copy_streaming_avx2(dst, src, bytes);
    else std::memcpy(dst, src, bytes);
}

// Copies documents uniq[first .. last) of the table into `dst` back to back, on the pool's threads.  Nothing
// in here allocates or throws.
void pack_documents(const espn_table *t, PackPool &pool, const int64_t *uniq, int64_t first, int64_t last, uint8_t *dst)
{
    const size_t row_bytes = (size_t)t->dim * t->elem_bytes;
    const int64_t n = last - first;
    const int parts = (int)std::min<int64_t>(std::min(pool.parts(), kPackThreads), std::max<int64_t>(1, n / 64));
    // part x takes documents [cut[x], cut[x + 1]); where its bytes start in dst follows from the lengths
    int64_t cut[kPackThreads + 1];
    size_t at[kPackThreads + 1];
    at[0] = 0;
    for (int x = 0; x <= parts; ++x) cut[x] = first + n * x / parts;
    for (int x = 0; x < parts; ++x) {
        size_t rows = 0;
        for (int64_t u = cut[x]; u < cut[x + 1]; ++u) rows += (size_t)(t->off_host[uniq[u] + 1] - t->off_host[uniq[u]]);
        at[x + 1] = at[x] + rows * row_bytes;
    }
    static const bool avx2 = __builtin_cpu_supports("avx2");
    pool.run(parts, [&](int x) {
        uint8_t *out = dst + at[x];
        for (int64_t u = cut[x]; u < cut[x + 1]; ++u) {
            const int64_t id = uniq[u];
            const size_t bytes = (size_t)(t->off_host[id + 1] - t->off_host[id]) * row_bytes;
            if (u + 1 < cut[x + 1])          // the next document's first lines, while this one is copied
                __builtin_prefetch(t->emb_host + (size_t)t->off_host[uniq[u + 1]] * row_bytes);
            copy_document(out, t->emb_host + (size_t)t->off_host[id] * row_bytes, bytes, avx2);
            out += bytes;
        }
        __atomic_thread_fence(__ATOMIC_SEQ_CST);     // the streaming stores are out before the buffer is handed on
    });
}

// Everything espn_prefetch_packed enqueues once the batch has been found valid.  The slot's bitmap and row map
// are written LAST, after the row copies: if anything fails on the way the slot advertises no document.
// Documents [0, n_packed) of the lists are packed and sent, documents [n_packed, n_uniq) are copied from the other
// slots that hold them (`handed_rows` rows in all).
int enqueue_packed(espn_table *table, PackState &p, StagingSlot &s, int64_t n_packed, int64_t n_uniq, int64_t rows,
                   int64_t handed_rows, hipStream_t st)
{
    const int64_t *off = table->off_host;
    const size_t row_bytes = (size_t)table->dim * table->elem_bytes;
    if (n_uniq == 0) return ESPN_OK;
    HIP_TRY(hipMemcpyAsync(s.uniq, p.uniq, sizeof(int64_t) * (size_t)n_uniq, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(s.other_row, p.row0, sizeof(int64_t) * (size_t)n_uniq, hipMemcpyHostToDevice, st));
    if (n_uniq > n_packed)
        HIP_TRY(hipMemcpyAsync(s.handed + n_packed, p.from + n_packed, sizeof(int64_t) * (size_t)(n_uniq - n_packed),
                               hipMemcpyHostToDevice, st));
    HIP_TRY(hipEventRecord(p.lists_sent, st));
    p.lists_in_flight = true;
    if (n_uniq > n_packed) {
        // first, while the host packs: what the other slots hold moves inside HBM
        espn::SlotRows all{};
        for (int x = 0; x < table->n_slots; ++x) all.rows[x] = static_cast<const uint4 *>(table->slot[x].rows);
        const unsigned blocks = (unsigned)std::min<int64_t>((n_uniq - n_packed + 3) / 4, 4096);
        hipLaunchKernelGGL(espn::staging_handover_kernel, dim3(blocks), dim3(256), 0, st, all, table->off_dev, s.uniq,
                           s.other_row, s.handed, n_packed, n_uniq, static_cast<uint4 *>(s.rows), (int)(row_bytes / 16));
        HIP_TRY(hipGetLastError());
    }
    // rows: whole documents are packed into a pinned buffer while the previous buffer is on its way
    int64_t u = 0;
    int which = 0;
    while (u < n_packed) {
        int64_t last = u;
        size_t bytes = 0;
        while (last < n_packed) {
            const size_t len = (size_t)(off[p.uniq[last] + 1] - off[p.uniq[last]]) * row_bytes;
            if (bytes + len > kPackBytes) break;
            bytes += len;
            ++last;
        }
        if (p.in_flight[which]) HIP_TRY(hipEventSynchronize(p.sent[which]));      // the buffer is free again
        pack_documents(table, p.pool, p.uniq, u, last, static_cast<uint8_t *>(p.buf[which]));
        if (bytes > 0) {
            HIP_TRY(hipMemcpyAsync(static_cast<uint8_t *>(s.rows) + (size_t)p.row0[u] * row_bytes, p.buf[which], bytes,
                                   hipMemcpyHostToDevice, st));
            HIP_TRY(hipEventRecord(p.sent[which], st));
            p.in_flight[which] = true;
        }
        u = last;
        which ^= 1;
    }
    hipLaunchKernelGGL(espn::staging_publish_kernel, dim3((unsigned)((n_uniq + 255) / 256)), dim3(256), 0, st, s.uniq,
                       s.other_row, n_uniq, (unsigned long long)rows, (unsigned long long)handed_rows, s.bits, s.row_map,
                       s.counters);
    HIP_TRY(hipGetLastError());
    return ESPN_OK;
}
}  // namespace

ESPN_API int espn_prefetch_packed(espn_table *table, const int64_t *cand_host, int32_t B, int32_t K, int32_t slot,
                                  void *side_stream)
{
    if (int rc = check_slot(table, slot)) return rc;
    if (B < 0 || K < 0) return fail(ESPN_ERR_ARG, "B = %d, K = %d: negative size", B, K);
    if (B > 0 && K > 0 && !cand_host) return fail(ESPN_ERR_ARG, "cand_host is NULL");
    if (!table->emb_host && table->total_rows > 0)
        return fail(ESPN_ERR_UNSUPPORTED, "the packing engine reads the table on the host: the table is HBM-resident");
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    if (int rc = make_pack_state(table)) return rc;
    PackState &p = *table->pack;
    hipStream_t st = static_cast<hipStream_t>(side_stream);
    StagingSlot &s = table->slot[slot];
    const int64_t *off = table->off_host;
    const size_t row_bytes = (size_t)table->dim * table->elem_bytes;

    // the lists of the previous call may still be on their way to the device
    if (p.lists_in_flight) {
        HIP_TRY(hipEventSynchronize(p.lists_sent));
        p.lists_in_flight = false;
    }
    // The distinct documents of the batch and their lengths.  The threads take a share of the pairs each and claim
    // documents in the bitmap (1 M pairs, 325 000 distinct documents of an 8.8 M table: 11 ms on one thread, most of
    // it waiting for the documents' offsets); a thread's finds go to its own stretch of `found` (id, length), and
    // the stretches are then put together in thread order.  Which thread claims a document that several list is a
    // race with one winner: the order of the documents in the slot may differ from run to run, nothing else.
    const int64_t n_pairs = (int64_t)B * K;
    try {
        if (p.found.size() < 2 * (size_t)n_pairs) p.found.resize(2 * (size_t)n_pairs);
    } catch (...) {
        return fail(ESPN_ERR_NOMEM, "host allocation failed");
    }
    const int finders = (int)std::min<int64_t>(std::min(p.pool.parts(), kPackThreads), std::max<int64_t>(1, n_pairs / 8192));
    int64_t n_found[kPackThreads] = {}, first_bad[kPackThreads], first_large[kPackThreads];
    p.pool.run(finders, [&](int x) {
        const int64_t begin = n_pairs * x / finders, end = n_pairs * (x + 1) / finders;
        int64_t *mine = p.found.data() + 2 * begin, n = 0;
        first_bad[x] = first_large[x] = -1;
        for (int64_t i = begin; i < end; ++i) {
            const int64_t id = cand_host[i];
            if (id < 0 || id >= table->n_docs) {
                if (first_bad[x] < 0) first_bad[x] = i;
                continue;
            }
            const uint64_t bit = 1ull << (id & 63);
            if (__atomic_fetch_or(&p.seen[(size_t)id >> 6], bit, __ATOMIC_RELAXED) & bit) continue;
            const int64_t len = off[id + 1] - off[id];
            if ((size_t)len * row_bytes > kPackBytes && first_large[x] < 0) first_large[x] = i;
            mine[2 * n] = id;
            mine[2 * n + 1] = len;
            ++n;
        }
        n_found[x] = n;
    });
    int64_t n_uniq = 0, rows = 0;
    for (int x = 0; x < finders; ++x) n_uniq += n_found[x];
    // leave the bitmap clear, whatever comes next
    p.pool.run(finders, [&](int x) {
        const int64_t *mine = p.found.data() + 2 * (n_pairs * x / finders);
        for (int64_t u = 0; u < n_found[x]; ++u)
            __atomic_store_n(&p.seen[(size_t)mine[2 * u] >> 6], (uint64_t)0, __ATOMIC_RELAXED);
    });
    // errors, the first in list order: nothing has been enqueued
    for (int x = 0; x < finders; ++x)
        if (first_bad[x] >= 0)
            return fail(ESPN_ERR_ID_RANGE, "candidate %lld of the batch is %lld, outside [0, %lld)", (long long)first_bad[x],
                        (long long)cand_host[first_bad[x]], (long long)table->n_docs);
    for (int x = 0; x < finders; ++x)
        if (first_large[x] >= 0) {
            const int64_t id = cand_host[first_large[x]];
            return fail(ESPN_ERR_UNSUPPORTED, "document %lld holds %zu bytes, more than a pack buffer", (long long)id,
                        (size_t)(off[id + 1] - off[id]) * row_bytes);
        }
    if (n_uniq > table->capacity_docs)
        return fail(ESPN_ERR_NOMEM, "the batch needs more than the %lld rows / %lld documents a staging slot holds",
                    (long long)table->capacity_rows, (long long)table->capacity_docs);
    {
        int64_t at = 0;
        for (int x = 0; x < finders; ++x) {
            const int64_t *mine = p.found.data() + 2 * (n_pairs * x / finders);
            for (int64_t u = 0; u < n_found[x]; ++u, ++at) {
                p.uniq[at] = mine[2 * u];
                p.row0[at] = mine[2 * u + 1];           // for now: the document's length
                rows += mine[2 * u + 1];
            }
        }
    }
    if (rows > table->capacity_rows)
        return fail(ESPN_ERR_NOMEM, "the batch needs more than the %lld rows / %lld documents a staging slot holds",
                    (long long)table->capacity_rows, (long long)table->capacity_docs);

    // Which of them another slot still holds since an earlier packed prefetch (Zipf lists: a third of a batch's
    // distinct documents were in the batch before): those are copied inside HBM instead of being packed and sent.
    // The lists are put in the order (packed ..., handed over ...), so that what is packed fills the slot's first rows
    // back to back, and the slot row of every document follows from the lengths.
    // Same ordering as espn_prefetch: after the last re-rank that read the slot, and after the last prefetch into
    // every other slot (which may be reading this one).  (Enqueued before the host's books are touched: from here on
    // a failure gives the slot a new prefetch number, so that nothing is ever taken from it on the strength of them.)
    HIP_TRY(hipStreamWaitEvent(st, s.consumed, 0));
    for (int i = 0; i < table->n_slots; ++i)
        if (i != slot) HIP_TRY(hipStreamWaitEvent(st, table->slot[i].ready, 0));
    const uint64_t gen = s.filled_at = ++table->prefetches;
    uint64_t slot_gen[espn::MAX_SLOTS] = {};
    for (int x = 0; x < table->n_slots; ++x) slot_gen[x] = x == slot ? 0 : table->slot[x].filled_at;
    const int parts = (int)std::min<int64_t>(std::min(p.pool.parts(), kPackThreads), std::max<int64_t>(1, n_uniq / 4096));
    p.pool.run(parts, [&](int x) {
        for (int64_t u = n_uniq * x / parts; u < n_uniq * (x + 1) / parts; ++u) {
            const int64_t id = p.uniq[u], w = p.where[(size_t)id];
            int64_t from = -1;
            if (w >= 0) {
                const uint64_t then = slot_gen[w >> espn::OTHER_SHIFT];
                if (then != 0 && (uint32_t)then == p.where_gen[(size_t)id]) from = w;
            }
            p.from[u] = from;
        }
    });
    int64_t n_packed = 0, handed_rows = 0;
    {
        int64_t *ids = p.scratch.data(), *lens = ids + table->capacity_docs, *froms = lens + table->capacity_docs;
        int64_t n_handed = 0;
        for (int64_t u = 0; u < n_uniq; ++u) {
            if (p.from[u] < 0) {
                p.uniq[n_packed] = p.uniq[u];
                p.row0[n_packed] = p.row0[u];
                ++n_packed;
            } else {
                ids[n_handed] = p.uniq[u];
                lens[n_handed] = p.row0[u];
                froms[n_handed] = p.from[u];
                handed_rows += p.row0[u];
                ++n_handed;
            }
        }
        for (int64_t h = 0; h < n_handed; ++h) {
            p.uniq[n_packed + h] = ids[h];
            p.row0[n_packed + h] = lens[h];
            p.from[n_packed + h] = froms[h];
        }
        int64_t at = 0;
        for (int64_t u = 0; u < n_uniq; ++u) {
            const int64_t len = p.row0[u];
            p.row0[u] = at;
            at += len;
        }
    }
    // ... and this slot is where they all are from now on
    p.pool.run(parts, [&](int x) {
        for (int64_t u = n_uniq * x / parts; u < n_uniq * (x + 1) / parts; ++u) {
            p.where[(size_t)p.uniq[u]] = ((int64_t)slot << espn::OTHER_SHIFT) | p.row0[u];
            p.where_gen[(size_t)p.uniq[u]] = (uint32_t)gen;
        }
    });

    const int64_t n_words = (table->n_docs + 31) / 32 + 1;
    const dim3 clear_grid((unsigned)std::min<int64_t>((n_words + 255) / 256, 1024));
    hipLaunchKernelGGL(espn::staging_clear_kernel, clear_grid, dim3(256), 0, st, s.bits, n_words, s.counters);
    const hipError_t cleared = hipGetLastError();
    int status = cleared == hipSuccess ? enqueue_packed(table, p, s, n_packed, n_uniq, rows, handed_rows, st)
                                       : fail(ESPN_ERR_HIP, "launching the clear kernel failed: %s", hipGetErrorString(cleared));
    // (the clear kernel has run by then and the publish kernel has not been enqueued: the slot holds nothing,
    // and a staged re-rank of this batch reports ESPN_ERR_SHAPE through espn_table_check; a new prefetch number
    // keeps later prefetches from taking documents out of it)
    if (status != ESPN_OK) s.filled_at = ++table->prefetches;
    const hipError_t e = hipEventRecord(s.ready, st);
    if (status == ESPN_OK && e != hipSuccess) status = fail(ESPN_ERR_HIP, "hipEventRecord failed: %s", hipGetErrorString(e));
    return status;
}

ESPN_API int espn_rerank_staged(espn_table *table, int32_t slot, const void *q, const int64_t *cand, int32_t B,
                                int32_t Q, int32_t K, int32_t k, int64_t *out_ids, float *out_scores,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    if (int rc = check_slot(table, slot)) return rc;
    if (int rc = check_batch(table, q, cand, B, Q, K)) return rc;
    if (int rc = check_rerank_outputs(B, K, k, out_ids, out_scores, workspace, workspace_bytes)) return rc;
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    StagingSlot &s = table->slot[slot];
    HIP_TRY(hipStreamWaitEvent(st, s.ready, 0));
    const espn::DocSource src{s.rows, table->off_dev, s.row_map, s.bits, table->n_docs, table->scale_dev, nullptr};
    if (int rc = enqueue_rerank(table, src, plain_batch(q, cand, Q, K), B, k, k, out_ids, out_scores, workspace, nullptr, st))
        return rc;
    HIP_TRY(hipEventRecord(s.consumed, st));
    return ESPN_OK;
}

ESPN_API int espn_staging_counters(espn_table *table, int32_t slot, void *stream, uint64_t *out4)
{
    if (int rc = check_slot(table, slot)) return rc;
    if (!out4) return fail(ESPN_ERR_ARG, "out4 is NULL");
    DeviceScope scope(table->device);
    if (!scope.ok) return fail(ESPN_ERR_HIP, "cannot select device %d", table->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned long long c[4] = {0, 0, 0, 0};
    HIP_TRY(hipMemcpyAsync(c, table->slot[slot].counters, sizeof(c), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    out4[0] = c[0];
    out4[1] = c[1];
    out4[2] = (c[1] - c[2]) * (uint64_t)table->dim * (uint64_t)table->elem_bytes;
    out4[3] = (uint64_t)table->capacity_rows;
    return ESPN_OK;
}
