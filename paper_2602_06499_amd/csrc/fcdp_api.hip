// C ABI of libfcdp: argument checks, stream/event ordering, the host cache,
// the dirty-state flags, and the calls into the kernel launchers.
#include <hip/hip_runtime.h>

#include <sys/syscall.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "fcdp_internal.h"

using fcdp::fail;

// fcdp_materialize_layer_static stages the host-cache image in this array
// instead of a caller-provided staging buffer.  Every device the library
// runs on holds its own copy of the array, at its own address, from the
// moment the code object is loaded until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress; kernels and copies get the
// address that call returns (StaticCtx::ptr below).
static __device__ __align__(256) unsigned char scratch[FCDP_STATIC_STAGING_BYTES];

namespace {

fcdp_status hip_fail(hipError_t e, const char *what)
{
    return fail(FCDP_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define FCDP_HIP(call, what)                                                   \
    do {                                                                       \
        hipError_t e_ = (call);                                                \
        if (e_ != hipSuccess) return hip_fail(e_, what);                       \
    } while (0)

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Debugging aid (tuning knob debug_poison): no sizes cross the boundary, so a
// buffer that is too small cannot be refused in normal operation; with the
// knob on, every device buffer a call is about to read or write is looked up
// with hipMemGetAddressRange and must lie inside ONE allocation with at least
// `bytes` bytes from `p` on.  A pointer the runtime cannot place (a mapped
// host alias, a sub-range it does not track) is let through.  Catches the
// mistakes a caller's own allocator does not hide: an allocation of the
// wrong element size, a shard buffer sized S instead of N_pad, a short tail.
fcdp_status check_extent(const void *p, size_t bytes, const char *fn, const char *what)
{
    if (!p || bytes == 0) return FCDP_OK;
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    hipError_t e = hipMemGetAddressRange(&base, &size, const_cast<void *>(p));
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return FCDP_OK;
    }
    const size_t off = static_cast<size_t>(static_cast<const char *>(p) - static_cast<const char *>(base));
    if (off > size || bytes > size - off)
        return fail(FCDP_ESIZE, std::string(fn) + ": " + what + " needs " + std::to_string(bytes) +
                                    " bytes but its allocation ends after " + std::to_string(size - std::min(off, size)));
    return FCDP_OK;
}

// ----------------------------------------------------------------- events
// A ring of timing-disabled events for "record on A, wait on B" edges, and a
// small table that remembers, per staging buffer, the event recorded after
// the last scatter that read it.
struct DeviceCtx {
    std::mutex mu;
    std::vector<hipEvent_t> ring;
    size_t next = 0;
    struct StagingUse {
        void *staging = nullptr;
        hipEvent_t done = nullptr;
        uint64_t stamp = 0;
    };
    StagingUse uses[8];
    uint64_t clock = 0;
    // bytes of layer images sent over the host link (any thread may add)
    std::atomic<int64_t> stored_bytes{0}, fetched_bytes{0};
    // completion events of the host-link copies still in flight, oldest
    // first, and events ready for reuse; both guarded by mu
    std::deque<hipEvent_t> copies_in_flight;
    std::vector<hipEvent_t> copy_events_free;
};

DeviceCtx g_ctx[fcdp::kMaxDevices];
constexpr size_t kRing = 64;

// ---------------------------------------------------------- kernel timing
struct TimedLaunch {
    int32_t kind;
    hipEvent_t start, stop;
};
struct TimingCtx {
    std::vector<hipEvent_t> pool;    // 2 * capacity timing events, created once
    std::vector<TimedLaunch> taken;  // launches recorded so far
    size_t next = 0;
    bool on = false;
};
TimingCtx g_timing[fcdp::kMaxDevices];

TimingCtx *timing_ctx()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= fcdp::kMaxDevices) return nullptr;
    return &g_timing[dev];
}

// Hands out one start/stop pair for a launch of the given kind (nulls when
// timing is off or the pool is used up).
fcdp::LaunchEvents timing_events(int32_t kind)
{
    fcdp::LaunchEvents ev;
    TimingCtx *c = timing_ctx();
    if (!c || !c->on || c->next + 2 > c->pool.size()) return ev;
    ev.start = c->pool[c->next];
    ev.stop = c->pool[c->next + 1];
    c->next += 2;
    c->taken.push_back({kind, static_cast<hipEvent_t>(ev.start), static_cast<hipEvent_t>(ev.stop)});
    return ev;
}

fcdp_status current_ctx(DeviceCtx **out)
{
    int dev = 0;
    FCDP_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= fcdp::kMaxDevices)
        return fail(FCDP_ESIZE, "device ordinal beyond 15 is not supported");
    *out = &g_ctx[dev];
    return FCDP_OK;
}

// dst stream waits for everything enqueued so far on src stream.  Record and
// wait happen under the lock (neither blocks), so two threads never hold the
// same event of the ring between its record and its wait.
fcdp_status order_after(DeviceCtx *ctx, hipStream_t src, hipStream_t dst)
{
    if (src == dst) return FCDP_OK;
    std::lock_guard<std::mutex> lk(ctx->mu);
    hipEvent_t ev;
    if (ctx->ring.size() < kRing) {
        FCDP_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming), "hipEventCreate");
        ctx->ring.push_back(ev);
    } else {
        ev = ctx->ring[ctx->next];
        ctx->next = (ctx->next + 1) % kRing;
    }
    FCDP_HIP(hipEventRecord(ev, src), "hipEventRecord");
    FCDP_HIP(hipStreamWaitEvent(dst, ev, 0), "hipStreamWaitEvent");
    return FCDP_OK;
}

// Back-pressure on host-link copies: call before enqueueing one (may block on
// the host until the oldest queued copy has finished), then copy_enqueued()
// right after it.  The wait happens outside the lock: the event waited for
// has been taken off the list, so no other thread can record it meanwhile.
fcdp_status copy_admit(DeviceCtx *ctx)
{
    const int64_t cap = fcdp::tuning().max_copies_in_flight;
    if (cap <= 0) return FCDP_OK;
    for (;;) {
        hipEvent_t oldest = nullptr;
        {
            std::lock_guard<std::mutex> lk(ctx->mu);
            // retire finished copies without blocking
            while (!ctx->copies_in_flight.empty() && hipEventQuery(ctx->copies_in_flight.front()) == hipSuccess) {
                ctx->copy_events_free.push_back(ctx->copies_in_flight.front());
                ctx->copies_in_flight.pop_front();
            }
            (void)hipGetLastError(); // hipEventQuery reports "not ready" as an error code
            if (static_cast<int64_t>(ctx->copies_in_flight.size()) < cap) return FCDP_OK;
            oldest = ctx->copies_in_flight.front();
            ctx->copies_in_flight.pop_front();
        }
        hipError_t e = hipEventSynchronize(oldest);
        {
            std::lock_guard<std::mutex> lk(ctx->mu);
            ctx->copy_events_free.push_back(oldest);
        }
        if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
    }
}

fcdp_status copy_enqueued(DeviceCtx *ctx, hipStream_t copy)
{
    if (fcdp::tuning().max_copies_in_flight <= 0) return FCDP_OK;
    std::lock_guard<std::mutex> lk(ctx->mu);
    hipEvent_t e = nullptr;
    if (!ctx->copy_events_free.empty()) {
        e = ctx->copy_events_free.back();
        ctx->copy_events_free.pop_back();
    } else {
        FCDP_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming), "hipEventCreate");
    }
    hipError_t err = hipEventRecord(e, copy);
    if (err != hipSuccess) {
        ctx->copy_events_free.push_back(e);
        return hip_fail(err, "hipEventRecord");
    }
    ctx->copies_in_flight.push_back(e);
    return FCDP_OK;
}

fcdp_status staging_slot(DeviceCtx *ctx, void *staging, DeviceCtx::StagingUse **out)
{
    std::lock_guard<std::mutex> lk(ctx->mu);
    DeviceCtx::StagingUse *lru = &ctx->uses[0];
    for (auto &u : ctx->uses) {
        if (u.staging == staging) {
            u.stamp = ++ctx->clock;
            *out = &u;
            return FCDP_OK;
        }
        if (u.stamp < lru->stamp) lru = &u;
    }
    if (!lru->done)
        FCDP_HIP(hipEventCreateWithFlags(&lru->done, hipEventDisableTiming), "hipEventCreate");
    else if (lru->staging) {
        // Recycling a slot: its buffer loses its tracking, so drain the old
        // reader now (rare: more than 8 staging buffers in rotation).
        FCDP_HIP(hipEventSynchronize(lru->done), "hipEventSynchronize");
    }
    lru->staging = nullptr; // "no reader recorded yet"
    lru->stamp = ++ctx->clock;
    *out = lru;
    return FCDP_OK;
}

// ---------------------------------------------------------- device tables
fcdp_status upload(const std::vector<fcdp::Piece> &v, fcdp::Piece **out)
{
    *out = nullptr;
    if (v.empty()) return FCDP_OK;
    const size_t bytes = v.size() * sizeof(fcdp::Piece);
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) return fail(FCDP_ENOMEM, std::string("hipMalloc(piece table): ") + hipGetErrorString(e));
    e = hipMemcpy(p, v.data(), bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(p);
        return hip_fail(e, "hipMemcpy(piece table)");
    }
    *out = static_cast<fcdp::Piece *>(p);
    return FCDP_OK;
}

fcdp_status tables_for_current_device(const fcdp_layout *L, const fcdp::DeviceTables **out)
{
    int dev = 0;
    FCDP_HIP(hipGetDevice(&dev), "hipGetDevice");
    std::lock_guard<std::mutex> lk(L->mu);
    for (const auto &d : L->dev)
        if (d.device == dev) {
            *out = &d;
            return FCDP_OK;
        }
    if (L->dev.capacity() < fcdp::kMaxDevices) L->dev.reserve(fcdp::kMaxDevices);
    if (L->dev.size() >= fcdp::kMaxDevices)
        return fail(FCDP_ESIZE, "layout used on more than 16 devices");
    fcdp::DeviceTables d;
    d.device = dev;
    fcdp_status st;
    if ((st = upload(L->unflatten.pieces, &d.unflatten)) != FCDP_OK) return st;
    if ((st = upload(L->flatten.pieces, &d.flatten)) != FCDP_OK) return st;
    if ((st = upload(L->pack.pieces, &d.pack)) != FCDP_OK) return st;
    if ((st = upload(L->unpack.pieces, &d.unpack)) != FCDP_OK) return st;
    L->dev.push_back(d); // reserved above: earlier pointers stay valid
    *out = &L->dev.back();
    return FCDP_OK;
}

// Runs one tensor-windowed piece table.
fcdp_status run_windowed(const fcdp::PieceTable &tab, const fcdp::Piece *dev_pieces,
                         fcdp::TensorSide side, int32_t T,
                         const void *const *small, int32_t n_small,
                         const void *const *tensors, bool nt, int64_t wg_per_cu,
                         hipStream_t st, const char *what, int32_t kind, int64_t max_wgs = 0,
                         int64_t block = 0)
{
    const int64_t n_win = static_cast<int64_t>(tab.win_begin.size()) - 1;
    for (int64_t w = 0; w < n_win; ++w) {
        const int64_t b = tab.win_begin[w], e = tab.win_begin[w + 1];
        if (e <= b) continue;
        fcdp::CopyLaunch c;
        c.pieces = dev_pieces + b;
        c.n_pieces = e - b;
        c.tensor_side = side;
        c.tensor_base = static_cast<int32_t>(w * fcdp::kTensorWindow);
        c.small_ptrs = small;
        c.n_small = n_small;
        c.tensor_ptrs = tensors + c.tensor_base;
        c.n_tensor = std::min<int32_t>(fcdp::kTensorWindow, T - c.tensor_base);
        c.nt = nt;
        c.wg_per_cu = wg_per_cu;
        c.max_wgs = max_wgs;
        c.block = block;
        c.ev = timing_events(kind); // one pair per launch (per tensor window)
        hipError_t err = static_cast<hipError_t>(fcdp::launch_copy(c, st));
        if (err != hipSuccess) return hip_fail(err, what);
    }
    return FCDP_OK;
}

fcdp_status check_tensor_ptrs(const fcdp_layout *L, const void *const *tensor_ptrs, const char *fn)
{
    if (!tensor_ptrs) return fail(FCDP_EINVAL, std::string(fn) + ": tensor_ptrs is NULL");
    for (int32_t t = 0; t < L->T; ++t) {
        if (L->numel[t] == 0) continue;
        if (!tensor_ptrs[t]) return fail(FCDP_EINVAL, std::string(fn) + ": a tensor pointer is NULL");
        if (!aligned16(tensor_ptrs[t])) return fail(FCDP_EALIGN, std::string(fn) + ": a tensor pointer is not 16-byte aligned");
    }
    return FCDP_OK;
}

fcdp_status check_shard_ptrs(const fcdp_layout *L, const void *const *shard_ptrs, const char *fn)
{
    if (!shard_ptrs) return fail(FCDP_EINVAL, std::string(fn) + ": shard_ptrs is NULL");
    for (int32_t r = 0; r < L->G; ++r) {
        if (!shard_ptrs[r]) return fail(FCDP_EINVAL, std::string(fn) + ": a shard pointer is NULL");
        if (!aligned16(shard_ptrs[r])) return fail(FCDP_EALIGN, std::string(fn) + ": a shard pointer is not 16-byte aligned");
    }
    return FCDP_OK;
}

// Device address of a mapped pinned host buffer, or FCDP_ENOTPINNED.
fcdp_status mapped_alias(void *host, const char *fn, void **alias)
{
    hipPointerAttribute_t attr;
    std::memset(&attr, 0, sizeof attr);
    hipError_t e = hipPointerGetAttributes(&attr, host);
    if (e != hipSuccess) {
        (void)hipGetLastError(); // clear the sticky error of an unknown pointer
        return fail(FCDP_ENOTPINNED, std::string(fn) + ": host_cache is not known to HIP as pinned host memory");
    }
    if (attr.type != hipMemoryTypeHost || !attr.devicePointer)
        return fail(FCDP_ENOTPINNED, std::string(fn) + ": host_cache is not mapped pinned host memory");
    *alias = attr.devicePointer;
    return FCDP_OK;
}

// FCDP_OK if [host, host + bytes) is pinned host memory known to HIP (mapped
// or not), else FCDP_ENOTPINNED.  With pageable memory hipMemcpyAsync stops
// being asynchronous, and the overlap of the cache traffic with the kernels,
// which is what the host cache is for, is silently gone.
fcdp_status require_pinned(const void *host, size_t bytes, const char *fn)
{
    const char *ends[2] = {static_cast<const char *>(host),
                           static_cast<const char *>(host) + (bytes ? bytes - 1 : 0)};
    for (const char *p : ends) {
        hipPointerAttribute_t attr;
        std::memset(&attr, 0, sizeof attr);
        hipError_t e = hipPointerGetAttributes(&attr, p);
        if (e != hipSuccess) (void)hipGetLastError(); // clear the error an unknown pointer leaves
        if (e != hipSuccess || attr.type != hipMemoryTypeHost)
            return fail(FCDP_ENOTPINNED, std::string(fn) + ": host_cache is not pinned host memory "
                                                           "(allocate it with fcdp_host_cache_alloc or hipHostMalloc)");
    }
    return FCDP_OK;
}

// The device alias of mapped pinned host memory, or NULL; leaves no error.
void *alias_or_null(void *host)
{
    hipPointerAttribute_t attr;
    std::memset(&attr, 0, sizeof attr);
    if (hipPointerGetAttributes(&attr, host) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return attr.type == hipMemoryTypeHost ? attr.devicePointer : nullptr;
}

// debug_poison: fill every tensor of the layer on `st`
fcdp_status poison_tensors(const fcdp_layout *L, void *const *tensor_ptrs, hipStream_t st)
{
    for (int32_t t = 0; t < L->T; ++t) {
        if (L->numel[t] == 0) continue;
        hipError_t e = static_cast<hipError_t>(fcdp::launch_fill(
            tensor_ptrs[t], static_cast<size_t>(L->numel[t]) * L->esz, fcdp::kPoison, st));
        if (e != hipSuccess) return hip_fail(e, "launch poison fill");
    }
    return FCDP_OK;
}

// H <- concat(shards): after the producers of the shards (everything on
// `compute` so far), on the `copy` stream.
// `shard_ptrs` are the n_shards consecutive shards whose image `host_cache`
// takes (all G of them for a whole layer).
fcdp_status enqueue_store(const fcdp_layout *L, DeviceCtx *ctx, const void *const *shard_ptrs, int32_t n_shards,
                          void *host_cache, void *store_alias, int store_cache,
                          hipStream_t compute, hipStream_t copy)
{
    const fcdp::Tuning &tune = fcdp::tuning();
    const size_t shard_bytes = static_cast<size_t>(L->S) * L->esz;
    const size_t flat_bytes = shard_bytes * static_cast<size_t>(n_shards);
    fcdp_status st;
    // H <- concat(shards): after the producers of the shards, beside the scatter
    if ((st = order_after(ctx, compute, copy)) != FCDP_OK) return st;
    char *h = static_cast<char *>(host_cache);
    if (tune.debug_poison) {
        // through the mapping, in copy-stream order like the store itself
        if (void *pa = store_alias ? store_alias : alias_or_null(host_cache)) {
            hipError_t e = static_cast<hipError_t>(fcdp::launch_fill(pa, flat_bytes, fcdp::kPoison, copy, tune.link_max_wgs));
            if (e != hipSuccess) return hip_fail(e, "launch poison fill (host cache)");
        }
    }
    // contiguous shards (one gather buffer) go out as a single copy
    bool contiguous = true;
    for (int32_t r = 1; r < n_shards; ++r)
        if (static_cast<const char *>(shard_ptrs[r]) != static_cast<const char *>(shard_ptrs[0]) + r * shard_bytes)
            contiguous = false;
    if (store_cache == FCDP_STORE_ZEROCOPY) {
        // a few workgroups write the image through the host mapping
        fcdp::PlainCopy shape;
        shape.chunk = tune.link_chunk_bytes;
        shape.block = tune.link_block;
        shape.unroll = 4;
        shape.max_wgs = tune.link_max_wgs;
        shape.nt = 0;
        char *ha = static_cast<char *>(store_alias);
        const int32_t n_copies = contiguous ? 1 : n_shards;
        const size_t each = contiguous ? flat_bytes : shard_bytes;
        for (int32_t r = 0; r < n_copies; ++r) {
            shape.ev = timing_events(FCDP_KERNEL_STORE_ZEROCOPY);
            hipError_t e = static_cast<hipError_t>(fcdp::launch_plain_copy(ha + r * each, shard_ptrs[r], each, copy, shape));
            if (e != hipSuccess) return hip_fail(e, "launch zero-copy store");
        }
    } else if (contiguous) {
        if ((st = copy_admit(ctx)) != FCDP_OK) return st;
        FCDP_HIP(hipMemcpyAsync(h, shard_ptrs[0], flat_bytes, hipMemcpyDeviceToHost, copy), "hipMemcpyAsync(D2H)");
        if ((st = copy_enqueued(ctx, copy)) != FCDP_OK) return st;
    } else {
        for (int32_t r = 0; r < n_shards; ++r) {
            if ((st = copy_admit(ctx)) != FCDP_OK) return st;
            FCDP_HIP(hipMemcpyAsync(h + r * shard_bytes, shard_ptrs[r], shard_bytes, hipMemcpyDeviceToHost, copy), "hipMemcpyAsync(D2H)");
            if ((st = copy_enqueued(ctx, copy)) != FCDP_OK) return st;
        }
    }
    ctx->stored_bytes += static_cast<int64_t>(flat_bytes);
    return FCDP_OK;
}


// ------------------------------------------- allocation-free staged fetch

// Per device: the array's device address (the array's name is only a
// host-side handle for hipGetSymbolAddress, never a device address), and the
// two events the entry point needs, all made once at set-up
// (fcdp_layout_prepare) so that the entry point itself creates nothing.
struct StaticCtx {
    std::mutex mu;
    void *ptr = nullptr;          // device address of `scratch` on this device
    hipEvent_t copied = nullptr;  // the H2D copy into the array has finished
    hipEvent_t read_done = nullptr; // the last scatter that read the array has finished
    bool read_recorded = false;
    bool ready = false;
};
StaticCtx g_static[fcdp::kMaxDevices];

// Set-up for the current device; idempotent.
fcdp_status static_setup_current_device()
{
    int dev = 0;
    FCDP_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= fcdp::kMaxDevices)
        return fail(FCDP_ESIZE, "device ordinal beyond 15 is not supported");
    StaticCtx &c = g_static[dev];
    std::lock_guard<std::mutex> lk(c.mu);
    if (c.ready) return FCDP_OK;
    void *p = nullptr;
    FCDP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
    if (!p || !aligned16(p)) return fail(FCDP_EHIP, "hipGetSymbolAddress(scratch) gave an unusable address");
    if (!c.copied) FCDP_HIP(hipEventCreateWithFlags(&c.copied, hipEventDisableTiming), "hipEventCreate");
    if (!c.read_done) FCDP_HIP(hipEventCreateWithFlags(&c.read_done, hipEventDisableTiming), "hipEventCreate");
    c.ptr = p;
    c.ready = true;
    return FCDP_OK;
}

// The layout's tables on the current device if they were uploaded, else NULL.
const fcdp::DeviceTables *tables_if_prepared(const fcdp_layout *L, int dev)
{
    std::lock_guard<std::mutex> lk(L->mu);
    for (const auto &d : L->dev)
        if (d.device == dev) return &d;
    return nullptr;
}

} // namespace

extern "C" {

void fcdp_layout_destroy(fcdp_layout *L)
{
    if (!L) return;
    int cur = -1;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    for (auto &d : L->dev) {
        if (have_cur && d.device != cur) (void)hipSetDevice(d.device);
        if (d.unflatten) (void)hipFree(d.unflatten);
        if (d.flatten) (void)hipFree(d.flatten);
        if (d.pack) (void)hipFree(d.pack);
        if (d.unpack) (void)hipFree(d.unpack);
        if (have_cur && d.device != cur) (void)hipSetDevice(cur);
    }
    delete L;
}

fcdp_status fcdp_layout_prepare(const fcdp_layout *L)
try {
    if (!L) return fail(FCDP_EINVAL, "fcdp_layout_prepare: layout is NULL");
    const fcdp::DeviceTables *d = nullptr;
    fcdp_status st = tables_for_current_device(L, &d);
    if (st != FCDP_OK) return st;
    return static_setup_current_device();
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_layout_prepare: out of host memory");
}

fcdp_status fcdp_materialize_layer(const fcdp_layout *L, fcdp_source src,
                                   const void *const *shard_ptrs,
                                   void *host_cache, void *staging,
                                   void *const *tensor_ptrs, int store_cache,
                                   fcdp_stream compute_, fcdp_stream copy_)
try {
    const char *fn = "fcdp_materialize_layer";
    if (!L) return fail(FCDP_EINVAL, std::string(fn) + ": layout is NULL");
    if (src != FCDP_SRC_DEVICE_SHARDS && src != FCDP_SRC_HOST_DMA && src != FCDP_SRC_HOST_ZEROCOPY &&
        src != FCDP_SRC_DEVICE_RESIDENT && src != FCDP_SRC_HOST_SCATTER_DMA)
        return fail(FCDP_EINVAL, std::string(fn) + ": unknown source");
    if (store_cache != FCDP_STORE_NONE && store_cache != FCDP_STORE_DMA && store_cache != FCDP_STORE_ZEROCOPY)
        return fail(FCDP_EINVAL, std::string(fn) + ": unknown store_cache mode");
    fcdp_status st = check_tensor_ptrs(L, reinterpret_cast<const void *const *>(tensor_ptrs), fn);
    if (st != FCDP_OK) return st;
    if (src == FCDP_SRC_DEVICE_RESIDENT) {
        // the tensors still hold the layer since its forward pass
        if (store_cache) return fail(FCDP_EINVAL, std::string(fn) + ": store_cache is only valid with FCDP_SRC_DEVICE_SHARDS");
        return FCDP_OK;
    }
    hipStream_t compute = static_cast<hipStream_t>(compute_);
    hipStream_t copy = static_cast<hipStream_t>(copy_);
    const size_t flat_bytes = static_cast<size_t>(L->N_pad) * L->esz;
    const size_t shard_bytes = static_cast<size_t>(L->S) * L->esz;
    void *zc_alias = nullptr;
    if (src == FCDP_SRC_DEVICE_SHARDS) {
        if ((st = check_shard_ptrs(L, shard_ptrs, fn)) != FCDP_OK) return st;
        if (store_cache && !host_cache)
            return fail(FCDP_EINVAL, std::string(fn) + ": store_cache needs host_cache");
    } else {
        if (store_cache)
            return fail(FCDP_EINVAL, std::string(fn) + ": store_cache is only valid with FCDP_SRC_DEVICE_SHARDS");
        if (!host_cache) return fail(FCDP_EINVAL, std::string(fn) + ": host_cache is NULL");
        if (!aligned16(host_cache)) return fail(FCDP_EALIGN, std::string(fn) + ": host_cache is not 16-byte aligned");
        if (src == FCDP_SRC_HOST_DMA) {
            if (!staging) return fail(FCDP_EINVAL, std::string(fn) + ": FCDP_SRC_HOST_DMA needs a staging buffer");
            if (!aligned16(staging)) return fail(FCDP_EALIGN, std::string(fn) + ": staging is not 16-byte aligned");
        }
        if (src == FCDP_SRC_HOST_ZEROCOPY && flat_bytes) {
            if ((st = mapped_alias(host_cache, fn, &zc_alias)) != FCDP_OK) return st;
        } else if (flat_bytes && (st = require_pinned(host_cache, flat_bytes, fn)) != FCDP_OK) {
            return st;
        }
    }
    if (store_cache && !aligned16(host_cache))
        return fail(FCDP_EALIGN, std::string(fn) + ": host_cache is not 16-byte aligned");
    if (store_cache == FCDP_STORE_DMA && flat_bytes && (st = require_pinned(host_cache, flat_bytes, fn)) != FCDP_OK)
        return st;
    void *store_alias = nullptr;
    if (store_cache == FCDP_STORE_ZEROCOPY && flat_bytes) {
        if ((st = mapped_alias(host_cache, fn, &store_alias)) != FCDP_OK) return st;
    }
    if (L->N == 0 && !(store_cache && flat_bytes)) return FCDP_OK;

    DeviceCtx *ctx = nullptr;
    if ((st = current_ctx(&ctx)) != FCDP_OK) return st;
    const fcdp::DeviceTables *tabs = nullptr;
    if ((st = tables_for_current_device(L, &tabs)) != FCDP_OK) return st;
    const fcdp::Tuning &tune = fcdp::tuning();

    if (tune.debug_poison) {
        for (int32_t t = 0; t < L->T; ++t)
            if ((st = check_extent(tensor_ptrs[t], static_cast<size_t>(L->numel[t]) * L->esz, fn, "a tensor")) != FCDP_OK) return st;
        if (src == FCDP_SRC_DEVICE_SHARDS)
            for (int32_t r = 0; r < L->G; ++r)
                if ((st = check_extent(shard_ptrs[r], shard_bytes, fn, "a shard")) != FCDP_OK) return st;
        if (src == FCDP_SRC_HOST_DMA && (st = check_extent(staging, flat_bytes, fn, "staging")) != FCDP_OK) return st;
        if ((st = poison_tensors(L, tensor_ptrs, compute)) != FCDP_OK) return st;
    }

    const void *small[FCDP_MAX_G];
    if (src == FCDP_SRC_DEVICE_SHARDS) {
        if (store_cache && flat_bytes) {
            if ((st = enqueue_store(L, ctx, shard_ptrs, L->G, host_cache, store_alias, store_cache, compute, copy)) != FCDP_OK)
                return st;
        }
        for (int32_t r = 0; r < L->G; ++r) small[r] = shard_ptrs[r];
        return run_windowed(L->unflatten, tabs->unflatten, fcdp::TensorSide::Dst, L->T, small, L->G,
                            reinterpret_cast<const void *const *>(tensor_ptrs), tune.copy_nt != 0,
                            tune.copy_wg_per_cu, compute, "launch unflatten", FCDP_KERNEL_UNFLATTEN);
    }
    if (src == FCDP_SRC_HOST_DMA) {
        DeviceCtx::StagingUse *use = nullptr;
        if ((st = staging_slot(ctx, staging, &use)) != FCDP_OK) return st;
        if (use->staging == staging)
            FCDP_HIP(hipStreamWaitEvent(copy, use->done, 0), "hipStreamWaitEvent(staging)");
        if (tune.debug_poison) {
            hipError_t pe = static_cast<hipError_t>(fcdp::launch_fill(staging, flat_bytes, fcdp::kPoison, copy));
            if (pe != hipSuccess) return hip_fail(pe, "launch poison fill (staging)");
        }
        if ((st = copy_admit(ctx)) != FCDP_OK) return st;
        FCDP_HIP(hipMemcpyAsync(staging, host_cache, flat_bytes, hipMemcpyHostToDevice, copy), "hipMemcpyAsync(H2D)");
        if ((st = copy_enqueued(ctx, copy)) != FCDP_OK) return st;
        if ((st = order_after(ctx, copy, compute)) != FCDP_OK) return st;
        for (int32_t r = 0; r < L->G; ++r) small[r] = static_cast<const char *>(staging) + r * shard_bytes;
        st = run_windowed(L->unflatten, tabs->unflatten, fcdp::TensorSide::Dst, L->T, small, L->G,
                          reinterpret_cast<const void *const *>(tensor_ptrs), tune.copy_nt != 0,
                          tune.copy_wg_per_cu, compute, "launch unflatten", FCDP_KERNEL_UNFLATTEN);
        if (st != FCDP_OK) return st;
        {
            std::lock_guard<std::mutex> lk(ctx->mu);
            FCDP_HIP(hipEventRecord(use->done, compute), "hipEventRecord(staging)");
            use->staging = staging;
        }
        ctx->fetched_bytes += static_cast<int64_t>(flat_bytes);
        return FCDP_OK;
    }
    if (src == FCDP_SRC_HOST_SCATTER_DMA) {
        // the tensors may still be read by earlier work on `compute`
        if ((st = order_after(ctx, compute, copy)) != FCDP_OK) return st;
        const char *h = static_cast<const char *>(host_cache);
        for (int32_t t = 0; t < L->T; ++t) {
            if (L->numel[t] == 0) continue;
            if ((st = copy_admit(ctx)) != FCDP_OK) return st;
            FCDP_HIP(hipMemcpyAsync(tensor_ptrs[t], h + L->off[t] * L->esz, static_cast<size_t>(L->numel[t]) * L->esz,
                                    hipMemcpyHostToDevice, copy), "hipMemcpyAsync(H2D, per tensor)");
            if ((st = copy_enqueued(ctx, copy)) != FCDP_OK) return st;
        }
        ctx->fetched_bytes += static_cast<int64_t>(flat_bytes);
        return order_after(ctx, copy, compute);
    }
    // zero-copy: the kernel's loads cross the host link
    if ((st = order_after(ctx, copy, compute)) != FCDP_OK) return st;
    for (int32_t r = 0; r < L->G; ++r) small[r] = static_cast<const char *>(zc_alias) + r * shard_bytes;
    ctx->fetched_bytes += static_cast<int64_t>(flat_bytes);
    return run_windowed(L->unflatten, tabs->unflatten, fcdp::TensorSide::Dst, L->T, small, L->G,
                        reinterpret_cast<const void *const *>(tensor_ptrs), false, 0, compute,
                        "launch zero-copy unflatten", FCDP_KERNEL_UNFLATTEN_ZEROCOPY, tune.link_max_wgs,
                        tune.link_max_wgs > 0 ? tune.link_block : 0);
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_materialize_layer: out of host memory");
}

fcdp_status fcdp_materialize_layer_static(const fcdp_layout *L, void *host_cache,
                                          void *const *tensor_ptrs, fcdp_stream compute_,
                                          fcdp_stream copy_)
try {
    const char *fn = "fcdp_materialize_layer_static";
    if (!L) return fail(FCDP_EINVAL, std::string(fn) + ": layout is NULL");
    fcdp_status st = check_tensor_ptrs(L, reinterpret_cast<const void *const *>(tensor_ptrs), fn);
    if (st != FCDP_OK) return st;
    if (!host_cache) return fail(FCDP_EINVAL, std::string(fn) + ": host_cache is NULL");
    if (!aligned16(host_cache)) return fail(FCDP_EALIGN, std::string(fn) + ": host_cache is not 16-byte aligned");
    const size_t flat_bytes = static_cast<size_t>(L->N_pad) * L->esz;
    const size_t shard_bytes = static_cast<size_t>(L->S) * L->esz;
    if (flat_bytes > FCDP_STATIC_STAGING_BYTES)
        return fail(FCDP_ESIZE, std::string(fn) + ": the padded layer (" + std::to_string(flat_bytes) +
                                    " bytes) exceeds FCDP_STATIC_STAGING_BYTES (" +
                                    std::to_string(static_cast<size_t>(FCDP_STATIC_STAGING_BYTES)) + ")");
    if (L->N == 0) return FCDP_OK;
    if ((st = require_pinned(host_cache, flat_bytes, fn)) != FCDP_OK) return st;
    int dev = 0;
    FCDP_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= fcdp::kMaxDevices)
        return fail(FCDP_ESIZE, "device ordinal beyond 15 is not supported");
    StaticCtx &c = g_static[dev];
    const fcdp::DeviceTables *tabs = tables_if_prepared(L, dev);
    std::lock_guard<std::mutex> lk(c.mu);
    if (!tabs || !c.ready)
        return fail(FCDP_ESTATE, std::string(fn) + ": call fcdp_layout_prepare for this layout on this device first "
                                                   "(this entry point uploads and allocates nothing)");
    hipStream_t compute = static_cast<hipStream_t>(compute_);
    hipStream_t copy = static_cast<hipStream_t>(copy_);
    const fcdp::Tuning &tune = fcdp::tuning();
    // the array may still be read by the scatter of the previous call
    if (c.read_recorded) FCDP_HIP(hipStreamWaitEvent(copy, c.read_done, 0), "hipStreamWaitEvent(scratch)");
    FCDP_HIP(hipMemcpyAsync(c.ptr, host_cache, flat_bytes, hipMemcpyHostToDevice, copy), "hipMemcpyAsync(H2D)");
    if (copy != compute) {
        FCDP_HIP(hipEventRecord(c.copied, copy), "hipEventRecord");
        FCDP_HIP(hipStreamWaitEvent(compute, c.copied, 0), "hipStreamWaitEvent");
    }
    const void *small[FCDP_MAX_G];
    for (int32_t r = 0; r < L->G; ++r) small[r] = static_cast<const char *>(c.ptr) + r * shard_bytes;
    st = run_windowed(L->unflatten, tabs->unflatten, fcdp::TensorSide::Dst, L->T, small, L->G,
                      reinterpret_cast<const void *const *>(tensor_ptrs), tune.copy_nt != 0,
                      tune.copy_wg_per_cu, compute, "launch unflatten", FCDP_KERNEL_UNFLATTEN);
    if (st != FCDP_OK) return st;
    FCDP_HIP(hipEventRecord(c.read_done, compute), "hipEventRecord(scratch)");
    c.read_recorded = true;
    g_ctx[dev].fetched_bytes += static_cast<int64_t>(flat_bytes);
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_materialize_layer_static: out of host memory");
}

fcdp_status fcdp_flatten_to_shards(const fcdp_layout *L, const void *const *tensor_ptrs,
                                   void *const *shard_ptrs, fcdp_stream stream)
try {
    const char *fn = "fcdp_flatten_to_shards";
    if (!L) return fail(FCDP_EINVAL, std::string(fn) + ": layout is NULL");
    fcdp_status st = check_tensor_ptrs(L, tensor_ptrs, fn);
    if (st != FCDP_OK) return st;
    if ((st = check_shard_ptrs(L, reinterpret_cast<const void *const *>(shard_ptrs), fn)) != FCDP_OK) return st;
    if (L->N_pad == 0) return FCDP_OK;
    const fcdp::DeviceTables *tabs = nullptr;
    if ((st = tables_for_current_device(L, &tabs)) != FCDP_OK) return st;
    const void *small[FCDP_MAX_G];
    for (int32_t r = 0; r < L->G; ++r) small[r] = shard_ptrs[r];
    const fcdp::Tuning &tune = fcdp::tuning();
    return run_windowed(L->flatten, tabs->flatten, fcdp::TensorSide::Src, L->T, small, L->G, tensor_ptrs,
                        tune.copy_nt != 0, tune.copy_wg_per_cu, static_cast<hipStream_t>(stream), "launch flatten",
                        FCDP_KERNEL_FLATTEN);
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_flatten_to_shards: out of host memory");
}

fcdp_status fcdp_cache_store(const fcdp_layout *L, const void *const *shard_ptrs, void *host_cache,
                             int store_mode, fcdp_stream compute_, fcdp_stream copy_)
try {
    const char *fn = "fcdp_cache_store";
    if (!L) return fail(FCDP_EINVAL, std::string(fn) + ": layout is NULL");
    if (store_mode != FCDP_STORE_DMA && store_mode != FCDP_STORE_ZEROCOPY)
        return fail(FCDP_EINVAL, std::string(fn) + ": store_mode must be FCDP_STORE_DMA or FCDP_STORE_ZEROCOPY");
    fcdp_status st = check_shard_ptrs(L, shard_ptrs, fn);
    if (st != FCDP_OK) return st;
    if (!host_cache) return fail(FCDP_EINVAL, std::string(fn) + ": host_cache is NULL");
    if (!aligned16(host_cache)) return fail(FCDP_EALIGN, std::string(fn) + ": host_cache is not 16-byte aligned");
    if (L->N_pad == 0) return FCDP_OK;
    void *alias = nullptr;
    if (store_mode == FCDP_STORE_ZEROCOPY && (st = mapped_alias(host_cache, fn, &alias)) != FCDP_OK) return st;
    if (store_mode == FCDP_STORE_DMA &&
        (st = require_pinned(host_cache, static_cast<size_t>(L->N_pad) * L->esz, fn)) != FCDP_OK)
        return st;
    DeviceCtx *ctx = nullptr;
    if ((st = current_ctx(&ctx)) != FCDP_OK) return st;
    return enqueue_store(L, ctx, shard_ptrs, L->G, host_cache, alias, store_mode,
                         static_cast<hipStream_t>(compute_), static_cast<hipStream_t>(copy_));
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_store: out of host memory");
}

// ------------------------------------------------ one GPU's share of a node
namespace {
fcdp_status check_node_slice(const fcdp_layout *L, int32_t first_shard, int32_t n_shards, const char *fn)
{
    if (first_shard < 0 || n_shards < 1 || first_shard > L->G - n_shards)
        return fail(FCDP_EINVAL, std::string(fn) + ": shards [first_shard, first_shard + n_shards) must lie in [0, G)");
    return FCDP_OK;
}
} // namespace

fcdp_status fcdp_cache_store_node_slice(const fcdp_layout *L, int32_t first_shard, int32_t n_shards,
                                        const void *const *shard_ptrs, void *host_slice,
                                        fcdp_stream compute_, fcdp_stream copy_)
try {
    const char *fn = "fcdp_cache_store_node_slice";
    if (!L) return fail(FCDP_EINVAL, std::string(fn) + ": layout is NULL");
    fcdp_status st = check_node_slice(L, first_shard, n_shards, fn);
    if (st != FCDP_OK) return st;
    if (!shard_ptrs) return fail(FCDP_EINVAL, std::string(fn) + ": shard_ptrs is NULL");
    for (int32_t r = first_shard; r < first_shard + n_shards; ++r) {
        if (!shard_ptrs[r]) return fail(FCDP_EINVAL, std::string(fn) + ": a shard pointer of the slice is NULL");
        if (!aligned16(shard_ptrs[r])) return fail(FCDP_EALIGN, std::string(fn) + ": a shard pointer is not 16-byte aligned");
    }
    if (!host_slice) return fail(FCDP_EINVAL, std::string(fn) + ": host_slice is NULL");
    if (!aligned16(host_slice)) return fail(FCDP_EALIGN, std::string(fn) + ": host_slice is not 16-byte aligned");
    const size_t slice_bytes = static_cast<size_t>(L->S) * L->esz * static_cast<size_t>(n_shards);
    if (slice_bytes == 0) return FCDP_OK;
    if ((st = require_pinned(host_slice, slice_bytes, fn)) != FCDP_OK) return st;
    DeviceCtx *ctx = nullptr;
    if ((st = current_ctx(&ctx)) != FCDP_OK) return st;
    if (fcdp::tuning().debug_poison)
        for (int32_t r = first_shard; r < first_shard + n_shards; ++r)
            if ((st = check_extent(shard_ptrs[r], static_cast<size_t>(L->S) * L->esz, fn, "a shard")) != FCDP_OK) return st;
    return enqueue_store(L, ctx, shard_ptrs + first_shard, n_shards, host_slice, nullptr, FCDP_STORE_DMA,
                         static_cast<hipStream_t>(compute_), static_cast<hipStream_t>(copy_));
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_store_node_slice: out of host memory");
}

fcdp_status fcdp_materialize_layer_node_slice(const fcdp_layout *L, int32_t first_shard, int32_t n_shards,
                                              const void *const *shard_ptrs, void *host_slice,
                                              void *staging_slice, void *const *tensor_ptrs,
                                              fcdp_stream compute_, fcdp_stream copy_)
try {
    const char *fn = "fcdp_materialize_layer_node_slice";
    if (!L) return fail(FCDP_EINVAL, std::string(fn) + ": layout is NULL");
    fcdp_status st = check_node_slice(L, first_shard, n_shards, fn);
    if (st != FCDP_OK) return st;
    if ((st = check_tensor_ptrs(L, reinterpret_cast<const void *const *>(tensor_ptrs), fn)) != FCDP_OK) return st;
    if (!shard_ptrs && n_shards < L->G) return fail(FCDP_EINVAL, std::string(fn) + ": shard_ptrs is NULL");
    for (int32_t r = 0; r < L->G; ++r) {
        if (r >= first_shard && r < first_shard + n_shards) continue; // the slice comes from the host
        if (!shard_ptrs[r]) return fail(FCDP_EINVAL, std::string(fn) + ": a shard pointer outside the slice is NULL");
        if (!aligned16(shard_ptrs[r])) return fail(FCDP_EALIGN, std::string(fn) + ": a shard pointer is not 16-byte aligned");
    }
    if (!host_slice) return fail(FCDP_EINVAL, std::string(fn) + ": host_slice is NULL");
    if (!aligned16(host_slice)) return fail(FCDP_EALIGN, std::string(fn) + ": host_slice is not 16-byte aligned");
    if (!staging_slice) return fail(FCDP_EINVAL, std::string(fn) + ": staging_slice is NULL");
    if (!aligned16(staging_slice)) return fail(FCDP_EALIGN, std::string(fn) + ": staging_slice is not 16-byte aligned");
    const size_t shard_bytes = static_cast<size_t>(L->S) * L->esz;
    const size_t slice_bytes = shard_bytes * static_cast<size_t>(n_shards);
    if (L->N == 0) return FCDP_OK;
    if ((st = require_pinned(host_slice, slice_bytes, fn)) != FCDP_OK) return st;
    hipStream_t compute = static_cast<hipStream_t>(compute_);
    hipStream_t copy = static_cast<hipStream_t>(copy_);
    DeviceCtx *ctx = nullptr;
    if ((st = current_ctx(&ctx)) != FCDP_OK) return st;
    const fcdp::DeviceTables *tabs = nullptr;
    if ((st = tables_for_current_device(L, &tabs)) != FCDP_OK) return st;
    const fcdp::Tuning &tune = fcdp::tuning();
    if (tune.debug_poison) {
        for (int32_t t = 0; t < L->T; ++t)
            if ((st = check_extent(tensor_ptrs[t], static_cast<size_t>(L->numel[t]) * L->esz, fn, "a tensor")) != FCDP_OK) return st;
        for (int32_t r = 0; r < L->G; ++r)
            if ((r < first_shard || r >= first_shard + n_shards) &&
                (st = check_extent(shard_ptrs[r], shard_bytes, fn, "a shard")) != FCDP_OK) return st;
        if ((st = check_extent(staging_slice, slice_bytes, fn, "staging_slice")) != FCDP_OK) return st;
        if ((st = poison_tensors(L, tensor_ptrs, compute)) != FCDP_OK) return st;
    }
    DeviceCtx::StagingUse *use = nullptr;
    if ((st = staging_slot(ctx, staging_slice, &use)) != FCDP_OK) return st;
    if (use->staging == staging_slice)
        FCDP_HIP(hipStreamWaitEvent(copy, use->done, 0), "hipStreamWaitEvent(staging)");
    if (tune.debug_poison) {
        hipError_t pe = static_cast<hipError_t>(fcdp::launch_fill(staging_slice, slice_bytes, fcdp::kPoison, copy));
        if (pe != hipSuccess) return hip_fail(pe, "launch poison fill (staging)");
    }
    if ((st = copy_admit(ctx)) != FCDP_OK) return st;
    FCDP_HIP(hipMemcpyAsync(staging_slice, host_slice, slice_bytes, hipMemcpyHostToDevice, copy), "hipMemcpyAsync(H2D)");
    if ((st = copy_enqueued(ctx, copy)) != FCDP_OK) return st;
    if ((st = order_after(ctx, copy, compute)) != FCDP_OK) return st;
    const void *small[FCDP_MAX_G];
    for (int32_t r = 0; r < L->G; ++r)
        small[r] = (r >= first_shard && r < first_shard + n_shards)
                       ? static_cast<const char *>(staging_slice) + static_cast<size_t>(r - first_shard) * shard_bytes
                       : shard_ptrs[r];
    st = run_windowed(L->unflatten, tabs->unflatten, fcdp::TensorSide::Dst, L->T, small, L->G,
                      reinterpret_cast<const void *const *>(tensor_ptrs), tune.copy_nt != 0,
                      tune.copy_wg_per_cu, compute, "launch unflatten", FCDP_KERNEL_UNFLATTEN);
    if (st != FCDP_OK) return st;
    {
        std::lock_guard<std::mutex> lk(ctx->mu);
        FCDP_HIP(hipEventRecord(use->done, compute), "hipEventRecord(staging)");
        use->staging = staging_slice;
    }
    ctx->fetched_bytes += static_cast<int64_t>(slice_bytes);
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_materialize_layer_node_slice: out of host memory");
}

fcdp_status fcdp_link_bytes(int32_t reset, int64_t *stored, int64_t *fetched)
try {
    DeviceCtx *ctx = nullptr;
    fcdp_status st = current_ctx(&ctx);
    if (st != FCDP_OK) return st;
    if (stored) *stored = reset ? ctx->stored_bytes.exchange(0) : ctx->stored_bytes.load();
    if (fetched) *fetched = reset ? ctx->fetched_bytes.exchange(0) : ctx->fetched_bytes.load();
    if (reset && !stored) ctx->stored_bytes = 0;
    if (reset && !fetched) ctx->fetched_bytes = 0;
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_link_bytes: out of host memory");
}

fcdp_status fcdp_reduce_grad_shard(const void *const *partial_ptrs, int32_t G, int64_t elem_offset,
                                   int64_t count, fcdp_dtype in, fcdp_dtype out, void *out_shard,
                                   fcdp_stream stream)
try {
    return fcdp_reduce_grad_shard_scaled(partial_ptrs, G, elem_offset, count, in, out, 1.0f, out_shard, stream);
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_reduce_grad_shard: out of host memory");
}

fcdp_status fcdp_reduce_grad_shard_scaled(const void *const *partial_ptrs, int32_t G, int64_t elem_offset,
                                          int64_t count, fcdp_dtype in, fcdp_dtype out, float scale,
                                          void *out_shard, fcdp_stream stream)
try {
    const char *fn = "fcdp_reduce_grad_shard";
    if (!std::isfinite(scale)) return fail(FCDP_EINVAL, std::string(fn) + ": scale is not finite");
    if (!partial_ptrs) return fail(FCDP_EINVAL, std::string(fn) + ": partial_ptrs is NULL");
    if (G < 1) return fail(FCDP_EINVAL, std::string(fn) + ": G must be >= 1");
    if (G > FCDP_MAX_G) return fail(FCDP_ESIZE, std::string(fn) + ": G exceeds FCDP_MAX_G (64)");
    if (count < 0 || elem_offset < 0) return fail(FCDP_EINVAL, std::string(fn) + ": negative count or offset");
    if ((in != FCDP_BF16 && in != FCDP_F32) || (out != FCDP_BF16 && out != FCDP_F32))
        return fail(FCDP_EINVAL, std::string(fn) + ": unknown dtype");
    if (!out_shard) return fail(FCDP_EINVAL, std::string(fn) + ": out_shard is NULL");
    if (!aligned16(out_shard)) return fail(FCDP_EALIGN, std::string(fn) + ": out_shard is not 16-byte aligned");
    const int64_t ie = in == FCDP_F32 ? 4 : 2, oe = out == FCDP_F32 ? 4 : 2;
    const char *ob = static_cast<const char *>(out_shard);
    const char *oe_ = ob + count * oe;
    for (int32_t g = 0; g < G; ++g) {
        if (!partial_ptrs[g]) return fail(FCDP_EINVAL, std::string(fn) + ": a partial pointer is NULL");
        if (!aligned16(partial_ptrs[g])) return fail(FCDP_EALIGN, std::string(fn) + ": a partial pointer is not 16-byte aligned");
        const char *pb = static_cast<const char *>(partial_ptrs[g]) + elem_offset * ie;
        const char *pe = pb + count * ie;
        const bool overlap = count > 0 && pb < oe_ && ob < pe;
        if (overlap && !(pb == ob && ie == oe))
            return fail(FCDP_EINVAL, std::string(fn) + ": out_shard overlaps an input other than exactly in place");
    }
    if (fcdp::tuning().debug_poison) {
        fcdp_status st;
        for (int32_t g = 0; g < G; ++g)
            if ((st = check_extent(partial_ptrs[g], static_cast<size_t>(elem_offset + count) * ie, fn, "a partial")) != FCDP_OK) return st;
        if ((st = check_extent(out_shard, static_cast<size_t>(count) * oe, fn, "out_shard")) != FCDP_OK) return st;
    }
    hipError_t e = static_cast<hipError_t>(fcdp::launch_reduce(partial_ptrs, G, elem_offset, count, in, out, scale, out_shard, stream,
                                                               count > 0 ? timing_events(FCDP_KERNEL_REDUCE) : fcdp::LaunchEvents()));
    if (e != hipSuccess) return hip_fail(e, "launch reduce");
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_reduce_grad_shard_scaled: out of host memory");
}

fcdp_status fcdp_reduce_trainable_shard(const fcdp_layout *L, const void *const *flat_grad_ptrs,
                                        int32_t rank, fcdp_dtype in, fcdp_dtype out, void *out_shard,
                                        fcdp_stream stream)
try {
    return fcdp_reduce_trainable_shard_scaled(L, flat_grad_ptrs, rank, in, out, 1.0f, out_shard, stream);
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_reduce_trainable_shard: out of host memory");
}

fcdp_status fcdp_reduce_trainable_shard_scaled(const fcdp_layout *L, const void *const *flat_grad_ptrs,
                                               int32_t rank, fcdp_dtype in, fcdp_dtype out, float scale,
                                               void *out_shard, fcdp_stream stream)
try {
    const char *fn = "fcdp_reduce_trainable_shard";
    if (!std::isfinite(scale)) return fail(FCDP_EINVAL, std::string(fn) + ": scale is not finite");
    if (!L) return fail(FCDP_EINVAL, std::string(fn) + ": layout is NULL");
    if (!flat_grad_ptrs) return fail(FCDP_EINVAL, std::string(fn) + ": flat_grad_ptrs is NULL");
    if (rank < 0 || rank >= L->G) return fail(FCDP_EINVAL, std::string(fn) + ": rank out of range");
    if ((in != FCDP_BF16 && in != FCDP_F32) || (out != FCDP_BF16 && out != FCDP_F32))
        return fail(FCDP_EINVAL, std::string(fn) + ": unknown dtype");
    if (!out_shard) return fail(FCDP_EINVAL, std::string(fn) + ": out_shard is NULL");
    if (!aligned16(out_shard)) return fail(FCDP_EALIGN, std::string(fn) + ": out_shard is not 16-byte aligned");
    const int64_t ie = in == FCDP_F32 ? 4 : 2, oe = out == FCDP_F32 ? 4 : 2;
    const int64_t Sp = L->N_packed / L->G;
    const char *ob = static_cast<const char *>(out_shard);
    for (int32_t g = 0; g < L->G; ++g) {
        if (!flat_grad_ptrs[g]) return fail(FCDP_EINVAL, std::string(fn) + ": a gradient pointer is NULL");
        if (!aligned16(flat_grad_ptrs[g])) return fail(FCDP_EALIGN, std::string(fn) + ": a gradient pointer is not 16-byte aligned");
        const char *pb = static_cast<const char *>(flat_grad_ptrs[g]);
        if (Sp > 0 && pb < ob + Sp * oe && ob < pb + L->N_pad * ie)
            return fail(FCDP_EINVAL, std::string(fn) + ": out_shard overlaps an input");
    }
    if (Sp == 0) return FCDP_OK;
    // this rank's slice [lo, hi) of the packed order, cut by the trainable runs
    const int64_t lo = static_cast<int64_t>(rank) * Sp, hi = lo + Sp;
    std::vector<fcdp::ReduceRuns> batches(1);
    auto add = [&](int64_t src, int64_t dst, int64_t count) {
        if (batches.back().n_runs == fcdp::kMaxReduceRuns) batches.emplace_back();
        fcdp::ReduceRuns &b = batches.back();
        b.src_off[b.n_runs] = src;
        b.dst_off[b.n_runs] = dst;
        b.count[b.n_runs] = count;
        ++b.n_runs;
    };
    int64_t c = 0; // packed position of the current tensor
    for (int32_t t = 0; t < L->T; ++t) {
        if (!L->trainable[t]) continue;
        const int64_t a = std::max(c, lo), b = std::min(c + L->numel[t], hi);
        if (b > a) add(L->off[t] + (a - c), a - lo, b - a);
        c += L->numel[t];
    }
    if (hi > std::max(lo, L->N_t)) add(-1, std::max(lo, L->N_t) - lo, hi - std::max(lo, L->N_t)); // zero tail
    for (const fcdp::ReduceRuns &b : batches) {
        hipError_t e = static_cast<hipError_t>(fcdp::launch_reduce_runs(
            flat_grad_ptrs, L->G, b, in, out, scale, out_shard, stream, timing_events(FCDP_KERNEL_REDUCE_TRAINABLE)));
        if (e != hipSuccess) return hip_fail(e, "launch trainable reduce");
    }
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_reduce_trainable_shard_scaled: out of host memory");
}

static fcdp_status pack_or_unpack(const fcdp_layout *L, const void *src, void *dst, bool pack,
                                  fcdp_stream stream, const char *fn)
{
    if (!L) return fail(FCDP_EINVAL, std::string(fn) + ": layout is NULL");
    if (!src || !dst) return fail(FCDP_EINVAL, std::string(fn) + ": NULL buffer");
    if (!aligned16(src) || !aligned16(dst)) return fail(FCDP_EALIGN, std::string(fn) + ": buffer not 16-byte aligned");
    const char *flat = static_cast<const char *>(pack ? src : dst);
    const char *packed = static_cast<const char *>(pack ? dst : src);
    const int64_t fb = L->N_pad * L->esz, pb = L->N_packed * L->esz;
    if (fb > 0 && pb > 0 && flat < packed + pb && packed < flat + fb)
        return fail(FCDP_EINVAL, std::string(fn) + ": flat and packed overlap");
    const fcdp::PieceTable &tab = pack ? L->pack : L->unpack;
    if (tab.pieces.empty()) return FCDP_OK;
    if (fcdp::tuning().debug_poison) {
        fcdp_status ce;
        if ((ce = check_extent(flat, static_cast<size_t>(fb), fn, "flat")) != FCDP_OK) return ce;
        if ((ce = check_extent(packed, static_cast<size_t>(pb), fn, "packed")) != FCDP_OK) return ce;
    }
    const fcdp::DeviceTables *tabs = nullptr;
    fcdp_status st = tables_for_current_device(L, &tabs);
    if (st != FCDP_OK) return st;
    const void *small[2] = {src, dst};
    fcdp::CopyLaunch c;
    c.pieces = pack ? tabs->pack : tabs->unpack;
    c.n_pieces = static_cast<int64_t>(tab.pieces.size());
    c.tensor_side = fcdp::TensorSide::None;
    c.small_ptrs = small;
    c.n_small = 2;
    c.nt = false;
    c.wg_per_cu = 0;
    c.ev = timing_events(pack ? FCDP_KERNEL_PACK : FCDP_KERNEL_UNPACK);
    hipError_t e = static_cast<hipError_t>(fcdp::launch_copy(c, stream));
    if (e != hipSuccess) return hip_fail(e, fn);
    return FCDP_OK;
}

fcdp_status fcdp_pack_trainable(const fcdp_layout *L, const void *flat, void *packed, fcdp_stream stream)
try {
    return pack_or_unpack(L, flat, packed, true, stream, "fcdp_pack_trainable");
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_pack_trainable: out of host memory");
}

fcdp_status fcdp_unpack_trainable(const fcdp_layout *L, const void *packed, void *flat, fcdp_stream stream)
try {
    return pack_or_unpack(L, packed, flat, false, stream, "fcdp_unpack_trainable");
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_unpack_trainable: out of host memory");
}

fcdp_status fcdp_unpack_trainable_node_slice(const fcdp_layout *L, int32_t first_shard, int32_t n_shards,
                                             const void *packed, void *flat_slice, fcdp_stream stream)
try {
    const char *fn = "fcdp_unpack_trainable_node_slice";
    if (!L) return fail(FCDP_EINVAL, std::string(fn) + ": layout is NULL");
    fcdp_status st = check_node_slice(L, first_shard, n_shards, fn);
    if (st != FCDP_OK) return st;
    if (!packed || !flat_slice) return fail(FCDP_EINVAL, std::string(fn) + ": NULL buffer");
    if (!aligned16(packed) || !aligned16(flat_slice))
        return fail(FCDP_EALIGN, std::string(fn) + ": buffer not 16-byte aligned");
    const int64_t shard_bytes = L->S * L->esz;
    const int64_t lo = first_shard * shard_bytes, hi = lo + n_shards * shard_bytes; // the slice's flat byte range
    const int64_t pb = L->N_packed * L->esz;
    const char *sl = static_cast<const char *>(flat_slice), *pk = static_cast<const char *>(packed);
    if (hi > lo && pb > 0 && sl < pk + pb && pk < sl + (hi - lo))
        return fail(FCDP_EINVAL, std::string(fn) + ": flat_slice and packed overlap");
    // the table is in ascending destination order and cut at shard boundaries: the pieces
    // that write into [lo, hi) are one contiguous part of it
    const std::vector<fcdp::Piece> &pcs = L->unpack.pieces;
    const auto first = std::lower_bound(pcs.begin(), pcs.end(), lo,
                                        [](const fcdp::Piece &p, int64_t v) { return p.dst_off < v; });
    const auto last = std::lower_bound(first, pcs.end(), hi,
                                       [](const fcdp::Piece &p, int64_t v) { return p.dst_off < v; });
    if (first == last) return FCDP_OK;               // no trainable element lives in this slice
    if (fcdp::tuning().debug_poison) {
        if ((st = check_extent(flat_slice, static_cast<size_t>(hi - lo), fn, "flat_slice")) != FCDP_OK) return st;
        if ((st = check_extent(packed, static_cast<size_t>(pb), fn, "packed")) != FCDP_OK) return st;
    }
    const fcdp::DeviceTables *tabs = nullptr;
    if ((st = tables_for_current_device(L, &tabs)) != FCDP_OK) return st;
    // the pieces carry offsets into the whole flat buffer: hand the kernel the address the
    // whole buffer would start at; only [lo, hi) of it is touched
    const void *small[2] = {packed, reinterpret_cast<void *>(reinterpret_cast<uintptr_t>(flat_slice) -
                                                            static_cast<uintptr_t>(lo))};
    fcdp::CopyLaunch c;
    c.pieces = tabs->unpack + (first - pcs.begin());
    c.n_pieces = static_cast<int64_t>(last - first);
    c.tensor_side = fcdp::TensorSide::None;
    c.small_ptrs = small;
    c.n_small = 2;
    c.nt = false;
    c.wg_per_cu = 0;
    c.ev = timing_events(FCDP_KERNEL_UNPACK);
    hipError_t e = static_cast<hipError_t>(fcdp::launch_copy(c, stream));
    if (e != hipSuccess) return hip_fail(e, fn);
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_unpack_trainable_node_slice: out of host memory");
}

// ------------------------------------------------------------- host cache

fcdp_status fcdp_host_cache_alloc(size_t bytes, int numa_node, void **host, void **dev_alias)
try {
    const char *fn = "fcdp_host_cache_alloc";
    if (!host || !dev_alias) return fail(FCDP_EINVAL, std::string(fn) + ": NULL output pointer");
    *host = nullptr;
    *dev_alias = nullptr;
    if (bytes == 0) return fail(FCDP_EINVAL, std::string(fn) + ": zero bytes");
    if (numa_node >= 1024) return fail(FCDP_EINVAL, std::string(fn) + ": numa_node out of range");
    unsigned flags = hipHostMallocMapped | hipHostMallocPortable;
    bool policy_set = false;
    std::string note;
#ifdef SYS_set_mempolicy
    unsigned long mask[16] = {0};
    if (numa_node >= 0) {
        mask[numa_node / (8 * sizeof(unsigned long))] |= 1ul << (numa_node % (8 * sizeof(unsigned long)));
        // MPOL_PREFERRED = 1: take pages from this node while it has any
        if (syscall(SYS_set_mempolicy, 1, mask, sizeof(mask) * 8) == 0) {
            policy_set = true;
            flags |= hipHostMallocNumaUser;
        } else {
            note = "fcdp_host_cache_alloc: NUMA policy refused by the kernel; allocated without it";
        }
    }
#else
    if (numa_node >= 0) note = "fcdp_host_cache_alloc: no NUMA policy call on this platform";
#endif
    void *p = nullptr;
    hipError_t e = hipHostMalloc(&p, bytes, flags);
#ifdef SYS_set_mempolicy
    if (policy_set) (void)syscall(SYS_set_mempolicy, 0 /* MPOL_DEFAULT */, nullptr, 0);
#endif
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(FCDP_ENOMEM, std::string(fn) + ": hipHostMalloc: " + hipGetErrorString(e));
    }
    void *d = nullptr;
    e = hipHostGetDevicePointer(&d, p, 0);
    if (e != hipSuccess) {
        (void)hipHostFree(p);
        return hip_fail(e, "hipHostGetDevicePointer");
    }
    *host = p;
    *dev_alias = d;
    fcdp::set_error(note);
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_host_cache_alloc: out of host memory");
}

fcdp_status fcdp_host_cache_free(void *host)
try {
    if (!host) return FCDP_OK;
    FCDP_HIP(hipHostFree(host), "hipHostFree");
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_host_cache_free: out of host memory");
}

// ------------------------------------------------------------ dirty state
} // extern "C"

struct fcdp_cache_state {
    std::vector<uint8_t> dirty;    // [layer][class]
    std::vector<uint8_t> pending;  // [layer][class]: handed out for storing in this forward pass
    std::vector<uint8_t> resident; // [layer]: kept on the device until its backward pass
    double tau = 0.0;
    int32_t L = 0;
};

extern "C" {

fcdp_status fcdp_cache_state_create(int32_t n_layers, fcdp_cache_state **out)
try {
    if (!out) return fail(FCDP_EINVAL, "fcdp_cache_state_create: out is NULL");
    *out = nullptr;
    if (n_layers < 1) return fail(FCDP_EINVAL, "fcdp_cache_state_create: n_layers must be >= 1");
    fcdp_cache_state *s = new (std::nothrow) fcdp_cache_state;
    if (!s) return fail(FCDP_ENOMEM, "fcdp_cache_state_create: out of host memory");
    s->L = n_layers;
    s->dirty.assign(static_cast<size_t>(n_layers) * 2, 1); // Alg. 1: everything starts dirty
    s->pending.assign(static_cast<size_t>(n_layers) * 2, 0);
    s->resident.assign(static_cast<size_t>(n_layers), 0);
    *out = s;
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_state_create: out of host memory");
}

void fcdp_cache_state_destroy(fcdp_cache_state *s) { delete s; }

static bool host_mode_ok(fcdp_source m)
{
    return m == FCDP_SRC_HOST_DMA || m == FCDP_SRC_HOST_ZEROCOPY || m == FCDP_SRC_HOST_SCATTER_DMA;
}

fcdp_status fcdp_cache_state_forward_source(fcdp_cache_state *s, int32_t layer, int32_t klass,
                                            fcdp_source host_mode, fcdp_source *src, int32_t *store_cache)
try {
    const char *fn = "fcdp_cache_state_forward_source";
    if (!s || !src || !store_cache) return fail(FCDP_EINVAL, std::string(fn) + ": NULL argument");
    if (layer < 0 || layer >= s->L || klass < 0 || klass > 1) return fail(FCDP_EINVAL, std::string(fn) + ": layer or class out of range");
    if (!host_mode_ok(host_mode)) return fail(FCDP_EINVAL, std::string(fn) + ": host_mode must be a host source");
    uint8_t &d = s->dirty[static_cast<size_t>(layer) * 2 + klass];
    if (d) {
        *src = FCDP_SRC_DEVICE_SHARDS; // inter-node gather result, then H <- p
        *store_cache = 1;
        d = 0;
        s->pending[static_cast<size_t>(layer) * 2 + klass] = 1;
    } else {
        *src = host_mode;
        *store_cache = 0;
    }
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_state_forward_source: out of host memory");
}

fcdp_status fcdp_cache_state_backward_source(const fcdp_cache_state *s, int32_t layer, int32_t klass,
                                             fcdp_source host_mode, fcdp_source *src)
try {
    const char *fn = "fcdp_cache_state_backward_source";
    if (!s || !src) return fail(FCDP_EINVAL, std::string(fn) + ": NULL argument");
    if (layer < 0 || layer >= s->L || klass < 0 || klass > 1) return fail(FCDP_EINVAL, std::string(fn) + ": layer or class out of range");
    if (!host_mode_ok(host_mode)) return fail(FCDP_EINVAL, std::string(fn) + ": host_mode must be a host source");
    if (s->resident[layer]) {
        *src = FCDP_SRC_DEVICE_RESIDENT;
        return FCDP_OK;
    }
    if (s->dirty[static_cast<size_t>(layer) * 2 + klass])
        return fail(FCDP_ESTATE, std::string(fn) + ": backward before the forward pass stored this layer");
    *src = host_mode;
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_state_backward_source: out of host memory");
}

fcdp_status fcdp_cache_state_optimizer_step(fcdp_cache_state *s)
try {
    if (!s) return fail(FCDP_EINVAL, "fcdp_cache_state_optimizer_step: NULL state");
    for (int32_t l = 0; l < s->L; ++l) {
        s->dirty[static_cast<size_t>(l) * 2 + 1] = 1;
        s->pending[static_cast<size_t>(l) * 2] = s->pending[static_cast<size_t>(l) * 2 + 1] = 0;
        s->resident[l] = 0;
    }
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_state_optimizer_step: out of host memory");
}

fcdp_status fcdp_cache_state_mark_dirty(fcdp_cache_state *s, int32_t layer, int32_t klass)
try {
    const char *fn = "fcdp_cache_state_mark_dirty";
    if (!s) return fail(FCDP_EINVAL, std::string(fn) + ": NULL state");
    if (layer < 0 || layer >= s->L || klass < 0 || klass > 1) return fail(FCDP_EINVAL, std::string(fn) + ": layer or class out of range");
    s->dirty[static_cast<size_t>(layer) * 2 + klass] = 1;
    s->pending[static_cast<size_t>(layer) * 2 + klass] = 0;
    s->resident[layer] = 0;
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_state_mark_dirty: out of host memory");
}

fcdp_status fcdp_cache_state_set_tau(fcdp_cache_state *s, double tau)
try {
    if (!s) return fail(FCDP_EINVAL, "fcdp_cache_state_set_tau: NULL state");
    if (!(tau >= 0.0 && tau <= 1.0)) return fail(FCDP_EINVAL, "fcdp_cache_state_set_tau: tau must be in [0, 1]");
    s->tau = tau;
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_state_set_tau: out of host memory");
}

fcdp_status fcdp_cache_state_place(fcdp_cache_state *s, int32_t layer, int64_t used_bytes,
                                   int64_t total_bytes, int32_t *keep)
try {
    const char *fn = "fcdp_cache_state_place";
    if (!s || !keep) return fail(FCDP_EINVAL, std::string(fn) + ": NULL argument");
    if (layer < 0 || layer >= s->L) return fail(FCDP_EINVAL, std::string(fn) + ": layer out of range");
    if (total_bytes <= 0 || used_bytes < 0 || used_bytes > total_bytes)
        return fail(FCDP_EINVAL, std::string(fn) + ": need 0 <= used_bytes <= total_bytes, total_bytes > 0");
    const double util = static_cast<double>(used_bytes) / static_cast<double>(total_bytes);
    const bool k = util < s->tau; // Sec. 4.4: below the threshold the layer stays on the device
    for (int c = 0; c < 2; ++c) {
        uint8_t &p = s->pending[static_cast<size_t>(layer) * 2 + c];
        if (k && p) s->dirty[static_cast<size_t>(layer) * 2 + c] = 1; // not stored after all
        p = 0;
    }
    s->resident[layer] = k ? 1 : 0;
    *keep = k ? 1 : 0;
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_state_place: out of host memory");
}

fcdp_status fcdp_cache_state_release(fcdp_cache_state *s, int32_t layer)
try {
    if (!s) return fail(FCDP_EINVAL, "fcdp_cache_state_release: NULL state");
    if (layer < 0 || layer >= s->L) return fail(FCDP_EINVAL, "fcdp_cache_state_release: layer out of range");
    s->resident[layer] = 0;
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_cache_state_release: out of host memory");
}

int32_t fcdp_cache_state_is_dirty(const fcdp_cache_state *s, int32_t layer, int32_t klass)
{
    if (!s || layer < 0 || layer >= s->L || klass < 0 || klass > 1) return -1;
    return s->dirty[static_cast<size_t>(layer) * 2 + klass];
}

// ----------------------------------------------------------------- tuning

fcdp_status fcdp_tuning_set(const char *name, int64_t v)
try {
    if (!name) return fail(FCDP_EINVAL, "fcdp_tuning_set: name is NULL");
    fcdp::Tuning &t = fcdp::tuning();
    const std::string n(name);
    auto pow2 = [](int64_t x) { return x > 0 && (x & (x - 1)) == 0; };
    if (n == "copy_chunk_bytes") {
        if (v < 4096 || v > (1 << 24) || v % 4096) return fail(FCDP_EINVAL, "copy_chunk_bytes: multiple of 4096 in 4096..16 MiB");
        t.copy_chunk_bytes = v;
    } else if (n == "copy_block") {
        if (v < 64 || v > 1024 || !pow2(v)) return fail(FCDP_EINVAL, "copy_block: power of two in 64..1024");
        t.copy_block = v;
    } else if (n == "copy_unroll") {
        if (v != 1 && v != 2 && v != 4 && v != 8) return fail(FCDP_EINVAL, "copy_unroll: 1, 2, 4 or 8");
        t.copy_unroll = v;
    } else if (n == "copy_wg_per_cu") {
        if (v < 0 || v > 64) return fail(FCDP_EINVAL, "copy_wg_per_cu: 0..64");
        t.copy_wg_per_cu = v;
    } else if (n == "link_max_wgs") {
        if (v < 0 || v > 65536) return fail(FCDP_EINVAL, "link_max_wgs: 0..65536");
        t.link_max_wgs = v;
    } else if (n == "link_block") {
        if (v < 64 || v > 1024 || !pow2(v)) return fail(FCDP_EINVAL, "link_block: power of two in 64..1024");
        t.link_block = v;
    } else if (n == "link_chunk_bytes") {
        if (v < 4096 || v > (1 << 24) || v % 4096) return fail(FCDP_EINVAL, "link_chunk_bytes: multiple of 4096 in 4096..16 MiB");
        t.link_chunk_bytes = v;
    } else if (n == "copy_nt") {
        if (v < 0 || v > 3) return fail(FCDP_EINVAL, "copy_nt: 0..3 (bit 0 loads, bit 1 stores)");
        t.copy_nt = v;
    } else if (n == "max_copies_in_flight") {
        if (v < 0 || v > 4096) return fail(FCDP_EINVAL, "max_copies_in_flight: 0..4096");
        t.max_copies_in_flight = v;
    } else if (n == "reduce_block") {
        if (v < 64 || v > 256 || !pow2(v)) return fail(FCDP_EINVAL, "reduce_block: power of two in 64..256");
        t.reduce_block = v;
    } else if (n == "reduce_phased") {
        if (v < 0 || v > 2) return fail(FCDP_EINVAL, "reduce_phased: 0, 1 or 2");
        t.reduce_phased = v;
    } else if (n == "reduce_phase_rotate") {
        if (v < 0 || v > 2) return fail(FCDP_EINVAL, "reduce_phase_rotate: 0, 1 or 2");
        t.reduce_phase_rotate = v;
    } else if (n == "reduce_phase_waves") {
        if (v < 0 || v > 2) return fail(FCDP_EINVAL, "reduce_phase_waves: 0, 1 or 2");
        t.reduce_phase_waves = v;
    } else if (n == "debug_poison") {
        if (v != 0 && v != 1) return fail(FCDP_EINVAL, "debug_poison: 0 or 1");
        t.debug_poison = v;
    } else {
        return fail(FCDP_EINVAL, "fcdp_tuning_set: unknown knob " + n);
    }
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_tuning_set: out of host memory");
}

int64_t fcdp_tuning_get(const char *name)
{
    if (!name) return -1;
    const fcdp::Tuning &t = fcdp::tuning();
    const std::string n(name);
    if (n == "copy_chunk_bytes") return t.copy_chunk_bytes;
    if (n == "copy_block") return t.copy_block;
    if (n == "copy_unroll") return t.copy_unroll;
    if (n == "copy_wg_per_cu") return t.copy_wg_per_cu;
    if (n == "link_max_wgs") return t.link_max_wgs;
    if (n == "link_block") return t.link_block;
    if (n == "link_chunk_bytes") return t.link_chunk_bytes;
    if (n == "copy_nt") return t.copy_nt;
    if (n == "max_copies_in_flight") return t.max_copies_in_flight;
    if (n == "reduce_block") return t.reduce_block;
    if (n == "reduce_phased") return t.reduce_phased;
    if (n == "reduce_phase_waves") return t.reduce_phase_waves;
    if (n == "reduce_phase_rotate") return t.reduce_phase_rotate;
    if (n == "debug_poison") return t.debug_poison;
    if (n == "last_reduce_shape") return fcdp::last_reduce_shape();
    return -1;
}

fcdp_status fcdp_probe_copy(void *dst, const void *src, size_t bytes, fcdp_stream stream)
try {
    if (!dst || !src) return fail(FCDP_EINVAL, "fcdp_probe_copy: NULL buffer");
    if (!aligned16(dst) || !aligned16(src)) return fail(FCDP_EALIGN, "fcdp_probe_copy: buffer not 16-byte aligned");
    if (bytes & 1) return fail(FCDP_EINVAL, "fcdp_probe_copy: bytes must be even");
    fcdp::PlainCopy shape;
    if (bytes) shape.ev = timing_events(FCDP_KERNEL_PROBE_COPY);
    hipError_t e = static_cast<hipError_t>(fcdp::launch_plain_copy(dst, src, bytes, stream, shape));
    if (e != hipSuccess) return hip_fail(e, "launch plain copy");
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_probe_copy: out of host memory");
}

fcdp_status fcdp_probe_reduce_stream(void *dst, const void *src, int32_t G, int64_t count,
                                     fcdp_dtype out, fcdp_stream stream)
try {
    const char *fn = "fcdp_probe_reduce_stream";
    if (!dst || !src) return fail(FCDP_EINVAL, std::string(fn) + ": NULL buffer");
    if (!aligned16(dst) || !aligned16(src)) return fail(FCDP_EALIGN, std::string(fn) + ": buffer not 16-byte aligned");
    if (G < 1) return fail(FCDP_EINVAL, std::string(fn) + ": G must be >= 1");
    if (G > FCDP_MAX_G) return fail(FCDP_ESIZE, std::string(fn) + ": G exceeds FCDP_MAX_G (64)");
    if (count < 0 || count % 1024) return fail(FCDP_EINVAL, std::string(fn) + ": count must be a non-negative multiple of 1024");
    if (out != FCDP_BF16 && out != FCDP_F32) return fail(FCDP_EINVAL, std::string(fn) + ": unknown dtype");
    const char *s0 = static_cast<const char *>(src), *d0 = static_cast<const char *>(dst);
    if (count > 0 && s0 < d0 + count * (out == FCDP_F32 ? 4 : 2) && d0 < s0 + static_cast<int64_t>(G) * count * 4)
        return fail(FCDP_EINVAL, std::string(fn) + ": dst overlaps src");
    hipError_t e = static_cast<hipError_t>(fcdp::launch_reduce_stream_calibration(
        dst, src, G, count, out, stream, count > 0 ? timing_events(FCDP_KERNEL_PROBE_STREAM) : fcdp::LaunchEvents()));
    if (e != hipSuccess) return hip_fail(e, "launch reduce calibration stream");
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_probe_reduce_stream: out of host memory");
}

fcdp_status fcdp_timing_enable(int32_t capacity)
try {
    if (capacity < 0 || capacity > (1 << 20)) return fail(FCDP_EINVAL, "fcdp_timing_enable: capacity must be in 0..2^20");
    TimingCtx *c = timing_ctx();
    if (!c) return fail(FCDP_EHIP, "fcdp_timing_enable: no current device");
    for (hipEvent_t e : c->pool) (void)hipEventDestroy(e);
    c->pool.clear();
    c->taken.clear();
    c->next = 0;
    c->on = false;
    if (capacity == 0) return FCDP_OK;
    c->pool.reserve(static_cast<size_t>(capacity) * 2);
    for (int32_t i = 0; i < capacity * 2; ++i) {
        hipEvent_t e;
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) return hip_fail(err, "hipEventCreate");
        c->pool.push_back(e);
    }
    c->on = true;
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_timing_enable: out of host memory");
}

fcdp_status fcdp_timing_collect(int32_t kind, int64_t *launches, double *total_ms)
try {
    if (!launches || !total_ms) return fail(FCDP_EINVAL, "fcdp_timing_collect: NULL output");
    *launches = 0;
    *total_ms = 0.0;
    TimingCtx *c = timing_ctx();
    if (!c) return fail(FCDP_EHIP, "fcdp_timing_collect: no current device");
    std::vector<TimedLaunch> keep;
    for (const TimedLaunch &t : c->taken) {
        if (t.kind != kind) {
            keep.push_back(t);
            continue;
        }
        FCDP_HIP(hipEventSynchronize(t.stop), "hipEventSynchronize");
        float ms = 0.f;
        FCDP_HIP(hipEventElapsedTime(&ms, t.start, t.stop), "hipEventElapsedTime");
        *total_ms += ms;
        *launches += 1;
    }
    c->taken.swap(keep);
    if (c->taken.empty()) c->next = 0; // every event is free again
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_timing_collect: out of host memory");
}

} // extern "C"
