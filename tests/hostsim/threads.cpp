// Two host threads issue data calls at the same time against the stand-in HIP
// runtime (device memory = host memory, a launch runs on the calling thread),
// built with ThreadSanitizer by tests/test_hostsim_sanitizers.py.  Each thread
// owns its staging buffer, tensors and gradient buffers, as the header asks;
// what they share is what the library says it guards: the per-device event
// ring, the staging-buffer table, the list of copies in flight and the link
// counters, plus one immutable layout.  A data race in the library's host
// code is a TSan report; wrong bytes are a non-zero exit.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "fcdp.h"

namespace {

constexpr int kT = 4, kG = 3, kIters = 200;
const int64_t kNumel[kT] = {3001, 64, 7777, 5};

int worker(const fcdp_layout *L, int id, const std::vector<uint16_t> &flat, void *host_cache, int *failures)
{
    const int64_t Np = fcdp_layout_padded_numel(L), S = fcdp_layout_shard_numel(L);
    const int64_t *off = fcdp_layout_offsets(L);
    std::vector<uint16_t> staging(Np), staging_slice(S), shards(flat);
    std::vector<std::vector<uint16_t>> tensors(kT);
    void *tptr[kT];
    const void *sptr[kG];
    for (int t = 0; t < kT; ++t) {
        tensors[t].assign(kNumel[t] + 8, 0);
        tptr[t] = tensors[t].data();
    }
    for (int r = 0; r < kG; ++r) sptr[r] = shards.data() + r * S;
    std::vector<float> p0(5000, 1.5f), p1(5000, 0.25f), out(5000);
    const void *pp[2] = {p0.data(), p1.data()};
    void *stream_a = reinterpret_cast<void *>(uintptr_t(0x1000 + id * 16)),
         *stream_b = reinterpret_cast<void *>(uintptr_t(0x2000 + id * 16));
    for (int it = 0; it < kIters; ++it) {
        fcdp_status st;
        switch (it % 5) {
        case 0:
            st = fcdp_materialize_layer(L, FCDP_SRC_HOST_DMA, nullptr, host_cache, staging.data(), tptr,
                                        FCDP_STORE_NONE, stream_a, stream_b);
            break;
        case 1:
            st = fcdp_materialize_layer(L, FCDP_SRC_HOST_SCATTER_DMA, nullptr, host_cache, nullptr, tptr,
                                        FCDP_STORE_NONE, stream_a, stream_b);
            break;
        case 2:
            st = fcdp_materialize_layer(L, FCDP_SRC_DEVICE_SHARDS, sptr, nullptr, nullptr, tptr,
                                        FCDP_STORE_NONE, stream_a, stream_b);
            break;
        case 3:
            st = fcdp_materialize_layer(L, FCDP_SRC_HOST_ZEROCOPY, nullptr, host_cache, nullptr, tptr,
                                        FCDP_STORE_NONE, stream_a, stream_b);
            break;
        default: // shard 1 from the host, the others from the device
            st = fcdp_materialize_layer_node_slice(L, 1, 1, sptr, static_cast<char *>(host_cache) + S * 2,
                                                   staging_slice.data(), tptr, stream_a, stream_b);
            break;
        }
        if (st != FCDP_OK) {
            std::printf("thread %d: call failed: %s\n", id, fcdp_last_error());
            ++*failures;
            return 1;
        }
        for (int t = 0; t < kT; ++t)
            if (std::memcmp(tensors[t].data(), flat.data() + off[t], kNumel[t] * 2) != 0) ++*failures;
        if (fcdp_reduce_grad_shard(pp, 2, 0, 5000, FCDP_F32, FCDP_F32, out.data(), stream_a) != FCDP_OK ||
            out[0] != 1.75f || out[4999] != 1.75f)
            ++*failures;
        int64_t stored = 0, fetched = 0;
        if (fcdp_link_bytes(0, &stored, &fetched) != FCDP_OK) ++*failures;
    }
    return 0;
}

} // namespace

int main()
{
    fcdp_layout *L = nullptr;
    if (fcdp_layout_build(kNumel, nullptr, kT, kG, 2, 64, &L) != FCDP_OK) return 2;
    if (fcdp_layout_prepare(L) != FCDP_OK) return 2;
    const int64_t Np = fcdp_layout_padded_numel(L);
    std::vector<uint16_t> flat(Np, 0);
    for (int64_t i = 0; i < fcdp_layout_numel(L); ++i) flat[i] = static_cast<uint16_t>(i * 31 + 5);
    void *host = nullptr, *alias = nullptr;
    if (fcdp_host_cache_alloc(static_cast<size_t>(Np) * 2, -1, &host, &alias) != FCDP_OK) return 2;
    std::memcpy(host, flat.data(), static_cast<size_t>(Np) * 2);
    if (fcdp_tuning_set("max_copies_in_flight", 1) != FCDP_OK) return 2; // every copy passes the back-pressure
    int64_t s0, f0;
    fcdp_link_bytes(1, &s0, &f0);
    int fail_a = 0, fail_b = 0;
    std::thread a(worker, L, 0, std::cref(flat), host, &fail_a);
    std::thread b(worker, L, 1, std::cref(flat), host, &fail_b);
    a.join();
    b.join();
    int64_t stored = 0, fetched = 0;
    fcdp_link_bytes(0, &stored, &fetched);
    // 3 of every 5 iterations fetch one padded image and 1 of 5 one shard, in both threads
    const int64_t want = 2LL * (kIters / 5) * (3 * Np * 2 + fcdp_layout_shard_numel(L) * 2);
    if (fetched != want) {
        std::printf("link counter lost updates: %lld, expected %lld\n", (long long)fetched, (long long)want);
        return 1;
    }
    fcdp_host_cache_free(host);
    fcdp_layout_destroy(L);
    if (fail_a || fail_b) {
        std::printf("wrong results: %d %d\n", fail_a, fail_b);
        return 1;
    }
    std::printf("threads ok\n");
    return 0;
}
