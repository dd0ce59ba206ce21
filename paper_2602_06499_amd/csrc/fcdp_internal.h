// Internal declarations shared by the host-side translation units of libfcdp.
#ifndef FCDP_INTERNAL_H
#define FCDP_INTERNAL_H

#include <cstdint>
#include <mutex>
#include <string>
#include <vector>

#include "fcdp.h"

namespace fcdp {

// One unit of copy work: nbytes bytes from buffer src_idx at byte offset
// src_off to buffer dst_idx at byte offset dst_off.  src_idx < 0 means "write
// zeros".  A piece never crosses a tensor, shard or chunk boundary, so every
// workgroup moves a bounded, nearly equal number of bytes.
struct Piece {
    int64_t src_off;
    int64_t dst_off;
    int32_t nbytes;
    int32_t src_idx;
    int32_t dst_idx;
    int32_t reserved;
};
static_assert(sizeof(Piece) == 32, "Piece must stay 32 bytes");

// Which side of a piece table indexes the (possibly long) per-tensor pointer
// list; the other side indexes the short list (shards, or a single buffer).
enum class TensorSide { Dst, Src, None };

struct PieceTable {
    std::vector<Piece> pieces;
    // For tables whose tensor side can exceed one launch's pointer window:
    // [win_begin[w], win_begin[w+1]) are the pieces whose tensor index lies in
    // window w (tensors [w*kTensorWindow, (w+1)*kTensorWindow)).
    std::vector<int64_t> win_begin;
};

constexpr int kTensorWindow = 256; // per-launch tensor pointers (kernarg)
constexpr int kMaxDevices = 16;

struct DeviceTables {
    int device = -1;
    Piece *unflatten = nullptr;
    Piece *flatten = nullptr;
    Piece *pack = nullptr;
    Piece *unpack = nullptr;
};

struct Segment {
    int64_t t, r, dst_off, src_off, len;
};

} // namespace fcdp

struct fcdp_layout {
    int32_t T = 0, G = 1, esz = 2, q = 64;
    int64_t N = 0, N_pad = 0, S = 0, N_t = 0, N_packed = 0;
    int64_t chunk_bytes = 0;
    std::vector<int64_t> numel, off;
    std::vector<uint8_t> trainable;
    std::vector<fcdp::Segment> segments;
    fcdp::PieceTable unflatten, flatten, pack, unpack;
    // device copies, filled lazily per device
    mutable std::mutex mu;
    mutable std::vector<fcdp::DeviceTables> dev;
};

namespace fcdp {

void set_error(const std::string &msg);
const std::string &last_error_ref();
fcdp_status fail(fcdp_status st, const std::string &msg);
// for catch-all handlers at the C boundary: records msg if that is possible
// without throwing, and returns st
fcdp_status fail_noexcept(fcdp_status st, const char *msg) noexcept;

// tuning knobs (see fcdp_tuning_set)
struct Tuning {
    // Measured best on MI355X (Llama 7B/13B/70B-shaped layers): many small
    // workgroups, two 16-byte vectors per lane, non-temporal access.
    int64_t copy_chunk_bytes = 4096;  // piece size cap; multiple of 4096
    int64_t copy_block = 128;         // threads per workgroup: 64..1024
    int64_t copy_unroll = 1;          // 16-byte vectors in flight per thread
    int64_t copy_wg_per_cu = 0;       // 0 = one workgroup per piece
    int64_t copy_nt = 3;              // non-temporal: bit 0 loads, bit 1 stores
    // kernels whose loads or stores cross the host link (zero-copy fetch and
    // store): a bounded number of workgroups keeps enough bytes in flight for
    // the link and leaves the rest of the GPU to other work; 0 = no bound
    int64_t link_max_wgs = 64;
    int64_t link_block = 256;
    int64_t link_chunk_bytes = 16384; // bytes per workgroup iteration (store)
    // most host-link copies (DMA stores and fetches) in flight per device; a
    // call that would exceed it first waits on the host for the oldest one.
    // Measured on MI355X / ROCm 7: with up to 4 large pinned copies queued
    // both directions run at the full link rate; from 6 on the stores fall
    // to 20-30 GB/s.  2 is also the depth double buffering needs.  0 = off
    int64_t max_copies_in_flight = 2;
    int64_t reduce_block = 64;
    // The phased reduce (persistent waves keep their sums in registers and
    // store them after the last load of a phase) against one tile per
    // workgroup, stored as soon as it is summed: 0 never phased, 1 phased
    // whenever the slices are 16-byte aligned and long enough, 2 phased where
    // it measured faster (by G and the two element types)
    int64_t reduce_phased = 2;
    // waves per SIMD of the phased kernel: 0 by rule (one when every load group
    // is full, two otherwise), 1 or 2 forced (1 falls back to 2 for other G)
    int64_t reduce_phase_waves = 0;
    int64_t reduce_phase_rotate = 1;
    // debugging aid, off by default (the environment variable FCDP_DEBUG_POISON=1
    // turns it on at load): outputs are filled with kPoison before the work that
    // writes them is enqueued, so a consumer that misses a wait reads poison
    // instead of stale bytes that happen to be right
    int64_t debug_poison = 0;
};
constexpr uint16_t kPoison = 0x7FC1; // a bf16 NaN; 0x7FC17FC1 is an fp32 NaN
Tuning &tuning();

// host-side table construction (fcdp_layout.cpp)
fcdp_status build_tables(fcdp_layout *L);

// Timing events attached to one kernel dispatch (both null = untimed).  They
// take the dispatch's own start and end timestamps, not those of barrier
// packets around it.
struct LaunchEvents {
    void *start = nullptr; // hipEvent_t
    void *stop = nullptr;
};

// kernel launchers (fcdp_kernels.hip).  All return a hipError_t as int.
struct CopyLaunch {
    const Piece *pieces = nullptr;  // device
    int64_t n_pieces = 0;
    TensorSide tensor_side = TensorSide::None;
    int32_t tensor_base = 0;        // first tensor index of this window
    const void *const *small_ptrs = nullptr; // host array, n_small entries
    int32_t n_small = 0;
    const void *const *tensor_ptrs = nullptr; // host array (window start)
    int32_t n_tensor = 0;
    bool nt = true;
    int64_t wg_per_cu = 0;
    int64_t max_wgs = 0;            // absolute cap on workgroups, 0 = none
    int64_t block = 0;              // threads per workgroup, 0 = copy_block
    LaunchEvents ev;                // optional start/stop timing events
};
int launch_copy(const CopyLaunch &c, void *stream);
int launch_reduce(const void *const *partials, int32_t G, int64_t elem_offset,
                  int64_t count, int in_dtype, int out_dtype, float scale, void *out,
                  void *stream, const LaunchEvents &ev = LaunchEvents());
struct PlainCopy {
    int64_t chunk = 0, block = 0, unroll = 0, max_wgs = 0; // 0 = the copy_* knobs
    int nt = -1;                                           // -1 = copy_nt
    LaunchEvents ev;
};
// Rank-order reduction over a few runs: run k sums `count[k]` elements that
// start at element src_off[k] of every partial into out + dst_off[k]; a run
// with src_off < 0 writes zeros.
constexpr int kMaxReduceRuns = 32;
struct ReduceRuns {
    int32_t n_runs = 0;
    int64_t src_off[kMaxReduceRuns];
    int64_t dst_off[kMaxReduceRuns];
    int64_t count[kMaxReduceRuns];
};
int launch_reduce_runs(const void *const *partials, int32_t G, const ReduceRuns &runs,
                       int in_dtype, int out_dtype, float scale, void *out, void *stream,
                       const LaunchEvents &ev = LaunchEvents());
int launch_reduce_stream_calibration(void *dst, const void *src, int32_t G, int64_t count,
                                     int out_dtype, void *stream, const LaunchEvents &ev = LaunchEvents());
int launch_plain_copy(void *dst, const void *src, size_t bytes, void *stream,
                      const PlainCopy &shape = PlainCopy());
// dst 16-byte aligned, bytes even; max_wgs 0 = up to 16384 workgroups
int launch_fill(void *dst, size_t bytes, uint16_t pattern, void *stream, int64_t max_wgs = 0);
int device_cu_count();
// What the last launch_reduce of the process used: 0 one tile per workgroup,
// 1 or 2 the phased kernel with that many waves per SIMD.
int last_reduce_shape();

} // namespace fcdp
#endif
