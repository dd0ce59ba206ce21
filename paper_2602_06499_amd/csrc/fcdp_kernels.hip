// HIP kernels of libfcdp for gfx950 (MI355X) and their launchers.
//
//   copy_pieces  -- the scatter/gather engine behind unflatten (shards ->
//                   tensors, from HBM or straight from mapped host memory),
//                   flatten, pack and unpack.  Pure byte movement, bound by
//                   HBM (or by the host link when the source is host memory).
//   reduce_ranks -- rank-order fp32 sum of G partial gradient slices with an
//                   optional bf16 (nearest-even) store.  Bound by HBM reads.
//   reduce_runs  -- the same sum over the trainable ranges of G unpacked flat
//                   gradients, written in packed order (pack and reduce in
//                   one launch); launch-bound at PEFT sizes.
//   plain_copy   -- contiguous copy with the same inner loop; the known-size
//                   reference for counter calibration.
//   fill_pattern -- 16-bit pattern fill behind the debug poison.
//
// Nothing here is a contraction, so no MFMA and no LDS staging: every byte is
// read once and written once, there is no reuse to stage.  What matters is
// 16-byte coalesced access per lane, enough independent loads in flight per
// wave to cover HBM latency, and equal bytes per workgroup.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <atomic>
#include <cstdint>

#include "fcdp_internal.h"

namespace fcdp {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// 16-byte vectors that are only 4- or 2-byte aligned: the compiler picks the
// widest access the target allows for that alignment.
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 u32x2_a2 __attribute__((aligned(2)));

constexpr int kMaxSmall = FCDP_MAX_G;

// All buffer pointers of one launch sit in a single table: entries
// [0, kMaxSmall) are the short list (shards, or flat/packed), entries from
// kMaxSmall on are the tensor window.  A piece's indices are turned into
// table slots by adding src_bias / dst_bias, which the host sets per launch,
// so the kernel selects its two pointers without any branch on the kind of
// copy.  (A three-way branch here was compiled to code that left the
// destination pointer unset on one path.)
struct CopyArgs {
    const Piece *pieces;
    int64_t n_pieces;
    int32_t src_bias;
    int32_t dst_bias;
    char *ptrs[kMaxSmall + kTensorWindow];
};

// Loads 16 bytes from an address that is ALIGN-byte aligned (16, 4 or 2).
// The under-aligned typedefs are named here directly: a typedef's alignment
// does not survive being passed as a template type argument.
template <int ALIGN, bool NT>
__device__ __forceinline__ u32x4 load16(const char *p)
{
    if constexpr (ALIGN >= 16) {
        const u32x4 *vp = reinterpret_cast<const u32x4 *>(p);
        if constexpr (NT) return __builtin_nontemporal_load(vp);
        else return *vp;
    } else if constexpr (ALIGN >= 4) {
        const u32x4_a4 *vp = reinterpret_cast<const u32x4_a4 *>(p);
        u32x4_a4 v;
        if constexpr (NT) v = __builtin_nontemporal_load(vp);
        else v = *vp;
        return u32x4{v.x, v.y, v.z, v.w};
    } else {
        const u32x4_a2 *vp = reinterpret_cast<const u32x4_a2 *>(p);
        u32x4_a2 v;
        if constexpr (NT) v = __builtin_nontemporal_load(vp);
        else v = *vp;
        return u32x4{v.x, v.y, v.z, v.w};
    }
}

template <bool NT>
__device__ __forceinline__ void store16(char *p, u32x4 v)
{
    u32x4 *vp = reinterpret_cast<u32x4 *>(p);
    if constexpr (NT)
        __builtin_nontemporal_store(v, vp);
    else
        *vp = v;
}

// Copies nvec 16-byte vectors from s to d; d is 16-byte aligned, s is
// ALIGN-byte aligned.  UNROLL independent loads are issued per thread before the
// first store.
// HINT: bit 0 = non-temporal loads, bit 1 = non-temporal stores.
template <int ALIGN, int UNROLL, int HINT>
__device__ __forceinline__ void copy_body(const char *s, char *d, uint32_t nvec,
                                          uint32_t tid, uint32_t nthreads)
{
    const uint32_t step = nthreads * UNROLL;
    uint32_t base = 0;
    for (; base + step <= nvec; base += step) {
        u32x4 r[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            r[u] = load16<ALIGN, (HINT & 1) != 0>(s + (size_t)(base + u * nthreads + tid) * 16);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            store16<(HINT & 2) != 0>(d + (size_t)(base + u * nthreads + tid) * 16, r[u]);
    }
    if (base < nvec) {
        u32x4 r[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t i = base + u * nthreads + tid;
            if (i < nvec) r[u] = load16<ALIGN, (HINT & 1) != 0>(s + (size_t)i * 16);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t i = base + u * nthreads + tid;
            if (i < nvec) store16<(HINT & 2) != 0>(d + (size_t)i * 16, r[u]);
        }
    }
}

template <int UNROLL, int HINT>
__device__ __forceinline__ void zero_body(char *d, uint32_t nvec, uint32_t tid,
                                          uint32_t nthreads)
{
    for (uint32_t i = tid; i < nvec; i += nthreads)
        store16<(HINT & 2) != 0>(d + (size_t)i * 16, u32x4{0u, 0u, 0u, 0u});
}

// One piece: n bytes (even), s and d both at least 2-byte aligned.
template <int UNROLL, int HINT>
__device__ __forceinline__ void copy_piece(const char *s, char *d, uint32_t n,
                                           bool zero, uint32_t tid,
                                           uint32_t nthreads)
{
    // head: 2-byte units until d reaches a 16-byte boundary
    uint32_t head = static_cast<uint32_t>((16u - (reinterpret_cast<uintptr_t>(d) & 15u)) & 15u);
    if (head > n) head = n;
    if (tid < (head >> 1)) {
        uint16_t v = zero ? uint16_t(0) : reinterpret_cast<const uint16_t *>(s)[tid];
        reinterpret_cast<uint16_t *>(d)[tid] = v;
    }
    s += head;
    d += head;
    n -= head;
    const uint32_t nvec = n >> 4;
    if (zero) {
        zero_body<UNROLL, HINT>(d, nvec, tid, nthreads);
    } else {
        const uint32_t mis = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(s) & 15u);
        if (mis == 0)
            copy_body<16, UNROLL, HINT>(s, d, nvec, tid, nthreads);
        else if ((mis & 3u) == 0)
            copy_body<4, UNROLL, HINT>(s, d, nvec, tid, nthreads);
        else
            copy_body<2, UNROLL, HINT>(s, d, nvec, tid, nthreads);
    }
    // tail: the last n % 16 bytes, 2-byte units
    const uint32_t done = nvec << 4;
    const uint32_t tail = n - done;
    if (tid < (tail >> 1)) {
        uint16_t v = zero ? uint16_t(0)
                          : reinterpret_cast<const uint16_t *>(s + done)[tid];
        reinterpret_cast<uint16_t *>(d + done)[tid] = v;
    }
}

template <int UNROLL, int HINT>
__global__ void copy_pieces(const CopyArgs a)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t nthreads = blockDim.x;
    for (int64_t pi = blockIdx.x; pi < a.n_pieces; pi += gridDim.x) {
        // The table is written by the host before the launch and never by a
        // kernel, so it may be read through the constant address space: the
        // 32-byte record then arrives by one scalar load, straight into the
        // scalar registers that the pointer look-ups and the address
        // arithmetic below use (measured: 0.8-1.3 % on the large layers, the
        // whole gap to a plain copy; a vector load plus seven readfirstlanes
        // before).
        typedef const Piece __attribute__((address_space(4))) *ConstPiece;
        const ConstPiece cp = (ConstPiece)(uintptr_t)(a.pieces + pi);
        const int32_t src_idx = cp->src_idx;
        const int32_t dst_idx = cp->dst_idx;
        const int64_t src_off = cp->src_off;
        const int64_t dst_off = cp->dst_off;
        const uint32_t nbytes = static_cast<uint32_t>(cp->nbytes);
        const bool zero = src_idx < 0;
        char *d = a.ptrs[dst_idx + a.dst_bias] + dst_off;
        // a zero-fill piece reads nothing: point its source at slot 0, unused
        const char *s = a.ptrs[zero ? 0 : src_idx + a.src_bias] + src_off;
        copy_piece<UNROLL, HINT>(s, d, nbytes, zero, tid, nthreads);
    }
}

struct PlainArgs {
    const char *src;
    char *dst;
    size_t bytes;
    size_t n_chunks; // ceil(bytes / chunk), from the host (no 64-bit division in the kernel)
    uint32_t chunk;
};

template <int UNROLL, int HINT>
__global__ void plain_copy(const PlainArgs a)
{
    for (size_t c = blockIdx.x; c < a.n_chunks; c += gridDim.x) {
        const size_t o = c * a.chunk;
        const uint32_t n = static_cast<uint32_t>(a.bytes - o < a.chunk ? a.bytes - o : a.chunk);
        copy_piece<UNROLL, HINT>(a.src + o, a.dst + o, n, false, threadIdx.x, blockDim.x);
    }
}

// Fills a 16-byte aligned buffer of an even number of bytes with a repeated
// 16-bit pattern (the debug poison).
struct FillArgs {
    char *dst;
    size_t bytes;
    uint32_t pattern; // the 16-bit pattern in both halves
};

__global__ void __launch_bounds__(256) fill_pattern(const FillArgs a)
{
    const size_t nvec = a.bytes >> 4;
    const u32x4 v{a.pattern, a.pattern, a.pattern, a.pattern};
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < nvec; i += stride)
        reinterpret_cast<u32x4 *>(a.dst)[i] = v;
    const size_t t = (nvec << 4) + 2 * static_cast<size_t>(threadIdx.x);
    if (blockIdx.x == 0 && t < a.bytes)
        *reinterpret_cast<uint16_t *>(a.dst + t) = static_cast<uint16_t>(a.pattern);
}

// ------------------------------------------------------------------ reduce

struct ReduceArgs {
    const char *p[FCDP_MAX_G]; // already offset to the slice start
    char *out;
    int64_t count;
    int32_t G;
    float scale; // multiplies the finished sum; 1.0f leaves every value as it is
    int32_t spp;    // phased kernel: steps per wave
    int32_t rotate; // phased kernel: start each full run at step w mod spp
};

__device__ __forceinline__ uint32_t bf16_rne_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Loads four consecutive elements of partial g as fp32.
template <bool IN_F32, bool ALIGNED, bool NT>
__device__ __forceinline__ void load4(const char *base, int64_t vec, float (&v)[4])
{
    if constexpr (IN_F32) {
        const char *p = base + vec * 16;
        u32x4 r;
        r = load16<ALIGNED ? 16 : 4, NT>(p);
        v[0] = __uint_as_float(r.x);
        v[1] = __uint_as_float(r.y);
        v[2] = __uint_as_float(r.z);
        v[3] = __uint_as_float(r.w);
    } else {
        const char *p = base + vec * 8;
        u32x2 r;
        if constexpr (ALIGNED) {
            const u32x2 *vp = reinterpret_cast<const u32x2 *>(p);
            if constexpr (NT) r = __builtin_nontemporal_load(vp);
            else r = *vp;
        } else {
            const u32x2_a2 *vp = reinterpret_cast<const u32x2_a2 *>(p);
            u32x2_a2 t = *vp;
            r = u32x2{t.x, t.y};
        }
        v[0] = __uint_as_float(r.x << 16);
        v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16);
        v[3] = __uint_as_float(r.y & 0xffff0000u);
    }
}

template <bool OUT_F32, bool NT>
__device__ __forceinline__ void store4(char *out, int64_t vec, const float (&a)[4])
{
    if constexpr (OUT_F32) {
        u32x4 r{__float_as_uint(a[0]), __float_as_uint(a[1]),
                __float_as_uint(a[2]), __float_as_uint(a[3])};
        store16<NT>(out + vec * 16, r);
    } else {
        u32x2 r{bf16_rne_bits(a[0]) | (bf16_rne_bits(a[1]) << 16),
                bf16_rne_bits(a[2]) | (bf16_rne_bits(a[3]) << 16)};
        u32x2 *vp = reinterpret_cast<u32x2 *>(out + vec * 8);
        if constexpr (NT) __builtin_nontemporal_store(r, vp);
        else *vp = r;
    }
}

#ifndef FCDP_REDUCE_UNROLL
#define FCDP_REDUCE_UNROLL 4 // 4-element vectors per thread
#endif
#ifndef FCDP_REDUCE_NT
#define FCDP_REDUCE_NT 1     // non-temporal loads
#endif
#ifndef FCDP_REDUCE_NT_STORE
#define FCDP_REDUCE_NT_STORE 1 // non-temporal stores
#endif
constexpr int kGroup = 8;    // partials loaded back to back before their adds
constexpr int kReduceUnroll = FCDP_REDUCE_UNROLL;
constexpr bool kReduceNT = FCDP_REDUCE_NT != 0;
constexpr bool kReduceNTStore = FCDP_REDUCE_NT_STORE != 0;

// Adds partials g0 .. g0+K-1 to acc, strictly in that order.  All K*UNROLL
// loads are issued before the first add.
template <int K, bool IN_F32, bool ALIGNED, int UNROLL, bool NT>
__device__ __forceinline__ void add_group(const ReduceArgs &a, int g0,
                                          const int64_t (&idx)[UNROLL],
                                          float (&acc)[UNROLL][4])
{
    float v[K][UNROLL][4];
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            load4<IN_F32, ALIGNED, NT>(a.p[g0 + k], idx[u], v[k][u]);
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[u][c] = acc[u][c] + v[k][u][c];
}

// One tile = blockDim.x * UNROLL vectors of four elements starting at b0.
// GUARD tiles (the last, partial one) clamp their load index to the last
// vector and skip the stores beyond it, so no load is predicated.
template <bool GUARD, int REM, bool IN_F32, bool OUT_F32, bool ALIGNED, int UNROLL, bool NT>
__device__ __forceinline__ void reduce_tile(const ReduceArgs &a, int64_t b0, int64_t nvec)
{
    int64_t idx[UNROLL], lidx[UNROLL];
    float acc[UNROLL][4];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        idx[u] = b0 + static_cast<int64_t>(u) * blockDim.x + threadIdx.x;
        lidx[u] = GUARD ? (idx[u] < nvec ? idx[u] : nvec - 1) : idx[u];
        // -0.0f is the identity of IEEE addition for every value including
        // -0.0f itself, so "acc = -0 + p_0" equals "acc = p_0" bit for bit
        // and rank 0 needs no special case.
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[u][c] = -0.0f;
    }
    const int full = a.G - REM;
    for (int g = 0; g < full; g += kGroup)
        add_group<kGroup, IN_F32, ALIGNED, UNROLL, NT>(a, g, lidx, acc);
    if constexpr (REM > 0)
        add_group<REM, IN_F32, ALIGNED, UNROLL, NT>(a, full, lidx, acc);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[u][c] = acc[u][c] * a.scale;
        if (!GUARD || idx[u] < nvec) store4<OUT_F32, kReduceNTStore>(a.out, idx[u], acc[u]);
    }
}

// REM = G mod kGroup is a template parameter, so the rank loop is a counted
// loop of full groups plus one fixed-size group: no data-dependent branch
// sits between the loads and the adds.  The adds run strictly in rank
// order, one binary32 rounding each; the result does not depend on the
// launch shape.
template <int REM, bool IN_F32, bool OUT_F32, bool ALIGNED, int UNROLL, bool NT>
__global__ void __launch_bounds__(256) reduce_ranks(const ReduceArgs a)
{
    const int64_t nvec = a.count >> 2;
    const int64_t per_block = static_cast<int64_t>(blockDim.x) * UNROLL;
    for (int64_t b0 = static_cast<int64_t>(blockIdx.x) * per_block; b0 < nvec;
         b0 += static_cast<int64_t>(gridDim.x) * per_block) {
        if (b0 + per_block <= nvec)
            reduce_tile<false, REM, IN_F32, OUT_F32, ALIGNED, UNROLL, NT>(a, b0, nvec);
        else
            reduce_tile<true, REM, IN_F32, OUT_F32, ALIGNED, UNROLL, NT>(a, b0, nvec);
    }
    // the last count % 4 elements, one thread each
    const int64_t k = (nvec << 2) + threadIdx.x;
    if (blockIdx.x == 0 && k < a.count) {
        float acc = -0.0f;
        for (int g = 0; g < a.G; ++g) {
            float v;
            if constexpr (IN_F32)
                v = reinterpret_cast<const float *>(a.p[g])[k];
            else
                v = __uint_as_float(static_cast<uint32_t>(
                        reinterpret_cast<const uint16_t *>(a.p[g])[k]) << 16);
            acc = acc + v;
        }
        acc = acc * a.scale;
        if constexpr (OUT_F32)
            reinterpret_cast<float *>(a.out)[k] = acc;
        else
            reinterpret_cast<uint16_t *>(a.out)[k] =
                static_cast<uint16_t>(bf16_rne_bits(acc));
    }
}

// ---- calibration stream for the reduce ----------------------------------
// The reduce's G : 1 mix of reads and writes from ONE contiguous buffer: tile
// t (1024 elements of output, one workgroup of 64 threads, four vectors per
// lane as in reduce_ranks) sums the G consecutive 4 KiB sub-tiles that start
// at element t * G * 1024 of src, in order, and stores the tile as soon as it
// is summed.  Same loads, adds and stores per output element as reduce_ranks;
// what differs is the address pattern (one stream instead of G), so its rate
// is the ceiling of that kernel design for a given G.
struct StreamArgs {
    const char *src;
    char *out;
    int64_t tiles;
    int32_t G;
};

template <bool OUT_F32>
__global__ void __launch_bounds__(64) reduce_stream_calibration(const StreamArgs a)
{
    constexpr int kVecPerTile = 256; // 64 lanes x 4 vectors
    for (int64_t t = blockIdx.x; t < a.tiles; t += gridDim.x) {
        float acc[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[u][c] = -0.0f;
        const char *base = a.src + t * a.G * (kVecPerTile * 16);
        for (int g0 = 0; g0 < a.G; g0 += kGroup) {
            float v[kGroup][4][4];
#pragma unroll
            for (int k = 0; k < kGroup; ++k) {
                const int g = g0 + k < a.G ? g0 + k : a.G - 1; // clamp: the load is issued, the add is not
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    load4<true, true, kReduceNT>(base + static_cast<int64_t>(g) * (kVecPerTile * 16),
                                                 u * 64 + threadIdx.x, v[k][u]);
            }
#pragma unroll
            for (int k = 0; k < kGroup; ++k)
                if (g0 + k < a.G)
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[u][c] = acc[u][c] + v[k][u][c];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            store4<OUT_F32, kReduceNTStore>(a.out, t * kVecPerTile + u * 64 + threadIdx.x, acc[u]);
    }
}

// ---- phased reduce: reads and writes kept apart in time -------------------
// Measured on MI355X: a read stream of G partials runs at 7.0 TB/s, and the
// same stream with the output written as it is produced at 6.0 TB/s, although
// the output is only 3-11 % of the bytes: stores that trickle into a
// read-dominated stream cost the memory system far more than their bytes.
// Here the whole chip reads for a while and then writes for a while.  The
// grid is persistent: ONE wave per SIMD, all resident at once, and every
// wave owns one contiguous run of steps (a step = 64 lanes x one 16-byte
// unit of each partial).  A wave sums up to 104 steps of every
// partial, keeps the finished sums in registers (4 per fp32 step and lane;
// with one wave per SIMD a lane has 512 registers, 256 of them accumulation
// registers that the compiler uses as backing store) and stores them only
// after its last load of the phase.  All waves have the same work, so they
// reach their stores at about the same time and the stores arrive at the
// memory as one burst.  With 104 steps one launch holds 1024 waves x
// 104 KiB = 109 MB of fp32 sums on a 256-CU part, i.e. the whole shard of
// every Llama-shaped layer here; longer inputs take several launches.  Fewer,
// fatter waves measured faster at every step of the way (G = 32, fp32 out,
// fraction of the HBM peak): 16 steps at four waves per SIMD 0.80, 24 at
// three 0.83, 48 at two 0.85, 96 at one 0.87; so did a contiguous run per
// wave against steps dealt round robin.  The adds per element stay in rank
// order, one wave and lane owns an element from its first load to its
// store, and the launch shape changes nothing in the result.
// Two shapes of the same kernel are built: one wave per SIMD holding 104 steps
// (416 sums per lane), and two waves per SIMD holding 52 steps each.  The
// first is the faster one when every load group is full (G a multiple of 8):
// with a single wave on a SIMD nothing hides the round trip of a short last
// group (measured at a 25 M-element shard: G = 16 0.85 of the peak, G = 9 0.74,
// G = 1 0.33), which the second wave of the other shape does.
constexpr int kPhasedBlock = 256;                          // four waves
constexpr int kPhaseSteps1 = 104, kPhaseSteps2 = 52;       // steps of 4 elements per lane held per phase
constexpr int kPhasedMinStepsPerWave = 8; // below this the one-tile-per-workgroup kernel is used
constexpr int kPhasedGroup = 8; // partials loaded back to back before their adds (4 or 6 measured 1-3 % slower)

// One lane's share of a step: 16 bytes of one partial = E elements (4 fp32
// or 8 bf16), widened to fp32 only when they are added, so that the loads of
// a group wait in 4 registers each.
template <bool IN_F32>
__device__ __forceinline__ void widen_unit(const u32x4 r, float (&v)[IN_F32 ? 4 : 8])
{
    if constexpr (IN_F32) {
        v[0] = __uint_as_float(r.x);
        v[1] = __uint_as_float(r.y);
        v[2] = __uint_as_float(r.z);
        v[3] = __uint_as_float(r.w);
    } else {
        v[0] = __uint_as_float(r.x << 16);
        v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16);
        v[3] = __uint_as_float(r.y & 0xffff0000u);
        v[4] = __uint_as_float(r.z << 16);
        v[5] = __uint_as_float(r.z & 0xffff0000u);
        v[6] = __uint_as_float(r.w << 16);
        v[7] = __uint_as_float(r.w & 0xffff0000u);
    }
}

// The loads of partials g0 .. g0+K-1 of one unit, issued back to back.
template <int K, bool NT>
__device__ __forceinline__ void issue_group(const ReduceArgs &a, int g0, int64_t unit,
                                            u32x4 (&r)[K])
{
#pragma unroll
    for (int k = 0; k < K; ++k) r[k] = load16<16, NT>(a.p[g0 + k] + unit * 16);
}

// Adds the K loaded partials to acc in their order.
template <int K, bool IN_F32>
__device__ __forceinline__ void consume_group(const u32x4 (&r)[K], float (&acc)[IN_F32 ? 4 : 8])
{
    constexpr int E = IN_F32 ? 4 : 8;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        float v[E];
        widen_unit<IN_F32>(r[k], v);
#pragma unroll
        for (int c = 0; c < E; ++c) acc[c] = acc[c] + v[c];
    }
}

// Adds partials g0 .. g0+K-1 of one unit to acc in that order; the K loads
// are issued before the first add.
template <int K, bool IN_F32, bool NT>
__device__ __forceinline__ void add_group1(const ReduceArgs &a, int g0, int64_t unit,
                                           float (&acc)[IN_F32 ? 4 : 8])
{
    u32x4 r[K];
    issue_group<K, NT>(a, g0, unit, r);
    consume_group<K, IN_F32>(r, acc);
}

// What a lane holds of a step until the phase's stores.  For fp32 output
// these are the sums themselves, added up in place and scaled at the store.
// For bf16 output they are the scaled sums already rounded, two to a word:
// half the registers, and the rounding arithmetic is done while loads are in
// flight instead of in front of the stores.
template <bool OUT_F32, int E>
struct HeldUnit;
template <int E>
struct HeldUnit<true, E> {
    float f[E];
};
template <int E>
struct HeldUnit<false, E> {
    uint32_t w[E / 2];
};

// Where the sums of the step in progress are added up: in place for fp32
// output, in a temporary for bf16 output.
template <int E>
__device__ __forceinline__ float (&sums_of(HeldUnit<true, E> &h, float (&)[E]))[E] { return h.f; }
template <int E>
__device__ __forceinline__ float (&sums_of(HeldUnit<false, E> &, float (&t)[E]))[E] { return t; }

// A finished step's sums into their held form (nothing to do for fp32).
template <int E>
__device__ __forceinline__ void finish_unit(const float (&)[E], float, HeldUnit<true, E> &) {}
template <int E>
__device__ __forceinline__ void finish_unit(const float (&t)[E], float scale, HeldUnit<false, E> &h)
{
#pragma unroll
    for (int c = 0; c < E / 2; ++c)
        h.w[c] = bf16_rne_bits(t[2 * c] * scale) | (bf16_rne_bits(t[2 * c + 1] * scale) << 16);
}

// Plain stores: with all stores of the chip in one burst they measured 1-2 %
// faster than non-temporal ones.
template <int E>
__device__ __forceinline__ void store_held(char *out, int64_t unit, float scale,
                                           const HeldUnit<true, E> &h)
{
#pragma unroll
    for (int q = 0; q < E / 4; ++q)
        store16<false>(out + unit * (E * 4) + q * 16,
                       u32x4{__float_as_uint(h.f[4 * q] * scale), __float_as_uint(h.f[4 * q + 1] * scale),
                             __float_as_uint(h.f[4 * q + 2] * scale),
                             __float_as_uint(h.f[4 * q + 3] * scale)});
}
template <int E>
__device__ __forceinline__ void store_held(char *out, int64_t unit, float,
                                           const HeldUnit<false, E> &h)
{
    if constexpr (E == 4)
        *reinterpret_cast<u32x2 *>(out + unit * 8) = u32x2{h.w[0], h.w[1]};
    else
        store16<false>(out + unit * 16, u32x4{h.w[0], h.w[1], h.w[2], h.w[3]});
}

// Needs 16-byte aligned input slices and output (the launcher falls back to
// reduce_ranks otherwise).  A unit is 16 bytes of input = E elements; a step
// is 64 units, one per lane; a wave holds up to STEPS = STEPS4 * 4 / E
// steps, i.e. at most STEPS4 * 4 words per lane whatever the types.  WPE =
// waves per SIMD the register budget is cut for (1: 512 registers, 2: 256).
// For bf16 output a step's sums are scaled and rounded while the first loads
// of the next step are in flight, so that this arithmetic, like the adds,
// runs under memory latency and only the stores are left for the end (at one
// wave per SIMD and G = 8 that alone is 0.73 -> 0.83 of the HBM peak).
template <int STEPS4, int WPE, int REM, bool IN_F32, bool OUT_F32, bool NT>
__global__ void __launch_bounds__(kPhasedBlock, WPE) // threads, waves per SIMD
reduce_phased(const ReduceArgs a)
{
    constexpr int E = IN_F32 ? 4 : 8;
    constexpr int STEPS = STEPS4 * 4 / E;
    constexpr int K0 = REM > 0 ? REM : kPhasedGroup; // the first group when no group is full
    const int64_t n_units = a.count / E;
    const int64_t n_steps = (n_units + 63) >> 6;
    const int64_t w = static_cast<int64_t>(blockIdx.x) * (kPhasedBlock / 64) +
                      __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
    const int lane = static_cast<int>(threadIdx.x & 63u);
    const int full = a.G - REM; // REM = G mod kPhasedGroup
    {
        // this wave's run: steps [s0, s0 + spp)
        const int64_t s0 = w * a.spp;
        // A wave whose whole run exists may start it at step w mod spp and wrap around
        // (the launcher asks for that where equal positions in every run would make the
        // chip read a comb of addresses that the memory maps badly).
        const int rot = (a.rotate && s0 + a.spp <= n_steps)
                            ? static_cast<int>(static_cast<uint32_t>(w) % static_cast<uint32_t>(a.spp)) : 0;
        HeldUnit<OUT_F32, E> held[STEPS];
        float tmp[2][E]; // bf16 output: the sums of the step in progress and of the one before it
#pragma unroll
        for (int j = 0; j <= STEPS; ++j) {
            const int64_t s = s0 + (j + rot < a.spp ? j + rot : j + rot - a.spp);
            // the same for every lane of the wave; an active step follows active steps only
            // (a rotated run is active throughout)
            const bool active = j < STEPS && j < a.spp && s < n_steps;
            const bool prev_active = j > 0 && (j - 1) < a.spp && (rot != 0 || s0 + j - 1 < n_steps);
            if (active) {
                const int64_t idx = (s << 6) + lane;
                // the last step may be partial: clamp the load index, skip the store
                const int64_t lidx = idx < n_units ? idx : n_units - 1;
                float (&cur)[E] = sums_of<E>(held[j < STEPS ? j : 0], tmp[j & 1]);
                if constexpr (OUT_F32) {
#pragma unroll
                    for (int c = 0; c < E; ++c) cur[c] = -0.0f; // the identity of IEEE addition, also for -0
                    for (int g = 0; g < full; g += kPhasedGroup)
                        add_group1<kPhasedGroup, IN_F32, NT>(a, g, lidx, cur);
                    if constexpr (REM > 0) add_group1<REM, IN_F32, NT>(a, full, lidx, cur);
                } else if (REM == 0 || full > 0) {
                    // the step before is rounded between the first loads of this one and their adds
                    u32x4 r[kPhasedGroup];
                    issue_group<kPhasedGroup, NT>(a, 0, lidx, r);
                    if (j > 0) finish_unit<E>(tmp[(j - 1) & 1], a.scale, held[j > 0 ? j - 1 : 0]);
#pragma unroll
                    for (int c = 0; c < E; ++c) cur[c] = -0.0f;
                    consume_group<kPhasedGroup, IN_F32>(r, cur);
                    for (int g = kPhasedGroup; g < full; g += kPhasedGroup)
                        add_group1<kPhasedGroup, IN_F32, NT>(a, g, lidx, cur);
                    if constexpr (REM > 0) add_group1<REM, IN_F32, NT>(a, full, lidx, cur);
                } else {
                    u32x4 r[K0];
                    issue_group<K0, NT>(a, 0, lidx, r);
                    if (j > 0) finish_unit<E>(tmp[(j - 1) & 1], a.scale, held[j > 0 ? j - 1 : 0]);
#pragma unroll
                    for (int c = 0; c < E; ++c) cur[c] = -0.0f;
                    consume_group<K0, IN_F32>(r, cur);
                }
            } else if (prev_active) {
                finish_unit<E>(tmp[(j - 1) & 1], a.scale, held[j > 0 ? j - 1 : 0]);
            }
        }
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
            const int64_t s = s0 + (j + rot < a.spp ? j + rot : j + rot - a.spp);
            if (j < a.spp && s < n_steps) {
                const int64_t idx = (s << 6) + lane;
                if (idx < n_units) store_held<E>(a.out, idx, a.scale, held[j]);
            }
        }
    }
    // the last count % E elements, one thread each
    const int64_t k = n_units * E + threadIdx.x;
    if (blockIdx.x == 0 && k < a.count) {
        float acc = -0.0f;
        for (int g = 0; g < a.G; ++g) {
            float v;
            if constexpr (IN_F32)
                v = reinterpret_cast<const float *>(a.p[g])[k];
            else
                v = __uint_as_float(static_cast<uint32_t>(
                        reinterpret_cast<const uint16_t *>(a.p[g])[k]) << 16);
            acc = acc + v;
        }
        acc = acc * a.scale;
        if constexpr (OUT_F32)
            reinterpret_cast<float *>(a.out)[k] = acc;
        else
            reinterpret_cast<uint16_t *>(a.out)[k] =
                static_cast<uint16_t>(bf16_rne_bits(acc));
    }
}

// ---- reduce over runs (trainable ranges of unpacked gradients) ------------
// A LoRA layer's shard is a few tens of thousands of elements, so the kernel is
// launch-bound: small pieces spread it over enough workgroups (measured:
// 256..2048 elements per piece are within noise of each other, 4.2-4.5 us).
constexpr int kRunPieceElems = 512; // elements one workgroup reduces
constexpr int kRunBlock = 128;      // one 4-element vector per thread

struct ReduceRunArgs {
    int32_t first_piece[kMaxReduceRuns + 1]; // prefix sums; unused = INT32_MAX
    int32_t G;
    float scale;
    int64_t src_off[kMaxReduceRuns]; // elements; < 0: the run is zeros
    int64_t dst_off[kMaxReduceRuns];
    int64_t count[kMaxReduceRuns];
    const char *p[FCDP_MAX_G];
    char *out;
};

template <bool IN_F32>
__device__ __forceinline__ float load_elem(const char *base, int64_t e)
{
    if constexpr (IN_F32)
        return reinterpret_cast<const float *>(base)[e];
    else
        return __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t *>(base)[e]) << 16);
}

template <bool OUT_F32>
__device__ __forceinline__ void store_elem(char *base, int64_t e, float v)
{
    if constexpr (OUT_F32)
        reinterpret_cast<float *>(base)[e] = v;
    else
        reinterpret_cast<uint16_t *>(base)[e] = static_cast<uint16_t>(bf16_rne_bits(v));
}

// Workgroup i reduces piece i: up to kRunPieceElems elements of one run.  The
// run is found from the block index by counting prefix sums held in the
// kernel argument.  Element offsets are arbitrary, so loads use
// element-aligned vectors and stores fall back to single elements when the
// destination is not vector aligned.  Same arithmetic and order as
// reduce_ranks.
template <bool IN_F32, bool OUT_F32>
__global__ void __launch_bounds__(256) reduce_runs(const ReduceRunArgs a)
{
    const int32_t total = a.first_piece[kMaxReduceRuns];
    for (int32_t i = blockIdx.x; i < total; i += gridDim.x) {
        int32_t r = 0;
#pragma unroll
        for (int k = 1; k < kMaxReduceRuns; ++k) r += (i >= a.first_piece[k]) ? 1 : 0;
        const int64_t e0 = static_cast<int64_t>(i - a.first_piece[r]) * kRunPieceElems;
        int64_t n = a.count[r] - e0;
        if (n > kRunPieceElems) n = kRunPieceElems;
        const int64_t so = a.src_off[r];
        const int64_t s = so + e0, d = a.dst_off[r] + e0;
        constexpr int64_t oes = OUT_F32 ? 4 : 2;
        const bool vec_store = ((reinterpret_cast<uintptr_t>(a.out) + d * oes) & (OUT_F32 ? 15 : 7)) == 0;
        const int64_t nvec = n >> 2;
        for (int64_t v = threadIdx.x; v < nvec; v += blockDim.x) {
            float acc[4] = {-0.0f, -0.0f, -0.0f, -0.0f};
            if (so >= 0) {
                const int64_t sb = s * (IN_F32 ? 4 : 2);
                int g = 0;
                // four ranks' loads are issued before their adds; the adds
                // stay in rank order
                for (; g + 4 <= a.G; g += 4) {
                    float x[4][4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) load4<IN_F32, false, false>(a.p[g + k] + sb, v, x[k]);
#pragma unroll
                    for (int k = 0; k < 4; ++k)
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[c] = acc[c] + x[k][c];
                }
                for (; g < a.G; ++g) {
                    float x[4];
                    load4<IN_F32, false, false>(a.p[g] + sb, v, x);
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] = acc[c] + x[c];
                }
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = 0.0f;
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] = acc[c] * a.scale;
            if (vec_store) {
                store4<OUT_F32, false>(a.out + d * oes, v, acc);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) store_elem<OUT_F32>(a.out, d + v * 4 + c, acc[c]);
            }
        }
        const int64_t k = (nvec << 2) + threadIdx.x;
        if (k < n) {
            float acc = -0.0f;
            if (so >= 0) {
                for (int g = 0; g < a.G; ++g) acc = acc + load_elem<IN_F32>(a.p[g], s + k);
            } else {
                acc = 0.0f;
            }
            store_elem<OUT_F32>(a.out, d + k, acc * a.scale);
        }
    }
}

std::atomic<int> g_cu_count[kMaxDevices]; // 0 = not asked yet; any thread may fill it in
std::atomic<int> g_last_reduce_shape{0};  // what the last launch_reduce of the process picked

// Launches `kernel`; with timing events the dispatch itself carries them.
template <typename K, typename A>
hipError_t launch_one(K kernel, dim3 grid, dim3 block, hipStream_t st, const LaunchEvents &ev, const A &args)
{
    if (ev.start || ev.stop) // either may be null: a call of several dispatches starts on its first, stops on its last
        hipExtLaunchKernelGGL(kernel, grid, block, 0, st, static_cast<hipEvent_t>(ev.start),
                              static_cast<hipEvent_t>(ev.stop), 0, args);
    else
        hipLaunchKernelGGL(kernel, grid, block, 0, st, args);
    return hipGetLastError();
}

template <int UNROLL>
hipError_t launch_copy_h(const CopyArgs &args, dim3 grid, dim3 block, int hint, hipStream_t st,
                         const LaunchEvents &ev)
{
    switch (hint & 3) {
    case 0: return launch_one(copy_pieces<UNROLL, 0>, grid, block, st, ev, args);
    case 1: return launch_one(copy_pieces<UNROLL, 1>, grid, block, st, ev, args);
    case 2: return launch_one(copy_pieces<UNROLL, 2>, grid, block, st, ev, args);
    default: return launch_one(copy_pieces<UNROLL, 3>, grid, block, st, ev, args);
    }
}

template <int UNROLL>
hipError_t launch_plain_h(const PlainArgs &args, dim3 grid, dim3 block, int hint, hipStream_t st,
                          const LaunchEvents &ev)
{
    switch (hint & 3) {
    case 0: return launch_one(plain_copy<UNROLL, 0>, grid, block, st, ev, args);
    case 1: return launch_one(plain_copy<UNROLL, 1>, grid, block, st, ev, args);
    case 2: return launch_one(plain_copy<UNROLL, 2>, grid, block, st, ev, args);
    default: return launch_one(plain_copy<UNROLL, 3>, grid, block, st, ev, args);
    }
}

template <int REM, bool IN_F32, bool OUT_F32, bool ALIGNED>
hipError_t launch_reduce_r(const ReduceArgs &args, dim3 grid, dim3 block, hipStream_t st,
                           const LaunchEvents &ev)
{
    return launch_one(reduce_ranks<REM, IN_F32, OUT_F32, ALIGNED, kReduceUnroll, kReduceNT>,
                      grid, block, st, ev, args);
}

template <int REM, bool IN_F32, bool OUT_F32>
hipError_t launch_phased_r(const ReduceArgs &args, dim3 grid, dim3 block, hipStream_t st,
                           const LaunchEvents &ev)
{
    if constexpr (REM < kPhasedGroup)
        return launch_one(reduce_phased<kPhaseSteps2, 2, REM, IN_F32, OUT_F32, kReduceNT>, grid, block, st, ev, args);
    else
        return hipErrorInvalidValue; // not reachable: REM = G mod kPhasedGroup
}

// waves_per_simd 1: only built for G a multiple of the load group
template <bool IN_F32, bool OUT_F32>
hipError_t launch_phased_t(const ReduceArgs &args, int waves_per_simd, dim3 grid, dim3 block, hipStream_t st,
                           const LaunchEvents &ev)
{
    if (waves_per_simd == 1)
        return launch_one(reduce_phased<kPhaseSteps1, 1, 0, IN_F32, OUT_F32, kReduceNT>, grid, block, st, ev, args);
    switch (args.G % kPhasedGroup) {
    case 0: return launch_phased_r<0, IN_F32, OUT_F32>(args, grid, block, st, ev);
    case 1: return launch_phased_r<1, IN_F32, OUT_F32>(args, grid, block, st, ev);
    case 2: return launch_phased_r<2, IN_F32, OUT_F32>(args, grid, block, st, ev);
    case 3: return launch_phased_r<3, IN_F32, OUT_F32>(args, grid, block, st, ev);
    case 4: return launch_phased_r<4, IN_F32, OUT_F32>(args, grid, block, st, ev);
    case 5: return launch_phased_r<5, IN_F32, OUT_F32>(args, grid, block, st, ev);
    case 6: return launch_phased_r<6, IN_F32, OUT_F32>(args, grid, block, st, ev);
    default: return launch_phased_r<7, IN_F32, OUT_F32>(args, grid, block, st, ev);
    }
}

template <bool IN_F32, bool OUT_F32, bool ALIGNED>
hipError_t launch_reduce_t(const ReduceArgs &args, dim3 grid, dim3 block, hipStream_t st,
                           const LaunchEvents &ev)
{
    switch (args.G % kGroup) {
    case 0: return launch_reduce_r<0, IN_F32, OUT_F32, ALIGNED>(args, grid, block, st, ev);
    case 1: return launch_reduce_r<1, IN_F32, OUT_F32, ALIGNED>(args, grid, block, st, ev);
    case 2: return launch_reduce_r<2, IN_F32, OUT_F32, ALIGNED>(args, grid, block, st, ev);
    case 3: return launch_reduce_r<3, IN_F32, OUT_F32, ALIGNED>(args, grid, block, st, ev);
    case 4: return launch_reduce_r<4, IN_F32, OUT_F32, ALIGNED>(args, grid, block, st, ev);
    case 5: return launch_reduce_r<5, IN_F32, OUT_F32, ALIGNED>(args, grid, block, st, ev);
    case 6: return launch_reduce_r<6, IN_F32, OUT_F32, ALIGNED>(args, grid, block, st, ev);
    default: return launch_reduce_r<7, IN_F32, OUT_F32, ALIGNED>(args, grid, block, st, ev);
    }
}

} // namespace

int last_reduce_shape() { return g_last_reduce_shape.load(std::memory_order_relaxed); }

int device_cu_count()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (dev < 0 || dev >= kMaxDevices) return 256;
    int n = g_cu_count[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        g_cu_count[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

int launch_copy(const CopyLaunch &c, void *stream)
{
    if (c.n_pieces <= 0) return hipSuccess;
    CopyArgs args;
    args.pieces = c.pieces;
    args.n_pieces = c.n_pieces;
    for (int i = 0; i < kMaxSmall; ++i)
        args.ptrs[i] = i < c.n_small
            ? const_cast<char *>(static_cast<const char *>(c.small_ptrs[i])) : nullptr;
    for (int i = 0; i < kTensorWindow; ++i)
        args.ptrs[kMaxSmall + i] = i < c.n_tensor
            ? const_cast<char *>(static_cast<const char *>(c.tensor_ptrs[i])) : nullptr;
    switch (c.tensor_side) {
    case TensorSide::Dst: // short list -> tensors
        args.src_bias = 0;
        args.dst_bias = kMaxSmall - c.tensor_base;
        break;
    case TensorSide::Src: // tensors -> short list
        args.src_bias = kMaxSmall - c.tensor_base;
        args.dst_bias = 0;
        break;
    default:              // one source buffer (slot 0) -> one destination (slot 1)
        args.src_bias = 0;
        args.dst_bias = 1;
        break;
    }
    const Tuning &t = tuning();
    int64_t grid = c.n_pieces;
    if (c.wg_per_cu > 0)
        grid = std::min<int64_t>(grid, c.wg_per_cu * device_cu_count());
    if (c.max_wgs > 0) grid = std::min<int64_t>(grid, c.max_wgs);
    grid = std::min<int64_t>(grid, 0x7fffffff);
    const dim3 g(static_cast<unsigned>(grid)),
        b(static_cast<unsigned>(c.block > 0 ? c.block : t.copy_block));
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int unroll = static_cast<int>(t.copy_unroll);
    const int hint = c.nt ? static_cast<int>(t.copy_nt) : 0;
    if (unroll >= 8) return launch_copy_h<8>(args, g, b, hint, st, c.ev);
    if (unroll >= 4) return launch_copy_h<4>(args, g, b, hint, st, c.ev);
    if (unroll >= 2) return launch_copy_h<2>(args, g, b, hint, st, c.ev);
    return launch_copy_h<1>(args, g, b, hint, st, c.ev);
}

int launch_reduce_runs(const void *const *partials, int32_t G, const ReduceRuns &runs,
                       int in_dtype, int out_dtype, float scale, void *out, void *stream,
                       const LaunchEvents &ev)
{
    if (runs.n_runs <= 0) return hipSuccess;
    ReduceRunArgs args;
    int64_t total = 0;
    for (int k = 0; k < kMaxReduceRuns; ++k) {
        if (k < runs.n_runs) {
            args.first_piece[k] = static_cast<int32_t>(total);
            args.src_off[k] = runs.src_off[k];
            args.dst_off[k] = runs.dst_off[k];
            args.count[k] = runs.count[k];
            total += (runs.count[k] + kRunPieceElems - 1) / kRunPieceElems;
        } else {
            args.first_piece[k] = 0x7fffffff;
            args.src_off[k] = args.dst_off[k] = args.count[k] = 0;
        }
    }
    if (total <= 0) return hipSuccess;
    if (total >= 0x7fffffff) return hipErrorInvalidValue;
    args.first_piece[kMaxReduceRuns] = static_cast<int32_t>(total);
    args.G = G;
    args.scale = scale;
    for (int g = 0; g < FCDP_MAX_G; ++g)
        args.p[g] = g < G ? static_cast<const char *>(partials[g]) : nullptr;
    args.out = static_cast<char *>(out);
    const dim3 grid(static_cast<unsigned>(total)), block(kRunBlock);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool inf = in_dtype == FCDP_F32, outf = out_dtype == FCDP_F32;
    if (inf && outf) return launch_one(reduce_runs<true, true>, grid, block, st, ev, args);
    if (inf && !outf) return launch_one(reduce_runs<true, false>, grid, block, st, ev, args);
    if (!inf && outf) return launch_one(reduce_runs<false, true>, grid, block, st, ev, args);
    return launch_one(reduce_runs<false, false>, grid, block, st, ev, args);
}

int launch_fill(void *dst, size_t bytes, uint16_t pattern, void *stream, int64_t max_wgs)
{
    if (bytes == 0) return hipSuccess;
    FillArgs a;
    a.dst = static_cast<char *>(dst);
    a.bytes = bytes;
    a.pattern = static_cast<uint32_t>(pattern) | (static_cast<uint32_t>(pattern) << 16);
    int64_t grid = static_cast<int64_t>(((bytes >> 4) + 255) / 256);
    grid = std::max<int64_t>(1, std::min<int64_t>(grid, max_wgs > 0 ? max_wgs : 16384));
    hipLaunchKernelGGL(fill_pattern, dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
    return hipGetLastError();
}

int launch_plain_copy(void *dst, const void *src, size_t bytes, void *stream,
                      const PlainCopy &shape)
{
    if (bytes == 0) return hipSuccess;
    const Tuning &t = tuning();
    const uint32_t chunk = static_cast<uint32_t>(shape.chunk > 0 ? shape.chunk : t.copy_chunk_bytes);
    const int64_t block = shape.block > 0 ? shape.block : t.copy_block;
    const int unroll = static_cast<int>(shape.unroll > 0 ? shape.unroll : t.copy_unroll);
    const int hint = shape.nt >= 0 ? shape.nt : static_cast<int>(t.copy_nt);
    size_t n_chunks = (bytes + chunk - 1) / chunk;
    int64_t grid = static_cast<int64_t>(std::min<size_t>(n_chunks, 0x7fffffff));
    if (shape.max_wgs > 0)
        grid = std::min<int64_t>(grid, shape.max_wgs);
    else if (t.copy_wg_per_cu > 0)
        grid = std::min<int64_t>(grid, t.copy_wg_per_cu * device_cu_count());
    const dim3 g(static_cast<unsigned>(grid)), b(static_cast<unsigned>(block));
    hipStream_t st = static_cast<hipStream_t>(stream);
    PlainArgs pa;
    pa.src = static_cast<const char *>(src);
    pa.dst = static_cast<char *>(dst);
    pa.bytes = bytes;
    pa.n_chunks = n_chunks;
    pa.chunk = chunk;
    if (unroll >= 8) return launch_plain_h<8>(pa, g, b, hint, st, shape.ev);
    if (unroll >= 4) return launch_plain_h<4>(pa, g, b, hint, st, shape.ev);
    if (unroll >= 2) return launch_plain_h<2>(pa, g, b, hint, st, shape.ev);
    return launch_plain_h<1>(pa, g, b, hint, st, shape.ev);
}

int launch_reduce_stream_calibration(void *dst, const void *src, int32_t G, int64_t count,
                                     int out_dtype, void *stream, const LaunchEvents &ev)
{
    if (count <= 0) return hipSuccess;
    StreamArgs a;
    a.src = static_cast<const char *>(src);
    a.out = static_cast<char *>(dst);
    a.tiles = count / 1024;
    a.G = G;
    const dim3 grid(static_cast<unsigned>(std::min<int64_t>(a.tiles, 0x7fffffff))), block(64);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (out_dtype == FCDP_F32) return launch_one(reduce_stream_calibration<true>, grid, block, st, ev, a);
    return launch_one(reduce_stream_calibration<false>, grid, block, st, ev, a);
}

int launch_reduce(const void *const *partials, int32_t G, int64_t elem_offset,
                  int64_t count, int in_dtype, int out_dtype, float scale, void *out,
                  void *stream, const LaunchEvents &ev)
{
    if (count <= 0) return hipSuccess;
    const int64_t in_esz = in_dtype == FCDP_F32 ? 4 : 2;
    ReduceArgs args;
    bool aligned = true;
    for (int g = 0; g < FCDP_MAX_G; ++g) {
        if (g < G) {
            args.p[g] = static_cast<const char *>(partials[g]) + elem_offset * in_esz;
            if (reinterpret_cast<uintptr_t>(args.p[g]) & 15u) aligned = false;
        } else {
            args.p[g] = nullptr;
        }
    }
    args.out = static_cast<char *>(out);
    args.count = count;
    args.G = G;
    args.scale = scale;
    const Tuning &t = tuning();
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool inf = in_dtype == FCDP_F32, outf = out_dtype == FCDP_F32;
    // The persistent grid: every wave resident at once.  Where each kernel pays by G
    // and type pair (20 launches each on MI355X, a 25 M-element shard, G = 1..64,
    // fractions of the HBM peak): with G a multiple of 8 the one-wave-per-SIMD shape
    // is the fastest from G = 8 on (0.83-0.86 against 0.75-0.81 for one tile per
    // workgroup), bf16 partials into a bf16 shard at G = 8 aside (two waves 0.78,
    // one 0.77).  For other G the two-wave shape wins from G = 3 on when both types
    // are equal (fp32 0.80-0.83 against 0.77-0.80, bf16 0.78-0.82 against 0.72-0.76),
    // from G = 5 on for fp32 partials into a bf16 shard (0.81-0.84 against 0.78-0.81)
    // and from G = 12 on for bf16 partials into an fp32 shard; below that one tile
    // per workgroup is faster (at G = 1 by 0.78 against 0.51).
    // And by length: a launch has a fixed cost (the ramp, the tail, the store burst),
    // so a phased launch must be long.  One launch holds C = waves x held steps.  A
    // longer input takes full launches of C steps and then what is left (the kernel
    // boundary keeps one launch's stores out of the next one's reads: 0.80 of the
    // peak at 200 M elements, against 0.66 with the passes inside one kernel and 0.73
    // for one tile per workgroup).  What a launch of fewer than C steps runs: the
    // one-wave shape from 0.7 C on (below that it falls behind the others: at half
    // of C 0.76 against 0.80 at G = 8); the two-wave shape from 0.46 C on, for G = 8
    // only where it is the rule's pick anyway (at G = 8 it merely ties with one tile
    // per workgroup there, at G >= 12 it is 3-6 points ahead); otherwise one tile
    // per workgroup (at 0.3 C: 0.80-0.81 against 0.67-0.77).
    const int64_t wpb = kPhasedBlock / 64;
    const int64_t epu = inf ? 4 : 8;                       // elements per 16-byte unit
    const int64_t out_esz = outf ? 4 : 2;
    const int64_t n_steps = (count / epu + 63) / 64;
    const int64_t W1 = static_cast<int64_t>(device_cu_count()) * 4; // waves at one per SIMD
    static_assert(kPhaseSteps1 == 2 * kPhaseSteps2, "both shapes hold the same number of steps per launch");
    const int64_t cap1 = kPhaseSteps1 * 4 / epu;           // steps a wave holds at one per SIMD
    const int64_t C = W1 * cap1;                           // steps per launch, either shape
    const bool can_phase = aligned && (reinterpret_cast<uintptr_t>(out) & 15u) == 0;
    // waves per SIMD for a launch of `steps` steps; 0 = one tile per workgroup
    auto shape_for = [&](int64_t steps) {
        int wps = 0;
        if (!can_phase) return 0;
        if (t.reduce_phased == 1) {
            wps = t.reduce_phase_waves ? static_cast<int>(t.reduce_phase_waves) : (G % kPhasedGroup == 0 ? 1 : 2);
            if (wps == 1 && G % kPhasedGroup != 0) wps = 2; // the one-wave shape is built for full groups only
            if (steps < W1 * wps * kPhasedMinStepsPerWave) wps = 0;
        } else if (t.reduce_phased == 2) {
            if (G % kPhasedGroup == 0) wps = (G == 8 && !inf && !outf) ? 2 : 1;
            else if (G >= 12 || (G >= 3 && inf == outf) || (G >= 5 && inf && !outf)) wps = 2;
            if (wps && t.reduce_phase_waves) wps = static_cast<int>(t.reduce_phase_waves);
            if (wps == 1 && G % kPhasedGroup != 0) wps = 2;
            if (wps == 1 && steps * 10 < C * 7) wps = G >= 12 ? 2 : 0;
            if (wps == 2 && steps * 100 < C * 46) wps = 0;
        }
        return wps;
    };
    g_last_reduce_shape.store(shape_for(std::min(n_steps, C)), std::memory_order_relaxed);
    int64_t s_begin = 0;                                   // steps already launched
    while (s_begin < n_steps) {
        const int64_t steps = std::min(n_steps - s_begin, C);
        const int wps = shape_for(steps);
        if (wps == 0) break;                               // the rest goes to one tile per workgroup
        const int64_t W = W1 * wps;
        const dim3 g(static_cast<unsigned>(W / wpb)), b(kPhasedBlock);
        const int64_t e_begin = s_begin * 64 * epu;        // a multiple of 1 KiB of input: alignment is kept
        const bool last = s_begin + steps == n_steps;
        ReduceArgs ra = args;
        for (int32_t r = 0; r < G; ++r) ra.p[r] = args.p[r] + e_begin * in_esz;
        ra.out = args.out + e_begin * out_esz;
        ra.count = last ? count - e_begin : steps * 64 * epu;
        const int64_t spp = (steps + W - 1) / W;           // <= the steps a wave of this shape holds
        ra.spp = static_cast<int32_t>(spp);
        // Runs of 43 or 86 KiB (3 x 43 KiB = 128 KiB + 1 KiB) measured 4-14 % slower than
        // their neighbours at every G and size tried when all waves start their run
        // at its first step; started at step w mod spp they run like the neighbours.
        ra.rotate = t.reduce_phase_rotate == 2 ? 1 : (t.reduce_phase_rotate == 1 ? (spp % 43 == 0) : 0);
        // with timing on, the call's interval runs from its first dispatch to its last
        LaunchEvents le;
        le.start = s_begin == 0 ? ev.start : nullptr;
        le.stop = last ? ev.stop : nullptr;
        hipError_t e;
        if (inf && outf) e = launch_phased_t<true, true>(ra, wps, g, b, st, le);
        else if (inf && !outf) e = launch_phased_t<true, false>(ra, wps, g, b, st, le);
        else if (!inf && outf) e = launch_phased_t<false, true>(ra, wps, g, b, st, le);
        else e = launch_phased_t<false, false>(ra, wps, g, b, st, le);
        if (e != hipSuccess) return e;
        s_begin += steps;
    }
    if (s_begin >= n_steps && s_begin > 0) return hipSuccess;
    // one tile per workgroup, for everything or for what the phased launches left
    const int64_t e_begin = s_begin * 64 * epu;
    for (int32_t r = 0; r < G; ++r) args.p[r] += e_begin * in_esz;
    args.out += e_begin * out_esz;
    args.count = count - e_begin;
    args.spp = args.rotate = 0;
    LaunchEvents le;
    le.start = s_begin == 0 ? ev.start : nullptr;
    le.stop = ev.stop;
    const int64_t nvec = args.count >> 2;
    const int64_t block = t.reduce_block;
    int64_t grid = (nvec + block * kReduceUnroll - 1) / (block * kReduceUnroll);
    grid = std::max<int64_t>(1, std::min<int64_t>(grid, 0x7fffffff));
    const dim3 g(static_cast<unsigned>(grid)), b(static_cast<unsigned>(block));
    if (inf && outf)
        return aligned ? launch_reduce_t<true, true, true>(args, g, b, st, le)
                       : launch_reduce_t<true, true, false>(args, g, b, st, le);
    if (inf && !outf)
        return aligned ? launch_reduce_t<true, false, true>(args, g, b, st, le)
                       : launch_reduce_t<true, false, false>(args, g, b, st, le);
    if (!inf && outf)
        return aligned ? launch_reduce_t<false, true, true>(args, g, b, st, le)
                       : launch_reduce_t<false, true, false>(args, g, b, st, le);
    return aligned ? launch_reduce_t<false, false, true>(args, g, b, st, le)
                   : launch_reduce_t<false, false, false>(args, g, b, st, le);
}

} // namespace fcdp
