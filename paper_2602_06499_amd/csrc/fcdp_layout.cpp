// Host side of libfcdp: the flat-parameter offset table, the tensor x shard
// segment list, and the piece tables the copy kernels walk.  No GPU needed.
//
// Layout (the paper does not print one; Sec. 2.1 and Sec. 6.1 fix only that
// every rank holds an equal 1/G shard): tensors end to end in the given
// order, zero tail padding up to a multiple of G*q, shard r = flat range
// [r*S, (r+1)*S).
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <new>

#include "fcdp_internal.h"

namespace fcdp {

namespace {

thread_local std::string g_last_error;

// Appends pieces for one contiguous run of `nbytes` bytes.  Cuts fall on
// multiples of `chunk` of the destination offset, so every piece after the
// first of a run starts chunk-aligned in its destination buffer.
void emit_run(std::vector<Piece> &out, int32_t src_idx, int64_t src_off,
              int32_t dst_idx, int64_t dst_off, int64_t nbytes, int64_t chunk)
{
    while (nbytes > 0) {
        int64_t room = chunk - (dst_off % chunk);
        int64_t n = std::min(room, nbytes);
        Piece p;
        p.src_off = src_idx < 0 ? 0 : src_off;
        p.dst_off = dst_off;
        p.nbytes = static_cast<int32_t>(n);
        p.src_idx = src_idx;
        p.dst_idx = dst_idx;
        p.reserved = 0;
        out.push_back(p);
        src_off += n;
        dst_off += n;
        nbytes -= n;
    }
}

void index_windows(PieceTable &tab, TensorSide side, int32_t T)
{
    const int64_t n_win = std::max<int64_t>(1, (T + kTensorWindow - 1) / kTensorWindow);
    tab.win_begin.assign(n_win + 1, static_cast<int64_t>(tab.pieces.size()));
    tab.win_begin[0] = 0;
    int64_t w = 0;
    for (int64_t i = 0; i < static_cast<int64_t>(tab.pieces.size()); ++i) {
        const Piece &p = tab.pieces[i];
        const int32_t t = side == TensorSide::Dst ? p.dst_idx : p.src_idx;
        const int64_t pw = t / kTensorWindow;
        while (w < pw) tab.win_begin[++w] = i;
    }
    while (w < n_win) tab.win_begin[++w] = static_cast<int64_t>(tab.pieces.size());
}

} // namespace

void set_error(const std::string &msg) { g_last_error = msg; }

fcdp_status fail_noexcept(fcdp_status st, const char *msg) noexcept
{
    try {
        g_last_error = msg;
    } catch (...) {
        g_last_error.clear(); // never throws
    }
    return st;
}

fcdp_status fail(fcdp_status st, const std::string &msg)
{
    g_last_error = msg;
    return st;
}

const std::string &last_error_ref() { return g_last_error; }

Tuning &tuning()
{
    static Tuning t = [] {
        Tuning v;
        const char *e = std::getenv("FCDP_DEBUG_POISON");
        if (e && e[0] && e[0] != '0') v.debug_poison = 1;
        return v;
    }();
    return t;
}

fcdp_status build_tables(fcdp_layout *L)
{
    const int64_t e = L->esz;
    const int64_t chunk = L->chunk_bytes;
    const int64_t S = L->S;

    // tensor x shard overlaps, in (tensor, shard) order
    L->segments.clear();
    for (int32_t t = 0; t < L->T; ++t) {
        const int64_t lo_t = L->off[t], hi_t = L->off[t + 1];
        if (hi_t == lo_t) continue;
        const int64_t r0 = lo_t / S, r1 = (hi_t - 1) / S;
        for (int64_t r = r0; r <= r1; ++r) {
            const int64_t lo = std::max(lo_t, r * S);
            const int64_t hi = std::min(hi_t, (r + 1) * S);
            L->segments.push_back({t, r, lo - lo_t, lo - r * S, hi - lo});
        }
    }

    // unflatten: shard r -> tensor t;  flatten: tensor t -> shard r
    L->unflatten.pieces.clear();
    L->flatten.pieces.clear();
    for (const Segment &s : L->segments) {
        emit_run(L->unflatten.pieces, static_cast<int32_t>(s.r), s.src_off * e,
                 static_cast<int32_t>(s.t), s.dst_off * e, s.len * e, chunk);
        emit_run(L->flatten.pieces, static_cast<int32_t>(s.t), s.dst_off * e,
                 static_cast<int32_t>(s.r), s.src_off * e, s.len * e, chunk);
    }
    // flatten also zero-fills the tail padding [N, N_pad)
    for (int64_t i = L->N; i < L->N_pad;) {
        const int64_t r = i / S;
        const int64_t hi = std::min(L->N_pad, (r + 1) * S);
        emit_run(L->flatten.pieces, -1, 0, static_cast<int32_t>(r),
                 (i - r * S) * e, (hi - i) * e, chunk);
        i = hi;
    }
    index_windows(L->unflatten, TensorSide::Dst, L->T);
    // flatten pieces are in tensor order except the zero-fill pieces at the
    // end (src_idx = -1), which are valid in every window: keep them out of
    // the window index and let the launcher add them to the last window.
    {
        PieceTable &f = L->flatten;
        int64_t n_copy = 0;
        for (const Piece &p : f.pieces)
            if (p.src_idx >= 0) ++n_copy;
        PieceTable only_copy;
        only_copy.pieces.assign(f.pieces.begin(), f.pieces.begin() + n_copy);
        index_windows(only_copy, TensorSide::Src, L->T);
        f.win_begin = only_copy.win_begin;
        f.win_begin.back() = static_cast<int64_t>(f.pieces.size());
    }

    // pack / unpack: runs of consecutive trainable tensors are contiguous in
    // both the flat and the packed buffer, so they are merged into one run.
    L->pack.pieces.clear();
    L->unpack.pieces.clear();
    int64_t c = 0;
    for (int32_t t = 0; t < L->T;) {
        if (!L->trainable[t] || L->numel[t] == 0) {
            ++t;
            continue;
        }
        int32_t u = t;
        int64_t run = 0;
        while (u < L->T && (L->trainable[u] || L->numel[u] == 0)) {
            run += L->numel[u];
            ++u;
        }
        emit_run(L->pack.pieces, 0, L->off[t] * e, 0, c * e, run * e, chunk);
        // unpack pieces are also cut at the shard boundaries of the flat buffer, so that the
        // pieces that write one range of shards are a contiguous part of the table (a GPU that
        // holds only its node slice of the flat image unpacks exactly those)
        for (int64_t lo = L->off[t], done = 0; done < run;) {
            const int64_t hi = std::min(L->off[t] + run, S > 0 ? (lo / S + 1) * S : L->off[t] + run);
            emit_run(L->unpack.pieces, 0, (c + done) * e, 0, lo * e, (hi - lo) * e, chunk);
            done += hi - lo;
            lo = hi;
        }
        c += run;
        t = u;
    }
    if (L->N_packed > L->N_t)
        emit_run(L->pack.pieces, -1, 0, 0, L->N_t * e,
                 (L->N_packed - L->N_t) * e, chunk);
    L->pack.win_begin = {0, static_cast<int64_t>(L->pack.pieces.size())};
    L->unpack.win_begin = {0, static_cast<int64_t>(L->unpack.pieces.size())};
    return FCDP_OK;
}

} // namespace fcdp

using fcdp::fail;

extern "C" {

fcdp_status fcdp_layout_build(const int64_t *numel, const uint8_t *trainable,
                              int32_t n_tensors, int32_t G, int32_t elem_size,
                              int32_t pad_quantum, fcdp_layout **out)
try {
    if (!out) return fail(FCDP_EINVAL, "fcdp_layout_build: out is NULL");
    *out = nullptr;
    if (!numel) return fail(FCDP_EINVAL, "fcdp_layout_build: numel is NULL");
    if (n_tensors < 1)
        return fail(FCDP_EINVAL, "fcdp_layout_build: n_tensors must be >= 1");
    if (G < 1) return fail(FCDP_EINVAL, "fcdp_layout_build: G must be >= 1");
    if (G > FCDP_MAX_G)
        return fail(FCDP_ESIZE, "fcdp_layout_build: G exceeds FCDP_MAX_G (64)");
    if (elem_size != 2 && elem_size != 4)
        return fail(FCDP_EINVAL, "fcdp_layout_build: elem_size must be 2 or 4");
    if (pad_quantum < 1 || pad_quantum > (1 << 20))
        return fail(FCDP_EINVAL, "fcdp_layout_build: pad_quantum must be in 1..2^20");
    // 1 TiB of flat bytes is far beyond one GPU's memory and keeps the piece
    // tables small enough to build
    const int64_t limit = (int64_t(1) << 40) / elem_size - (int64_t(1) << 27);
    int64_t N = 0;
    for (int32_t t = 0; t < n_tensors; ++t) {
        if (numel[t] < 0)
            return fail(FCDP_EINVAL, "fcdp_layout_build: negative numel");
        if (numel[t] > limit - N)
            return fail(FCDP_ESIZE, "fcdp_layout_build: flat size overflows");
        N += numel[t];
    }
    fcdp_layout *L = new (std::nothrow) fcdp_layout;
    if (!L) return fail(FCDP_ENOMEM, "fcdp_layout_build: out of host memory");
    try {
        L->T = n_tensors;
        L->G = G;
        L->esz = elem_size;
        L->q = pad_quantum;
        L->numel.assign(numel, numel + n_tensors);
        L->trainable.assign(n_tensors, 1);
        if (trainable)
            for (int32_t t = 0; t < n_tensors; ++t)
                L->trainable[t] = trainable[t] ? 1 : 0;
        L->off.assign(n_tensors + 1, 0);
        for (int32_t t = 0; t < n_tensors; ++t)
            L->off[t + 1] = L->off[t] + numel[t];
        const int64_t Q = static_cast<int64_t>(G) * pad_quantum;
        L->N = N;
        L->N_pad = (N + Q - 1) / Q * Q;
        L->S = L->N_pad / G;
        L->N_t = 0;
        for (int32_t t = 0; t < n_tensors; ++t)
            if (L->trainable[t]) L->N_t += numel[t];
        L->N_packed = (L->N_t + Q - 1) / Q * Q;
        L->chunk_bytes = fcdp::tuning().copy_chunk_bytes;
        // never more than ~4M pieces per table
        const int64_t min_chunk = ((L->N_pad * elem_size) >> 22) / 4096 * 4096 + 4096;
        if (L->chunk_bytes < min_chunk) L->chunk_bytes = min_chunk;
        if (L->S > 0) {
            fcdp_status st = fcdp::build_tables(L);
            if (st != FCDP_OK) {
                delete L;
                return st;
            }
        } else {
            L->unflatten.win_begin = {0, 0};
            L->flatten.win_begin = {0, 0};
            L->pack.win_begin = {0, 0};
            L->unpack.win_begin = {0, 0};
        }
    } catch (const std::bad_alloc &) {
        delete L;
        return fail(FCDP_ENOMEM, "fcdp_layout_build: out of host memory");
    }
    *out = L;
    return FCDP_OK;
} catch (...) {
    return fcdp::fail_noexcept(FCDP_ENOMEM, "fcdp_layout_build: out of host memory");
}

int32_t fcdp_layout_n_tensors(const fcdp_layout *L) { return L ? L->T : -1; }
int32_t fcdp_layout_G(const fcdp_layout *L) { return L ? L->G : -1; }
int32_t fcdp_layout_elem_size(const fcdp_layout *L) { return L ? L->esz : -1; }
int64_t fcdp_layout_numel(const fcdp_layout *L) { return L ? L->N : -1; }
int64_t fcdp_layout_padded_numel(const fcdp_layout *L) { return L ? L->N_pad : -1; }
int64_t fcdp_layout_shard_numel(const fcdp_layout *L) { return L ? L->S : -1; }
int64_t fcdp_layout_trainable_numel(const fcdp_layout *L) { return L ? L->N_t : -1; }
int64_t fcdp_layout_packed_numel(const fcdp_layout *L) { return L ? L->N_packed : -1; }
const int64_t *fcdp_layout_offsets(const fcdp_layout *L)
{
    return L ? L->off.data() : nullptr;
}

int64_t fcdp_layout_segments(const fcdp_layout *L, int64_t *rows, int64_t cap)
{
    if (!L) return -1;
    const int64_t n = static_cast<int64_t>(L->segments.size());
    if (rows)
        for (int64_t i = 0; i < n && i < cap; ++i) {
            const fcdp::Segment &s = L->segments[i];
            rows[i * 5 + 0] = s.t;
            rows[i * 5 + 1] = s.r;
            rows[i * 5 + 2] = s.dst_off;
            rows[i * 5 + 3] = s.src_off;
            rows[i * 5 + 4] = s.len;
        }
    return n;
}

int64_t fcdp_layout_copy_plan(const fcdp_layout *L, int32_t which, int64_t *rows, int64_t cap)
{
    if (!L || which < 0 || which > 3) return -1;
    const fcdp::PieceTable &tab = which == 0 ? L->unflatten : which == 1 ? L->flatten
                                  : which == 2 ? L->pack : L->unpack;
    const int64_t n = static_cast<int64_t>(tab.pieces.size());
    if (rows)
        for (int64_t i = 0; i < n && i < cap; ++i) {
            const fcdp::Piece &p = tab.pieces[i];
            rows[i * 5 + 0] = p.src_idx;
            rows[i * 5 + 1] = p.src_off;
            rows[i * 5 + 2] = p.dst_idx;
            rows[i * 5 + 3] = p.dst_off;
            rows[i * 5 + 4] = p.nbytes;
        }
    return n;
}

const char *fcdp_status_string(fcdp_status st)
{
    switch (st) {
    case FCDP_OK: return "FCDP_OK";
    case FCDP_EINVAL: return "FCDP_EINVAL: invalid argument";
    case FCDP_ESIZE: return "FCDP_ESIZE: size beyond a documented limit";
    case FCDP_EALIGN: return "FCDP_EALIGN: base pointer not 16-byte aligned";
    case FCDP_ENOTPINNED: return "FCDP_ENOTPINNED: not mapped pinned host memory";
    case FCDP_ESTATE: return "FCDP_ESTATE: cache-state call out of order";
    case FCDP_ENOMEM: return "FCDP_ENOMEM: allocation failed";
    case FCDP_EHIP: return "FCDP_EHIP: HIP runtime error";
    }
    return "unknown fcdp_status";
}

const char *fcdp_last_error(void) { return fcdp::last_error_ref().c_str(); }

} // extern "C"
