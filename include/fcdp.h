/*
 * fcdp.h -- C ABI of the FCDP per-layer hot path for one AMD MI355X (gfx950).
 *
 * What the path is (paper Sec. 2.1, Sec. 4.3-4.5, Alg. 1, Sec. 6.1-6.3): under
 * fully sharded data parallelism each of the G ranks keeps a 1/G shard of a
 * layer's flat parameter buffer; the full per-tensor parameters are rebuilt
 * before the forward and again before the backward computation; FCDP keeps
 * the forward copy in pinned host memory and rebuilds the backward copy from
 * there; gradients are summed over ranks and each rank keeps the shard that
 * matches its parameter shard; under PEFT only trainable parameters travel.
 * This library is the part of that path that runs on one GPU.  Peers' shards
 * and partial gradients are ordinary device buffers handed in by the caller.
 *
 * Flat layout (the paper inherits it from its substrate and does not print
 * it; this is the reading used here): the T tensors of a layer are laid end
 * to end in the order given to fcdp_layout_build, tightly packed; the total
 * N is padded with zero elements at the tail to N_pad, a multiple of
 * G*pad_quantum; shard r is the flat range [r*S, (r+1)*S), S = N_pad/G.
 *
 * Conventions for every call below
 *   - "dev ptr" is a device address valid on the current HIP device; "host
 *     ptr" is an ordinary host address.  Arrays of pointers (shard_ptrs,
 *     tensor_ptrs, partial_ptrs) are HOST arrays whose entries are dev ptrs;
 *     they are read during the call and may be freed right after it returns.
 *   - Ownership: the caller owns every data buffer.  The library owns only
 *     fcdp_layout / fcdp_cache_state objects and memory returned by
 *     fcdp_host_cache_alloc (freed with fcdp_host_cache_free).
 *   - Streams are hipStream_t values passed as void* (NULL = the default
 *     stream).  Data calls only enqueue work; they never synchronise the
 *     device, with two exceptions: the first data call on a layout uploads
 *     the layout's tables (call fcdp_layout_prepare beforehand to avoid
 *     that), and a call that would put more than max_copies_in_flight (a
 *     tuning knob, default 2) host-link DMA copies in flight first waits on
 *     the host for the oldest of them.
 *   - Stream capture: the calls that only launch kernels may be recorded into
 *     a HIP graph: fcdp_materialize_layer with FCDP_SRC_DEVICE_SHARDS and no
 *     store, fcdp_flatten_to_shards, the reduce entry points, pack and
 *     unpack; call fcdp_layout_prepare first and keep timing disabled.  The
 *     host-cache sources and the store use events and host-side waits and
 *     must stay outside a capture.
 *   - Every data base pointer must be 16-byte aligned (FCDP_EALIGN if not).
 *     Offsets inside a buffer may be any element index.
 *   - Errors: a status code is returned, nothing is thrown (every entry
 *     point catches what its host code could throw, e.g. on exhausted host
 *     memory, and returns FCDP_ENOMEM) and nothing aborts.  All argument checks precede the first enqueue, so a call that
 *     fails an argument check has no side effect.  fcdp_last_error() gives a
 *     thread-local text for the last failing call on the calling thread.
 *   - Zero-element tensors, N = 0 and N_t = 0 are legal no-ops.
 *   - Threads: a layout is immutable and may be shared.  Data calls may come
 *     from several threads: the event ring, the staging-buffer table, the
 *     list of copies in flight and the link counters of a device are guarded,
 *     and a thread that has to wait for the oldest copy in flight waits
 *     without holding that guard.  Calls that share a staging buffer, a cache
 *     state object, the static staging array or the timing pool (i.e. any
 *     data call while timing is enabled) must be serialised by the caller.
 */
#ifndef FCDP_H
#define FCDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fcdp_layout fcdp_layout;           /* immutable after build */
typedef struct fcdp_cache_state fcdp_cache_state; /* dirty flags, host only */
typedef void *fcdp_stream;                        /* a hipStream_t */

typedef enum {
    FCDP_OK = 0,
    FCDP_EINVAL = 1,     /* NULL pointer, bad count, bad enum, aliasing */
    FCDP_ESIZE = 2,      /* a size beyond a documented limit */
    FCDP_EALIGN = 3,     /* a base pointer that is not 16-byte aligned */
    FCDP_ENOTPINNED = 4, /* host_cache is not mapped pinned host memory */
    FCDP_ESTATE = 5,     /* cache-state call out of order */
    FCDP_ENOMEM = 6,     /* allocation failed */
    FCDP_EHIP = 7        /* a HIP runtime call failed; see fcdp_last_error */
} fcdp_status;

typedef enum { FCDP_BF16 = 0, FCDP_F32 = 1 } fcdp_dtype;

typedef enum {
    FCDP_SRC_DEVICE_SHARDS = 0, /* cache miss: scatter the G gathered shards */
    FCDP_SRC_HOST_DMA = 1,      /* cache hit: DMA host cache -> staging, scatter */
    FCDP_SRC_HOST_ZEROCOPY = 2, /* cache hit: kernel reads the mapped host cache */
    FCDP_SRC_DEVICE_RESIDENT = 3, /* kept on the device since the forward pass: nothing to do */
    FCDP_SRC_HOST_SCATTER_DMA = 4 /* cache hit: one DMA copy per tensor, no kernel, no staging */
} fcdp_source;

/* store_cache argument of fcdp_materialize_layer */
typedef enum {
    FCDP_STORE_NONE = 0,
    FCDP_STORE_DMA = 1,      /* hipMemcpyAsync device -> pinned host */
    FCDP_STORE_ZEROCOPY = 2  /* a small kernel writes through the host mapping */
} fcdp_store;

#define FCDP_MAX_G 64 /* most shards / gradient partials per call */

/* ------------------------------------------------------------ offset table
 * Builds the layout of one layer: every rank keeps an equal 1/G share of the
 * flat parameter buffer (Sec. 2.1; the per-GPU parameter memory of Sec. 6.1).
 *   numel[t]      elements of tensor t (>= 0), t in [0, n_tensors)
 *   trainable[t]  1 = trainable (W_t), 0 = frozen (W_f); NULL = all trainable
 *                 (Sec. 4.5: parameters are classified once, at initialisation)
 *   G             number of ranks = shards, 1..FCDP_MAX_G
 *   elem_size     bytes per element, 2 (bf16) or 4
 *   pad_quantum   q: N_pad is a multiple of G*q (64 in all shipped configs)
 * Host-only; needs no GPU.  *out is owned by the library until
 * fcdp_layout_destroy.  Errors: FCDP_EINVAL, FCDP_ESIZE (G > FCDP_MAX_G or
 * a flat size that would overflow), FCDP_ENOMEM.
 */
fcdp_status fcdp_layout_build(const int64_t *numel, const uint8_t *trainable,
                              int32_t n_tensors, int32_t G, int32_t elem_size,
                              int32_t pad_quantum, fcdp_layout **out);
void fcdp_layout_destroy(fcdp_layout *layout);

int32_t fcdp_layout_n_tensors(const fcdp_layout *layout);
int32_t fcdp_layout_G(const fcdp_layout *layout);
int32_t fcdp_layout_elem_size(const fcdp_layout *layout);
int64_t fcdp_layout_numel(const fcdp_layout *layout);           /* N      */
int64_t fcdp_layout_padded_numel(const fcdp_layout *layout);    /* N_pad  */
int64_t fcdp_layout_shard_numel(const fcdp_layout *layout);     /* S      */
int64_t fcdp_layout_trainable_numel(const fcdp_layout *layout); /* N_t    */
int64_t fcdp_layout_packed_numel(const fcdp_layout *layout);    /* N_t up to G*q */
/* off[0..T]; borrowed, valid until destroy */
const int64_t *fcdp_layout_offsets(const fcdp_layout *layout);
/* Segment list: every non-empty (tensor x shard) overlap in (tensor, shard)
 * order, rows of 5 int64 (t, r, dst_off, src_off, len): len elements of
 * shard r starting at src_off form tensor t's elements from dst_off.
 * Returns the number of rows; writes at most cap rows. */
int64_t fcdp_layout_segments(const fcdp_layout *layout, int64_t *rows,
                             int64_t cap);
/* The copy plan a kernel walks, for inspection and host-side checking:
 * which = 0 unflatten (shards -> tensors), 1 flatten (tensors -> shards),
 * 2 pack (flat -> packed), 3 unpack (packed -> flat).  Rows of 5 int64
 * (src_idx, src_byte_off, dst_idx, dst_byte_off, nbytes); src_idx = -1 means
 * "write zeros".  Indices are shard or tensor numbers (0 for flat/packed).
 * Returns the number of rows (-1 on a bad argument); writes at most cap. */
int64_t fcdp_layout_copy_plan(const fcdp_layout *layout, int32_t which,
                              int64_t *rows, int64_t cap);
/* Uploads the layout's copy tables to the current device (synchronous,
 * idempotent) and, once per device, looks up the address of the library's
 * static staging array and creates the events
 * fcdp_materialize_layer_static uses.  Data calls other than that one do
 * the upload on first use if it was not called. */
fcdp_status fcdp_layout_prepare(const fcdp_layout *layout);

/* ---------------------------------------------------- layer materialization
 * Rebuilds the T per-tensor parameter buffers of one layer.
 *
 * FCDP_SRC_DEVICE_SHARDS (forward, cache miss; Sec. 4.3 forward pass, Alg. 1:
 * the dirty branch's inter-node gather): tensor_t[j] =
 * shard_{(off_t+j) div S}[(off_t+j) mod S].  If store_cache != FCDP_STORE_NONE
 * the padded flat image concat(shard_0..shard_{G-1}) is also copied to
 * host_cache on the `copy` stream (Alg. 1: the dirty branch's refresh of
 * the host copy, GPU to host), ordered
 * after everything enqueued on `compute` before this call; the shards must
 * stay unmodified until that copy has completed in `copy`-stream order.
 * FCDP_STORE_DMA uses hipMemcpyAsync; FCDP_STORE_ZEROCOPY uses a kernel with a
 * bounded number of workgroups that writes through the host mapping
 * (host_cache must then be mapped pinned memory, else FCDP_ENOTPINNED).
 *
 * FCDP_SRC_HOST_DMA (backward / clean forward, cache hit; Sec. 4.3 backward
 * pass, Alg. 1: the load of the cached copy from the host): host_cache is
 * copied to `staging` on the
 * `copy` stream, then the scatter runs on `compute` after it.  The library
 * remembers the last scatter that read each staging buffer and makes the
 * next copy into that buffer wait for it, so alternating two staging
 * buffers overlaps the fetch of one layer with the scatter of another.
 *
 * FCDP_SRC_HOST_SCATTER_DMA: every tensor is contiguous in the cached flat
 * image, so T copies on `copy` move host_cache[off_t .. off_t + n_t) straight
 * into tensor t; no staging buffer and no kernel.  The copies wait for what
 * is enqueued on `compute` before the call (earlier readers of the tensors),
 * and `compute` waits for the copies.
 *
 * FCDP_SRC_HOST_ZEROCOPY: one kernel on `compute` reads host_cache through
 * its device mapping and writes the tensors; ordered after everything
 * enqueued on `copy` before this call.  host_cache must be mapped pinned
 * host memory (fcdp_host_cache_alloc), else FCDP_ENOTPINNED.
 *
 *   shard_ptrs   host array of G dev ptrs, S*elem_size bytes each
 *                (DEVICE_SHARDS only, else may be NULL)
 *   host_cache   host ptr to N_pad*elem_size bytes of pinned memory; read
 *                for HOST_*, written when store_cache is set; else may be NULL.
 *                Every host-link path checks it: memory HIP does not know as
 *                pinned host memory (malloc, numpy, pageable) is refused with
 *                FCDP_ENOTPINNED before anything is enqueued, because a copy
 *                from or to pageable memory is not asynchronous and would
 *                silently serialise the cache traffic with the kernels; the
 *                zero-copy paths also need it mapped (fcdp_host_cache_alloc)
 *   staging      dev ptr to N_pad*elem_size bytes (HOST_DMA only)
 *   tensor_ptrs  host array of T dev ptrs, numel[t]*elem_size bytes each
 *                (entries of zero-element tensors are ignored)
 * Results are valid in `compute`-stream order (tensors) and `copy`-stream
 * order (host_cache).  Padding is never read into a tensor.
 */
fcdp_status fcdp_materialize_layer(const fcdp_layout *layout, fcdp_source src,
                                   const void *const *shard_ptrs,
                                   void *host_cache, void *staging,
                                   void *const *tensor_ptrs, int store_cache,
                                   fcdp_stream compute, fcdp_stream copy);

/* The FCDP_SRC_HOST_DMA fetch for callers that cannot allocate device memory
 * or pass a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It does what fcdp_materialize_layer(layout,
 * FCDP_SRC_HOST_DMA, NULL, host_cache, staging, tensor_ptrs, FCDP_STORE_NONE,
 * compute, copy) does, with the staging buffer taken from a fixed array of
 * FCDP_STATIC_STAGING_BYTES bytes that is part of the library's device image
 * (every GPU the library runs on holds one until the process ends).  The call
 * itself allocates nothing, uploads nothing and creates no event: the
 * layout's tables, the array's address and the two events it uses are made by
 * fcdp_layout_prepare, which must have been called for this layout on the
 * current device (else FCDP_ESTATE).
 *   host_cache   host ptr to N_pad*elem_size bytes of pinned memory
 *   tensor_ptrs  host array of T dev ptrs, as for fcdp_materialize_layer
 * Errors: N_pad*elem_size > FCDP_STATIC_STAGING_BYTES -> FCDP_ESIZE (nothing
 * is enqueued); NULL / misaligned pointers as for fcdp_materialize_layer.
 * The array needs no clearing: each call overwrites the N_pad*elem_size bytes
 * it then reads, and bytes left by an earlier, larger layer are never read.
 * All calls on one GPU share the array.  A call orders its copy after the
 * previous call's scatter, so calls issued one after another from one thread
 * (or serialised by the caller) are safe on any streams; calls issued
 * concurrently from several threads on one GPU race on the array's contents
 * and must be serialised by the caller.  The copy is not counted against
 * max_copies_in_flight (it is at most FCDP_STATIC_STAGING_BYTES long). */
#define FCDP_STATIC_STAGING_BYTES (32u << 20)
fcdp_status fcdp_materialize_layer_static(const fcdp_layout *layout,
                                          void *host_cache,
                                          void *const *tensor_ptrs,
                                          fcdp_stream compute,
                                          fcdp_stream copy);

/* The cache store alone (Alg. 1: the dirty branch's refresh of the host
 * copy), for callers that decide after
 * the layer's forward computation whether to offload it (Sec. 4.4): copies
 * concat(shard_0..shard_{G-1}) to host_cache on `copy`, ordered after what is
 * enqueued on `compute` at the time of the call.  store_mode is FCDP_STORE_DMA
 * or FCDP_STORE_ZEROCOPY; arguments as for fcdp_materialize_layer. */
fcdp_status fcdp_cache_store(const fcdp_layout *layout,
                             const void *const *shard_ptrs, void *host_cache,
                             int store_mode, fcdp_stream compute,
                             fcdp_stream copy);

/* One GPU's share when a node has g GPUs (Sec. 4.3, backward pass: each GPU
 * loads its 1/g part of the cached layer from host memory over its own link,
 * then the node's GPUs exchange their parts; Sec. 5.1: the node caches the
 * layer once, about 2W bytes per node).  This GPU's part is the n_shards
 * consecutive rank shards [first_shard, first_shard + n_shards), n_shards =
 * G/g in the paper's setting (any 1..G here).
 *
 * fcdp_cache_store_node_slice: host_slice <- shard_first .. shard_{first +
 * n_shards - 1} by DMA on `copy`, ordered after what is enqueued on `compute`.
 *   shard_ptrs   host array of G dev ptrs; only the entries of the slice are
 *                read (the others may be NULL)
 *   host_slice   pinned host ptr, n_shards*S*elem_size bytes
 *
 * fcdp_materialize_layer_node_slice: the layer's tensors from this GPU's
 * cached part and the parts the peers delivered.  host_slice is copied to
 * staging_slice on `copy` (with the same staging-buffer bookkeeping as
 * FCDP_SRC_HOST_DMA, so two staging slices alternate without host waits),
 * then one scatter on `compute` reads the slice's shards from staging_slice
 * and every other shard from shard_ptrs.
 *   shard_ptrs     host array of G dev ptrs; entries outside the slice are
 *                  the peers' shards, S*elem_size bytes each, valid in
 *                  compute-stream order (how they got there -- an exchange
 *                  over the node's links -- is not this library's business);
 *                  entries inside the slice are ignored
 *   host_slice     pinned host ptr, n_shards*S*elem_size bytes
 *   staging_slice  dev ptr, n_shards*S*elem_size bytes
 * Over the host link go n_shards*S*elem_size bytes per call (fcdp_link_bytes
 * counts that).  Errors: FCDP_EINVAL (NULL, a slice outside [0, G)),
 * FCDP_EALIGN, FCDP_ENOTPINNED, FCDP_EHIP. */
fcdp_status fcdp_cache_store_node_slice(const fcdp_layout *layout,
                                        int32_t first_shard, int32_t n_shards,
                                        const void *const *shard_ptrs,
                                        void *host_slice, fcdp_stream compute,
                                        fcdp_stream copy);
fcdp_status fcdp_materialize_layer_node_slice(const fcdp_layout *layout,
                                              int32_t first_shard,
                                              int32_t n_shards,
                                              const void *const *shard_ptrs,
                                              void *host_slice,
                                              void *staging_slice,
                                              void *const *tensor_ptrs,
                                              fcdp_stream compute,
                                              fcdp_stream copy);

/* Inverse of the scatter, for initialisation and tests: writes the G shards
 * from the T tensors and zero-fills the tail padding. */
fcdp_status fcdp_flatten_to_shards(const fcdp_layout *layout,
                                   const void *const *tensor_ptrs,
                                   void *const *shard_ptrs, fcdp_stream stream);

/* ------------------------------------------------------ gradient-shard sum
 * The local half of the gradient reduce-scatter (Sec. 2.1; Sec. 6.2
 * the gradient reduce-scatter; Alg. 1: the reduce-scatter of the trainable gradients): for k in
 * [0, count)
 *     acc = p_0[e0+k];  acc = acc + p_g[e0+k]  for g = 1..G-1, in that order
 *     out[k] = acc                      (out == FCDP_F32)
 *     out[k] = bf16(acc), nearest-even  (out == FCDP_BF16)
 * in IEEE binary32 with one rounding per addition, denormals kept.  The sum,
 * not the mean, is produced.  NaN in gives NaN out; which NaN payload is not
 * specified.
 *   partial_ptrs  host array of G dev ptrs to rank g's buffer base
 *   elem_offset   e0: r*S for a whole flat gradient, 0 if the pointers
 *                 already address the slice
 *   in            dtype of the partials (FCDP_F32 or FCDP_BF16)
 *   out_shard     dev ptr, count elements of dtype `out`.  It may be exactly
 *                 partial_ptrs[g] + e0 for one g when in == out (in place);
 *                 any other overlap with an input is FCDP_EINVAL.
 * Errors: G outside 1..FCDP_MAX_G -> FCDP_ESIZE; count < 0 or e0 < 0 ->
 * FCDP_EINVAL.
 */
fcdp_status fcdp_reduce_grad_shard(const void *const *partial_ptrs, int32_t G,
                                   int64_t elem_offset, int64_t count,
                                   fcdp_dtype in, fcdp_dtype out,
                                   void *out_shard, fcdp_stream stream);

/* Gradient-shard sum of the trainable parameters straight from G unpacked
 * flat gradients: pack and reduce in one launch (Alg. 1: the reduce-scatter of the
 * trainable gradients; Sec. 4.5: only trainable parameters take part).  With Sp =
 * packed_numel / G and pk(.) the packed order of fcdp_pack_trainable,
 *     out[k] = sum over g = 0..G-1, in that order, of grad_g[flat index of
 *              packed element rank*Sp + k],     k in [0, Sp)
 * under the arithmetic of fcdp_reduce_grad_shard; packed positions beyond
 * N_t (the zero tail) give +0.
 *   flat_grad_ptrs  host array of G dev ptrs (G = the layout's G), each a
 *                   flat gradient of N_pad elements of dtype `in`
 *   rank            which shard of the packed buffer to produce, 0..G-1
 *   out_shard       dev ptr, Sp elements of dtype `out`; must not overlap
 *                   any input
 */
fcdp_status fcdp_reduce_trainable_shard(const fcdp_layout *layout,
                                        const void *const *flat_grad_ptrs,
                                        int32_t rank, fcdp_dtype in,
                                        fcdp_dtype out, void *out_shard,
                                        fcdp_stream stream);

/* The two sums above followed by one multiplication.  Alg. 1 names the
 * collective (a reduce-scatter of the trainable gradients) without saying whether ranks are
 * summed or averaged; scale = 1/G gives the mean, and a loss-scale's inverse
 * can ride along.  For every output element
 *     acc = the rank-order sum as defined above
 *     out[k] = acc * scale               one more binary32 rounding
 *     (then the bf16 rounding when out == FCDP_BF16)
 * The scale multiplies the finished sum, never the terms, and it is a
 * multiplication by the given float (not a division by G).  scale = 1 gives
 * the unscaled entry points' results bit for bit; zero-tail positions of the
 * trainable variant give (+0) * scale.  A scale that is not finite is
 * FCDP_EINVAL; all other arguments and errors are those of the unscaled
 * entry points. */
fcdp_status fcdp_reduce_grad_shard_scaled(const void *const *partial_ptrs,
                                          int32_t G, int64_t elem_offset,
                                          int64_t count, fcdp_dtype in,
                                          fcdp_dtype out, float scale,
                                          void *out_shard, fcdp_stream stream);
fcdp_status fcdp_reduce_trainable_shard_scaled(const fcdp_layout *layout,
                                               const void *const *flat_grad_ptrs,
                                               int32_t rank, fcdp_dtype in,
                                               fcdp_dtype out, float scale,
                                               void *out_shard,
                                               fcdp_stream stream);

/* --------------------------------------------------- PEFT pack and unpack
 * Under PEFT only trainable parameters cross the node boundary (Sec. 4.5,
 * Alg. 1's dirty branch and its reduce-scatter of grad W_t).
 * Pack: the flat ranges of the trainable tensors, in tensor order, are
 * copied end to end into `packed`; packed[N_t .. packed_numel) is set to 0.
 * Unpack: the inverse writes; no other byte of `flat` is written (frozen
 * parameters and the tail padding are left as they are).
 *   flat    dev ptr, N_pad elements (unpack: may also be the device alias of
 *           a mapped host cache, which refreshes H for W_t only)
 *   packed  dev ptr, packed_numel elements
 * flat and packed must not overlap.
 */
fcdp_status fcdp_pack_trainable(const fcdp_layout *layout, const void *flat,
                                void *packed, fcdp_stream stream);
fcdp_status fcdp_unpack_trainable(const fcdp_layout *layout,
                                  const void *packed, void *flat,
                                  fcdp_stream stream);
/* Unpack for a GPU that holds only its node slice of the flat image (the
 * shards [first_shard, first_shard + n_shards), see
 * fcdp_materialize_layer_node_slice): writes the trainable elements that
 * fall into those shards and nothing else.
 *   packed      dev ptr, packed_numel elements (the whole packed buffer)
 *   flat_slice  dev ptr, n_shards*S elements: the slice, e.g. the device
 *               alias of this GPU's part of the mapped host cache (Alg. 1's
 *               refresh of H for W_t, on this GPU's share)
 * Errors as for fcdp_unpack_trainable, FCDP_EINVAL for a slice outside [0, G). */
fcdp_status fcdp_unpack_trainable_node_slice(const fcdp_layout *layout,
                                             int32_t first_shard,
                                             int32_t n_shards,
                                             const void *packed,
                                             void *flat_slice,
                                             fcdp_stream stream);

/* ------------------------------------------------------------- host cache
 * Pinned, device-mapped host memory for the cache H (Sec. 4.4, host memory:
 * allocated once, kept for the whole run, updated in place,
 * taken from the NUMA node local to the GPU).  numa_node >= 0 binds the
 * pages to that node (best effort: if the kernel refuses the policy the
 * allocation still succeeds and fcdp_last_error() says so); -1 = no policy.
 * *host is the host address, *dev_alias the address kernels use.
 */
fcdp_status fcdp_host_cache_alloc(size_t bytes, int numa_node, void **host,
                                  void **dev_alias);
fcdp_status fcdp_host_cache_free(void *host);

/* ------------------------------------------------------------ dirty state
 * The cache-validity flags of Alg. 1, per (layer, class) with class 0 =
 * frozen, 1 = trainable.  All flags start dirty (nothing is cached yet).
 * forward_source: a dirty class must be served from the gathered device
 * shards and stored (*src = DEVICE_SHARDS, *store_cache = 1) and becomes
 * clean; a clean class is served from the host cache (*src = host_mode,
 * *store_cache = 0).  backward_source: always the host cache; FCDP_ESTATE if
 * the class is still dirty (no forward has stored it).  optimizer_step marks
 * the trainable class of every layer dirty (frozen stays clean for ever).
 * host_mode must be one of the three FCDP_SRC_HOST_* sources.
 */
fcdp_status fcdp_cache_state_create(int32_t n_layers, fcdp_cache_state **out);
void fcdp_cache_state_destroy(fcdp_cache_state *state);
fcdp_status fcdp_cache_state_forward_source(fcdp_cache_state *state,
                                            int32_t layer, int32_t klass,
                                            fcdp_source host_mode,
                                            fcdp_source *src,
                                            int32_t *store_cache);
fcdp_status fcdp_cache_state_backward_source(const fcdp_cache_state *state,
                                             int32_t layer, int32_t klass,
                                             fcdp_source host_mode,
                                             fcdp_source *src);
fcdp_status fcdp_cache_state_optimizer_step(fcdp_cache_state *state);
/* forward_source marks a class clean when it hands it out for storing,
 * before the store is enqueued.  If that store (fcdp_materialize_layer with
 * store_cache, or fcdp_cache_store) then fails, the host image was never
 * written: call this to make the class dirty again, so that backward_source
 * answers FCDP_ESTATE instead of serving it and the next forward pass takes
 * the miss path.  Also ends the layer's device residency. */
fcdp_status fcdp_cache_state_mark_dirty(fcdp_cache_state *state, int32_t layer,
                                        int32_t klass);
/* 1 dirty, 0 clean, -1 bad argument */
int32_t fcdp_cache_state_is_dirty(const fcdp_cache_state *state, int32_t layer,
                                  int32_t klass);

/* Adaptive placement (Sec. 4.4, adaptive GPU caching).  tau in [0, 1]; the
 * default 0 offloads every layer (the plain schedule of Sec. 4.3).
 * fcdp_cache_state_place is the decision at the "cache on CPU" point of a
 * layer, after its forward computation: utilisation = used_bytes /
 * total_bytes of device memory as the caller measures it at that moment.
 *   *keep = 1  utilisation < tau: the layer's parameters stay on the device
 *              until its backward pass; the caller issues neither store nor
 *              fetch, backward_source answers FCDP_SRC_DEVICE_RESIDENT, and
 *              every class that forward_source had just handed out for
 *              storing is dirty again (the host copy was not refreshed);
 *   *keep = 0  offload as usual (the caller issues the store now).
 * fcdp_cache_state_release ends a layer's residency (after its backward
 * pass); fcdp_cache_state_optimizer_step ends all of them. */
fcdp_status fcdp_cache_state_set_tau(fcdp_cache_state *state, double tau);
fcdp_status fcdp_cache_state_place(fcdp_cache_state *state, int32_t layer,
                                   int64_t used_bytes, int64_t total_bytes,
                                   int32_t *keep);
fcdp_status fcdp_cache_state_release(fcdp_cache_state *state, int32_t layer);

/* Bytes of layer images this process has moved over the host link through
 * the library on the current device since the last reset: N_pad*elem_size per
 * cache store (device to host) and per cache fetch (host to device), counted
 * the same way for every mode (the zero-copy and per-tensor fetches leave the
 * tail padding, fewer than G*pad_quantum elements, off the wire).  The
 * counters are atomic; data calls from several threads may add to them. */
fcdp_status fcdp_link_bytes(int32_t reset, int64_t *stored, int64_t *fetched);

/* ------------------------------------------------------------------- misc */
const char *fcdp_status_string(fcdp_status status);
const char *fcdp_last_error(void);

/* Launch-shape knobs for measurement sweeps.  Unknown name or a value outside
 * its range -> FCDP_EINVAL.  Not needed for normal use; the defaults are the
 * measured best on MI355X.  Process-wide, not synchronised with data calls.
 *   copy_chunk_bytes      piece size of the copy plans, multiple of 4096 in
 *                         4096..16 MiB (4096); applies to layouts built later
 *   copy_block            threads per workgroup of the copy kernels, power of
 *                         two in 64..1024 (128)
 *   copy_unroll           16-byte vectors in flight per lane: 1, 2, 4, 8 (1)
 *   copy_nt               non-temporal hint, bit 0 loads, bit 1 stores (3)
 *   copy_wg_per_cu        cap on workgroups per compute unit, 0 = none (0)
 *   reduce_block          threads per workgroup of the one-tile-per-workgroup
 *                         reduce kernel, 64..256 (64)
 *   reduce_phased         which reduce kernel runs: 0 one tile per workgroup,
 *                         stored as soon as it is summed; 1 the phased kernel
 *                         (a persistent grid whose waves keep their sums in
 *                         registers and store them after their last load, so
 *                         that the chip reads, then writes) whenever slices
 *                         and output are 16-byte aligned and at least 8 steps
 *                         per wave long; 2 the phased kernel where it measured
 *                         faster (2): G a multiple of 8 takes it at one wave
 *                         per SIMD (bf16 partials into a bf16 shard at G = 8:
 *                         two); other G take it at two waves per SIMD from
 *                         G = 3 on when partials and shard have one type, from
 *                         G = 5 on for fp32 partials into a bf16 shard, from
 *                         G = 12 on for bf16 partials into an fp32 shard; and
 *                         by length: an input beyond what one launch holds
 *                         (waves x held steps: 27.26 M elements on a 256-CU
 *                         part) takes full launches and then the rest; a
 *                         launch filled below 0.7 of that takes two waves
 *                         per SIMD if G >= 12, else one tile per workgroup,
 *                         as does any launch filled below 0.46.
 *                         The result is the same bits either way.
 *   reduce_phase_waves    waves per SIMD of the phased kernel: 1 (104 steps
 *                         held per wave; built for G a multiple of 8 only,
 *                         other G take 2), 2 (52 steps), 0 by rule (0)
 *   reduce_phase_rotate   where a wave of the phased kernel starts its run
 *                         of steps: 0 at the first step, 2 at step
 *                         (wave index mod run length), wrapping around,
 *                         1 the second only for the run lengths at which
 *                         the first measured slow (1)
 *   link_max_wgs          workgroups of the zero-copy fetch / store kernels,
 *                         0 = no bound (64)
 *   link_block            their threads per workgroup (256)
 *   link_chunk_bytes      bytes per workgroup trip of the store kernel (16384)
 *   max_copies_in_flight  host-link DMA copies queued before a call blocks
 *                         on the oldest, 0 = no bound (2)
 *   debug_poison          0 or 1 (0; the environment variable
 *                         FCDP_DEBUG_POISON=1 turns it on at load).  A debugging
 *                         aid: fcdp_materialize_layer first fills every tensor
 *                         of the layer with the 16-bit pattern 0x7FC1 (a bf16
 *                         NaN) on `compute`, the staging buffer on `copy` ahead
 *                         of the fetch, and a store first fills a mapped host
 *                         cache on `copy`; a consumer that misses one of the
 *                         documented waits then reads NaNs instead of stale
 *                         bytes that may happen to be right.  Results are
 *                         unchanged; each call costs one more pass.  With
 *                         the knob on the data calls also look every device
 *                         buffer up with hipMemGetAddressRange: one that does
 *                         not lie inside a single allocation with at least
 *                         the documented number of bytes is FCDP_ESIZE
 *                         before anything is enqueued (no sizes cross this
 *                         boundary, so normal operation cannot check them).
 * Read only (fcdp_tuning_set answers FCDP_EINVAL, as for an unknown name):
 *   last_reduce_shape     what the last fcdp_reduce_grad_shard[_scaled] of the
 *                         process launched (first, if it took several
 *                         launches): 0 one tile per workgroup, 1 or 2 the
 *                         phased kernel with that many waves per SIMD */
fcdp_status fcdp_tuning_set(const char *name, int64_t value);
int64_t fcdp_tuning_get(const char *name); /* -1 if unknown */

/* Kernel timing for measurement.  While enabled, every kernel dispatch the
 * library makes on the current device carries a start and a stop event that
 * take the dispatch's own begin and end timestamps on its stream (at most
 * `capacity` dispatches are kept; later ones are not timed).  A reduce that
 * takes several dispatches (an input longer than one launch of the phased
 * kernel holds) counts as one: its start is taken on the first dispatch and
 * its stop on the last.  fcdp_timing_collect waits for the recorded launches
 * of one kind, returns how many there were and the sum of their durations in
 * milliseconds, and forgets them.  fcdp_timing_enable(0) disables timing and
 * frees the events.  Not thread-safe against concurrent data calls. */
typedef enum {
    FCDP_KERNEL_UNFLATTEN = 0,          /* shards or staging -> tensors */
    FCDP_KERNEL_UNFLATTEN_ZEROCOPY = 1, /* mapped host cache -> tensors */
    FCDP_KERNEL_FLATTEN = 2,
    FCDP_KERNEL_REDUCE = 3,
    FCDP_KERNEL_PACK = 4,
    FCDP_KERNEL_UNPACK = 5,
    FCDP_KERNEL_STORE_ZEROCOPY = 6,
    FCDP_KERNEL_PROBE_COPY = 7,
    FCDP_KERNEL_REDUCE_TRAINABLE = 8,
    FCDP_KERNEL_PROBE_STREAM = 9
} fcdp_kernel_kind;
fcdp_status fcdp_timing_enable(int32_t capacity);
fcdp_status fcdp_timing_collect(int32_t kind, int64_t *launches, double *total_ms);

/* A plain contiguous device copy of `bytes` bytes with the same inner loop as
 * the scatter kernels; the known-size reference used to calibrate hardware
 * byte counters and to state the copy speed this GPU reaches. */
fcdp_status fcdp_probe_copy(void *dst, const void *src, size_t bytes,
                            fcdp_stream stream);

/* The gradient-shard sum's mix of G reads to 1 write as ONE contiguous
 * stream, the known-pattern reference next to which the reduce kernels are
 * measured: tile t of dst (1024 elements) is the sum, in order, of the G
 * consecutive 1024-element sub-tiles of src that start at element
 * t * G * 1024, stored as soon as it is summed (same loads, adds and stores
 * per output element as the one-tile-per-workgroup reduce kernel).
 *   src    dev ptr, G * count fp32 elements
 *   dst    dev ptr, count elements of dtype `out`; must not overlap src
 *   count  a multiple of 1024 (else FCDP_EINVAL) */
fcdp_status fcdp_probe_reduce_stream(void *dst, const void *src, int32_t G,
                                     int64_t count, fcdp_dtype out,
                                     fcdp_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* FCDP_H */
