/*
 * fcdp_oracle.c -- plain CPU oracle for the FCDP per-layer hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product (the HIP library, its
 * Python binding) may include, link or call this file; only the tests, the
 * smoke check and the benchmark's cpu_baseline leg do.  It shares no code,
 * header, table or constant with the HIP path.
 *
 * Every function below is the definition of the operation written out as
 * scalar loops, one element at a time, in the order the definition states.
 * There is no blocking, no vector code and no reordering; speed is whatever
 * "gcc -O2" makes of it.
 *
 * Notation (paper Sec. 6.1 plus the flat-parameter layout the problem
 * statement fixes): a layer has T tensors with n[t] elements; off[t] is the
 * running sum; N = off[T]; Q = G*q (q = 64); N_pad = ceil(N/Q)*Q;
 * S = N_pad/G.  Flat index i lives in shard (i div S) at position (i mod S).
 * Each of the G data-parallel ranks owns one shard of S = W_l/G elements
 * (the sharding of Sec. 2.1; the per-GPU parameter memory of Sec. 6.1).
 *
 * Parity pins: every function here is pinned by tests that do not use it to
 * check itself (invariants, closed forms from Sec. 5.1 / Sec. 6.1, numpy and
 * PyTorch-CPU library routines, pure-Python brute force on tiny layers).
 * No function is "parity unpinned".
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_EINVAL 1

/* ------------------------------------------------------------------ layout */

/*
 * Offset table.  off has T+1 entries.  (Sec. 2.1 / Sec. 6.1: parameters are
 * split evenly over all G GPUs.  The paper does not print the layout it
 * inherits; the reading used here: tensors end to end in the order given,
 * tightly packed, zero elements at the tail up to a multiple of G*q.)
 */
int fcdp_oracle_layout(const int64_t *n, int32_t T, int32_t G, int32_t q,
                       int64_t *off, int64_t *N_out, int64_t *N_pad_out,
                       int64_t *S_out)
{
    if (T < 0 || G < 1 || q < 1) return ORACLE_EINVAL;
    off[0] = 0;
    for (int32_t t = 0; t < T; ++t) {
        if (n[t] < 0) return ORACLE_EINVAL;
        off[t + 1] = off[t] + n[t];
    }
    int64_t N = off[T];
    int64_t Q = (int64_t)G * (int64_t)q;
    int64_t N_pad = ((N + Q - 1) / Q) * Q;
    *N_out = N;
    *N_pad_out = N_pad;
    *S_out = N_pad / G;
    return ORACLE_OK;
}

/* Copy one element of esz bytes. */
static void put_elem(unsigned char *dst, int64_t di, const unsigned char *src,
                     int64_t si, int32_t esz)
{
    for (int32_t b = 0; b < esz; ++b)
        dst[di * esz + b] = src[si * esz + b];
}

/*
 * Flatten: flat[off[t]+j] = tensor_t[j]; flat[N..N_pad) = 0.
 * flat has N_pad elements of esz bytes.
 */
int fcdp_oracle_flatten(const void *const *tensors, const int64_t *n,
                        int32_t T, int32_t G, int32_t q, int32_t esz,
                        void *flat)
{
    if (G < 1 || q < 1) return ORACLE_EINVAL;
    unsigned char *f = (unsigned char *)flat;
    int64_t off_t = 0;
    for (int32_t t = 0; t < T; ++t) {
        if (n[t] < 0) return ORACLE_EINVAL;
        const unsigned char *src = (const unsigned char *)tensors[t];
        for (int64_t j = 0; j < n[t]; ++j)
            put_elem(f, off_t + j, src, j, esz);
        off_t += n[t];
    }
    int64_t N = off_t;
    int64_t Q = (int64_t)G * (int64_t)q;
    int64_t N_pad = ((N + Q - 1) / Q) * Q;
    for (int64_t i = N; i < N_pad; ++i)
        for (int32_t b = 0; b < esz; ++b)
            f[i * esz + b] = 0;
    return ORACLE_OK;
}

/* shard_r[k] = flat[r*S + k]  for every rank r. */
int fcdp_oracle_split(const void *flat, int64_t S, int32_t G, int32_t esz,
                      void *const *shards)
{
    const unsigned char *f = (const unsigned char *)flat;
    for (int32_t r = 0; r < G; ++r) {
        unsigned char *s = (unsigned char *)shards[r];
        for (int64_t k = 0; k < S; ++k)
            put_elem(s, k, f, (int64_t)r * S + k, esz);
    }
    return ORACLE_OK;
}

/*
 * Materialize from G rank shards (the receive side of the forward
 * all-gather, Sec. 4.3 forward pass; Alg. 1: the dirty branch's inter-node gather):
 *   tensor_t[j] = shard_{(off_t+j) div S}[(off_t+j) mod S].
 * Padding is never read.
 */
int fcdp_oracle_materialize_from_shards(const void *const *shards, int64_t S,
                                        int32_t G, const int64_t *n, int32_t T,
                                        int32_t esz, void *const *tensors)
{
    int64_t off_t = 0;
    for (int32_t t = 0; t < T; ++t) {
        unsigned char *dst = (unsigned char *)tensors[t];
        for (int64_t j = 0; j < n[t]; ++j) {
            int64_t i = off_t + j;
            int64_t r = i / S;
            int64_t k = i % S;
            if (r >= G) return ORACLE_EINVAL;
            put_elem(dst, j, (const unsigned char *)shards[r], k, esz);
        }
        off_t += n[t];
    }
    return ORACLE_OK;
}

/*
 * Materialize from the host cache H_l, which holds the padded flat image of
 * the layer in shard order (Sec. 4.3 backward pass; Alg. 1: the load of the
 * cached copy from the host
 * followed by the intra-node gather, which on one GPU is the whole layer):
 *   tensor_t[j] = H[off_t + j].
 */
int fcdp_oracle_materialize_from_flat(const void *flat, const int64_t *n,
                                      int32_t T, int32_t esz,
                                      void *const *tensors)
{
    const unsigned char *f = (const unsigned char *)flat;
    int64_t off_t = 0;
    for (int32_t t = 0; t < T; ++t) {
        unsigned char *dst = (unsigned char *)tensors[t];
        for (int64_t j = 0; j < n[t]; ++j)
            put_elem(dst, j, f, off_t + j, esz);
        off_t += n[t];
    }
    return ORACLE_OK;
}

/*
 * Cache store (Alg. 1: the dirty branch's refresh of the host copy, GPU to host): H = concat(shard_0 ..
 * shard_{G-1}), padding included.
 */
int fcdp_oracle_cache_store(const void *const *shards, int64_t S, int32_t G,
                            int32_t esz, void *H)
{
    unsigned char *h = (unsigned char *)H;
    for (int32_t r = 0; r < G; ++r)
        for (int64_t k = 0; k < S; ++k)
            put_elem(h, (int64_t)r * S + k, (const unsigned char *)shards[r],
                     k, esz);
    return ORACLE_OK;
}

/*
 * Segment list: every non-empty intersection of a tensor's flat range with a
 * shard's flat range, in (tensor, shard) order.  Row = (t, r, dst_off,
 * src_off, len): len elements go from shard r at src_off to tensor t at
 * dst_off.  Returns the number of rows; writes at most cap rows of 5 int64.
 */
int64_t fcdp_oracle_segments(const int64_t *n, int32_t T, int32_t G, int32_t q,
                             int64_t *rows, int64_t cap)
{
    int64_t N = 0;
    for (int32_t t = 0; t < T; ++t) N += n[t];
    int64_t Q = (int64_t)G * (int64_t)q;
    int64_t N_pad = ((N + Q - 1) / Q) * Q;
    int64_t S = N_pad / G;
    int64_t count = 0;
    int64_t off_t = 0;
    for (int32_t t = 0; t < T; ++t) {
        for (int32_t r = 0; r < G; ++r) {
            int64_t lo = off_t > (int64_t)r * S ? off_t : (int64_t)r * S;
            int64_t hi_t = off_t + n[t];
            int64_t hi_r = ((int64_t)r + 1) * S;
            int64_t hi = hi_t < hi_r ? hi_t : hi_r;
            if (hi > lo) {
                if (count < cap) {
                    rows[count * 5 + 0] = t;
                    rows[count * 5 + 1] = r;
                    rows[count * 5 + 2] = lo - off_t;
                    rows[count * 5 + 3] = lo - (int64_t)r * S;
                    rows[count * 5 + 4] = hi - lo;
                }
                ++count;
            }
        }
        off_t += n[t];
    }
    return count;
}

/* ------------------------------------------------------------------ reduce */

static float bits_to_f32(uint32_t u)
{
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static uint32_t f32_to_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return u;
}

/* bf16 -> fp32 is exact: the 16 bits become the upper half of the word. */
static float bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }

/*
 * fp32 -> bf16, round to nearest, ties to even, on the upper 16 bits.
 * NaN stays NaN (quiet bit forced, sign kept); +-Inf is kept; a finite value
 * that rounds past the largest bf16 becomes +-Inf.
 */
uint16_t fcdp_oracle_bf16_rne(float x)
{
    uint32_t u = f32_to_bits(x);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

void fcdp_oracle_bf16_rne_array(const float *x, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = fcdp_oracle_bf16_rne(x[i]);
}

/*
 * Gradient-shard reduction (the local half of the reduce-scatter, Sec. 6.2
 * the gradient reduce-scatter; Alg. 1: the reduce-scatter of the trainable gradients):
 *   acc = p_0[e0+k]; acc = acc + p_g[e0+k] for g = 1 .. G-1, in that order,
 * in IEEE binary32 (one rounding per add; built without fast-math and
 * without contraction, so the compiler keeps this order), and
 *   out[k] = acc (fp32)  or  bf16_rne(acc).
 * in_dtype / out_dtype: 0 = bf16, 1 = fp32.  partials[g] is rank g's buffer
 * base; e0 is the element offset of this rank's slice (r*S).
 */
int fcdp_oracle_reduce(const void *const *partials, int32_t G, int64_t e0,
                       int64_t count, int32_t in_dtype, int32_t out_dtype,
                       void *out)
{
    if (G < 1 || count < 0) return ORACLE_EINVAL;
    for (int64_t k = 0; k < count; ++k) {
        float acc;
        if (in_dtype == 1)
            acc = ((const float *)partials[0])[e0 + k];
        else
            acc = bf16_to_f32(((const uint16_t *)partials[0])[e0 + k]);
        for (int32_t g = 1; g < G; ++g) {
            float v;
            if (in_dtype == 1)
                v = ((const float *)partials[g])[e0 + k];
            else
                v = bf16_to_f32(((const uint16_t *)partials[g])[e0 + k]);
            acc = acc + v;
        }
        if (out_dtype == 1)
            ((float *)out)[k] = acc;
        else
            ((uint16_t *)out)[k] = fcdp_oracle_bf16_rne(acc);
    }
    return ORACLE_OK;
}

/*
 * The same reduction followed by one multiplication (the mean over ranks when
 * scale = 1/G; Alg. 1 names the collective, not whether it sums or averages,
 * so both are offered):
 *   acc as above, then acc = acc * scale, one more binary32 rounding,
 *   out[k] = acc (fp32)  or  bf16_rne(acc).
 * The scale multiplies the finished sum, never the terms.
 */
int fcdp_oracle_reduce_scaled(const void *const *partials, int32_t G,
                              int64_t e0, int64_t count, int32_t in_dtype,
                              int32_t out_dtype, float scale, void *out)
{
    if (G < 1 || count < 0) return ORACLE_EINVAL;
    for (int64_t k = 0; k < count; ++k) {
        float acc;
        if (in_dtype == 1)
            acc = ((const float *)partials[0])[e0 + k];
        else
            acc = bf16_to_f32(((const uint16_t *)partials[0])[e0 + k]);
        for (int32_t g = 1; g < G; ++g) {
            float v;
            if (in_dtype == 1)
                v = ((const float *)partials[g])[e0 + k];
            else
                v = bf16_to_f32(((const uint16_t *)partials[g])[e0 + k]);
            acc = acc + v;
        }
        acc = acc * scale;
        if (out_dtype == 1)
            ((float *)out)[k] = acc;
        else
            ((uint16_t *)out)[k] = fcdp_oracle_bf16_rne(acc);
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------- pack/unpack */

/*
 * Pack (what travels under PEFT is the trainable subset only, Sec. 4.5 and
 * Alg. 1's dirty branch): walk tensors in order; every trainable tensor's
 * flat range is appended to packed; packed is then zero-filled up to
 * packed_numel = ceil(N_t / Q) * Q.  Returns N_t through *Nt_out.
 */
int fcdp_oracle_pack(const void *flat, const int64_t *n,
                     const uint8_t *trainable, int32_t T, int32_t G, int32_t q,
                     int32_t esz, void *packed, int64_t *Nt_out)
{
    const unsigned char *f = (const unsigned char *)flat;
    unsigned char *p = (unsigned char *)packed;
    int64_t off_t = 0, c = 0;
    for (int32_t t = 0; t < T; ++t) {
        if (trainable[t]) {
            for (int64_t j = 0; j < n[t]; ++j)
                put_elem(p, c + j, f, off_t + j, esz);
            c += n[t];
        }
        off_t += n[t];
    }
    int64_t Q = (int64_t)G * (int64_t)q;
    int64_t Np = ((c + Q - 1) / Q) * Q;
    for (int64_t i = c; i < Np; ++i)
        for (int32_t b = 0; b < esz; ++b) p[i * esz + b] = 0;
    *Nt_out = c;
    return ORACLE_OK;
}

/*
 * Unpack: the inverse writes, flat[off_t + j] = packed[c_t + j] for trainable
 * t; no other element of flat is written (frozen parameters and the tail
 * padding stay as they are).
 */
int fcdp_oracle_unpack(const void *packed, const int64_t *n,
                       const uint8_t *trainable, int32_t T, int32_t esz,
                       void *flat)
{
    const unsigned char *p = (const unsigned char *)packed;
    unsigned char *f = (unsigned char *)flat;
    int64_t off_t = 0, c = 0;
    for (int32_t t = 0; t < T; ++t) {
        if (trainable[t]) {
            for (int64_t j = 0; j < n[t]; ++j)
                put_elem(f, off_t + j, p, c + j, esz);
            c += n[t];
        }
        off_t += n[t];
    }
    return ORACLE_OK;
}
