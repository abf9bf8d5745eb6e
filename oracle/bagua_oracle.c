/*
 * bagua_oracle.c -- plain CPU definition of the compression hot path behind the
 * communication primitives of "BAGUA: Scaling up Distributed Learning with System
 * Relaxations" (Section 3.2 "Communication Primitives", Section 3.4 "Implementations
 * of Primitives", Section 3.5 "Tensor Bucketing and Memory Flattening").
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, obviously-correct reference that
 * the GPU library is checked against.  It shares no code with the GPU library, is never
 * loaded by the product path, and is only used by tests/, the smoke check and the
 * "cpu_baseline" leg of the benchmark.
 *
 * Everything is scalar C in IEEE-754 binary32, one rounding per written operation
 * (build with -ffp-contract=off, never -ffast-math, no -march flags), round-to-nearest-even.
 * The only parallelism is an optional OpenMP "parallel for" over independent chunks
 * (or peers), which cannot change any result bit.
 *
 * ---------------------------------------------------------------------------------
 * Readings of the paper taken here (the paper leaves these open):
 *
 *  R0  The lossy compression function Q of C_LP_S is left to the developer (Section 3.2,
 *      text under the C_LP_S equations).  Two Qs are defined here:
 *        MinMax-u8: per chunk of C consecutive elements, 256 uniformly spaced levels from
 *                   the chunk minimum to the chunk maximum, round to nearest level;
 *        Sign-1bit: per chunk, one bit per element (v >= 0) and one scale = mean |v|.
 *  R1  Error compensation (C_LP_S equations, Section 3.2).  The printed equations carry
 *      the stored error with a minus sign and index it inconsistently; the text says the
 *      state keeps the error of the previous compression so that it is compensated.
 *      Reading: v = x + delta ;  delta' = v - Q(v)  (same for the server state epsilon).
 *  R2  The primitives are stated as sums over workers / neighbours (C_FP_S, C_LP_S,
 *      D_FP_S, D_LP_S equations).  This build returns the average: the sum taken in
 *      ascending worker order, then one multiplication by fl(1/k) (fl(1/3) on the ring).
 *  R3  Quantiser rounding: round-half-to-even (rintf), then clamp to [0,255]; a NaN
 *      intermediate clamps to 0.
 *  R4  A chunk whose max equals its min encodes to all-zero codes and step 0.
 *  R5  min/max compare -0 and +0 as equal; the stored values are canonicalised by
 *      adding +0.0f.  NaN/Inf inputs are outside the preconditions.
 *  R6  Order of the per-chunk sum of |v| in the sign codec: 64 accumulators over groups
 *      of four elements, then a 6-level xor butterfly (function ordered_abs_sum below).
 *  R7  Ring topology (Section 3.4, "ring" peer allocation): N(i) = {i-1, i, i+1} mod k
 *      with uniform weight 1/3, all peers updated simultaneously from the old values.
 *  R8  D_LP_S (Section 3.2 equation, Section 3.4 last paragraph) is realised as
 *      compressed-difference exchange with a public copy xhat_i of every peer's
 *      replica: the wire carries Q(x_i - xhat_i).
 *  R9  Bit order of the sign codec: bit b of 32-bit word w is element 32w+b of the bucket.
 *  R10 Flatten (Section 3.5): tensors are copied to caller-given element offsets of one
 *      contiguous bucket, everything not covered by a tensor is +0.0f.
 *  R11 Bucket size and bucketing heuristic are not given (Section 3.1 "Bucketing"): the
 *      benchmark workloads use greedy 25 MiB buckets in definition order, padded to a multiple
 *      of k*C (that rule lives with the workload generators, not here).
 *  R12 Chunks are counted over the whole padded bucket, so each of the k ScatterReduce
 *      partitions (Section 3.4) is a whole number of chunks and one pass over n elements
 *      equals k servers each doing n/k; the server error state epsilon is one fp32[n] buffer,
 *      the concatenation of the k servers' partitions.
 *  R13 Chunk sizes come from the benchmark configurations (4096, 8192, 2048); any multiple of
 *      256 in [256, 16384] is accepted.
 *  R14 Scale of the sign codec: sum * fl(1/C) for a full chunk with C a power of two (an exact
 *      scaling), otherwise sum / (float)length.
 *  R15 A chunk whose range is so small that 255/range overflows follows the same formula
 *      (inf clamps to 255, NaN to 0).
 *  R16 The optimizer that follows the primitive on the flattened bucket is not fixed by the
 *      paper: SGD with optional weight decay and momentum (oracle_decompress_sgd_step).
 *  R17 Random peer strategy: N(i) = {i, peer[i]}, weight 1/2 (oracle_peer_avg_fp).
 *  R18 Hierarchical C_LP_S, intra-node stage: uncompressed average of the local workers, then
 *      the leader's Q with its error state (oracle_reduce_compress_minmax_u8).
 *  R20 1-bit Adam (Section 4.1 names it as C_LP_S with error compensation; its steps are those of
 *      the published algorithm it cites): Adam without bias correction; after the warm-up the
 *      variance is frozen, every worker forms its local momentum beta1*m + (1-beta1)*g and
 *      compresses that; the decoded average replaces the momentum and drives the update
 *      (oracle_momentum_sign_compress_ef, oracle_decompress_adam_step).
 *
 * Status codes: 0 ok, 1 invalid argument.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

/* Number of OpenMP threads used for the loops over independent chunks (default 1). */
void oracle_set_threads(int t) { g_threads = t < 1 ? 1 : t; }
int oracle_get_threads(void) { return g_threads; }
int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int chunk_ok(size_t chunk) { return chunk >= 256 && chunk <= 16384 && chunk % 256 == 0; }
static size_t num_chunks(size_t n, size_t chunk) { return (n + chunk - 1) / chunk; }

/* ------------------------------------------------------------------ MinMax-u8 codec */

/* Quantisation step of a chunk from its stored (min,max): fl(fl(max-min)/255), 0 for a flat chunk (R4). */
static float minmax_step(float mn, float mx)
{
    float r = mx - mn;
    if (r == 0.0f) return 0.0f;
    return r / 255.0f;
}

/* Dequantise one code: fl(mn + fl(code*step)), two roundings. */
static float minmax_dequant(float mn, float step, uint8_t code)
{
    float p = (float)code * step;
    return mn + p;
}

/*
 * One chunk of Q := MinMax-u8 applied to v = x (+ residual), with the error update of
 * the C_LP_S equations under reading R1.  v is materialised in a scratch array first so
 * that the three stages (carry-in, statistics, quantise) read as in the definition.
 */
static void minmax_compress_chunk(const float* x, float* residual, size_t len,
                                  uint8_t* codes, float* mn_out, float* mx_out, float* v)
{
    size_t i;
    for (i = 0; i < len; ++i) v[i] = residual ? x[i] + residual[i] : x[i];

    float mn = v[0], mx = v[0];
    for (i = 1; i < len; ++i) {
        if (v[i] < mn) mn = v[i];
        if (v[i] > mx) mx = v[i];
    }
    mn = mn + 0.0f; /* R5: -0 -> +0 */
    mx = mx + 0.0f;

    float r = mx - mn;
    float step = minmax_step(mn, mx);
    float inv = (r == 0.0f) ? 0.0f : 255.0f / r;

    for (i = 0; i < len; ++i) {
        uint8_t c = 0;
        if (r != 0.0f) {
            float d = v[i] - mn;
            float t = d * inv;
            float q = rintf(t);            /* R3: half to even */
            if (!(q >= 0.0f)) q = 0.0f;    /* also catches NaN */
            if (q > 255.0f) q = 255.0f;
            c = (uint8_t)q;
        }
        codes[i] = c;
        if (residual) {
            float deq = minmax_dequant(mn, step, c);
            residual[i] = v[i] - deq;
        }
    }
    *mn_out = mn;
    *mx_out = mx;
}

/*
 * Worker side of C_LP_S (Section 3.2): codes = Q(x + delta), delta <- (x + delta) - Q(x + delta).
 * residual may be NULL (no error compensation: codes = Q(x)).
 * minmax holds (min,max) pairs, one per chunk.
 */
int oracle_compress_minmax_u8(const float* x, float* residual, size_t n, size_t chunk,
                              uint8_t* codes, float* minmax)
{
    if (!x || !codes || !minmax || n == 0 || !chunk_ok(chunk)) return 1;
    ptrdiff_t nc = (ptrdiff_t)num_chunks(n, chunk);
    ptrdiff_t c;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (c = 0; c < nc; ++c) {
        size_t lo = (size_t)c * chunk;
        size_t len = (lo + chunk <= n) ? chunk : n - lo;
        float* v = (float*)malloc(len * sizeof(float));
        minmax_compress_chunk(x + lo, residual ? residual + lo : NULL, len, codes + lo,
                              &minmax[2 * c], &minmax[2 * c + 1], v);
        free(v);
    }
    return 0;
}

/* Decompression of MinMax-u8: out_i = fl(mn + fl(code_i * step)). */
int oracle_decompress_minmax_u8(const uint8_t* codes, const float* minmax, size_t n, size_t chunk,
                                float* out)
{
    if (!codes || !minmax || !out || n == 0 || !chunk_ok(chunk)) return 1;
    ptrdiff_t nc = (ptrdiff_t)num_chunks(n, chunk);
    ptrdiff_t c;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (c = 0; c < nc; ++c) {
        size_t lo = (size_t)c * chunk;
        size_t len = (lo + chunk <= n) ? chunk : n - lo;
        float mn = minmax[2 * c], mx = minmax[2 * c + 1];
        float step = minmax_step(mn, mx);
        for (size_t i = 0; i < len; ++i) out[lo + i] = minmax_dequant(mn, step, codes[lo + i]);
    }
    return 0;
}

/*
 * Server side of C_LP_S (Section 3.2; steps 3-5 of ScatterReduce, Section 3.4) with
 * Q := MinMax-u8:  a = (sum_j deq_j) * fl(1/k) in ascending j (R2);
 * codes' = Q(a + epsilon);  epsilon <- (a + epsilon) - Q(a + epsilon);
 * out_fp32 (optional) = decompressed codes' = the tensor every worker ends up with.
 */
int oracle_drr_minmax_u8(const uint8_t* const* codes_in, const float* const* minmax_in, int k,
                         float* server_residual, size_t n, size_t chunk,
                         uint8_t* codes_out, float* minmax_out, float* out_fp32)
{
    if (!codes_in || !minmax_in || k < 1 || k > 32 || !codes_out || !minmax_out || n == 0 ||
        !chunk_ok(chunk))
        return 1;
    for (int j = 0; j < k; ++j)
        if (!codes_in[j] || !minmax_in[j]) return 1;
    float inv_k = 1.0f / (float)k;
    ptrdiff_t nc = (ptrdiff_t)num_chunks(n, chunk);
    ptrdiff_t c;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (c = 0; c < nc; ++c) {
        size_t lo = (size_t)c * chunk;
        size_t len = (lo + chunk <= n) ? chunk : n - lo;
        float* a = (float*)malloc(len * sizeof(float));
        float* v = (float*)malloc(len * sizeof(float));
        for (size_t i = 0; i < len; ++i) {
            float s = 0.0f;
            for (int j = 0; j < k; ++j) {
                float mn = minmax_in[j][2 * c], mx = minmax_in[j][2 * c + 1];
                float deq = minmax_dequant(mn, minmax_step(mn, mx), codes_in[j][lo + i]);
                s = (j == 0) ? deq : s + deq;
            }
            a[i] = s * inv_k;
        }
        minmax_compress_chunk(a, server_residual ? server_residual + lo : NULL, len,
                              codes_out + lo, &minmax_out[2 * c], &minmax_out[2 * c + 1], v);
        if (out_fp32) {
            float mn = minmax_out[2 * c], mx = minmax_out[2 * c + 1];
            float step = minmax_step(mn, mx);
            for (size_t i = 0; i < len; ++i)
                out_fp32[lo + i] = minmax_dequant(mn, step, codes_out[lo + i]);
        }
        free(a);
        free(v);
    }
    return 0;
}

/* ------------------------------------------------------------- decentralised averaging */

/*
 * D_FP_S on a ring (Section 3.2 equation; Section 3.4 "ring"), reading R7/R2:
 * x_i' = ((x_{i-1} + x_i) + x_{i+1}) * fl(1/3), indices mod k, from the old values.
 * Outputs must not alias inputs.
 */
int oracle_ring_avg_fp(const float* const* x_in, float* const* x_out, int k, size_t n)
{
    if (!x_in || !x_out || k < 1 || k > 32 || n == 0) return 1;
    for (int i = 0; i < k; ++i)
        if (!x_in[i] || !x_out[i]) return 1;
    float third = 1.0f / 3.0f;
    for (int i = 0; i < k; ++i) {
        const float* l = x_in[(i + k - 1) % k];
        const float* m = x_in[i];
        const float* r = x_in[(i + 1) % k];
        float* o = x_out[i];
        ptrdiff_t e;
#pragma omp parallel for schedule(static) num_threads(g_threads)
        for (e = 0; e < (ptrdiff_t)n; ++e) {
            float s = l[e] + m[e];
            s = s + r[e];
            o[e] = s * third;
        }
    }
    return 0;
}

/*
 * D_LP_S on a ring, one round, reading R8.  For every peer i:
 *   d_i = x_i - xhat_i ;  (codes_i, minmax_i) = Q(d_i) without error state ;
 *   xhat_i <- xhat_i + dequant(codes_i, minmax_i)          (what every holder of the copy does)
 * then, from the updated copies,
 *   x_i' = ((xhat_{i-1} + xhat_i) + xhat_{i+1}) * fl(1/3) + (x_i - xhat_i).
 * xhat is updated in place; x_out must not alias x_in or xhat.
 */
int oracle_ring_avg_lp(const float* const* x_in, float* const* x_out, float* const* xhat,
                       uint8_t* const* codes, float* const* minmax, int k, size_t n, size_t chunk)
{
    if (!x_in || !x_out || !xhat || !codes || !minmax || k < 1 || k > 32 || n == 0 ||
        !chunk_ok(chunk))
        return 1;
    for (int i = 0; i < k; ++i)
        if (!x_in[i] || !x_out[i] || !xhat[i] || !codes[i] || !minmax[i]) return 1;
    float* d = (float*)malloc(n * sizeof(float));
    float* q = (float*)malloc(n * sizeof(float));
    if (!d || !q) { free(d); free(q); return 1; }
    for (int i = 0; i < k; ++i) {
        for (size_t e = 0; e < n; ++e) d[e] = x_in[i][e] - xhat[i][e];
        oracle_compress_minmax_u8(d, NULL, n, chunk, codes[i], minmax[i]);
        oracle_decompress_minmax_u8(codes[i], minmax[i], n, chunk, q);
        for (size_t e = 0; e < n; ++e) xhat[i][e] = xhat[i][e] + q[e];
    }
    free(d);
    free(q);
    float third = 1.0f / 3.0f;
    for (int i = 0; i < k; ++i) {
        const float* l = xhat[(i + k - 1) % k];
        const float* m = xhat[i];
        const float* r = xhat[(i + 1) % k];
        ptrdiff_t e;
#pragma omp parallel for schedule(static) num_threads(g_threads)
        for (e = 0; e < (ptrdiff_t)n; ++e) {
            float s = l[e] + m[e];
            s = s + r[e];
            float avg = s * third;
            float own = x_in[i][e] - m[e];
            x_out[i][e] = avg + own;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------- Sign-1bit codec */

/*
 * Sum of |v| over one chunk in the fixed order of reading R6: the chunk is cut into groups
 * of four consecutive elements (missing ones count as +0.0f); group m is reduced as
 * (|a|+|b|) + (|c|+|d|) and added to accumulator m mod 64; the 64 accumulators are then
 * combined by a butterfly acc[l] <- acc[l] + acc[l xor s] for s = 1,2,4,8,16,32.
 */
static float ordered_abs_sum(const float* v, size_t len)
{
    float acc[64], nxt[64];
    for (int l = 0; l < 64; ++l) acc[l] = 0.0f;
    size_t groups = (len + 3) / 4;
    for (size_t m = 0; m < groups; ++m) {
        float e[4];
        for (int t = 0; t < 4; ++t) {
            size_t i = 4 * m + t;
            e[t] = (i < len) ? fabsf(v[i]) : 0.0f;
        }
        float p = e[0] + e[1];
        float q = e[2] + e[3];
        float g = p + q;
        acc[m % 64] = acc[m % 64] + g;
    }
    for (int s = 1; s < 64; s <<= 1) {
        for (int l = 0; l < 64; ++l) nxt[l] = acc[l] + acc[l ^ s];
        for (int l = 0; l < 64; ++l) acc[l] = nxt[l];
    }
    return acc[0];
}

/* scale = mean |v| of a chunk of length len out of nominal size chunk. */
static float sign_scale(const float* v, size_t len, size_t chunk)
{
    float s = ordered_abs_sum(v, len);
    int pow2 = (chunk & (chunk - 1)) == 0;
    if (len == chunk && pow2) return s * (1.0f / (float)chunk);
    return s / (float)len;
}

/* One chunk of Q := Sign-1bit on v = x (+ residual). lo = bucket index of the first element. */
static void sign_compress_chunk(const float* x, float* residual, size_t lo, size_t len, size_t chunk,
                                uint32_t* bits, float* scale_out, float* v)
{
    for (size_t i = 0; i < len; ++i) v[i] = residual ? x[i] + residual[i] : x[i];
    float scale = sign_scale(v, len, chunk);
    for (size_t i = 0; i < len; ++i) {
        int b = (v[i] >= 0.0f) ? 1 : 0;
        size_t g = lo + i;
        if (b) bits[g >> 5] |= (uint32_t)1 << (g & 31);
        if (residual) {
            float deq = b ? scale : -scale;
            residual[i] = v[i] - deq;
        }
    }
    *scale_out = scale;
}

/*
 * 1-bit worker-side compression with error compensation (the Q used by "1-bit Adam",
 * Section 4.1 "Bagua Algorithms", inside the C_LP_S equations of Section 3.2).
 * bits has ceil(n/32) words, unused tail bits are 0; scale has one float per chunk.
 */
int oracle_sign_compress_ef(const float* x, float* residual, size_t n, size_t chunk,
                            uint32_t* bits, float* scale)
{
    if (!x || !bits || !scale || n == 0 || !chunk_ok(chunk)) return 1;
    memset(bits, 0, ((n + 31) / 32) * sizeof(uint32_t));
    ptrdiff_t nc = (ptrdiff_t)num_chunks(n, chunk);
    ptrdiff_t c;
    /* chunk is a multiple of 256, so chunks never share a 32-bit word */
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (c = 0; c < nc; ++c) {
        size_t lo = (size_t)c * chunk;
        size_t len = (lo + chunk <= n) ? chunk : n - lo;
        float* v = (float*)malloc(len * sizeof(float));
        sign_compress_chunk(x + lo, residual ? residual + lo : NULL, lo, len, chunk, bits,
                            &scale[c], v);
        free(v);
    }
    return 0;
}

/* Decompression of Sign-1bit: out_i = bit_i ? +scale_c : -scale_c. */
int oracle_decompress_sign(const uint32_t* bits, const float* scale, size_t n, size_t chunk, float* out)
{
    if (!bits || !scale || !out || n == 0 || !chunk_ok(chunk)) return 1;
    for (size_t i = 0; i < n; ++i) {
        float s = scale[i / chunk];
        out[i] = ((bits[i >> 5] >> (i & 31)) & 1u) ? s : -s;
    }
    return 0;
}

/* Server side of C_LP_S with Q := Sign-1bit (same structure as oracle_drr_minmax_u8). */
int oracle_drr_sign(const uint32_t* const* bits_in, const float* const* scale_in, int k,
                    float* server_residual, size_t n, size_t chunk,
                    uint32_t* bits_out, float* scale_out, float* out_fp32)
{
    if (!bits_in || !scale_in || k < 1 || k > 32 || !bits_out || !scale_out || n == 0 ||
        !chunk_ok(chunk))
        return 1;
    for (int j = 0; j < k; ++j)
        if (!bits_in[j] || !scale_in[j]) return 1;
    memset(bits_out, 0, ((n + 31) / 32) * sizeof(uint32_t));
    float inv_k = 1.0f / (float)k;
    ptrdiff_t nc = (ptrdiff_t)num_chunks(n, chunk);
    ptrdiff_t c;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (c = 0; c < nc; ++c) {
        size_t lo = (size_t)c * chunk;
        size_t len = (lo + chunk <= n) ? chunk : n - lo;
        float* a = (float*)malloc(len * sizeof(float));
        float* v = (float*)malloc(len * sizeof(float));
        for (size_t i = 0; i < len; ++i) {
            size_t g = lo + i;
            float s = 0.0f;
            for (int j = 0; j < k; ++j) {
                float sc = scale_in[j][c];
                float deq = ((bits_in[j][g >> 5] >> (g & 31)) & 1u) ? sc : -sc;
                s = (j == 0) ? deq : s + deq;
            }
            a[i] = s * inv_k;
        }
        sign_compress_chunk(a, server_residual ? server_residual + lo : NULL, lo, len, chunk,
                            bits_out, &scale_out[c], v);
        if (out_fp32) {
            float sc = scale_out[c];
            for (size_t i = 0; i < len; ++i) {
                size_t g = lo + i;
                out_fp32[g] = ((bits_out[g >> 5] >> (g & 31)) & 1u) ? sc : -sc;
            }
        }
        free(a);
        free(v);
    }
    return 0;
}

/* --------------------------------------------------------------------------- flatten */

/*
 * Bucket flatten (Section 3.5 "Tensor Bucketing and Memory Flattening"; Section 3.1
 * "Flattening"), reading R10.  dst_offset ascending, tensors must not overlap and must
 * fit in the bucket.
 */
int oracle_bucket_flatten(const float* const* src, const size_t* numel, const size_t* dst_offset,
                          size_t T, float* bucket, size_t bucket_numel)
{
    if (!bucket || bucket_numel == 0 || (T && (!src || !numel || !dst_offset))) return 1;
    size_t prev_end = 0;
    for (size_t t = 0; t < T; ++t) {
        if (numel[t] && !src[t]) return 1;
        if (dst_offset[t] < prev_end) return 1;
        if (dst_offset[t] + numel[t] > bucket_numel) return 1;
        prev_end = dst_offset[t] + numel[t];
    }
    for (size_t e = 0; e < bucket_numel; ++e) bucket[e] = 0.0f;
    for (size_t t = 0; t < T; ++t)
        for (size_t e = 0; e < numel[t]; ++e) bucket[dst_offset[t] + e] = src[t][e];
    return 0;
}

/* ------------------------------------------------------- decode fused into the optimizer step */

/*
 * Last step of C_LP_S on every worker followed by the bucket-level model update (Section 3.5:
 * the stochastic-gradient optimizer also runs on the flattened bucket; Appendix listing: the
 * primitive is followed by optimizer.step()).  The optimizer is left open by the paper; reading
 * R16: plain SGD with optional weight decay and momentum (no dampening, no Nesterov), one
 * rounding per operation in this order:
 *     g = decode(codes, meta)                         (MinMax-u8 or Sign-1bit, as above)
 *     if weight_decay != 0:  g = g + weight_decay * p
 *     if momentum buffer:    m = momentum * m + g ;  u = m     else u = g
 *     p = p - lr * u
 * A zero-initialised momentum buffer reproduces the usual "first step: m = g".
 */
/* The update above for a decoded gradient g (shared by every codec's step). */
static void sgd_update(const float* g, size_t n, float* param, float* momentum_buf, float lr, float momentum,
                       float weight_decay)
{
    for (size_t i = 0; i < n; ++i) {
        float gi = g[i];
        if (weight_decay != 0.0f) {
            float w = weight_decay * param[i];
            gi = gi + w;
        }
        float u = gi;
        if (momentum_buf) {
            float t = momentum * momentum_buf[i];
            float m = t + gi;
            momentum_buf[i] = m;
            u = m;
        }
        float s = lr * u;
        param[i] = param[i] - s;
    }
}

int oracle_decompress_sgd_step(int codec, const void* codes, const float* meta, size_t n, size_t chunk,
                               float* param, float* momentum_buf, float lr, float momentum, float weight_decay)
{
    if ((codec != 0 && codec != 1) || !codes || !meta || !param || n == 0 || !chunk_ok(chunk)) return 1;
    float* g = (float*)malloc(n * sizeof(float));
    if (!g) return 1;
    int rc = codec == 0 ? oracle_decompress_minmax_u8((const uint8_t*)codes, meta, n, chunk, g)
                        : oracle_decompress_sign((const uint32_t*)codes, meta, n, chunk, g);
    if (rc) { free(g); return rc; }
    sgd_update(g, n, param, momentum_buf, lr, momentum, weight_decay);
    free(g);
    return 0;
}

int oracle_decompress_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep, float* out);

/* The same step after a top-K round (Section 3.2 names top-K as the aggressive Q): g = decode of the sparse entries,
 * +0 everywhere else, then the identical update on EVERY element (so weight decay and momentum act on all of them). */
int oracle_decompress_sgd_step_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep,
                                    float* param, float* momentum_buf, float lr, float momentum, float weight_decay)
{
    if (!idx || !val || !param || n == 0 || !chunk_ok(chunk) || keep < 1 || keep > chunk) return 1;
    float* g = (float*)malloc(n * sizeof(float));
    if (!g) return 1;
    int rc = oracle_decompress_topk(idx, val, n, chunk, keep, g);
    if (!rc) sgd_update(g, n, param, momentum_buf, lr, momentum, weight_decay);
    free(g);
    return rc;
}

/* ------------------------------------------------ decentralised averaging, "random" peer strategy */

/*
 * D_FP_S with the random peer allocation of Section 3.4 (each worker exchanges with one peer
 * chosen for the round; "Decen-32bits" of Section 4.1 uses it).  peer[i] is the worker that
 * worker i exchanges with in this round; reading R17: N(i) = {i, peer[i]} with weight 1/2,
 *     x_i' = (x_i + x_peer[i]) * 0.5f        from the old values (outputs must not alias inputs).
 * peer[i] == i leaves the replica unchanged.  For a matching (peer[peer[i]] == i) both partners
 * receive the same bits and the replica mean is preserved.
 */
int oracle_peer_avg_fp(const float* const* x_in, float* const* x_out, const int* peer, int k, size_t n)
{
    if (!x_in || !x_out || !peer || k < 1 || k > 32 || n == 0) return 1;
    for (int i = 0; i < k; ++i)
        if (!x_in[i] || !x_out[i] || peer[i] < 0 || peer[i] >= k) return 1;
    for (int i = 0; i < k; ++i) {
        const float* a = x_in[i];
        const float* b = x_in[peer[i]];
        for (size_t e = 0; e < n; ++e) {
            float s = a[e] + b[e];
            x_out[i][e] = s * 0.5f;
        }
    }
    return 0;
}

/* ------------------------------------------------------ hierarchical C_LP_S: intra-node step */

/*
 * First stage of the hierarchical variant of C_LP_S (Section 3.5 "Hierarchical Communications"):
 * the tensors of the k_local workers of one node are aggregated WITHOUT compression, and only the
 * node leader compresses the aggregate for the inter-node exchange (which is the ordinary server
 * step among leaders, oracle_drr_minmax_u8, followed by a broadcast and a local decode).
 * Reading R18 (consistent with R2): the aggregate is the average, a = (x_0 + x_1 + ...) * fl(1/k_local)
 * summed in ascending worker order; the leader's error state enters as in R1:
 *     codes = Q(a + delta),  delta <- (a + delta) - decode(codes).
 * With k_local == 1 this is not the plain worker-side compression bit for bit only because of the
 * multiplication by 1.0f, which is exact: the results are identical.
 */
int oracle_reduce_compress_minmax_u8(const float* const* x, int k_local, float* residual, size_t n,
                                     size_t chunk, uint8_t* codes, float* minmax)
{
    if (!x || k_local < 1 || k_local > 32 || !codes || !minmax || n == 0 || !chunk_ok(chunk)) return 1;
    for (int j = 0; j < k_local; ++j)
        if (!x[j]) return 1;
    float* a = (float*)malloc(n * sizeof(float));
    if (!a) return 1;
    float inv = 1.0f / (float)k_local;
    for (size_t i = 0; i < n; ++i) {
        float s = x[0][i];
        for (int j = 1; j < k_local; ++j) s = s + x[j][i];
        a[i] = s * inv;
    }
    int rc = oracle_compress_minmax_u8(a, residual, n, chunk, codes, minmax);
    free(a);
    return rc;
}

/*
 * Inverse of the flatten (Section 3.5): copy every tensor's range of the bucket back to the
 * tensor; bucket elements not covered by a tensor are ignored.  Same layout rules as
 * oracle_bucket_flatten.
 */
int oracle_bucket_unflatten(const float* bucket, size_t bucket_numel, float* const* dst, const size_t* numel,
                            const size_t* src_offset, size_t T)
{
    if (!bucket || bucket_numel == 0 || (T && (!dst || !numel || !src_offset))) return 1;
    size_t prev_end = 0;
    for (size_t t = 0; t < T; ++t) {
        if (numel[t] && !dst[t]) return 1;
        if (src_offset[t] < prev_end) return 1;
        if (src_offset[t] + numel[t] > bucket_numel) return 1;
        prev_end = src_offset[t] + numel[t];
    }
    for (size_t t = 0; t < T; ++t)
        for (size_t e = 0; e < numel[t]; ++e) dst[t][e] = bucket[src_offset[t] + e];
    return 0;
}

/* --------------------------------------------------------------------------- Top-K codec */

/*
 * A third compression function Q: per-chunk top-K sparsification, the example of an aggressive
 * compression for which the paper says error compensation matters most (Section 3.2, last
 * sentences on C_LP_S).  Reading R19: per chunk of C elements keep the `keep` entries of largest
 * |v| (ties: the lower index wins; |v| is compared through its IEEE bit pattern, so -0 == +0);
 * a chunk is encoded as `keep` (index, value) pairs in ascending index order, index = position
 * inside the chunk as u16, value = fl(v + 0.0f) (v itself, with -0 stored as +0, so that summing the
 * kept entries of several workers sparsely or densely gives the same bits); a last chunk shorter than `keep` keeps everything and
 * pads the remaining slots with index 0xFFFF, value +0.0f.  decode = 0 everywhere except the kept
 * positions.  The error update of C_LP_S is then exact: delta' = v at dropped positions, +0 at kept.
 */
typedef struct { uint32_t key; uint32_t pos; } topk_item;

static int topk_cmp(const void* a, const void* b)
{
    const topk_item* x = (const topk_item*)a;
    const topk_item* y = (const topk_item*)b;
    if (x->key != y->key) return x->key > y->key ? -1 : 1;   /* larger magnitude first */
    return x->pos < y->pos ? -1 : (x->pos > y->pos ? 1 : 0); /* then lower index */
}

static void topk_compress_chunk(const float* v, size_t len, size_t keep, uint16_t* idx, float* val, float* residual)
{
    topk_item* items = (topk_item*)malloc(len * sizeof(topk_item));
    uint8_t* sel = (uint8_t*)calloc(len, 1);
    for (size_t i = 0; i < len; ++i) {
        uint32_t bits;
        memcpy(&bits, &v[i], 4);
        items[i].key = bits & 0x7fffffffu;
        items[i].pos = (uint32_t)i;
    }
    qsort(items, len, sizeof(topk_item), topk_cmp);
    size_t kk = keep < len ? keep : len;
    for (size_t s = 0; s < kk; ++s) sel[items[s].pos] = 1;
    size_t o = 0;
    for (size_t i = 0; i < len; ++i) {
        if (sel[i]) {
            idx[o] = (uint16_t)i;
            val[o] = v[i] + 0.0f; /* -0 is stored as +0, as for the MinMax statistics (R5) */
            ++o;
        }
        if (residual) residual[i] = sel[i] ? 0.0f : v[i];
    }
    for (; o < keep; ++o) {
        idx[o] = 0xFFFFu;
        val[o] = 0.0f;
    }
    free(items);
    free(sel);
}

/* Worker side of C_LP_S with Q = top-K: idx u16[nc*keep], val fp32[nc*keep]. */
int oracle_compress_topk(const float* x, float* residual, size_t n, size_t chunk, size_t keep,
                         uint16_t* idx, float* val)
{
    if (!x || !idx || !val || n == 0 || !chunk_ok(chunk) || keep < 1 || keep > chunk) return 1;
    ptrdiff_t nc = (ptrdiff_t)num_chunks(n, chunk);
    ptrdiff_t c;
#pragma omp parallel for schedule(static) num_threads(g_threads)
    for (c = 0; c < nc; ++c) {
        size_t lo = (size_t)c * chunk;
        size_t len = (lo + chunk <= n) ? chunk : n - lo;
        float* v = (float*)malloc(len * sizeof(float));
        for (size_t i = 0; i < len; ++i) v[i] = residual ? x[lo + i] + residual[lo + i] : x[lo + i];
        topk_compress_chunk(v, len, keep, idx + (size_t)c * keep, val + (size_t)c * keep,
                            residual ? residual + lo : NULL);
        free(v);
    }
    return 0;
}

int oracle_decompress_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep, float* out)
{
    if (!idx || !val || !out || n == 0 || !chunk_ok(chunk) || keep < 1 || keep > chunk) return 1;
    size_t nc = num_chunks(n, chunk);
    for (size_t i = 0; i < n; ++i) out[i] = 0.0f;
    for (size_t c = 0; c < nc; ++c) {
        size_t lo = c * chunk;
        size_t len = (lo + chunk <= n) ? chunk : n - lo;
        for (size_t s = 0; s < keep; ++s) {
            uint16_t p = idx[c * keep + s];
            if (p == 0xFFFFu) continue;
            if (p >= len) return 1;
            out[lo + p] = val[c * keep + s];
        }
    }
    return 0;
}

/* Server side of C_LP_S with Q = top-K: dense average of the k decoded buckets (ascending j), + epsilon, Q again. */
int oracle_drr_topk(const uint16_t* const* idx_in, const float* const* val_in, int k, float* server_residual,
                    size_t n, size_t chunk, size_t keep, uint16_t* idx_out, float* val_out, float* out_fp32)
{
    if (!idx_in || !val_in || k < 1 || k > 32 || !idx_out || !val_out || n == 0 || !chunk_ok(chunk) || keep < 1 ||
        keep > chunk)
        return 1;
    float* a = (float*)malloc(n * sizeof(float));
    float* d = (float*)malloc(n * sizeof(float));
    if (!a || !d) { free(a); free(d); return 1; }
    float inv_k = 1.0f / (float)k;
    for (int j = 0; j < k; ++j) {
        if (!idx_in[j] || !val_in[j] || oracle_decompress_topk(idx_in[j], val_in[j], n, chunk, keep, d)) {
            free(a); free(d); return 1;
        }
        for (size_t i = 0; i < n; ++i) a[i] = (j == 0) ? d[i] : a[i] + d[i];
    }
    for (size_t i = 0; i < n; ++i) a[i] = a[i] * inv_k;
    int rc = oracle_compress_topk(a, server_residual, n, chunk, keep, idx_out, val_out);
    if (!rc && out_fp32) rc = oracle_decompress_topk(idx_out, val_out, n, chunk, keep, out_fp32);
    free(a);
    free(d);
    return rc;
}

/* ----------------------------------------------------------- centralised, full precision */

/*
 * C_FP_S (Section 3.2, "Centralized, Full Precision": every worker ends up with the sum of all
 * replicas, the Allreduce result).  With reading R2 the average is returned: the ascending-order
 * fp32 sum times fl(1/k).  This is C_LP_S with Q = identity and no error state.
 */
int oracle_centralized_avg_fp(const float* const* x, int k, size_t n, float* out)
{
    if (!x || k < 1 || k > 32 || n == 0 || !out) return 1;
    for (int j = 0; j < k; ++j)
        if (!x[j]) return 1;
    float inv = 1.0f / (float)k;
    for (size_t i = 0; i < n; ++i) {
        float s = x[0][i];
        for (int j = 1; j < k; ++j) s = s + x[j][i];
        out[i] = s * inv;
    }
    return 0;
}

/*
 * D_LP_S with the random peer allocation (Section 3.4: the low-precision primitive uses the same
 * peer selection as the full-precision one and compresses before sending).  Readings R8 and R17
 * combined: every peer publishes Q(x_i - xhat_i) and all holders advance xhat_i, then
 *     x_i' = (xhat_i + xhat_peer[i]) * 0.5f + (x_i - xhat_i)        (updated xhat).
 */
int oracle_peer_avg_lp(const float* const* x_in, float* const* x_out, float* const* xhat,
                       uint8_t* const* codes, float* const* minmax, const int* peer, int k, size_t n,
                       size_t chunk)
{
    if (!x_in || !x_out || !xhat || !codes || !minmax || !peer || k < 1 || k > 32 || n == 0 || !chunk_ok(chunk))
        return 1;
    for (int i = 0; i < k; ++i)
        if (!x_in[i] || !x_out[i] || !xhat[i] || !codes[i] || !minmax[i] || peer[i] < 0 || peer[i] >= k) return 1;
    float* d = (float*)malloc(n * sizeof(float));
    float* q = (float*)malloc(n * sizeof(float));
    if (!d || !q) { free(d); free(q); return 1; }
    for (int i = 0; i < k; ++i) {
        for (size_t e = 0; e < n; ++e) d[e] = x_in[i][e] - xhat[i][e];
        oracle_compress_minmax_u8(d, NULL, n, chunk, codes[i], minmax[i]);
        oracle_decompress_minmax_u8(codes[i], minmax[i], n, chunk, q);
        for (size_t e = 0; e < n; ++e) xhat[i][e] = xhat[i][e] + q[e];
    }
    free(d);
    free(q);
    for (int i = 0; i < k; ++i) {
        const float* a = xhat[i];
        const float* b = xhat[peer[i]];
        for (size_t e = 0; e < n; ++e) {
            float s = a[e] + b[e];
            float avg = s * 0.5f;
            float own = x_in[i][e] - a[e];
            x_out[i][e] = avg + own;
        }
    }
    return 0;
}


/* ------------------------------------------------------------------ Adam-type bucket optimizer */

/*
 * Decode fused into an Adam-type update of the flattened bucket (Section 3.5: the optimizer runs on
 * the bucket; Section 4.1: QSGD and 1-bit Adam are C_LP_S followed by the optimizer).  Reading R20,
 * one rounding per operation, in this order, with omb = 1.0f - beta in fp32:
 *   d = decode(codes, meta)
 *   variance_frozen == 0 (d is the averaged gradient):
 *       m = beta1*m + omb1*d ;  v = beta2*v + omb2*(d*d)
 *   variance_frozen != 0 (compression stage of 1-bit Adam, d is the averaged momentum):
 *       m = d ;  v unchanged
 *   u = m / (sqrtf(v) + eps) ;  if weight_decay != 0:  u = u + weight_decay*p ;  p = p - lr*u
 */
/* The update above for a decoded tensor d (shared by every codec's step). */
static void adam_update(const float* d, size_t n, float* param, float* m, float* v, float lr, float beta1, float beta2,
                        float eps, float weight_decay, int variance_frozen)
{
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    for (size_t i = 0; i < n; ++i) {
        float mi, vi = v[i];
        if (variance_frozen) {
            mi = d[i];
        } else {
            float a = beta1 * m[i];
            float b = omb1 * d[i];
            mi = a + b;
            float c = beta2 * vi;
            float dd = d[i] * d[i];
            float e = omb2 * dd;
            vi = c + e;
            v[i] = vi;
        }
        m[i] = mi;
        float root = sqrtf(vi);
        float denom = root + eps;
        float u = mi / denom;
        if (weight_decay != 0.0f) {
            float w = weight_decay * param[i];
            u = u + w;
        }
        float step = lr * u;
        param[i] = param[i] - step;
    }
}

int oracle_decompress_adam_step(int codec, const void* codes, const float* meta, size_t n, size_t chunk,
                                float* param, float* m, float* v, float lr, float beta1, float beta2, float eps,
                                float weight_decay, int variance_frozen)
{
    if ((codec != 0 && codec != 1) || !codes || !meta || !param || !m || !v || n == 0 || !chunk_ok(chunk)) return 1;
    float* d = (float*)malloc(n * sizeof(float));
    if (!d) return 1;
    int rc = codec == 0 ? oracle_decompress_minmax_u8((const uint8_t*)codes, meta, n, chunk, d)
                        : oracle_decompress_sign((const uint32_t*)codes, meta, n, chunk, d);
    if (rc) { free(d); return rc; }
    adam_update(d, n, param, m, v, lr, beta1, beta2, eps, weight_decay, variance_frozen);
    free(d);
    return 0;
}

/* The same step after a top-K round: d = decode of the sparse entries, +0 everywhere else, then the identical update
 * on EVERY element (where nothing was kept the momentum decays by beta1, the variance by beta2, and the parameter
 * still moves by the decayed momentum). */
int oracle_decompress_adam_step_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep,
                                     float* param, float* m, float* v, float lr, float beta1, float beta2, float eps,
                                     float weight_decay, int variance_frozen)
{
    if (!idx || !val || !param || !m || !v || n == 0 || !chunk_ok(chunk) || keep < 1 || keep > chunk) return 1;
    float* d = (float*)malloc(n * sizeof(float));
    if (!d) return 1;
    int rc = oracle_decompress_topk(idx, val, n, chunk, keep, d);
    if (!rc) adam_update(d, n, param, m, v, lr, beta1, beta2, eps, weight_decay, variance_frozen);
    free(d);
    return rc;
}

/*
 * Worker side of the compression stage of 1-bit Adam (reading R20): the local momentum
 *   u = beta1*m + omb1*g        (m: the momentum all workers share after the previous step; not written)
 * is compressed with the sign codec and the worker's error state exactly as oracle_sign_compress_ef does.
 */
int oracle_momentum_sign_compress_ef(const float* g, const float* m, float beta1, float* residual, size_t n,
                                     size_t chunk, uint32_t* bits, float* scale)
{
    if (!g || !m || !bits || !scale || n == 0 || !chunk_ok(chunk)) return 1;
    float* u = (float*)malloc(n * sizeof(float));
    if (!u) return 1;
    const float omb1 = 1.0f - beta1;
    for (size_t i = 0; i < n; ++i) {
        float a = beta1 * m[i];
        float b = omb1 * g[i];
        u[i] = a + b;
    }
    int rc = oracle_sign_compress_ef(u, residual, n, chunk, bits, scale);
    free(u);
    return rc;
}
