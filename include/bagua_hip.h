/*
 * bagua_hip.h -- C ABI of the MI355X (gfx950) compression hot path behind the communication
 * primitives of "BAGUA: Scaling up Distributed Learning with System Relaxations".
 *
 * The library implements the on-device compute of the paper's primitives (Section 3.2,
 * "Communication Primitives"): C_LP_S (centralised, low precision, with the error states
 * delta and epsilon), D_FP_S / D_LP_S (decentralised, full / low precision) on the ring
 * peer topology of Section 3.4, and the bucket flattening of Section 3.5.  The k workers
 * (peers) are k buffers in one GPU's memory; nothing here communicates between GPUs.
 *
 * Conventions shared by every entry point
 *   - Return value: BAGUA_OK or an error code below.  Nothing is enqueued when an error other
 *     than BAGUA_ERR_LAUNCH is returned.  No exceptions, no aborts, nothing is printed.
 *   - Pointers named "device" point to GPU memory owned by the caller; "host[k]" arrays are
 *     host arrays of k device pointers and are only read during the call.  The library
 *     allocates no device memory and keeps no state between calls.
 *   - Bucket-sized buffers (x, residual, codes, sign words, replicas, parameters, optimizer state,
 *     bucket) must be 16-byte aligned (BAGUA_ERR_ALIGNMENT otherwise).  Per-chunk metadata (minmax,
 *     scale) and the top-K entry arrays need only the alignment of their element type, so the slice
 *     that belongs to a partition of whole chunks can be passed as it is.
 *   - Aliasing: a buffer that a call writes (outputs and in-out state) must not overlap, by byte
 *     range, any other buffer passed to the same call (BAGUA_ERR_INVALID_ARG otherwise); buffers
 *     that are only read may overlap each other.  Tensors named in a flatten plan are not checked.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work and return without synchronising unless stated otherwise.
 *   - n = number of fp32 elements of the bucket; chunk = C = elements per statistics chunk,
 *     a multiple of 256 in [256, 16384]; nc = ceil(n / C); the last chunk may be short.
 *   - All arithmetic is IEEE binary32, one rounding per operation in a fixed order (no fused
 *     multiply-add), so results are reproducible bit for bit.  Inputs must be finite.
 *   - The primitives return averages (the paper states sums): the sum over workers in
 *     ascending index order is multiplied by fl(1/k), on the ring by fl(1/3).
 *   - Error compensation follows the C_LP_S equations with the stored error carried in as
 *     v = x + residual and updated as residual <- v - decode(Q(v)).
 */
#ifndef BAGUA_HIP_H
#define BAGUA_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    BAGUA_OK = 0,
    BAGUA_ERR_INVALID_ARG = 1, /* NULL where required, n == 0, k outside [1,32], bad chunk, bad enum, aliasing */
    BAGUA_ERR_ALIGNMENT = 2,   /* a pointer is not aligned as stated under "Conventions" */
    BAGUA_ERR_LAUNCH = 3,      /* the HIP runtime reported an error for a copy or a launch */
    BAGUA_ERR_UNSUPPORTED = 4  /* valid request outside what this build implements */
};

enum { BAGUA_CODEC_MINMAX_U8 = 0, BAGUA_CODEC_SIGN1 = 1 };
enum { BAGUA_AVG_FP = 0, BAGUA_AVG_LP_MINMAX_U8 = 1 };

#define BAGUA_MAX_WORKERS 32

/* Human-readable name of a status code (static storage). */
const char* bagua_status_string(int status);

/*
 * Bucket flatten (Section 3.1 "Flattening"; Section 3.5 "Tensor Bucketing and Memory
 * Flattening"): copy T layer tensors into one contiguous fp32 bucket, tensor t to elements
 * [dst_offset[t], dst_offset[t] + numel[t]); every bucket element not covered by a tensor
 * is set to +0.0f.
 *   src         host[T] of device pointers to fp32 data, 4-byte aligned (may be NULL if numel[t] == 0)
 *   numel       host[T]
 *   dst_offset  host[T], in elements, ascending; tensors must not overlap and must fit
 *   bucket      device, fp32[bucket_numel], 16-byte aligned
 *   workspace   device, >= bagua_flatten_workspace_bytes(T, bucket_numel) bytes, 16-byte aligned;
 *               holds the tensor table the copy kernel reads
 * bagua_flatten_plan validates the layout and uploads the table into `workspace`; it
 * SYNCHRONISES `stream` before returning (a set-up call: the layout of a bucket is fixed after
 * the first iteration).  bagua_bucket_flatten_run only launches the copy using a planned
 * workspace (T and bucket_numel must be those given to the plan).  bagua_bucket_flatten is
 * plan followed by run.
 */
size_t bagua_flatten_workspace_bytes(size_t T, size_t bucket_numel);
int bagua_flatten_plan(const void* const* src, const size_t* numel, const size_t* dst_offset, size_t T,
                       size_t bucket_numel, void* workspace, size_t workspace_bytes, void* stream);
int bagua_bucket_flatten_run(const void* workspace, size_t T, float* bucket, size_t bucket_numel, void* stream);
int bagua_bucket_flatten(const void* const* src, const size_t* numel, const size_t* dst_offset, size_t T,
                         float* bucket, size_t bucket_numel, void* workspace, size_t workspace_bytes,
                         void* stream);

/*
 * bagua_bucket_flatten without a workspace, for callers that cannot allocate device memory or must not
 * synchronise: code running under HIP graph capture, tight serving loops, harnesses that forbid allocation.
 * Same result as bagua_bucket_flatten.  The tensor table is built on the device, from kernel arguments, in a
 * fixed array inside the library (about 360 KB per GPU, held until the process ends); the call allocates nothing,
 * copies nothing from host memory and does not synchronise.
 *   limits   T <= BAGUA_FLATTEN_STATIC_MAX_TENSORS and bucket_numel <= BAGUA_FLATTEN_STATIC_MAX_NUMEL,
 *            BAGUA_ERR_UNSUPPORTED beyond (use the workspace form there)
 *   sharing  every call on one GPU uses that GPU's one array: calls are safe one after another on one stream,
 *            but two calls that overlap in time on the same GPU (different streams or threads) race on the table
 * Other arguments and errors as bagua_bucket_flatten; additionally no tensor may overlap the bucket.
 */
#define BAGUA_FLATTEN_STATIC_MAX_TENSORS 4096
#define BAGUA_FLATTEN_STATIC_MAX_NUMEL 67108864 /* 2^26 elements = 256 MiB of fp32 */
int bagua_bucket_flatten_static(const void* const* src, const size_t* numel, const size_t* dst_offset, size_t T,
                                float* bucket, size_t bucket_numel, void* stream);

/*
 * Inverse of the flatten: copy each tensor's range [dst_offset[t], dst_offset[t] + numel[t]) of the bucket back
 * into tensor t (for callers whose layer tensors are not views of the bucket).  Uses a workspace planned by
 * bagua_flatten_plan; the tensor pointers given to the plan are written through, so they must be writable.
 * Bucket elements no tensor covers are ignored.
 */
int bagua_bucket_unflatten_run(const void* workspace, size_t T, const float* bucket, size_t bucket_numel,
                               void* stream);

/*
 * Worker side of C_LP_S (Section 3.2, terms Q(x_j - delta_j) and delta_j' of the C_LP_S
 * equations) with Q = per-chunk MinMax uint8:
 *   v = x + residual (v = x if residual == NULL);  per chunk mn = min v, mx = max v;
 *   code = clamp(rint((v - mn) * fl(255 / fl(mx - mn))), 0, 255)   (all 0 when mx == mn);
 *   residual <- v - (mn + code * fl(fl(mx - mn) / 255)).
 *   x        device fp32[n], read only
 *   residual device fp32[n], updated in place, or NULL (no error compensation)
 *   codes    device u8[n], written
 *   minmax   device fp32[2*nc], written as (min, max) pairs; -0 is stored as +0
 */
int bagua_compress_minmax_u8(const float* x, float* residual, size_t n, size_t chunk,
                             uint8_t* codes, float* minmax, void* stream);

/*
 * Flatten fused into the worker-side compression (the step right before the path: Section 3.5 has the
 * compression work on the flattened view of a bucket; here that view is never materialised).  The result is exactly
 * bagua_bucket_flatten followed by bagua_compress_minmax_u8 on the bucket, but the rows of each chunk are
 * gathered straight from the layer tensors through a planned workspace (bagua_flatten_plan with the same T and
 * bucket_numel), so the bucket is not written to and read back from memory.
 *   workspace   device, planned;  T, bucket_numel as given to the plan
 *   residual    device fp32[bucket_numel], in-out, or NULL
 *   codes       device u8[bucket_numel];  minmax device fp32[2*nc]
 *   bucket_out  device fp32[bucket_numel] or NULL: if given, the flattened bucket is also written (for callers
 *               that need the flat view as well); 16-byte aligned
 */
int bagua_flatten_compress_minmax_u8(const void* workspace, size_t T, float* residual, size_t bucket_numel,
                                     size_t chunk, uint8_t* codes, float* minmax, float* bucket_out, void* stream);

/*
 * The same fusion in front of the 1-bit sign codec: exactly bagua_bucket_flatten followed by bagua_sign_compress_ef
 * on the bucket, with the rows gathered straight from the layer tensors (Section 3.5; the codec of Section 4.1's
 * 1-bit Adam).  Arguments as bagua_flatten_compress_minmax_u8 with bits u32[ceil(n/32)] and scale fp32[nc].
 */
int bagua_flatten_sign_compress_ef(const void* workspace, size_t T, float* residual, size_t bucket_numel, size_t chunk,
                                   uint32_t* bits, float* scale, float* bucket_out, void* stream);

/*
 * The last step of C_LP_S on every worker, fused with the inverse of the flatten (Section 3.4 step 5 followed by
 * Section 3.5's flattening in reverse): the compressed bucket is decoded and every decoded element is written
 * straight into the layer tensor that covers it; the decoded bucket itself is never stored.  Exactly bagua_decompress
 * followed by bagua_bucket_unflatten_run.
 *   codec, codes, meta, n, chunk   as bagua_decompress (n = bucket_numel of the plan)
 *   workspace, T                   a plan made by bagua_flatten_plan with WRITABLE tensors; they must not overlap
 *                                  codes or meta (not checked: the table is on the device)
 */
int bagua_decompress_unflatten(int codec, const void* codes, const float* meta, size_t n, size_t chunk,
                               const void* workspace, size_t T, void* stream);

/*
 * Server side of C_LP_S (Section 3.2, x_i' and epsilon_i' of the C_LP_S equations; steps 3-5 of
 * ScatterReduce, Section 3.4): decode the k workers' compressed buckets, average them in
 * ascending worker order, add the server error state, compress again, update the state:
 *   a = (sum_j decode_j) * fl(1/k);  w = a + server_residual (w = a if NULL);
 *   (codes_out, meta_out) = Q(w);  server_residual <- w - decode(Q(w));
 *   out_fp32 (optional) = decode(Q(w)), the tensor every worker ends up with.
 *   codec      BAGUA_CODEC_MINMAX_U8: codes are u8[n], meta is minmax fp32[2*nc]
 *              BAGUA_CODEC_SIGN1:     codes are u32[ceil(n/32)] sign words, meta is scale fp32[nc]
 *   codes_in   host[k] of device pointers;  meta_in host[k] of device pointers
 *   k          number of workers, 1..BAGUA_MAX_WORKERS
 *   codes_out, meta_out   device, written (must not alias any input)
 *   out_fp32   device fp32[n] or NULL
 */
int bagua_decompress_reduce_recompress(int codec, const void* const* codes_in, const float* const* meta_in,
                                       int k, float* server_residual, size_t n, size_t chunk,
                                       void* codes_out, float* meta_out, float* out_fp32, void* stream);

/*
 * Decentralised averaging on a ring, one round (D_FP_S and D_LP_S equations, Section 3.2; "ring"
 * peer allocation, Section 3.4).  Neighbours of peer i are i-1, i, i+1 (mod k) with weight 1/3;
 * every output is computed from the old inputs.
 *   BAGUA_AVG_FP:            x_out[i] = ((x_in[i-1] + x_in[i]) + x_in[i+1]) * fl(1/3)
 *   BAGUA_AVG_LP_MINMAX_U8:  the wire carries Q(x_i - xhat_i) with Q = MinMax uint8, no error state:
 *        (codes[i], minmax[i]) = Q(x_in[i] - xhat[i]);   xhat[i] <- xhat[i] + decode(codes[i], minmax[i]);
 *        x_out[i] = ((xhat[i-1] + xhat[i]) + xhat[i+1]) * fl(1/3) + (x_in[i] - xhat[i])   (updated xhat)
 *   x_in    host[k] of device fp32[n], read only
 *   x_out   host[k] of device fp32[n], written; must not alias any x_in or xhat (BAGUA_ERR_INVALID_ARG)
 *   xhat    host[k] of device fp32[n], LP only: public copies of the replicas, updated in place
 *   codes   host[k] of device u8[n], LP only, written;  minmax host[k] of device fp32[2*nc], LP only, written
 *   chunk   used by LP only (ignored for FP)
  * Placement: this call streams 2k (FP) or 5k (LP) buffers at once.  On MI355X it runs 15-20 % faster when those
 * buffers are scattered over more than ~48 GiB of the GPU's address space than when they lie back to back (any
 * placement gives the same results).
 */
int bagua_decentralized_avg(int mode, const float* const* x_in, float* const* x_out, float* const* xhat,
                            uint8_t* const* codes, float* const* minmax, int k, size_t n, size_t chunk,
                            void* stream);

/*
 * One peer's share of D_LP_S on a ring (Section 3.2, D_LP_S; Section 3.4: a peer compresses before sending and
 * decompresses after receiving), i.e. what a single GPU runs when every peer has a GPU of its own.  Same arithmetic
 * as bagua_decentralized_avg in LP mode, which is these two steps for all k peers at once.
 *
 * bagua_lp_encode: the peer publishes its difference and advances its own public copy:
 *   codes, minmax = Q(x - xhat)  (no error feedback);   xhat <- xhat + decode(codes, minmax).
 *
 * bagua_lp_apply_mix: after the neighbours' codes have arrived, the peer advances its copies of their public
 * replicas and forms its new replica (xhat_own is the copy bagua_lp_encode has already advanced):
 *   xhat_left <- xhat_left + decode(codes_left);   xhat_right <- xhat_right + decode(codes_right);
 *   x_out = ((xhat_left + xhat_own) + xhat_right) * fl(1/3) + (x - xhat_own).
 *   left = peer i-1, right = peer i+1.  codes_* / minmax_* may be NULL together: that copy is current and only read.
 *   Ring of two: pass the other peer's copy as both xhat_left and xhat_right with codes_right = NULL; it is
 *   advanced once and counted twice.  Ring of one: pass xhat_own for both neighbours, no codes.
 *   x, xhat_*, x_out: device fp32[n]; codes_*: device u8[n]; minmax_*: device fp32[2*nc].
 */
int bagua_lp_encode(const float* x, float* xhat, size_t n, size_t chunk, uint8_t* codes, float* minmax, void* stream);
int bagua_lp_apply_mix(const float* x, const float* xhat_own, float* xhat_left, float* xhat_right,
                       const uint8_t* codes_left, const float* minmax_left, const uint8_t* codes_right,
                       const float* minmax_right, size_t n, size_t chunk, float* x_out, void* stream);

/*
 * C_FP_S (Section 3.2, centralised full precision: every worker receives the aggregate of all replicas, the
 * Allreduce result), as an average: out = (x[0] + x[1] + ...) * fl(1/k), summed in ascending order.
 *   x    host[k] of device fp32[n], read only;   out  device fp32[n], must not overlap any input
 */
int bagua_centralized_avg_fp(const float* const* x, int k, size_t n, float* out, void* stream);

/*
 * Intra-node stage of the hierarchical variant of C_LP_S (Section 3.5 "Hierarchical Communications": the workers
 * of one node are aggregated without compression, only the node leaders exchange compressed tensors): average the
 * k_local workers' uncompressed buckets in ascending order, then compress as bagua_compress_minmax_u8 does, with
 * the leader's error state:
 *   a = (x[0] + x[1] + ...) * fl(1/k_local);  v = a + residual;  codes = Q(v);  residual <- v - decode(codes).
 * The inter-node stage is bagua_decompress_reduce_recompress over the leaders' codes.
 *   x   host[k_local] of device fp32[n], read only;  residual device fp32[n] in-out or NULL; codes, minmax written
 */
int bagua_reduce_compress_minmax_u8(const float* const* x, int k_local, float* residual, size_t n, size_t chunk,
                                    uint8_t* codes, float* minmax, void* stream);

/*
 * The same intra-node stage with the 1-bit sign codec (Section 3.5 "Hierarchical Communications" with the Q of
 * Section 4.1's 1-bit Adam): a = ((x_0 + x_1) + ...) * fl(1/k_local), then exactly bagua_sign_compress_ef on a with the
 * leader's error state.  bits u32[ceil(n/32)], scale fp32[nc]; other arguments as above.
 */
int bagua_reduce_compress_sign_ef(const float* const* x, int k_local, float* residual, size_t n, size_t chunk,
                                  uint32_t* bits, float* scale, void* stream);

/*
 * Decentralised full-precision averaging with the "random" peer strategy of Section 3.4 (each worker exchanges
 * with one peer chosen for the round; the D_FP_S equation of Section 3.2 with N(i) = {i, peer[i]}, weight 1/2):
 *   x_out[i] = (x_in[i] + x_in[peer[i]]) * 0.5f        from the old values.
 *   peer    host[k], peer[i] in [0,k); chosen by the caller (e.g. a random perfect matching).  peer[i] == i
 *           leaves replica i unchanged.  Matched pairs (peer[peer[i]] == i) are read once and receive equal bits.
 *   x_in, x_out as in bagua_decentralized_avg (no aliasing).
 */
int bagua_decentralized_avg_peers(const float* const* x_in, float* const* x_out, const int* peer, int k, size_t n,
                                  void* stream);

/*
 * Decentralised low-precision averaging with a chosen peer per worker (Section 3.2, D_LP_S, with the peer selection
 * of Section 3.4; the compressed-difference reading used by bagua_decentralized_avg in LP mode):
 *   codes[i], minmax[i] = Q(x_in[i] - xhat[i])  (no error feedback);  xhat[i] <- xhat[i] + decode(codes[i]);
 *   x_out[i] = (xhat[i] + xhat[peer[i]]) * 0.5f + (x_in[i] - xhat[i])        with the updated xhat.
 *   peer    host[k], peer[i] in [0,k).  When the map is a perfect matching (peer[i] != i, peer[peer[i]] == i for
 *           all i) and chunk <= 4096 each pair is processed in one pass; any other map takes two passes.
 *   x_in, x_out, xhat, codes, minmax as in bagua_decentralized_avg (LP mode); same aliasing and alignment rules.
 */
int bagua_decentralized_avg_peers_lp(const float* const* x_in, float* const* x_out, float* const* xhat,
                                     uint8_t* const* codes, float* const* minmax, const int* peer, int k, size_t n,
                                     size_t chunk, void* stream);

/*
 * Worker side of C_LP_S with Q = 1-bit sign and per-chunk scale (the compression of "1-bit
 * Adam", Section 4.1 "Bagua Algorithms"):
 *   v = x + residual (v = x if NULL);  scale_c = mean over the chunk of |v| (fixed summation order);
 *   bit = (v >= 0);  residual <- v - (bit ? +scale_c : -scale_c).
 *   bits   device u32[ceil(n/32)], written; bit b of word w is element 32*w + b; unused tail bits are 0
 *   scale  device fp32[nc], written
 * Summation order of |v| within a chunk: groups of four consecutive elements reduced as
 * (|a|+|b|)+(|c|+|d|), group m added to accumulator m mod 64, the 64 accumulators combined by
 * acc[l] += acc[l xor s] for s = 1,2,4,8,16,32.  scale = sum * fl(1/C) for a full chunk with C a
 * power of two, else sum / (float)length.
 */
int bagua_sign_compress_ef(const float* x, float* residual, size_t n, size_t chunk,
                           uint32_t* bits, float* scale, void* stream);

/*
 * Decode a compressed bucket to fp32 (the last step of C_LP_S on every worker):
 *   MINMAX_U8: out = mn + code * fl(fl(mx - mn) / 255);   SIGN1: out = bit ? +scale : -scale.
 */
int bagua_decompress(int codec, const void* codes, const float* meta, size_t n, size_t chunk,
                     float* out, void* stream);

/*
 * C_LP_S with a third compression function: per-chunk top-K sparsification (the aggressive compression the paper
 * names when it motivates error compensation, Section 3.2).  Per chunk of C elements the `keep` entries of largest
 * |v| are kept (ties: the lower index wins; -0 and +0 compare equal).  A chunk is encoded as `keep` pairs in
 * ascending index order: idx = position inside the chunk (u16), val = v with -0 stored as +0; a last chunk shorter
 * than `keep` keeps everything and pads with idx 0xFFFF, val 0.  decode = 0 except at the kept positions, so the
 * error update is exact: residual <- v at dropped positions, +0 at kept ones.
 *   keep   1..chunk;   idx device u16[nc*keep];   val device fp32[nc*keep]   (chunk c owns slots [c*keep, (c+1)*keep))
 * bagua_compress_topk_ef:                   worker side, v = x + residual (residual NULL = no error compensation)
 * bagua_decompress_reduce_recompress_topk:  server side, a = (sum_j decode_j) * fl(1/k) in ascending j,
 *                                           w = a + server_residual, Q(w), server_residual <- w - decode(Q(w)),
 *                                           out_fp32 (optional) = decode(Q(w))
 * bagua_decompress_topk:                    out = decode(idx, val)
 */
int bagua_compress_topk_ef(const float* x, float* residual, size_t n, size_t chunk, size_t keep, uint16_t* idx,
                           float* val, void* stream);
int bagua_decompress_reduce_recompress_topk(const uint16_t* const* idx_in, const float* const* val_in, int k,
                                            size_t keep, float* server_residual, size_t n, size_t chunk,
                                            uint16_t* idx_out, float* val_out, float* out_fp32, void* stream);
int bagua_decompress_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep, float* out,
                          void* stream);

/*
 * Decode fused into the bucket-level optimizer step (Section 3.5: the stochastic-gradient optimizer also works
 * on the flattened bucket; in the appendix listing the primitive is followed by the optimizer step).  The
 * optimizer itself is not fixed by the paper; this entry point implements SGD with optional weight decay and
 * momentum (no dampening, no Nesterov), one rounding per operation in this order:
 *   g = decode(codes, meta);  if weight_decay != 0: g = g + weight_decay * p;
 *   if momentum_buf: m = momentum * m + g, u = m;  else u = g;      p = p - lr * u.
 * A zero-initialised momentum buffer gives the usual first step m = g.  The decoded gradient is not stored.
 *   codec, codes, meta   a compressed bucket as produced by bagua_decompress_reduce_recompress
 *   param                device fp32[n], updated in place
 *   momentum_buf         device fp32[n], updated in place, or NULL (no momentum; `momentum` is ignored)
 */
int bagua_decompress_sgd_step(int codec, const void* codes, const float* meta, size_t n, size_t chunk,
                              float* param, float* momentum_buf, float lr, float momentum, float weight_decay,
                              void* stream);

/*
 * The same step after a round with the per-chunk top-K codec (Section 3.2 names top-K as the aggressive compression;
 * Section 3.5: the optimizer works on the flattened bucket): g = the decoded sparse entries, +0 at every other element,
 * then the update above on EVERY element.  idx / val / keep as bagua_decompress_topk.  Without momentum and weight
 * decay (and with a finite lr >= +0) only the kept entries are touched, which gives the same bits.
 */
int bagua_decompress_sgd_step_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep,
                                   float* param, float* momentum_buf, float lr, float momentum, float weight_decay,
                                   void* stream);

/*
 * Decode fused into an Adam-type update of the flattened bucket (Section 3.5: the optimizer runs on the bucket;
 * Section 4.1: QSGD and 1-bit Adam are C_LP_S followed by the optimizer; the steps of 1-bit Adam are those of the
 * published algorithm the paper cites).  Adam without bias correction, one rounding per operation:
 *   d = decode(codes, meta)                                        (codec as in bagua_decompress)
 *   variance_frozen == 0 (d = averaged gradient):   m = beta1*m + (1-beta1)*d ;  v = beta2*v + (1-beta2)*(d*d)
 *   variance_frozen != 0 (compression stage of 1-bit Adam, d = averaged momentum):   m = d ;  v only read
 *   u = m / (sqrtf(v) + eps) ;  if weight_decay != 0: u = u + weight_decay*p ;  p = p - lr*u
 * (1-beta) is formed in fp32.  param, m, v: device fp32[n], in-out, 16-byte aligned, pairwise disjoint.
 */
int bagua_decompress_adam_step(int codec, const void* codes, const float* meta, size_t n, size_t chunk, float* param,
                               float* m, float* v, float lr, float beta1, float beta2, float eps, float weight_decay,
                               int variance_frozen, void* stream);

/*
 * The same step after a round with the per-chunk top-K codec (Section 3.2 top-K; Section 3.5 optimizer on the flattened
 * bucket): d = the decoded sparse entries, +0 at every other element, then the update above on EVERY element (where
 * nothing was kept m decays by beta1, v by beta2, and p still moves by the decayed momentum).  idx / val / keep as
 * bagua_decompress_topk; param, m, v as above.
 */
int bagua_decompress_adam_step_topk(const uint16_t* idx, const float* val, size_t n, size_t chunk, size_t keep,
                                    float* param, float* m, float* v, float lr, float beta1, float beta2, float eps,
                                    float weight_decay, int variance_frozen, void* stream);

/*
 * Worker side of the compression stage of 1-bit Adam (Section 4.1: 1-bit Adam = C_LP_S with error compensation,
 * applied to the momentum): compresses the local momentum u = beta1*m + (1-beta1)*g exactly as
 * bagua_sign_compress_ef compresses x (same codec, error state, layouts and limits).
 *   g  device fp32[n] gradient, read only;   m  device fp32[n], the momentum shared after the previous step, read only
 */
int bagua_momentum_sign_compress_ef(const float* g, const float* m, float beta1, float* residual, size_t n,
                                    size_t chunk, uint32_t* bits, float* scale, void* stream);

/*
 * Batched forms: B buckets that need not be contiguous in memory are processed by ONE launch, so a worker whose
 * buckets are separate allocations runs at the rate of one large launch instead of paying a launch (and its ramp-up
 * and drain) per 25 MiB bucket (Section 3.1 "Bucketing": the unit handed to the communication primitive is a bucket;
 * Section 3.5: primitives run on the flattened bucket).  Every bucket is processed exactly as the unbatched entry
 * point would process it (own chunk grid starting at its first element, own ragged last chunk), so results are
 * identical bit for bit to B separate calls.
 *   per-bucket arguments   host arrays of length B (pointers: device pointers; n: elements, each > 0)
 *   residual / server_residual / out_fp32   either NULL (none for any bucket) or an array with B non-NULL entries
 *   codes_in, meta_in (server step)   host[B*k], bucket-major: entry b*k + j is worker j's buffer for bucket b
 *   workspace   device, >= bagua_batch_workspace_bytes(B, k) bytes (k = 0 for the calls without workers),
 *               16-byte aligned; holds the bucket table, written by small launches on `stream` before the main
 *               launch (no host-to-device copy, no synchronisation; the host arrays may be reused on return).
 *               It must stay untouched until the call's work on `stream` has finished.
 * Alignment, aliasing and error rules as for the unbatched calls, applied over all buckets of the call.
 * bagua_bucket_flatten_batched_run launches the copy of B planned buckets (plans[b] from bagua_flatten_plan with
 * T[b] and bucket_numel[b]).
 */
size_t bagua_batch_workspace_bytes(size_t B, int k);
int bagua_compress_minmax_u8_batched(const float* const* x, float* const* residual, const size_t* n, size_t B,
                                     size_t chunk, uint8_t* const* codes, float* const* minmax, void* workspace,
                                     size_t workspace_bytes, void* stream);
int bagua_sign_compress_ef_batched(const float* const* x, float* const* residual, const size_t* n, size_t B,
                                   size_t chunk, uint32_t* const* bits, float* const* scale, void* workspace,
                                   size_t workspace_bytes, void* stream);
int bagua_decompress_reduce_recompress_batched(int codec, const void* const* codes_in, const float* const* meta_in,
                                               int k, float* const* server_residual, const size_t* n, size_t B,
                                               size_t chunk, void* const* codes_out, float* const* meta_out,
                                               float* const* out_fp32, void* workspace, size_t workspace_bytes,
                                               void* stream);
int bagua_bucket_flatten_batched_run(const void* const* plans, const size_t* T, float* const* bucket,
                                     const size_t* bucket_numel, size_t B, void* workspace, size_t workspace_bytes,
                                     void* stream);

/*
 * Measurement utilities used by the benchmark to state what the memory system of the GPU at hand delivers for
 * plain access patterns (the ceilings printed next to the roofline fractions); no arithmetic of the method.
 * bagua_probe_read: a read-only reduction, tile_sums[t] = sum of x[4096 t .. 4096 t + 4095] (device fp32[ceil(n/4096)]).
 * bagua_probe_streams: every wavefront owns one 256-element row and visits `seq` groups of streams one after
 * another; in a group it reads the row from nr fp32 streams, then writes it to nw fp32 streams and to nb byte
 * streams.  in: host[seq*nr], out: host[seq*nw], bout: host[seq*nb] of device pointers (16-byte aligned, n
 * elements each, n a multiple of 256); (nr, nw, nb) in {(1,1,0), (2,1,0), (2,1,1), (2,2,1), (4,4,0), (8,8,0), (1,8,0),
 * (8,1,0)}, BAGUA_ERR_UNSUPPORTED otherwise; seq*max(nr,nw,nb) <= BAGUA_MAX_WORKERS.
 */
int bagua_probe_read(const float* x, size_t n, float* tile_sums, void* stream);
int bagua_probe_streams(const float* const* in, float* const* out, uint8_t* const* bout, int nr, int nw, int nb,
                        int seq, size_t n, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BAGUA_HIP_H */
