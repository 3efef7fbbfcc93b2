/*
 * cgx.h -- C ABI of the MI355X (gfx950) implementation of the compute a rank
 * performs in CGX's compressed all-reduce (arXiv 2111.08617): bucketed
 * stochastic quantization of a fused gradient buffer, and the matching
 * dequantize-and-reduce / requantize of a Scatter-Reduce-Allgather.
 *
 * Common conventions
 *   Plan.  A fused buffer of n elements is described by L layers:
 *   layer_offsets[0..L] (host, int64, layer_offsets[0] = 0, non-decreasing,
 *   layer_offsets[L] = n; empty layers are allowed and skipped) and
 *   bits_per_layer[0..L-1] (host, uint8: 0 = pass-through, 1..8 = quantize to
 *   that many bits).  `bucket` is the bucket size in elements: a multiple of 32
 *   in [32, 8192] (powers of two take the vectorised kernel paths; the others
 *   a generic, several times slower one).  Buckets restart at every layer's
 *   first element; a layer's last bucket may be short.  Layers may start at any
 *   element (only the buffers' base addresses must be aligned, see Memory).
 *   (Paper Sec. 4.1: fused buffers keep the layer offsets, compression is per
 *   layer, small layers travel uncompressed; Sec. 4.3: buckets with per-bucket
 *   scaling meta-data.)
 *
 *   Packed stream.  For each non-empty layer, in order, one segment padded with
 *   zero bytes to a multiple of 16 bytes:
 *     quantized layer of len elements at b bits: ceil(len*b/8) bytes holding
 *       the codes as an LSB-first bitstream (code j in stream bits
 *       [j*b, (j+1)*b); stream bit t is bit t&7 of byte t>>3);
 *     pass-through layer: its len elements verbatim in the storage type.
 *   Meta.  Two floats {unit, min} per bucket, buckets numbered in layer order
 *   over the quantized layers.  A code q stands for fma(q, unit, min).
 *
 *   Memory.  Every pointer marked "device" is device memory owned by the
 *   caller, 16-byte aligned, valid until the work queued on `stream` has run.
 *   Pointers marked "host" are read during the call and may be reused on
 *   return.  `stream` is a hipStream_t passed as void* (NULL = the default
 *   stream).  No call synchronises the stream.
 *
 *   Plan tables and graph capture.  The library keeps a small device-resident
 *   table per distinct plan.  It is built on the first call with that plan,
 *   which allocates device memory and copies synchronously; later calls with the
 *   same plan only queue kernels.  (cgx_quantize on binary32 input and
 *   cgx_requantize, cgx_quantize on binary16 gradients of 2^24 elements or more,
 *   and the fused call on 2^27 or more, keep tables of their own beside the one
 *   the other calls share.)  At most 64 tables are kept: when a 65th arrives
 *   the least recently used one is freed, which waits for the device;
 *   cgx_shutdown() frees them all.
 *   A call on a stream that is capturing a graph records its launches into the
 *   graph, and those read the plan's table on every replay.  Therefore:
 *     - the table must exist before the capture: run the same call once, not
 *       captured, first; a captured call whose plan has no table yet returns
 *       CGX_ERR_CAPTURE and records nothing (it neither allocates nor copies in
 *       the middle of a capture), and the capture can go on;
 *     - a table used by a captured call is pinned: it is never the one freed for
 *       a new plan, so the graph stays valid however many other plans follow;
 *       only cgx_shutdown() frees it, after which such graphs must not be
 *       replayed;
 *     - no first call with a new plan may run while ANOTHER thread captures in
 *       the global capture mode (the runtime forbids allocations then).
 *
 *   Errors.  Every function returns CGX_OK or a negative cgx_status.  Argument
 *   errors are found on the host before anything is queued; nothing is written
 *   in that case.  Inputs must be finite with |x| < 2^126; other values do not
 *   fault but give unspecified codes.
 */
#ifndef CGX_H
#define CGX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CGX_OK = 0,
    CGX_ERR_NULL = -1,     /* a required pointer is NULL */
    CGX_ERR_SIZE = -2,     /* n or L negative, or n does not match layer_offsets[L] */
    CGX_ERR_OFFSETS = -3,  /* layer_offsets[0] != 0 or offsets decrease */
    CGX_ERR_BITS = -4,     /* a bits_per_layer entry above 8 */
    CGX_ERR_BUCKET = -5,   /* bucket not a multiple of 32 in [32, 8192] */
    CGX_ERR_PEERS = -6,    /* W outside [1, CGX_MAX_PEERS] */
    CGX_ERR_DTYPE = -7,    /* unknown storage type */
    CGX_ERR_HIP = -8,      /* the HIP runtime reported an error */
    CGX_ERR_ALIGN = -9,    /* a device pointer is not 16-byte aligned */
    CGX_ERR_CAPACITY = -10, /* the plan is larger than a no-allocation entry point's fixed tables */
    CGX_ERR_CAPTURE = -11  /* the stream is capturing a graph and the plan's tables do not exist yet */
} cgx_status;

typedef enum {
    CGX_F32 = 0,           /* gradient stored as IEEE binary32 */
    CGX_F16 = 1            /* gradient stored as IEEE binary16, arithmetic in binary32 */
} cgx_dtype;

#define CGX_MAX_PEERS 64
#define CGX_MAX_FUSED_PEERS 16   /* cgx_dequant_reduce_requantize takes at most this many chunks */

/*
 * Sizes of the packed stream and of the meta array for a plan (pure host
 * computation; follows the layout above).  Either output pointer may be NULL.
 */
int cgx_sizes(int64_t n, int32_t L, const int64_t *layer_offsets /* host [L+1] */,
              const uint8_t *bits_per_layer /* host [L] */, int32_t bucket, cgx_dtype dt,
              size_t *packed_bytes, size_t *meta_bytes);

/*
 * Bucketed stochastic quantization of a fused buffer (paper Sec. 2.3, "Gradient
 * Quantization": the rounding rule q(v_i, s); Sec. 4.3, buckets; Sec. 4.1, per-layer parameters).
 * Per bucket: mn = min, mx = max, Lv = 2^b - 1, unit = (mx - mn) / Lv,
 * inv16 = (Lv * 65536) / (mx - mn); unit = inv16 = 0 for a constant or
 * degenerate bucket; a zero minimum is stored as +0.  Per element with buffer
 * index i: T = trunc((x - mn) * inv16), code = min((T + u) >> 16, Lv), where u
 * is the 16-bit draw of a counter-based generator keyed on (seed, i).  All
 * arithmetic is binary32 without fused operations.  The rule's probability p of
 * taking the upper level is thereby cut to 16 bits: a code goes up with
 * probability floor(p * 65536) / 65536, never more than p and less than 2^-16
 * below it, so the expected value of a code lies at most 2^-16 of a step (on
 * average 2^-17) below the unbiased one; values on the grid (p = 0) stay exact.
 *   grad    device, n elements of dt
 *   packed  device, at least packed_bytes; every byte of it is written
 *   meta    device, at least meta_bytes
 */
int cgx_quantize(const void *grad, int64_t n, int32_t L, const int64_t *layer_offsets,
                 const uint8_t *bits_per_layer, int32_t bucket, uint64_t seed, cgx_dtype dt,
                 void *packed, void *meta, void *stream);

/*
 * Dequantize W compressed chunks of the same plan and sum them (paper Sec. 4:
 * compression is not associative, so chunks are decompressed before the sum;
 * Sec. 4.1, Scatter-Reduce-Allgather, first round on a rank's own share).
 * sum[i] = deq_0[i] + deq_1[i] + ... in that order in binary32, where
 * deq_w[i] = fma(code, unit, min) for quantized layers and the stored value,
 * widened to binary32, for pass-through layers.
 *   packed, meta  host arrays of W device pointers (chunk w's stream and meta)
 *   sum           device, n floats
 * A rank's share of a larger buffer is passed as a plan over the share alone.
 */
int cgx_dequant_reduce(const void *const *packed, const void *const *meta, int32_t W,
                       int64_t n, int32_t L, const int64_t *layer_offsets,
                       const uint8_t *bits_per_layer, int32_t bucket, cgx_dtype dt,
                       float *sum, void *stream);

/*
 * The same reduction when the rank's own contribution to its share is still uncompressed
 * (paper Sec. 4.1, Scatter-Reduce-Allgather: a node receives its chunk from all OTHER
 * nodes and aggregates it with its own): sum[i] = local[i] + deq_0[i] + ... + deq_{W-1}[i],
 * in that order in binary32, local widened to binary32 first.
 *   local  device, n elements of local_dt (binary32 or binary16), 16-byte aligned
 */
int cgx_dequant_reduce_add(const void *local, cgx_dtype local_dt, const void *const *packed,
                           const void *const *meta, int32_t W, int64_t n, int32_t L,
                           const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket,
                           cgx_dtype dt, float *sum, void *stream);

/*
 * Decompress one chunk into the gradient's storage type (paper Sec. 4.1,
 * Scatter-Reduce-Allgather, after the second round: every rank decompresses the
 * aggregated chunks it gathered): out[i] = fma(code, unit, min), or the stored value for
 * pass-through layers, rounded to nearest even when out_dt is CGX_F16.
 *   packed, meta  device, one chunk of the plan (pass-through layers stored as dt)
 *   out           device, n elements of out_dt
 */
int cgx_dequantize(const void *packed, const void *meta, int64_t n, int32_t L,
                   const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket,
                   cgx_dtype dt, cgx_dtype out_dt, void *out, void *stream);

/*
 * Compress the aggregated chunk again before it is broadcast (paper Sec. 4.1,
 * Scatter-Reduce-Allgather, second round): cgx_quantize on binary32 input.
 * Pass-through layers are written as binary32.
 */
int cgx_requantize(const float *sum, int64_t n, int32_t L, const int64_t *layer_offsets,
                   const uint8_t *bits_per_layer, int32_t bucket, uint64_t seed,
                   void *packed, void *meta, void *stream);

/*
 * cgx_dequant_reduce followed by cgx_requantize in one pass: the binary32 sums stay in
 * registers and never reach memory (paper Sec. 4.1, Scatter-Reduce-Allgather: a rank
 * aggregates its chunk and compresses the aggregate again before broadcasting it).  The
 * output is byte for byte what cgx_dequant_reduce into a buffer and cgx_requantize of that
 * buffer with the same seed would give: packed_out has the layout of the plan with dt =
 * CGX_F32 (pass-through layers hold the binary32 sums), meta_out its meta.
 *   packed, meta          host arrays of W device pointers, chunks of the plan with storage dt
 *   packed_out, meta_out  device, sizes from cgx_sizes(..., CGX_F32, ...)
 * W must be in [1, CGX_MAX_FUSED_PEERS] (CGX_ERR_PEERS otherwise).
 */
int cgx_dequant_reduce_requantize(const void *const *packed, const void *const *meta, int32_t W,
                                  int64_t n, int32_t L, const int64_t *layer_offsets,
                                  const uint8_t *bits_per_layer, int32_t bucket, cgx_dtype dt,
                                  uint64_t seed, void *packed_out, void *meta_out, void *stream);

/*
 * The calls above with a bucket size per layer (paper Sec. 4.1: compression parameters are
 * per layer, the bucket size among them; Sec. "Layer-wise Adaptive Quantization": bit-widths
 * and bucket sizes are mapped to the layers).  buckets_per_layer[0..L-1] (host, int32) gives
 * every layer its own bucket size, each a multiple of 32 in [32, 8192] (CGX_ERR_BUCKET
 * otherwise; the entries of pass-through and empty layers are checked but not used).
 * Layout, meta numbering (buckets in layer order), draws, sums and errors are those of the
 * calls above; with all entries equal the results are byte for byte those of the call with
 * that one size.  A call queues one launch for each of the three size classes in use among its
 * quantized layers (32-64, 96-2048, above 2048: each class has its own kernel instantiation)
 * and keeps one device table per class.
 */
int cgx_layered_sizes(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                      const int32_t *buckets_per_layer /* host [L] */, cgx_dtype dt, size_t *packed_bytes,
                      size_t *meta_bytes);
int cgx_layered_quantize(const void *grad, int64_t n, int32_t L, const int64_t *layer_offsets,
                         const uint8_t *bits_per_layer, const int32_t *buckets_per_layer, uint64_t seed,
                         cgx_dtype dt, void *packed, void *meta, void *stream);
int cgx_layered_dequant_reduce(const void *const *packed, const void *const *meta, int32_t W, int64_t n,
                               int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                               const int32_t *buckets_per_layer, cgx_dtype dt, float *sum, void *stream);
int cgx_layered_dequant_reduce_add(const void *local, cgx_dtype local_dt, const void *const *packed,
                                   const void *const *meta, int32_t W, int64_t n, int32_t L,
                                   const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                                   const int32_t *buckets_per_layer, cgx_dtype dt, float *sum, void *stream);
int cgx_layered_dequantize(const void *packed, const void *meta, int64_t n, int32_t L,
                           const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                           const int32_t *buckets_per_layer, cgx_dtype dt, cgx_dtype out_dt, void *out,
                           void *stream);
int cgx_layered_requantize(const float *sum, int64_t n, int32_t L, const int64_t *layer_offsets,
                           const uint8_t *bits_per_layer, const int32_t *buckets_per_layer, uint64_t seed,
                           void *packed, void *meta, void *stream);
int cgx_layered_dequant_reduce_requantize(const void *const *packed, const void *const *meta, int32_t W,
                                          int64_t n, int32_t L, const int64_t *layer_offsets,
                                          const uint8_t *bits_per_layer, const int32_t *buckets_per_layer,
                                          cgx_dtype dt, uint64_t seed, void *packed_out, void *meta_out,
                                          void *stream);
/* cgx_layer_sqerrors and its workspace size for a chunk written by cgx_layered_quantize. */
int cgx_layered_stats_workspace(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                                const int32_t *buckets_per_layer, cgx_dtype dt, size_t *bytes);
int cgx_layered_layer_sqerrors(const void *grad, const void *packed, const void *meta, int64_t n, int32_t L,
                               const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                               const int32_t *buckets_per_layer, cgx_dtype dt, double *sqerr, void *workspace,
                               size_t workspace_bytes, void *stream);

/*
 * The norm-and-sign form of the quantizer: Q_s of paper Sec. 2.3
 * (Q_s(v_i) = ||v|| sign(v_i) q(|v_i| / ||v||, s)) applied per bucket (Sec. 4.3)
 * with per-layer widths (Sec. 4.1) and with the bucket's LARGEST MAGNITUDE as
 * ||v|| (the l-infinity norm: a variant of the printed form, which uses the l2
 * norm; with it all s levels are in use).  Same plan, layout of the packed stream,
 * draws, pass-through layers, summation order and error codes as the calls
 * above; what differs:
 *   - the norm of a bucket is its largest magnitude (so that |v_i| / ||v||
 *     covers [0, 1] and no summation order enters the result);
 *   - level = min((trunc(|x| * inv16) + u) >> 16, s), s = 2^(b-1) - 1; b must
 *     be in 2..8 (CGX_ERR_BITS for a 1-bit layer);
 *   - a b-bit code is the signed level sign(x) * level in -s..s as a two's
 *     complement number (the sign is that of the value's sign bit; level 0 has
 *     the one code 0);
 *   - meta is ONE float per bucket, unit = ||v|| / s (0 for an all-zero or
 *     degenerate bucket, as is inv16 = (s * 65536) / ||v||);
 *   - the value of a code is (float)signed_level * unit, one binary32
 *     multiplication.
 * cgx_qsgd_sizes: packed_bytes as cgx_sizes, meta_bytes = 4 * buckets.
 * cgx_qsgd_quantize: as cgx_quantize (dt = CGX_F32 serves as the requantize
 * of a reduced chunk).  cgx_qsgd_dequant_reduce: as cgx_dequant_reduce.
 * cgx_qsgd_dequant_reduce_requantize: as cgx_dequant_reduce_requantize.
 */
int cgx_qsgd_sizes(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                   int32_t bucket, cgx_dtype dt, size_t *packed_bytes, size_t *meta_bytes);
int cgx_qsgd_quantize(const void *grad, int64_t n, int32_t L, const int64_t *layer_offsets,
                      const uint8_t *bits_per_layer, int32_t bucket, uint64_t seed, cgx_dtype dt,
                      void *packed, void *meta, void *stream);
int cgx_qsgd_dequant_reduce(const void *const *packed, const void *const *meta, int32_t W, int64_t n,
                            int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                            int32_t bucket, cgx_dtype dt, float *sum, void *stream);
int cgx_qsgd_dequant_reduce_requantize(const void *const *packed, const void *const *meta, int32_t W,
                                       int64_t n, int32_t L, const int64_t *layer_offsets,
                                       const uint8_t *bits_per_layer, int32_t bucket, cgx_dtype dt,
                                       uint64_t seed, void *packed_out, void *meta_out, void *stream);

/* The norm-and-sign calls with a bucket size per layer (see the cgx_layered_* calls above). */
int cgx_qsgd_layered_sizes(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                           const int32_t *buckets_per_layer, cgx_dtype dt, size_t *packed_bytes,
                           size_t *meta_bytes);
int cgx_qsgd_layered_quantize(const void *grad, int64_t n, int32_t L, const int64_t *layer_offsets,
                              const uint8_t *bits_per_layer, const int32_t *buckets_per_layer, uint64_t seed,
                              cgx_dtype dt, void *packed, void *meta, void *stream);
int cgx_qsgd_layered_dequant_reduce(const void *const *packed, const void *const *meta, int32_t W, int64_t n,
                                    int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                                    const int32_t *buckets_per_layer, cgx_dtype dt, float *sum, void *stream);
int cgx_qsgd_layered_dequant_reduce_requantize(const void *const *packed, const void *const *meta, int32_t W,
                                               int64_t n, int32_t L, const int64_t *layer_offsets,
                                               const uint8_t *bits_per_layer, const int32_t *buckets_per_layer,
                                               cgx_dtype dt, uint64_t seed, void *packed_out, void *meta_out,
                                               void *stream);

/*
 * Per-layer statistics for the layer-wise adaptive scheme (paper Sec. "Layer-wise
 * Adaptive Quantization").  Sums are binary64; squares of binary32 values and
 * differences of two binary32 values are exact in binary64, so only the additions
 * round, and their order is fixed (no atomics): a result is reproducible bit for bit
 * and lies within (140 + tiles_of_the_layer / 64) * 2^-53, relative, of the exact sum.
 *
 * cgx_layer_sqnorms: sqnorm[l] = sum of x_i^2 over layer l of buf (n elements of dt):
 * the squared "norm(G_l)" of Algorithm 1 when buf holds the accumulated gradient.
 * cgx_layer_sqerrors / cgx_qsgd_layer_sqerrors: sqerr[l] = sum over layer l of
 * (grad_i - value of its code)^2 for a chunk written by cgx_quantize /
 * cgx_qsgd_quantize from grad with the same plan: the squared l2 norm of the
 * compression error that the problem definition bounds by alpha * E_4; 0 for
 * pass-through and empty layers.
 *   sqnorm, sqerr  device, L doubles (8-byte aligned), every entry written
 *   workspace      device, 16-byte aligned, at least the bytes cgx_layer_stats_workspace
 *                  reports for the same plan (bits_per_layer = NULL and any valid bucket
 *                  for cgx_layer_sqnorms); holds one partial sum per wavefront work item
 *                  during the call, contents unspecified afterwards; CGX_ERR_SIZE if it
 *                  is too small.  Calls that share a workspace must not overlap.
 */
int cgx_layer_stats_workspace(int64_t n, int32_t L, const int64_t *layer_offsets,
                              const uint8_t *bits_per_layer /* NULL: for cgx_layer_sqnorms */,
                              int32_t bucket, cgx_dtype dt, size_t *bytes);
int cgx_layer_sqnorms(const void *buf, int64_t n, int32_t L, const int64_t *layer_offsets, cgx_dtype dt,
                      double *sqnorm, void *workspace, size_t workspace_bytes, void *stream);
int cgx_layer_sqerrors(const void *grad, const void *packed, const void *meta, int64_t n, int32_t L,
                       const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket,
                       cgx_dtype dt, double *sqerr, void *workspace, size_t workspace_bytes, void *stream);
int cgx_qsgd_layer_sqerrors(const void *grad, const void *packed, const void *meta, int64_t n, int32_t L,
                            const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket,
                            cgx_dtype dt, double *sqerr, void *workspace, size_t workspace_bytes,
                            void *stream);

/*
 * cgx_layer_sqnorms for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same result, bit for bit, as
 * cgx_layer_sqnorms; no workspace argument: the tile table, its numbering and the partial sums
 * live in a fixed array of 11.1 MB inside the library's device
 * code, one copy per GPU, held until the process ends.  The call allocates nothing on the
 * device (no hipMalloc, no hipFree, no table cache) and copies nothing from host memory on the
 * stream: the layer table travels in kernel arguments, ceil((L + 1) / 192) small launches
 * ahead of the three that compute.
 * Limits: L <= CGX_NOALLOC_MAX_LAYERS, and at most CGX_NOALLOC_MAX_TILES work items (a layer of
 * len elements takes ceil(len / 8192) of them); beyond either the call returns
 * CGX_ERR_CAPACITY and queues nothing.  The other errors are those of cgx_layer_sqnorms.
 * Every call on a GPU uses that GPU's one array: calls on different streams of one GPU, or
 * from different threads, must not overlap (calls queued on one stream are ordered and safe).
 */
#define CGX_NOALLOC_MAX_LAYERS 4096
#define CGX_NOALLOC_MAX_TILES 262144
int cgx_layer_sqnorms_noalloc(const void *buf, int64_t n, int32_t L, const int64_t *layer_offsets, cgx_dtype dt,
                              double *sqnorm, void *stream);

/*
 * Bit-width assigners of the layer-wise adaptive scheme (same section; host only, no
 * device work).  Inputs: the layer table, one non-negative number per layer
 * (layer_norms: the l2 norm of the layer's accumulated gradient, i.e. the square root of
 * cgx_layer_sqnorms' output), bits_in (0 marks a layer that stays uncompressed, as in
 * every plan), and k candidate widths in 1..8 (any order; used in ascending order).
 * bits_out[l] is 0 for layers with bits_in[l] == 0 or no elements, else one of the
 * candidates; it is a valid bits_per_layer for every call above.
 *
 * cgx_assign_bits_kmeans (Algorithm 1): each taking-part layer is the point
 * (size, norm), both axes scaled to [0, 1] by their minimum and maximum over those
 * layers (an axis without spread becomes 0).  Lloyd's k-means with k clusters: the
 * points are ordered by norm - size (ties: layer order), cluster c starts at the point
 * of rank floor((c + 1/2) * M / k); every point goes to its nearest centroid (squared
 * Euclidean distance, ties to the lowest index); centroids become the means of their
 * points (an empty cluster keeps its centroid); stop when nothing moves or after
 * max_iter rounds.  Non-empty clusters are ranked by centroid norm - size, ascending;
 * rank r of m gets candidate number round_half_up(r * (k - 1) / (m - 1)) (m = 1: the
 * largest), so large layers with small gradients get the fewest bits.  With M <= k
 * points every point is its own cluster.
 * cgx_assign_bits_linear (the sort-and-interpolate heuristic): layers ordered by
 * norm / size, ascending (ties: layer order); rank r of M gets candidate number
 * floor(r * k / M).
 * Errors: CGX_ERR_NULL, CGX_ERR_SIZE (L < 0, k outside 1..64, max_iter < 1),
 * CGX_ERR_OFFSETS, CGX_ERR_BITS (a candidate outside 1..8, bits_in above 8).
 */
int cgx_assign_bits_kmeans(int32_t L, const int64_t *layer_offsets /* host [L+1] */,
                           const double *layer_norms /* host [L] */, const uint8_t *bits_in /* host [L] */,
                           const uint8_t *candidates /* host [k] */, int32_t k, int32_t max_iter,
                           uint8_t *bits_out /* host [L] */);
int cgx_assign_bits_linear(int32_t L, const int64_t *layer_offsets, const double *layer_norms,
                           const uint8_t *bits_in, const uint8_t *candidates, int32_t k, uint8_t *bits_out);

/*
 * Bucket sizes to go with assigned widths (same section: bit-widths and bucket sizes are mapped
 * to the layers linearly; no rule is printed for the sizes).  The position of a layer's width
 * among the ascending width candidates decides, linearly, its position among the DESCENDING
 * bucket candidates, so the layers with the fewest bits also get the longest buckets: width
 * number i of k takes bucket number round_half_up(i * (kb - 1) / (k - 1)) of kb (k = 1: the
 * longest).  Layers with width 0 get the longest size (unused, but valid for cgx_layered_*).
 * buckets_out is a valid buckets_per_layer for the cgx_layered_* calls.  Host only.
 * Errors: CGX_ERR_NULL, CGX_ERR_SIZE (L < 0, k or kb outside 1..64), CGX_ERR_BITS (a candidate
 * outside 1..8, or a width that is neither 0 nor a candidate), CGX_ERR_BUCKET (a bucket
 * candidate that is not a multiple of 32 in [32, 8192]).
 */
int cgx_assign_buckets_from_bits(int32_t L, const uint8_t *bits_per_layer /* host [L] */,
                                 const uint8_t *width_candidates /* host [k] */, int32_t k,
                                 const int32_t *bucket_candidates /* host [kb] */, int32_t kb,
                                 int32_t *buckets_out /* host [L] */);

/* Human-readable name of a status code (static storage). */
const char *cgx_status_string(int status);

/* Frees the cached plan tables.  Call with no work of this library in flight. */
int cgx_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* CGX_H */
