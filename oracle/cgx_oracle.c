/*
 * cgx_oracle.c -- plain CPU oracle for bucketed stochastic gradient quantization
 * and the matching dequantize-and-reduce step of a compressed scatter-reduce.
 *
 * THIS IS TEST INFRASTRUCTURE.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code with the GPU
 * library and the product path never routes through it.
 *
 * What it follows (CGX paper, arXiv 2111.08617):
 *   - Sec. 2.3 "Gradient Quantization", the definition of q(v_i, s): a value
 *     normalised to a in [0,1] falls in the interval [l/s, (l+1)/s] and is
 *     rounded to level l+1 with probability p = a*s - l, else to level l.
 *   - Sec. 4.3 "Efficient Quantization": the vector is split into buckets,
 *     each compressed independently, with scaling meta-data kept per bucket.
 *   - Sec. 4.1 "The Native CGX Framework" (layer filters): compression is done
 *     per layer using the layer offsets inside the fused buffer; small layers
 *     (bias, normalisation) travel uncompressed.
 *   - Sec. 4.1 "Choosing a Reduction Scheme" (Scatter-Reduce-Allgather) and
 *     Sec. 4 on non-associativity: a rank decompresses every received chunk
 *     and only then sums; the aggregated chunk is compressed again.
 *
 * The paper leaves every bit-level choice open.  The readings used here:
 *   - scaling is affine per bucket: mn = min, mx = max, s = Lv = 2^b - 1
 *     intervals, a = (x - mn) / (mx - mn); meta = {unit, mn} with
 *     unit = (mx - mn) / Lv.
 *   - all quantizer arithmetic is IEEE binary32, round to nearest even, no
 *     fused operations, subnormals kept (the integer code is decided in the
 *     kernel's precision).
 *   - the probability p is resolved to 16 bits: with S = (x - mn) * inv16,
 *     inv16 = (Lv * 65536) / (mx - mn), T = trunc(S) and a uniform 16-bit
 *     draw u, the code is q = min(floor((T + u) / 65536), Lv).  So level
 *     l = floor(T / 65536) goes up with probability (T mod 65536) / 65536,
 *     which is p truncated to 16 bits.
 *   - u comes from a counter-based generator keyed on (seed, element index in
 *     the buffer passed to the call): one 32-bit word per aligned pair of
 *     elements, low half for the even element, high half for the odd one.
 *     PARITY UNPINNED for the generator's stream: the paper only says "with
 *     probability"; the tests pin its statistical quality, not its bits.
 *   - codes of one layer form an LSB-first bitstream (code j occupies stream
 *     bits [j*b, (j+1)*b), stream bit t is bit t&7 of byte t>>3); each layer's
 *     segment is zero padded to a multiple of 16 bytes; segments follow each
 *     other in layer order.  Pass-through layers (bits == 0) are copied in
 *     their storage type.
 *   - dequantized value = fma(q, unit, mn) in binary32; the reduce adds the
 *     peers in ascending order in binary32 (sum32) and, separately, evaluates
 *     sum_w (mn_w + q_w * unit_w) in binary64 (sum64).
 *   - the second half of the file holds the norm-and-sign form of the same
 *     quantizer (the formula Q_s of Sec. 2.3 taken literally), with its own
 *     header comment.
 *
 * Build:  gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)

enum { DT_F32 = 0, DT_F16 = 1 };

/* ---- storage types ------------------------------------------------------ */

/* IEEE binary16 -> binary32, written out from the format definition. */
static float half_to_float(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int exp = (h >> 10) & 0x1f;
    int man = h & 0x3ff;
    float v;
    if (exp == 0)
        v = ldexpf((float)man, -24);            /* zero and subnormals: man * 2^-24 */
    else if (exp == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexpf((float)(man | 0x400), exp - 25); /* (1024 + man) * 2^(exp-15-10) */
    return sign ? -v : v;
}

/* binary32 -> binary16, round to nearest, ties to even, from the format definition:
 * normal results are (1024 + m) * 2^(e-10) with e in [-14, 15], subnormal ones m * 2^-24. */
static uint16_t float_to_half(float f)
{
    uint16_t sign = signbit(f) ? 0x8000u : 0u;
    float a = fabsf(f);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0f) return (uint16_t)(sign | 0x7c00u);   /* half way between the largest half and 2^16, or above */
    if (a < 6.103515625e-05f) {                              /* below 2^-14: subnormal, units of 2^-24 */
        int m = (int)nearbyintf(ldexpf(a, 24));              /* exact scaling; ties to even */
        return (uint16_t)(sign | m);                         /* m == 1024 is the smallest normal */
    }
    int e;
    float frac = frexpf(a, &e);                              /* a = frac * 2^e, frac in [0.5, 1) */
    int m = (int)nearbyintf(ldexpf(frac, 11));               /* in [1024, 2048] */
    e -= 1;                                                  /* a = (m / 1024) * 2^e */
    if (m == 2048) { m = 1024; e += 1; }
    return (uint16_t)(sign | ((e + 15) << 10) | (m - 1024));
}

void oracle_float_to_half(const float *in, int64_t count, uint16_t *out)
{
    for (int64_t k = 0; k < count; k++) out[k] = float_to_half(in[k]);
}

static float load_elem(const void *buf, int64_t i, int dt)
{
    if (dt == DT_F16)
        return half_to_float(((const uint16_t *)buf)[i]);
    return ((const float *)buf)[i];
}

static int elem_size(int dt) { return dt == DT_F16 ? 2 : 4; }

/* ---- counter-based generator -------------------------------------------- */

/* A 32-bit avalanche finalizer of the multiply / xor-shift family
 * (two odd multipliers, three xor-shifts); it is a bijection on 32 bits. */
static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

/* One 32-bit word per (seed, pair index).  The key folds the seed and the
 * upper half of the pair index; the lower half is the counter. */
uint32_t oracle_rng32(uint64_t seed, uint64_t pair)
{
    uint32_t seed_lo = (uint32_t)seed, seed_hi = (uint32_t)(seed >> 32);
    uint32_t pair_lo = (uint32_t)pair, pair_hi = (uint32_t)(pair >> 32);
    uint32_t key = mix32(seed_lo ^ mix32(seed_hi ^ 0x9e3779b9U ^ pair_hi));
    return mix32(pair_lo ^ key);
}

/* The 16-bit uniform draw of element i. */
uint32_t oracle_u16(uint64_t seed, uint64_t i)
{
    uint32_t r = oracle_rng32(seed, i >> 1);
    return (i & 1) ? (r >> 16) : (r & 0xffffU);
}

/* Draws of elements i0 .. i0+count-1, for the statistical tests of the generator. */
void oracle_fill_u16(uint64_t seed, uint64_t i0, int64_t count, uint16_t *out)
{
    for (int64_t k = 0; k < count; k++) out[k] = (uint16_t)oracle_u16(seed, i0 + (uint64_t)k);
}

/* ---- layout -------------------------------------------------------------- */

static uint64_t round_up16(uint64_t v) { return (v + 15u) & ~(uint64_t)15u; }

static int check_plan(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                      int32_t bucket, int dt)
{
    if (n < 0 || L < 0 || (L > 0 && (!off || !bits))) return ORACLE_ERR_ARG;
    if (bucket < 32 || bucket > 8192 || bucket % 32) return ORACLE_ERR_ARG;
    if (dt != DT_F32 && dt != DT_F16) return ORACLE_ERR_ARG;
    if (L == 0) return n == 0 ? ORACLE_OK : ORACLE_ERR_ARG;
    if (off[0] != 0 || off[L] != n) return ORACLE_ERR_ARG;
    for (int32_t l = 0; l < L; l++) {
        if (off[l + 1] < off[l]) return ORACLE_ERR_ARG;
        if (bits[l] > 8) return ORACLE_ERR_ARG;
    }
    return ORACLE_OK;
}

/*
 * A bucket size per layer (CGX paper Sec. 4.1: compression parameters, the bucket size among
 * them, are per layer; the adaptive scheme maps bit-widths and bucket sizes to layers):
 * layer_buckets == NULL means `bucket` for every layer.
 */
static int check_layer_buckets(int32_t L, const int32_t *layer_buckets)
{
    if (!layer_buckets) return ORACLE_OK;
    for (int32_t l = 0; l < L; l++)
        if (layer_buckets[l] < 32 || layer_buckets[l] > 8192 || layer_buckets[l] % 32) return ORACLE_ERR_ARG;
    return ORACLE_OK;
}
static int32_t bucket_of(int32_t l, int32_t bucket, const int32_t *layer_buckets)
{
    return layer_buckets ? layer_buckets[l] : bucket;
}

/* Bytes of layer l's segment in the packed stream and its bucket count. */
static void layer_extent(int64_t len, int b, int32_t bucket, int dt,
                         uint64_t *seg_bytes, uint64_t *n_buckets)
{
    if (len == 0) { *seg_bytes = 0; *n_buckets = 0; return; }
    if (b == 0) {
        *seg_bytes = round_up16((uint64_t)len * elem_size(dt));
        *n_buckets = 0;
    } else {
        *seg_bytes = round_up16(((uint64_t)len * b + 7) / 8);
        *n_buckets = ((uint64_t)len + bucket - 1) / bucket;
    }
}

static int sizes_impl(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket,
                      const int32_t *layer_buckets, int32_t dt, uint64_t *packed_bytes, uint64_t *meta_bytes)
{
    int rc = check_plan(n, L, off, bits, layer_buckets ? 32 : bucket, dt);
    if (rc) return rc;
    rc = check_layer_buckets(L, layer_buckets);
    if (rc) return rc;
    uint64_t pb = 0, nb = 0;
    for (int32_t l = 0; l < L; l++) {
        uint64_t s, k;
        layer_extent(off[l + 1] - off[l], bits[l], bucket_of(l, bucket, layer_buckets), dt, &s, &k);
        pb += s;
        nb += k;
    }
    if (packed_bytes) *packed_bytes = pb;
    if (meta_bytes) *meta_bytes = 8 * nb;
    return ORACLE_OK;
}

int oracle_sizes(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                 int32_t bucket, int32_t dt, uint64_t *packed_bytes, uint64_t *meta_bytes)
{
    return sizes_impl(n, L, off, bits, bucket, NULL, dt, packed_bytes, meta_bytes);
}

int oracle_layered_sizes(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                         const int32_t *layer_buckets, int32_t dt, uint64_t *packed_bytes, uint64_t *meta_bytes)
{
    if (L > 0 && !layer_buckets) return ORACLE_ERR_ARG;
    return sizes_impl(n, L, off, bits, 32, layer_buckets, dt, packed_bytes, meta_bytes);
}

/* ---- quantize ------------------------------------------------------------ */

/* Scale of one bucket: min, max, step and the 16.16 fixed-point multiplier. */
static void bucket_scale(const void *grad, int64_t first, int64_t count, int dt, int b,
                         float *unit, float *mn, float *inv16)
{
    float lo = load_elem(grad, first, dt), hi = lo;
    for (int64_t j = 1; j < count; j++) {
        float x = load_elem(grad, first + j, dt);
        if (x < lo) lo = x;
        if (x > hi) hi = x;
    }
    if (lo == 0.0f) lo = 0.0f;      /* a zero minimum is stored as +0, whatever its sign was */
    int levels = (1 << b) - 1;      /* Lv: number of intervals; codes are 0..Lv */
    float range = hi - lo;
    float u = range / (float)levels;
    float iv = (float)(levels * 65536) / range;
    if (!(u > 0.0f) || !isfinite(u) || !isfinite(iv)) {
        u = 0.0f;                   /* constant or degenerate bucket: every code is 0 */
        iv = 0.0f;
    }
    *unit = u;
    *mn = lo;
    *inv16 = iv;
}

/* Code of one element given its bucket's scale and its 16-bit draw. */
static uint32_t quantize_elem(float x, float mn, float inv16, int b, uint32_t u16)
{
    uint32_t levels = (1u << b) - 1u;
    float d = x - mn;
    float S = d * inv16;            /* position on the grid, in units of 1/65536 of a step */
    uint64_t T;                     /* trunc(S), saturating; not-a-number gives 0 */
    if (!(S >= 0.0f)) T = 0;
    else if (S >= 4294967296.0f) T = 0xffffffffu;
    else T = (uint64_t)S;
    uint64_t q = (T + u16) >> 16;   /* floor((T + u) / 65536): up iff (T mod 65536) + u >= 65536 */
    return q > levels ? levels : (uint32_t)q;
}

static void put_bits(uint8_t *stream, uint64_t bitpos, uint32_t code, int b)
{
    for (int k = 0; k < b; k++) {
        uint64_t t = bitpos + (uint64_t)k;
        if ((code >> k) & 1u) stream[t >> 3] |= (uint8_t)(1u << (t & 7));
    }
}

static uint32_t get_bits(const uint8_t *stream, uint64_t bitpos, int b)
{
    uint32_t code = 0;
    for (int k = 0; k < b; k++) {
        uint64_t t = bitpos + (uint64_t)k;
        code |= (uint32_t)((stream[t >> 3] >> (t & 7)) & 1u) << k;
    }
    return code;
}

/*
 * Quantize a fused buffer.  If draws != NULL it supplies the 16-bit draw of
 * every element (draws[i] for buffer index i) instead of the generator: the
 * tests use that to enumerate the rounding rule exhaustively.
 */
static int quantize_impl(const void *grad, int64_t n, int32_t L, const int64_t *off,
                         const uint8_t *bits, int32_t uniform_bucket, const int32_t *layer_buckets,
                         uint64_t seed, int32_t dt,
                         const uint16_t *draws, uint64_t index_base, uint8_t *packed, float *meta)
{
    int rc = check_plan(n, L, off, bits, layer_buckets ? 32 : uniform_bucket, dt);
    if (rc) return rc;
    rc = check_layer_buckets(L, layer_buckets);
    if (rc) return rc;
    uint64_t seg_start = 0, bucket0 = 0;
    for (int32_t l = 0; l < L; l++) {
        int64_t first = off[l], len = off[l + 1] - off[l];
        int b = bits[l];
        const int32_t bucket = bucket_of(l, uniform_bucket, layer_buckets);
        uint64_t seg_bytes, n_buckets;
        layer_extent(len, b, bucket, dt, &seg_bytes, &n_buckets);
        if (len == 0) continue;
        uint8_t *seg = packed + seg_start;
        memset(seg, 0, seg_bytes);
        if (b == 0) {
            memcpy(seg, (const uint8_t *)grad + (uint64_t)first * elem_size(dt),
                   (uint64_t)len * elem_size(dt));
        } else {
            /* buckets restart at the layer's first element; the last may be short */
#pragma omp parallel for schedule(static)
            for (int64_t k = 0; k < (int64_t)n_buckets; k++) {
                int64_t j0 = k * bucket;
                int64_t count = len - j0 < bucket ? len - j0 : bucket;
                float unit, mn, inv16;
                bucket_scale(grad, first + j0, count, dt, b, &unit, &mn, &inv16);
                meta[2 * (bucket0 + k) + 0] = unit;
                meta[2 * (bucket0 + k) + 1] = mn;
                for (int64_t j = j0; j < j0 + count; j++) {
                    uint64_t i = (uint64_t)(first + j);      /* index in the buffer handed in */
                    uint32_t u16 = draws ? draws[i] : oracle_u16(seed, index_base + i);
                    uint32_t q = quantize_elem(load_elem(grad, first + j, dt), mn, inv16, b, u16);
                    put_bits(seg, (uint64_t)j * b, q, b);
                }
            }
        }
        seg_start += seg_bytes;
        bucket0 += n_buckets;
    }
    return ORACLE_OK;
}

int oracle_quantize(const void *grad, int64_t n, int32_t L, const int64_t *off,
                    const uint8_t *bits, int32_t bucket, uint64_t seed, int32_t dt,
                    uint8_t *packed, float *meta)
{
    return quantize_impl(grad, n, L, off, bits, bucket, NULL, seed, dt, NULL, 0, packed, meta);
}

/*
 * The same for a window of a larger buffer: element i of `grad` is element
 * index_base + i of that buffer, which only matters for the draws (they are keyed on
 * the position in the whole buffer).  Lets a test check a slice of a buffer too
 * large to hand to the oracle in one piece.
 */
int oracle_quantize_window(const void *grad, int64_t n, int32_t L, const int64_t *off,
                           const uint8_t *bits, int32_t bucket, uint64_t seed, int32_t dt,
                           uint64_t index_base, uint8_t *packed, float *meta)
{
    return quantize_impl(grad, n, L, off, bits, bucket, NULL, seed, dt, NULL, index_base, packed, meta);
}

/* Every layer with its own bucket size (see check_layer_buckets). */
int oracle_layered_quantize(const void *grad, int64_t n, int32_t L, const int64_t *off,
                            const uint8_t *bits, const int32_t *layer_buckets, uint64_t seed, int32_t dt,
                            uint8_t *packed, float *meta)
{
    if (L > 0 && !layer_buckets) return ORACLE_ERR_ARG;
    return quantize_impl(grad, n, L, off, bits, 32, layer_buckets, seed, dt, NULL, 0, packed, meta);
}

int oracle_quantize_with_draws(const void *grad, int64_t n, int32_t L, const int64_t *off,
                               const uint8_t *bits, int32_t bucket, int32_t dt,
                               const uint16_t *draws, uint8_t *packed, float *meta)
{
    if (!draws) return ORACLE_ERR_ARG;
    return quantize_impl(grad, n, L, off, bits, bucket, NULL, 0, dt, draws, 0, packed, meta);
}

/* ---- dequantize and reduce ---------------------------------------------- */

/*
 * For every element of the buffer: sum over the W peers of the dequantized
 * value (pass-through layers: of the stored value), optionally preceded by the
 * rank's own uncompressed value local[i] (local == NULL: no such term).
 *   sum32[i]: binary32; terms are local[i] widened to binary32, then
 *             deq_w = fmaf(q, unit, mn) for w = 0..W-1, added in that order.
 *   sum64[i]: binary64 evaluation of local + sum_w (mn_w + q_w * unit_w).
 *   abs64[i]: binary64 sum of the absolute values of the terms, the scale of the tolerance.
 * Any of the three outputs may be NULL.
 */
static int reduce_impl(const void *local, int32_t local_dt, const uint8_t *const *packed,
                       const float *const *meta, int32_t W, int64_t n, int32_t L, const int64_t *off,
                       const uint8_t *bits, int32_t uniform_bucket, const int32_t *layer_buckets, int32_t dt,
                       float *sum32, double *sum64, double *abs64)
{
    int rc = check_plan(n, L, off, bits, layer_buckets ? 32 : uniform_bucket, dt);
    if (rc) return rc;
    rc = check_layer_buckets(L, layer_buckets);
    if (rc) return rc;
    if (W < 1 || !packed || !meta) return ORACLE_ERR_ARG;
    if (local && local_dt != DT_F32 && local_dt != DT_F16) return ORACLE_ERR_ARG;
    uint64_t seg_start = 0, bucket0 = 0;
    for (int32_t l = 0; l < L; l++) {
        int64_t first = off[l], len = off[l + 1] - off[l];
        int b = bits[l];
        const int32_t bucket = bucket_of(l, uniform_bucket, layer_buckets);
        uint64_t seg_bytes, n_buckets;
        layer_extent(len, b, bucket, dt, &seg_bytes, &n_buckets);
        if (len == 0) continue;
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < len; j++) {
            float acc32 = 0.0f;
            double acc64 = 0.0, accabs = 0.0;
            int started = 0;
            if (local) {
                acc32 = load_elem(local, first + j, local_dt);
                acc64 = (double)acc32;
                accabs = fabs(acc64);
                started = 1;
            }
            for (int32_t w = 0; w < W; w++) {
                const uint8_t *seg = packed[w] + seg_start;
                float v32;
                double v64;
                if (b == 0) {
                    v32 = load_elem(seg, j, dt);
                    v64 = (double)v32;
                } else {
                    uint64_t g = bucket0 + (uint64_t)(j / bucket);
                    float unit = meta[w][2 * g + 0], mn = meta[w][2 * g + 1];
                    uint32_t q = get_bits(seg, (uint64_t)j * b, b);
                    v32 = fmaf((float)q, unit, mn);
                    v64 = (double)mn + (double)q * (double)unit;
                }
                acc32 = started ? acc32 + v32 : v32;
                started = 1;
                acc64 += v64;
                accabs += fabs(v64);
            }
            if (sum32) sum32[first + j] = acc32;
            if (sum64) sum64[first + j] = acc64;
            if (abs64) abs64[first + j] = accabs;
        }
        seg_start += seg_bytes;
        bucket0 += n_buckets;
    }
    return ORACLE_OK;
}

int oracle_dequant_reduce_add(const void *local, int32_t local_dt, const uint8_t *const *packed,
                              const float *const *meta, int32_t W, int64_t n, int32_t L, const int64_t *off,
                              const uint8_t *bits, int32_t bucket, int32_t dt, float *sum32, double *sum64,
                              double *abs64)
{
    return reduce_impl(local, local_dt, packed, meta, W, n, L, off, bits, bucket, NULL, dt, sum32, sum64, abs64);
}

int oracle_layered_dequant_reduce(const uint8_t *const *packed, const float *const *meta, int32_t W,
                                  int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                                  const int32_t *layer_buckets, int32_t dt, float *sum32, double *sum64,
                                  double *abs64)
{
    if (L > 0 && !layer_buckets) return ORACLE_ERR_ARG;
    return reduce_impl(NULL, DT_F32, packed, meta, W, n, L, off, bits, 32, layer_buckets, dt, sum32, sum64, abs64);
}

int oracle_layered_dequant_reduce_add(const void *local, int32_t local_dt, const uint8_t *const *packed,
                                      const float *const *meta, int32_t W, int64_t n, int32_t L,
                                      const int64_t *off, const uint8_t *bits, const int32_t *layer_buckets,
                                      int32_t dt, float *sum32, double *sum64, double *abs64)
{
    if (L > 0 && !layer_buckets) return ORACLE_ERR_ARG;
    return reduce_impl(local, local_dt, packed, meta, W, n, L, off, bits, 32, layer_buckets, dt, sum32, sum64,
                       abs64);
}

int oracle_dequant_reduce(const uint8_t *const *packed, const float *const *meta, int32_t W,
                          int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                          int32_t bucket, int32_t dt, float *sum32, double *sum64, double *abs64)
{
    return oracle_dequant_reduce_add(NULL, DT_F32, packed, meta, W, n, L, off, bits, bucket, dt, sum32, sum64,
                                     abs64);
}

/* Codes of a quantized buffer, one byte per element (pass-through layers give 0xff). */
int oracle_unpack_codes(const uint8_t *packed, int64_t n, int32_t L, const int64_t *off,
                        const uint8_t *bits, int32_t bucket, int32_t dt, uint8_t *codes)
{
    int rc = check_plan(n, L, off, bits, bucket, dt);
    if (rc) return rc;
    uint64_t seg_start = 0;
    for (int32_t l = 0; l < L; l++) {
        int64_t first = off[l], len = off[l + 1] - off[l];
        int b = bits[l];
        uint64_t seg_bytes, n_buckets;
        layer_extent(len, b, bucket, dt, &seg_bytes, &n_buckets);
        for (int64_t j = 0; j < len; j++)
            codes[first + j] = b ? (uint8_t)get_bits(packed + seg_start, (uint64_t)j * b, b) : 0xff;
        seg_start += seg_bytes;
    }
    return ORACLE_OK;
}

/* ======================================================================== *
 * The norm-and-sign form of the quantizer, as the paper prints it
 * (Sec. 2.3: Q_s(v_i) = ||v|| * sign(v_i) * q(|v_i| / ||v||, s)), per bucket.
 *
 * Readings: the norm is the maximum absolute value of the bucket (so that
 * |v_i| / ||v|| covers [0, 1] and no summation order enters the result);
 * s = 2^(b-1) - 1 intervals, b >= 2; meta is ONE float per bucket,
 * unit = ||v|| / s; the level is drawn exactly as in the min/max form:
 * inv16 = (s * 65536) / ||v||, T = trunc(|v_i| * inv16),
 * level = min(floor((T + u) / 65536), s).  The paper gives no bit format for
 * sign(v_i) * level: the b-bit code is that product, the signed level in
 * -s..s, in two's complement (so sign(0) * 0 = 0 has one code, and a negative
 * v_i whose level is 0 decodes to +0).  The value of a code is
 * (float)signed_level * unit, one binary32 multiplication.  Layout, draws,
 * pass-through layers and the order of the sum are those of the min/max form.
 * ======================================================================== */

static int check_qsgd_bits(int32_t L, const uint8_t *bits)
{
    for (int32_t l = 0; l < L; l++)
        if (bits[l] == 1) return ORACLE_ERR_ARG;     /* a sign bit alone carries no level */
    return ORACLE_OK;
}

int oracle_qsgd_sizes(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                      int32_t bucket, int32_t dt, uint64_t *packed_bytes, uint64_t *meta_bytes)
{
    uint64_t mb = 0;
    int rc = oracle_sizes(n, L, off, bits, bucket, dt, packed_bytes, &mb);
    if (rc) return rc;
    if (check_qsgd_bits(L, bits)) return ORACLE_ERR_ARG;
    if (meta_bytes) *meta_bytes = mb / 2;            /* one float per bucket instead of two */
    return ORACLE_OK;
}

int oracle_qsgd_layered_sizes(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                              const int32_t *layer_buckets, int32_t dt, uint64_t *packed_bytes,
                              uint64_t *meta_bytes)
{
    uint64_t mb = 0;
    int rc = oracle_layered_sizes(n, L, off, bits, layer_buckets, dt, packed_bytes, &mb);
    if (rc) return rc;
    if (check_qsgd_bits(L, bits)) return ORACLE_ERR_ARG;
    if (meta_bytes) *meta_bytes = mb / 2;
    return ORACLE_OK;
}

static int qsgd_quantize_impl(const void *grad, int64_t n, int32_t L, const int64_t *off,
                              const uint8_t *bits, int32_t uniform_bucket, const int32_t *layer_buckets,
                              uint64_t seed, int32_t dt, const uint16_t *draws, uint64_t index_base,
                              uint8_t *packed, float *meta)
{
    int rc = check_plan(n, L, off, bits, layer_buckets ? 32 : uniform_bucket, dt);
    if (rc) return rc;
    rc = check_layer_buckets(L, layer_buckets);
    if (rc) return rc;
    if (check_qsgd_bits(L, bits)) return ORACLE_ERR_ARG;
    uint64_t seg_start = 0, bucket0 = 0;
    for (int32_t l = 0; l < L; l++) {
        int64_t first = off[l], len = off[l + 1] - off[l];
        int b = bits[l];
        const int32_t bucket = bucket_of(l, uniform_bucket, layer_buckets);
        uint64_t seg_bytes, n_buckets;
        layer_extent(len, b, bucket, dt, &seg_bytes, &n_buckets);
        if (len == 0) continue;
        uint8_t *seg = packed + seg_start;
        memset(seg, 0, seg_bytes);
        if (b == 0) {
            memcpy(seg, (const uint8_t *)grad + (uint64_t)first * elem_size(dt), (uint64_t)len * elem_size(dt));
        } else {
            const uint32_t s = (1u << (b - 1)) - 1u;         /* intervals of the level grid */
#pragma omp parallel for schedule(static)
            for (int64_t k = 0; k < (int64_t)n_buckets; k++) {
                int64_t j0 = k * bucket;
                int64_t count = len - j0 < bucket ? len - j0 : bucket;
                float norm = 0.0f;
                for (int64_t j = j0; j < j0 + count; j++) {
                    float a = fabsf(load_elem(grad, first + j, dt));
                    if (a > norm) norm = a;
                }
                float unit = norm / (float)s;
                float inv16 = (float)(s * 65536u) / norm;
                if (!(unit > 0.0f) || !isfinite(unit) || !isfinite(inv16)) {
                    unit = 0.0f;
                    inv16 = 0.0f;
                }
                meta[bucket0 + k] = unit;
                for (int64_t j = j0; j < j0 + count; j++) {
                    uint64_t i = (uint64_t)(first + j);
                    uint32_t u16 = draws ? draws[i] : oracle_u16(seed, index_base + i);
                    float x = load_elem(grad, first + j, dt);
                    float S = fabsf(x) * inv16;
                    uint64_t T;
                    if (!(S >= 0.0f)) T = 0;
                    else if (S >= 4294967296.0f) T = 0xffffffffu;
                    else T = (uint64_t)S;
                    uint64_t level = (T + u16) >> 16;
                    if (level > s) level = s;
                    int32_t signed_level = signbit(x) ? -(int32_t)level : (int32_t)level;
                    uint32_t code = (uint32_t)signed_level & ((1u << b) - 1u);
                    put_bits(seg, (uint64_t)j * b, code, b);
                }
            }
        }
        seg_start += seg_bytes;
        bucket0 += n_buckets;
    }
    return ORACLE_OK;
}

int oracle_qsgd_quantize(const void *grad, int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                         int32_t bucket, uint64_t seed, int32_t dt, uint8_t *packed, float *meta)
{
    return qsgd_quantize_impl(grad, n, L, off, bits, bucket, NULL, seed, dt, NULL, 0, packed, meta);
}

/* A window of a larger buffer (see oracle_quantize_window), and a bucket size per layer. */
int oracle_qsgd_quantize_window(const void *grad, int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                                int32_t bucket, uint64_t seed, int32_t dt, uint64_t index_base, uint8_t *packed,
                                float *meta)
{
    return qsgd_quantize_impl(grad, n, L, off, bits, bucket, NULL, seed, dt, NULL, index_base, packed, meta);
}

int oracle_qsgd_layered_quantize(const void *grad, int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                                 const int32_t *layer_buckets, uint64_t seed, int32_t dt, uint8_t *packed,
                                 float *meta)
{
    if (L > 0 && !layer_buckets) return ORACLE_ERR_ARG;
    return qsgd_quantize_impl(grad, n, L, off, bits, 32, layer_buckets, seed, dt, NULL, 0, packed, meta);
}

int oracle_qsgd_quantize_with_draws(const void *grad, int64_t n, int32_t L, const int64_t *off,
                                    const uint8_t *bits, int32_t bucket, int32_t dt, const uint16_t *draws,
                                    uint8_t *packed, float *meta)
{
    if (!draws) return ORACLE_ERR_ARG;
    return qsgd_quantize_impl(grad, n, L, off, bits, bucket, NULL, 0, dt, draws, 0, packed, meta);
}

/* Sum over the W peers of the decoded values; outputs as in oracle_dequant_reduce. */
static int qsgd_reduce_impl(const uint8_t *const *packed, const float *const *meta, int32_t W, int64_t n,
                            int32_t L, const int64_t *off, const uint8_t *bits, int32_t uniform_bucket,
                            const int32_t *layer_buckets, int32_t dt, float *sum32, double *sum64, double *abs64)
{
    int rc = check_plan(n, L, off, bits, layer_buckets ? 32 : uniform_bucket, dt);
    if (rc) return rc;
    rc = check_layer_buckets(L, layer_buckets);
    if (rc) return rc;
    if (check_qsgd_bits(L, bits) || W < 1 || !packed || !meta) return ORACLE_ERR_ARG;
    uint64_t seg_start = 0, bucket0 = 0;
    for (int32_t l = 0; l < L; l++) {
        int64_t first = off[l], len = off[l + 1] - off[l];
        int b = bits[l];
        const int32_t bucket = bucket_of(l, uniform_bucket, layer_buckets);
        uint64_t seg_bytes, n_buckets;
        layer_extent(len, b, bucket, dt, &seg_bytes, &n_buckets);
        if (len == 0) continue;
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < len; j++) {
            float acc32 = 0.0f;
            double acc64 = 0.0, accabs = 0.0;
            for (int32_t w = 0; w < W; w++) {
                const uint8_t *seg = packed[w] + seg_start;
                float v32;
                double v64;
                if (b == 0) {
                    v32 = load_elem(seg, j, dt);
                    v64 = (double)v32;
                } else {
                    float unit = meta[w][bucket0 + (uint64_t)(j / bucket)];
                    uint32_t code = get_bits(seg, (uint64_t)j * b, b);
                    /* two's complement of width b: the top bit weighs -2^(b-1) */
                    int32_t level = (int32_t)code - (int32_t)((code >> (b - 1)) << b);
                    v32 = (float)level * unit;
                    v64 = (double)level * (double)unit;
                }
                acc32 = (w == 0) ? v32 : acc32 + v32;
                acc64 += v64;
                accabs += fabs(v64);
            }
            if (sum32) sum32[first + j] = acc32;
            if (sum64) sum64[first + j] = acc64;
            if (abs64) abs64[first + j] = accabs;
        }
        seg_start += seg_bytes;
        bucket0 += n_buckets;
    }
    return ORACLE_OK;
}

int oracle_qsgd_dequant_reduce(const uint8_t *const *packed, const float *const *meta, int32_t W, int64_t n,
                               int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int32_t dt,
                               float *sum32, double *sum64, double *abs64)
{
    return qsgd_reduce_impl(packed, meta, W, n, L, off, bits, bucket, NULL, dt, sum32, sum64, abs64);
}

int oracle_qsgd_layered_dequant_reduce(const uint8_t *const *packed, const float *const *meta, int32_t W,
                                       int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                                       const int32_t *layer_buckets, int32_t dt, float *sum32, double *sum64,
                                       double *abs64)
{
    if (L > 0 && !layer_buckets) return ORACLE_ERR_ARG;
    return qsgd_reduce_impl(packed, meta, W, n, L, off, bits, 32, layer_buckets, dt, sum32, sum64, abs64);
}

/* ======================================================================== *
 * Per-layer statistics for the layer-wise adaptive scheme (Sec. "Layer-wise
 * Adaptive Quantization"): the squared l2 norm of every layer of a fused
 * buffer (the second coordinate of Algorithm 1's points is its square root)
 * and the squared l2 norm of the compression error of every layer (the
 * quantity the problem definition bounds by alpha * E_4).  Sums are carried in
 * long double and rounded to binary64 once, so the oracle's own rounding is
 * far below the tolerance the GPU sums are checked with.
 * ======================================================================== */

int oracle_layer_sqnorms(const void *buf, int64_t n, int32_t L, const int64_t *off, int32_t dt, double *out)
{
    if (n < 0 || L < 0 || (L > 0 && (!off || !out)) || (dt != DT_F32 && dt != DT_F16)) return ORACLE_ERR_ARG;
    if (L == 0) return n == 0 ? ORACLE_OK : ORACLE_ERR_ARG;
    if (off[0] != 0 || off[L] != n) return ORACLE_ERR_ARG;
    for (int32_t l = 0; l < L; l++) {
        if (off[l + 1] < off[l]) return ORACLE_ERR_ARG;
        long double acc = 0.0L;
        for (int64_t i = off[l]; i < off[l + 1]; i++) {
            long double x = (long double)load_elem(buf, i, dt);
            acc += x * x;
        }
        out[l] = (double)acc;
    }
    return ORACLE_OK;
}

/* out[l] = sum over the layer of (x_i - value of its code)^2, the value being the binary32 one
 * the dequantizer returns; 0 for pass-through layers.  scheme 0: min/max form (meta {unit, mn}),
 * scheme 1: norm-and-sign form (meta unit). */
static int sqerrors_impl(int32_t scheme, const void *grad, const uint8_t *packed, const float *meta, int64_t n,
                         int32_t L, const int64_t *off, const uint8_t *bits, int32_t uniform_bucket,
                         const int32_t *layer_buckets, int32_t dt, double *out)
{
    int rc = check_plan(n, L, off, bits, layer_buckets ? 32 : uniform_bucket, dt);
    if (rc) return rc;
    rc = check_layer_buckets(L, layer_buckets);
    if (rc) return rc;
    if ((scheme != 0 && scheme != 1) || (scheme == 1 && check_qsgd_bits(L, bits))) return ORACLE_ERR_ARG;
    if (L > 0 && !out) return ORACLE_ERR_ARG;
    uint64_t seg_start = 0, bucket0 = 0;
    for (int32_t l = 0; l < L; l++) {
        int64_t first = off[l], len = off[l + 1] - off[l];
        int b = bits[l];
        const int32_t bucket = bucket_of(l, uniform_bucket, layer_buckets);
        uint64_t seg_bytes, n_buckets;
        layer_extent(len, b, bucket, dt, &seg_bytes, &n_buckets);
        long double acc = 0.0L;
        if (b != 0) {
            const uint8_t *seg = packed + seg_start;
            for (int64_t j = 0; j < len; j++) {
                uint64_t g = bucket0 + (uint64_t)(j / bucket);
                uint32_t code = get_bits(seg, (uint64_t)j * b, b);
                float v;
                if (scheme == 1) {
                    int32_t level = (int32_t)code - (int32_t)((code >> (b - 1)) << b);
                    v = (float)level * meta[g];
                } else {
                    v = fmaf((float)code, meta[2 * g], meta[2 * g + 1]);
                }
                long double d = (long double)load_elem(grad, first + j, dt) - (long double)v;
                acc += d * d;
            }
        }
        out[l] = (double)acc;
        seg_start += seg_bytes;
        bucket0 += n_buckets;
    }
    return ORACLE_OK;
}

int oracle_layer_sqerrors(int32_t scheme, const void *grad, const uint8_t *packed, const float *meta, int64_t n,
                          int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int32_t dt,
                          double *out)
{
    return sqerrors_impl(scheme, grad, packed, meta, n, L, off, bits, bucket, NULL, dt, out);
}

/* The same for a chunk written with a bucket size per layer (min/max form). */
int oracle_layered_layer_sqerrors(const void *grad, const uint8_t *packed, const float *meta, int64_t n, int32_t L,
                                  const int64_t *off, const uint8_t *bits, const int32_t *layer_buckets,
                                  int32_t dt, double *out)
{
    if (L > 0 && !layer_buckets) return ORACLE_ERR_ARG;
    return sqerrors_impl(0, grad, packed, meta, n, L, off, bits, 32, layer_buckets, dt, out);
}
