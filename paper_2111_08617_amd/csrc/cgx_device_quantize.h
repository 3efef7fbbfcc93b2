// Device code of the quantizer: encoding of chunks, rows, wide buckets, short ends and
// generic tiles, and the pass-through copy (shared by the quantize and the fused kernels).
#pragma once

#include "cgx_device.h"

namespace cgx {
namespace {

// ---------------------------------------------------------------- quantize

// The 8 codes of one group, packed: element j of the group has buffer index
// 2 * pair0 + odd + j, key = generator key of the tile.  odd (0 or 1, uniform over a tile: groups
// start 8 elements apart) tells whether the group starts on the upper half of a generator word;
// then its 8 draws are the 16-bit halves 1..8 of words pair0 .. pair0 + 4 instead of halves
// 0..7 of words pair0 .. pair0 + 3.  ODD = false: the plan has no such tile (odd == 0 always),
// and neither the fifth word nor the selection is paid; the host picks the instantiation.
template <int SCHEME, int BITS, bool ODD>
__device__ __forceinline__ uint64_t encode_group(const float (&x)[8], const Scale &s, uint32_t pair0, uint32_t key,
                                                 uint32_t odd)
{
    constexpr uint32_t kLevels = top_level<SCHEME>(BITS);
    uint32_t word[5];
#pragma unroll
    for (int k = 0; k < 4 + int(ODD); k++) word[k] = mix32((pair0 + k) ^ key);
    uint64_t acc = 0;
#pragma unroll
    for (int k = 0; k < 4; k++) {
        // the pair's two draws
        const uint32_t w = ODD ? __builtin_amdgcn_alignbit(word[k + 1], word[k], 16u * odd) : word[k];
        const uint64_t q0 = code_of<SCHEME>(x[2 * k], s, w & 0xffffU, kLevels, BITS);
        const uint64_t q1 = code_of<SCHEME>(x[2 * k + 1], s, w >> 16, kLevels, BITS);
        acc |= q0 << (2 * k * BITS);
        acc |= q1 << ((2 * k + 1) * BITS);
    }
    return acc;
}

// Minimum and maximum (kNormSign: +0 and the largest magnitude) of a lane's chunk, folded into mn / mx.
template <int SCHEME>
__device__ __forceinline__ void lane_extent(const float (&x)[G][8], float &mn, float &mx)
{
#pragma unroll
    for (int r = 0; r < G; r++)
#pragma unroll
        for (int j = 0; j < 8; j++) {
            if (SCHEME == kNormSign) {
                mx = __builtin_fmaxf(mx, __builtin_fabsf(x[r][j]));
            } else {
                mn = __builtin_fminf(mn, x[r][j]);
                mx = __builtin_fmaxf(mx, x[r][j]);
            }
        }
}

// Codes of a chunk whose elements all take the scale s: staged, then sent out.
template <int SCHEME, int BITS, bool ODD>
__device__ __forceinline__ void encode_chunk(const float (&x)[G][8], const Scale &s, const LaneMap &map,
                                             int64_t first, uint32_t key, uint8_t *__restrict__ out,
                                             uint4v *stage, int lane)
{
#pragma unroll
    for (int r = 0; r < G; r++) {
        const uint32_t pair0 = uint32_t(uint64_t(first + map.group(r)) >> 1);
        stage_codes<BITS>(reinterpret_cast<uint8_t *>(stage) + (map.group(r) >> 3) * BITS,
                          encode_group<SCHEME, BITS, ODD>(x[r], s, pair0, key, uint32_t(first) & 1u));
    }
    // the chunk's codes leave as whole 16-byte vectors, consecutive across lanes
    wave_lds_fence();
    flush_stage(stage, reinterpret_cast<uint4v *>(out), kChunk * BITS / 128, lane);
    wave_lds_fence();
}

// One chunk held in registers (x) -> meta of its buckets and its packed codes.
// first = buffer index of the chunk's first element; key = generator key of the tile.
// meta_chunk points at the meta of the chunk's first bucket.
template <int SCHEME, int BITS, bool ODD>
__device__ __forceinline__ void quantize_chunk(const float (&x)[G][8], const LaneMap &map, int lane, int64_t first,
                                               uint32_t key, float *__restrict__ meta_chunk,
                                               uint8_t *__restrict__ out, uint4v *stage)
{
    constexpr uint32_t kLevels = top_level<SCHEME>(BITS);
    float mn = SCHEME == kNormSign ? 0.0f : x[0][0], mx = mn;
    lane_extent<SCHEME>(x, mn, mx);
    if (SCHEME == kNormSign)
        group_max(mx, map.lg, lane);
    else
        group_minmax(mn, mx, map.lg, lane);
    const Scale s = bucket_scale(mn, mx, int(kLevels));
    if (map.lp == 0) store_meta<SCHEME>(meta_chunk, map.bi, s);
    encode_chunk<SCHEME, BITS, ODD>(x, s, map, first, key, out, stage, lane);
}

// The same for buckets of 32 or 64 elements, with the chunk held row by row: group r of lane l
// is elements [512 r + 8 l, 512 r + 8 l + 8) of the chunk, so every load instruction of the
// caller covers 64 consecutive groups (with the bucket-major mapping a lane's four groups would
// be one or two whole buckets and each load instruction would touch 32 or 64 separate lines,
// 16 to 64 bytes of each: measured 21 % of the HBM peak at 32-element buckets).  A bucket is
// bucket / 8 neighbouring lanes of one row; a lane serves four buckets and pays the two
// divisions four times.
template <int SCHEME, int BITS, bool ODD>
__device__ __forceinline__ void quantize_chunk_rows(const float (&x)[G][8], int bucket, int lane, int64_t first,
                                                    uint32_t key, float *__restrict__ meta_chunk,
                                                    uint8_t *__restrict__ out, uint4v *stage)
{
    constexpr uint32_t kLevels = top_level<SCHEME>(BITS);
    constexpr int kRow = kWave * 8;                  // elements per row
    const int lg = bucket == 32 ? 2 : 3;             // log2(lanes per bucket)
    const int buckets_per_row = kRow / bucket;
#pragma unroll
    for (int r = 0; r < G; r++) {
        float mn, mx;
        if (SCHEME == kNormSign) {
            mn = 0.0f;
            mx = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; j++) mx = __builtin_fmaxf(mx, __builtin_fabsf(x[r][j]));
            group_max(mx, lg, lane);
        } else {
            mn = x[r][0];
            mx = x[r][0];
#pragma unroll
            for (int j = 1; j < 8; j++) {
                mn = __builtin_fminf(mn, x[r][j]);
                mx = __builtin_fmaxf(mx, x[r][j]);
            }
            group_minmax(mn, mx, lg, lane);
        }
        const Scale s = bucket_scale(mn, mx, int(kLevels));
        if ((lane & ((1 << lg) - 1)) == 0) store_meta<SCHEME>(meta_chunk, r * buckets_per_row + (lane >> lg), s);
        const int e = r * kRow + lane * 8;           // the group's first element within the chunk
        const uint32_t pair0 = uint32_t(uint64_t(first + e) >> 1);
        stage_codes<BITS>(reinterpret_cast<uint8_t *>(stage) + (e >> 3) * BITS,
                          encode_group<SCHEME, BITS, ODD>(x[r], s, pair0, key, uint32_t(first) & 1u));
    }
    wave_lds_fence();
    flush_stage(stage, reinterpret_cast<uint4v *>(out), kChunk * BITS / 128, lane);
    wave_lds_fence();
}

// A chunk that starts on a 16-byte boundary, fetched through the wave's LDS area: every load
// instruction moves 1 KB of consecutive bytes straight into LDS (no registers held while in
// flight), and each lane then reads its groups from there.  Read into registers directly, a
// lane's 32 consecutive bytes come from two instructions that each cover every other 16 bytes
// of 2 KB; a kernel that only moves bytes loses 5 to 9 % of its rate with that pattern.
// The area must hold the chunk as stored (kChunk elements of DT).
template <int DT>
__device__ __forceinline__ void chunk_through_lds(const void *__restrict__ grad, int64_t first, const LaneMap &map,
                                                  float (&x)[G][8], uint4v *stage, int lane)
{
    constexpr int S = DT == CGX_F16 ? 2 : 4;
    constexpr int kVecs = kChunk * S / 16;
    static_assert(kVecs % kWave == 0, "whole load instructions");
    const uint4v *src = reinterpret_cast<const uint4v *>(reinterpret_cast<const uint8_t *>(grad) + first * S);
#pragma unroll
    for (int k = 0; k < kVecs / kWave; k++) load_to_lds16(src + k * kWave + lane, stage + k * kWave);
    wait_vector_memory();
    wave_lds_fence();
#pragma unroll
    for (int r = 0; r < G; r++) {
        if (DT == CGX_F16) {
            const half8v h = *reinterpret_cast<const half8v *>(reinterpret_cast<const _Float16 *>(stage) + map.group(r));
#pragma unroll
            for (int j = 0; j < 8; j++) x[r][j] = float(h[j]);
        } else {
            const float4v *p = reinterpret_cast<const float4v *>(reinterpret_cast<const float *>(stage) + map.group(r));
            const float4v a = p[0], b = p[1];
#pragma unroll
            for (int j = 0; j < 4; j++) {
                x[r][j] = a[j];
                x[r][4 + j] = b[j];
            }
        }
    }
    wave_lds_fence();      // the codes are staged in the same area
}

// VIA_LDS: every vectorised tile of the plan starts on a 16-byte boundary of the buffer (a property
// of the tile table; the host picks the instantiation).
template <int SCHEME, int DT, int BITS, bool ODD, bool VIA_LDS = false>
__device__ __forceinline__ void quantize_fast(const void *__restrict__ grad, uint8_t *__restrict__ packed,
                                              float *__restrict__ meta, const Tile &tile, int bucket,
                                              uint32_t seed_lo, uint32_t seed_hi, int lane, uint4v *stage)
{
    const LaneMap map(tile, bucket, lane);
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    const int chunks = int(tile.count / kChunk);
    const int buckets_per_chunk = kChunk / bucket;
    for (int c = 0; c < chunks; c++) {
        const int64_t first = tile.elem0 + int64_t(c) * kChunk;
        float x[G][8];
        if constexpr (VIA_LDS) {
            chunk_through_lds<DT>(grad, first, map, x, stage, lane);
        } else {
#pragma unroll
            for (int r = 0; r < G; r++) load8<DT>(grad, first + map.group(r), x[r]);
        }
        quantize_chunk<SCHEME, BITS, ODD>(x, map, lane, first, key,
                                     meta + kMetaFloats<SCHEME> * (tile.bucket0 + c * buckets_per_chunk),
                                     packed + tile.packed_off + int64_t(c) * (kChunk * BITS / 8), stage);
    }
}

// quantize_fast for buckets of 32 or 64 elements (row-by-row mapping).
template <int SCHEME, int DT, int BITS, bool ODD>
__device__ __forceinline__ void quantize_fast_rows(const void *__restrict__ grad, uint8_t *__restrict__ packed,
                                                   float *__restrict__ meta, const Tile &tile, int bucket,
                                                   uint32_t seed_lo, uint32_t seed_hi, int lane, uint4v *stage)
{
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    const int chunks = int(tile.count / kChunk);
    const int buckets_per_chunk = kChunk / bucket;
    for (int c = 0; c < chunks; c++) {
        const int64_t first = tile.elem0 + int64_t(c) * kChunk;
        float x[G][8];
#pragma unroll
        for (int r = 0; r < G; r++) load8<DT>(grad, first + r * (kWave * 8) + lane * 8, x[r]);
        quantize_chunk_rows<SCHEME, BITS, ODD>(x, bucket, lane, first, key,
                                          meta + kMetaFloats<SCHEME> * (tile.bucket0 + c * buckets_per_chunk),
                                          packed + tile.packed_off + int64_t(c) * (kChunk * BITS / 8), stage);
    }
}

// A tile that is one whole bucket of 2 or 4 chunks: a first pass over the chunks finds the
// scale, a second one reads them again (from the caches: 16 or 32 KB read a moment ago) and
// cuts the codes.  Row-by-row mapping (LaneMap with the whole wave as one bucket).
template <int SCHEME, int DT, int BITS, bool ODD>
__device__ __forceinline__ void quantize_wide(const void *__restrict__ grad, uint8_t *__restrict__ packed,
                                              float *__restrict__ meta, const Tile &tile, int bucket,
                                              uint32_t seed_lo, uint32_t seed_hi, int lane, uint4v *stage)
{
    constexpr uint32_t kLevels = top_level<SCHEME>(BITS);
    const LaneMap map(tile, bucket, lane);
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    const int chunks = int(tile.count / kChunk);
    float mn = SCHEME == kNormSign ? 0.0f : __builtin_inff(), mx = SCHEME == kNormSign ? 0.0f : -__builtin_inff();
    for (int c = 0; c < chunks; c++) {
        float x[G][8];
#pragma unroll
        for (int r = 0; r < G; r++) {
            Raw8<DT> raw;
            raw.load_keep(grad, tile.elem0 + int64_t(c) * kChunk + map.group(r));   // read again below
            raw.widen(x[r]);
        }
        lane_extent<SCHEME>(x, mn, mx);
    }
    if (SCHEME == kNormSign)
        group_max(mx, 6, lane);
    else
        group_minmax(mn, mx, 6, lane);
    const Scale s = bucket_scale(mn, mx, int(kLevels));
    if (lane == 0) store_meta<SCHEME>(meta, tile.bucket0, s);
    for (int c = 0; c < chunks; c++) {
        const int64_t first = tile.elem0 + int64_t(c) * kChunk;
        float x[G][8];
#pragma unroll
        for (int r = 0; r < G; r++) load8<DT>(grad, first + map.group(r), x[r]);
        encode_chunk<SCHEME, BITS, ODD>(x, s, map, first, key, packed + tile.packed_off + int64_t(c) * (kChunk * BITS / 8),
                                   stage, lane);
    }
}

// x holds the tile's elements in the chunk mapping, 0 where there is none -> meta and codes.
template <int SCHEME, int BITS, bool ODD>
__device__ __forceinline__ void quantize_tail_regs(const float (&x)[G][8], const TailShape &shape, const LaneMap &map,
                                                   int lane, int64_t first, uint32_t key, float *__restrict__ meta,
                                                   uint8_t *__restrict__ out, uint4v *stage)
{
    constexpr uint32_t kLevels = top_level<SCHEME>(BITS);
    // kNormSign: the zeros of the missing elements are neutral for the largest magnitude
    float mn = SCHEME == kNormSign ? 0.0f : __builtin_inff(), mx = SCHEME == kNormSign ? 0.0f : -__builtin_inff();
#pragma unroll
    for (int r = 0; r < G; r++) {
        const int v = shape.valid(map.group(r));
#pragma unroll
        for (int j = 0; j < 8; j++) {
            if (SCHEME == kNormSign) {
                mx = __builtin_fmaxf(mx, __builtin_fabsf(x[r][j]));
            } else {
                mn = __builtin_fminf(mn, j < v ? x[r][j] : __builtin_inff());
                mx = __builtin_fmaxf(mx, j < v ? x[r][j] : -__builtin_inff());
            }
        }
    }
    if (SCHEME == kNormSign)
        group_max(mx, map.lg, lane);
    else
        group_minmax(mn, mx, map.lg, lane);
    const Scale s = bucket_scale(mn, mx, int(kLevels));
    if (map.lp == 0 && map.bi < shape.buckets) store_meta<SCHEME>(meta, map.bi, s);
#pragma unroll
    for (int r = 0; r < G; r++) {
        const int v = shape.valid(map.group(r));
        const uint32_t pair0 = uint32_t(uint64_t(first + map.group(r)) >> 1);
        uint64_t codes = encode_group<SCHEME, BITS, ODD>(x[r], s, pair0, key, uint32_t(first) & 1u);
        codes &= v == 8 ? ~uint64_t(0) : (uint64_t(1) << (v * BITS)) - 1u;       // nothing past the layer's end
        stage_codes<BITS>(reinterpret_cast<uint8_t *>(stage) + (map.group(r) >> 3) * BITS, codes);
    }
    // every group of the chunk has been staged (zeros past the end), so whole vectors can leave:
    // they carry the zero padding of the layer's segment with them
    wave_lds_fence();
    flush_stage(stage, reinterpret_cast<uint4v *>(out), shape.nvecs, lane);
    wave_lds_fence();
}

template <int SCHEME, int DT, int BITS, bool ODD>
__device__ __forceinline__ void quantize_tail(const void *__restrict__ grad, uint8_t *__restrict__ packed,
                                              float *__restrict__ meta, const Tile &tile, int bucket,
                                              uint32_t seed_lo, uint32_t seed_hi, int lane, uint4v *stage)
{
    const LaneMap map(tile, bucket, lane);
    const TailShape shape = TailShape::of<BITS>(tile, bucket);
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    float x[G][8];
#pragma unroll
    for (int r = 0; r < G; r++) {
        const int e = map.group(r), v = shape.valid(e);
        if (v == 8) {
            load8<DT>(grad, tile.elem0 + e, x[r]);
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++) x[r][j] = j < v ? load_elem<DT>(grad, tile.elem0 + e + j) : 0.0f;
        }
    }
    quantize_tail_regs<SCHEME, BITS, ODD>(x, shape, map, lane, tile.elem0, key,
                                          meta + kMetaFloats<SCHEME> * tile.bucket0, packed + tile.packed_off, stage);
}

// LDS a wave needs for a tile of kind kQuantAny: its codes, a minimum and a maximum per group, a scale per bucket.
constexpr int kAnyStageBytes = kChunk + 2 * (kChunk / 8) * 4 + kWave * 8;

// x holds the tile row by row (zeros where there is no group) -> meta of its buckets and its packed codes.
// The scale of a bucket comes from a per-group minimum / maximum parked in LDS: the lanes are split into
// groups of P (a power of two, 64 / P >= buckets), each of which folds the entries of one bucket.
template <int SCHEME, int BITS, bool ODD>
__device__ __forceinline__ void quantize_any_regs(const float (&x)[G][8], const AnyShape &shape, const Tile &tile,
                                                  uint32_t key, float *__restrict__ meta, uint8_t *__restrict__ out,
                                                  uint4v *stage, int lane)
{
    constexpr uint32_t kLevels = top_level<SCHEME>(BITS);
    uint8_t *codes = reinterpret_cast<uint8_t *>(stage);
    float *gmn = reinterpret_cast<float *>(codes + kChunk), *gmx = gmn + kChunk / 8;
    float2 *scales = reinterpret_cast<float2 *>(gmx + kChunk / 8);
#pragma unroll
    for (int r = 0; r < G; r++) {
        const int Gi = r * kWave + lane;
        float mn = SCHEME == kNormSign ? 0.0f : x[r][0], mx = SCHEME == kNormSign ? 0.0f : x[r][0];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            if (SCHEME == kNormSign) {
                mx = __builtin_fmaxf(mx, __builtin_fabsf(x[r][j]));
            } else {
                mn = __builtin_fminf(mn, x[r][j]);
                mx = __builtin_fmaxf(mx, x[r][j]);
            }
        }
        if (Gi < shape.groups) {
            gmn[Gi] = mn;
            gmx[Gi] = mx;
        }
    }
    wave_lds_fence();
    const int lgP = 31 - __builtin_clz(uint32_t(kWave / shape.m));      // floor(log2(64 / buckets))
    const int bucket_of_lane = lane >> lgP, part = lane & ((1 << lgP) - 1);
    float mn = SCHEME == kNormSign ? 0.0f : __builtin_inff(), mx = SCHEME == kNormSign ? 0.0f : -__builtin_inff();
    if (bucket_of_lane < shape.m) {
        for (int g = part; g < shape.gb; g += 1 << lgP) {
            if (SCHEME != kNormSign) mn = __builtin_fminf(mn, gmn[bucket_of_lane * shape.gb + g]);
            mx = __builtin_fmaxf(mx, gmx[bucket_of_lane * shape.gb + g]);
        }
    }
    if (SCHEME == kNormSign)
        group_max(mx, lgP, lane);
    else
        group_minmax(mn, mx, lgP, lane);
    if (bucket_of_lane < shape.m && part == 0) {
        const Scale s = bucket_scale(mn, mx, int(kLevels));
        store_meta<SCHEME>(meta, uint32_t(bucket_of_lane), s);
        scales[bucket_of_lane] = make_float2(s.mn, s.inv16);
    }
    wave_lds_fence();
#pragma unroll
    for (int r = 0; r < G; r++) {
        const int Gi = r * kWave + lane;
        if (Gi < shape.groups) {
            const float2 sc = scales[shape.bucket_of(Gi)];
            const Scale s{0.0f, sc.x, sc.y};
            const uint32_t pair0 = uint32_t(uint64_t(tile.elem0 + int64_t(Gi) * 8) >> 1);
            stage_codes<BITS>(codes + Gi * BITS, encode_group<SCHEME, BITS, ODD>(x[r], s, pair0, key, uint32_t(tile.elem0) & 1u));
        }
    }
    wave_lds_fence();
    // the tile's codes are groups * BITS bytes, a multiple of 4, at a multiple of 4 in the stream
    const int dwords = shape.groups * BITS / 4;
    uint32_t *dst = reinterpret_cast<uint32_t *>(out);
    for (int v = lane; v < dwords; v += kWave) stream_store(dst + v, reinterpret_cast<const uint32_t *>(codes)[v]);
    if (uint32_t(lane) < tile.pad) out[shape.groups * BITS + lane] = 0;        // the layer's zero padding
    wave_lds_fence();
}

template <int SCHEME, int DT, int BITS, bool ODD>
__device__ __forceinline__ void quantize_any(const void *__restrict__ grad, uint8_t *__restrict__ packed,
                                             float *__restrict__ meta, const Tile &tile, int bucket,
                                             uint32_t seed_lo, uint32_t seed_hi, int lane, uint4v *stage)
{
    const AnyShape shape(tile, bucket);
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    float x[G][8];
#pragma unroll
    for (int r = 0; r < G; r++) {
        const int Gi = r * kWave + lane;
        if (Gi < shape.groups) {
            load8<DT>(grad, tile.elem0 + int64_t(Gi) * 8, x[r]);
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++) x[r][j] = 0.0f;
        }
    }
    quantize_any_regs<SCHEME, BITS, ODD>(x, shape, tile, key, meta + kMetaFloats<SCHEME> * tile.bucket0,
                                         packed + tile.packed_off, stage, lane);
}

// Any bucket size, any alignment, ragged last bucket: one bucket at a time, two passes.
// value(j) gives element j of the tile (called twice per element).  With BATCH the values
// of a pass are fetched 8 at a time so that plain loads overlap; without it (value() is
// itself a reduction over the peers) they are taken one by one.
template <int SCHEME, bool BATCH, typename Value>
__device__ __forceinline__ void quantize_generic(Value value, uint8_t *__restrict__ out,
                                                 float *__restrict__ meta, const Tile &tile, uint32_t pad,
                                                 int bucket, uint32_t seed_lo, uint32_t seed_hi, int lane)
{
    const int b = int(tile_bits(tile));
    const uint32_t levels = top_level<SCHEME>(b);
    // kNormSign: the maximum runs over magnitudes and the minimum stays +0
    const auto seen = [](float x) { return SCHEME == kNormSign ? __builtin_fabsf(x) : x; };
    for (uint32_t k0 = 0; k0 < tile.count; k0 += uint32_t(bucket)) {
        const uint32_t cnt = tile.count - k0 < uint32_t(bucket) ? tile.count - k0 : uint32_t(bucket);
        float mn = SCHEME == kNormSign ? 0.0f : __builtin_inff(), mx = SCHEME == kNormSign ? 0.0f : -__builtin_inff();
        if (BATCH) {
            for (uint32_t j0 = 0; j0 < cnt; j0 += 8 * kWave) {
                float x[8];
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    const uint32_t j = j0 + u * kWave + lane;
                    x[u] = value(k0 + (j < cnt ? j : 0));           // clamped: the bucket's first element again
                }
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    if (SCHEME != kNormSign) mn = __builtin_fminf(mn, x[u]);
                    mx = __builtin_fmaxf(mx, seen(x[u]));
                }
            }
        } else {
            for (uint32_t j = lane; j < cnt; j += kWave) {
                const float x = value(k0 + j);
                if (SCHEME != kNormSign) mn = __builtin_fminf(mn, x);
                mx = __builtin_fmaxf(mx, seen(x));
            }
        }
        if (SCHEME == kNormSign)
            group_max(mx, 6, lane);
        else
            group_minmax(mn, mx, 6, lane);
        const Scale s = bucket_scale(mn, mx, int(levels));
        if (lane == 0) store_meta<SCHEME>(meta, tile.bucket0 + k0 / uint32_t(bucket), s);

        const uint32_t groups = (cnt + 7) / 8;
        for (uint32_t g = lane; g < groups; g += kWave) {
            const uint32_t valid = cnt - g * 8 < 8 ? cnt - g * 8 : 8;
            const uint64_t i0 = uint64_t(tile.elem0) + k0 + g * 8;
            uint64_t acc = 0;
            if (BATCH) {
                float x[8];
#pragma unroll
                for (uint32_t j = 0; j < 8; j++) x[j] = value(k0 + g * 8 + (j < valid ? j : 0));
#pragma unroll
                for (uint32_t j = 0; j < 8; j++) {
                    const uint64_t q = code_of<SCHEME>(x[j], s, draw16(seed_lo, seed_hi, i0 + j), levels, b);
                    if (j < valid) acc |= q << (j * b);
                }
            } else {
                for (uint32_t j = 0; j < valid; j++) {
                    const uint64_t q =
                        code_of<SCHEME>(value(k0 + g * 8 + j), s, draw16(seed_lo, seed_hi, i0 + j), levels, b);
                    acc |= q << (j * b);
                }
            }
            const uint32_t nbytes = (valid * b + 7) / 8;
            uint8_t *p = out + uint64_t(k0 / 8 + g) * b;
            for (uint32_t k = 0; k < nbytes; k++) p[k] = uint8_t(acc >> (8 * k));
        }
    }
    if (pad) {
        const uint64_t end = (uint64_t(tile.count) * b + 7) / 8;
        if (uint32_t(lane) < pad) out[end + lane] = 0;
    }
}

// Pass-through tile of the quantize kernel: verbatim copy, then the layer's zero padding.
template <int DT>
__device__ __forceinline__ void copy_tile(const void *__restrict__ grad, uint8_t *__restrict__ packed, const Tile &tile,
                          bool fast, int lane)
{
    constexpr int S = DT == CGX_F16 ? 2 : 4;
    const uint8_t *src = reinterpret_cast<const uint8_t *>(grad) + tile.elem0 * S;
    uint8_t *dst = packed + tile.packed_off;
    const uint32_t bytes = tile.count * S;
    uint32_t done = 0;
    if (fast) {
        const uint32_t vecs = bytes / 16;
        for (uint32_t v = lane; v < vecs; v += kWave)
            reinterpret_cast<uint4v *>(dst)[v] = reinterpret_cast<const uint4u2 *>(src)[v];
        done = vecs * 16;
    } else if (DT == CGX_F16) {
        for (uint32_t e = lane; e < tile.count; e += kWave)
            reinterpret_cast<uint16_t *>(dst)[e] = reinterpret_cast<const uint16_t *>(src)[e];
        done = bytes;
    } else {
        for (uint32_t e = lane; e < tile.count; e += kWave)
            reinterpret_cast<uint32_t *>(dst)[e] = reinterpret_cast<const uint32_t *>(src)[e];
        done = bytes;
    }
    for (uint32_t k = done + lane; k < bytes + tile.pad; k += kWave) dst[k] = k < bytes ? src[k] : uint8_t(0);
}

}  // namespace
}  // namespace cgx
