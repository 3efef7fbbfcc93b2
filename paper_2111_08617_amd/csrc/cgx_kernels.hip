// gfx950 kernels: bucketed stochastic quantization of a fused gradient buffer
// and dequantize-and-reduce of W compressed chunks.
//
// One wavefront (64 lanes) owns one tile of the plan.  In the vectorised path a
// wave takes a chunk of kChunk = 2048 elements per pass: each lane holds 4 groups
// of 8 consecutive elements, all of the same bucket (a bucket of B elements
// spans B/32 neighbouring lanes), so
//   - the bucket minimum / maximum is a lane-local reduction over 32 values
//     followed by a log2(B/32)-step butterfly across lanes (DPP within a row of
//     16 lanes, ds_swizzle across rows, a permute across the two halves);
//   - the two divisions of the bucket scale are paid once per 32 elements;
//   - 8 consecutive codes pack into exactly b bytes, so no code straddles lanes.
// The gradient is read from HBM once; a bucket lives in registers between the
// reduction and the rounding (paper Sec. 4.3: parallel bucket norm computation,
// vectorized loads and stores).  All streaming traffic is non-temporal and every
// store instruction writes whole lines: packed codes and sums are staged in LDS
// and leave lane-contiguous; the reduce fetches each peer's packed bytes straight
// into LDS (global_load_lds_dwordx4).
//
// The arithmetic of the code decision is binary32 without contraction and must
// stay as written: the packed output is compared bit for bit with a CPU
// implementation of the same definition.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "cgx_kernels.h"

namespace cgx {
namespace {

constexpr int kWave = 64;
#ifndef CGX_WAVES_PER_BLOCK
#define CGX_WAVES_PER_BLOCK 4
#endif
constexpr int kWavesPerBlock = CGX_WAVES_PER_BLOCK;
constexpr int kBlock = kWave * kWavesPerBlock;

typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------- generator

// 32-bit avalanche finalizer (xor-shift 16, odd multiply, xor-shift 15, odd
// multiply, xor-shift 16).
__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// Key of a 2^32-pair block: folds the seed and the upper half of the pair index.
__device__ __forceinline__ uint32_t rng_key(uint32_t seed_lo, uint32_t seed_hi, uint32_t pair_hi)
{
    return mix32(seed_lo ^ mix32(seed_hi ^ 0x9e3779b9U ^ pair_hi));
}

// 16-bit draw of element i (slow path: key recomputed per element).
__device__ __forceinline__ uint32_t draw16(uint32_t seed_lo, uint32_t seed_hi, uint64_t i)
{
    const uint64_t pair = i >> 1;
    const uint32_t r = mix32(uint32_t(pair) ^ rng_key(seed_lo, seed_hi, uint32_t(pair >> 32)));
    return (i & 1) ? (r >> 16) : (r & 0xffffU);
}

// ---------------------------------------------------------------- cross-lane

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    const int s = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(s, s, CTRL, 0xf, 0xf, false));
}

__device__ __forceinline__ float swizzle_xor16(float v)
{
    // bit-mask mode: and 0x1f, or 0, xor 0x10 -> lane ^ 16 within each half
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401f));
}

__device__ __forceinline__ float permute_xor32(float v, int lane)
{
    return __builtin_bit_cast(float,
                              __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, v)));
}

// Minimum and maximum over groups of 2^lg neighbouring lanes, result in every lane.
__device__ __forceinline__ void group_minmax(float &mn, float &mx, int lg, int lane)
{
    if (lg >= 1) {   // lane ^ 1: quad_perm [1,0,3,2]
        mn = __builtin_fminf(mn, dpp_move<0xB1>(mn));
        mx = __builtin_fmaxf(mx, dpp_move<0xB1>(mx));
    }
    if (lg >= 2) {   // lane ^ 2: quad_perm [2,3,0,1]
        mn = __builtin_fminf(mn, dpp_move<0x4E>(mn));
        mx = __builtin_fmaxf(mx, dpp_move<0x4E>(mx));
    }
    if (lg >= 3) {   // quads are uniform now: row_half_mirror pairs each quad with its neighbour
        mn = __builtin_fminf(mn, dpp_move<0x141>(mn));
        mx = __builtin_fmaxf(mx, dpp_move<0x141>(mx));
    }
    if (lg >= 4) {   // row_mirror pairs the two halves of a row of 16
        mn = __builtin_fminf(mn, dpp_move<0x140>(mn));
        mx = __builtin_fmaxf(mx, dpp_move<0x140>(mx));
    }
    if (lg >= 5) {
        mn = __builtin_fminf(mn, swizzle_xor16(mn));
        mx = __builtin_fmaxf(mx, swizzle_xor16(mx));
    }
    if (lg >= 6) {
        mn = __builtin_fminf(mn, permute_xor32(mn, lane));
        mx = __builtin_fmaxf(mx, permute_xor32(mx, lane));
    }
}

// ---------------------------------------------------------------- bucket scale

struct Scale {
    float unit, mn, inv16;
};

// unit = (mx - mn) / Lv, inv16 = (Lv * 65536) / (mx - mn), both IEEE divisions;
// a constant or degenerate bucket gets unit = inv16 = 0; a zero minimum is +0.
__device__ __forceinline__ Scale bucket_scale(float mn, float mx, int bits)
{
    const int levels = (1 << bits) - 1;
    if (mn == 0.0f) mn = 0.0f;
    const float range = mx - mn;
    float unit = __fdiv_rn(range, float(levels));
    float inv16 = __fdiv_rn(float(levels * 65536), range);
    if (!(unit > 0.0f) || !__builtin_isfinite(unit) || !__builtin_isfinite(inv16)) {
        unit = 0.0f;
        inv16 = 0.0f;
    }
    return Scale{unit, mn, inv16};
}

__device__ __forceinline__ uint32_t code_of(float x, const Scale &s, uint32_t draw, uint32_t levels)
{
    const float d = __fsub_rn(x, s.mn);
    const float S = __fmul_rn(d, s.inv16);
    const uint32_t T = uint32_t(S);                 // v_cvt_u32_f32: truncates, saturates
    const uint32_t q = (T + draw) >> 16;
    return q < levels ? q : levels;
}

// ---------------------------------------------------------------- element access

template <int DT>
__device__ __forceinline__ float load_elem(const void *buf, int64_t i)
{
    if (DT == CGX_F16) return float(reinterpret_cast<const _Float16 *>(buf)[i]);
    return reinterpret_cast<const float *>(buf)[i];
}

#ifndef CGX_NT_LOAD
#define CGX_NT_LOAD 1
#endif
#ifndef CGX_NT_STORE
#define CGX_NT_STORE 1
#endif
#ifndef CGX_PIPELINE
#define CGX_PIPELINE 0
#endif

template <typename T>
__device__ __forceinline__ T stream_load(const T *p)
{
#if CGX_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

template <typename T>
__device__ __forceinline__ void stream_store(T *p, T v)
{
#if CGX_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

#ifndef CGX_STAGE_OUT
#define CGX_STAGE_OUT 1
#endif

// Orders this wave's LDS writes before its later LDS reads (a wave's LDS operations
// execute in order; this only keeps the compiler from moving them).
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Streams `vecs` 16-byte vectors from the wave's LDS staging area to global memory,
// lane-contiguous (each store instruction writes 1 KB of consecutive addresses).
__device__ __forceinline__ void flush_stage(const uint4v *stage, uint4v *dst, int vecs, int lane)
{
    for (int v = lane; v < vecs; v += kWave) stream_store(dst + v, stage[v]);
}

// 8 consecutive elements starting at element e (16-byte aligned address), as stored.
template <int DT>
struct Raw8;
template <>
struct Raw8<CGX_F32> {
    float4v a, b;
    __device__ __forceinline__ void load(const void *buf, int64_t e)
    {
        const float4v *p = reinterpret_cast<const float4v *>(reinterpret_cast<const float *>(buf) + e);
        a = stream_load(p);
        b = stream_load(p + 1);
    }
    __device__ __forceinline__ void widen(float (&x)[8]) const
    {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            x[j] = a[j];
            x[4 + j] = b[j];
        }
    }
};
template <>
struct Raw8<CGX_F16> {
    half8v h;
    __device__ __forceinline__ void load(const void *buf, int64_t e)
    {
        h = stream_load(reinterpret_cast<const half8v *>(reinterpret_cast<const _Float16 *>(buf) + e));
    }
    __device__ __forceinline__ void widen(float (&x)[8]) const
    {
#pragma unroll
        for (int j = 0; j < 8; j++) x[j] = float(h[j]);
    }
};

template <int DT>
__device__ __forceinline__ void load8(const void *buf, int64_t e, float (&x)[8])
{
    Raw8<DT> raw;
    raw.load(buf, e);
    raw.widen(x);
}

// b bytes holding 8 codes, to a b-byte aligned address.
template <int BITS>
__device__ __forceinline__ void store_codes(uint8_t *p, uint64_t acc)
{
    if (BITS == 8) {
        stream_store(reinterpret_cast<uint64_t *>(p), acc);
    } else if (BITS == 4) {
        stream_store(reinterpret_cast<uint32_t *>(p), uint32_t(acc));
    } else if (BITS == 2) {
        stream_store(reinterpret_cast<uint16_t *>(p), uint16_t(acc));
    } else {
#pragma unroll
        for (int k = 0; k < BITS; k++) p[k] = uint8_t(acc >> (8 * k));
    }
}

// Same, into the LDS staging area (plain stores).
template <int BITS>
__device__ __forceinline__ void stage_codes(uint8_t *p, uint64_t acc)
{
    if (BITS == 8) {
        *reinterpret_cast<uint64_t *>(p) = acc;
    } else if (BITS == 4) {
        *reinterpret_cast<uint32_t *>(p) = uint32_t(acc);
    } else if (BITS == 2) {
        *reinterpret_cast<uint16_t *>(p) = uint16_t(acc);
    } else {
#pragma unroll
        for (int k = 0; k < BITS; k++) p[k] = uint8_t(acc >> (8 * k));
    }
}

template <int BITS>
__device__ __forceinline__ uint64_t load_codes(const uint8_t *p)
{
    if (BITS == 8) return stream_load(reinterpret_cast<const uint64_t *>(p));
    if (BITS == 4) return stream_load(reinterpret_cast<const uint32_t *>(p));
    if (BITS == 2) return stream_load(reinterpret_cast<const uint16_t *>(p));
    uint64_t acc = 0;
#pragma unroll
    for (int k = 0; k < BITS; k++) acc |= uint64_t(p[k]) << (8 * k);
    return acc;
}

// ---------------------------------------------------------------- quantize

template <int DT, int BITS>
__device__ __forceinline__ void quantize_fast(const void *__restrict__ grad, uint8_t *__restrict__ packed,
                                              float2 *__restrict__ meta, const Tile &tile, int bucket,
                                              uint32_t seed_lo, uint32_t seed_hi, int lane, uint4v *stage)
{
    constexpr uint32_t kLevels = (1u << BITS) - 1u;
    constexpr int G = kGroups;
    const int lg = int(tile_lpb_log2(tile));
    const int bi = lane >> lg;                       // bucket of this lane within the chunk
    const int lp = lane & ((1 << lg) - 1);           // lane within the bucket
    const int row = 8 << lg;                         // elements between a lane's groups = bucket / G
    const int e_lane = bi * bucket + lp * 8;
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    const int chunks = int(tile.count / kChunk);
    const int buckets_per_chunk = kChunk / bucket;

    Raw8<DT> raw[G];
#pragma unroll
    for (int r = 0; r < G; r++) raw[r].load(grad, tile.elem0 + e_lane + r * row);

    for (int c = 0; c < chunks; c++) {
        const int64_t e0 = tile.elem0 + int64_t(c) * kChunk + e_lane;
        float x[G][8];
#pragma unroll
        for (int r = 0; r < G; r++) raw[r].widen(x[r]);
#if CGX_PIPELINE
        if (c + 1 < chunks) {                        // next chunk's loads fly while this one is processed
#pragma unroll
            for (int r = 0; r < G; r++) raw[r].load(grad, e0 + kChunk + r * row);
        }
#endif

        float mn = x[0][0], mx = x[0][0];
#pragma unroll
        for (int r = 0; r < G; r++)
#pragma unroll
            for (int j = 0; j < 8; j++) {
                mn = __builtin_fminf(mn, x[r][j]);
                mx = __builtin_fmaxf(mx, x[r][j]);
            }
        group_minmax(mn, mx, lg, lane);
        const Scale s = bucket_scale(mn, mx, BITS);
        if (lp == 0) meta[tile.bucket0 + c * buckets_per_chunk + bi] = make_float2(s.unit, s.mn);

        uint8_t *out = packed + tile.packed_off + int64_t(c) * (kChunk * BITS / 8);
#pragma unroll
        for (int r = 0; r < G; r++) {
            const uint32_t pair0 = uint32_t(uint64_t(e0 + r * row) >> 1);
            uint64_t acc = 0;
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const uint32_t w = mix32((pair0 + k) ^ key);
                const uint64_t q0 = code_of(x[r][2 * k], s, w & 0xffffU, kLevels);
                const uint64_t q1 = code_of(x[r][2 * k + 1], s, w >> 16, kLevels);
                acc |= q0 << (2 * k * BITS);
                acc |= q1 << ((2 * k + 1) * BITS);
            }
#if CGX_STAGE_OUT
            stage_codes<BITS>(reinterpret_cast<uint8_t *>(stage) + ((e_lane + r * row) >> 3) * BITS, acc);
#else
            store_codes<BITS>(out + ((e_lane + r * row) >> 3) * BITS, acc);
#endif
        }
#if CGX_STAGE_OUT
        // the chunk's codes leave as whole 16-byte vectors, consecutive across lanes
        wave_lds_fence();
        flush_stage(stage, reinterpret_cast<uint4v *>(out), kChunk * BITS / 128, lane);
        wave_lds_fence();
#endif
#if !CGX_PIPELINE
        if (c + 1 < chunks) {
#pragma unroll
            for (int r = 0; r < G; r++) raw[r].load(grad, e0 + kChunk + r * row);
        }
#endif
    }
}

// Any bucket size, any alignment, ragged last bucket: one bucket at a time, two passes.
// Loads are issued in batches of 8 so that a pass costs few memory round trips.
template <int DT>
__device__ void quantize_slow(const void *__restrict__ grad, uint8_t *__restrict__ packed,
                              float2 *__restrict__ meta, const Tile &tile, int bucket, uint32_t seed_lo,
                              uint32_t seed_hi, int lane)
{
    const int b = int(tile_bits(tile));
    const uint32_t levels = (1u << b) - 1u;
    uint8_t *out = packed + tile.packed_off;
    for (uint32_t k0 = 0; k0 < tile.count; k0 += uint32_t(bucket)) {
        const uint32_t cnt = tile.count - k0 < uint32_t(bucket) ? tile.count - k0 : uint32_t(bucket);
        const int64_t base = tile.elem0 + k0;
        float mn = __builtin_inff(), mx = -__builtin_inff();
        for (uint32_t j0 = 0; j0 < cnt; j0 += 8 * kWave) {
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const uint32_t j = j0 + u * kWave + lane;
                x[u] = load_elem<DT>(grad, base + (j < cnt ? j : 0));     // clamped: element 0 again
            }
#pragma unroll
            for (int u = 0; u < 8; u++) {
                mn = __builtin_fminf(mn, x[u]);
                mx = __builtin_fmaxf(mx, x[u]);
            }
        }
        group_minmax(mn, mx, 6, lane);
        const Scale s = bucket_scale(mn, mx, b);
        if (lane == 0) meta[tile.bucket0 + k0 / uint32_t(bucket)] = make_float2(s.unit, s.mn);

        const uint32_t groups = (cnt + 7) / 8;
        for (uint32_t g = lane; g < groups; g += kWave) {
            const uint32_t valid = cnt - g * 8 < 8 ? cnt - g * 8 : 8;
            float x[8];
#pragma unroll
            for (uint32_t j = 0; j < 8; j++) x[j] = load_elem<DT>(grad, base + g * 8 + (j < valid ? j : 0));
            uint64_t acc = 0;
#pragma unroll
            for (uint32_t j = 0; j < 8; j++) {
                const uint64_t i = uint64_t(base + g * 8 + j);
                const uint64_t q = code_of(x[j], s, draw16(seed_lo, seed_hi, i), levels);
                if (j < valid) acc |= q << (j * b);
            }
            const uint32_t nbytes = (valid * b + 7) / 8;
            uint8_t *p = out + uint64_t(k0 / 8 + g) * b;
            for (uint32_t k = 0; k < nbytes; k++) p[k] = uint8_t(acc >> (8 * k));
        }
    }
    if (tile.pad) {
        const uint64_t end = (uint64_t(tile.count) * b + 7) / 8;
        if (uint32_t(lane) < tile.pad) out[end + lane] = 0;
    }
}

// Pass-through tile of the quantize kernel: verbatim copy, then the layer's zero padding.
template <int DT>
__device__ void copy_tile(const void *__restrict__ grad, uint8_t *__restrict__ packed, const Tile &tile,
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
            reinterpret_cast<uint4v *>(dst)[v] = reinterpret_cast<const uint4v *>(src)[v];
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

template <int DT>
__global__ __launch_bounds__(kBlock) void quantize_kernel(const void *__restrict__ grad,
                                                           const Tile *__restrict__ tiles, int64_t n_tiles,
                                                           int bucket, uint32_t seed_lo, uint32_t seed_hi,
                                                           uint8_t *__restrict__ packed,
                                                           float2 *__restrict__ meta)
{
    // per-wave staging area for a chunk's packed codes (at most kChunk bytes, at 8 bits)
    __shared__ uint4v stage_all[kWavesPerBlock][kChunk / 16];
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = int(threadIdx.x) & 63;
    uint4v *stage = stage_all[wave];
    const int64_t stride = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t t = int64_t(blockIdx.x) * kWavesPerBlock + wave; t < n_tiles; t += stride) {
        const Tile tile = tiles[t];
        const uint32_t kind = tile_kind(tile);
        if (kind == kQuantFast) {
            switch (tile_bits(tile)) {
            case 1: quantize_fast<DT, 1>(grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane, stage); break;
            case 2: quantize_fast<DT, 2>(grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane, stage); break;
            case 3: quantize_fast<DT, 3>(grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane, stage); break;
            case 4: quantize_fast<DT, 4>(grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane, stage); break;
            case 5: quantize_fast<DT, 5>(grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane, stage); break;
            case 6: quantize_fast<DT, 6>(grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane, stage); break;
            case 7: quantize_fast<DT, 7>(grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane, stage); break;
            default: quantize_fast<DT, 8>(grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane, stage); break;
            }
        } else if (kind == kQuantSlow) {
            quantize_slow<DT>(grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane);
        } else {
            copy_tile<DT>(grad, packed, tile, kind == kCopyFast, lane);
        }
    }
}

// ---------------------------------------------------------------- dequantize + reduce

// Codes of one group of 8 elements as floats.
template <int BITS>
__device__ __forceinline__ void codes_to_float(uint64_t v, float (&f)[8])
{
    if (BITS == 8) {
        const uint32_t lo = uint32_t(v), hi = uint32_t(v >> 32);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            f[j] = float((lo >> (8 * j)) & 0xffu);
            f[4 + j] = float((hi >> (8 * j)) & 0xffu);
        }
    } else if (BITS == 4) {
        const uint32_t w = uint32_t(v);
        const uint32_t even = w & 0x0f0f0f0fu, odd = (w >> 4) & 0x0f0f0f0fu;   // one code per byte
#pragma unroll
        for (int j = 0; j < 4; j++) {
            f[2 * j] = float((even >> (8 * j)) & 0xffu);
            f[2 * j + 1] = float((odd >> (8 * j)) & 0xffu);
        }
    } else if (BITS == 2) {
        const uint32_t w = uint32_t(v);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const uint32_t t = (w >> (2 * j)) & 0x0303u;     // codes j and j + 4, one per byte
            f[j] = float(t & 0xffu);
            f[4 + j] = float((t >> 8) & 0xffu);
        }
    } else {
        constexpr uint64_t kMask = (1u << BITS) - 1u;
#pragma unroll
        for (int j = 0; j < 8; j++) f[j] = float(uint32_t((v >> (j * BITS)) & kMask));
    }
}

// b bytes holding 8 codes, read back from the LDS staging area.
template <int BITS>
__device__ __forceinline__ uint64_t staged_codes(const uint8_t *p)
{
    if (BITS == 8) return *reinterpret_cast<const uint64_t *>(p);
    if (BITS == 4) return *reinterpret_cast<const uint32_t *>(p);
    if (BITS == 2) return *reinterpret_cast<const uint16_t *>(p);
    uint64_t acc = 0;
#pragma unroll
    for (int k = 0; k < BITS; k++) acc |= uint64_t(p[k]) << (8 * k);
    return acc;
}

// One 16-byte vector per lane from global memory straight into LDS, without passing
// through registers: lane l's vector lands at lds_base + 16 * l (lds_base is wave-uniform).
__device__ __forceinline__ void load_to_lds16(const uint4v *gptr, uint4v *lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gptr,
                                     (__attribute__((address_space(3))) void *)lds_base, 16, 0,
                                     CGX_NT_LOAD ? 2 : 0);
}

// Waits until every outstanding vector-memory operation of this wave has completed
// (s_waitcnt vmcnt(0); the export and LDS counters are left alone).
__device__ __forceinline__ void wait_vector_memory()
{
    __builtin_amdgcn_s_waitcnt(0x0f70);
}

// Folds peers w0 .. w0+WB-1 into acc.  Each peer's share of the chunk (kChunk*BITS/8 bytes)
// is fetched as whole 16-byte vectors, consecutive across lanes, directly into the wave's
// LDS staging area, and read back by the lanes that own the codes.
template <int BITS, int WB>
__device__ __forceinline__ void reduce_peers(const PeerPtrs &peers, int w0, int64_t in_off, uint32_t g,
                                             const int (&code_off)[kGroups], float (&acc)[kGroups][8],
                                             uint4v *stage, int lane)
{
    constexpr int kBytes = kChunk * BITS / 8;        // per peer
    constexpr int kVecs = kBytes / 16;
    constexpr int kPerLane = (kVecs + kWave - 1) / kWave;
    float2 m[WB];
#pragma unroll
    for (int i = 0; i < WB; i++) {
        const uint4v *in = reinterpret_cast<const uint4v *>(peers.packed[w0 + i] + in_off);
#pragma unroll
        for (int k = 0; k < kPerLane; k++) {
            const int v = lane + k * kWave;
            if (kVecs % kWave == 0 || v < kVecs) load_to_lds16(in + v, stage + i * kVecs + k * kWave);
        }
        m[i] = peers.meta[w0 + i][g];
    }
    wait_vector_memory();
    wave_lds_fence();
    const uint8_t *codes = reinterpret_cast<const uint8_t *>(stage);
#pragma unroll
    for (int i = 0; i < WB; i++) {
#pragma unroll
        for (int r = 0; r < kGroups; r++) {
            float f[8];
            codes_to_float<BITS>(staged_codes<BITS>(codes + i * kBytes + code_off[r]), f);
#pragma unroll
            for (int j = 0; j < 8; j++) acc[r][j] = __fadd_rn(acc[r][j], __builtin_fmaf(f[j], m[i].x, m[i].y));
        }
#ifndef CGX_SCHED_PEERS
#define CGX_SCHED_PEERS 2
#endif
        // keep the scheduler from hoisting every peer's LDS reads to the top (registers)
        if (CGX_SCHED_PEERS && (i % CGX_SCHED_PEERS) == CGX_SCHED_PEERS - 1) __builtin_amdgcn_sched_barrier(0);
    }
    wave_lds_fence();
}

template <int BITS>
__device__ __forceinline__ void reduce_fast(const PeerPtrs &peers, int W, bool accumulate,
                                            float *__restrict__ sum, const Tile &tile, int bucket, int lane,
                                            uint4v *stage)
{
    constexpr int G = kGroups;
    // peers staged together: their packed bytes fit the staging area (one chunk of sums,
    // kChunk * 4 bytes)
    constexpr int kBytes = kChunk * BITS / 8;
    // (bit widths whose codes are read back byte by byte take fewer peers at a time: the
    // byte reads of a whole block are in flight together and each holds a register)
    constexpr bool kByteReads = BITS != 1 && BITS != 2 && BITS != 4 && BITS != 8;
    constexpr int kWide = kByteReads ? (BITS == 3 ? 2 : 1) : (8 * kBytes <= kChunk * 4 ? 8 : 4);
    static_assert(kWide * kBytes <= kChunk * 4, "staging area too small");
    const int lg = int(tile_lpb_log2(tile));
    const int bi = lane >> lg;
    const int lp = lane & ((1 << lg) - 1);
    const int row = 8 << lg;
    const int e_lane = bi * bucket + lp * 8;
    const int chunks = int(tile.count / kChunk);
    const int buckets_per_chunk = kChunk / bucket;
    int code_off[G];
#pragma unroll
    for (int r = 0; r < G; r++) code_off[r] = ((e_lane + r * row) >> 3) * BITS;

    for (int c = 0; c < chunks; c++) {
        const int64_t e_chunk = tile.elem0 + int64_t(c) * kChunk;
        const int64_t in_off = tile.packed_off + int64_t(c) * kBytes;
        const uint32_t g = tile.bucket0 + c * buckets_per_chunk + bi;
        // -0 is the identity of binary32 addition for every addend, signed zeros included,
        // so the first peer's value enters the sum unchanged
        float acc[G][8];
        if (accumulate) {
#pragma unroll
            for (int r = 0; r < G; r++) load8<CGX_F32>(sum, e_chunk + e_lane + r * row, acc[r]);
        } else {
#pragma unroll
            for (int r = 0; r < G; r++)
#pragma unroll
                for (int j = 0; j < 8; j++) acc[r][j] = -0.0f;
        }
        int w = 0;
        if (kWide >= 8)
            for (; w + 8 <= W; w += 8) reduce_peers<BITS, 8>(peers, w, in_off, g, code_off, acc, stage, lane);
        if (kWide >= 4)
            for (; w + 4 <= W; w += 4) reduce_peers<BITS, 4>(peers, w, in_off, g, code_off, acc, stage, lane);
        if (kWide >= 2)
            for (; w + 2 <= W; w += 2) reduce_peers<BITS, 2>(peers, w, in_off, g, code_off, acc, stage, lane);
        for (; w < W; w++) reduce_peers<BITS, 1>(peers, w, in_off, g, code_off, acc, stage, lane);

        // the sums leave through LDS as well, so that every store instruction writes 1 KB of
        // consecutive addresses
#pragma unroll
        for (int r = 0; r < G; r++) {
            float4v *p = reinterpret_cast<float4v *>(stage) + ((e_lane + r * row) >> 2);
            p[0] = float4v{acc[r][0], acc[r][1], acc[r][2], acc[r][3]};
            p[1] = float4v{acc[r][4], acc[r][5], acc[r][6], acc[r][7]};
        }
        wave_lds_fence();
        flush_stage(stage, reinterpret_cast<uint4v *>(sum + e_chunk), kChunk / 4, lane);
        wave_lds_fence();
    }
}

// Calls f(w0, std::integral_constant<int, WB>) for consecutive blocks of 8, 4, 2, 1 peers
// covering 0..W-1 in order, so that a block's loads can be issued together.
template <typename F>
__device__ __forceinline__ void for_peer_blocks(int W, F f)
{
    int w = 0;
    for (; w + 8 <= W; w += 8) f(w, std::integral_constant<int, 8>());
    if (w + 4 <= W) {
        f(w, std::integral_constant<int, 4>());
        w += 4;
    }
    if (w + 2 <= W) {
        f(w, std::integral_constant<int, 2>());
        w += 2;
    }
    if (w < W) f(w, std::integral_constant<int, 1>());
}

// Any bucket size, any alignment, ragged tiles: one element per lane and pass.
__device__ void reduce_slow(const PeerPtrs &peers, int W, bool accumulate, float *__restrict__ sum,
                            const Tile &tile, int bucket, int lane)
{
    const int b = int(tile_bits(tile));
    const uint32_t mask = (1u << b) - 1u;
    for (uint32_t j = lane; j < tile.count; j += kWave) {
        const uint32_t g = tile.bucket0 + j / uint32_t(bucket);
        const uint64_t bit = uint64_t(j) * b;
        const int64_t at = tile.packed_off + int64_t(bit >> 3);
        const uint32_t shift = uint32_t(bit & 7);
        const bool two = shift + b > 8;                  // a code spans at most two bytes
        float acc = accumulate ? sum[tile.elem0 + j] : -0.0f;
        for_peer_blocks(W, [&](int w0, auto wb) {
            constexpr int WB = decltype(wb)::value;
            uint32_t lo[WB], hi[WB];
            float2 m[WB];
#pragma unroll
            for (int i = 0; i < WB; i++) {
                const uint8_t *p = peers.packed[w0 + i] + at;
                lo[i] = p[0];
                hi[i] = two ? p[1] : 0u;
                m[i] = peers.meta[w0 + i][g];
            }
#pragma unroll
            for (int i = 0; i < WB; i++) {
                const uint32_t q = ((lo[i] | (hi[i] << 8)) >> shift) & mask;
                acc = __fadd_rn(acc, __builtin_fmaf(float(q), m[i].x, m[i].y));
            }
        });
        sum[tile.elem0 + j] = acc;
    }
}

// Pass-through tile of the reduce kernel: plain ordered sum of the stored values.
template <int DT>
__device__ void reduce_copy(const PeerPtrs &peers, int W, bool accumulate, float *__restrict__ sum,
                            const Tile &tile, bool fast, int lane)
{
    const uint32_t groups = fast ? tile.count / 8 : 0;
    for (uint32_t g = lane; g < groups; g += kWave) {
        float acc[8];
        if (accumulate) {
            load8<CGX_F32>(sum, tile.elem0 + g * 8, acc);
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++) acc[j] = -0.0f;
        }
        for_peer_blocks(W, [&](int w0, auto wb) {
            constexpr int WB = decltype(wb)::value;
            Raw8<DT> raw[WB];
#pragma unroll
            for (int i = 0; i < WB; i++) raw[i].load(peers.packed[w0 + i] + tile.packed_off, int64_t(g) * 8);
#pragma unroll
            for (int i = 0; i < WB; i++) {
                float x[8];
                raw[i].widen(x);
#pragma unroll
                for (int j = 0; j < 8; j++) acc[j] = __fadd_rn(acc[j], x[j]);
            }
        });
        float4v *p = reinterpret_cast<float4v *>(sum + tile.elem0 + g * 8);
        p[0] = float4v{acc[0], acc[1], acc[2], acc[3]};
        p[1] = float4v{acc[4], acc[5], acc[6], acc[7]};
    }
    for (uint32_t j = groups * 8 + lane; j < tile.count; j += kWave) {
        float acc = accumulate ? sum[tile.elem0 + j] : -0.0f;
        for_peer_blocks(W, [&](int w0, auto wb) {
            constexpr int WB = decltype(wb)::value;
            float x[WB];
#pragma unroll
            for (int i = 0; i < WB; i++) x[i] = load_elem<DT>(peers.packed[w0 + i] + tile.packed_off, j);
#pragma unroll
            for (int i = 0; i < WB; i++) acc = __fadd_rn(acc, x[i]);
        });
        sum[tile.elem0 + j] = acc;
    }
}

__global__ __launch_bounds__(kBlock) void reduce_kernel(const PeerPtrs peers, int W, int dt, bool accumulate,
                                                         const Tile *__restrict__ tiles, int64_t n_tiles,
                                                         int bucket, float *__restrict__ sum)
{
    // per-wave staging area for a chunk of binary32 sums
    __shared__ uint4v stage_all[kWavesPerBlock][kChunk / 4];
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = int(threadIdx.x) & 63;
    uint4v *stage = stage_all[wave];
    const int64_t stride = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t t = int64_t(blockIdx.x) * kWavesPerBlock + wave; t < n_tiles; t += stride) {
        const Tile tile = tiles[t];
        const uint32_t kind = tile_kind(tile);
        if (kind == kQuantFast) {
            switch (tile_bits(tile)) {
            case 1: reduce_fast<1>(peers, W, accumulate, sum, tile, bucket, lane, stage); break;
            case 2: reduce_fast<2>(peers, W, accumulate, sum, tile, bucket, lane, stage); break;
            case 3: reduce_fast<3>(peers, W, accumulate, sum, tile, bucket, lane, stage); break;
            case 4: reduce_fast<4>(peers, W, accumulate, sum, tile, bucket, lane, stage); break;
            case 5: reduce_fast<5>(peers, W, accumulate, sum, tile, bucket, lane, stage); break;
            case 6: reduce_fast<6>(peers, W, accumulate, sum, tile, bucket, lane, stage); break;
            case 7: reduce_fast<7>(peers, W, accumulate, sum, tile, bucket, lane, stage); break;
            default: reduce_fast<8>(peers, W, accumulate, sum, tile, bucket, lane, stage); break;
            }
        } else if (kind == kQuantSlow) {
            reduce_slow(peers, W, accumulate, sum, tile, bucket, lane);
        } else if (dt == CGX_F16) {
            reduce_copy<CGX_F16>(peers, W, accumulate, sum, tile, kind == kCopyFast, lane);
        } else {
            reduce_copy<CGX_F32>(peers, W, accumulate, sum, tile, kind == kCopyFast, lane);
        }
    }
}

inline unsigned grid_for(int64_t n_tiles, const LaunchConfig &cfg)
{
    int64_t blocks = (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (cfg.max_blocks > 0 && blocks > cfg.max_blocks) blocks = cfg.max_blocks;
    if (blocks > 0x7fffffff) blocks = 0x7fffffff;
    return unsigned(blocks);
}

}  // namespace

hipError_t launch_quantize(const void *grad, int dt, const Tile *tiles, int64_t n_tiles, int32_t bucket,
                           uint64_t seed, void *packed, void *meta, const LaunchConfig &cfg,
                           hipStream_t stream)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(grid_for(n_tiles, cfg)), block(kBlock);
    const uint32_t seed_lo = uint32_t(seed), seed_hi = uint32_t(seed >> 32);
    if (dt == CGX_F16)
        hipLaunchKernelGGL(quantize_kernel<CGX_F16>, grid, block, 0, stream, grad, tiles, n_tiles, int(bucket),
                           seed_lo, seed_hi, static_cast<uint8_t *>(packed), static_cast<float2 *>(meta));
    else
        hipLaunchKernelGGL(quantize_kernel<CGX_F32>, grid, block, 0, stream, grad, tiles, n_tiles, int(bucket),
                           seed_lo, seed_hi, static_cast<uint8_t *>(packed), static_cast<float2 *>(meta));
    return hipGetLastError();
}

hipError_t launch_dequant_reduce(const PeerPtrs &peers, int W, int dt, const Tile *tiles, int64_t n_tiles,
                                 int32_t bucket, bool accumulate, float *sum, const LaunchConfig &cfg,
                                 hipStream_t stream)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(grid_for(n_tiles, cfg)), block(kBlock);
    hipLaunchKernelGGL(reduce_kernel, grid, block, 0, stream, peers, W, dt, accumulate, tiles, n_tiles,
                       int(bucket), sum);
    return hipGetLastError();
}

}  // namespace cgx
