// gfx950 kernels: bucketed stochastic quantization of a fused gradient buffer,
// dequantize-and-reduce of W compressed chunks, and the two fused into one pass.
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

// The peers' pointer table is a kernel argument (256 bytes).  The kernels read it where the
// dispatch packet put it, in the constant-address-space kernarg segment, with scalar loads at
// computed offsets; taken as an ordinary by-value parameter it would be copied into 64 scalar
// registers at entry and, in the larger kernels, spilled to scratch to be indexed.
typedef const __attribute__((address_space(4))) PeerPtrs KernargPeers;

// The table when it is the kernel's FIRST parameter (offset 0 of the kernarg segment).
__device__ __forceinline__ KernargPeers &first_kernel_argument()
{
    return *(KernargPeers *)__builtin_amdgcn_kernarg_segment_ptr();
}

constexpr int kWave = 64;
#ifndef CGX_WAVES_PER_BLOCK
#define CGX_WAVES_PER_BLOCK 4
#endif
constexpr int kWavesPerBlock = CGX_WAVES_PER_BLOCK;
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int G = kGroups;               // groups of 8 elements per lane and chunk

typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
// The same vectors at the alignment of ONE element: a layer may start anywhere in the fused
// buffer, so accesses on the gradient / sum side promise no more than that.  Global memory takes
// 16-byte accesses at any alignment in this execution mode (the instructions are the same; only
// the lines touched by an instruction shift), which keeps unaligned layers on the vectorised path.
typedef float4v float4u __attribute__((aligned(4)));
typedef half8v half8u __attribute__((aligned(2)));
typedef uint4v uint4u2 __attribute__((aligned(2)));

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

// 16-bit draw of element i (generic path: key recomputed per element).
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

// Maximum alone, same exchange pattern.
__device__ __forceinline__ void group_max(float &mx, int lg, int lane)
{
    if (lg >= 1) mx = __builtin_fmaxf(mx, dpp_move<0xB1>(mx));
    if (lg >= 2) mx = __builtin_fmaxf(mx, dpp_move<0x4E>(mx));
    if (lg >= 3) mx = __builtin_fmaxf(mx, dpp_move<0x141>(mx));
    if (lg >= 4) mx = __builtin_fmaxf(mx, dpp_move<0x140>(mx));
    if (lg >= 5) mx = __builtin_fmaxf(mx, swizzle_xor16(mx));
    if (lg >= 6) mx = __builtin_fmaxf(mx, permute_xor32(mx, lane));
}

// ---------------------------------------------------------------- the two quantizers
//
// kMinMax: affine per bucket.  A b-bit code is a level 0..2^b-1 between the bucket's minimum
// and maximum; meta = {unit, minimum} (float2 per bucket); value = fma(level, unit, minimum).
// kNormSign: the norm-and-sign form printed in Sec. 2.2 (Q_s), with the bucket's largest
// magnitude as the norm.  A b-bit code (b >= 2) is sign(x) times a level 0..s,
// s = 2^(b-1)-1, of |x| / norm, as a two's complement number (decoding, done once per peer
// and element, is then a sign-extending conversion and a multiplication; encoding, done once
// per element, pays the negation); meta = unit = norm / s (one float per bucket);
// value = float(signed level) * unit.
// Both resolve the rounding probability to 16 bits with the same draws.
enum Scheme { kMinMax = kSchemeMinMax, kNormSign = kSchemeNormSign };

template <int SCHEME>
__device__ __forceinline__ constexpr uint32_t top_level(int bits)
{
    return SCHEME == kNormSign ? (1u << (bits - 1)) - 1u : (1u << bits) - 1u;
}

// floats of meta per bucket
template <int SCHEME>
constexpr int kMetaFloats = SCHEME == kNormSign ? 1 : 2;

struct Scale {
    float unit, mn, inv16;
};

// unit = (mx - mn) / Lv, inv16 = (Lv * 65536) / (mx - mn), both IEEE divisions;
// a constant or degenerate bucket gets unit = inv16 = 0; a zero minimum is +0.
// (kNormSign calls it with mn = +0 and mx = the largest magnitude.)
__device__ __forceinline__ Scale bucket_scale(float mn, float mx, int levels)
{
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

// bits is the code width (only kNormSign uses it, to cut the two's complement code).
template <int SCHEME>
__device__ __forceinline__ uint32_t code_of(float x, const Scale &s, uint32_t draw, uint32_t levels, int bits)
{
    const float d = SCHEME == kNormSign ? __builtin_fabsf(x) : __fsub_rn(x, s.mn);
    const float S = __fmul_rn(d, s.inv16);
    const uint32_t T = uint32_t(S);                 // v_cvt_u32_f32: truncates, saturates
    const uint32_t q = (T + draw) >> 16;
    const uint32_t level = q < levels ? q : levels;
    if (SCHEME == kNormSign) {
        const uint32_t neg = uint32_t(__builtin_bit_cast(int32_t, x) >> 31);    // all ones for a set sign bit
        return ((level ^ neg) - neg) & ((1u << bits) - 1u);
    }
    return level;
}

template <int SCHEME>
__device__ __forceinline__ void store_meta(float *meta, uint32_t g, const Scale &s)
{
    if (SCHEME == kNormSign)
        meta[g] = s.unit;
    else
        reinterpret_cast<float2 *>(meta)[g] = make_float2(s.unit, s.mn);
}

// {unit, offset} of bucket g (kNormSign: offset unused).
template <int SCHEME>
__device__ __forceinline__ float2 load_meta(const float *meta, uint32_t g)
{
    if (SCHEME == kNormSign) return make_float2(meta[g], 0.0f);
    return reinterpret_cast<const float2 *>(meta)[g];
}

// Value of a code whose (kNormSign: signed) level is f.
template <int SCHEME>
__device__ __forceinline__ float decode(float f, float2 m)
{
    if (SCHEME == kNormSign) return __fmul_rn(f, m.x);
    return __builtin_fmaf(f, m.x, m.y);
}

// ---------------------------------------------------------------- memory helpers

// Streaming data is touched once: non-temporal loads and stores keep it from
// displacing anything and (measured) raise the sustained HBM rate, provided each
// instruction covers whole lines.
template <typename T>
__device__ __forceinline__ T stream_load(const T *p)
{
    return __builtin_nontemporal_load(p);
}

template <typename T>
__device__ __forceinline__ void stream_store(T *p, T v)
{
    __builtin_nontemporal_store(v, p);
}
// (Pointers to the element-aligned vector types below must not go through these templates:
// a template argument drops the alignment of the typedef.  Their accesses call the builtins.)

template <int DT>
__device__ __forceinline__ float load_elem(const void *buf, int64_t i)
{
    if (DT == CGX_F16) return float(reinterpret_cast<const _Float16 *>(buf)[i]);
    return reinterpret_cast<const float *>(buf)[i];
}

// 8 consecutive elements starting at element e (16-byte aligned address), as stored.
template <int DT>
struct Raw8;
template <>
struct Raw8<CGX_F32> {
    float4v a, b;
    __device__ __forceinline__ void load(const void *buf, int64_t e)
    {
        const float4u *p = reinterpret_cast<const float4u *>(reinterpret_cast<const float *>(buf) + e);
        a = __builtin_nontemporal_load(p);
        b = __builtin_nontemporal_load(p + 1);
    }
    // the same with ordinary loads: for data that is read again shortly
    __device__ __forceinline__ void load_keep(const void *buf, int64_t e)
    {
        const float4u *p = reinterpret_cast<const float4u *>(reinterpret_cast<const float *>(buf) + e);
        a = p[0];
        b = p[1];
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
        h = __builtin_nontemporal_load(reinterpret_cast<const half8u *>(reinterpret_cast<const _Float16 *>(buf) + e));
    }
    __device__ __forceinline__ void load_keep(const void *buf, int64_t e)
    {
        h = *reinterpret_cast<const half8u *>(reinterpret_cast<const _Float16 *>(buf) + e);
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

// The same to an element-aligned destination (sums).
__device__ __forceinline__ void flush_stage_to_elements(const uint4v *stage, uint4u2 *dst, int vecs, int lane)
{
    for (int v = lane; v < vecs; v += kWave) __builtin_nontemporal_store(stage[v], dst + v);
}

// One 16-byte vector per lane from global memory straight into LDS, without passing
// through registers: lane l's vector lands at lds_base + 16 * l (lds_base is wave-uniform).
__device__ __forceinline__ void load_to_lds16(const uint4v *gptr, uint4v *lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gptr,
                                     (__attribute__((address_space(3))) void *)lds_base, 16, 0, 2 /* nt */);
}

// Waits until every outstanding vector-memory operation of this wave has completed
// (s_waitcnt vmcnt(0); the export and LDS counters are left alone).
__device__ __forceinline__ void wait_vector_memory()
{
    __builtin_amdgcn_s_waitcnt(0x0f70);
}

// b bytes holding 8 codes into the LDS staging area at a multiple of b bytes: exactly b bytes
// are written (the neighbours belong to other lanes); for the odd widths the copy is lowered
// to a few unaligned LDS stores (LDS accepts any alignment in this execution mode).
template <int BITS>
__device__ __forceinline__ void stage_codes(uint8_t *p, uint64_t acc)
{
    if (BITS == 8)
        *reinterpret_cast<uint64_t *>(p) = acc;
    else if (BITS == 4)
        *reinterpret_cast<uint32_t *>(p) = uint32_t(acc);
    else if (BITS == 2)
        *reinterpret_cast<uint16_t *>(p) = uint16_t(acc);
    else
        __builtin_memcpy(p, &acc, BITS);
}

// Bytes staged_codes may read past the b bytes of a group (their content is ignored).
template <int BITS>
constexpr int kStagedOverRead = (BITS == 3 || BITS == 5 || BITS == 6 || BITS == 7) ? 8 : 0;

// The b bytes holding 8 codes at byte offset off (a multiple of b) of a 4-byte aligned LDS
// area; bits above 8 * b of the result are unspecified.  Power-of-two widths read their
// naturally aligned unit.  The odd widths read the aligned dwords that cover the group and
// shift: unaligned LDS reads work but run at a fraction of the aligned rate (measured: the
// 3-bit reduce was LDS-bound with them).
template <int BITS>
__device__ __forceinline__ uint64_t staged_codes(const uint8_t *base, int off)
{
    if (BITS == 8) return *reinterpret_cast<const uint64_t *>(base + off);
    if (BITS == 4) return *reinterpret_cast<const uint32_t *>(base + off);
    if (BITS == 2) return *reinterpret_cast<const uint16_t *>(base + off);
    if (BITS == 1) return base[off];
    const uint32_t *w = reinterpret_cast<const uint32_t *>(base) + (off >> 2);
    const uint32_t shift = uint32_t(off & 3) * 8u;
    const uint32_t d0 = w[0], d1 = w[1];
    // 3 and 5 bits: shift + 8 * b <= 64, two dwords cover the group; 6 and 7 bits: three
    const uint32_t d2 = (BITS == 6 || BITS == 7) ? w[2] : 0u;
    const uint32_t lo = __builtin_amdgcn_alignbit(d1, d0, shift);      // ({d1, d0} >> shift), low 32 bits
    const uint32_t hi = BITS == 3 ? 0u : __builtin_amdgcn_alignbit(d2, d1, shift);
    return (uint64_t(hi) << 32) | lo;
}

// Calls f(w0, std::integral_constant<int, WB>) for consecutive blocks of at most MAXB
// (8, 4, 2, 1) peers covering 0..W-1 in order, so that a block's loads can be issued together.
template <int MAXB, typename F>
__device__ __forceinline__ void for_peer_blocks(int W, F f)
{
    int w = 0;
    if (MAXB >= 8)
        for (; w + 8 <= W; w += 8) f(w, std::integral_constant<int, 8>());
    if (MAXB >= 4)
        for (; w + 4 <= W; w += 4) f(w, std::integral_constant<int, 4>());
    if (MAXB >= 2)
        for (; w + 2 <= W; w += 2) f(w, std::integral_constant<int, 2>());
    for (; w < W; w++) f(w, std::integral_constant<int, 1>());
}

// Where a lane's groups sit inside a chunk of the vectorised path.
struct LaneMap {
    int lg;          // log2(lanes per bucket)
    int bi;          // bucket of this lane within the chunk
    int lp;          // lane within the bucket
    int row;         // elements between a lane's groups = bucket / G
    int e_lane;      // first element of the lane's group 0, relative to the chunk
    __device__ __forceinline__ LaneMap(const Tile &tile, int bucket, int lane)
    {
        lg = int(tile_lpb_log2(tile));
        bi = lane >> lg;
        lp = lane & ((1 << lg) - 1);
        row = 8 << lg;
        e_lane = bi * bucket + lp * 8;
    }
    __device__ __forceinline__ int group(int r) const { return e_lane + r * row; }
};

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

template <int SCHEME, int DT, int BITS, bool ODD>
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
#pragma unroll
        for (int r = 0; r < G; r++) load8<DT>(grad, first + map.group(r), x[r]);
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

// The short end of a layer (fewer elements than a chunk, whole buckets and possibly a ragged last
// one) goes through the chunk code with the missing elements masked.
struct TailShape {
    int count;       // elements of the tile
    int buckets;     // its buckets (the last one may be short)
    int nvecs;       // 16-byte vectors of its packed bytes (the layer's zero padding included)
    template <int BITS>
    __device__ __forceinline__ static TailShape of(const Tile &tile, int bucket)
    {
        TailShape t;
        t.count = int(tile.count);
        t.buckets = (t.count + bucket - 1) / bucket;
        t.nvecs = ((t.count * BITS + 7) / 8 + 15) / 16;
        return t;
    }
    // how many of the 8 elements of the group that starts at chunk element e exist
    __device__ __forceinline__ int valid(int e) const { return count - e >= 8 ? 8 : count - e > 0 ? count - e : 0; }
};

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

// Runs CALL with BITS = bits as a constant (kNormSign has no 1-bit codes: the entry points
// reject such plans, and nothing is instantiated for them).
#define CGX_FOR_BITS(bits, CALL)                      \
    switch (bits) {                                   \
    case 1: { constexpr int BITS = 1; if constexpr (SCHEME != kNormSign) { CALL; } } break;  \
    case 2: { constexpr int BITS = 2; CALL; } break;  \
    case 3: { constexpr int BITS = 3; CALL; } break;  \
    case 4: { constexpr int BITS = 4; CALL; } break;  \
    case 5: { constexpr int BITS = 5; CALL; } break;  \
    case 6: { constexpr int BITS = 6; CALL; } break;  \
    case 7: { constexpr int BITS = 7; CALL; } break;  \
    default: { constexpr int BITS = 8; CALL; } break; \
    }

// MAP: how the vectorised tiles of the plan are laid over the lanes, fixed by the call's bucket
// size: kMapBuckets for 128..2048 (bucket-major), kMapRows for 32 and 64 (row by row; needs more
// registers, so a kernel of its own keeps the others' occupancy), kMapWide for 4096 and 8192
// (a tile is one bucket of several chunks).
enum LaneMapping { kMapBuckets = 0, kMapRows = 1, kMapWide = 2 };

inline int mapping_of(int bucket) { return bucket <= 64 ? kMapRows : bucket > kChunk ? kMapWide : kMapBuckets; }

// ODD: some vectorised tile of the plan starts on an odd element index (see encode_group).
template <int SCHEME, int DT, int MAP, bool ODD>
__global__ __launch_bounds__(kBlock) void quantize_kernel(const void *__restrict__ grad,
                                                           const Tile *__restrict__ tiles, int64_t n_tiles,
                                                           int bucket, uint32_t seed_lo, uint32_t seed_hi,
                                                           uint8_t *__restrict__ packed,
                                                           float *__restrict__ meta)
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
        if (is_vector_kind(kind)) {
            if constexpr (MAP == kMapRows) {
                CGX_FOR_BITS(tile_bits(tile), (quantize_fast_rows<SCHEME, DT, BITS, ODD>(grad, packed, meta, tile, bucket,
                                                                                      seed_lo, seed_hi, lane, stage)))
            } else if constexpr (MAP == kMapWide) {
                CGX_FOR_BITS(tile_bits(tile), (quantize_wide<SCHEME, DT, BITS, ODD>(grad, packed, meta, tile, bucket,
                                                                                 seed_lo, seed_hi, lane, stage)))
            } else {
                CGX_FOR_BITS(tile_bits(tile), (quantize_fast<SCHEME, DT, BITS, ODD>(grad, packed, meta, tile, bucket,
                                                                                 seed_lo, seed_hi, lane, stage)))
            }
        } else if (kind == kQuantTail) {
            CGX_FOR_BITS(tile_bits(tile), (quantize_tail<SCHEME, DT, BITS, ODD>(grad, packed, meta, tile, bucket,
                                                                                  seed_lo, seed_hi, lane, stage)))
        } else if (kind == kQuantSlow) {
            quantize_generic<SCHEME, true>([&](uint32_t j) { return load_elem<DT>(grad, tile.elem0 + j); },
                                           packed + tile.packed_off, meta, tile, tile.pad, bucket, seed_lo,
                                           seed_hi, lane);
        } else {
            copy_tile<DT>(grad, packed, tile, kind == kCopyFast, lane);
        }
    }
}

// ---------------------------------------------------------------- dequantize + reduce

// Levels of one group of 8 codes as floats (kNormSign: signed levels).
template <int SCHEME, int BITS>
__device__ __forceinline__ void codes_to_float(uint64_t v, float (&f)[8])
{
    if (SCHEME == kNormSign) {
        if (BITS == 8) {
            const uint32_t lo = uint32_t(v), hi = uint32_t(v >> 32);
#pragma unroll
            for (int j = 0; j < 4; j++) {
                f[j] = float(int32_t(int8_t(lo >> (8 * j))));
                f[4 + j] = float(int32_t(int8_t(hi >> (8 * j))));
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; j++)      // sign-extending field extract
                f[j] = float(int32_t(uint32_t(v >> (j * BITS)) << (32 - BITS)) >> (32 - BITS));
        }
    } else if (BITS == 8) {
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

// Folds peers w0 .. w0+WB-1 into acc.  Each peer's share of the chunk (kChunk*BITS/8 bytes)
// is fetched as whole 16-byte vectors, consecutive across lanes, directly into the wave's
// LDS staging area, and read back by the lanes that own the codes.
// TAIL: the chunk is the short end of a layer; only its first nvecs 16-byte vectors exist in the
// packed streams (what lies behind them in LDS is stale, and so are the sums of elements past
// the end: the caller drops them).
template <int SCHEME, int BITS, int WB, bool TAIL, typename Peers>
__device__ __forceinline__ void reduce_peers(Peers &peers, int w0, int64_t in_off, uint32_t g,
                                             const int (&code_off)[G], float (&acc)[G][8], uint4v *stage,
                                             int lane, int nvecs)
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
            if (TAIL ? v < nvecs : (kVecs % kWave == 0 || v < kVecs)) load_to_lds16(in + v, stage + i * kVecs + k * kWave);
        }
        m[i] = load_meta<SCHEME>(peers.meta[w0 + i], g);
    }
    wait_vector_memory();
    wave_lds_fence();
    const uint8_t *codes = reinterpret_cast<const uint8_t *>(stage);
#pragma unroll
    for (int i = 0; i < WB; i++) {
#pragma unroll
        for (int r = 0; r < G; r++) {
            float f[8];
            codes_to_float<SCHEME, BITS>(staged_codes<BITS>(codes + i * kBytes, code_off[r]), f);
#pragma unroll
            for (int j = 0; j < 8; j++) acc[r][j] = __fadd_rn(acc[r][j], decode<SCHEME>(f[j], m[i]));
        }
        // keep the scheduler from hoisting every peer's LDS reads to the top (registers)
        if (i % 2 == 1) __builtin_amdgcn_sched_barrier(0);
    }
    wave_lds_fence();
}

// Sum over the W peers of one chunk's dequantized values, added to acc in peer order.
template <int SCHEME, int BITS, bool TAIL = false, typename Peers>
__device__ __forceinline__ void reduce_chunk(Peers &peers, int W, int64_t in_off, uint32_t g,
                                             const LaneMap &map, float (&acc)[G][8], uint4v *stage, int lane,
                                             int nvecs = 0)
{
    // peers staged together: 8 if their packed bytes fit the staging area (one chunk of sums,
    // kChunk * 4 bytes), else 4; the odd widths take 4 (their two or three dwords per group
    // and peer are all in flight together: at 8 peers the 3-bit path alone raised the fused
    // kernel from 106 to 125 registers, which cost every other width up to 50 % there)
    constexpr int kBytes = kChunk * BITS / 8;
    constexpr bool kOddWidth = kStagedOverRead<BITS> != 0;
    constexpr int kWide = (kOddWidth || 8 * kBytes > kChunk * 4) ? 4 : 8;
    static_assert(kWide * kBytes + kStagedOverRead<BITS> <= kChunk * 4, "staging area too small");
    int code_off[G];
#pragma unroll
    for (int r = 0; r < G; r++) code_off[r] = (map.group(r) >> 3) * BITS;
    for_peer_blocks<kWide>(W, [&](int w0, auto wb) {
        reduce_peers<SCHEME, BITS, decltype(wb)::value, TAIL>(peers, w0, in_off, g, code_off, acc, stage, lane, nvecs);
    });
}

// -0 is the identity of binary32 addition for every addend, signed zeros included, so
// the first peer's value enters the sum unchanged.
__device__ __forceinline__ void clear_sums(float (&acc)[G][8])
{
#pragma unroll
    for (int r = 0; r < G; r++)
#pragma unroll
        for (int j = 0; j < 8; j++) acc[r][j] = -0.0f;
}

// What a reduction starts from and where it goes: element e of the tile's buffer is
// init[e] (binary32 or binary16; init == nullptr: nothing) and is written to out[e]
// (binary32, or binary16 rounded to nearest even).
struct SumIo {
    const void *init;
    int init_dt;
    void *out;
    int out_dt;
};

__device__ __forceinline__ void init8(const SumIo &io, int64_t e, float (&acc)[8])
{
    if (!io.init) {
#pragma unroll
        for (int j = 0; j < 8; j++) acc[j] = -0.0f;
    } else if (io.init_dt == CGX_F16) {
        load8<CGX_F16>(io.init, e, acc);
    } else {
        load8<CGX_F32>(io.init, e, acc);
    }
}

__device__ __forceinline__ float init1(const SumIo &io, int64_t e)
{
    if (!io.init) return -0.0f;
    return io.init_dt == CGX_F16 ? load_elem<CGX_F16>(io.init, e) : load_elem<CGX_F32>(io.init, e);
}

__device__ __forceinline__ void store1(const SumIo &io, int64_t e, float v)
{
    if (io.out_dt == CGX_F16)
        reinterpret_cast<_Float16 *>(io.out)[e] = _Float16(v);
    else
        reinterpret_cast<float *>(io.out)[e] = v;
}

// 8 consecutive results to a 16-byte aligned position.
__device__ __forceinline__ void store8(const SumIo &io, int64_t e, const float (&acc)[8])
{
    if (io.out_dt == CGX_F16) {
        half8v h;
#pragma unroll
        for (int j = 0; j < 8; j++) h[j] = _Float16(acc[j]);
        *reinterpret_cast<half8u *>(reinterpret_cast<_Float16 *>(io.out) + e) = h;
    } else {
        float4u *p = reinterpret_cast<float4u *>(reinterpret_cast<float *>(io.out) + e);
        p[0] = float4v{acc[0], acc[1], acc[2], acc[3]};
        p[1] = float4v{acc[4], acc[5], acc[6], acc[7]};
    }
}

template <int SCHEME, int BITS, typename Peers>
__device__ __forceinline__ void reduce_fast(Peers &peers, int W, const SumIo &io, const Tile &tile,
                                            int bucket, int lane, uint4v *stage)
{
    const LaneMap map(tile, bucket, lane);
    const int chunks = int(tile.count / kChunk);
    const int buckets_per_chunk = kChunk / bucket;
    for (int c = 0; c < chunks; c++) {
        const int64_t first = tile.elem0 + int64_t(c) * kChunk;
        float acc[G][8];
#pragma unroll
        for (int r = 0; r < G; r++) init8(io, first + map.group(r), acc[r]);
        reduce_chunk<SCHEME, BITS>(peers, W, tile.packed_off + int64_t(c) * (kChunk * BITS / 8),
                                   tile.bucket0 + c * buckets_per_chunk + map.bi, map, acc, stage, lane);
        // the results leave through LDS as well, so that every store instruction writes 1 KB of
        // consecutive addresses
        if (io.out_dt == CGX_F16) {
#pragma unroll
            for (int r = 0; r < G; r++) {
                half8v h;
#pragma unroll
                for (int j = 0; j < 8; j++) h[j] = _Float16(acc[r][j]);
                reinterpret_cast<half8v *>(stage)[map.group(r) >> 3] = h;
            }
            wave_lds_fence();
            flush_stage_to_elements(stage, reinterpret_cast<uint4u2 *>(reinterpret_cast<_Float16 *>(io.out) + first),
                                    kChunk / 8, lane);
        } else {
#pragma unroll
            for (int r = 0; r < G; r++) {
                float4v *p = reinterpret_cast<float4v *>(stage) + (map.group(r) >> 2);
                p[0] = float4v{acc[r][0], acc[r][1], acc[r][2], acc[r][3]};
                p[1] = float4v{acc[r][4], acc[r][5], acc[r][6], acc[r][7]};
            }
            wave_lds_fence();
            flush_stage_to_elements(stage, reinterpret_cast<uint4u2 *>(reinterpret_cast<float *>(io.out) + first),
                                    kChunk / 4, lane);
        }
        wave_lds_fence();
    }
}

// Sums of the short end of a layer, in the chunk mapping: acc[r][j] is valid for j < valid(group r).
template <int SCHEME, int BITS, typename Peers>
__device__ __forceinline__ void reduce_tail_regs(Peers &peers, int W, const Tile &tile,
                                                 const TailShape &shape, const LaneMap &map, float (&acc)[G][8],
                                                 uint4v *stage, int lane)
{
    // lanes past the last bucket read its meta (and produce sums nobody uses)
    const int bi = map.bi < shape.buckets ? map.bi : shape.buckets - 1;
    reduce_chunk<SCHEME, BITS, true>(peers, W, tile.packed_off, tile.bucket0 + uint32_t(bi), map, acc, stage, lane,
                                     shape.nvecs);
}

// Start values come in and sums go out through the staging area, element by element over the
// elements that exist (coalesced; light on registers).
template <int SCHEME, int BITS, typename Peers>
__device__ __forceinline__ void reduce_tail(Peers &peers, int W, const SumIo &io, const Tile &tile,
                                            int bucket, int lane, uint4v *stage)
{
    const LaneMap map(tile, bucket, lane);
    const TailShape shape = TailShape::of<BITS>(tile, bucket);
    float *staged = reinterpret_cast<float *>(stage);
    for (int e = lane; e < kChunk; e += kWave) staged[e] = e < shape.count ? init1(io, tile.elem0 + e) : -0.0f;
    wave_lds_fence();
    float acc[G][8];
#pragma unroll
    for (int r = 0; r < G; r++) {
        const float4v *p = reinterpret_cast<const float4v *>(staged + map.group(r));
        const float4v a = p[0], b = p[1];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            acc[r][j] = a[j];
            acc[r][4 + j] = b[j];
        }
    }
    wave_lds_fence();
    reduce_tail_regs<SCHEME, BITS>(peers, W, tile, shape, map, acc, stage, lane);
#pragma unroll
    for (int r = 0; r < G; r++) {
        float4v *p = reinterpret_cast<float4v *>(staged + map.group(r));
        p[0] = float4v{acc[r][0], acc[r][1], acc[r][2], acc[r][3]};
        p[1] = float4v{acc[r][4], acc[r][5], acc[r][6], acc[r][7]};
    }
    wave_lds_fence();
    for (int e = lane; e < shape.count; e += kWave) store1(io, tile.elem0 + e, staged[e]);
    wave_lds_fence();
}

// Ordered sum over the peers of element j of a generic quantized tile (start = the value
// the sum starts from).
template <int SCHEME, typename Peers>
__device__ __forceinline__ float generic_sum(Peers &peers, int W, const Tile &tile, int bucket,
                                             uint32_t j, float start)
{
    const int b = int(tile_bits(tile));
    const uint32_t mask = (1u << b) - 1u;
    const uint32_t g = tile.bucket0 + j / uint32_t(bucket);
    const uint64_t bit = uint64_t(j) * b;
    const int64_t at = tile.packed_off + int64_t(bit >> 3);
    const uint32_t shift = uint32_t(bit & 7);
    const bool two = shift + b > 8;                  // a code spans at most two bytes
    float acc = start;
    for_peer_blocks<8>(W, [&](int w0, auto wb) {
        constexpr int WB = decltype(wb)::value;
        uint32_t lo[WB], hi[WB];
        float2 m[WB];
#pragma unroll
        for (int i = 0; i < WB; i++) {
            const uint8_t *p = peers.packed[w0 + i] + at;
            lo[i] = p[0];
            hi[i] = two ? p[1] : 0u;
            m[i] = load_meta<SCHEME>(peers.meta[w0 + i], g);
        }
#pragma unroll
        for (int i = 0; i < WB; i++) {
            const uint32_t code = ((lo[i] | (hi[i] << 8)) >> shift) & mask;
            const float level = SCHEME == kNormSign ? float(int32_t(code << (32 - b)) >> (32 - b)) : float(code);
            acc = __fadd_rn(acc, decode<SCHEME>(level, m[i]));
        }
    });
    return acc;
}

// Any bucket size, any alignment, ragged tiles: one element per lane and pass.
template <int SCHEME, typename Peers>
__device__ void reduce_slow(Peers &peers, int W, const SumIo &io, const Tile &tile, int bucket, int lane)
{
    for (uint32_t j = lane; j < tile.count; j += kWave)
        store1(io, tile.elem0 + j, generic_sum<SCHEME>(peers, W, tile, bucket, j, init1(io, tile.elem0 + j)));
}

// Ordered sum over the peers of 8 consecutive elements of a pass-through tile (16-byte
// aligned) and of a single element.
template <int DT, typename Peers>
__device__ __forceinline__ void copy_sum8(Peers &peers, int W, const Tile &tile, uint32_t g,
                                          float (&acc)[8])
{
    for_peer_blocks<8>(W, [&](int w0, auto wb) {
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
}

template <int DT, typename Peers>
__device__ __forceinline__ float copy_sum1(Peers &peers, int W, const Tile &tile, uint32_t j, float start)
{
    float acc = start;
    for_peer_blocks<8>(W, [&](int w0, auto wb) {
        constexpr int WB = decltype(wb)::value;
        float x[WB];
#pragma unroll
        for (int i = 0; i < WB; i++) x[i] = load_elem<DT>(peers.packed[w0 + i] + tile.packed_off, j);
#pragma unroll
        for (int i = 0; i < WB; i++) acc = __fadd_rn(acc, x[i]);
    });
    return acc;
}

// Pass-through tile of the reduce kernels: plain ordered sum of the stored values; element j
// of the tile starts from / goes to position e0 + j of io.
template <int DT, typename Peers>
__device__ void reduce_copy(Peers &peers, int W, const SumIo &io, int64_t e0, const Tile &tile, bool fast,
                            int lane)
{
    const uint32_t groups = fast ? tile.count / 8 : 0;
    for (uint32_t g = lane; g < groups; g += kWave) {
        float acc[8];
        init8(io, e0 + int64_t(g) * 8, acc);
        copy_sum8<DT>(peers, W, tile, g, acc);
        store8(io, e0 + int64_t(g) * 8, acc);
    }
    for (uint32_t j = groups * 8 + lane; j < tile.count; j += kWave)
        store1(io, e0 + j, copy_sum1<DT>(peers, W, tile, j, init1(io, e0 + j)));
}

// TAILS: the short ends of layers take the masked chunk path.  That path costs the kernel one
// register too many for its occupancy (and fencing it in by attribute cost 9 % on one of the
// benchmark plans), so the host asks for it only where short ends are a real share of the work;
// elsewhere the few there are go through the generic path, overlapped with everything else.
template <int SCHEME, bool TAILS>
__global__ __launch_bounds__(kBlock) void reduce_kernel(const PeerPtrs peers_argument, int W, int dt, const SumIo io,
                                                         const Tile *__restrict__ tiles, int64_t n_tiles,
                                                         int bucket)
{
    // the vectorised tiles index the table with constants (it then sits in scalar registers);
    // the other kinds index it at run time and read it from the kernarg segment
    const PeerPtrs &peers = peers_argument;
    KernargPeers &peers_in_memory = first_kernel_argument();
    // per-wave staging area: a chunk of binary32 results, or the packed bytes of a block of peers
    __shared__ uint4v stage_all[kWavesPerBlock][kChunk / 4];
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = int(threadIdx.x) & 63;
    uint4v *stage = stage_all[wave];
    const int64_t stride = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t t = int64_t(blockIdx.x) * kWavesPerBlock + wave; t < n_tiles; t += stride) {
        const Tile tile = tiles[t];
        const uint32_t kind = tile_kind(tile);
        if (is_vector_kind(kind)) {      // a wide tile is chunks of one bucket: kChunk / bucket == 0 below
            CGX_FOR_BITS(tile_bits(tile), (reduce_fast<SCHEME, BITS>(peers, W, io, tile, bucket, lane, stage)))
        } else if (TAILS && kind == kQuantTail) {
            if constexpr (TAILS) {
                CGX_FOR_BITS(tile_bits(tile),
                             (reduce_tail<SCHEME, BITS>(peers_in_memory, W, io, tile, bucket, lane, stage)))
            }
        } else if (kind == kQuantSlow || kind == kQuantTail) {
            reduce_slow<SCHEME>(peers_in_memory, W, io, tile, bucket, lane);
        } else if (dt == CGX_F16) {
            reduce_copy<CGX_F16>(peers_in_memory, W, io, tile.elem0, tile, kind == kCopyFast, lane);
        } else {
            reduce_copy<CGX_F32>(peers_in_memory, W, io, tile.elem0, tile, kind == kCopyFast, lane);
        }
    }
}

// ---------------------------------------------------------------- fused reduce + requantize

// The sums of a chunk never leave the registers: reduce_chunk feeds quantize_chunk.
template <int SCHEME, int BITS, bool ODD, typename Peers>
__device__ __forceinline__ void fused_fast(Peers &peers, int W, const Tile &tile, int64_t out_off,
                                           int bucket, uint32_t seed_lo, uint32_t seed_hi,
                                           uint8_t *__restrict__ packed_out, float *__restrict__ meta_out,
                                           int lane, uint4v *stage)
{
    const LaneMap map(tile, bucket, lane);
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    const int chunks = int(tile.count / kChunk);
    const int buckets_per_chunk = kChunk / bucket;
    for (int c = 0; c < chunks; c++) {
        float acc[G][8];
        clear_sums(acc);
        reduce_chunk<SCHEME, BITS>(peers, W, tile.packed_off + int64_t(c) * (kChunk * BITS / 8),
                                   tile.bucket0 + c * buckets_per_chunk + map.bi, map, acc, stage, lane);
        quantize_chunk<SCHEME, BITS, ODD>(acc, map, lane, tile.elem0 + int64_t(c) * kChunk, key,
                                     meta_out + kMetaFloats<SCHEME> * (tile.bucket0 + c * buckets_per_chunk),
                                     packed_out + out_off + int64_t(c) * (kChunk * BITS / 8), stage);
    }
}

// A tile that is one whole bucket of 2 or 4 chunks: the sums are formed twice, once for the
// scale and once for the codes (they would not fit the registers, and the chunks' bytes come
// from the caches the second time).
template <int SCHEME, int BITS, bool ODD, typename Peers>
__device__ __forceinline__ void fused_wide(Peers &peers, int W, const Tile &tile, int64_t out_off,
                                           int bucket, uint32_t seed_lo, uint32_t seed_hi,
                                           uint8_t *__restrict__ packed_out, float *__restrict__ meta_out,
                                           int lane, uint4v *stage)
{
    constexpr uint32_t kLevels = top_level<SCHEME>(BITS);
    const LaneMap map(tile, bucket, lane);
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    const int chunks = int(tile.count / kChunk);
    float mn = SCHEME == kNormSign ? 0.0f : __builtin_inff(), mx = SCHEME == kNormSign ? 0.0f : -__builtin_inff();
    Scale s{0.0f, 0.0f, 0.0f};
    // both passes in one loop, so that the reduction is instantiated once
    for (int it = 0; it < 2 * chunks; it++) {
        const bool second = it >= chunks;
        const int c = second ? it - chunks : it;
        float acc[G][8];
        clear_sums(acc);
        reduce_chunk<SCHEME, BITS>(peers, W, tile.packed_off + int64_t(c) * (kChunk * BITS / 8), tile.bucket0, map,
                                   acc, stage, lane);
        if (second) {
            encode_chunk<SCHEME, BITS, ODD>(acc, s, map, tile.elem0 + int64_t(c) * kChunk, key,
                                       packed_out + out_off + int64_t(c) * (kChunk * BITS / 8), stage, lane);
            continue;
        }
        lane_extent<SCHEME>(acc, mn, mx);
        if (c == chunks - 1) {
            if (SCHEME == kNormSign)
                group_max(mx, 6, lane);
            else
                group_minmax(mn, mx, 6, lane);
            s = bucket_scale(mn, mx, int(kLevels));
            if (lane == 0) store_meta<SCHEME>(meta_out, tile.bucket0, s);
        }
    }
}

// The short end of a layer: masked sums feed the masked quantizer.
template <int SCHEME, int BITS, bool ODD, typename Peers>
__device__ __forceinline__ void fused_tail(Peers &peers, int W, const Tile &tile, int64_t out_off, int bucket,
                                           uint32_t seed_lo, uint32_t seed_hi, uint8_t *__restrict__ packed_out,
                                           float *__restrict__ meta_out, int lane, uint4v *stage)
{
    const LaneMap map(tile, bucket, lane);
    const TailShape shape = TailShape::of<BITS>(tile, bucket);
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    float acc[G][8];
    clear_sums(acc);
    reduce_tail_regs<SCHEME, BITS>(peers, W, tile, shape, map, acc, stage, lane);
#pragma unroll
    for (int r = 0; r < G; r++) {
        const int v = shape.valid(map.group(r));
#pragma unroll
        for (int j = 0; j < 8; j++)
            if (j >= v) acc[r][j] = 0.0f;            // stale LDS bytes decoded to anything
    }
    quantize_tail_regs<SCHEME, BITS, ODD>(acc, shape, map, lane, tile.elem0, key,
                                          meta_out + kMetaFloats<SCHEME> * tile.bucket0, packed_out + out_off, stage);
}

// tiles_in follows the layout of the chunks (storage type dt), tiles_out that of the
// output (binary32 pass-through layers); the two tables list the same tiles in the same order.
// WIDE: the call's bucket is longer than a chunk (see quantize_kernel's MAP).
template <int SCHEME, bool WIDE, bool ODD>
__global__ __launch_bounds__(kBlock) void fused_kernel(const PeerPtrs peers_argument, int W, int dt,
                                                        const Tile *__restrict__ tiles_in,
                                                        const Tile *__restrict__ tiles_out, int64_t n_tiles,
                                                        int bucket, uint32_t seed_lo, uint32_t seed_hi,
                                                        uint8_t *__restrict__ packed_out,
                                                        float *__restrict__ meta_out)
{
    (void)peers_argument;
    KernargPeers &peers = first_kernel_argument();
    __shared__ uint4v stage_all[kWavesPerBlock][kChunk / 4];
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = int(threadIdx.x) & 63;
    uint4v *stage = stage_all[wave];
    const int64_t stride = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t t = int64_t(blockIdx.x) * kWavesPerBlock + wave; t < n_tiles; t += stride) {
        const Tile tile = tiles_in[t];
        const int64_t out_off = tiles_out[t].packed_off;
        const uint32_t out_pad = tiles_out[t].pad;
        const uint32_t kind = tile_kind(tile);
        if (is_vector_kind(kind)) {
            if constexpr (WIDE) {
                CGX_FOR_BITS(tile_bits(tile), (fused_wide<SCHEME, BITS, ODD>(peers, W, tile, out_off, bucket, seed_lo,
                                                                         seed_hi, packed_out, meta_out, lane, stage)))
            } else {
                CGX_FOR_BITS(tile_bits(tile), (fused_fast<SCHEME, BITS, ODD>(peers, W, tile, out_off, bucket, seed_lo,
                                                                         seed_hi, packed_out, meta_out, lane, stage)))
            }
        } else if (kind == kQuantTail) {
            CGX_FOR_BITS(tile_bits(tile), (fused_tail<SCHEME, BITS, ODD>(peers, W, tile, out_off, bucket, seed_lo,
                                                                         seed_hi, packed_out, meta_out, lane, stage)))
        } else if (kind == kQuantSlow) {
            quantize_generic<SCHEME, false>(
                [&](uint32_t j) { return generic_sum<SCHEME>(peers, W, tile, bucket, j, -0.0f); },
                packed_out + out_off, meta_out, tile, out_pad, bucket, seed_lo, seed_hi, lane);
        } else {
            // pass-through: the sum is written as binary32 into the output stream, then its padding
            const SumIo io{nullptr, CGX_F32, packed_out + out_off, CGX_F32};
            if (dt == CGX_F16)
                reduce_copy<CGX_F16>(peers, W, io, 0, tile, kind == kCopyFast, lane);
            else
                reduce_copy<CGX_F32>(peers, W, io, 0, tile, kind == kCopyFast, lane);
            uint8_t *end = packed_out + out_off + uint64_t(tile.count) * 4;
            if (uint32_t(lane) < out_pad) end[lane] = 0;
        }
    }
}

// ---------------------------------------------------------------- per-layer statistics
//
// Squared l2 norms per layer (of a buffer, or of the compression error x - value(code)) for
// the layer-wise adaptive scheme (paper Sec. "Layer-wise Adaptive Quantization").  Two
// launches: one wave per tile leaves a binary64 partial sum in partial[slot of the tile]; then
// one wave per layer adds the layer's partials.  No atomics, so a result does not depend on
// the order in which waves finish.  Squares of binary32 values and differences of two
// binary32 values are exact in binary64; only the additions round.

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

__device__ __forceinline__ double square(float x)
{
    const double d = double(x);
    return d * d;
}

// Sum of squares of a run of elements of the buffer (tile of a pass-through plan).
template <int DT>
__device__ __forceinline__ double sqnorm_tile(const void *__restrict__ buf, const Tile &tile, bool fast, int lane)
{
    double s = 0.0;
    const uint32_t groups = fast ? tile.count / 8 : 0;
    for (uint32_t g0 = 0; g0 < groups; g0 += 4 * kWave) {
        Raw8<DT> raw[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const uint32_t g = g0 + u * kWave + lane;
            raw[u].load(buf, tile.elem0 + int64_t(g < groups ? g : g0) * 8);    // clamped; masked below
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            float x[8];
            raw[u].widen(x);
            if (g0 + u * kWave + lane < groups) {
#pragma unroll
                for (int j = 0; j < 8; j++) s += square(x[j]);
            }
        }
    }
    for (uint32_t j = groups * 8 + lane; j < tile.count; j += kWave) s += square(load_elem<DT>(buf, tile.elem0 + j));
    return s;
}

template <int DT>
__global__ __launch_bounds__(kBlock) void sqnorm_kernel(const void *__restrict__ buf,
                                                         const Tile *__restrict__ tiles,
                                                         const uint32_t *__restrict__ slots, int64_t n_tiles,
                                                         double *__restrict__ partial)
{
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = int(threadIdx.x) & 63;
    const int64_t stride = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t t = int64_t(blockIdx.x) * kWavesPerBlock + wave; t < n_tiles; t += stride) {
        const Tile tile = tiles[t];
        const double s = wave_sum(sqnorm_tile<DT>(buf, tile, tile_kind(tile) == kCopyFast, lane));
        if (lane == 0) partial[slots[t]] = s;
    }
}

// Squared error of a vectorised tile: the codes are decoded as in the reduce (one peer) and
// compared with the gradient they were cut from.
template <int SCHEME, int DT, int BITS, typename Peers>
__device__ __forceinline__ double sqerror_fast(const void *__restrict__ grad, Peers &chunk,
                                               const Tile &tile, int bucket, int lane, uint4v *stage)
{
    const LaneMap map(tile, bucket, lane);
    const int chunks = int(tile.count / kChunk);
    const int buckets_per_chunk = kChunk / bucket;
    double s = 0.0;
    for (int c = 0; c < chunks; c++) {
        const int64_t first = tile.elem0 + int64_t(c) * kChunk;
        float x[G][8], v[G][8];
#pragma unroll
        for (int r = 0; r < G; r++) load8<DT>(grad, first + map.group(r), x[r]);
        clear_sums(v);
        reduce_chunk<SCHEME, BITS>(chunk, 1, tile.packed_off + int64_t(c) * (kChunk * BITS / 8),
                                   tile.bucket0 + c * buckets_per_chunk + map.bi, map, v, stage, lane);
#pragma unroll
        for (int r = 0; r < G; r++)
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const double d = double(x[r][j]) - double(v[r][j]);
                s += d * d;
            }
    }
    return s;
}

template <int SCHEME, int DT>
__global__ __launch_bounds__(kBlock) void sqerror_kernel(const PeerPtrs chunk_argument, const void *__restrict__ grad,
                                                          const Tile *__restrict__ tiles,
                                                          const uint32_t *__restrict__ slots, int64_t n_tiles,
                                                          int bucket, double *__restrict__ partial)
{
    (void)chunk_argument;
    KernargPeers &chunk = first_kernel_argument();
    __shared__ uint4v stage_all[kWavesPerBlock][kChunk / 4];
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = int(threadIdx.x) & 63;
    uint4v *stage = stage_all[wave];
    const int64_t stride = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t t = int64_t(blockIdx.x) * kWavesPerBlock + wave; t < n_tiles; t += stride) {
        const Tile tile = tiles[t];
        const uint32_t kind = tile_kind(tile);
        double s = 0.0;                              // pass-through tiles: no error
        if (is_vector_kind(kind)) {
            CGX_FOR_BITS(tile_bits(tile), (s = sqerror_fast<SCHEME, DT, BITS>(grad, chunk, tile, bucket, lane, stage)))
        } else if (kind == kQuantSlow || kind == kQuantTail) {
            for (uint32_t j = lane; j < tile.count; j += kWave) {
                const double d = double(load_elem<DT>(grad, tile.elem0 + j)) -
                                 double(generic_sum<SCHEME>(chunk, 1, tile, bucket, j, -0.0f));
                s += d * d;
            }
        }
        s = wave_sum(s);
        if (lane == 0) partial[slots[t]] = s;
    }
}

// out[l] = sum of the partials of layer l, numbers layer_first[l] .. layer_first[l + 1] - 1.
// One block per layer: the largest layers own tens of thousands of partials, so the loads are
// spread over 16 waves and issued four at a time; the order of the additions is fixed.
constexpr int kSumBlock = 1024;

__global__ __launch_bounds__(kSumBlock) void layer_sum_kernel(const double *__restrict__ partial,
                                                               const int64_t *__restrict__ layer_first,
                                                               double *__restrict__ out)
{
    __shared__ double wave_part[kSumBlock / kWave];
    const int64_t l = blockIdx.x;
    const int tid = int(threadIdx.x), lane = tid & 63, wave = tid >> 6;
    const int64_t a = layer_first[l], b = layer_first[l + 1];
    double s = 0.0;
    for (int64_t i0 = a; i0 < b; i0 += 4 * kSumBlock) {
        double v[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int64_t i = i0 + u * kSumBlock + tid;
            v[u] = i < b ? partial[i] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < 4; u++) s += v[u];
    }
    s = wave_sum(s);
    if (lane == 0) wave_part[wave] = s;
    __syncthreads();
    if (wave == 0) {
        const double t = wave_sum(lane < kSumBlock / kWave ? wave_part[lane] : 0.0);
        if (lane == 0) out[l] = t;
    }
}

// ---------------------------------------------------------------- streaming probe

// Measurement aid: moves read_bytes in and write_bytes out with the access style of the
// kernels above (one wave per slice, lane-contiguous non-temporal 16-byte vectors) and no
// arithmetic to speak of.  Its rate is what the memory system gives a kernel with that
// read:write mix at that size.
__global__ __launch_bounds__(kBlock) void stream_probe_kernel(const uint4v *__restrict__ src, int64_t read_vecs,
                                                               uint4v *__restrict__ dst, int64_t write_vecs,
                                                               int64_t waves)
{
    const int64_t wave = int64_t(blockIdx.x) * kWavesPerBlock + (int(threadIdx.x) >> 6);
    const int lane = int(threadIdx.x) & 63;
    if (wave >= waves) return;
    const int64_t r0 = read_vecs * wave / waves, r1 = read_vecs * (wave + 1) / waves;
    const int64_t w0 = write_vecs * wave / waves, w1 = write_vecs * (wave + 1) / waves;
    uint4v acc = {0u, 0u, 0u, 0u};
    for (int64_t v = r0 + lane; v < r1; v += 8 * kWave) {
        uint4v x[8];
#pragma unroll
        for (int u = 0; u < 8; u++) {
            const int64_t i = v + u * kWave;
            x[u] = i < r1 ? stream_load(src + i) : uint4v{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < 8; u++) acc += x[u];
    }
    for (int64_t v = w0 + lane; v < w1; v += kWave) stream_store(dst + v, acc + uint32_t(v));
}

inline unsigned grid_for(int64_t n_tiles, const LaunchConfig &cfg)
{
    int64_t blocks = (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (cfg.max_blocks > 0 && blocks > cfg.max_blocks) blocks = cfg.max_blocks;
    if (blocks > 0x7fffffff) blocks = 0x7fffffff;
    return unsigned(blocks);
}

}  // namespace

hipError_t launch_quantize(int scheme, const void *grad, int dt, const Tile *tiles, int64_t n_tiles, bool odd_tiles,
                           int32_t bucket, uint64_t seed, void *packed, void *meta, const LaunchConfig &cfg,
                           hipStream_t stream)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(grid_for(n_tiles, cfg)), block(kBlock);
    const uint32_t seed_lo = uint32_t(seed), seed_hi = uint32_t(seed >> 32);
    using Kernel = void (*)(const void *, const Tile *, int64_t, int, uint32_t, uint32_t, uint8_t *, float *);
#define CGX_QUANTIZE_MAPS(S, D, O) \
    {quantize_kernel<S, D, kMapBuckets, O>, quantize_kernel<S, D, kMapRows, O>, quantize_kernel<S, D, kMapWide, O>}
    static const Kernel table[2][2][2][3] = {
        {{CGX_QUANTIZE_MAPS(kMinMax, CGX_F32, false), CGX_QUANTIZE_MAPS(kMinMax, CGX_F16, false)},
         {CGX_QUANTIZE_MAPS(kNormSign, CGX_F32, false), CGX_QUANTIZE_MAPS(kNormSign, CGX_F16, false)}},
        {{CGX_QUANTIZE_MAPS(kMinMax, CGX_F32, true), CGX_QUANTIZE_MAPS(kMinMax, CGX_F16, true)},
         {CGX_QUANTIZE_MAPS(kNormSign, CGX_F32, true), CGX_QUANTIZE_MAPS(kNormSign, CGX_F16, true)}}};
#undef CGX_QUANTIZE_MAPS
    const Kernel kernel = table[odd_tiles][scheme == kSchemeNormSign][dt == CGX_F16][mapping_of(bucket)];
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, grad, tiles, n_tiles, int(bucket), seed_lo, seed_hi,
                       static_cast<uint8_t *>(packed), static_cast<float *>(meta));
    return hipGetLastError();
}

hipError_t launch_dequant_reduce(int scheme, const PeerPtrs &peers, int W, int dt, const Tile *tiles, int64_t n_tiles,
                                 bool many_tails,
                                 int32_t bucket, const void *init, int init_dt, void *out, int out_dt,
                                 const LaunchConfig &cfg, hipStream_t stream)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(grid_for(n_tiles, cfg)), block(kBlock);
    const SumIo io{init, init_dt, out, out_dt};
    const auto kernel = scheme == kSchemeNormSign
                            ? (many_tails ? reduce_kernel<kNormSign, true> : reduce_kernel<kNormSign, false>)
                            : (many_tails ? reduce_kernel<kMinMax, true> : reduce_kernel<kMinMax, false>);
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, peers, W, dt, io, tiles, n_tiles, int(bucket));
    return hipGetLastError();
}

hipError_t launch_dequant_reduce_requantize(int scheme, const PeerPtrs &peers, int W, int dt, const Tile *tiles_in,
                                            const Tile *tiles_out, int64_t n_tiles, bool odd_tiles, int32_t bucket,
                                            uint64_t seed, void *packed_out, void *meta_out,
                                            const LaunchConfig &cfg, hipStream_t stream)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(grid_for(n_tiles, cfg)), block(kBlock);
    const bool wide = mapping_of(bucket) == kMapWide;
    using Kernel = void (*)(const PeerPtrs, int, int, const Tile *, const Tile *, int64_t, int, uint32_t, uint32_t,
                            uint8_t *, float *);
    static const Kernel table[2][2][2] = {
        {{fused_kernel<kMinMax, false, false>, fused_kernel<kMinMax, true, false>},
         {fused_kernel<kNormSign, false, false>, fused_kernel<kNormSign, true, false>}},
        {{fused_kernel<kMinMax, false, true>, fused_kernel<kMinMax, true, true>},
         {fused_kernel<kNormSign, false, true>, fused_kernel<kNormSign, true, true>}}};
    const Kernel kernel = table[odd_tiles][scheme == kSchemeNormSign][wide];
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, peers, W, dt, tiles_in, tiles_out, n_tiles, int(bucket),
                       uint32_t(seed), uint32_t(seed >> 32), static_cast<uint8_t *>(packed_out),
                       static_cast<float *>(meta_out));
    return hipGetLastError();
}

hipError_t launch_layer_sqnorms(const void *buf, int dt, const Tile *tiles, const uint32_t *slots, int64_t n_tiles,
                                const int64_t *layer_first, int32_t L, double *partial, double *out,
                                const LaunchConfig &cfg, hipStream_t stream)
{
    if (L == 0) return hipSuccess;
    const dim3 block(kBlock);
    if (n_tiles > 0) {
        const dim3 grid(grid_for(n_tiles, cfg));
        const auto kernel = dt == CGX_F16 ? sqnorm_kernel<CGX_F16> : sqnorm_kernel<CGX_F32>;
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, buf, tiles, slots, n_tiles, partial);
    }
    hipLaunchKernelGGL(layer_sum_kernel, dim3(unsigned(L)), dim3(kSumBlock), 0, stream,
                       static_cast<const double *>(partial), layer_first, out);
    return hipGetLastError();
}

hipError_t launch_layer_sqerrors(int scheme, const void *grad, int dt, const void *packed, const void *meta,
                                 const Tile *tiles, const uint32_t *slots, int64_t n_tiles,
                                 const int64_t *layer_first, int32_t L, int32_t bucket, double *partial,
                                 double *out, const LaunchConfig &cfg, hipStream_t stream)
{
    if (L == 0) return hipSuccess;
    const dim3 block(kBlock);
    if (n_tiles > 0) {
        const dim3 grid(grid_for(n_tiles, cfg));
        PeerPtrs chunk{};
        chunk.packed[0] = static_cast<const uint8_t *>(packed);
        chunk.meta[0] = static_cast<const float *>(meta);
        const auto kernel =
            scheme == kSchemeNormSign
                ? (dt == CGX_F16 ? sqerror_kernel<kNormSign, CGX_F16> : sqerror_kernel<kNormSign, CGX_F32>)
                : (dt == CGX_F16 ? sqerror_kernel<kMinMax, CGX_F16> : sqerror_kernel<kMinMax, CGX_F32>);
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, chunk, grad, tiles, slots, n_tiles, int(bucket), partial);
    }
    hipLaunchKernelGGL(layer_sum_kernel, dim3(unsigned(L)), dim3(kSumBlock), 0, stream,
                       static_cast<const double *>(partial), layer_first, out);
    return hipGetLastError();
}

hipError_t launch_stream_probe(const void *src, size_t read_bytes, void *dst, size_t write_bytes, hipStream_t stream)
{
    const int64_t read_vecs = int64_t(read_bytes / 16), write_vecs = int64_t(write_bytes / 16);
    const int64_t larger = read_vecs > write_vecs ? read_vecs : write_vecs;
    const int64_t waves = (larger + 511) / 512;                 // 8 KB of the larger side per wave
    if (waves == 0) return hipSuccess;
    const dim3 grid(unsigned((waves + kWavesPerBlock - 1) / kWavesPerBlock)), block(kBlock);
    hipLaunchKernelGGL(stream_probe_kernel, grid, block, 0, stream, static_cast<const uint4v *>(src), read_vecs,
                       static_cast<uint4v *>(dst), write_vecs, waves);
    return hipGetLastError();
}

}  // namespace cgx
