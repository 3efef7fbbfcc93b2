// Shared device code of the gfx950 kernels (included by the .hip files; everything here has
// internal linkage).
//
// The kernels: bucketed stochastic quantization of a fused gradient buffer (cgx_quantize.hip),
// dequantize-and-reduce of W compressed chunks (cgx_reduce.hip), the two fused into one pass
// (cgx_fused.hip), per-layer statistics and the streaming probe (cgx_stats.hip).
//
// One wavefront (64 lanes) owns one tile of the plan.  In the vectorised path a
// wave takes a chunk of kChunk elements per pass: each lane holds kGroups groups
// of 8 consecutive elements, all of the same bucket (a bucket of B elements
// spans B / (8 kGroups) neighbouring lanes).  kGroups is fixed per translation unit
// (CGX_GROUPS: 4 unless the build says otherwise, i.e. chunks of 2048 elements; the
// binary32 quantizer is also built with 2), so
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
#pragma once

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

// The table when the parameter starts byte_offset bytes into the kernarg segment.  (The kernels are built
// with their first 16 dwords of arguments preloaded into scalar registers by the dispatcher, which
// spares every wave one dependent scalar load ahead of its tile descriptor; the arguments a wave needs
// first therefore come first and the 256-byte table last.)
__device__ __forceinline__ KernargPeers &kernel_argument_peers(size_t byte_offset)
{
    return *(KernargPeers *)((const __attribute__((address_space(4))) char *)__builtin_amdgcn_kernarg_segment_ptr() +
                             byte_offset);
}

#ifndef CGX_GROUPS
#define CGX_GROUPS 4
#endif
constexpr int kGroups = CGX_GROUPS;            // groups of 8 elements per lane and chunk
// (names of the launchers of files that are compiled once per chunk size)
#define CGX_CONCAT2(a, b) a##b
#define CGX_CONCAT(a, b) CGX_CONCAT2(a, b)
constexpr int kChunk = chunk_of(kGroups);      // elements a wave takes per pass of the vectorised path

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
typedef uint4v uint4u4 __attribute__((aligned(4)));

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

// The smaller / larger of two numbers as the instruction gives it.  fminf / fmaxf compile to the same
// instruction behind one more per operand that quiets a signalling NaN (a value that has crossed lanes
// as an integer is not known to be quiet): four of the eight instructions of a butterfly step.  The
// operands here are minima and maxima of the gradient; with a NaN among them the bucket's result is
// unspecified anyway.
__device__ __forceinline__ float min_plain(float a, float b)
{
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

__device__ __forceinline__ float max_plain(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// min / max of a lane's value and the value of its partner lane under one of the four lane patterns
// that stay within a row of 16, in one instruction (the partner's value is the first operand, fetched
// through the data-parallel-primitive path).  Such an operand must not have been written by the two
// vector instructions before it; the compiler does not look into this text, hence the s_nop.
#define CGX_DPP_EXCHANGE(NAME, OP, PATTERN)                                                            \
    __device__ __forceinline__ float NAME(float v)                                                     \
    {                                                                                                  \
        /* in place: a lane whose partner is switched off keeps its own value */                       \
        asm("s_nop 1\n\t" OP " %0, %0, %0 " PATTERN " row_mask:0xf bank_mask:0xf" : "+v"(v));         \
        return v;                                                                                      \
    }
CGX_DPP_EXCHANGE(min_xor1, "v_min_f32_dpp", "quad_perm:[1,0,3,2]")
CGX_DPP_EXCHANGE(max_xor1, "v_max_f32_dpp", "quad_perm:[1,0,3,2]")
CGX_DPP_EXCHANGE(min_xor2, "v_min_f32_dpp", "quad_perm:[2,3,0,1]")
CGX_DPP_EXCHANGE(max_xor2, "v_max_f32_dpp", "quad_perm:[2,3,0,1]")
CGX_DPP_EXCHANGE(min_half_mirror, "v_min_f32_dpp", "row_half_mirror")
CGX_DPP_EXCHANGE(max_half_mirror, "v_max_f32_dpp", "row_half_mirror")
CGX_DPP_EXCHANGE(min_mirror, "v_min_f32_dpp", "row_mirror")
CGX_DPP_EXCHANGE(max_mirror, "v_max_f32_dpp", "row_mirror")
#undef CGX_DPP_EXCHANGE

// Minimum and maximum over groups of 2^lg neighbouring lanes, result in every lane.  Every lane of the
// wave takes part (the callers are in wave-uniform control flow).
__device__ __forceinline__ void group_minmax(float &mn, float &mx, int lg, int lane)
{
    if (lg >= 1) {   // lane ^ 1
        mn = min_xor1(mn);
        mx = max_xor1(mx);
    }
    if (lg >= 2) {   // lane ^ 2
        mn = min_xor2(mn);
        mx = max_xor2(mx);
    }
    if (lg >= 3) {   // quads are uniform now: row_half_mirror pairs each quad with its neighbour
        mn = min_half_mirror(mn);
        mx = max_half_mirror(mx);
    }
    if (lg >= 4) {   // row_mirror pairs the two halves of a row of 16
        mn = min_mirror(mn);
        mx = max_mirror(mx);
    }
    if (lg >= 5) {
        mn = min_plain(mn, swizzle_xor16(mn));
        mx = max_plain(mx, swizzle_xor16(mx));
    }
    if (lg >= 6) {
        mn = min_plain(mn, permute_xor32(mn, lane));
        mx = max_plain(mx, permute_xor32(mx, lane));
    }
}

// Maximum alone, same exchange pattern.
__device__ __forceinline__ void group_max(float &mx, int lg, int lane)
{
    if (lg >= 1) mx = max_xor1(mx);
    if (lg >= 2) mx = max_xor2(mx);
    if (lg >= 3) mx = max_half_mirror(mx);
    if (lg >= 4) mx = max_mirror(mx);
    if (lg >= 5) mx = max_plain(mx, swizzle_xor16(mx));
    if (lg >= 6) mx = max_plain(mx, permute_xor32(mx, lane));
}

// ---------------------------------------------------------------- the two quantizers
//
// kMinMax: affine per bucket.  A b-bit code is a level 0..2^b-1 between the bucket's minimum
// and maximum; meta = {unit, minimum} (float2 per bucket); value = fma(level, unit, minimum).
// kNormSign: a variant of the norm-and-sign form Q_s printed in Sec. 2.3: the norm is the bucket's
// largest magnitude (l-infinity) where the paper prints the l2 norm.  A b-bit code (b >= 2) is sign(x) times a level 0..s,
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

// The same to an element-aligned destination (sums), with the cache policy (StorePolicy, cgx_kernels.h) the host
// chose for the call:
//   kStoreStream   non-temporal: results larger than the memory-side cache
//   kStoreKeep     written through at device scope (sc1).  Measured: a result of about 100 MB then
//                  stays in the 256 MB memory-side cache, the launch that writes it gets 7 % shorter and the
//                  one that reads it next 10 %; results of several hundred MB gain 3 % in the writer and
//                  lose 7 % in the reader, so the host asks for it only below a size (see reduce_impl)
//   kStoreThrough  written through at system scope, non-temporal (sc0 sc1 nt): for calls that write
//                  eight bytes per byte they read (cgx_dequantize).  An arithmetic-free kernel in that mix
//                  sustains 0.61 of the HBM peak with non-temporal loads and stores, 0.75 with ordinary
//                  loads and these stores (8 KB per wave), and 0.91 with 4 KB per wave
__device__ __forceinline__ void flush_stage_to_elements(const uint4v *stage, uint4u2 *dst, int vecs, int lane, int policy)
{
    if (policy == kStoreKeep) {
        for (int v = lane; v < vecs; v += kWave)
            asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(dst + v), "v"(stage[v]) : "memory");
    } else if (policy == kStoreThrough) {
        for (int v = lane; v < vecs; v += kWave)
            asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" : : "v"(dst + v), "v"(stage[v]) : "memory");
    } else {
        for (int v = lane; v < vecs; v += kWave) __builtin_nontemporal_store(stage[v], dst + v);
    }
}

// One 16-byte vector per lane from global memory straight into LDS, without passing
// through registers: lane l's vector lands at lds_base + 16 * l (lds_base is wave-uniform).
__device__ __forceinline__ void load_to_lds16(const uint4v *gptr, uint4v *lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gptr,
                                     (__attribute__((address_space(3))) void *)lds_base, 16, 0, 2 /* nt */);
}

// The same as an ordinary (cached) load: in a call that mostly writes, the few bytes it reads come
// in faster this way (see kStoreThrough).
__device__ __forceinline__ void load_to_lds16_cached(const uint4v *gptr, uint4v *lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gptr,
                                     (__attribute__((address_space(3))) void *)lds_base, 16, 0, 0);
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

// A tile of whole buckets of a size that is no power of two (kQuantAny): held row by row, group Gi = 64 r +
// lane of the tile's count / 8 groups of 8 elements is group r of lane `lane`; a bucket is bucket / 8
// consecutive groups.
struct AnyShape {
    int groups;      // groups of 8 elements in the tile
    int gb;          // groups per bucket
    int m;           // buckets in the tile (at most 21: the smallest such bucket is 96)
    uint32_t inv;    // ceil(2^16 / gb): (Gi * inv) >> 16 == Gi / gb for Gi < 256 and gb <= 256 (checked exhaustively)
    __device__ __forceinline__ AnyShape(const Tile &tile, int bucket)
    {
        groups = int(tile.count >> 3);
        gb = bucket >> 3;
        m = int(tile.count) / bucket;
        inv = (65536u + uint32_t(gb) - 1u) / uint32_t(gb);
    }
    __device__ __forceinline__ int bucket_of(int Gi) const { return int((uint32_t(Gi) * inv) >> 16); }
};

// One dword per lane from global memory straight into LDS: lane l's dword lands at lds_base + 4 * l.
__device__ __forceinline__ void load_to_lds4(const uint32_t *gptr, uint32_t *lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gptr,
                                     (__attribute__((address_space(3))) void *)lds_base, 4, 0, 2 /* nt */);
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

inline unsigned grid_for(int64_t n_tiles, const LaunchConfig &cfg)
{
    int64_t blocks = (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (cfg.max_blocks > 0 && blocks > cfg.max_blocks) blocks = cfg.max_blocks;
    if (blocks > 0x7fffffff) blocks = 0x7fffffff;
    return unsigned(blocks);
}

}  // namespace
}  // namespace cgx
