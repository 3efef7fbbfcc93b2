// Device code of the dequantize-and-reduce: decoding of staged codes, the peers' loop, sums of
// chunks, short ends, generic and pass-through tiles (shared by the reduce, fused and
// statistics kernels).
#pragma once

#include "cgx_device.h"

namespace cgx {
namespace {

// ---------------------------------------------------------------- dequantize + reduce

// Keeps a value opaque to the optimiser at no cost.  The byte-wise decoders below put one code
// into every byte of a register and convert the bytes with v_cvt_f32_ubyte0..3; seeing through
// the mask, the compiler would instead extract every code with a v_bfe_u32 of its own and
// convert byte 0 (two instructions of the slow issue class per code instead of one).
__device__ __forceinline__ uint32_t opaque(uint32_t v)
{
    asm("" : "+v"(v));
    return v;
}

// The four bytes of t as floats.
__device__ __forceinline__ void bytes_to_float(uint32_t t, float &b0, float &b1, float &b2, float &b3)
{
    b0 = float(t & 0xffu);
    b1 = float((t >> 8) & 0xffu);
    b2 = float((t >> 16) & 0xffu);
    b3 = float(t >> 24);
}

// Levels of one group of 8 codes as floats (kNormSign: signed levels).  Of the signed widths
// only 4 bits takes the byte-wise form: with 2 and 8 bits as well the reduce kernel needs 129
// to 131 registers, one wave per SIMD less.
template <int SCHEME, int BITS>
__device__ __forceinline__ void codes_to_float(uint64_t v, float (&f)[8])
{
    constexpr bool kSigned = SCHEME == kNormSign;
    if (BITS == 8 && !kSigned) {
        bytes_to_float(uint32_t(v), f[0], f[1], f[2], f[3]);
        bytes_to_float(uint32_t(v >> 32), f[4], f[5], f[6], f[7]);
    } else if (BITS == 4) {
        // one code per byte: even codes in one register, odd ones in another.  kSigned: a code is
        // a two's complement nibble; with its sign bit flipped it reads level + 8 in 1..15
        constexpr uint32_t kFlip = kSigned ? 0x88888888u : 0u;
        const uint32_t w = uint32_t(v) ^ kFlip;
        const uint32_t even = opaque(w & 0x0f0f0f0fu), odd = opaque((w >> 4) & 0x0f0f0f0fu);
        bytes_to_float(even, f[0], f[2], f[4], f[6]);
        bytes_to_float(odd, f[1], f[3], f[5], f[7]);
        if (kSigned) {
#pragma unroll
            for (int j = 0; j < 8; j++) f[j] -= 8.0f;
        }
    } else if (BITS == 2 && !kSigned) {
        const uint32_t w = uint32_t(v);
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const uint32_t t = opaque((w >> (2 * j)) & 0x0303u);     // codes j and j + 4, one per byte
            f[j] = float(t & 0xffu);
            f[4 + j] = float((t >> 8) & 0xffu);
        }
    } else if (kSigned) {
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
    } else {
        constexpr uint64_t kMask = (1u << BITS) - 1u;
#pragma unroll
        for (int j = 0; j < 8; j++) f[j] = float(uint32_t((v >> (j * BITS)) & kMask));
    }
}

// ---- two conversions per instruction (min/max codes of 2 and 4 bits)
//
// A code q <= 15 alone in a byte is also the 8-bit float (E4M3) q / 512: the subnormals and the
// first binade of that format form one linear grid.  v_cvt_pk_f32_fp8 converts two bytes per
// instruction, exactly, and fma(q / 512, unit * 512, mn) is bit for bit fma(float(q), unit, mn):
// scaling by a power of two is exact unless unit * 512 overflows, which the caller rules out per
// peer.  A pair of conversions costs a SIMD little more than one v_cvt_f32_ubyte.
template <int SCHEME, int BITS>
constexpr bool kPairedConversion = SCHEME == kMinMax && BITS == 4;
constexpr float kPairedScale = 512.0f;

// false: unit * 512 would not be finite (or unit is not) and the codes take the plain conversion
__device__ __forceinline__ bool paired_usable(float2 m) { return __builtin_fabsf(m.x) < 0x1p118f; }

// Levels / 512 of one group of 8 codes.
template <int BITS>
__device__ __forceinline__ void codes_to_scaled_float(uint64_t v, float (&f)[8])
{
    typedef float float2v __attribute__((ext_vector_type(2)));
    const uint32_t w = uint32_t(v);
    if (BITS == 4) {
        const uint32_t even = w & 0x0f0f0f0fu, odd = (w >> 4) & 0x0f0f0f0fu;
        const float2v e0 = __builtin_amdgcn_cvt_pk_f32_fp8(even, false), e1 = __builtin_amdgcn_cvt_pk_f32_fp8(even, true);
        const float2v o0 = __builtin_amdgcn_cvt_pk_f32_fp8(odd, false), o1 = __builtin_amdgcn_cvt_pk_f32_fp8(odd, true);
        f[0] = e0.x, f[2] = e0.y, f[4] = e1.x, f[6] = e1.y;
        f[1] = o0.x, f[3] = o0.y, f[5] = o1.x, f[7] = o1.y;
    } else {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const float2v p = __builtin_amdgcn_cvt_pk_f32_fp8((w >> (2 * j)) & 0x0303u, false);     // codes j and j + 4
            f[j] = p.x, f[4 + j] = p.y;
        }
    }
}

// Folds peers w0 .. w0+WB-1 into acc.  Each peer's share of the chunk (kChunk*BITS/8 bytes)
// is fetched as whole 16-byte vectors, consecutive across lanes, directly into the wave's
// LDS staging area, and read back by the lanes that own the codes.
// TAIL: the chunk is the short end of a layer; only its first nvecs 16-byte vectors exist in the
// packed streams (what lies behind them in LDS is stale, and so are the sums of elements past
// the end: the caller drops them).
// PAIRED: the two-per-instruction conversion above; the result says whether every peer's unit allowed it:
// if not, acc holds garbage and the caller forms the sums again without PAIRED.
template <int SCHEME, int BITS, int WB, bool TAIL, bool PAIRED, typename Peers>
__device__ __forceinline__ bool reduce_peers(Peers &peers, int w0, int64_t in_off, uint32_t g,
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
            if (TAIL ? v < nvecs : (kVecs % kWave == 0 || v < kVecs)) {
                // a block of one peer is what a decompression (W = 1) consists of: ordinary loads there
                if (WB == 1)
                    load_to_lds16_cached(in + v, stage + i * kVecs + k * kWave);
                else
                    load_to_lds16(in + v, stage + i * kVecs + k * kWave);
            }
        }
        m[i] = load_meta<SCHEME>(peers.meta[w0 + i], g);
    }
    wait_vector_memory();
    wave_lds_fence();
    const uint8_t *codes = reinterpret_cast<const uint8_t *>(stage);
    bool usable = true;
#pragma unroll
    for (int i = 0; i < WB; i++) {
        if constexpr (PAIRED && kPairedConversion<SCHEME, BITS>) {
            usable = usable && paired_usable(m[i]);
            m[i].x *= kPairedScale;
        }
#pragma unroll
        for (int r = 0; r < G; r++) {
            float f[8];
            if constexpr (PAIRED && kPairedConversion<SCHEME, BITS>)
                codes_to_scaled_float<BITS>(staged_codes<BITS>(codes + i * kBytes, code_off[r]), f);
            else
                codes_to_float<SCHEME, BITS>(staged_codes<BITS>(codes + i * kBytes, code_off[r]), f);
#pragma unroll
            for (int j = 0; j < 8; j++) acc[r][j] = __fadd_rn(acc[r][j], decode<SCHEME>(f[j], m[i]));
        }
        // keep the scheduler from hoisting every peer's LDS reads to the top (registers)
        if (i % 2 == 1) __builtin_amdgcn_sched_barrier(0);
    }
    wave_lds_fence();
    return __builtin_amdgcn_ballot_w64(!usable) == 0;
}

// Sum over the W peers of one chunk's dequantized values, added to acc in peer order.
// PAIRED: as in reduce_peers; false is returned when the sums have to be formed again without it.
template <int SCHEME, int BITS, bool TAIL = false, bool PAIRED = false, typename Peers>
__device__ __forceinline__ bool reduce_chunk(Peers &peers, int W, int64_t in_off, uint32_t g,
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
    bool good = true;
    for_peer_blocks<kWide>(W, [&](int w0, auto wb) {
        good &= reduce_peers<SCHEME, BITS, decltype(wb)::value, TAIL, PAIRED>(peers, w0, in_off, g, code_off, acc, stage,
                                                                             lane, nvecs);
    });
    return good;
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
    int keep;          // StorePolicy of the result: see flush_stage_to_elements
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
        // (the plain conversion: this kernel is bound by memory, and the paired one costs it registers)
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
                                    kChunk / 8, lane, io.keep);
        } else {
#pragma unroll
            for (int r = 0; r < G; r++) {
                float4v *p = reinterpret_cast<float4v *>(stage) + (map.group(r) >> 2);
                p[0] = float4v{acc[r][0], acc[r][1], acc[r][2], acc[r][3]};
                p[1] = float4v{acc[r][4], acc[r][5], acc[r][6], acc[r][7]};
            }
            wave_lds_fence();
            flush_stage_to_elements(stage, reinterpret_cast<uint4u2 *>(reinterpret_cast<float *>(io.out) + first),
                                    kChunk / 4, lane, io.keep);
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

// Sums of a tile of whole buckets of a size that is no power of two (kQuantAny), row by row: acc[r] belongs to
// group Gi = 64 r + lane (valid for Gi < shape.groups).  Two peers at a time: their codes (a multiple of 4
// bytes at a multiple of 4 in the stream) and the meta of the tile's buckets go straight into LDS, one dword
// per lane and instruction.
template <int SCHEME, int BITS, typename Peers>
__device__ __forceinline__ void reduce_any_regs(Peers &peers, int W, const Tile &tile, const AnyShape &shape,
                                                float (&acc)[G][8], uint4v *stage, int lane)
{
    constexpr int kPeerBytes = kChunk * BITS / 8 + 16 + kWave * 8;      // codes (+ over-read), unit[64], offset[64]
    static_assert(2 * kPeerBytes <= kChunk * 4, "staging area too small");
    constexpr int kMetaAt = kChunk * BITS / 8 + 16;
    const int dwords = shape.groups * BITS / 4;
    uint8_t *area = reinterpret_cast<uint8_t *>(stage);
    for_peer_blocks<2>(W, [&](int w0, auto wb) {
        constexpr int WB = decltype(wb)::value;
#pragma unroll
        for (int i = 0; i < WB; i++) {
            const uint32_t *in = reinterpret_cast<const uint32_t *>(peers.packed[w0 + i] + tile.packed_off);
            uint32_t *codes = reinterpret_cast<uint32_t *>(area + i * kPeerBytes);
            for (int v0 = 0; v0 < dwords; v0 += kWave)
                if (v0 + lane < dwords) load_to_lds4(in + v0 + lane, codes + v0);
            // meta of bucket j of the tile: lane j fetches it (kMinMax: unit and minimum, two dwords)
            const uint32_t *m = reinterpret_cast<const uint32_t *>(peers.meta[w0 + i]) + size_t(kMetaFloats<SCHEME>) * tile.bucket0;
            uint32_t *unit = reinterpret_cast<uint32_t *>(area + i * kPeerBytes + kMetaAt);
            if (lane < shape.m) {
                load_to_lds4(m + kMetaFloats<SCHEME> * lane, unit);
                if (SCHEME != kNormSign) load_to_lds4(m + kMetaFloats<SCHEME> * lane + 1, unit + kWave);
            }
        }
        wait_vector_memory();
        wave_lds_fence();
#pragma unroll
        for (int i = 0; i < WB; i++) {
            const uint8_t *codes = area + i * kPeerBytes;
            const float *unit = reinterpret_cast<const float *>(area + i * kPeerBytes + kMetaAt);
#pragma unroll
            for (int r = 0; r < G; r++) {
                const int Gi = r * kWave + lane;
                if (Gi < shape.groups) {
                    const int j = shape.bucket_of(Gi);
                    const float2 m = make_float2(unit[j], SCHEME == kNormSign ? 0.0f : unit[kWave + j]);
                    float f[8];
                    codes_to_float<SCHEME, BITS>(staged_codes<BITS>(codes, Gi * BITS), f);
#pragma unroll
                    for (int k = 0; k < 8; k++) acc[r][k] = __fadd_rn(acc[r][k], decode<SCHEME>(f[k], m));
                }
            }
        }
        wave_lds_fence();
    });
}

template <int SCHEME, int BITS, typename Peers>
__device__ __forceinline__ void reduce_any(Peers &peers, int W, const SumIo &io, const Tile &tile, int bucket,
                                           int lane, uint4v *stage)
{
    const AnyShape shape(tile, bucket);
    float acc[G][8];
#pragma unroll
    for (int r = 0; r < G; r++) {
        const int Gi = r * kWave + lane;
        if (Gi < shape.groups) {
            init8(io, tile.elem0 + int64_t(Gi) * 8, acc[r]);
        } else {
#pragma unroll
            for (int k = 0; k < 8; k++) acc[r][k] = -0.0f;
        }
    }
    reduce_any_regs<SCHEME, BITS>(peers, W, tile, shape, acc, stage, lane);
    // the sums leave through LDS as whole vectors: count is a multiple of 32 elements
    if (io.out_dt == CGX_F16) {
#pragma unroll
        for (int r = 0; r < G; r++) {
            const int Gi = r * kWave + lane;
            half8v h;
#pragma unroll
            for (int k = 0; k < 8; k++) h[k] = _Float16(acc[r][k]);
            if (Gi < shape.groups) reinterpret_cast<half8v *>(stage)[Gi] = h;
        }
        wave_lds_fence();
        flush_stage_to_elements(stage, reinterpret_cast<uint4u2 *>(reinterpret_cast<_Float16 *>(io.out) + tile.elem0),
                                shape.groups, lane, io.keep);
    } else {
#pragma unroll
        for (int r = 0; r < G; r++) {
            const int Gi = r * kWave + lane;
            if (Gi < shape.groups) {
                float4v *p = reinterpret_cast<float4v *>(stage) + 2 * Gi;
                p[0] = float4v{acc[r][0], acc[r][1], acc[r][2], acc[r][3]};
                p[1] = float4v{acc[r][4], acc[r][5], acc[r][6], acc[r][7]};
            }
        }
        wave_lds_fence();
        flush_stage_to_elements(stage, reinterpret_cast<uint4u2 *>(reinterpret_cast<float *>(io.out) + tile.elem0),
                                2 * shape.groups, lane, io.keep);
    }
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
__device__ __forceinline__ void reduce_slow(Peers &peers, int W, const SumIo &io, const Tile &tile, int bucket, int lane)
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
__device__ __forceinline__ void reduce_copy(Peers &peers, int W, const SumIo &io, int64_t e0, const Tile &tile, bool fast,
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

}  // namespace
}  // namespace cgx
