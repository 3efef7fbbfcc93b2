// cgx_dequant_reduce_requantize: the fused kernel and its launcher.
#include "cgx_device_quantize.h"
#include "cgx_device_reduce.h"

namespace cgx {
namespace {

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
        const int64_t in_off = tile.packed_off + int64_t(c) * (kChunk * BITS / 8);
        const uint32_t g = tile.bucket0 + c * buckets_per_chunk + map.bi;
        if (!reduce_chunk<SCHEME, BITS, false, true>(peers, W, in_off, g, map, acc, stage, lane)) {
            // a unit of 2^118 or more (or none at all): once more with the plain conversion
            clear_sums(acc);
            reduce_chunk<SCHEME, BITS>(peers, W, in_off, g, map, acc, stage, lane);
        }
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

// Whole buckets of a size that is no power of two: the row-by-row sums feed the row-by-row quantizer.
template <int SCHEME, int BITS, bool ODD, typename Peers>
__device__ __forceinline__ void fused_any(Peers &peers, int W, const Tile &tile, int64_t out_off, uint32_t out_pad,
                                          int bucket, uint32_t seed_lo, uint32_t seed_hi,
                                          uint8_t *__restrict__ packed_out, float *__restrict__ meta_out, int lane,
                                          uint4v *stage)
{
    const AnyShape shape(tile, bucket);
    const uint32_t key = rng_key(seed_lo, seed_hi, uint32_t((uint64_t(tile.elem0) >> 1) >> 32));
    float acc[G][8];
    clear_sums(acc);
    reduce_any_regs<SCHEME, BITS>(peers, W, tile, shape, acc, stage, lane);
    Tile out = tile;                                 // the same elements and buckets at their place in the output stream
    out.pad = out_pad;
    quantize_any_regs<SCHEME, BITS, ODD>(acc, shape, out, key, meta_out + kMetaFloats<SCHEME> * tile.bucket0,
                                         packed_out + out_off, stage, lane);
}

// tiles_in follows the layout of the chunks (storage type dt), tiles_out that of the
// output (binary32 pass-through layers); the two tables list the same tiles in the same order.
// WIDE: the call's bucket is longer than a chunk (see quantize_kernel's MAP).
struct FusedArguments {       // the kernarg segment's layout: offset of the peers' table behind the scalars
    const Tile *tiles_in, *tiles_out;
    int64_t n_tiles;
    int W, dt;
    uint32_t seed_lo, seed_hi;
    uint8_t *packed_out;
    float *meta_out;
    PeerPtrs peers;
};

template <int SCHEME, bool WIDE, bool ODD>
__global__ __launch_bounds__(kBlock) void fused_kernel(const Tile *__restrict__ tiles_in,
                                                        const Tile *__restrict__ tiles_out, int64_t n_tiles, int W,
                                                        int dt, uint32_t seed_lo, uint32_t seed_hi,
                                                        uint8_t *__restrict__ packed_out,
                                                        float *__restrict__ meta_out, const PeerPtrs peers_argument)
{
    (void)peers_argument;
    KernargPeers &peers = kernel_argument_peers(offsetof(FusedArguments, peers));
    __shared__ uint4v stage_all[kWavesPerBlock][kChunk / 4];
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    int lane_of_wave = int(threadIdx.x) & 63;
    uint4v *stage = stage_all[wave];
    const int64_t stride = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t t = int64_t(blockIdx.x) * kWavesPerBlock + wave; t < n_tiles; t += stride) {
        // the lane index is made opaque once per tile: otherwise everything that depends on the
        // lane alone (offsets, masks, of every bit width's path) is hoisted out of this loop and
        // stays in registers across all of it
        asm volatile("" : "+v"(lane_of_wave));
        const int lane = lane_of_wave;
        const Tile tile = tiles_in[t];
        const int bucket = tile_bucket(tile);       // per tile: a launch may mix sizes of one lane mapping
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
        } else if (!WIDE && kind == kQuantAny) {
            if constexpr (!WIDE) {
                CGX_FOR_BITS(tile_bits(tile), (fused_any<SCHEME, BITS, ODD>(peers, W, tile, out_off, out_pad, bucket, seed_lo,
                                                                            seed_hi, packed_out, meta_out, lane, stage)))
            }
        } else if (kind == kQuantSlow || kind == kQuantAny) {
            quantize_generic<SCHEME, false>(
                [&](uint32_t j) { return generic_sum<SCHEME>(peers, W, tile, bucket, j, -0.0f); },
                packed_out + out_off, meta_out, tile, out_pad, bucket, seed_lo, seed_hi, lane);
        } else {
            // pass-through: the sum is written as binary32 into the output stream, then its padding
            const SumIo io{nullptr, CGX_F32, packed_out + out_off, CGX_F32, 0};
            if (dt == CGX_F16)
                reduce_copy<CGX_F16>(peers, W, io, 0, tile, kind == kCopyFast, lane);
            else
                reduce_copy<CGX_F32>(peers, W, io, 0, tile, kind == kCopyFast, lane);
            uint8_t *end = packed_out + out_off + uint64_t(tile.count) * 4;
            if (uint32_t(lane) < out_pad) end[lane] = 0;
        }
    }
}

}  // namespace

hipError_t launch_dequant_reduce_requantize(int scheme, const PeerPtrs &peers, int W, int dt, const Tile *tiles_in,
                                            const Tile *tiles_out, int64_t n_tiles, bool odd_tiles, int32_t bucket,
                                            uint64_t seed, void *packed_out, void *meta_out,
                                            const LaunchConfig &cfg, hipStream_t stream)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(grid_for(n_tiles, cfg)), block(kBlock);
    const bool wide = mapping_of(bucket, kChunk) == kMapWide;
    using Kernel = void (*)(const Tile *, const Tile *, int64_t, int, int, uint32_t, uint32_t, uint8_t *, float *,
                            const PeerPtrs);
    static const Kernel table[2][2][2] = {
        {{fused_kernel<kMinMax, false, false>, fused_kernel<kMinMax, true, false>},
         {fused_kernel<kNormSign, false, false>, fused_kernel<kNormSign, true, false>}},
        {{fused_kernel<kMinMax, false, true>, fused_kernel<kMinMax, true, true>},
         {fused_kernel<kNormSign, false, true>, fused_kernel<kNormSign, true, true>}}};
    const Kernel kernel = table[odd_tiles][scheme == kSchemeNormSign][wide];
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, tiles_in, tiles_out, n_tiles, W, dt, uint32_t(seed),
                       uint32_t(seed >> 32), static_cast<uint8_t *>(packed_out), static_cast<float *>(meta_out), peers);
    return hipGetLastError();
}

}  // namespace cgx
