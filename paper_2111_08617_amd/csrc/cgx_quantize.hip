// cgx_quantize / cgx_requantize / cgx_qsgd_quantize: the quantize kernel and its launcher.
#include "cgx_device_quantize.h"

namespace cgx {
namespace {

// ODD: some vectorised tile of the plan starts on an odd element index (see encode_group).
// VIA_LDS: every vectorised tile starts on a 16-byte boundary and the bucket-major mapping reads its
// chunks through LDS (see chunk_through_lds); never together with ODD.
template <int SCHEME, int DT, int MAP, bool ODD, bool VIA_LDS = false>
__global__ __launch_bounds__(kBlock) void quantize_kernel(const void *__restrict__ grad,
                                                           const Tile *__restrict__ tiles, int64_t n_tiles,
                                                           uint32_t seed_lo, uint32_t seed_hi,
                                                           uint8_t *__restrict__ packed,
                                                           float *__restrict__ meta)
{
    // per-wave staging area for a chunk's packed codes (at most kChunk bytes, at 8 bits), and with
    // VIA_LDS for the chunk as stored
    constexpr int kInputBytes = VIA_LDS ? kChunk * (DT == CGX_F16 ? 2 : 4) : kChunk;
    constexpr int kStageBytes = (MAP == kMapBuckets && kAnyStageBytes > kInputBytes) ? kAnyStageBytes : kInputBytes;
    __shared__ uint4v stage_all[kWavesPerBlock][kStageBytes / 16];
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    int lane_of_wave = int(threadIdx.x) & 63;
    uint4v *stage = stage_all[wave];
    const int64_t stride = int64_t(gridDim.x) * kWavesPerBlock;
    int64_t t = int64_t(blockIdx.x) * kWavesPerBlock + wave;
    if (t >= n_tiles) return;
    Tile upcoming = tiles[t];
    for (; t < n_tiles; t += stride) {
        // the lane index is made opaque once per tile: otherwise everything that depends on the
        // lane alone (offsets, masks, of every bit width's path) is hoisted out of this loop and
        // stays in registers across all of it
        asm volatile("" : "+v"(lane_of_wave));
        const int lane = lane_of_wave;
        const Tile tile = upcoming;
        // a wave that takes more than one tile has the next descriptor on its way meanwhile
        if (t + stride < n_tiles) upcoming = tiles[t + stride];
        const int bucket = tile_bucket(tile);       // per tile: a launch may mix sizes of one lane mapping
        const uint32_t kind = tile_kind(tile);
        if (is_vector_kind(kind)) {
            if constexpr (MAP == kMapRows) {
                CGX_FOR_BITS(tile_bits(tile), (quantize_fast_rows<SCHEME, DT, BITS, ODD>(grad, packed, meta, tile, bucket,
                                                                                      seed_lo, seed_hi, lane, stage)))
            } else if constexpr (MAP == kMapWide) {
                CGX_FOR_BITS(tile_bits(tile), (quantize_wide<SCHEME, DT, BITS, ODD>(grad, packed, meta, tile, bucket,
                                                                                 seed_lo, seed_hi, lane, stage)))
            } else {
                CGX_FOR_BITS(tile_bits(tile), (quantize_fast<SCHEME, DT, BITS, ODD, VIA_LDS>(
                                                  grad, packed, meta, tile, bucket, seed_lo, seed_hi, lane, stage)))
            }
        } else if (kind == kQuantTail) {
            CGX_FOR_BITS(tile_bits(tile), (quantize_tail<SCHEME, DT, BITS, ODD>(grad, packed, meta, tile, bucket,
                                                                                  seed_lo, seed_hi, lane, stage)))
        } else if (MAP == kMapBuckets && kind == kQuantAny) {
            if constexpr (MAP == kMapBuckets) {
                CGX_FOR_BITS(tile_bits(tile), (quantize_any<SCHEME, DT, BITS, ODD>(grad, packed, meta, tile, bucket,
                                                                                     seed_lo, seed_hi, lane, stage)))
            }
        } else if (kind == kQuantSlow || kind == kQuantAny) {
            quantize_generic<SCHEME, true>([&](uint32_t j) { return load_elem<DT>(grad, tile.elem0 + j); },
                                           packed + tile.packed_off, meta, tile, tile.pad, bucket, seed_lo,
                                           seed_hi, lane);
        } else {
            copy_tile<DT>(grad, packed, tile, kind == kCopyFast, lane);
        }
    }
}

}  // namespace

// This file is compiled once per chunk size (CGX_GROUPS = 2 and 4): launch_quantize_g2, launch_quantize_g4.
hipError_t CGX_CONCAT(launch_quantize_g, CGX_GROUPS)(int scheme, const void *grad, int dt, const Tile *tiles, int64_t n_tiles, bool odd_tiles,
                           bool aligned_tiles, int32_t bucket, uint64_t seed, void *packed, void *meta,
                           const LaunchConfig &cfg, hipStream_t stream)
{
    if (n_tiles == 0) return hipSuccess;
    // Four fifths of the waves that one tile each would take: every fourth wave takes a second tile, whose
    // descriptor it fetches while it works on the first.  For the kernel of 1024-element chunks on plans of up to
    // 2^19 tiles.  Measured by kernel trace, the two grids alternating on one box: ResNet-50 plan (25 k tiles)
    // 20.9 -> 20.0 us, the requantize of a 13.7 M-element share 12.6 -> 11.9 us, full BERT-base buffer 77.6 ->
    // 76.3 us, a 44 M-element share 34.6 -> 34.2 us; the 1.3 G-element buffer (1.28 M tiles) 978 -> 988 us and
    // binary16 input (2048-element chunks, two per tile) 25.5 -> 26.7 us on a small buffer, hence the limits.
    // With one and a half tiles per wave the gain is gone from 100 M elements on, with two it is a loss.
    LaunchConfig shaped = cfg;
    if (kGroups == 2 && cfg.max_blocks == 0 && cfg.quantize_tiles_per_wave_x4 > 4 && n_tiles <= (int64_t(1) << 19)) {
        const int64_t blocks = (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
        shaped.max_blocks = int((blocks * 4 + cfg.quantize_tiles_per_wave_x4 - 1) / cfg.quantize_tiles_per_wave_x4);
    }
    const dim3 grid(grid_for(n_tiles, shaped)), block(kBlock);
    const uint32_t seed_lo = uint32_t(seed), seed_hi = uint32_t(seed >> 32);
    using Kernel = void (*)(const void *, const Tile *, int64_t, uint32_t, uint32_t, uint8_t *, float *);
#define CGX_QUANTIZE_MAPS(S, D, O) \
    {quantize_kernel<S, D, kMapBuckets, O>, quantize_kernel<S, D, kMapRows, O>, quantize_kernel<S, D, kMapWide, O>}
    static const Kernel table[2][2][2][3] = {
        {{CGX_QUANTIZE_MAPS(kMinMax, CGX_F32, false), CGX_QUANTIZE_MAPS(kMinMax, CGX_F16, false)},
         {CGX_QUANTIZE_MAPS(kNormSign, CGX_F32, false), CGX_QUANTIZE_MAPS(kNormSign, CGX_F16, false)}},
        {{CGX_QUANTIZE_MAPS(kMinMax, CGX_F32, true), CGX_QUANTIZE_MAPS(kMinMax, CGX_F16, true)},
         {CGX_QUANTIZE_MAPS(kNormSign, CGX_F32, true), CGX_QUANTIZE_MAPS(kNormSign, CGX_F16, true)}}};
#undef CGX_QUANTIZE_MAPS
    static const Kernel through_lds[2][2] = {
        {quantize_kernel<kMinMax, CGX_F32, kMapBuckets, false, true>, quantize_kernel<kMinMax, CGX_F16, kMapBuckets, false, true>},
        {quantize_kernel<kNormSign, CGX_F32, kMapBuckets, false, true>, quantize_kernel<kNormSign, CGX_F16, kMapBuckets, false, true>}};
    const bool via_lds = aligned_tiles && !odd_tiles && mapping_of(bucket, kChunk) == kMapBuckets && cfg.via_lds;
    const Kernel kernel = via_lds ? through_lds[scheme == kSchemeNormSign][dt == CGX_F16]
                                  : table[odd_tiles][scheme == kSchemeNormSign][dt == CGX_F16][mapping_of(bucket, kChunk)];
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, grad, tiles, n_tiles, seed_lo, seed_hi,
                       static_cast<uint8_t *>(packed), static_cast<float *>(meta));
    return hipGetLastError();
}

}  // namespace cgx
