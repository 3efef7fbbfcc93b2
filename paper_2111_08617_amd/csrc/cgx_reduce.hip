// cgx_dequant_reduce and its relatives: the reduce kernel and its launcher.
#include "cgx_device_reduce.h"

namespace cgx {
namespace {

// TAILS: the short ends of layers take the masked chunk path.  The kernel with that path is
// about 1 % slower on plans that hardly use it (and, when it was added, needed one register
// more than the kernel's occupancy allows).  Without it a short end goes through the generic
// path, a chain of dependent round trips for one tile: hidden behind the rest of a long launch,
// it outlasts a short one (6 % of a 25 us launch with a single short end).  The host asks for
// it when there is a short end and the plan has fewer than 16384 tiles, or when short ends are
// at least 1/512 of the tiles.
// The arguments as the kernarg segment lays them out (each at its natural alignment, in order): gives the
// offset of the peers' table behind the scalars.
struct ReduceArguments {
    const Tile *tiles;
    int64_t n_tiles;
    int W, dt;
    const void *init;
    void *out;
    int init_dt, out_dt, keep;
    PeerPtrs peers;
};

template <int SCHEME, bool TAILS>
__global__ __launch_bounds__(kBlock) void reduce_kernel(const Tile *__restrict__ tiles, int64_t n_tiles, int W, int dt,
                                                         const void *init, void *out, int init_dt, int out_dt,
                                                         int keep, const PeerPtrs peers_argument)
{
    // the vectorised tiles index the table with constants (it then sits in scalar registers);
    // the other kinds index it at run time and read it from the kernarg segment
    const PeerPtrs &peers = peers_argument;
    KernargPeers &peers_in_memory = kernel_argument_peers(offsetof(ReduceArguments, peers));
    const SumIo io{init, init_dt, out, out_dt, keep};
    // per-wave staging area: a chunk of binary32 results, or the packed bytes of a block of peers
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
        const Tile tile = tiles[t];
        const int bucket = tile_bucket(tile);       // per tile: a launch may mix sizes of one lane mapping
        const uint32_t kind = tile_kind(tile);
        if (is_vector_kind(kind)) {      // a wide tile is chunks of one bucket: kChunk / bucket == 0 below
            CGX_FOR_BITS(tile_bits(tile), (reduce_fast<SCHEME, BITS>(peers, W, io, tile, bucket, lane, stage)))
        } else if (TAILS && kind == kQuantTail) {
            if constexpr (TAILS) {
                CGX_FOR_BITS(tile_bits(tile),
                             (reduce_tail<SCHEME, BITS>(peers_in_memory, W, io, tile, bucket, lane, stage)))
            }
        } else if (kind == kQuantAny) {
            CGX_FOR_BITS(tile_bits(tile), (reduce_any<SCHEME, BITS>(peers_in_memory, W, io, tile, bucket, lane, stage)))
        } else if (kind == kQuantSlow || kind == kQuantTail) {
            reduce_slow<SCHEME>(peers_in_memory, W, io, tile, bucket, lane);
        } else if (dt == CGX_F16) {
            reduce_copy<CGX_F16>(peers_in_memory, W, io, tile.elem0, tile, kind == kCopyFast, lane);
        } else {
            reduce_copy<CGX_F32>(peers_in_memory, W, io, tile.elem0, tile, kind == kCopyFast, lane);
        }
    }
}

}  // namespace

// This file is compiled once per chunk size (CGX_GROUPS = 2 and 4): launch_dequant_reduce_g2, launch_dequant_reduce_g4.
hipError_t CGX_CONCAT(launch_dequant_reduce_g, CGX_GROUPS)(int scheme, const PeerPtrs &peers, int W, int dt, const Tile *tiles, int64_t n_tiles,
                                 bool many_tails,
                                 int32_t bucket, const void *init, int init_dt, void *out, int out_dt,
                                 int store_policy, const LaunchConfig &cfg, hipStream_t stream)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(grid_for(n_tiles, cfg)), block(kBlock);
    const SumIo io{init, init_dt, out, out_dt, store_policy};
    const auto kernel = scheme == kSchemeNormSign
                            ? (many_tails ? reduce_kernel<kNormSign, true> : reduce_kernel<kNormSign, false>)
                            : (many_tails ? reduce_kernel<kMinMax, true> : reduce_kernel<kMinMax, false>);
    (void)bucket;
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, tiles, n_tiles, W, dt, io.init, io.out, io.init_dt, io.out_dt, io.keep,
                       peers);
    return hipGetLastError();
}

}  // namespace cgx
