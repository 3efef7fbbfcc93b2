// Launchers of the gfx950 kernels (implemented in cgx_quantize.hip, cgx_reduce.hip, cgx_fused.hip
// and cgx_stats.hip).
#pragma once

#include <hip/hip_runtime.h>

#include "cgx_plan.h"

namespace cgx {

constexpr int kPeersPerLaunch = 16;   // chunks one reduce launch reads; more peers take more launches

// The two quantizers the kernels implement (`scheme` below): affine between the bucket's
// minimum and maximum (meta: two floats per bucket), and sign plus level of |x| / max|x|
// (meta: one float per bucket).
enum { kSchemeMinMax = 0, kSchemeNormSign = 1 };

struct PeerPtrs {
    const uint8_t *packed[kPeersPerLaunch];
    const float *meta[kPeersPerLaunch];
};

// Tunables (set once from the environment at first use; see cgx_api.cpp).
struct LaunchConfig {
    int chunks_per_tile = 0;   // fast-tile length in chunks of kChunk elements; 0: chosen per call
    int max_blocks = 0;        // 0: one wave per tile; >0: persistent grid of at most this many blocks
    int via_lds = 1;           // quantize and squared errors: fetch aligned chunks of the buffer through LDS
    int quantize_groups = 0;   // 2 or 4: chunk size of every quantize call; 0: chosen per call
    long keep_sums_max_bytes = 128l << 20;   // reduce: results up to this size are kept in the memory-side cache
    int dequantize_through = 1;              // cgx_dequantize: stores written through at system scope
    int reduce_groups = 0;                   // 2 or 4: chunk size of every reduce call (0: chosen per call)
    int quantize_tiles_per_wave_x4 = 5;      // quantize: tiles per wave of the grid, in quarters (4: one wave per tile)
};

// odd_tiles: some vectorised tile starts on an odd element index (the kernels then take the
// variant that can draw across generator words; a property of the tile table).
// aligned_tiles: every vectorised tile starts on a 16-byte boundary of the buffer (its chunks can then be
// fetched through LDS with whole-line loads).
// The quantize kernel is built for chunks of 1024 elements (_g2: two groups of 8 per lane) and of 2048
// (_g4); `tiles` must have been built for that chunk size.
hipError_t launch_quantize_g2(int scheme, const void *grad, int dt, const Tile *tiles, int64_t n_tiles, bool odd_tiles,
                              bool aligned_tiles, int32_t bucket, uint64_t seed, void *packed, void *meta,
                              const LaunchConfig &cfg, hipStream_t stream);
hipError_t launch_quantize_g4(int scheme, const void *grad, int dt, const Tile *tiles, int64_t n_tiles, bool odd_tiles,
                              bool aligned_tiles, int32_t bucket, uint64_t seed, void *packed, void *meta,
                              const LaunchConfig &cfg, hipStream_t stream);
// Chunk size of every other kernel (reduce, fused, statistics).
constexpr int kDefaultChunk = chunk_of(4);

// How a reduce writes its result (see flush_stage_to_elements in cgx_device.h).
enum StorePolicy { kStoreStream = 0, kStoreKeep = 1, kStoreThrough = 2 };

// out[e] = init[e] + deq_0[e] + ... + deq_{W-1}[e] in that order (init == nullptr: no such
// term), W <= kPeersPerLaunch; init is binary32 or binary16, out binary32 or binary16.
// store_policy (StorePolicy): the result is streamed (non-temporal), written through at device scope (it then stays
// in the memory-side cache if it is small enough; the caller decides by size), or written through at system scope,
// non-temporal (calls that mostly write: a decompression).
// many_tails: the short ends of layers are a real share of the plan's tiles (the kernel then
// takes them through the masked chunk path instead of the generic one).
// (two builds: chunks of 1024 elements, which a decompression takes, and of 2048)
hipError_t launch_dequant_reduce_g2(int scheme, const PeerPtrs &peers, int W, int dt, const Tile *tiles, int64_t n_tiles,
                                 bool many_tails,
                                 int32_t bucket, const void *init, int init_dt, void *out, int out_dt,
                                 int store_policy, const LaunchConfig &cfg, hipStream_t stream);
hipError_t launch_dequant_reduce_g4(int scheme, const PeerPtrs &peers, int W, int dt, const Tile *tiles, int64_t n_tiles,
                                 bool many_tails,
                                 int32_t bucket, const void *init, int init_dt, void *out, int out_dt,
                                 int store_policy, const LaunchConfig &cfg, hipStream_t stream);

// packed_out / meta_out = quantize(deq_0 + ... + deq_{W-1}) without the binary32 sum ever
// reaching memory; tiles_in describes the chunks (storage type dt), tiles_out the output
// (binary32 pass-through); W <= kPeersPerLaunch.
hipError_t launch_dequant_reduce_requantize(int scheme, const PeerPtrs &peers, int W, int dt, const Tile *tiles_in,
                                            const Tile *tiles_out, int64_t n_tiles, bool odd_tiles, int32_t bucket,
                                            uint64_t seed, void *packed_out, void *meta_out,
                                            const LaunchConfig &cfg, hipStream_t stream);

// Per-layer squared l2 norms of buf (tiles of a plan whose layers are all pass-through) and
// of the compression error grad - dequantize(packed, meta) (tiles of the chunk's plan).
// slots / layer_first number the tiles per layer (see build_tiles); partial holds one double
// per tile; out one double per layer (all device memory).
hipError_t launch_layer_sqnorms(const void *buf, int dt, const Tile *tiles, const uint32_t *slots, int64_t n_tiles,
                                const int64_t *layer_first, int32_t L, double *partial, double *out,
                                const LaunchConfig &cfg, hipStream_t stream);
hipError_t launch_layer_sqerrors(int scheme, const void *grad, int dt, const void *packed, const void *meta,
                                 const Tile *tiles, const uint32_t *slots, int64_t n_tiles, bool aligned_tiles,
                                 const int64_t *layer_first, int32_t L, double *partial,
                                 double *out, const LaunchConfig &cfg, hipStream_t stream, bool sum_layers = true);
// (sum_layers = false: only the tiles' partial sums are written; a plan served by several tile
// tables adds them up after the last one)

// launch_layer_sqnorms with every table and the partial sums in a fixed device array of the
// library: no allocation, nothing copied from host memory on the stream.  off / first: host
// arrays [L + 1], layer offsets and the number of each layer's first tile (runs of kCopyTile
// elements); L <= CGX_NOALLOC_MAX_LAYERS and first[L] <= CGX_NOALLOC_MAX_TILES (caller-checked).
hipError_t launch_layer_sqnorms_noalloc(const void *buf, int dt, const int64_t *off, const int64_t *first, int32_t L,
                                        double *out, hipStream_t stream);

// Measurement aid (cgx_diag.h): streams read_bytes in and write_bytes out (multiples of 16) with the
// access style of the kernels and no arithmetic, in the given launch shape (checked by the caller).
struct ProbeShape {
    int slice_bytes = 8192;
    int block_threads = 256;
    int load_policy = 1;
    int store_policy = 1;
    int xcd_contiguous = 0;
    int max_blocks = 0;
    int paired_loads = 0;
    int alu_ops_per_pass = 0;
    int lds_bytes_per_block = 0;
};
hipError_t launch_stream_probe(const void *src, size_t read_bytes, void *dst, size_t write_bytes,
                               const ProbeShape &shape, hipStream_t stream);
// The issue-rate probe: the text of instruction form number `form` (nullptr past the last), and one launch
// of `blocks` blocks of 256 threads that each run 16 * iterations instructions of that form per wave and
// leave one word per thread in out.
const char *issue_probe_form(int form);
hipError_t launch_issue_probe(int form, int blocks, int iterations, void *out, hipStream_t stream);

}  // namespace cgx
