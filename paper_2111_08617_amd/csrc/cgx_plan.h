// Host-side plan: validation of the layer table, sizes of the packed stream
// and meta array, and the tile table the kernels walk.
//
// A tile is a contiguous run of elements of ONE layer that one wavefront
// processes: whole buckets of a quantized layer (paper Sec. 4.3: buckets are
// compressed independently; Sec. 4.1: layers are never mixed) or a piece of a
// pass-through layer.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/cgx.h"

#if defined(__HIPCC__)
#define CGX_HOST_DEVICE __host__ __device__
#else
#define CGX_HOST_DEVICE
#endif

namespace cgx {

// A chunk is what a wavefront handles per pass of the vectorised path: 64 lanes x `groups` groups
// of 8 consecutive elements.  A kernel is compiled for one chunk size (2 groups = 1024 elements or
// 4 groups = 2048 elements) and walks a tile table built for that size: a vectorised tile is a
// whole number of chunks.
constexpr int chunk_of(int groups) { return 64 * 8 * groups; }
// Elements per pass-through tile.
constexpr int kCopyTile = 8192;

enum TileKind : uint32_t {
    kQuantSlow = 0,  // any bucket size, any alignment, ragged last bucket
    kQuantFast = 1,  // power-of-two bucket <= chunk, whole chunks
    kCopyFast = 3,   // pass-through, 16-byte vectors
    kQuantWide = 4,  // one whole power-of-two bucket longer than a chunk (4096, 8192)
    kQuantTail = 5,  // power-of-two bucket <= chunk, the last tile of a layer, shorter than a chunk
    kQuantAny = 6    // whole buckets of a size that is no power of two (a multiple of 32, at most a chunk in all)
};

// Chunk-shaped quantized tiles (whole chunks of the bucket-major or row-by-row mapping).
CGX_HOST_DEVICE inline bool is_vector_kind(uint32_t kind) { return kind == kQuantFast || kind == kQuantWide; }
// Tiles that stream (everything else costs several dependent memory round trips and goes first in the table).
CGX_HOST_DEVICE inline bool is_streamed_kind(uint32_t kind) { return is_vector_kind(kind) || kind == kQuantAny; }

struct Tile {               // 32 bytes, read by the kernels with scalar loads
    int64_t elem0;          // first element, index in the fused buffer
    int64_t packed_off;     // byte offset of the tile's payload in the packed stream
    uint32_t bucket0;       // index of the tile's first bucket in the meta array
    uint32_t count;         // elements in the tile
    uint32_t info;          // bits [0:3] bit width, [4:7] TileKind, [8:11] log2(lanes per bucket), [12:20] bucket / 32
    uint32_t pad;           // zero bytes to append after the payload (last tile of a layer)
};
static_assert(sizeof(Tile) == 32, "tile layout is shared with the kernels");

CGX_HOST_DEVICE inline uint32_t tile_bits(const Tile &t) { return t.info & 15u; }
CGX_HOST_DEVICE inline uint32_t tile_kind(const Tile &t) { return (t.info >> 4) & 15u; }
CGX_HOST_DEVICE inline uint32_t tile_lpb_log2(const Tile &t) { return (t.info >> 8) & 15u; }
// Bucket size of a quantized tile (0 for pass-through tiles): info bits [12:20] hold bucket / 32.
CGX_HOST_DEVICE inline int tile_bucket(const Tile &t) { return int((t.info >> 12) & 0x1ffu) * 32; }

// How the vectorised tiles of a bucket size are laid over the lanes, which fixes the kernel
// instantiation of a launch: kMapBuckets for 96..chunk (bucket-major), kMapRows for 32 and 64
// (row by row; needs more registers, so a kernel of its own keeps the others' occupancy),
// kMapWide above the chunk size (a tile is one bucket of several chunks).  One launch serves
// every bucket size of one class.
enum LaneMapping { kMapBuckets = 0, kMapRows = 1, kMapWide = 2 };
inline int mapping_of(int bucket, int chunk) { return bucket <= 64 ? kMapRows : bucket > chunk ? kMapWide : kMapBuckets; }

struct PlanShape {
    size_t packed_bytes = 0;
    size_t meta_bytes = 0;
    uint64_t n_buckets = 0;
};

// Returns CGX_OK or the status code of the first violated rule.
int validate_plan(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int dt);
// The same rule for a bucket size per layer (every entry, also those of pass-through layers).
int validate_layer_buckets(int32_t L, const int32_t *layer_buckets);

// Sizes only (layout rules of cgx.h).  The plan must be valid.  layer_buckets, if not null,
// gives every layer its own bucket size and `bucket` is ignored.
PlanShape plan_shape(int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int dt,
                     const int32_t *layer_buckets = nullptr);

// Tile table for kernels with chunks of `chunk` elements.  `chunks_per_tile` bounds the length of
// fast tiles.
// With `slots` and `layer_first` (both or neither): numbering the tiles layer by layer and,
// inside a layer, by first element, tile t of the table has number slots[t], and layer l owns
// the numbers layer_first[l] .. layer_first[l + 1] - 1 (the per-layer statistics keep one
// partial sum per tile and add them up in that order).
// With layer_buckets (a bucket size per layer) the table holds the tiles of the layers whose
// bucket size has the lane mapping of `bucket` (mapping_of at this chunk size) only, at their places in the whole
// plan's streams: a launch runs one kernel instantiation, so such a plan takes one launch per
// mapping in use (at most three).  The pass-through layers belong to the launch with
// with_copies set.
void build_tiles(int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int dt, int chunk,
                 int chunks_per_tile, std::vector<Tile> &tiles, std::vector<uint32_t> *slots = nullptr,
                 std::vector<int64_t> *layer_first = nullptr, const int32_t *layer_buckets = nullptr,
                 bool with_copies = true);

}  // namespace cgx
