// Plan validation, sizes and tile table (host only; no HIP calls here).
#include "cgx_plan.h"

#include <algorithm>

namespace cgx {

static inline uint64_t round_up16(uint64_t v) { return (v + 15u) & ~uint64_t(15); }
static inline int elem_size(int dt) { return dt == CGX_F16 ? 2 : 4; }

int validate_plan(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int dt)
{
    if (n < 0 || L < 0) return CGX_ERR_SIZE;
    if (L > 0 && (!off || !bits)) return CGX_ERR_NULL;
    if (dt != CGX_F32 && dt != CGX_F16) return CGX_ERR_DTYPE;
    if (bucket < 32 || bucket > 8192 || bucket % 32) return CGX_ERR_BUCKET;
    if (L == 0) return n == 0 ? CGX_OK : CGX_ERR_SIZE;
    if (off[0] != 0) return CGX_ERR_OFFSETS;
    for (int32_t l = 0; l < L; l++) {
        if (off[l + 1] < off[l]) return CGX_ERR_OFFSETS;
        if (bits[l] > 8) return CGX_ERR_BITS;
    }
    if (off[L] != n) return CGX_ERR_SIZE;
    // bucket indices are 32-bit in the tile table
    if (n / 32 > int64_t(0xfffffff0u)) return CGX_ERR_SIZE;
    return CGX_OK;
}

int validate_layer_buckets(int32_t L, const int32_t *layer_buckets)
{
    if (L > 0 && !layer_buckets) return CGX_ERR_NULL;
    for (int32_t l = 0; l < L; l++)
        if (layer_buckets[l] < 32 || layer_buckets[l] > 8192 || layer_buckets[l] % 32) return CGX_ERR_BUCKET;
    return CGX_OK;
}

// Payload bytes (before padding) and buckets of one layer.
static inline void layer_extent(int64_t len, int b, int32_t bucket, int dt, uint64_t &payload, uint64_t &buckets)
{
    if (b == 0) {
        payload = uint64_t(len) * elem_size(dt);
        buckets = 0;
    } else {
        payload = (uint64_t(len) * b + 7) / 8;
        buckets = (uint64_t(len) + bucket - 1) / bucket;
    }
}

PlanShape plan_shape(int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int dt,
                     const int32_t *layer_buckets)
{
    PlanShape s;
    for (int32_t l = 0; l < L; l++) {
        int64_t len = off[l + 1] - off[l];
        if (len == 0) continue;
        uint64_t payload, buckets;
        layer_extent(len, bits[l], layer_buckets ? layer_buckets[l] : bucket, dt, payload, buckets);
        s.packed_bytes += round_up16(payload);
        s.n_buckets += buckets;
    }
    s.meta_bytes = size_t(8 * s.n_buckets);
    return s;
}

static inline bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
static inline int log2i(int v) { int k = 0; while ((1 << k) < v) k++; return k; }

// All element pairs of [e0, e0 + count) share the upper 32 bits of their pair
// index, so the generator's key is uniform over the tile.
static inline bool same_key_block(int64_t e0, int64_t count)
{
    return ((uint64_t(e0) >> 1) >> 32) == ((uint64_t(e0 + count - 1) >> 1) >> 32);
}

void build_tiles(int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int dt, int chunk,
                 int chunks_per_tile, std::vector<Tile> &tiles, std::vector<uint32_t> *slots,
                 std::vector<int64_t> *layer_first, const int32_t *layer_buckets, bool with_copies)
{
    tiles.clear();
    if (layer_first) layer_first->assign(size_t(L) + 1, 0);
    if (chunks_per_tile < 1) chunks_per_tile = 1;
    const int S = elem_size(dt);
    const int kChunk = chunk, kGroups = chunk / (64 * 8);
    const int launch_mapping = mapping_of(bucket, chunk);
    uint64_t seg = 0, bucket0 = 0;
    for (int32_t l = 0; l < L; l++) {
        const int64_t first = off[l], len = off[l + 1] - off[l];
        if (layer_first) (*layer_first)[size_t(l)] = int64_t(tiles.size());
        if (len == 0) continue;
        const int b = bits[l];
        uint64_t payload, buckets;
        const int32_t own_bucket = layer_buckets ? layer_buckets[l] : bucket;
        layer_extent(len, b, own_bucket, dt, payload, buckets);
        if (b == 0 ? !with_copies : mapping_of(own_bucket, chunk) != launch_mapping) {
            seg += round_up16(payload);                           // another launch's layer: only its extent counts
            bucket0 += buckets;
            continue;
        }
        const bool fast_bucket = is_pow2(own_bucket) && own_bucket <= kChunk;
        const bool wide_bucket = is_pow2(own_bucket) && own_bucket > kChunk;       // a bucket is 2, 4 or 8 chunks
        // 64 lanes x kGroups groups x 8 elements = kChunk, so a bucket spans bucket / (8 * kGroups) lanes
        const uint32_t lpb_log2 = fast_bucket ? uint32_t(log2i(own_bucket / (8 * kGroups))) : 0u;
        const uint32_t size_bits = uint32_t(own_bucket / 32) << 12;
        const uint32_t pad = uint32_t(round_up16(payload) - payload);
        // vector accesses on the gradient side are element-aligned, so a layer may start anywhere
        const bool aligned = true;
        const size_t first_tile = tiles.size();
        if (b == 0) {
            for (int64_t j = 0; j < len; j += kCopyTile) {
                Tile t{};
                t.elem0 = first + j;
                t.packed_off = int64_t(seg + uint64_t(j) * S);
                t.count = uint32_t(len - j < kCopyTile ? len - j : kCopyTile);
                t.info = uint32_t(kCopyFast) << 4;
                tiles.push_back(t);
            }
        } else {
            int64_t j = 0;
            if (fast_bucket && aligned) {
                const int64_t full_chunks = len / kChunk;
                for (int64_t c = 0; c < full_chunks;) {
                    int64_t k = full_chunks - c < chunks_per_tile ? full_chunks - c : chunks_per_tile;
                    // a tile must not straddle a 2^33-element block of the generator's key
                    while (k > 1 && !same_key_block(first + c * kChunk, k * kChunk)) k--;
                    Tile t{};
                    t.elem0 = first + c * kChunk;
                    t.packed_off = int64_t(seg + uint64_t(c) * kChunk * b / 8);
                    t.bucket0 = uint32_t(bucket0 + uint64_t(c) * kChunk / own_bucket);
                    t.count = uint32_t(k * kChunk);
                    const bool fast = same_key_block(t.elem0, t.count);
                    t.info = uint32_t(b) | uint32_t(fast ? kQuantFast : kQuantSlow) << 4 | lpb_log2 << 8 | size_bits;
                    tiles.push_back(t);
                    c += k;
                }
                j = full_chunks * kChunk;
            } else if (wide_bucket && aligned) {
                // one tile per whole bucket: its scale needs all of it (lanes-per-bucket field: the whole wave)
                const int64_t full = len / own_bucket;
                for (int64_t k = 0; k < full; k++) {
                    Tile t{};
                    t.elem0 = first + k * own_bucket;
                    t.packed_off = int64_t(seg + uint64_t(k) * own_bucket * b / 8);
                    t.bucket0 = uint32_t(bucket0 + uint64_t(k));
                    t.count = uint32_t(own_bucket);
                    const bool fast = same_key_block(t.elem0, t.count);
                    t.info = uint32_t(b) | uint32_t(fast ? kQuantWide : kQuantSlow) << 4 | 6u << 8 | size_bits;
                    tiles.push_back(t);
                }
                j = full * own_bucket;
            }
            // what is left (or the whole layer): whole buckets, about a chunk per tile
            const int64_t step = own_bucket >= kChunk ? own_bucket : int64_t(kChunk / own_bucket) * own_bucket;
            for (; j < len; j += step) {
                Tile t{};
                t.elem0 = first + j;
                t.packed_off = int64_t(seg + uint64_t(j) * b / 8);
                t.bucket0 = uint32_t(bucket0 + uint64_t(j) / own_bucket);
                t.count = uint32_t(len - j < step ? len - j : step);
                // the short end of a layer with power-of-two buckets runs through the chunk code, masked
                const bool tail = fast_bucket && j % kChunk == 0 && t.count < uint32_t(kChunk) &&
                                  same_key_block(t.elem0, t.count);
                // whole buckets of a size that is no power of two, a chunk or less in all: the streamed path
                // for any bucket size (the ragged end of a layer stays on the generic one)
                const bool any = !tail && !is_pow2(own_bucket) && own_bucket <= kChunk && t.count % uint32_t(own_bucket) == 0 &&
                                 t.count <= uint32_t(kChunk) && same_key_block(t.elem0, t.count);
                t.info = uint32_t(b) | uint32_t(tail ? kQuantTail : any ? kQuantAny : kQuantSlow) << 4 |
                         (tail ? lpb_log2 << 8 : 0u) | size_bits;
                tiles.push_back(t);
            }
        }
        if (tiles.size() > first_tile) tiles.back().pad = pad;
        seg += round_up16(payload);
        bucket0 += buckets;
    }
    // Waves take tiles in table order.  The generic and pass-through tiles cost several
    // dependent memory round trips each, so they go first and overlap with the stream
    // of vectorised tiles instead of forming the tail of the launch.
    if (layer_first) (*layer_first)[size_t(L)] = int64_t(tiles.size());
    std::vector<uint32_t> order(tiles.size());
    for (size_t i = 0; i < order.size(); i++) order[i] = uint32_t(i);
    std::stable_partition(order.begin(), order.end(),
                          [&](uint32_t i) { return !is_streamed_kind(tile_kind(tiles[i])); });
    std::vector<Tile> sorted(tiles.size());
    for (size_t i = 0; i < order.size(); i++) sorted[i] = tiles[order[i]];
    tiles.swap(sorted);
    if (slots) slots->swap(order);
}

}  // namespace cgx
