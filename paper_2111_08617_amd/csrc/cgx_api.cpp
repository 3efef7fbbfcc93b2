// extern "C" entry points of libcgx.so (see include/cgx.h): argument checks,
// the per-plan tile table cache, and kernel launches on the caller's stream.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <vector>

#include "../../include/cgx_diag.h"
#include "cgx_kernels.h"
#include "cgx_plan.h"

namespace {

using cgx::Tile;

struct CachedPlan {
    // identity
    int device = 0;
    int32_t bucket = 0;
    int dt = 0;
    uint64_t digest = 0;        // hash of (off, bits, layer_buckets): compared before the arrays themselves
    int chunk = 0;              // elements per chunk of the kernels that walk this table
    int chunks_per_tile = 0;
    std::vector<int64_t> off;
    std::vector<uint8_t> bits;
    std::vector<int32_t> layer_buckets;   // empty: `bucket` for every layer; else the table holds the
    bool with_copies = true;              // layers of size `bucket` (and the pass-through ones if with_copies)
    // content
    cgx::PlanShape shape;
    int64_t n_tiles = 0;
    int64_t plan_tiles = 0;     // tiles of the whole plan: n_tiles, or the sum over the launches of a layered plan
    bool odd_tiles = false;     // some vectorised quantized tile starts on an odd element index
    bool aligned_tiles = true;  // every vectorised quantized tile starts on a 16-byte boundary of the buffer
    bool many_tails = false;    // the reduce kernel with the masked path for short ends of layers pays (see get_plan)
    Tile *d_tiles = nullptr;
    // per-layer numbering of the tiles (for the statistics): slot of every tile, first slot of every layer
    uint32_t *d_slots = nullptr;
    int64_t *d_layer_first = nullptr;
    uint64_t last_use = 0;      // cache clock at the latest look-up
    bool pinned = false;        // a stream capture has recorded launches that read these tables: never dropped
};

void free_plan(CachedPlan &p)
{
    if (p.d_tiles) (void)hipFree(p.d_tiles);
    if (p.d_slots) (void)hipFree(p.d_slots);
    if (p.d_layer_first) (void)hipFree(p.d_layer_first);
    p.d_tiles = nullptr;
    p.d_slots = nullptr;
    p.d_layer_first = nullptr;
}

template <typename T>
bool upload(T **dst, const std::vector<T> &src)
{
    if (src.empty()) return true;
    const size_t bytes = src.size() * sizeof(T);
    if (hipMalloc(reinterpret_cast<void **>(dst), bytes) != hipSuccess) return false;
    return hipMemcpy(*dst, src.data(), bytes, hipMemcpyHostToDevice) == hipSuccess;
}

std::mutex g_mutex;
// A caller that keeps changing its plan (new bit widths every so often) must not grow the
// cache without bound: beyond kMaxPlans entries the least recently used one is dropped.  An
// entry handed out stays alive while its call uses it (shared ownership); its device tables
// are released when the last owner lets go, and hipFree waits for launches still reading them.
// The cache object itself is never destroyed, so nothing is freed during process exit, when
// the HIP runtime may already be gone.
constexpr size_t kMaxPlans = 64;
using PlanRef = std::shared_ptr<const CachedPlan>;
std::vector<std::shared_ptr<CachedPlan>> &g_plans = *new std::vector<std::shared_ptr<CachedPlan>>();
uint64_t g_clock = 0;

int env_int(const char *name, int fallback)
{
    const char *v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : fallback;
}

// Launch-shape overrides for the tests and for measurements (listed in include/cgx_diag.h): read once.
const cgx::LaunchConfig &launch_config()
{
    static const cgx::LaunchConfig cfg = [] {
        cgx::LaunchConfig c;
        c.chunks_per_tile = env_int("CGX_CHUNKS_PER_TILE", 0);
        c.max_blocks = env_int("CGX_MAX_BLOCKS", c.max_blocks);
        c.via_lds = env_int("CGX_VIA_LDS", c.via_lds);
        c.keep_sums_max_bytes = long(env_int("CGX_KEEP_SUMS_MB", int(c.keep_sums_max_bytes >> 20))) << 20;
        c.dequantize_through = env_int("CGX_DEQUANTIZE_THROUGH", c.dequantize_through);
        c.reduce_groups = env_int("CGX_REDUCE_GROUPS", 0) == 2 ? 2 : env_int("CGX_REDUCE_GROUPS", 0) == 4 ? 4 : 0;
        c.quantize_tiles_per_wave_x4 = env_int("CGX_QUANTIZE_TILES_PER_WAVE_X4", c.quantize_tiles_per_wave_x4);
        c.quantize_groups = env_int("CGX_QUANTIZE_GROUPS", 0) == 2 ? 2 : env_int("CGX_QUANTIZE_GROUPS", 0) == 4 ? 4 : 0;
        return c;
    }();
    return cfg;
}

// Chunks per vectorised tile.  One keeps the most loads in flight and wins wherever a wave's
// chunk is 4 KB of input or more.  Two cases differ on buffers that fill the chip many times over
// (measured; shorter buffers lose to the coarser tail of the launch):
//  - cgx_quantize on binary16, which is the heaviest in arithmetic per byte: a wave takes 2 chunks
//    (354 M elements: 155 -> 149 us; 4 chunks: 156 us);
//  - the fused reduce + requantize, which is bound by arithmetic: 2 chunks (3-6 % faster at
//    164-268 M elements for every width).
// Bucket sizes of a call: one for all layers, or one per layer (per_layer != nullptr).
struct Buckets {
    int32_t uniform;
    const int32_t *per_layer;
};

enum CallKind { kQuantizeCall, kFusedCall, kOtherCall };

// Elements per chunk of the kernel a call runs.  The quantizer of binary32 input takes chunks of 1024
// elements (4 KB per wave and pass: measured, a streaming kernel sustains about a tenth more with 4 KB
// per wave than with 8 KB, and the quantizer follows it: 0.74 -> 0.78 of the HBM peak on 1.3 G
// elements); on binary16 a chunk of 2048 elements is 4 KB already.  The reduce, fused and statistics
// kernels take 2048 (a peer's codes of a chunk then fill a whole load instruction at 4 bits).
// Bucket sizes between 1024 and 2048 take the quantizer of 2048-element chunks also on binary32 (one bucket per
// chunk, vectorised or streamed; with chunks of 1024 such a bucket is a two-pass tile or a generic one).
int chunk_length(CallKind call, int dt, const Buckets &buckets)
{
    const int forced = launch_config().quantize_groups;
    if (call != kQuantizeCall) return cgx::kDefaultChunk;
    if (forced > 0) return cgx::chunk_of(forced);
    const bool long_buckets = !buckets.per_layer && buckets.uniform > 1024 && buckets.uniform <= 2048;
    return cgx::chunk_of(dt == CGX_F32 && !long_buckets ? 2 : 4);
}

int tile_length(CallKind call, int dt, int64_t n)
{
    const int forced = launch_config().chunks_per_tile;
    if (forced > 0) return forced;
    if (call == kQuantizeCall && dt == CGX_F16 && n >= (int64_t(1) << 24)) return 2;
    if (call == kFusedCall && n >= (int64_t(1) << 27)) return 2;
    return 1;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// One launch per lane mapping in use (a launch runs one kernel instantiation; the bucket size
// itself travels in the tile descriptors), named by the smallest bucket size of that mapping;
// the first launch also carries the pass-through layers.
struct Launch {
    int32_t bucket;
    bool with_copies;
};
std::vector<Launch> launches_of(const Buckets &b, int32_t L, const int64_t *off, const uint8_t *bits, int chunk)
{
    if (!b.per_layer) return {{b.uniform, true}};
    int32_t smallest[3] = {0, 0, 0};
    for (int32_t l = 0; l < L; l++)
        if (bits[l] != 0 && off[l + 1] > off[l]) {
            int32_t &s = smallest[cgx::mapping_of(b.per_layer[l], chunk)];
            if (s == 0 || b.per_layer[l] < s) s = b.per_layer[l];
        }
    std::vector<Launch> out;
    for (int32_t s : smallest)
        if (s != 0) out.push_back({s, out.empty()});
    if (out.empty()) out.push_back({32, true});         // pass-through layers only
    return out;
}

// A 64-bit digest of the plan's arrays, eight bytes at a time (multiply and xor-shift per word): a look-up
// compares this one word per cached plan and the arrays themselves only on a match.
uint64_t plan_digest(int32_t L, const int64_t *off, const uint8_t *bits, const int32_t *layer_buckets)
{
    uint64_t h = 0x9e3779b97f4a7c15ull ^ uint64_t(L);
    const auto mix = [&h](const void *p, size_t bytes) {
        const unsigned char *c = static_cast<const unsigned char *>(p);
        for (size_t i = 0; i < bytes; i += 8) {
            uint64_t w = 0;
            std::memcpy(&w, c + i, bytes - i < 8 ? bytes - i : 8);
            h = (h ^ w) * 0xff51afd7ed558ccdull;
            h ^= h >> 32;
        }
    };
    mix(off, sizeof(int64_t) * (size_t(L) + 1));
    mix(bits, size_t(L));
    if (layer_buckets) mix(layer_buckets, sizeof(int32_t) * size_t(L));
    return h;
}

// Finds or builds the device-resident tile table of a (valid) plan for a call on `stream`.
// A graph that is being captured keeps the raw table pointers of the launches recorded into it, so a table
// found during a capture is pinned for the life of the library (never the one dropped for a new plan),
// and a table that does not exist yet is not built during a capture (that would allocate and copy
// synchronously in the middle of it): the call fails with CGX_ERR_CAPTURE and records nothing.
int get_plan(hipStream_t stream, int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int dt, int chunk,
             int chunks_per_tile, PlanRef *out, const int32_t *layer_buckets = nullptr, bool with_copies = true)
{
    const uint64_t digest = plan_digest(L, off, bits, layer_buckets);       // before the lock is taken
    std::lock_guard<std::mutex> lock(g_mutex);
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return CGX_ERR_HIP;
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    const bool capturing = hipStreamIsCapturing(stream, &capture) == hipSuccess && capture == hipStreamCaptureStatusActive;
    if (!capturing) (void)hipGetLastError();       // a refused query (legacy stream beside a capture) is not this call's error
    for (const auto &p : g_plans) {
        if (p->digest == digest && p->device == device && p->bucket == bucket && p->dt == dt &&
            p->chunk == chunk && p->chunks_per_tile == chunks_per_tile && p->bits.size() == size_t(L) &&
            p->with_copies == with_copies && p->layer_buckets.size() == (layer_buckets ? size_t(L) : 0) &&
            (!layer_buckets || L == 0 ||
             std::memcmp(p->layer_buckets.data(), layer_buckets, sizeof(int32_t) * size_t(L)) == 0) &&
            std::memcmp(p->bits.data(), bits, size_t(L)) == 0 &&
            std::memcmp(p->off.data(), off, sizeof(int64_t) * (size_t(L) + 1)) == 0) {
            p->last_use = ++g_clock;
            if (capturing) p->pinned = true;
            *out = p;
            return CGX_OK;
        }
    }
    if (capturing) return CGX_ERR_CAPTURE;
    std::shared_ptr<CachedPlan> plan(new CachedPlan, [](CachedPlan *p) {
        free_plan(*p);
        delete p;
    });
    plan->digest = digest;
    plan->device = device;
    plan->bucket = bucket;
    plan->dt = dt;
    plan->chunk = chunk;
    plan->chunks_per_tile = chunks_per_tile;
    plan->off.assign(off, off + L + 1);
    plan->bits.assign(bits, bits + L);
    if (layer_buckets) plan->layer_buckets.assign(layer_buckets, layer_buckets + L);
    plan->with_copies = with_copies;
    plan->shape = cgx::plan_shape(L, off, bits, bucket, dt, layer_buckets);
    std::vector<Tile> tiles;
    std::vector<uint32_t> slots;
    std::vector<int64_t> layer_first;
    cgx::build_tiles(L, off, bits, bucket, dt, chunk, chunks_per_tile, tiles, &slots, &layer_first, layer_buckets,
                     with_copies);
    if (tiles.size() > size_t(0xffffffffu)) return CGX_ERR_SIZE;
    plan->n_tiles = int64_t(tiles.size());
    plan->plan_tiles = plan->n_tiles;
    if (layer_buckets) {
        // The per-layer statistics number the tiles of the WHOLE plan layer by layer; this table
        // holds one launch's share of them, so its tiles take their numbers in that common order.
        std::vector<int64_t> common(size_t(L) + 1, 0);
        for (const Launch &other : launches_of(Buckets{bucket, layer_buckets}, L, off, bits, chunk)) {
            std::vector<Tile> their_tiles;
            std::vector<uint32_t> their_slots;
            std::vector<int64_t> their_first;
            cgx::build_tiles(L, off, bits, other.bucket, dt, chunk, chunks_per_tile, their_tiles, &their_slots, &their_first,
                             layer_buckets, other.with_copies);
            for (int32_t l = 0; l < L; l++) common[size_t(l) + 1] += their_first[size_t(l) + 1] - their_first[size_t(l)];
        }
        for (int32_t l = 0; l < L; l++) common[size_t(l) + 1] += common[size_t(l)];
        if (common[size_t(L)] > int64_t(0xffffffffu)) return CGX_ERR_SIZE;
        for (uint32_t &slot : slots) {
            const size_t l = size_t(std::upper_bound(layer_first.begin(), layer_first.end(), int64_t(slot)) -
                                    layer_first.begin()) - 1;
            slot = uint32_t(common[l] + (int64_t(slot) - layer_first[l]));
        }
        layer_first = common;
        plan->plan_tiles = common[size_t(L)];
    }
    for (const Tile &t : tiles)
        if ((cgx::is_streamed_kind(cgx::tile_kind(t)) || cgx::tile_kind(t) == cgx::kQuantTail) && (t.elem0 & 1))
            plan->odd_tiles = true;
    for (const Tile &t : tiles)
        if (cgx::is_vector_kind(cgx::tile_kind(t)) && (t.elem0 * (dt == CGX_F16 ? 2 : 4)) % 16 != 0)
            plan->aligned_tiles = false;
    int64_t tails = 0;
    for (const Tile &t : tiles) tails += cgx::tile_kind(t) == cgx::kQuantTail;
    // One short end that goes through the generic path is a chain of dependent round trips,
    // bucket after bucket: hidden in a long launch, it outlasts the rest of a short one.
    plan->many_tails = tails > 0 && (plan->n_tiles < 16384 || tails * 512 >= plan->n_tiles);
    if (!upload(&plan->d_tiles, tiles) || !upload(&plan->d_slots, slots) ||
        !upload(&plan->d_layer_first, layer_first)) {
        free_plan(*plan);
        return CGX_ERR_HIP;
    }
    plan->last_use = ++g_clock;
    if (g_plans.size() >= kMaxPlans) {
        // drop the least recently used table that no captured graph reads (if all are pinned the cache grows)
        size_t oldest = g_plans.size();
        for (size_t i = 0; i < g_plans.size(); i++)
            if (!g_plans[i]->pinned && (oldest == g_plans.size() || g_plans[i]->last_use < g_plans[oldest]->last_use))
                oldest = i;
        if (oldest != g_plans.size()) g_plans.erase(g_plans.begin() + long(oldest));
    }
    *out = plan;
    g_plans.push_back(std::move(plan));
    return CGX_OK;
}

// The tables of all launches of a call, looked up before its first launch: a call that fails for a
// missing table (CGX_ERR_CAPTURE) has then queued nothing.
int get_plans(hipStream_t stream, const std::vector<Launch> &launches, int32_t L, const int64_t *off,
              const uint8_t *bits, int dt, int chunk, int chunks_per_tile, const int32_t *layer_buckets,
              std::vector<PlanRef> *out)
{
    out->resize(launches.size());
    for (size_t i = 0; i < launches.size(); i++) {
        const int rc = get_plan(stream, L, off, bits, launches[i].bucket, dt, chunk, chunks_per_tile, &(*out)[i],
                                layer_buckets, launches[i].with_copies);
        if (rc != CGX_OK) return rc;
    }
    return CGX_OK;
}

// Plan check of an entry point: the common rules, and for the norm-and-sign quantizer no
// 1-bit layers (a sign bit alone carries no level).
int check_plan(int scheme, int64_t n, int32_t L, const int64_t *off, const uint8_t *bits, const Buckets &buckets,
               int dt)
{
    int rc = cgx::validate_plan(n, L, off, bits, buckets.per_layer ? 32 : buckets.uniform, dt);
    if (rc != CGX_OK) return rc;
    if (buckets.per_layer) {
        rc = cgx::validate_layer_buckets(L, buckets.per_layer);
        if (rc != CGX_OK) return rc;
    }
    if (scheme == cgx::kSchemeNormSign)
        for (int32_t l = 0; l < L; l++)
            if (bits[l] == 1) return CGX_ERR_BITS;
    return CGX_OK;
}

int quantize_impl(int scheme, const void *grad, int64_t n, int32_t L, const int64_t *off, const uint8_t *bits,
                  const Buckets &buckets, uint64_t seed, int dt, void *packed, void *meta, void *stream)
{
    int rc = check_plan(scheme, n, L, off, bits, buckets, dt);
    if (rc != CGX_OK) return rc;
    if (n == 0) return CGX_OK;
    const cgx::PlanShape shape = cgx::plan_shape(L, off, bits, buckets.uniform, dt, buckets.per_layer);
    if (!grad || !packed || (shape.meta_bytes && !meta)) return CGX_ERR_NULL;
    if (misaligned(grad) || misaligned(packed) || misaligned(meta)) return CGX_ERR_ALIGN;
    const int chunk = chunk_length(kQuantizeCall, dt, buckets);
    const auto launch_quantize = chunk == cgx::chunk_of(2) ? cgx::launch_quantize_g2 : cgx::launch_quantize_g4;
    const std::vector<Launch> launches = launches_of(buckets, L, off, bits, chunk);
    std::vector<PlanRef> plans;
    rc = get_plans(static_cast<hipStream_t>(stream), launches, L, off, bits, dt, chunk, tile_length(kQuantizeCall, dt, n),
                   buckets.per_layer, &plans);
    if (rc != CGX_OK) return rc;
    for (size_t i = 0; i < launches.size(); i++) {
        const Launch &launch = launches[i];
        const PlanRef &plan = plans[i];
        const hipError_t e = launch_quantize(scheme, grad, dt, plan->d_tiles, plan->n_tiles, plan->odd_tiles,
                                                  plan->aligned_tiles, launch.bucket, seed, packed, meta, launch_config(),
                                                  static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return CGX_ERR_HIP;
    }
    return CGX_OK;
}

// Shared body of the dequantize / reduce entry points: out = [local +] deq_0 + ... + deq_{W-1}.
int reduce_impl(int scheme, const void *const *packed, const void *const *meta, int32_t W, int64_t n, int32_t L,
                const int64_t *off, const uint8_t *bits, const Buckets &buckets, int dt, const void *local,
                int local_dt, bool want_local, void *out, int out_dt, void *stream)
{
    int rc = check_plan(scheme, n, L, off, bits, buckets, dt);
    if (rc != CGX_OK) return rc;
    if (W < 1 || W > CGX_MAX_PEERS) return CGX_ERR_PEERS;
    if (n == 0) return CGX_OK;
    const cgx::PlanShape shape = cgx::plan_shape(L, off, bits, buckets.uniform, dt, buckets.per_layer);
    if (!packed || !meta || !out || (want_local && !local)) return CGX_ERR_NULL;
    for (int w = 0; w < W; w++) {
        if (!packed[w] || (shape.meta_bytes && !meta[w])) return CGX_ERR_NULL;
        if (misaligned(packed[w]) || misaligned(meta[w])) return CGX_ERR_ALIGN;
    }
    if (misaligned(out) || misaligned(local)) return CGX_ERR_ALIGN;
    // A decompression (one chunk, nothing to add to) writes eight bytes per byte it reads; a kernel that only
    // moves bytes in that mix sustains 0.75 of the HBM peak with 8 KB written per wave and 0.91 with 4 KB, so it
    // takes the kernel of 1024-element chunks (buckets up to 1024 elements; longer ones keep 2048).
    const bool decompression = W == 1 && !local && launch_config().dequantize_through;
    const bool short_buckets = !buckets.per_layer && buckets.uniform <= 1024;
    const int forced = launch_config().reduce_groups;
    const int chunk = forced > 0 ? (short_buckets ? cgx::chunk_of(forced) : cgx::kDefaultChunk)
                      : decompression && short_buckets && out_dt == CGX_F32 ? cgx::chunk_of(2) : cgx::kDefaultChunk;
    const std::vector<Launch> launches = launches_of(buckets, L, off, bits, chunk);
    std::vector<PlanRef> plans;
    rc = get_plans(static_cast<hipStream_t>(stream), launches, L, off, bits, dt, chunk,
                   tile_length(kOtherCall, dt, n), buckets.per_layer, &plans);
    if (rc != CGX_OK) return rc;
    const auto launch_reduce = chunk == cgx::kDefaultChunk ? cgx::launch_dequant_reduce_g4 : cgx::launch_dequant_reduce_g2;
    for (size_t li = 0; li < launches.size(); li++) {
        const Launch &launch = launches[li];
        const PlanRef &plan = plans[li];
        // peers are folded in order, kPeersPerLaunch at a time, so the sum order is local, 0, 1, ..., W-1;
        // a later launch starts from the binary32 result of the one before (W <= kPeersPerLaunch
        // whenever the output is not binary32: only cgx_dequantize asks for that, with W = 1)
        for (int w0 = 0; w0 < W; w0 += cgx::kPeersPerLaunch) {
            const int k = W - w0 < cgx::kPeersPerLaunch ? W - w0 : cgx::kPeersPerLaunch;
            cgx::PeerPtrs peers{};
            for (int i = 0; i < k; i++) {
                peers.packed[i] = static_cast<const uint8_t *>(packed[w0 + i]);
                peers.meta[i] = static_cast<const float *>(meta[w0 + i]);
            }
            const void *init = w0 == 0 ? local : out;
            const int init_dt = w0 == 0 ? local_dt : CGX_F32;
            // a result that fits the 256 MB memory-side cache with room to spare is left there for the
            // call that consumes it (requantize, the optimizer): measured on 102 MB of sums, the reduce
            // runs 7 % and the requantize after it 10 % faster; on 658 MB the reader loses what the
            // writer gains.  A decompression's stores go through at system scope whatever the size.
            const bool small = int64_t(n) * (out_dt == CGX_F16 ? 2 : 4) <= launch_config().keep_sums_max_bytes;
            const int policy = decompression ? cgx::kStoreThrough : small ? cgx::kStoreKeep : cgx::kStoreStream;
            const hipError_t e = launch_reduce(scheme, peers, k, dt, plan->d_tiles, plan->n_tiles, plan->many_tails,
                                               launch.bucket, init, init_dt, out, out_dt, policy, launch_config(),
                                               static_cast<hipStream_t>(stream));
            if (e != hipSuccess) return CGX_ERR_HIP;
        }
    }
    return CGX_OK;
}

int fused_impl(int scheme, const void *const *packed, const void *const *meta, int32_t W, int64_t n, int32_t L,
               const int64_t *layer_offsets, const uint8_t *bits_per_layer, const Buckets &buckets, int dt,
               uint64_t seed, void *packed_out, void *meta_out, void *stream)
{
    int rc = check_plan(scheme, n, L, layer_offsets, bits_per_layer, buckets, dt);
    if (rc != CGX_OK) return rc;
    if (W < 1 || W > CGX_MAX_FUSED_PEERS) return CGX_ERR_PEERS;
    if (n == 0) return CGX_OK;
    const cgx::PlanShape shape =
        cgx::plan_shape(L, layer_offsets, bits_per_layer, buckets.uniform, dt, buckets.per_layer);
    if (!packed || !meta || !packed_out || (shape.meta_bytes && !meta_out)) return CGX_ERR_NULL;
    for (int w = 0; w < W; w++) {
        if (!packed[w] || (shape.meta_bytes && !meta[w])) return CGX_ERR_NULL;
        if (misaligned(packed[w]) || misaligned(meta[w])) return CGX_ERR_ALIGN;
    }
    if (misaligned(packed_out) || misaligned(meta_out)) return CGX_ERR_ALIGN;
    cgx::PeerPtrs peers{};
    for (int i = 0; i < W; i++) {
        peers.packed[i] = static_cast<const uint8_t *>(packed[i]);
        peers.meta[i] = static_cast<const float *>(meta[i]);
    }
    for (const Launch &launch : launches_of(buckets, L, layer_offsets, bits_per_layer, cgx::kDefaultChunk)) {
        PlanRef in, out;
        rc = get_plan(static_cast<hipStream_t>(stream), L, layer_offsets, bits_per_layer, launch.bucket, dt,
                      cgx::kDefaultChunk, tile_length(kFusedCall, dt, n), &in, buckets.per_layer, launch.with_copies);
        if (rc != CGX_OK) return rc;
        rc = get_plan(static_cast<hipStream_t>(stream), L, layer_offsets, bits_per_layer, launch.bucket, CGX_F32,
                      cgx::kDefaultChunk, tile_length(kFusedCall, dt, n), &out, buckets.per_layer, launch.with_copies);
        if (rc != CGX_OK) return rc;
        if (in->n_tiles != out->n_tiles) return CGX_ERR_SIZE;     // cannot happen: same tiling for both layouts
        const hipError_t e = cgx::launch_dequant_reduce_requantize(
            scheme, peers, W, dt, in->d_tiles, out->d_tiles, in->n_tiles, in->odd_tiles, launch.bucket, seed,
            packed_out, meta_out, launch_config(), static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return CGX_ERR_HIP;
    }
    return CGX_OK;
}

// Number of tiles (= doubles of workspace) of the plan the statistics walk; bits == nullptr:
// the all-pass-through plan cgx_layer_sqnorms uses.
int stats_tiles(int64_t n, int32_t L, const int64_t *off, const uint8_t *bits, int32_t bucket, int dt,
                int64_t *n_tiles)
{
    std::vector<uint8_t> zeros;
    if (!bits) {
        zeros.assign(size_t(L > 0 ? L : 0), 0);
        bits = zeros.data();
        bucket = 32;
    }
    const int rc = cgx::validate_plan(n, L, off, bits, bucket, dt);
    if (rc != CGX_OK) return rc;
    std::vector<Tile> tiles;
    cgx::build_tiles(L, off, bits, bucket, dt, cgx::kDefaultChunk, tile_length(kOtherCall, dt, n), tiles);
    *n_tiles = int64_t(tiles.size());
    return CGX_OK;
}

int sqerrors_impl(int scheme, const void *grad, const void *packed, const void *meta, int64_t n, int32_t L,
                  const int64_t *off, const uint8_t *bits, const Buckets &buckets, int dt, double *sqerr,
                  void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_plan(scheme, n, L, off, bits, buckets, dt);
    if (rc != CGX_OK) return rc;
    if (L == 0) return CGX_OK;
    const cgx::PlanShape shape = cgx::plan_shape(L, off, bits, buckets.uniform, dt, buckets.per_layer);
    if (!sqerr || (n > 0 && (!grad || !packed || !workspace)) || (shape.meta_bytes && !meta)) return CGX_ERR_NULL;
    if (misaligned(grad) || misaligned(packed) || misaligned(meta) || misaligned(workspace) ||
        (reinterpret_cast<uintptr_t>(sqerr) & 7u))
        return CGX_ERR_ALIGN;
    // every launch leaves its tiles' partial sums in the workspace; the last one adds them up layer by layer
    const std::vector<Launch> launches = launches_of(buckets, L, off, bits, cgx::kDefaultChunk);
    std::vector<PlanRef> plans;
    rc = get_plans(static_cast<hipStream_t>(stream), launches, L, off, bits, dt, cgx::kDefaultChunk,
                   tile_length(kOtherCall, dt, n), buckets.per_layer, &plans);
    if (rc != CGX_OK) return rc;
    for (const PlanRef &plan : plans)
        if (workspace_bytes < size_t(plan->plan_tiles) * sizeof(double)) return CGX_ERR_SIZE;
    for (size_t i = 0; i < launches.size(); i++) {
        const PlanRef &plan = plans[i];
        const hipError_t e = cgx::launch_layer_sqerrors(
            scheme, grad, dt, packed, meta, plan->d_tiles, plan->d_slots, plan->n_tiles, plan->aligned_tiles,
            plan->d_layer_first, L,
            static_cast<double *>(workspace), sqerr, launch_config(), static_cast<hipStream_t>(stream),
            i + 1 == launches.size());
        if (e != hipSuccess) return CGX_ERR_HIP;
    }
    return CGX_OK;
}

}  // namespace

extern "C" {

int cgx_sizes(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket,
              cgx_dtype dt, size_t *packed_bytes, size_t *meta_bytes)
{
    const int rc = cgx::validate_plan(n, L, layer_offsets, bits_per_layer, bucket, int(dt));
    if (rc != CGX_OK) return rc;
    const cgx::PlanShape s = cgx::plan_shape(L, layer_offsets, bits_per_layer, bucket, int(dt));
    if (packed_bytes) *packed_bytes = s.packed_bytes;
    if (meta_bytes) *meta_bytes = s.meta_bytes;
    return CGX_OK;
}

int cgx_quantize(const void *grad, int64_t n, int32_t L, const int64_t *layer_offsets,
                 const uint8_t *bits_per_layer, int32_t bucket, uint64_t seed, cgx_dtype dt, void *packed,
                 void *meta, void *stream)
{
    return quantize_impl(cgx::kSchemeMinMax, grad, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, seed, int(dt), packed, meta, stream);
}

int cgx_requantize(const float *sum, int64_t n, int32_t L, const int64_t *layer_offsets,
                   const uint8_t *bits_per_layer, int32_t bucket, uint64_t seed, void *packed, void *meta,
                   void *stream)
{
    return quantize_impl(cgx::kSchemeMinMax, sum, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, seed, CGX_F32, packed, meta, stream);
}

int cgx_dequant_reduce(const void *const *packed, const void *const *meta, int32_t W, int64_t n, int32_t L,
                       const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket, cgx_dtype dt,
                       float *sum, void *stream)
{
    return reduce_impl(cgx::kSchemeMinMax, packed, meta, W, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, int(dt), nullptr, CGX_F32,
                       false, sum, CGX_F32, stream);
}

int cgx_dequant_reduce_add(const void *local, cgx_dtype local_dt, const void *const *packed,
                           const void *const *meta, int32_t W, int64_t n, int32_t L,
                           const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket,
                           cgx_dtype dt, float *sum, void *stream)
{
    if (local_dt != CGX_F32 && local_dt != CGX_F16) return CGX_ERR_DTYPE;
    return reduce_impl(cgx::kSchemeMinMax, packed, meta, W, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, int(dt), local, int(local_dt),
                       true, sum, CGX_F32, stream);
}

int cgx_dequantize(const void *packed, const void *meta, int64_t n, int32_t L, const int64_t *layer_offsets,
                   const uint8_t *bits_per_layer, int32_t bucket, cgx_dtype dt, cgx_dtype out_dt, void *out,
                   void *stream)
{
    if (out_dt != CGX_F32 && out_dt != CGX_F16) return CGX_ERR_DTYPE;
    const void *const p[1] = {packed}, *const m[1] = {meta};
    return reduce_impl(cgx::kSchemeMinMax, p, m, 1, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, int(dt), nullptr, CGX_F32, false, out,
                       int(out_dt), stream);
}

int cgx_dequant_reduce_requantize(const void *const *packed, const void *const *meta, int32_t W, int64_t n,
                                  int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                                  int32_t bucket, cgx_dtype dt, uint64_t seed, void *packed_out, void *meta_out,
                                  void *stream)
{
    return fused_impl(cgx::kSchemeMinMax, packed, meta, W, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, int(dt), seed,
                      packed_out, meta_out, stream);
}

int cgx_layered_sizes(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                      const int32_t *buckets_per_layer, cgx_dtype dt, size_t *packed_bytes, size_t *meta_bytes)
{
    const int rc = check_plan(cgx::kSchemeMinMax, n, L, layer_offsets, bits_per_layer, Buckets{32, buckets_per_layer},
                              int(dt));
    if (rc != CGX_OK) return rc;
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    const cgx::PlanShape s = cgx::plan_shape(L, layer_offsets, bits_per_layer, 32, int(dt), buckets_per_layer);
    if (packed_bytes) *packed_bytes = s.packed_bytes;
    if (meta_bytes) *meta_bytes = s.meta_bytes;
    return CGX_OK;
}

int cgx_layered_quantize(const void *grad, int64_t n, int32_t L, const int64_t *layer_offsets,
                         const uint8_t *bits_per_layer, const int32_t *buckets_per_layer, uint64_t seed,
                         cgx_dtype dt, void *packed, void *meta, void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    return quantize_impl(cgx::kSchemeMinMax, grad, n, L, layer_offsets, bits_per_layer, Buckets{32, buckets_per_layer},
                         seed, int(dt), packed, meta, stream);
}

int cgx_layered_requantize(const float *sum, int64_t n, int32_t L, const int64_t *layer_offsets,
                           const uint8_t *bits_per_layer, const int32_t *buckets_per_layer, uint64_t seed,
                           void *packed, void *meta, void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    return quantize_impl(cgx::kSchemeMinMax, sum, n, L, layer_offsets, bits_per_layer, Buckets{32, buckets_per_layer},
                         seed, CGX_F32, packed, meta, stream);
}

int cgx_layered_dequant_reduce(const void *const *packed, const void *const *meta, int32_t W, int64_t n, int32_t L,
                               const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                               const int32_t *buckets_per_layer, cgx_dtype dt, float *sum, void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    return reduce_impl(cgx::kSchemeMinMax, packed, meta, W, n, L, layer_offsets, bits_per_layer,
                       Buckets{32, buckets_per_layer}, int(dt), nullptr, CGX_F32, false, sum, CGX_F32, stream);
}

int cgx_layered_dequant_reduce_add(const void *local, cgx_dtype local_dt, const void *const *packed,
                                   const void *const *meta, int32_t W, int64_t n, int32_t L,
                                   const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                                   const int32_t *buckets_per_layer, cgx_dtype dt, float *sum, void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    if (local_dt != CGX_F32 && local_dt != CGX_F16) return CGX_ERR_DTYPE;
    return reduce_impl(cgx::kSchemeMinMax, packed, meta, W, n, L, layer_offsets, bits_per_layer,
                       Buckets{32, buckets_per_layer}, int(dt), local, int(local_dt), true, sum, CGX_F32, stream);
}

int cgx_layered_dequantize(const void *packed, const void *meta, int64_t n, int32_t L, const int64_t *layer_offsets,
                           const uint8_t *bits_per_layer, const int32_t *buckets_per_layer, cgx_dtype dt,
                           cgx_dtype out_dt, void *out, void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    if (out_dt != CGX_F32 && out_dt != CGX_F16) return CGX_ERR_DTYPE;
    const void *const p[1] = {packed}, *const m[1] = {meta};
    return reduce_impl(cgx::kSchemeMinMax, p, m, 1, n, L, layer_offsets, bits_per_layer, Buckets{32, buckets_per_layer},
                       int(dt), nullptr, CGX_F32, false, out, int(out_dt), stream);
}

int cgx_layered_dequant_reduce_requantize(const void *const *packed, const void *const *meta, int32_t W, int64_t n,
                                          int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                                          const int32_t *buckets_per_layer, cgx_dtype dt, uint64_t seed,
                                          void *packed_out, void *meta_out, void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    return fused_impl(cgx::kSchemeMinMax, packed, meta, W, n, L, layer_offsets, bits_per_layer,
                      Buckets{32, buckets_per_layer}, int(dt), seed, packed_out, meta_out, stream);
}

int cgx_layered_stats_workspace(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                                const int32_t *buckets_per_layer, cgx_dtype dt, size_t *bytes)
{
    if (!bytes || (L > 0 && !buckets_per_layer)) return CGX_ERR_NULL;
    const Buckets buckets{32, buckets_per_layer};
    const int rc = check_plan(cgx::kSchemeMinMax, n, L, layer_offsets, bits_per_layer, buckets, int(dt));
    if (rc != CGX_OK) return rc;
    size_t tiles_of_plan = 0;
    for (const Launch &launch : launches_of(buckets, L, layer_offsets, bits_per_layer, cgx::kDefaultChunk)) {
        std::vector<Tile> tiles;
        cgx::build_tiles(L, layer_offsets, bits_per_layer, launch.bucket, int(dt), cgx::kDefaultChunk,
                         tile_length(kOtherCall, int(dt), n),
                         tiles, nullptr, nullptr, buckets_per_layer, launch.with_copies);
        tiles_of_plan += tiles.size();
    }
    *bytes = tiles_of_plan * sizeof(double);
    return CGX_OK;
}

int cgx_layered_layer_sqerrors(const void *grad, const void *packed, const void *meta, int64_t n, int32_t L,
                               const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                               const int32_t *buckets_per_layer, cgx_dtype dt, double *sqerr, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    return sqerrors_impl(cgx::kSchemeMinMax, grad, packed, meta, n, L, layer_offsets, bits_per_layer,
                         Buckets{32, buckets_per_layer}, int(dt), sqerr, workspace, workspace_bytes, stream);
}

int cgx_qsgd_sizes(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                   int32_t bucket, cgx_dtype dt, size_t *packed_bytes, size_t *meta_bytes)
{
    const int rc = check_plan(cgx::kSchemeNormSign, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, int(dt));
    if (rc != CGX_OK) return rc;
    const cgx::PlanShape s = cgx::plan_shape(L, layer_offsets, bits_per_layer, bucket, int(dt));
    if (packed_bytes) *packed_bytes = s.packed_bytes;
    if (meta_bytes) *meta_bytes = s.meta_bytes / 2;            // one float per bucket
    return CGX_OK;
}

int cgx_qsgd_quantize(const void *grad, int64_t n, int32_t L, const int64_t *layer_offsets,
                      const uint8_t *bits_per_layer, int32_t bucket, uint64_t seed, cgx_dtype dt, void *packed,
                      void *meta, void *stream)
{
    return quantize_impl(cgx::kSchemeNormSign, grad, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, seed, int(dt),
                         packed, meta, stream);
}

int cgx_qsgd_dequant_reduce(const void *const *packed, const void *const *meta, int32_t W, int64_t n, int32_t L,
                            const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket,
                            cgx_dtype dt, float *sum, void *stream)
{
    return reduce_impl(cgx::kSchemeNormSign, packed, meta, W, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, int(dt),
                       nullptr, CGX_F32, false, sum, CGX_F32, stream);
}

int cgx_qsgd_dequant_reduce_requantize(const void *const *packed, const void *const *meta, int32_t W, int64_t n,
                                       int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                                       int32_t bucket, cgx_dtype dt, uint64_t seed, void *packed_out,
                                       void *meta_out, void *stream)
{
    return fused_impl(cgx::kSchemeNormSign, packed, meta, W, n, L, layer_offsets, bits_per_layer, Buckets{bucket, nullptr}, int(dt),
                      seed, packed_out, meta_out, stream);
}

int cgx_qsgd_layered_sizes(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                           const int32_t *buckets_per_layer, cgx_dtype dt, size_t *packed_bytes, size_t *meta_bytes)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    const int rc = check_plan(cgx::kSchemeNormSign, n, L, layer_offsets, bits_per_layer, Buckets{32, buckets_per_layer},
                              int(dt));
    if (rc != CGX_OK) return rc;
    const cgx::PlanShape s = cgx::plan_shape(L, layer_offsets, bits_per_layer, 32, int(dt), buckets_per_layer);
    if (packed_bytes) *packed_bytes = s.packed_bytes;
    if (meta_bytes) *meta_bytes = s.meta_bytes / 2;
    return CGX_OK;
}

int cgx_qsgd_layered_quantize(const void *grad, int64_t n, int32_t L, const int64_t *layer_offsets,
                              const uint8_t *bits_per_layer, const int32_t *buckets_per_layer, uint64_t seed,
                              cgx_dtype dt, void *packed, void *meta, void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    return quantize_impl(cgx::kSchemeNormSign, grad, n, L, layer_offsets, bits_per_layer,
                         Buckets{32, buckets_per_layer}, seed, int(dt), packed, meta, stream);
}

int cgx_qsgd_layered_dequant_reduce(const void *const *packed, const void *const *meta, int32_t W, int64_t n,
                                    int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                                    const int32_t *buckets_per_layer, cgx_dtype dt, float *sum, void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    return reduce_impl(cgx::kSchemeNormSign, packed, meta, W, n, L, layer_offsets, bits_per_layer,
                       Buckets{32, buckets_per_layer}, int(dt), nullptr, CGX_F32, false, sum, CGX_F32, stream);
}

int cgx_qsgd_layered_dequant_reduce_requantize(const void *const *packed, const void *const *meta, int32_t W,
                                               int64_t n, int32_t L, const int64_t *layer_offsets,
                                               const uint8_t *bits_per_layer, const int32_t *buckets_per_layer,
                                               cgx_dtype dt, uint64_t seed, void *packed_out, void *meta_out,
                                               void *stream)
{
    if (L > 0 && !buckets_per_layer) return CGX_ERR_NULL;
    return fused_impl(cgx::kSchemeNormSign, packed, meta, W, n, L, layer_offsets, bits_per_layer,
                      Buckets{32, buckets_per_layer}, int(dt), seed, packed_out, meta_out, stream);
}

int cgx_layer_stats_workspace(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                              int32_t bucket, cgx_dtype dt, size_t *bytes)
{
    if (!bytes) return CGX_ERR_NULL;
    int64_t n_tiles = 0;
    const int rc = stats_tiles(n, L, layer_offsets, bits_per_layer, bucket, int(dt), &n_tiles);
    if (rc != CGX_OK) return rc;
    *bytes = size_t(n_tiles) * sizeof(double);
    return CGX_OK;
}

int cgx_layer_sqnorms(const void *buf, int64_t n, int32_t L, const int64_t *layer_offsets, cgx_dtype dt,
                      double *sqnorm, void *workspace, size_t workspace_bytes, void *stream)
{
    const std::vector<uint8_t> zeros(size_t(L > 0 ? L : 0), 0);
    int rc = cgx::validate_plan(n, L, layer_offsets, zeros.data(), 32, int(dt));
    if (rc != CGX_OK) return rc;
    if (L == 0) return CGX_OK;
    if (!sqnorm || (n > 0 && (!buf || !workspace))) return CGX_ERR_NULL;
    if (misaligned(buf) || misaligned(workspace) || (reinterpret_cast<uintptr_t>(sqnorm) & 7u)) return CGX_ERR_ALIGN;
    PlanRef plan;
    rc = get_plan(static_cast<hipStream_t>(stream), L, layer_offsets, zeros.data(), 32, int(dt), cgx::kDefaultChunk,
                  tile_length(kOtherCall, int(dt), n), &plan);
    if (rc != CGX_OK) return rc;
    if (workspace_bytes < size_t(plan->n_tiles) * sizeof(double)) return CGX_ERR_SIZE;
    const hipError_t e = cgx::launch_layer_sqnorms(buf, int(dt), plan->d_tiles, plan->d_slots, plan->n_tiles,
                                                   plan->d_layer_first, L, static_cast<double *>(workspace), sqnorm,
                                                   launch_config(), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CGX_OK : CGX_ERR_HIP;
}

int cgx_layer_sqnorms_noalloc(const void *buf, int64_t n, int32_t L, const int64_t *layer_offsets, cgx_dtype dt,
                              double *sqnorm, void *stream)
{
    // the checks of validate_plan that concern the layer table (this call has no widths), without
    // the heap: nothing here allocates
    if (n < 0 || L < 0) return CGX_ERR_SIZE;
    if (L > 0 && !layer_offsets) return CGX_ERR_NULL;
    if (dt != CGX_F32 && dt != CGX_F16) return CGX_ERR_DTYPE;
    if (L == 0) return n == 0 ? CGX_OK : CGX_ERR_SIZE;
    if (layer_offsets[0] != 0) return CGX_ERR_OFFSETS;
    for (int32_t l = 0; l < L; l++)
        if (layer_offsets[l + 1] < layer_offsets[l]) return CGX_ERR_OFFSETS;
    if (layer_offsets[L] != n || n / 32 > int64_t(0xfffffff0u)) return CGX_ERR_SIZE;
    if (L > CGX_NOALLOC_MAX_LAYERS) return CGX_ERR_CAPACITY;
    // number of each layer's first work item: runs of kCopyTile elements, layer by layer
    static thread_local int64_t first[CGX_NOALLOC_MAX_LAYERS + 1];
    first[0] = 0;
    for (int32_t l = 0; l < L; l++)
        first[l + 1] = first[l] + (layer_offsets[l + 1] - layer_offsets[l] + cgx::kCopyTile - 1) / cgx::kCopyTile;
    if (first[L] > CGX_NOALLOC_MAX_TILES) return CGX_ERR_CAPACITY;
    if (!sqnorm || (n > 0 && !buf)) return CGX_ERR_NULL;
    if (misaligned(buf) || (reinterpret_cast<uintptr_t>(sqnorm) & 7u)) return CGX_ERR_ALIGN;
    const hipError_t e = cgx::launch_layer_sqnorms_noalloc(buf, int(dt), layer_offsets, first, L, sqnorm,
                                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CGX_OK : CGX_ERR_HIP;
}

int cgx_layer_sqerrors(const void *grad, const void *packed, const void *meta, int64_t n, int32_t L,
                       const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket, cgx_dtype dt,
                       double *sqerr, void *workspace, size_t workspace_bytes, void *stream)
{
    return sqerrors_impl(cgx::kSchemeMinMax, grad, packed, meta, n, L, layer_offsets, bits_per_layer,
                         Buckets{bucket, nullptr}, int(dt), sqerr, workspace, workspace_bytes, stream);
}

int cgx_qsgd_layer_sqerrors(const void *grad, const void *packed, const void *meta, int64_t n, int32_t L,
                            const int64_t *layer_offsets, const uint8_t *bits_per_layer, int32_t bucket,
                            cgx_dtype dt, double *sqerr, void *workspace, size_t workspace_bytes, void *stream)
{
    return sqerrors_impl(cgx::kSchemeNormSign, grad, packed, meta, n, L, layer_offsets, bits_per_layer,
                         Buckets{bucket, nullptr}, int(dt), sqerr, workspace, workspace_bytes, stream);
}

int cgx_plan_tiles(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                   int32_t bucket, cgx_dtype dt, void *tiles_out, int64_t capacity, int64_t *n_tiles)
{
    return cgx_plan_tiles_chunk(n, L, layer_offsets, bits_per_layer, bucket, dt, cgx::kDefaultChunk, tiles_out, capacity,
                                n_tiles);
}

int cgx_plan_tiles_chunk(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                         int32_t bucket, cgx_dtype dt, int32_t chunk_elements, void *tiles_out, int64_t capacity,
                         int64_t *n_tiles)
{
    const int rc = cgx::validate_plan(n, L, layer_offsets, bits_per_layer, bucket, int(dt));
    if (rc != CGX_OK) return rc;
    if (chunk_elements != cgx::chunk_of(2) && chunk_elements != cgx::chunk_of(4)) return CGX_ERR_SIZE;
    if (!n_tiles || (capacity > 0 && !tiles_out)) return CGX_ERR_NULL;
    std::vector<Tile> tiles;
    cgx::build_tiles(L, layer_offsets, bits_per_layer, bucket, int(dt), chunk_elements, 1, tiles);
    *n_tiles = int64_t(tiles.size());
    const int64_t k = capacity < *n_tiles ? capacity : *n_tiles;
    if (k > 0) std::memcpy(tiles_out, tiles.data(), size_t(k) * sizeof(Tile));
    return CGX_OK;
}

int cgx_stream_probe_shaped(const void *src, size_t read_bytes, void *dst, size_t write_bytes,
                            const cgx_probe_shape *shape, void *stream)
{
    if (!shape || (read_bytes && !src) || (write_bytes && !dst)) return CGX_ERR_NULL;
    if (read_bytes % 16 || write_bytes % 16) return CGX_ERR_SIZE;
    if (misaligned(src) || misaligned(dst)) return CGX_ERR_ALIGN;
    const int32_t s = shape->slice_bytes, t = shape->block_threads;
    if (s < 1024 || s > (1 << 20) || (s & (s - 1)) || (t != 64 && t != 128 && t != 256 && t != 512 && t != 1024) ||
        shape->load_policy < 0 || shape->load_policy > 3 || shape->store_policy < 0 || shape->store_policy > 4 ||
        (shape->xcd_contiguous != 0 && shape->xcd_contiguous != 1) || shape->max_blocks < 0 ||
        (shape->paired_loads != 0 && shape->paired_loads != 1) || shape->alu_ops_per_pass < 0 ||
        shape->alu_ops_per_pass > 65536 || shape->lds_bytes_per_block < 0 || shape->lds_bytes_per_block > 65536)
        return CGX_ERR_SIZE;
    cgx::ProbeShape k;
    k.slice_bytes = s;
    k.block_threads = t;
    k.load_policy = shape->load_policy;
    k.store_policy = shape->store_policy;
    k.xcd_contiguous = shape->xcd_contiguous;
    k.max_blocks = shape->max_blocks;
    k.paired_loads = shape->paired_loads;
    k.alu_ops_per_pass = shape->alu_ops_per_pass;
    k.lds_bytes_per_block = shape->lds_bytes_per_block;
    const hipError_t e = cgx::launch_stream_probe(src, read_bytes, dst, write_bytes, k, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CGX_OK : CGX_ERR_HIP;
}

int cgx_stream_probe(const void *src, size_t read_bytes, void *dst, size_t write_bytes, void *stream)
{
    const cgx_probe_shape shape = {8192, 256, 1, 1, 0, 0, 0, 0, 0};      // the kernels' own style
    return cgx_stream_probe_shaped(src, read_bytes, dst, write_bytes, &shape, stream);
}

const char *cgx_issue_probe_form(int32_t form) { return cgx::issue_probe_form(form); }

int cgx_issue_probe(int32_t form, int32_t blocks, int32_t iterations, void *out, size_t out_bytes, void *stream)
{
    if (!out) return CGX_ERR_NULL;
    if (!cgx::issue_probe_form(form) || blocks < 1 || blocks > 65536 || iterations < 1 || iterations > (1 << 20) ||
        out_bytes < size_t(blocks) * 256 * 4)
        return CGX_ERR_SIZE;
    if (misaligned(out)) return CGX_ERR_ALIGN;
    const hipError_t e = cgx::launch_issue_probe(form, blocks, iterations, out, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CGX_OK : CGX_ERR_HIP;
}

const char *cgx_status_string(int status)
{
    switch (status) {
    case CGX_OK: return "ok";
    case CGX_ERR_NULL: return "a required pointer is NULL";
    case CGX_ERR_SIZE: return "n or L is negative, too large, or n does not match layer_offsets[L]";
    case CGX_ERR_OFFSETS: return "layer_offsets must start at 0 and never decrease";
    case CGX_ERR_BITS: return "bits_per_layer entries must be 0 (pass-through) or 1..8 (2..8 for the cgx_qsgd_ calls)";
    case CGX_ERR_BUCKET: return "bucket must be a multiple of 32 in [32, 8192]";
    case CGX_ERR_PEERS: return "W must be in [1, 64]";
    case CGX_ERR_DTYPE: return "unknown storage type";
    case CGX_ERR_HIP: return "the HIP runtime reported an error";
    case CGX_ERR_ALIGN: return "device pointers must be 16-byte aligned";
    case CGX_ERR_CAPTURE: return "the stream is capturing a graph and this plan's tables do not exist yet: run the call "
                                 "once outside the capture first";
    case CGX_ERR_CAPACITY: return "the plan exceeds the fixed tables of a no-allocation entry point "
                                  "(CGX_NOALLOC_MAX_LAYERS layers, CGX_NOALLOC_MAX_TILES work items)";
    default: return "unknown status";
    }
}

int cgx_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    int rc = CGX_OK;
    // the tables go away with their last owner; hipFree waits for work that still reads them
    g_plans.clear();
    return rc;
}

}  // extern "C"
