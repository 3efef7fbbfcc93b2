// Per-layer statistics of the adaptive scheme: kernels and launchers.
#include <mutex>

#include "cgx_device_reduce.h"

// Layout of the device array behind cgx_layer_sqnorms_noalloc (see the kernels further down):
// the layer table, the tile table with its numbering, and one partial sum per tile.
namespace cgx {
namespace {
constexpr int kStaticLayers = CGX_NOALLOC_MAX_LAYERS;
constexpr int64_t kStaticTiles = CGX_NOALLOC_MAX_TILES;

constexpr size_t round256(size_t v) { return (v + 255) & ~size_t(255); }

struct StaticLayout {                        // offsets into the array, each a multiple of 256 bytes
    static constexpr size_t kTable = (size_t(kStaticLayers) + 1) * sizeof(int64_t);
    static constexpr size_t off = 0;                                                  // int64 [L + 1]
    static constexpr size_t first = off + round256(kTable);                              // int64 [L + 1]
    static constexpr size_t partial = first + round256(kTable);                          // double [tiles]
    static constexpr size_t slots = partial + round256(size_t(kStaticTiles) * sizeof(double));     // uint32 [tiles]
    static constexpr size_t tiles = slots + round256(size_t(kStaticTiles) * sizeof(uint32_t));     // Tile [tiles]
    static constexpr size_t bytes = tiles + round256(size_t(kStaticTiles) * sizeof(Tile));
};

}  // namespace
}  // namespace cgx

// One copy per device, held from the load of the library's code until the process ends.  Host
// code never uses this name as an address: it asks the runtime for the array's device address
// (static_scratch below) and passes that to the kernels.
static __device__ __align__(256) unsigned char scratch[cgx::StaticLayout::bytes];

namespace cgx {
namespace {

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

// Sum of squares of a run of elements of the buffer (a tile of a pass-through plan: at most kCopyTile
// elements), formed by the kNormWaves waves of a block: each wave takes kCopyTile / kNormWaves
// elements (4 KB of binary32: the slice size at which a wave that only reads runs closest to the
// memory's peak; eight times that per wave reached 0.78 of it).
// Elements that no 16-byte load may fetch (a tile off the vector grid, or its last few) go to
// wave 0, one per lane and pass.
constexpr int kNormWaves = 8;
constexpr int kNormBlock = kNormWaves * kWave;

// 16 bytes as stored, widened.
template <int DT>
__device__ __forceinline__ double square_sum16(const uint4v &v)
{
    double s = 0.0;
    if (DT == CGX_F16) {
        const half8v h = __builtin_bit_cast(half8v, v);
#pragma unroll
        for (int j = 0; j < 8; j++) s += square(float(h[j]));
    } else {
        const float4v f = __builtin_bit_cast(float4v, v);
#pragma unroll
        for (int j = 0; j < 4; j++) s += square(f[j]);
    }
    return s;
}

template <int DT>
__device__ __forceinline__ double sqnorm_share(const void *__restrict__ buf, const Tile &tile, bool fast, int wave, int lane)
{
    // which lane squares which element does not matter to the sum: every load instruction takes 1 KB of
    // consecutive addresses, 16 bytes per lane
    constexpr uint32_t kPerVec = DT == CGX_F16 ? 8 : 4;
    constexpr int kLoads = kCopyTile / kNormWaves / kPerVec / kWave;       // per lane: 4 (binary32) or 2
    double s = 0.0;
    const uint32_t vecs = fast ? tile.count / kPerVec : 0;
    const uint32_t v0 = uint32_t(wave) * (kLoads * kWave);
    if (v0 < vecs) {
        // aligned like an element, not like a vector: a layer may start anywhere
        using Vec = std::conditional_t<DT == CGX_F16, uint4u2, uint4u4>;
        const Vec *base = reinterpret_cast<const Vec *>(static_cast<const uint8_t *>(buf) +
                                                        tile.elem0 * int64_t(DT == CGX_F16 ? 2 : 4));
        uint4v raw[kLoads];
#pragma unroll
        for (int u = 0; u < kLoads; u++) {
            const uint32_t v = v0 + u * kWave + lane;
            raw[u] = __builtin_nontemporal_load(base + (v < vecs ? v : v0));      // clamped; masked below
        }
#pragma unroll
        for (int u = 0; u < kLoads; u++)
            if (v0 + u * kWave + lane < vecs) s += square_sum16<DT>(raw[u]);
    }
    if (wave == 0)
        for (uint32_t j = vecs * kPerVec + lane; j < tile.count; j += kWave) s += square(load_elem<DT>(buf, tile.elem0 + j));
    return s;
}

// One block per tile; the waves' sums meet in LDS and are added in wave order.
template <int DT>
__global__ __launch_bounds__(kNormBlock) void sqnorm_kernel(const void *__restrict__ buf,
                                                             const Tile *__restrict__ tiles,
                                                             const uint32_t *__restrict__ slots, int64_t n_tiles,
                                                             double *__restrict__ partial)
{
    __shared__ double sums[kNormWaves];
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = int(threadIdx.x) & 63;
    for (int64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const Tile tile = tiles[t];
        const double s = wave_sum(sqnorm_share<DT>(buf, tile, tile_kind(tile) == kCopyFast, wave, lane));
        if (lane == 0) sums[wave] = s;
        __syncthreads();
        if (threadIdx.x == 0) {
            double total = sums[0];
#pragma unroll
            for (int w = 1; w < kNormWaves; w++) total += sums[w];
            partial[slots[t]] = total;
        }
        __syncthreads();                     // sums is free again before the next tile's results arrive
    }
}

// Blocks of the norm kernel: one per tile unless the configuration caps the grid.
inline unsigned norm_grid(int64_t n_tiles, const LaunchConfig &cfg)
{
    int64_t blocks = n_tiles;
    if (cfg.max_blocks > 0 && blocks > cfg.max_blocks) blocks = cfg.max_blocks;
    if (blocks > 0x7fffffff) blocks = 0x7fffffff;
    return unsigned(blocks);
}

// Squared error of a vectorised tile: the codes are decoded as in the reduce (one peer) and
// compared with the gradient they were cut from.
// VIA_LDS: every vectorised tile starts on a 16-byte boundary of the buffer (a property of the tile
// table; the host picks the instantiation).  The chunk of the gradient then comes in through LDS, 1 KB of
// consecutive bytes per load instruction, into an area of its own (x_stage) while the codes go to
// theirs, both in flight together; otherwise each lane loads its groups straight into registers.
template <int SCHEME, int DT, int BITS, bool VIA_LDS, typename Peers>
__device__ __forceinline__ double sqerror_fast(const void *__restrict__ grad, Peers &chunk,
                                               const Tile &tile, int bucket, int lane, uint4v *stage, uint4v *x_stage)
{
    constexpr int S = DT == CGX_F16 ? 2 : 4;
    constexpr int kVecs = kChunk * S / 16;
    const LaneMap map(tile, bucket, lane);
    const int chunks = int(tile.count / kChunk);
    const int buckets_per_chunk = kChunk / bucket;
    double s = 0.0;
    for (int c = 0; c < chunks; c++) {
        const int64_t first = tile.elem0 + int64_t(c) * kChunk;
        float x[G][8], v[G][8];
        if constexpr (VIA_LDS) {
            const uint4v *src = reinterpret_cast<const uint4v *>(reinterpret_cast<const uint8_t *>(grad) + first * S);
#pragma unroll
            for (int k = 0; k < kVecs / kWave; k++) load_to_lds16(src + k * kWave + lane, x_stage + k * kWave);
        } else {
#pragma unroll
            for (int r = 0; r < G; r++) load8<DT>(grad, first + map.group(r), x[r]);
        }
        clear_sums(v);
        // (waits for every load of this wave, the gradient's included)
        reduce_chunk<SCHEME, BITS>(chunk, 1, tile.packed_off + int64_t(c) * (kChunk * BITS / 8),
                                   tile.bucket0 + c * buckets_per_chunk + map.bi, map, v, stage, lane);
        if constexpr (VIA_LDS) {
#pragma unroll
            for (int r = 0; r < G; r++) {
                if (DT == CGX_F16) {
                    const half8v h = *reinterpret_cast<const half8v *>(reinterpret_cast<const _Float16 *>(x_stage) + map.group(r));
#pragma unroll
                    for (int j = 0; j < 8; j++) x[r][j] = float(h[j]);
                } else {
                    const float4v *p = reinterpret_cast<const float4v *>(reinterpret_cast<const float *>(x_stage) + map.group(r));
                    const float4v a = p[0], b = p[1];
#pragma unroll
                    for (int j = 0; j < 4; j++) {
                        x[r][j] = a[j];
                        x[r][4 + j] = b[j];
                    }
                }
            }
            wave_lds_fence();                // before the next chunk overwrites the area
        }
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

// LDS per wave: the staging area of one peer's codes (at most kChunk bytes, plus what the odd widths
// read past their last group), and with VIA_LDS a chunk of the gradient before it.
constexpr int kErrorCodeVecs = kChunk / 16;
constexpr int kErrorChunkVecs = kChunk / 4;

template <int SCHEME, int DT, bool VIA_LDS>
__global__ __launch_bounds__(kBlock) void sqerror_kernel(const PeerPtrs chunk_argument, const void *__restrict__ grad,
                                                          const Tile *__restrict__ tiles,
                                                          const uint32_t *__restrict__ slots, int64_t n_tiles,
                                                          double *__restrict__ partial)
{
    (void)chunk_argument;
    KernargPeers &chunk = first_kernel_argument();
    constexpr int kPerWave = VIA_LDS ? kErrorChunkVecs + kErrorCodeVecs : kErrorChunkVecs;
    __shared__ uint4v stage_all[kWavesPerBlock][kPerWave];
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = int(threadIdx.x) & 63;
    uint4v *x_stage = stage_all[wave];
    uint4v *stage = VIA_LDS ? x_stage + kErrorChunkVecs : x_stage;
    const int64_t stride = int64_t(gridDim.x) * kWavesPerBlock;
    for (int64_t t = int64_t(blockIdx.x) * kWavesPerBlock + wave; t < n_tiles; t += stride) {
        const Tile tile = tiles[t];
        const int bucket = tile_bucket(tile);
        const uint32_t kind = tile_kind(tile);
        double s = 0.0;                              // pass-through tiles: no error
        if (is_vector_kind(kind)) {
            CGX_FOR_BITS(tile_bits(tile),
                         (s = sqerror_fast<SCHEME, DT, BITS, VIA_LDS>(grad, chunk, tile, bucket, lane, stage, x_stage)))
        } else if (kind == kQuantSlow || kind == kQuantTail || kind == kQuantAny) {
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

// ---------------------------------------------------------------- statistics without allocations
//
// cgx_layer_sqnorms_noalloc: the tile table, its numbering and the partial sums live in a
// file-scope device array instead of library-allocated tables and a caller workspace, for callers
// that cannot allocate.  The layer table reaches the device through kernel arguments (a few
// hundred entries per launch), so that the call copies nothing from host memory on the stream;
// a kernel expands it into the same tile table the allocating call builds on the host, and the
// two statistics kernels above do the rest.

// A slice of the layer table as a kernel argument: layer offsets and first tile numbers.
constexpr int kSliceEntries = 192;
struct TableSlice {
    int64_t off[kSliceEntries];
    int64_t first[kSliceEntries];
};

// Entries [at, at + count) of both tables, from the kernel's arguments (the slice is the first
// parameter: read where the dispatch put it, indexed by the thread).
__global__ __launch_bounds__(kSliceEntries) void table_slice_kernel(const TableSlice slice_argument, int count, int at,
                                                                      int64_t *__restrict__ off,
                                                                      int64_t *__restrict__ first)
{
    (void)slice_argument;
    const __attribute__((address_space(4))) TableSlice &slice =
        *(const __attribute__((address_space(4))) TableSlice *)__builtin_amdgcn_kernarg_segment_ptr();
    const int i = int(threadIdx.x);
    if (i < count) {
        off[at + i] = slice.off[i];
        first[at + i] = slice.first[i];
    }
}

// The tiles of an all-pass-through plan, layer by layer (one block per layer): runs of kCopyTile
// elements, numbered in table order -- what build_tiles gives for such a plan.
__global__ __launch_bounds__(kBlock) void expand_tiles_kernel(const int64_t *__restrict__ off,
                                                               const int64_t *__restrict__ first,
                                                               Tile *__restrict__ tiles, uint32_t *__restrict__ slots)
{
    const int64_t l = blockIdx.x;
    const int64_t e0 = off[l], len = off[l + 1] - e0, a = first[l], b = first[l + 1];
    for (int64_t t = a + int(threadIdx.x); t < b; t += kBlock) {
        const int64_t j = (t - a) * kCopyTile;
        Tile tile{};
        tile.elem0 = e0 + j;
        tile.count = uint32_t(len - j < kCopyTile ? len - j : kCopyTile);
        tile.info = uint32_t(kCopyFast) << 4;
        tiles[t] = tile;
        slots[t] = uint32_t(t);
    }
}

// Device address of this device's copy of the array (looked up once per device).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char *g_scratch_ptr[kMaxDevices] = {};

hipError_t static_scratch(unsigned char **ptr)
{
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<unsigned char *>(p);
    }
    *ptr = g_scratch_ptr[device];
    return hipSuccess;
}

}  // namespace

hipError_t launch_layer_sqnorms(const void *buf, int dt, const Tile *tiles, const uint32_t *slots, int64_t n_tiles,
                                const int64_t *layer_first, int32_t L, double *partial, double *out,
                                const LaunchConfig &cfg, hipStream_t stream)
{
    if (L == 0) return hipSuccess;
    if (n_tiles > 0) {
        const auto kernel = dt == CGX_F16 ? sqnorm_kernel<CGX_F16> : sqnorm_kernel<CGX_F32>;
        hipLaunchKernelGGL(kernel, dim3(norm_grid(n_tiles, cfg)), dim3(kNormBlock), 0, stream, buf, tiles, slots, n_tiles,
                           partial);
    }
    hipLaunchKernelGGL(layer_sum_kernel, dim3(unsigned(L)), dim3(kSumBlock), 0, stream,
                       static_cast<const double *>(partial), layer_first, out);
    return hipGetLastError();
}

hipError_t launch_layer_sqnorms_noalloc(const void *buf, int dt, const int64_t *off, const int64_t *first, int32_t L,
                                        double *out, hipStream_t stream)
{
    if (L == 0) return hipSuccess;
    unsigned char *base = nullptr;
    const hipError_t e = static_scratch(&base);
    if (e != hipSuccess) return e;
    int64_t *d_off = reinterpret_cast<int64_t *>(base + StaticLayout::off);
    int64_t *d_first = reinterpret_cast<int64_t *>(base + StaticLayout::first);
    double *d_partial = reinterpret_cast<double *>(base + StaticLayout::partial);
    uint32_t *d_slots = reinterpret_cast<uint32_t *>(base + StaticLayout::slots);
    Tile *d_tiles = reinterpret_cast<Tile *>(base + StaticLayout::tiles);
    for (int at = 0; at <= L; at += kSliceEntries) {
        TableSlice slice{};
        const int count = L + 1 - at < kSliceEntries ? L + 1 - at : kSliceEntries;
        for (int i = 0; i < count; i++) {
            slice.off[i] = off[at + i];
            slice.first[i] = first[at + i];
        }
        hipLaunchKernelGGL(table_slice_kernel, dim3(1), dim3(kSliceEntries), 0, stream, slice, count, at, d_off, d_first);
    }
    const int64_t n_tiles = first[L];
    if (n_tiles > 0) {
        hipLaunchKernelGGL(expand_tiles_kernel, dim3(unsigned(L)), dim3(kBlock), 0, stream,
                           static_cast<const int64_t *>(d_off), static_cast<const int64_t *>(d_first), d_tiles, d_slots);
        const auto kernel = dt == CGX_F16 ? sqnorm_kernel<CGX_F16> : sqnorm_kernel<CGX_F32>;
        hipLaunchKernelGGL(kernel, dim3(norm_grid(n_tiles, LaunchConfig{})), dim3(kNormBlock), 0, stream, buf,
                           static_cast<const Tile *>(d_tiles), static_cast<const uint32_t *>(d_slots), n_tiles, d_partial);
    }
    hipLaunchKernelGGL(layer_sum_kernel, dim3(unsigned(L)), dim3(kSumBlock), 0, stream,
                       static_cast<const double *>(d_partial), static_cast<const int64_t *>(d_first), out);
    return hipGetLastError();
}

hipError_t launch_layer_sqerrors(int scheme, const void *grad, int dt, const void *packed, const void *meta,
                                 const Tile *tiles, const uint32_t *slots, int64_t n_tiles, bool aligned_tiles,
                                 const int64_t *layer_first, int32_t L, double *partial,
                                 double *out, const LaunchConfig &cfg, hipStream_t stream, bool sum_layers)
{
    if (L == 0) return hipSuccess;
    const dim3 block(kBlock);
    if (n_tiles > 0) {
        const dim3 grid(grid_for(n_tiles, cfg));
        PeerPtrs chunk{};
        chunk.packed[0] = static_cast<const uint8_t *>(packed);
        chunk.meta[0] = static_cast<const float *>(meta);
        using Kernel = void (*)(const PeerPtrs, const void *, const Tile *, const uint32_t *, int64_t, double *);
        static const Kernel table[2][2][2] = {
            {{sqerror_kernel<kMinMax, CGX_F32, false>, sqerror_kernel<kMinMax, CGX_F32, true>},
             {sqerror_kernel<kMinMax, CGX_F16, false>, sqerror_kernel<kMinMax, CGX_F16, true>}},
            {{sqerror_kernel<kNormSign, CGX_F32, false>, sqerror_kernel<kNormSign, CGX_F32, true>},
             {sqerror_kernel<kNormSign, CGX_F16, false>, sqerror_kernel<kNormSign, CGX_F16, true>}}};
        const Kernel kernel = table[scheme == kSchemeNormSign][dt == CGX_F16][aligned_tiles && cfg.via_lds];
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, chunk, grad, tiles, slots, n_tiles, partial);
    }
    if (sum_layers)
        hipLaunchKernelGGL(layer_sum_kernel, dim3(unsigned(L)), dim3(kSumBlock), 0, stream,
                           static_cast<const double *>(partial), layer_first, out);
    return hipGetLastError();
}

}  // namespace cgx
