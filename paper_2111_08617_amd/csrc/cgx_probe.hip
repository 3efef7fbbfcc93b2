// The streaming probe (include/cgx_diag.h): a kernel that only moves bytes, with the access
// style of the method's kernels (lane-contiguous 16-byte vectors, 1 KB per instruction and wave)
// and a launch shape and cache policies chosen by the caller.  A measurement aid: what it
// sustains at a given size and read:write mix is the ceiling the memory system sets for a
// streaming kernel of that shape.
#include "cgx_device.h"

namespace cgx {
namespace {

// The cache-policy bits are part of the instruction, so the accesses are written out.  The
// compiler does not track loads issued this way: wait_loads() stands between them and the first
// use of their results.
template <int POLICY>
__device__ __forceinline__ void probe_load(uint4v &v, const uint4v *p)
{
    if (POLICY == 0) asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p) : "memory");
    if (POLICY == 1) asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(v) : "v"(p) : "memory");
    if (POLICY == 2) asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
    if (POLICY == 3) asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1" : "=v"(v) : "v"(p) : "memory");
}

template <int POLICY>
__device__ __forceinline__ void probe_store(uint4v *p, uint4v v)
{
    if (POLICY == 0) asm volatile("global_store_dwordx4 %0, %1, off" : : "v"(p), "v"(v) : "memory");
    if (POLICY == 1) asm volatile("global_store_dwordx4 %0, %1, off nt" : : "v"(p), "v"(v) : "memory");
    if (POLICY == 2) asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
    if (POLICY == 3) asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" : : "v"(p), "v"(v) : "memory");
    if (POLICY == 4) asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}

// Every outstanding vector-memory operation of the wave has completed; the eight values are
// operands so that nothing that uses them can be moved ahead of the wait.
__device__ __forceinline__ void wait_loads(uint4v (&x)[8])
{
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])
                 :
                 : "memory");
}

constexpr int kPassVecs = 512;      // 16-byte vectors a wave keeps in flight: 8 loads of 1 KB

// Wave w moves vectors [w * read_per_wave, (w + 1) * read_per_wave) in (cut at read_vecs) and the
// same share of the output out, in parts of read_per_pass / write_per_pass vectors: the loads of a
// part (8 at a time), then its stores, which depend on what was loaded, as a kernel's results do.
// (The shares are computed on the host: a 64-bit division costs a wave hundreds of instructions.)
struct ProbeSplit {
    int64_t read_vecs, write_vecs, waves, blocks;
    int32_t read_per_wave, write_per_wave, read_per_pass, write_per_pass, passes, xcd_contiguous;
    int32_t paired_loads, alu_ops_per_pass;
};

template <int LOADS, int STORES>
__global__ __launch_bounds__(1024) void stream_probe_kernel(const uint4v *__restrict__ src,
                                                            uint4v *__restrict__ dst, const ProbeSplit s)
{
    const int waves_per_block = int(blockDim.x) >> 6;
    const int lane = int(threadIdx.x) & 63;
    const int64_t per_die = (s.blocks + 7) >> 3;
    for (int64_t b = blockIdx.x; b < (s.xcd_contiguous ? per_die * 8 : s.blocks); b += gridDim.x) {
        const int64_t block = s.xcd_contiguous ? (b & 7) * per_die + (b >> 3) : b;
        const int64_t wave = block * waves_per_block + (int(threadIdx.x) >> 6);
        if (wave >= s.waves) continue;
        const int64_t r0 = wave * s.read_per_wave, w0 = wave * s.write_per_wave;
        const int64_t r1 = r0 + s.read_per_wave < s.read_vecs ? r0 + s.read_per_wave : s.read_vecs;
        const int64_t w1 = w0 + s.write_per_wave < s.write_vecs ? w0 + s.write_per_wave : s.write_vecs;
        uint4v acc = {0u, 0u, 0u, 0u};
        for (int p = 0; p < s.passes; p++) {
            const int64_t ra = r0 + int64_t(p) * s.read_per_pass, wa = w0 + int64_t(p) * s.write_per_pass;
            const int64_t rb = ra + s.read_per_pass < r1 ? ra + s.read_per_pass : r1;
            const int64_t wb = wa + s.write_per_pass < w1 ? wa + s.write_per_pass : w1;
            for (int64_t v = ra; v < rb; v += kPassVecs) {
                uint4v x[8];
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    // paired: a lane's two vectors of a pair of loads are neighbours (32 consecutive bytes per
                    // lane, so each instruction covers every other 16 bytes of 2 KB), as in the quantizer's
                    // lane mapping; else every instruction covers 1 KB of consecutive bytes
                    const int64_t i = s.paired_loads ? v + (u >> 1) * (2 * kWave) + 2 * lane + (u & 1) : v + u * kWave + lane;
                    probe_load<LOADS>(x[u], src + (i < rb ? i : rb - 1));       // clamped: the part's last vector again
                }
                wait_loads(x);
#pragma unroll
                for (int u = 0; u < 8; u++) acc += x[u];
            }
            // stand-in for a kernel's arithmetic: a chain of dependent integer multiply-adds
            for (int k = 0; k < s.alu_ops_per_pass; k += 8) {
                acc[0] = acc[0] * 0x9e3779b1u + acc[1];
                acc[1] = acc[1] * 0x85ebca6bu + acc[2];
                acc[2] = acc[2] * 0xc2b2ae35u + acc[3];
                acc[3] = acc[3] * 0x27d4eb2fu + acc[0];
            }
            for (int64_t v = wa + lane; v < wb; v += kWave) probe_store<STORES>(dst + v, acc + uint32_t(v));
        }
    }
}

}  // namespace

hipError_t launch_stream_probe(const void *src, size_t read_bytes, void *dst, size_t write_bytes,
                               const ProbeShape &shape, hipStream_t stream)
{
    ProbeSplit s{};
    s.read_vecs = int64_t(read_bytes / 16);
    s.write_vecs = int64_t(write_bytes / 16);
    const int64_t larger = s.read_vecs > s.write_vecs ? s.read_vecs : s.write_vecs;
    const int64_t slice_vecs = shape.slice_bytes / 16;
    s.waves = (larger + slice_vecs - 1) / slice_vecs;
    if (s.waves == 0) return hipSuccess;
    const int waves_per_block = shape.block_threads / 64;
    s.blocks = (s.waves + waves_per_block - 1) / waves_per_block;
    s.passes = shape.slice_bytes > 8192 ? shape.slice_bytes / 8192 : 1;
    s.read_per_wave = int32_t((s.read_vecs + s.waves - 1) / s.waves);
    s.write_per_wave = int32_t((s.write_vecs + s.waves - 1) / s.waves);
    s.read_per_pass = (s.read_per_wave + s.passes - 1) / s.passes;
    s.write_per_pass = (s.write_per_wave + s.passes - 1) / s.passes;
    s.xcd_contiguous = shape.xcd_contiguous;
    s.paired_loads = shape.paired_loads;
    s.alu_ops_per_pass = shape.alu_ops_per_pass;
    int64_t grid = shape.xcd_contiguous ? (s.blocks + 7) / 8 * 8 : s.blocks;
    if (shape.max_blocks > 0 && grid > shape.max_blocks) grid = shape.max_blocks;
    if (grid > 0x7fffffff) grid = 0x7fffffff;
    using Kernel = void (*)(const uint4v *, uint4v *, const ProbeSplit);
#define CGX_PROBE_STORES(L) \
    {stream_probe_kernel<L, 0>, stream_probe_kernel<L, 1>, stream_probe_kernel<L, 2>, stream_probe_kernel<L, 3>, \
     stream_probe_kernel<L, 4>}
    static const Kernel table[4][5] = {CGX_PROBE_STORES(0), CGX_PROBE_STORES(1), CGX_PROBE_STORES(2),
                                       CGX_PROBE_STORES(3)};
#undef CGX_PROBE_STORES
    hipLaunchKernelGGL(table[shape.load_policy][shape.store_policy], dim3(unsigned(grid)),
                       dim3(unsigned(shape.block_threads)), size_t(shape.lds_bytes_per_block), stream, static_cast<const uint4v *>(src),
                       static_cast<uint4v *>(dst), s);
    return hipGetLastError();
}

}  // namespace cgx
