// The streaming probe (include/cgx_diag.h): a kernel that only moves bytes, with the access
// style of the method's kernels (lane-contiguous 16-byte vectors, 1 KB per instruction and wave)
// and a launch shape and cache policies chosen by the caller.  A measurement aid: what it
// sustains at a given size and read:write mix is the ceiling the memory system sets for a
// streaming kernel of that shape.  Behind it, the issue-rate probe: what one vector instruction form
// costs a SIMD.
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

// ---------------------------------------------------------------- issue-rate probe
//
// One vector instruction form, repeated in 16 independent chains per lane with no memory access
// in the loop: the time of a launch divided by the instructions each SIMD executed is what that
// form costs a SIMD with eight resident waves.  The forms are the ones the kernels' inner loops
// are made of, plus the alternatives that were weighed against them.  %0 is a chain's register
// (read and written), %1 and %2 other vector registers, %3 a scalar register.
#define CGX_ISSUE_FORMS(X)                                                                                       \
    X(0, "v_add_f32 %0, %1, %0")                                                                                 \
    X(1, "v_sub_f32 %0, %1, %0")                                                                                 \
    X(2, "v_mul_f32 %0, %1, %0")                                                                                 \
    X(3, "v_fmac_f32 %0, %1, %2")                                                                                \
    X(4, "v_fma_f32 %0, %0, %1, %2")                                                                             \
    X(5, "v_fma_f32 %0, %1, %3, %0")                                                                             \
    X(6, "v_add_f32 %0, %3, %0")                                                                                 \
    X(7, "v_and_b32 %0, %1, %0")                                                                                 \
    X(8, "v_and_b32 %0, 60, %0")                                                                                 \
    X(9, "v_and_b32 %0, 0x0f0f0f0f, %0")                                                                         \
    X(10, "v_and_b32 %0, %3, %0")                                                                                \
    X(11, "v_xor_b32 %0, %1, %0")                                                                                \
    X(12, "v_or_b32 %0, %1, %0")                                                                                 \
    X(13, "v_lshrrev_b32 %0, 4, %0")                                                                             \
    X(14, "v_lshlrev_b32 %0, 3, %0")                                                                             \
    X(15, "v_add_u32 %0, %1, %0")                                                                                \
    X(16, "v_mov_b32 %0, %1")                                                                                    \
    X(17, "v_cvt_f32_ubyte0 %0, %0")                                                                             \
    X(18, "v_cvt_f32_ubyte2 %0, %0")                                                                             \
    X(19, "v_cvt_u32_f32 %0, %0")                                                                                \
    X(20, "v_cvt_f16_f32 %0, %0")                                                                                \
    X(21, "v_cvt_f32_f16 %0, %0")                                                                                \
    X(22, "v_cvt_f32_fp8_sdwa %0, %0 src0_sel:BYTE_2")                                                           \
    X(23, "v_mul_lo_u32 %0, %1, %0")                                                                             \
    X(24, "v_min_f32 %0, %1, %0")                                                                                \
    X(25, "v_max_f32 %0, %1, %0")                                                                                \
    X(26, "v_min_u32_sdwa %0, %1, %0 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1")        \
    X(27, "v_xor_b32_sdwa %0, %1, %0 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1")        \
    X(28, "v_lshl_or_b32 %0, %0, 4, %1")                                                                         \
    X(29, "v_or3_b32 %0, %0, %1, %2")                                                                            \
    X(30, "v_xad_u32 %0, %0, %1, %2")                                                                            \
    X(31, "v_bfe_u32 %0, %0, 4, 4")                                                                              \
    X(32, "v_perm_b32 %0, %0, %1, %2")                                                                           \
    X(33, "v_alignbit_b32 %0, %0, %1, 8")                                                                        \
    X(34, "v_bitop3_b32 %0, %0, %1, %2 bitop3:0x80")                                                             \
    X(35, "v_mov_b32_dpp %0, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")                                 \
    X(36, "v_min_f32_dpp %0, %1, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")                             \
    X(37, "v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,0,0] op_sel_hi:[1,0,0]")                                       \
    X(38, "v_rcp_f32 %0, %0")
// four more forms are written out below: one whose result is a register pair, and three short sequences
// that decode a code by lookup (a table in LDS; a table in the lanes of a register, twice)
#define CGX_ISSUE_FORM_PAIR "v_cvt_pk_f32_fp8 %0:[2], %0 ; v_xor_b32 %0, %0[0], %0[1] (two results, folded by a v_xor_b32)"
#define CGX_ISSUE_FORM_TABLE \
    "v_lshrrev_b32 t, 7, %0 ; v_and_b32 t, 60, t ; v_add_u32 t, %1, t ; ds_read_b32 t, t ; v_add_f32 %0, t, %0 (the decode of a code by lookup: 16 entries in LDS, %1 the wave's table)"
#define CGX_ISSUE_FORM_LANES \
    "v_lshrrev_b32 t, 8, %0 ; ds_bpermute_b32 t, t, %1 ; v_add_f32 %0, t, %0 (the decode of a code by lookup in another lane's register, any of 64 lanes)"
#define CGX_ISSUE_FORM_LANES16 \
    "v_lshrrev_b32 t, 8, %0 ; v_and_b32 t, 60, t ; ds_bpermute_b32 t, t, %1 ; v_add_f32 %0, t, %0 (the same, 16 lanes)"

constexpr int kIssueForms = 43;
constexpr int kIssueChains = 16;

template <int FORM>
struct IssueForm;
#define CGX_ISSUE_FORM(N, TEXT)                                                              \
    template <>                                                                              \
    struct IssueForm<N> {                                                                    \
        static __device__ __forceinline__ void step(uint32_t &a, uint32_t b, uint32_t c, uint32_t s, const uint32_t *) \
        {                                                                                    \
            asm volatile(TEXT : "+v"(a) : "v"(b), "v"(c), "s"(s));                           \
        }                                                                                    \
    };
CGX_ISSUE_FORMS(CGX_ISSUE_FORM)
#undef CGX_ISSUE_FORM
template <>
struct IssueForm<kIssueForms - 4> {
    static __device__ __forceinline__ void step(uint32_t &a, uint32_t, uint32_t, uint32_t, const uint32_t *)
    {
        uint64_t pair;
        asm volatile("v_cvt_pk_f32_fp8 %0, %1" : "=v"(pair) : "v"(a));
        asm volatile("v_xor_b32 %0, %1, %2" : "=v"(a) : "v"(uint32_t(pair)), "v"(uint32_t(pair >> 32)));
    }
};
// The lookup is left to the compiler (it places the waits on LDS); every wave has a table of its own, whose 16
// dwords lie in 16 banks, so lanes that read different entries do not collide.
template <>
struct IssueForm<kIssueForms - 3> {
    static __device__ __forceinline__ void step(uint32_t &a, uint32_t, uint32_t, uint32_t, const uint32_t *table)
    {
        const float entry = __uint_as_float(*reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(table) + ((a >> 7) & 60u)));
        a = __float_as_uint(__uint_as_float(a) + entry);
    }
};

// The table in the lanes of one register: the permute takes bits 7:2 of its address for the lane it reads and
// touches no memory.
template <>
struct IssueForm<kIssueForms - 2> {
    static __device__ __forceinline__ void step(uint32_t &a, uint32_t, uint32_t c, uint32_t, const uint32_t *)
    {
        const float entry = __int_as_float(__builtin_amdgcn_ds_bpermute(int(a >> 8), int(c)));
        a = __float_as_uint(__uint_as_float(a) + entry);
    }
};
template <>
struct IssueForm<kIssueForms - 1> {
    static __device__ __forceinline__ void step(uint32_t &a, uint32_t, uint32_t c, uint32_t, const uint32_t *)
    {
        const float entry = __int_as_float(__builtin_amdgcn_ds_bpermute(int((a >> 8) & 60u), int(c)));
        a = __float_as_uint(__uint_as_float(a) + entry);
    }
};

template <int FORM>
__global__ __launch_bounds__(256) void issue_probe_kernel(uint32_t *__restrict__ out, int iterations, uint32_t scalar)
{
    __shared__ uint32_t tables[4][16];
    const uint32_t b = 0x3f800000u + 0x01010101u * (threadIdx.x & 63u), c = (b * 7u) | 1u;
    uint32_t *table = tables[(threadIdx.x >> 6) & 3u];
    if constexpr (FORM == kIssueForms - 3) {
        // entries of about 2^-20 .. 2^-19: the chains keep moving and stay finite
        if ((threadIdx.x & 63u) < 16u) table[threadIdx.x & 63u] = 0x35800000u + 0x00011111u * (threadIdx.x & 63u);
        __syncthreads();
    }
    uint32_t a[kIssueChains];
#pragma unroll
    for (int j = 0; j < kIssueChains; j++) a[j] = b * uint32_t(j + 3);
    for (int i = 0; i < iterations; i++) {
#pragma unroll
        for (int j = 0; j < kIssueChains; j++) IssueForm<FORM>::step(a[j], b, c, scalar, table);
    }
    uint32_t x = 0;
#pragma unroll
    for (int j = 0; j < kIssueChains; j++) x ^= a[j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = x;
}

template <int FORM>
void launch_issue_form(int form, unsigned blocks, uint32_t *out, int iterations, hipStream_t stream)
{
    if constexpr (FORM < kIssueForms) {
        if (form == FORM)
            hipLaunchKernelGGL(issue_probe_kernel<FORM>, dim3(blocks), dim3(256), 0, stream, out, iterations, 0x3f800000u);
        else
            launch_issue_form<FORM + 1>(form, blocks, out, iterations, stream);
    }
}

}  // namespace

const char *issue_probe_form(int form)
{
    static const char *const names[kIssueForms] = {
#define CGX_ISSUE_NAME(N, TEXT) TEXT,
        CGX_ISSUE_FORMS(CGX_ISSUE_NAME)
#undef CGX_ISSUE_NAME
        CGX_ISSUE_FORM_PAIR, CGX_ISSUE_FORM_TABLE, CGX_ISSUE_FORM_LANES, CGX_ISSUE_FORM_LANES16};
    return form >= 0 && form < kIssueForms ? names[form] : nullptr;
}

hipError_t launch_issue_probe(int form, int blocks, int iterations, void *out, hipStream_t stream)
{
    launch_issue_form<0>(form, unsigned(blocks), static_cast<uint32_t *>(out), iterations, stream);
    return hipGetLastError();
}

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
