/*
 * cgx_diag.h -- diagnostics and measurement aids of libcgx.so.  Nothing here is part of the
 * method of cgx.h: cgx_plan_tiles shows how the kernels split a plan into wavefront work
 * items, the cgx_stream_probe calls measure what the memory system gives a kernel that only
 * moves bytes.
 */
#ifndef CGX_DIAG_H
#define CGX_DIAG_H

#include "cgx.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Diagnostic: the table of wavefront work items ("tiles") the kernels walk for
 * a plan, written to host memory as 32-byte records
 *   { int64 first_element; int64 packed_byte_offset; uint32 first_bucket;
 *     uint32 elements; uint32 info; uint32 pad_bytes }
 * with info = bits | kind << 4 | log2(lanes per bucket) << 8 | (bucket / 32) << 12 (the last
 * two fields are 0 where they do not apply) and kind 0 = generic
 * quantize, 1 = vectorised quantize, 2 = element-wise copy, 3 = vectorised copy,
 * 4 = vectorised quantize of one whole bucket of 4096 or 8192 elements, 5 = the short end
 * of a layer (less than a chunk of 2048 elements) with power-of-two buckets, 6 = whole buckets
 * of a size that is no power of two, at most a chunk in all (streamed row by row; only the ragged
 * end of such a layer and sizes above the chunk take the generic kind 0).
 * Every element of every non-empty layer lies in exactly one tile and tiles never
 * cross layers (paper Sec. 4.1).  This is the table of one chunk per vectorised
 * tile that most calls walk: cgx_quantize on a binary16 gradient of 2^24 elements
 * or more, and the fused reduce + requantize on 2^27 elements or more, join 2
 * consecutive chunks of a layer into one tile (same bytes out; a wave's set-up is
 * spread over more input).  At most `capacity` records
 * are written; *n_tiles receives the full count.  Pure host computation.
 */
int cgx_plan_tiles(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                   int32_t bucket, cgx_dtype dt, void *tiles_out /* host */, int64_t capacity,
                   int64_t *n_tiles);
/*
 * The same table for kernels whose chunk is chunk_elements (1024 or 2048; CGX_ERR_SIZE otherwise).
 * cgx_plan_tiles gives the table of 2048-element chunks, which the reduce, fused and statistics
 * kernels and the binary16 quantizer walk; cgx_quantize on binary32 input, cgx_requantize and
 * cgx_dequantize to binary32 walk the table of 1024-element chunks (buckets of 2048 elements are then one-bucket tiles of
 * kind 4, like those of 4096 and 8192).
 */
int cgx_plan_tiles_chunk(int64_t n, int32_t L, const int64_t *layer_offsets, const uint8_t *bits_per_layer,
                         int32_t bucket, cgx_dtype dt, int32_t chunk_elements, void *tiles_out /* host */,
                         int64_t capacity, int64_t *n_tiles);

/*
 * One launch that reads read_bytes from src and writes write_bytes to dst (both device, 16-byte
 * aligned, sizes multiples of 16) with the kernels' access style (one wavefront per 8 KB slice
 * of the larger side, non-temporal 16-byte vectors, lane-contiguous) and no arithmetic.  Its
 * rate is what the memory system gives a kernel with that read:write mix at that size; the
 * benchmark reports it next to each kernel.  What is written to dst is unspecified.
 */
int cgx_stream_probe(const void *src, size_t read_bytes, void *dst, size_t write_bytes, void *stream);

/*
 * The same probe with its launch shape and cache policies chosen by the caller, for sweeps
 * that look for the best a streaming kernel can get at a given size and read:write mix.
 *   slice_bytes     bytes of the larger side one wavefront moves: a power of two in
 *                   [1024, 1048576]; the smaller side is split into as many slices.  A wave
 *                   works in passes of 8 KB (8 loads of 1 KB in flight), writing its share of
 *                   the output after each pass
 *   block_threads   64, 128, 256, 512 or 1024
 *   load_policy     0 plain, 1 nt, 2 sc1, 3 sc0 sc1   (cache-policy bits of the load instruction)
 *   store_policy    0 plain, 1 nt, 2 sc0 sc1, 3 sc0 sc1 nt, 4 sc1
 *   xcd_contiguous  0: block b takes slice group b; 1: blocks are renumbered so that the blocks
 *                   with equal b mod 8 (one accelerator die, if blocks go round the dies in turn)
 *                   walk one contiguous eighth of the buffers
 *   max_blocks      0: one block per slice group; > 0: at most this many blocks, each looping
 * Three more knobs make the probe resemble a kernel that also computes:
 *   paired_loads         1: a lane's two vectors of a pair of loads are neighbours in memory (32
 *                        consecutive bytes per lane; each load instruction covers every other 16 bytes
 *                        of 2 KB), the quantizer's lane mapping; 0: every instruction covers 1 KB
 *   alu_ops_per_pass     dependent vector instructions per lane executed between the loads of a pass and
 *                        its stores (0 to 65536; a multiply-add chain, rounded up to a multiple of 8)
 *   lds_bytes_per_block  dynamic LDS the launch asks for (0 to 65536): bounds the waves a compute unit
 *                        holds at once, as a kernel's registers or staging area would
 * CGX_ERR_SIZE for a value outside these sets.
 */
typedef struct {
    int32_t slice_bytes;
    int32_t block_threads;
    int32_t load_policy;
    int32_t store_policy;
    int32_t xcd_contiguous;
    int32_t max_blocks;
    int32_t paired_loads;
    int32_t alu_ops_per_pass;
    int32_t lds_bytes_per_block;
} cgx_probe_shape;
int cgx_stream_probe_shaped(const void *src, size_t read_bytes, void *dst, size_t write_bytes,
                            const cgx_probe_shape *shape /* host */, void *stream);

/*
 * What one vector instruction form costs: a launch of `blocks` blocks of 256 threads (1 to 65536) in
 * which every wavefront executes 16 * iterations instructions of form number `form` (1 to 2^20
 * iterations, 16 independent dependency chains per lane, nothing else in the loop).  With 8 resident
 * waves per SIMD (blocks = 8 * compute units), launch time * clock / (blocks * 4 * 16 * iterations /
 * (compute units * 4)) is the form's cost in cycles of a SIMD.  The forms are those of the kernels'
 * inner loops and the alternatives weighed against them (the last few are short sequences, a lookup in
 * LDS or in another lane's register followed by an addition, counted as one); cgx_issue_probe_form
 * returns the text of a form, NULL past the last one.  out (device, 16-byte aligned, out_bytes >= blocks * 1024) receives
 * one word per thread; its content is unspecified.  CGX_ERR_SIZE for a value outside these ranges.
 * The benchmark's --issue-rates mode prints the table; it is the evidence for pricing the fused
 * kernel, which is bound by the vector ALUs, and for the choice of its decoding instructions.
 */
const char *cgx_issue_probe_form(int32_t form);
int cgx_issue_probe(int32_t form, int32_t blocks, int32_t iterations, void *out, size_t out_bytes, void *stream);

/*
 * Launch-shape overrides, for the tests and for measurements.  The library reads these
 * environment variables once, at its first call; none of them changes a byte of any result (the
 * parity tests run the same inputs under several settings and compare digests):
 *   CGX_CHUNKS_PER_TILE=k   every vectorised tile holds up to k chunks (default: chosen per call)
 *   CGX_MAX_BLOCKS=k        persistent grids of at most k blocks (default: one wave per tile)
 *   CGX_QUANTIZE_GROUPS=2|4 chunk size of every quantize call: 1024 or 2048 elements (default:
 *                           1024 for binary32 input, 2048 for binary16)
 *   CGX_VIA_LDS=0           the quantizer reads its chunks straight into registers instead of
 *                           through LDS
 *   CGX_KEEP_SUMS_MB=k      the reduce writes results of up to k MB through at device scope so that
 *                           they stay in the memory-side cache (default 128; 0: always streamed)
 *   CGX_QUANTIZE_TILES_PER_WAVE_X4=k  grid of the binary32 quantizer on plans of up to 2^19 tiles: k/4 tiles per
 *                           wave (default 5: four fifths of the waves that one tile each would take; 4: one
 *                           wave per tile)
 *   CGX_REDUCE_GROUPS=2|4   chunk size of every reduce call with buckets of up to 1024 elements: 1024 or 2048
 *                           elements (default: 2048, and 1024 for cgx_dequantize to binary32)
 *   CGX_DEQUANTIZE_THROUGH=0  cgx_dequantize runs like a reduce of one chunk (2048-element chunks, the
 *                           reduce's store policy) instead of with 1024-element chunks and stores written
 *                           through at system scope
 */

#ifdef __cplusplus
}
#endif
#endif /* CGX_DIAG_H */
