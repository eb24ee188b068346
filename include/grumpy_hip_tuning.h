/*
 * grumpy_hip_tuning.h -- scheduling knobs and bandwidth-ceiling kernels of the fused lazy-array
 * evaluator.  Nothing here changes a result: the option keys below go through
 * gr_ctx_set_option (grumpy_hip.h) and choose how the kernels of a sub-graph (Section 3 of the
 * paper: one kernel per sub-graph, a point function evaluated per output index) are laid out
 * on the GPU; they exist for sweeps and for the benchmark, and their defaults are the measured
 * optima on MI355X.  The two streaming kernels give the practical HBM ceiling of the box, the
 * context for every "fraction of peak" figure.
 */
#ifndef GRUMPY_HIP_TUNING_H
#define GRUMPY_HIP_TUNING_H

#include "grumpy_hip.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Tuning keys of gr_ctx_set_option (0 = the library's own choice unless stated otherwise):
 *   "map_rows", "map_chunks"   per-lane patch of the map skeleton: rows, and chunks of four columns
 *   "map_bx"          lanes of a workgroup along the columns (power of two <= 256)
 *   "rowred_threads"  lanes that hold one row of a row-resident reduction: 16, 64, 128 or 256
 *   "rowred_rows"     rows a lane group of a row-resident reduction takes per launch when rows are
 *                     short (at most 64 elements) and reduce to one value each: 0 = 4 for 2^18 rows
 *                     or more, 1 = always one, 2..8 = that many
 *   "gemv_slabs", "gemv_unroll"  column-accumulate contraction: number of row slabs (first-stage
 *                     partial vectors) and rows in flight per lane, 8 or 16
 *   "gemm_bn"         width of the output tile of the matrix-product kernel: 32 or 128; 0 = 32 for
 *                     results of at most 96 columns and where the last 128-wide tile would be more
 *                     than half empty
 *   "gemm_kstep"      values of k per step of the matrix-product kernel's main loop (one barrier per
 *                     step): 16 (default), 32
 *   "gemm_split"      workgroups per output tile of a matrix product, each accumulating a part of K into
 *                     a partial tile that a second kernel combines in a fixed order: 1 .. 256; 0 (default) =
 *                     chosen by the planner (more than one only for fewer than 192 output tiles and K >= 256)
 *   "gemm_big"        1 (default) = matrix products whose operands are each contiguous along one of their
 *                     dimensions, with K a multiple of 16 (and of every split of K at least 32), use the kernels whose operand
 *                     tiles go from global memory straight into LDS: 256 x 256 tiles, one workgroup per
 *                     compute unit, where the result fills at least 85 % (65 % if M or N is not a multiple
 *                     of 128) of its rounds over the 256 compute units, else 128 x 128 tiles; 0 = the kernel
 *                     that stages tiles through registers for every product
 *   "nontemporal"     1 (default) = loads of arrays that are read once carry the non-temporal hint,
 *                     and so do the vector stores of a requested value of 192 MiB or more (not of
 *                     intermediate results of the request; except in kernels that read a transposed
 *                     operand through LDS tiles when output rows are not 64-byte aligned); 0 = none;
 *                     2 = every vector load; 8 = vector stores only; 9 = the loads of 1 and every
 *                     vector store
 *   "stage_transposed" 1 (default) = a map sub-graph reads operands whose contiguous dimension is the
 *                     row dimension of the iteration space (transposed views) through tiles
 *                     transposed in LDS; 0 = strided loads
 *   "stage_rows"      rows of such a tile (it has 64 columns): 0 = 128 where the iteration space has
 *                     128 rows or more, else 64; 64 = always 64
 *   "stage_diag"      1 (default) = kernels with such tiles take row blocks diagonally and give each
 *                     XCD a contiguous range of column blocks; 0 = row-major tile order
 *   "scan_min_threads", "scan_threads"
 *                     a scan along a non-contiguous axis that does not qualify for one pass over tiles
 *                     (see "scan_one_pass") gives each thread one line (four neighbouring lines with
 *                     dwordx4 loads); with fewer threads than scan_min_threads the lines are cut into
 *                     chunks so that about scan_threads threads run, at the price of a second read of
 *                     the input; 0 = 16384 / 65536 with dwordx4 loads, 32768 / 131072 with scalar loads
 *   "scan_polls"      polls a tile of a one-pass scan spends on each wait for a published total before
 *                     it recomputes its offset from the input (default 2^20; 0 = never wait: every
 *                     total that is not there yet is recomputed, which is how a test reaches that path)
 *   "scan_one_pass"   1 (default) = a scan of 4-byte values along a contiguous axis with few, long
 *                     lines (fewer than 512 lines of more than 32768 elements) reads its input once:
 *                     chained tiles that publish their totals (the map-scan primitive of Section 3.2
 *                     as a single kernel); 0 = chunk totals, a scan of the totals, then the chunks
 *                     with their offsets (three kernels, the input read twice); 2..24 = one pass
 *                     with tiles of that many 1024-element blocks.  Any value but 0 also lets a scan
 *                     of 4-byte values along a NON-contiguous axis (lines of 128 positions or more, the
 *                     innermost line dimension contiguous and a multiple of four) read its input once:
 *                     tiles of up to 256 neighbouring lines by up to 128 positions stay in registers,
 *                     publish their totals per line and collect their offsets from the tiles before
 *                     them; 0 = a thread per four lines, chunked as described above
 */

/* dst[i] = src[i] for `bytes` bytes (multiple of 16; both device pointers,
 * 16-byte aligned, not overlapping), launched on the context's stream. */
gr_status gr_stream_copy(gr_ctx* ctx, void* dst, const void* src, size_t bytes);
/* Reads `bytes` bytes (multiple of 16) and writes one 4-byte word per
 * workgroup to `sink` (device pointer, at least 16 KiB). */
gr_status gr_stream_read(gr_ctx* ctx, const void* src, size_t bytes, void* sink);

#ifdef __cplusplus
}
#endif
#endif /* GRUMPY_HIP_TUNING_H */
