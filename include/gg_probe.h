/* libgg_probe: measurement probes for gfx950 (MI355X).  NOT part of the hot path and never called by it.
 *
 * The grouped GEMM of libgg_fp8 (paper Sec. 2.1, Table 1) is judged against what this chip sustains, and the
 * datasheet gives only the matrix pipe's and HBM's peaks.  These calls measure the other ceilings the kernels
 * run into, with the same instructions and access shapes the kernels use and nothing else around them:
 *   - the matrix instruction in a register-only loop, alone and with the scale fusion of Sec. 2.1 behind it
 *     (one product per 128-wide scale block, started from zero, then 4 fp32 FMAs per 16x16 block);
 *   - the same loop with further scalar, vector and LDS instructions per matrix instruction;
 *   - a plain HBM read and a plain HBM copy;
 *   - the L2 -> LDS fetch stream (16 bytes per lane, straight into LDS) with no compute behind it;
 *   - the second GEMM kernel itself with parts of its K step left out (fetches, barrier, LDS reads).
 *
 * Every call is synchronous: it allocates its own device buffers, launches on the null stream, waits, frees, and
 * returns 0 or the hipError_t that stopped it (nothing is left allocated).  Results are written through host
 * pointers.  One GPU (the current device); not re-entrant.  `python bench.py --op ceilings` prints all of them.
 */
#ifndef GG_PROBE_H_
#define GG_PROBE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Register-only loop of FP8 (e4m3) matrix instructions on every SIMD of the chip: 8 waves per compute unit, no
 * memory access inside the loop.
 *   mode 0: v_mfma_f32_16x16x128_f8f6f4, each product added to its accumulator by the instruction itself
 *   mode 1: the same instruction started from zero, then acc += product * scale (4 fp32 FMAs): the inner loop of
 *           the block-scaled GEMM
 *   mode 2: v_mfma_f32_32x32x64_f8f6f4 accumulating
 *   mode 3: two v_mfma_f32_32x32x64_f8f6f4 per 128-wide scale block (the first from zero, the second on top of
 *           it), then 16 fp32 FMAs
 *   data_kind 0: every operand byte 0x38 (1.0); 1: bytes like e4m3-quantised normal samples scaled to the
 *           format's range; 2: uniformly random bytes (NaN codes replaced).  The chip's clock depends on how
 *           many operand bits toggle, so the three differ.
 * iters: loop trips per wave (each trip: 16 instructions of the 16x16x128 shape, or 8 of the 32x32x64 shape:
 *        the same 2 * 64 * 64 * 128 flop per trip per wave); > 0.
 * tflops_out (host): 1e-12 * flop / seconds of the timed launch (a warm-up launch precedes it). */
int gg_probe_mfma(int mode, int data_kind, int iters, double* tflops_out);

/* The loop of gg_probe_mfma mode 1 (16x16x128 from zero + 4 FMAs) on constant operands with further instructions
 * per matrix instruction that do no useful work: `extra_salu` scalar additions, `extra_valu` vector additions,
 * `extra_lds_reads` 16-byte LDS reads (conflict-free).  What each instruction a kernel puts beside the matrix
 * instruction costs in matrix-pipe time; with 8 waves per compute unit, as in the GEMM kernels.  Built combinations
 * (salu, valu, lds): (0,0,0) (2,0,0) (4,0,0) (8,0,0) (0,1,0) (0,2,0) (0,0,1) (0,0,2) (2,1,1) (2,1,2); anything else:
 * hipErrorInvalidValue. */
int gg_probe_issue_mix(int extra_salu, int extra_valu, int extra_lds_reads, int iters, double* tflops_out);

/* HBM streams over `bytes` (a multiple of 4096, larger than the caches for a meaningful figure).
 *   kind 0: read (16 bytes per lane, summed so the loads cannot be dropped)
 *   kind 1: copy (read `bytes`, write `bytes`)
 * gbytes_per_s_out (host): 1e-9 * bytes moved (kind 1: 2 * bytes) / seconds, best of `reps` >= 1 launches. */
int gg_probe_hbm(int kind, size_t bytes, int reps, double* gbytes_per_s_out);

/* The fetch stream of the GEMM kernels without their compute: 512-thread workgroups, one per compute unit, each
 * moving 64 KB per step (a K block of a 256 x 256 tile: 256 rows x 128 B of A and as much of B) into LDS with
 * 16-byte-per-lane buffer loads, `depth` steps in flight (1..7).
 *   pattern 0: every workgroup re-reads one contiguous 64 KB chunk (L2 hits, full cache lines in address order)
 *   pattern 1: every workgroup re-reads the same two column blocks [256 rows x 128 B, row pitch K] (L2 hits)
 *   pattern 2: the kernels' stream: per accelerator die 32 workgroups take a 4 x 8 block of tiles of a problem
 *              with K = 7168 and walk its 56 K blocks, so an A tile is fetched by 8 workgroups and a B tile by 4
 *              at about the same time: 12 of 64 fetches miss L2
 * gbytes_per_s_out: 1e-9 * bytes landed in LDS / seconds over the chip; bytes_per_clk_cu_out: the same per
 * compute unit and cycle of the nominal shader clock (hipDeviceAttributeClockRate). */
int gg_probe_lds_fetch(int pattern, int depth, int reps, double* gbytes_per_s_out, double* bytes_per_clk_cu_out);

/* The second GEMM kernel of libgg_fp8 (weights through registers; paper Sec. 2.1 arithmetic) in measurement builds
 * that LEAVE OUT parts of its K step, on a problem this call makes itself: `groups` equal groups of `rows_per_group`
 * rows, N = n, K = k (n % 256 == 0, k % 256 == 0, k >= 512; every tensor under 2 GiB), operand bytes like
 * e4m3-quantised normal samples, row-major activation scales.  What the step costs with and without each part says
 * where the time between the matrix pipe's minimum and the kernel's duration goes.
 *   tile_rows: 192 or 256 (the tiles 192x256 and 256x256 of the second kernel)
 *   left_out:  0 nothing (the kernel as the library launches it); 1 the fetches of the K steps; 2 every fetch goes
 *              to an out-of-range offset (issued, no traffic, the operands become zeros: compare cycles, not time);
 *              4 the barrier of the K step; 8 the LDS reads of activation fragments and scales; 16 the waits for the
 *              fetches (the data moves, nobody waits for it); 64 every fetch is an ordinary load into registers nobody
 *              reads (the same requests to memory, no LDS write).  Built sums: 5 = 1 + 4; 20 = 16 + 4;
 *              28 = 16 + 4 + 8; 92 = 28 + 64; 13 = 1 + 4 + 8 (matrix instructions, FMAs and bookkeeping only).
 *              32: nothing left out, but A and B are all zero bytes (the traffic of 0 at the power of 2).
 *              Anything else: hipErrorInvalidValue.  Only accesses and waits are removed, so every remaining access
 *              stays in bounds; the OUTPUT IS MEANINGLESS for every value but 0 and 32.
 *   reps:      timed launches (launches of the same build for about 150 ms precede them: the sustained clock)
 * us_out (host): microseconds per launch.  The shader clock differs between the builds (fewer operand bits moving,
 * higher clock): for cycles run the same call under `rocprofv3 --pmc GRBM_GUI_ACTIVE`. */
int gg_probe_gemm_kstep(int tile_rows, int left_out, int groups, int rows_per_group, int n, int k, int reps, double* us_out);

/* The weight-gradient kernel of libgg_fp8 (gg_fp8_grouped_gemm_wgrad: the variable-K grouped GEMM of training, which
 * the paper's title names and its text does not define) in measurement builds that LEAVE OUT parts of a token block's
 * work, on a problem this call makes itself: `groups` equal groups of `tokens_per_group` tokens (any count: a group
 * whose ends fall inside a 128-token block has masked first and last blocks), dW [groups, n, k] fp32 (n % 128 == 0,
 * k % 256 == 0; operands under 2 GiB, dW under 4 GiB), operand bytes like e4m3-quantised normal samples, block-major
 * scales.
 *   left_out:  sum of 1 the fetches of the token blocks, 2 the stores of dW, 4 the barrier of a block, 8 the byte
 *              masks of a group's first and last block, 16 the LDS reads that refill the operand registers.
 *              Built: 0 (the kernel as the library launches it), 1, 2, 3, 7, 11, 19, 31 (matrix instructions and
 *              FMAs only).  Anything else: hipErrorInvalidValue.  Only accesses, waits and masks are removed, so every
 *              remaining access stays in bounds; the OUTPUT IS MEANINGLESS for every value but 0.
 *   reps:      timed launches (launches of the same build for about 150 ms precede them: the sustained clock)
 * us_out (host): microseconds per launch. */
int gg_probe_wgrad_parts(int left_out, int groups, int tokens_per_group, int n, int k, int reps, double* us_out);

#ifdef __cplusplus
}
#endif
#endif
