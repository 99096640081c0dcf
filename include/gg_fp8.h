/* libgg_fp8 -- padding-free FP8 (e4m3) grouped GEMM with fine-grained block
 * scaling for AMD MI355X (gfx950).  C ABI; no C++ or framework types cross it.
 *
 * The operation (paper Sec. 2.1, Table 1; scaling granularity stated below the
 * table): G groups share N and K, group g owns M^g rows.  With
 *   A   [M_total, K]  e4m3 bytes, the groups' rows concatenated,
 *   SA  [M_total, ceil(K/128)]      one fp32 scale per (row, 128-wide K block),
 *   B   [G, N, K]     e4m3 bytes, B[g][n][k] = element (k, n) of the paper's B^g,
 *   SB  [G, ceil(N/128), ceil(K/128)]   one fp32 scale per 128x128 block of B^g (the last block along K and
 *                                   along N may be short: the ceilings of Table 1),
 *   group_offsets [G+1] int32       rows of group g are [off[g], off[g+1]),
 * the library writes, for every row r of group g and every n,
 *   C[r][n] = bf16( sum_kb  SA[r][kb] * SB[g][n/128][kb]
 *                           * sum_{k in block kb} dec(A[r][k]) * dec(B[g][n][k]) ).
 * Scales are dequantisation multipliers.  M^g is arbitrary (0, 1, not a
 * multiple of anything): only valid rows are read, computed and written; there
 * is no padded copy (the capability of Sec. 2.2, obtained here with bounded
 * buffer descriptors instead of a descriptor pool and two-phase stores).
 *
 * Conventions common to all entry points
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *    never allocates, frees or synchronises (except gg_fp8_check_offsets) and
 *    keeps no state between calls (beyond a per-device flag that a kernel's shared-memory limit has been
 *    raised); calls are asynchronous on `stream`
 *    (a hipStream_t passed as void*, NULL = the default stream).  Nothing but kernel launches is enqueued: the
 *    calls may be recorded into a HIP graph by stream capture (after one ordinary call per kernel on the device,
 *    which sets the kernel's shared-memory limit).
 *  - All matrices are row-major and dense (leading dimension = row length).
 *    A, B, C, A_pad, C_pad must be 16-byte aligned; SA, SB, offsets 4-byte.
 *  - N must be a positive multiple of 8 and K of 16 (16-byte stores and fetches; GG_ERR_UNSUPPORTED otherwise).
 *    Shapes with N % 128 != 0 or K % 128 != 0 run on a subset of the tile variants (the automatic choice knows
 *    them; asking explicitly for another variant returns GG_ERR_UNSUPPORTED).  The row kernels
 *    (gg_fp8_quantize_rows, gg_fp8_swiglu_quantize_rows) need whole 128-wide blocks.
 *  - group_offsets lives on the device and is trusted to be non-decreasing with
 *    0 <= off[0] and off[G] <= M_total.  If it is not, rows may be skipped or
 *    computed with the wrong group, but nothing outside C[0:M_total] is written.
 *    Rows of C outside [off[0], off[G]) are never written.
 *  - Return value: a gg_status.  On any error nothing has been enqueued.
 *    G == 0 or M_total == 0 returns GG_OK without a launch.
 */
#ifndef GG_FP8_H
#define GG_FP8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GG_OK = 0,
  GG_ERR_NULL = 1,        /* a required pointer is NULL                              */
  GG_ERR_SHAPE = 2,       /* G < 0, M_total < 0, N <= 0, K <= 0, or a size overflows */
  GG_ERR_UNSUPPORTED = 3, /* N % 8 or K % 16 nonzero, unknown variant, or a variant / row kernel that needs multiples of 128 */
  GG_ERR_WORKSPACE = 4,   /* workspace smaller than gg_fp8_workspace_bytes()         */
  GG_ERR_HIP = 5,         /* the HIP runtime refused a launch or a query             */
  GG_ERR_OFFSETS = 6      /* gg_fp8_check_offsets found invalid offsets              */
} gg_status;

/* Library version: major*10000 + minor*100 + patch. */
int gg_fp8_version(void);

/* Static, never-NULL description of a gg_status value. */
const char* gg_fp8_status_str(int status);

/* Bytes of device scratch a GEMM entry point needs for this problem size with the automatic variant choice
 * (gg_fp8_workspace_bytes; the same value serves the padded GEMM with M_total = M_pad_cap) or with an explicit
 * variant (gg_fp8_workspace_bytes_variant).  0 for all but the split-K variants ("-k2": the two halves of the K loop
 * of every tile are separate work units whose fp32 partial sums, 2 * M_total * N * 4 bytes, a second kernel adds and
 * rounds; paper Sec. 3.2, shapes with few rows per group).  `workspace` is a device buffer of at least that size,
 * 16-byte aligned, with any contents; it may be NULL when 0 bytes are needed.  Calls that may run at the same time
 * (different streams) need different workspaces.  A missing, short or misaligned workspace: GG_ERR_WORKSPACE. */
size_t gg_fp8_workspace_bytes(int G, int64_t M_total, int N, int K);
size_t gg_fp8_workspace_bytes_variant(int G, int64_t M_total, int N, int K, int variant);

/* The padding-free grouped GEMM defined at the top of this file (Sec. 2.1 and
 * 2.2).  One persistent kernel walks the (group, m-tile, n-tile) list derived
 * from group_offsets on the device; rows past the end of a group are neither
 * loaded (they read as zero) nor stored; the 16-row activation blocks of a tile that
 * lie past a group's end are not computed either (taller tile variants). */
int gg_fp8_grouped_gemm(const void* A, const float* SA, const void* B, const float* SB,
                        const int32_t* group_offsets, void* C,
                        int G, int64_t M_total, int N, int K,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Same operation with an explicit tile variant (for benchmarking and tests).
 * variant < 0 selects automatically, exactly like gg_fp8_grouped_gemm.
 * gg_fp8_num_variants() variants exist; gg_fp8_variant_name(v) describes one
 * ("BMxBN/waves/stages"), NULL if v is out of range. */
int gg_fp8_grouped_gemm_variant(const void* A, const float* SA, const void* B, const float* SB,
                                const int32_t* group_offsets, void* C,
                                int G, int64_t M_total, int N, int K,
                                void* workspace, size_t workspace_bytes, void* stream, int variant);
int gg_fp8_num_variants(void);
const char* gg_fp8_variant_name(int variant);
/* The variant gg_fp8_grouped_gemm would use for these sizes (the choice looks at
 * sizes only, never at device memory); a negative gg_status value if the sizes
 * are not supported. */
int gg_fp8_auto_variant(int G, int64_t M_total, int N, int K);
/* The same for gg_fp8_grouped_gemm_padded (and for the _ex call with GG_PADDED_GROUPS): the choice among the tile
 * heights that divide groups of 128-row blocks (the padded problem of Sec. 3). */
int gg_fp8_auto_variant_padded(int G, int64_t M_pad_cap, int N, int K);

/* gg_fp8_grouped_gemm_variant with C [M_total, N] written as IEEE binary16 instead of bfloat16: the paper says
 * "half-precision" and App. A only fixes 2 bytes per element, so both 2-byte formats are offered.  Same sum, same
 * order, one round-to-nearest-even step from the fp32 accumulator; magnitudes that round to 2^16 or more become
 * +-inf.  variant = -1 chooses automatically.  Everything else as for gg_fp8_grouped_gemm. */
int gg_fp8_grouped_gemm_f16(const void* A, const float* SA, const void* B, const float* SB,
                            const int32_t* group_offsets, void* C, int G, int64_t M_total, int N, int K,
                            void* workspace, size_t workspace_bytes, void* stream, int variant);

/* Options of the _ex entry points (bits of `flags`; any other bit: GG_ERR_UNSUPPORTED).
 *  GG_OUT_F16    C is IEEE binary16 instead of bfloat16 (as gg_fp8_grouped_gemm_f16).
 *  GG_SA_KMAJOR  the activation scales are stored K-block-major: SA [ceil(K/128), M_total], the scale of
 *                (row r, K block kb) at SA[kb * M_total + r].  Table 1 of the paper fixes the shape of the scale
 *                tensor, not its storage order; in this order the scales that one K block of a tile needs are
 *                contiguous, a few cache lines instead of one per row.  M_total * ceil(K/128) must stay below 2^29
 *                (GG_ERR_SHAPE otherwise).  Same arithmetic, bit-identical results.
 *  GG_PADDED_GROUPS  a promise that every group holds a multiple of 128 rows (the pad path of Sec. 3, what
 *                gg_fp8_grouped_gemm_padded passes): the automatic choice (variant = -1) then only considers tile
 *                heights that divide such groups, and reads M_total as a capacity (M_pad_cap).  Results do not
 *                depend on it.
 *  GG_OUT_BF16   gg_fp8_grouped_gemm_wgrad_ex only: its output is bfloat16 instead of fp32. */
enum { GG_OUT_F16 = 1, GG_SA_KMAJOR = 2, GG_PADDED_GROUPS = 4, GG_OUT_BF16 = 8 };

/* gg_fp8_grouped_gemm_variant with options (Sec. 2.1, 2.2 as above).  variant = -1 chooses automatically. */
int gg_fp8_grouped_gemm_ex(const void* A, const float* SA, const void* B, const float* SB,
                           const int32_t* group_offsets, void* C, int G, int64_t M_total, int N, int K,
                           void* workspace, size_t workspace_bytes, void* stream, int variant, unsigned flags);

/* gg_fp8_grouped_gemm_ex with a split-K variant, for callers that cannot allocate (code under HIP graph capture,
 * serving loops, harnesses that forbid hipMalloc): the partial sums live in a buffer built into the library, one
 * copy per GPU, instead of a caller's workspace, and the call allocates nothing.  variant: one of the "-k2" variants,
 * or -1 for the 128 x 256 one; flags: GG_OUT_F16 and GG_SA_KMAJOR.  M_total * N may be at most
 * gg_fp8_noalloc_max_elements() (4 Mi elements: 32 MiB of partial sums): GG_ERR_WORKSPACE beyond that, before
 * anything is enqueued.  Same results, bit for bit, as the _ex call with the same variant.  Every call on a GPU
 * uses that GPU's one buffer: calls that may overlap on one GPU (different streams) race; calls on one stream
 * are ordered and safe.  Other errors as for gg_fp8_grouped_gemm_ex (a variant that is not split-K:
 * GG_ERR_UNSUPPORTED). */
int gg_fp8_grouped_gemm_splitk_noalloc(const void* A, const float* SA, const void* B, const float* SB,
                                       const int32_t* group_offsets, void* C, int G, int64_t M_total, int N, int K,
                                       void* stream, int variant, unsigned flags);
size_t gg_fp8_noalloc_max_elements(void);

/* The first grouped GEMM of an expert MLP with the activation and the quantiser of the second GEMM's operand in
 * its epilogue (what gg_fp8_grouped_gemm followed by gg_fp8_swiglu_quantize_rows computes, without the bf16
 * intermediate [M_total, 2*I] ever reaching memory): B [G, 2*I, K] holds the gate projection in rows [0, I) and the
 * up projection in rows [I, 2*I) of every group, SB [G, 2*I/128, K/128] their scales;
 *   h = bf16(the block-scaled sums of Sec. 2.1),  act = bf16( silu(h_gate) * h_up ),
 * A2 [M_total, I] e4m3 and SA2 [M_total, I/128] from act by the recipe of gg_fp8_quantize_rows; act_out (bf16
 * [M_total, I]) receives act when it is not NULL.  Only valid rows are read, computed and written (Sec. 2.2), like
 * every kernel here; this is the "neighbouring kernel" of Sec. 4 moved into the GEMM.  Bit-identical to the
 * two-call sequence unless K % 8192 == 4096 (there the plain GEMM adds the K blocks in a rotated order).
 * flags: GG_SA_KMAJOR (applies to SA and to SA2) or 0.  variant: -1, or one of the second kernel's "-rb" variants
 * with 192, 224 or 256 rows.  I a multiple of 128, K a multiple of 256 and >= 512 (GG_ERR_UNSUPPORTED otherwise:
 * use the two calls); 2*I*K below 2^31.  A2, act_out 16-byte aligned.  Asynchronous on `stream`. */
int gg_fp8_grouped_gemm_swiglu(const void* A, const float* SA, const void* B, const float* SB,
                               const int32_t* group_offsets, void* A2, float* SA2, void* act_out,
                               int G, int64_t M_total, int I, int K, void* stream, int variant, unsigned flags);

/* The variable-K grouped GEMM of training: the weight gradient dW^g = dY^g^T X^g of the expert layer whose forward
 * pass gg_fp8_grouped_gemm computes, the contraction running over the tokens of each group, with no group padded
 * (the capability of Sec. 2.2 on the contraction dimension).  The paper's title names training and Sec. 4 the kernels
 * around the grouped GEMM, but the paper defines neither layouts nor scale granularity for this operation: the
 * definition is this library's own reading.
 *   XT  e4m3 [K, M_total]   X transposed: feature k of token r at XT[k * M_total + r] (the token index contiguous)
 *   SX  fp32 [ceil(M_total/128), K]   one scale per block of 128 tokens and feature, the scales of a block contiguous
 *       (what a K step of a tile needs is then a few cache lines, not one per feature); the token blocks are
 *       [128 j, 128 j + 128) of the concatenated token axis whatever the groups are (a block may hold tokens of
 *       several groups), so every fetch is 16-byte aligned and a group may start and end at ANY token
 *   DYT e4m3 [N, M_total], SDY fp32 [ceil(M_total/128), N]   the output gradient, transposed likewise
 *   group_offsets int32 [G+1] on the device: tokens of group g are [off[g], off[g+1]); clamped on the device like
 *       those of gg_fp8_grouped_gemm (a bad array garbles results, it cannot make the kernel leave the tensors)
 *   dW  fp32 [G, N, K], EVERY element written:
 *       dW[g][n][k] = sum_j SDY[j][n] * SX[j][k] * sum_{r in block j and in group g} dec(DYT[n][r]) * dec(XT[k][r])
 *       (blocks in ascending order; fp32 accumulation).  A group without tokens gets zeros.  Bytes of tokens outside
 *       a group never reach a product of that group, whatever they are (NaN codes included).
 * M_total a multiple of 16, N of 128, K of 256 (GG_ERR_UNSUPPORTED otherwise); K * M_total and N * M_total below
 * 2^31, K at most 2^20 (GG_ERR_SHAPE).  G == 0: GG_OK, nothing enqueued; M_total == 0 with G > 0: zeros are written
 * (XT, SX, DYT, SDY may then be NULL).  All pointers device memory, 16-byte aligned tensors.  No workspace, nothing
 * allocated, asynchronous on `stream`. */
int gg_fp8_grouped_gemm_wgrad(const void* XT, const float* SX, const void* DYT, const float* SDY,
                              const int32_t* group_offsets, float* dW, int G, int64_t M_total, int N, int K, void* stream);

/* The same with options.  flags: GG_OUT_BF16 (only this call takes it): dW is bfloat16 [G, N, K], the fp32 sum of
 * the definition above rounded once, to nearest even (half the output bytes, which are nine tenths of the operation's
 * traffic); 0: fp32, as gg_fp8_grouped_gemm_wgrad.  Any other bit: GG_ERR_UNSUPPORTED. */
int gg_fp8_grouped_gemm_wgrad_ex(const void* XT, const float* SX, const void* DYT, const float* SDY,
                                 const int32_t* group_offsets, void* dW, int G, int64_t M_total, int N, int K, void* stream,
                                 unsigned flags);

/* The producer of gg_fp8_grouped_gemm_wgrad's operands: the block quantiser of gg_fp8_quantize_rows (the 1x128
 * scaling stated below Table 1 of the paper) applied ALONG THE TOKENS, with the transpose that call wants.  The paper
 * defines neither the operation nor its layouts (Sec. 4 only names the kernels around the grouped GEMM).
 *   X        device, bf16 [T, K], token-major (an activation or an output-gradient tensor as the forward pass holds it)
 *   row_src  device, int32 [M_total]: output token r is row row_src[r] of X (the routing permutation); an index
 *            outside [0, T) stands for a row of zeros; NULL = identity
 *   XT       device, out, e4m3 bytes [K, M_total]: XT[k][r] = quantised X[row_src[r]][k]
 *   SX       device, out, fp32 [ceil(M_total / 128), K], block-major: SX[j][k] scales tokens [128 j, 128 j + 128) of
 *            feature k (the last block: the tokens that exist); amax, scale and rounding as in gg_fp8_quantize_rows
 * K a multiple of 64 and M_total a multiple of 16 (GG_ERR_UNSUPPORTED otherwise).  Bytes and scales are reproducible
 * bit for bit on the host.  XT 16-byte aligned.  Nothing is allocated; asynchronous on `stream`. */
int gg_fp8_quantize_cols(const void* X, const int32_t* row_src, void* XT, float* SX, int64_t T, int64_t M_total, int K,
                         void* stream);

/* ---- the pad-then-GEMM comparison path (the baseline of Sec. 3) ------------
 * Every group is copied to an offset that is a multiple of 128 rows, pad rows
 * are zero, the same GEMM kernels run on the aligned problem, and the valid
 * rows are gathered back.  Numerically identical to the padding-free path on
 * valid rows (the equivalence claimed in Sec. 3.2). */

/* Upper bound on the padded row count for ANY offsets with this G and M_total:
 * 128 * (ceil(M_total / 128) + G).  Size A_pad, SA_pad and C_pad with it. */
int64_t gg_fp8_padded_rows_cap(int G, int64_t M_total);

/* Writes padded_offsets[G+1] (padded_offsets[0] = 0, each group rounded up to a
 * multiple of 128 rows), copies the valid rows of A [M_total,K] and SA
 * [M_total,K/128] to A_pad [M_pad_cap,K] and SA_pad [M_pad_cap,K/128] and
 * zero-fills the pad rows of every group, i.e. every other row of
 * [0, padded_offsets[G]) (Sec. 3: the baseline allocates and fills the padded
 * problem, M_pad rows).  Rows from padded_offsets[G] up to M_pad_cap exist only
 * because the host cannot know M_pad without a synchronisation: they belong to
 * no group, no call of this library reads them, and they are left untouched.
 * M_pad_cap must be at least gg_fp8_padded_rows_cap(G, M_total) (GG_ERR_SHAPE
 * otherwise). */
int gg_fp8_pad(const void* A, const float* SA, const int32_t* group_offsets,
               void* A_pad, float* SA_pad, int32_t* padded_offsets,
               int G, int64_t M_total, int64_t M_pad_cap, int K, void* stream);

/* gg_fp8_pad with options: with GG_SA_KMAJOR, SA is [ceil(K/128), M_total] and SA_pad [ceil(K/128), M_pad_cap]
 * (the padded problem then goes to gg_fp8_grouped_gemm_ex with the same flag, M_total = M_pad_cap and
 * group_offsets = padded_offsets).  Other flag bits: GG_ERR_UNSUPPORTED. */
int gg_fp8_pad_ex(const void* A, const float* SA, const int32_t* group_offsets,
                  void* A_pad, float* SA_pad, int32_t* padded_offsets,
                  int G, int64_t M_total, int64_t M_pad_cap, int K, void* stream, unsigned flags);

/* The GEMM on the aligned problem: identical to gg_fp8_grouped_gemm with
 * M_total = M_pad_cap and group_offsets = padded_offsets.  Pad rows inside
 * [0, padded_offsets[G]) of C_pad are written (as zeros); rows beyond are not. */
int gg_fp8_grouped_gemm_padded(const void* A_pad, const float* SA_pad, const void* B, const float* SB,
                               const int32_t* padded_offsets, void* C_pad,
                               int G, int64_t M_pad_cap, int N, int K,
                               void* workspace, size_t workspace_bytes, void* stream);

/* Gathers the valid rows of C_pad [*, N] bf16 into C [M_total, N] bf16:
 * C[off[g] + i] = C_pad[padded_offsets[g] + i] for i < M^g. */
int gg_fp8_unpad(const void* C_pad, const int32_t* group_offsets, const int32_t* padded_offsets,
                 void* C, int G, int64_t M_total, int N, void* stream);

/* The step in front of the GEMM (the kind of kernel Sec. 4 of the paper says keeps working unchanged on the
 * padding-free layout): quantises rows of X [T, K] bf16 (device) to e4m3 bytes A [M_total, K] and 1x128 block
 * scales SA [M_total, K/128] (Table 1 and the paragraph below it), written in group-contiguous order:
 * output row r takes input row row_src[r] (device int32 [M_total]; NULL = identity).  Per (row, 128-wide K
 * block), in fp32: amax = max(max |x| with NaNs skipped, 2^-100), scale = amax / 448, byte = e4m3 round to
 * nearest even of clamp(x * (448 / amax), -448, 448); a NaN gives the byte 0x7F (so does an infinity: its
 * block has scale inf, its finite elements become 0).  A source index outside [0, T) stands for a row of
 * zeros (zero bytes, scales 2^-100 / 448).  X, A 16-byte aligned; K a multiple of 128 (GG_ERR_UNSUPPORTED
 * otherwise).  The caller owns every buffer; the call is asynchronous on `stream`. */
int gg_fp8_quantize_rows(const void* X, const int32_t* row_src, void* A, float* SA,
                         int64_t T, int64_t M_total, int K, void* stream);

/* The step between the two grouped GEMMs of an expert MLP, on the group-contiguous rows the first GEMM wrote
 * (again a kernel that Sec. 4 of the paper says runs unchanged on the padding-free layout): H [M_total, 2*I]
 * bf16 (device), columns [0, I) the gate projection and [I, 2*I) the up projection;
 * act = bf16 round-to-nearest-even of silu(gate) * up, silu(g) = g / (1 + exp(-g)), evaluated in fp32; then
 * A [M_total, I] e4m3 and SA [M_total, I/128] from act by exactly the recipe of gg_fp8_quantize_rows.
 * act_out (bf16 [M_total, I], device) receives act when it is not NULL.  I a multiple of 128
 * (GG_ERR_UNSUPPORTED otherwise); H, A, act_out 16-byte aligned.  Asynchronous on `stream`. */
int gg_fp8_swiglu_quantize_rows(const void* H, void* A, float* SA, void* act_out,
                                int64_t M_total, int I, void* stream);

/* The two row kernels with options: with GG_SA_KMAJOR they write the scales K-block-major, SA [K/128, M_total]
 * (resp. [I/128, M_total]), the order gg_fp8_grouped_gemm_ex takes with the same flag.  Bytes and scale values are
 * those of the plain entry points.  Other flag bits: GG_ERR_UNSUPPORTED. */
int gg_fp8_quantize_rows_ex(const void* X, const int32_t* row_src, void* A, float* SA,
                            int64_t T, int64_t M_total, int K, void* stream, unsigned flags);
int gg_fp8_swiglu_quantize_rows_ex(const void* H, void* A, float* SA, void* act_out,
                                   int64_t M_total, int I, void* stream, unsigned flags);

/* Debug helper, NOT for the hot path: synchronises `stream`, copies the G+1
 * offsets to the host and returns GG_ERR_OFFSETS unless they are non-decreasing
 * with 0 <= off[0] and off[G] <= M_total. */
int gg_fp8_check_offsets(const int32_t* group_offsets, int G, int64_t M_total, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GG_FP8_H */
