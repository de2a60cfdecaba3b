/*
 * flexgemm -- flexible mixed-precision GEMM and GETT-style tensor contraction for AMD MI355X
 * (gfx950).  C ABI of the shared library libflexgemm.so.
 *
 * The operations follow "Flexible Performant GEMM Kernels on GPUs" (arXiv 2009.12263):
 *   - Section 2.2:   the matrix unit computes D = A.B + C with FP16 A, B and FP32 C, D;
 *   - Section 4.3.2: the BLAS-like form C := alpha.A.B + beta.C with 'N'/'T' operands;
 *   - Section 5.1:   'N' = column-major, 'T' = row-major storage of an operand;
 *   - Section 5.2:   diagonal operands (only the diagonal is stored, zeros are never read,
 *                    inner-loop iterations off the diagonal are skipped);
 *   - Section 5.3:   fused elementwise operations and a bias vector (epilogue);
 *   - Section 5.4:   complex operands as four real products on split (planar) storage;
 *   - Section 5.5:   tensor contractions whose modes are mapped to GEMM tile coordinates
 *                    while tiles are loaded (GETT), never by separate transposition.
 *
 * General conventions
 *   - Every data pointer (matrix/tensor elements, bias) is a DEVICE pointer to memory the
 *     caller owns.  The library never allocates, frees, retains or copies caller memory.
 *   - The library owns one 64 MiB device workspace per GPU, allocated by fg_init() or by the
 *     first fg_gemm / fg_gemm_ex call that needs it and kept until the process ends.  It holds the
 *     partial products of split-K calls (outputs with too few tiles to fill the GPU and a long K,
 *     or the leftover tiles of the last, partly filled round of a larger output, are computed as
 *     partial products over ranges of K plus a reduction pass, the cross-workgroup reduction
 *     use of the epilogue in Section 4.2.5).  fg_gemm_plan() tells whether a problem is computed
 *     that way ("+splitk<n>" / "+tailsplitk<n>" in the plan name).  All such calls on one GPU share
 *     the workspace: calls on one stream are ordered anyway, and a call on another stream than the
 *     previous user's is made to wait on the device (an event recorded after that user's reduction
 *     pass) until the workspace is free, so calls on different streams may be issued freely; they
 *     are serialised, not run side by side.  The exception is a stream under graph capture: the
 *     caller orders captured split-K calls against other users of the workspace, and the workspace
 *     must exist before the capture begins (fg_init(); FG_ERR_UNSUPPORTED otherwise).  The partial
 *     products are added in a fixed order, so results do not depend on scheduling.
 *   - Every descriptor pointer (fg_matrix, fg_epilogue, mode/extent/stride arrays) is a HOST
 *     pointer, read only during the call.
 *   - Work is enqueued on `hip_stream` (a hipStream_t, NULL = the default stream) and the call
 *     returns without synchronising.  Calls on one stream execute in order.
 *   - Errors are reported by the return value only; nothing is launched when a call fails, and
 *     nothing is thrown or aborted across this boundary.  fg_last_error() gives a message.
 *   - Leading dimensions and strides are in ELEMENTS.
 *   - Alignment: the tiled kernels need element base pointers that are 16-byte aligned, leading
 *     dimensions of 16-bit operands that are multiples of 8 and of FP32 operands multiples of 4
 *     (Section 4.2.2: the aligned layouts that permit 128-bit accesses), and a K that is a
 *     multiple of 8.  A real, non-diagonal product that misses any of these (any leading
 *     dimension, pointers aligned to an element only, any K) is computed by a general kernel:
 *     same operation and options, much slower.  Complex, dual and diagonal products have no
 *     general kernel: FG_ERR_ALIGN (FG_ERR_UNSUPPORTED for K).  Pointers that are not aligned to
 *     an element are always FG_ERR_ALIGN.
 *   - Sizes: M and N are arbitrary; tiles that hang over the edge of a matrix are predicated
 *     (the paper requires inputs padded to the tile sizes and names predication as future work,
 *     Section 7).  M, N or K equal to zero is accepted: with M == 0 or N == 0 nothing is done;
 *     with K == 0 the product term is zero.  The tiled kernels may read (never write) up to 14
 *     bytes past the last element of A or B inside the same 16-byte chunk.  A matrix may be of
 *     any size in bytes (also above 2 GiB); what is bounded is the leading dimension
 *     (FG_ERR_UNSUPPORTED beyond): below 2^22 elements for an operand stored with K contiguous
 *     (A row-major, B column-major), below 2^24 for the other layouts of A and B, below 2^21
 *     for C and D; half of each for interleaved complex matrices.  M, N and K are at most 2^30.
 *   - D may alias C exactly (same pointer, layout and ld: the in-place BLAS form).  A and B
 *     must not overlap D.  With beta == 0 the C term is absent and C (Cin) is never read, so it may
 *     hold anything, NaN included (the BLAS convention).
 *   - Non-finite values: NaN and infinities in A, B, C or bias propagate into D as IEEE arithmetic
 *     produces them; with FG_ACT_RELU a NaN becomes 0 (relu(y) is the comparison y > 0 ? y : 0).
 *     Memory outside the described matrices (the padding between ld and the extent, the bytes
 *     after the last element) may hold anything: it never influences a result.
 */
#ifndef FLEXGEMM_H
#define FLEXGEMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FG_OK = 0,
    FG_ERR_NULL = 1,         /* a required pointer is NULL                                   */
    FG_ERR_SHAPE = 2,        /* negative size, leading dimension smaller than the extent     */
    FG_ERR_LAYOUT = 3,       /* layout / dtype value not valid for that operand              */
    FG_ERR_ALIGN = 4,        /* pointer or leading dimension not aligned as required         */
    FG_ERR_UNSUPPORTED = 5,  /* valid request that this version does not implement           */
    FG_ERR_MODES = 6,        /* inconsistent contraction description                         */
    FG_ERR_LAUNCH = 7        /* the HIP runtime refused the launch (no device, bad stream)   */
} fg_status;

typedef enum {
    FG_F16 = 0, FG_BF16 = 1,   /* A, B: IEEE binary16 / bfloat16 (FG_F16 also for C, D: see fg_gemm) */
    FG_F32 = 2,                /* C, D                                                           */
    FG_CF16 = 3,               /* A, B: interleaved complex, element = (re, im) as two binary16  */
    FG_CF32 = 4                /* C, D: interleaved complex, element = (re, im) as two binary32  */
} fg_dtype;

typedef enum {
    FG_COL = 0,   /* column-major ('N'): element (r, c) at r + c*ld                            */
    FG_ROW = 1,   /* row-major ('T'):    element (r, c) at c + r*ld                            */
    FG_DIAG = 2,  /* diagonal: `re` points at the min(rows, cols) diagonal entries; every other
                     element is zero and is never read; ld is ignored (A or B only)            */
    FG_ZERO = 3   /* all-zero matrix that is never read (C only; same as passing C == NULL)    */
} fg_layout;

typedef enum { FG_ACT_NONE = 0, FG_ACT_RELU = 1 } fg_act;       /* relu(y) = max(y, 0)         */

/* A matrix operand.  `im == NULL`: real matrix, or, with dtype FG_CF16 / FG_CF32, a complex matrix
 * in interleaved storage (Section 5.4: the real and imaginary part of an element are adjacent;
 * `re` points at the first real part; ld counts complex elements).  `im != NULL`: complex matrix
 * in planar-split storage, real parts at `re` and imaginary parts at `im`, both with the same
 * layout and ld. */
typedef struct {
    void   *re;
    void   *im;
    int32_t dtype;    /* fg_dtype  */
    int32_t layout;   /* fg_layout */
    int64_t ld;
} fg_matrix;

/* Operations fused into the store of D (Section 5.3): D = act(alpha.A.B + beta.C + bias). */
typedef struct {
    const float *bias;      /* device pointer or NULL                                           */
    int32_t      bias_dim;  /* 0: length M, bias[i] added to row i; 1: length N, bias[j] added
                               to column j                                                      */
    int32_t      act;       /* fg_act */
} fg_epilogue;

/*
 * D = act(alpha * op(A) * op(B) + beta * C + bias)       (Sections 2.2, 4.3.2, 5.1-5.4)
 *
 * op(A) is the logical M x K matrix and op(B) the logical K x N matrix described by A and B;
 * C and D are M x N.  16-bit elements are multiplied exactly and accumulated in FP32.
 *   A, B : both FG_F16 or both FG_BF16 (IEEE binary16 / bfloat16: the matrix unit multiplies
 *          either kind into FP32, Section 2.2); layout FG_COL, FG_ROW or FG_DIAG (at most one of
 *          A, B diagonal).  FG_BF16 is accepted for real, non-diagonal operands; otherwise
 *          FG_ERR_UNSUPPORTED.
 *   C    : FG_F32, FG_COL or FG_ROW with the same layout as D; NULL or FG_ZERO means no C term
 *          (beta is then ignored).
 *   D    : FG_F32, FG_COL or FG_ROW; written.
 *   C, D stored in lower precision (the type-conversion use of transforms, Section 4.2.3): D, and
 *          C if given, may both be FG_F16.  C is widened exactly when it is loaded, everything
 *          is computed in FP32 as above, and the result is rounded to nearest even when it is
 *          stored.  Any leading dimension and element-aligned pointers are accepted for them.
 *          For real FG_F16 A and B in FG_COL / FG_ROW layout without an addition on A and B, and
 *          with A, B, K meeting the alignment of the tiled kernels (FG_ERR_UNSUPPORTED or
 *          FG_ERR_ALIGN otherwise).
 *   ep   : NULL means no bias and no activation.
 * Complex: if A or B has `im`, the product is complex; this version needs `im` on both A and B
 * (FG_ERR_UNSUPPORTED otherwise), D must have `im`, C (if given) must have `im`, alpha and beta
 * are real, `ep` must be NULL or empty, and diagonal operands are not combined with complex.
 * Interleaved complex: A and B FG_CF16, D (and C if given) FG_CF32, all four interleaved (a mix
 * of planar and interleaved matrices is FG_ERR_UNSUPPORTED); the same rules otherwise.  The parts
 * are separated while tiles are copied into the LDS (the paper's split shared-memory layout).
 */
fg_status fg_gemm(int64_t M, int64_t N, int64_t K, float alpha,
                  const fg_matrix *A, const fg_matrix *B,
                  float beta, const fg_matrix *C,
                  const fg_matrix *D, const fg_epilogue *ep,
                  void *hip_stream);

/* Operations applied to elements right after they are loaded (the "transforms" of Section 4.3;
 * the last two rows of the fusion table of Section 5.3: ReLU on C, an addition on A and B). */
typedef struct {
    float   a_add;   /* every element of A becomes half(A_ik + a_add): a_add is rounded to FP16      */
    float   b_add;   /* (nearest even) and the sum is formed and rounded once in FP16; likewise B.   */
                     /* Both 0: A and B are used as stored.                                          */
    int32_t c_act;   /* fg_act applied to every element of C before it is scaled by beta             */
} fg_load_transforms;

/*
 * D = act(alpha * (A + a_add) * (B + b_add) + beta * c_act(C) + bias): fg_gemm with transforms on
 * the loaded elements.  `lt == NULL` is fg_gemm.  All arguments, requirements and errors as for
 * fg_gemm; in addition a non-zero a_add or b_add needs real FG_F16 operands in FG_COL or FG_ROW
 * layout (FG_ERR_UNSUPPORTED for complex, FG_BF16 or diagonal operands), and c_act needs a real
 * product.  Elements of A and B outside the M x K and K x N matrices stay zero.
 */
fg_status fg_gemm_ex(int64_t M, int64_t N, int64_t K, float alpha,
                     const fg_matrix *A, const fg_matrix *B,
                     float beta, const fg_matrix *C,
                     const fg_matrix *D, const fg_epilogue *ep,
                     const fg_load_transforms *lt, void *hip_stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): fg_gemm_ex with the same arguments, results and errors,
 * except that the partial products of a K split go to a 16 MiB array that is part of the library's
 * device image (one copy per GPU, held until the process ends) instead of the 64 MiB workspace.
 * The call makes the same plan as fg_gemm_ex, so its result is bit-identical; when that plan's
 * partial products need more than 16 MiB (tiles to split x K ranges x tile bytes, e.g. a 2048 x 2048
 * output split three ways) it returns FG_ERR_UNSUPPORTED and launches nothing.  It never calls
 * hipMalloc, hipFree or any allocating routine; for that to cover the runtime's own first-use
 * work (loading the kernels, looking up the array's address) call fg_init() once per device
 * beforehand.  Nothing in the array needs clearing between calls (every partial tile is written
 * whole before the reduction pass reads it).  All calls on one GPU share the array and are NOT
 * ordered against each other by the library: calls on one stream are safe, calls that overlap in
 * time on different streams of one GPU race.
 */
fg_status fg_gemm_noalloc(int64_t M, int64_t N, int64_t K, float alpha,
                          const fg_matrix *A, const fg_matrix *B,
                          float beta, const fg_matrix *C,
                          const fg_matrix *D, const fg_epilogue *ep,
                          const fg_load_transforms *lt, void *hip_stream);

/*
 * Dual-number product (Section 5.4): every element is x + eps.x' with eps^2 = 0, stored like the
 * planar complex matrices (value plane at `re`, dual plane at `im`), so
 *     D.re = alpha * A.re.B.re + beta * C.re
 *     D.im = alpha * (A.re.B.im + A.im.B.re) + beta * C.im
 * i.e. a product and its first derivative in one pass (three real products instead of the four
 * of a complex product).  Arguments, layouts, sizes and errors as for a complex fg_gemm without
 * epilogue: A, B FG_F16 with both planes, D (and C if given) with both planes, alpha and beta real.
 */
fg_status fg_gemm_dual(int64_t M, int64_t N, int64_t K, float alpha,
                       const fg_matrix *A, const fg_matrix *B,
                       float beta, const fg_matrix *C,
                       const fg_matrix *D, void *hip_stream);

/*
 * Cout[modesC] = alpha * sum over contracted modes of A[modesA] * B[modesB] + beta * Cin[modesC]
 *                                                                     (Sections 4.1 and 5.5)
 * A mode is an integer label; `mode_labels[n_modes]` lists the distinct labels and
 * `mode_extents[n_modes]` their extents.  modesX[nX] / stridesX[nX] give, for tensor X, its
 * modes in storage order and the element stride of each.  Every label that is used must appear
 * in two or in all three of {A, B, C}: modes shared by A and C become GEMM rows, modes shared by
 * B and C become GEMM columns, modes shared by A and B are summed over, and modes in all three
 * are batch modes (an independent contraction per index; FG_ERR_MODES for a mode in one tensor
 * only or listed twice in a tensor).  A, B are FP16 device tensors, Cin (NULL iff beta term
 * absent) and Cout FP32; Cout may equal Cin.  The tensors are never transposed in memory: the
 * mode-to-tile mapping happens while tiles are loaded and while the result is stored.
 * Fast path (the tiled matrix-unit kernels): in each of A and B some mode that is not a batch mode
 * has stride 1 and an extent that is a multiple of 8; every other stride of A and B is a multiple
 * of 8 elements and the base pointers are 16-byte aligned (so that 16-byte pieces along the
 * contiguous mode stay aligned); if both A and B are contiguous along a summed mode it is the same
 * one; there is a summed mode; A, B and C each span less than 2 GiB.  (The summed mode that is
 * walked fastest -- A's unit-stride mode if it is summed, else B's, else the first summed mode of A
 * -- is covered in steps of 64; an extent that is not a multiple of 64 costs the zero-filled
 * remainder of the last step.)  The row and column extents are otherwise arbitrary: tiles that
 * hang over the merged row or column extent are predicated like the edge tiles of fg_gemm.
 * A description that misses any of these is computed by a general kernel: the same mode mapping
 * with element-wise loads and 64-bit offsets, any strides, any extents, element-aligned pointers,
 * tensors of any size, outer products; much slower.  fg_contract_plan() tells which one serves a
 * description, and why.
 * Limits of both (FG_ERR_UNSUPPORTED): at most 4 modes of extent above 1 per group (rows, columns,
 * summed, batch); merged extents up to 2^30 and at most 2^20 batch indices; no negative strides.
 * Base pointers must be aligned to an element (FG_ERR_ALIGN).
 */
fg_status fg_contract(int32_t nA, const int32_t *modesA, const int64_t *stridesA, const void *A,
                      int32_t nB, const int32_t *modesB, const int64_t *stridesB, const void *B,
                      int32_t nC, const int32_t *modesC, const int64_t *stridesC,
                      const float *Cin, float *Cout,
                      int32_t n_modes, const int32_t *mode_labels, const int64_t *mode_extents,
                      float alpha, float beta, void *hip_stream);

/*
 * Name of the kernel fg_contract would use for this description (same descriptor arguments; the
 * data pointers are only inspected for alignment), as a NUL-terminated string in `buf`:
 * "gett_<layouts>_<tile>" or "gett_stream_..." for the tiled kernels (the latter when whole
 * lines of the result stream past the L2; a tile name ending in "_deep" is the 128x128 tile with a
 * ring of four buffers, for results of at most one such tile per compute unit), or "gett_general_64x64x32 (<reason>)" with the first
 * requirement of the tiled kernels that the description misses.  Returns what fg_contract would
 * return for the description.
 */
fg_status fg_contract_plan(int32_t nA, const int32_t *modesA, const int64_t *stridesA, const void *A,
                           int32_t nB, const int32_t *modesB, const int64_t *stridesB, const void *B,
                           int32_t nC, const int32_t *modesC, const int64_t *stridesC,
                           const float *Cin, float *Cout,
                           int32_t n_modes, const int32_t *mode_labels, const int64_t *mode_extents,
                           char *buf, int32_t buf_len);

/* Message for the most recent failing call on this thread ("" if none).  The pointer refers to
 * thread-local static storage: valid until the next library call on the same thread. */
const char *fg_last_error(void);

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t fg_version(void);

/*
 * Tuning aid, not part of the method: the planner's overrides FG_FORCE_TILE (0..5: tile shape; 0..2 for complex and
 * dual products, whose kernels have three),
 * FG_FORCE_SPLIT (n: K ranges for every tile) and FG_FORCE_TAIL (n: K ranges for the tiles of the
 * last round; 1: never) are environment variables read once, when the library is loaded.  This
 * call reads them again (for a process that changes its environment afterwards).
 */
void fg_reload_tuning(void);

/*
 * Optional: prepare every kernel variant on the current device (raise its LDS limit, query its
 * occupancy), allocate the split-K workspace and look up the static scratch array of fg_gemm_noalloc.  Without it each variant is prepared by the first
 * call that uses it, and the workspace is allocated by the first call that splits K.  After
 * fg_init() on a device, fg_gemm / fg_gemm_ex / fg_gemm_dual / fg_contract on that device do
 * nothing but enqueue one kernel (two or three when K is split) on the given stream, so they may be recorded into a HIP graph
 * (stream capture) and replayed.  Returns FG_OK or FG_ERR_LAUNCH.
 */
fg_status fg_init(void);

/*
 * Name of the kernel variant and block tile that fg_gemm would use for this problem, written as
 * a NUL-terminated string into `buf` (at most `buf_len` bytes), followed by "+splitk<n>" when K
 * is split into n ranges for every tile, or "+tailsplitk<n>" when only the tiles of the last round
 * are split.  A name ending in "_k32" is the kernel built on 16x16x32 matrix instructions, used for
 * outputs with a 256x256 tile for at least three quarters of the compute units; the others use 32x32x16 instructions.  Both
 * accumulate the same FP16 products in FP32, in a different order: results agree within the stated
 * tolerance and are bit-identical on integer-valued data.
 * This is the "params" choice of Section 4.2.1, made here by an estimate
 * of the run time of every tile shape and split.  `variant` (fg_plan_variant) names the operator: real FP16, planar complex, dual, real BF16,
 * interleaved complex, real FP16 with C and D stored as binary16, or real FP16 with a constant added to the
 * loaded A and B values (fg_gemm_ex with a_add or b_add).
 * Returns FG_OK, or the status fg_gemm would return for these sizes and layouts.
 */
typedef enum { FG_PLAN_REAL = 0, FG_PLAN_COMPLEX = 1, FG_PLAN_DUAL = 2, FG_PLAN_REAL_BF16 = 3,
               FG_PLAN_COMPLEX_INTERLEAVED = 4, FG_PLAN_REAL_F16_CD = 5, FG_PLAN_REAL_AB_ADD = 6 } fg_plan_variant;
fg_status fg_gemm_plan(int64_t M, int64_t N, int64_t K, int32_t layoutA, int32_t layoutB,
                       int32_t layoutD, int32_t variant, char *buf, int32_t buf_len);

/*
 * Measurement aid, not part of the method: launches a kernel that only issues
 * v_mfma_f32_32x32x16_f16 (iters * 32 per wave, 8 waves on each of the 256 compute units) on
 * operand fragments read from the first 48 KiB of `fp16_operands` (device pointer, 16-byte aligned,
 * `operand_bytes` bytes of FP16 values, at least 48 KiB, FG_ERR_SHAPE otherwise; e.g. the A matrix
 * of a workload) and writes the number of floating-point
 * operations of the launch to *flops_out (host).  Timed by the caller, it gives the MFMA rate the
 * chip sustains for that operand data: the engine clock is power-managed and dense MFMA power
 * depends on the operand values.  Returns FG_ERR_NULL / FG_ERR_SHAPE (iters outside 1..2^20) /
 * FG_ERR_ALIGN / FG_ERR_LAUNCH.
 */
fg_status fg_probe_mfma(const void *fp16_operands, int64_t operand_bytes, int32_t iters, int64_t *flops_out, void *hip_stream);

/*
 * The same measurement with v_mfma_f32_16x16x32_f16, the instruction of the "_k32" kernels
 * (iters * 64 per wave: the same number of floating-point operations per iteration, same
 * arguments, same return values).  On operand data that keeps the chip at its power limit the two
 * shapes sustain different rates.
 */
fg_status fg_probe_mfma_k32(const void *fp16_operands, int64_t operand_bytes, int32_t iters, int64_t *flops_out, void *hip_stream);

/*
 * Measurement aid: the matrix-instruction stream of fg_probe_mfma_k32 together with the other
 * instructions of the 256x256x64 kernel's K loop in its proportions -- per 64 matrix instructions
 * 24 fragment reads of 1 KB from LDS and 8 direct-to-LDS loads of 1 KB (from a window of at most
 * 4 MiB of `fp16_operands`, which needs at least 128 KiB) -- with no dependence between them, no
 * barrier and no epilogue.  Its rate is what the compute units sustain for that instruction mix on
 * that data, i.e. the bound of a K loop with this tile shape however it is scheduled.  Same
 * arguments and return values as fg_probe_mfma.
 */
fg_status fg_probe_kloop_mix(const void *fp16_operands, int64_t operand_bytes, int32_t iters, int64_t *flops_out, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FLEXGEMM_H */
