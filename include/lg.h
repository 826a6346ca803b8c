/*
 * lg.h -- C ABI of liblg: the paper's dense structured tensor ops on one AMD
 * MI355X (gfx950), fp32, row-major.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every data pointer is a DEVICE pointer to fp32 elements owned by the
 *    caller.  The library never allocates, frees or retains device memory.
 *    Between calls it keeps no state that results depend on (per process it
 *    remembers which kernels it has configured on which device, and
 *    lg_reduce_cols_static the address of its device array).
 *  - Extents, strides and leading dimensions are in ELEMENTS (int64_t).  A
 *    tensor is row-major: the last index is contiguous.  Operands follow the
 *    memref convention of Section 2.3 (pointer + sizes + strides); only the
 *    row stride of 2-D operands is free, N-D convolution operands are dense.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    A call only enqueues work on it and returns; it never synchronises.
 *  - Outputs are destination-passing operands (Section 3.4): with
 *    `accumulate` == 0 the output is overwritten and never read; with
 *    `accumulate` != 0 the computed value is added to what it holds.
 *  - Inputs must not overlap outputs.
 *  - Entry points may be called from several host threads at once (on their
 *    own streams or devices); what lg_reduce_cols_static shares between calls
 *    is stated there.
 *  - Return value: LG_OK or a negative LG_ERR_* code.  Arguments, workspace
 *    and launch limits of every kernel of a call are checked before the first
 *    kernel is enqueued: with LG_ERR_INVALID_ARG, LG_ERR_UNSUPPORTED or
 *    LG_ERR_WORKSPACE nothing has been enqueued.  LG_ERR_RUNTIME means the HIP
 *    runtime refused a launch; an op made of two kernels (a split reduction or
 *    contraction and the pass that combines its partial results) may then have
 *    its first kernel on the stream and the output must be taken as undefined.
 *    The library never aborts, throws or prints.
 *  - The HIP runtime keeps one "last error" per host thread, shared by all its
 *    users in the process.  An entry point that launches clears it on entry
 *    (an error another library left pending on the calling thread is dropped,
 *    not reported as this library's) and reads it after its own launches.
 *  - An output with a zero extent is a successful no-op.  A zero REDUCTION
 *    extent yields the neutral element 0 (or leaves an accumulated output
 *    unchanged), cf. the neutral padding value of Section 3.2.
 *  - `workspace` is caller-provided device scratch, 256-byte aligned, of at
 *    least the byte count the matching *_workspace_bytes() call returns (which
 *    may be 0, in which case NULL is accepted).  Its contents on entry are
 *    irrelevant and it may be reused once the stream has passed the call.
 *    It must not overlap any operand of the call (LG_ERR_INVALID_ARG).
 *  - Fast paths need 16-byte aligned base pointers and row lengths / leading
 *    dimensions that are multiples of 4 elements; anything else is handled by
 *    slower element-wise kernels with identical results, not rejected.
 */
#ifndef LG_H
#define LG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LG_OK 0
#define LG_ERR_INVALID_ARG (-1) /* null pointer, negative extent, ld < row length, stride/dilation < 1,
                                   window larger than the input, input overlapping output */
#define LG_ERR_UNSUPPORTED (-2) /* valid problem outside what the kernels index (an operand with
                                   2^31 or more elements in a dimension product the kernels
                                   address with 32 bits, or a grid beyond launch limits) */
#define LG_ERR_WORKSPACE (-3)   /* workspace missing, misaligned or too small */
#define LG_ERR_RUNTIME (-4)     /* the HIP runtime refused the launch */

/* Version of this ABI (major * 100 + minor). */
int lg_version(void);

/* Static, human-readable name of a status code. */
const char *lg_status_string(int status);

/*
 * Matrix multiplication, Section 4.6.1 equation (AB):
 *     C[m,n] (+)= sum_k A[m,k] * B[k,n]
 * A is M x K with row stride lda >= K, B is K x N with row stride ldb >= N,
 * C is M x N with row stride ldc >= N.  Products and sums are fp32 (matrix-core
 * FMA); the order of the k-sum is unspecified but fixed for a given shape, so
 * repeated calls give identical bits.
 * Workspace: lg_matmul_workspace_bytes(M, N, K); used to combine partial sums
 * when the k-range is split across workgroups.
 */
int lg_matmul(const float *A, const float *B, float *C,
              int64_t M, int64_t N, int64_t K,
              int64_t lda, int64_t ldb, int64_t ldc,
              int accumulate, void *workspace, size_t workspace_bytes, void *stream);
size_t lg_matmul_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * Matrix multiplication with one transposed operand, Section 4.6.1 equations (A^T B) and (A B^T):
 *     transA:  C[m,n] (+)= sum_k A[k,m] * B[k,n]      A is stored K x M (row stride lda >= M)
 *     transB:  C[m,n] (+)= sum_k A[m,k] * B[n,k]      B is stored N x K (row stride ldb >= K)
 * The transposition is folded into the operand load of the same kernel as lg_matmul (the
 * transposed operand is staged in the other shared-memory layout); nothing is transposed in
 * memory.  transA = transB = 0 is lg_matmul; both set is LG_ERR_UNSUPPORTED (it is not one of the
 * paper's variants).  Workspace: lg_matmul_workspace_bytes(M, N, K).
 */
int lg_matmul_t(const float *A, const float *B, float *C,
                int64_t M, int64_t N, int64_t K,
                int64_t lda, int64_t ldb, int64_t ldc,
                int transA, int transB,
                int accumulate, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Which decomposition lg_matmul (and lg_conv2d_nhwc_hwcf, for its implicit GEMM extents
 * M = N*OH*OW, N = F, K = KH*KW*C) picks for a shape: the workgroup tile block_m x block_n
 * and the number of k-slabs (1 = no split, no workspace).  Host-only query for tools that
 * attribute kernel time to shapes; any of the three output pointers may be NULL.
 * The answer is the planner's choice from the three extents.  What only the call itself can
 * see is not reflected: operands whose pitches or base addresses rule out 128-bit access or
 * exceed a kernel's 32-bit offsets fall back to the 64 x 64 tile, unsplit, and a product with
 * N <= 4 and M, K >= 1024 (a matrix times a few vectors) runs on a row-reduction kernel that
 * has no tile at all.
 */
int lg_matmul_plan(int64_t M, int64_t N, int64_t K, int *block_m, int *block_n, int *k_splits);

/*
 * 1 when that plan of lg_matmul runs fewer workgroups than output tiles, each walking over
 * several (short contractions with a large output: a tile's stores then drain under the next
 * tile's multiplications; Section 4.6.1 fixes what is computed, not the order of the tiles),
 * else 0, also for extents that are not positive (lg_matmul_t with transA walks tiles for the
 * same shapes).  A B^T, convolutions, accumulating calls, operands that rule out 128-bit
 * access and outputs whose rows do not start on 128-byte boundaries run one workgroup per tile,
 * on the tile the planner picks when it leaves the loop out (for such calls lg_matmul_plan
 * reports the loop's tile all the same: it sees the three extents only).
 */
int lg_matmul_plan_tile_loop(int64_t M, int64_t N, int64_t K);

/*
 * The same for lg_matmul_t: the plan may depend on the operand layout (a few dozen rows times a
 * large B stored N x K take k-slabs where AB does not).  lg_matmul_workspace_bytes(M, N, K) covers
 * the plan of every layout.  transA and transB both set is LG_ERR_INVALID_ARG.
 */
int lg_matmul_t_plan(int64_t M, int64_t N, int64_t K, int transA, int transB,
                     int *block_m, int *block_n, int *k_splits);

/*
 * The decomposition as a parameter (the paper's transformations take their tile sizes as
 * parameters and leave the choice to a search, Sections 3.2 and 4.1; here the menu of compiled
 * decompositions is numbered and the default entry points above pick from it with a cost
 * model).  These calls run one chosen entry of the menu on any shape: for autotuning by
 * measurement, and so that tests can hold every kernel variant to every shape.
 *
 *   lg_gemm_variants()       number of menu entries; variants are 0 .. that - 1.
 *   lg_gemm_variant_info()   workgroup block block_m x block_n, k depth per step block_k,
 *                            k_parts: into how many parts a workgroup cuts the k range among
 *                            its own wavefronts (1 for the LDS-tiled kernels), and tile_loop:
 *                            1 when the variant runs fewer workgroups than there are output
 *                            blocks, each walking over several (the chip's fill of workgroups,
 *                            or a third of the blocks if that is fewer), so that a block's
 *                            output stores drain under the next block's multiplications; such a
 *                            variant takes k_splits = 1 only, and runs as the same block
 *                            without the loop for A B^T, convolutions, operands
 *                            that rule out 128-bit accesses, and fewer than 9 blocks.  Any output
 *                            pointer may be NULL.  LG_ERR_INVALID_ARG for an unknown variant.
 *   lg_matmul_variant()      lg_matmul_t with the variant and the number of k-slabs across
 *                            workgroups (k_splits >= 1; the register-direct variants -- those
 *                            with block_m = 16 -- take only 1).  Slabs are whole multiples of
 *                            64 k, so fewer slabs than asked for may run.
 *   lg_conv2d_nhwc_hwcf_variant()   lg_conv2d_nhwc_hwcf likewise.
 *   lg_gemm_variant_workspace_bytes()   workspace those two need for (M, N, K) -- for the
 *                            convolution M = N*OH*OW, N = F, K = KH*KW*C -- 0 when k_splits
 *                            runs as one slab; same alignment rule as lg_matmul's workspace.
 * Arguments, layouts, ownership and errors are those of lg_matmul_t / lg_conv2d_nhwc_hwcf;
 * an unknown variant or a k_splits the variant does not take is LG_ERR_INVALID_ARG.  The
 * register-direct variants address their operands with 32-bit byte offsets: asked to run
 * an A or B of 4 GiB or more, or a leading dimension of 2^26 or more, they return
 * LG_ERR_UNSUPPORTED (the default entry points never pick them for such operands).
 */
int lg_gemm_variants(void);
int lg_gemm_variant_info(int variant, int *block_m, int *block_n, int *block_k, int *k_parts,
                         int *tile_loop);
size_t lg_gemm_variant_workspace_bytes(int64_t M, int64_t N, int64_t K, int variant, int k_splits);
int lg_matmul_variant(const float *A, const float *B, float *C,
                      int64_t M, int64_t N, int64_t K,
                      int64_t lda, int64_t ldb, int64_t ldc,
                      int transA, int transB, int accumulate,
                      int variant, int k_splits,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * 2-D convolution, Section 4.6.2 equation (2-D), NHWC input, HWCF filter:
 *     O[n,h,w,f] (+)= sum_{kh,kw,c} I[n, h*SH + kh*DH, w*SW + kw*DW, c] * Kf[kh,kw,c,f]
 * (cross-correlation: the filter is not flipped).  I is dense [N,H,W,C], Kf is
 * dense [KH,KW,C,F], O is dense [N,OH,OW,F] with the "valid" extents
 *     OH = (H - DH*(KH-1) - 1) / SH + 1,   OW = (W - DW*(KW-1) - 1) / SW + 1
 * (floor division); there is no padding.  LG_ERR_INVALID_ARG when the dilated
 * window does not fit in the input.  The 1-D op of the same section is the case
 * H = KH = 1.  Computed as an implicit GEMM of size (N*OH*OW) x F x (KH*KW*C).
 */
int lg_conv2d_nhwc_hwcf(const float *I, const float *Kf, float *O,
                        int64_t N, int64_t H, int64_t W, int64_t C,
                        int64_t KH, int64_t KW, int64_t F,
                        int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                        int accumulate, void *workspace, size_t workspace_bytes, void *stream);
int lg_conv2d_nhwc_hwcf_variant(const float *I, const float *Kf, float *O,
                                int64_t N, int64_t H, int64_t W, int64_t C,
                                int64_t KH, int64_t KW, int64_t F,
                                int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                                int accumulate, int variant, int k_splits,
                                void *workspace, size_t workspace_bytes, void *stream);

size_t lg_conv2d_workspace_bytes(int64_t N, int64_t H, int64_t W, int64_t C,
                                 int64_t KH, int64_t KW, int64_t F,
                                 int64_t SH, int64_t SW, int64_t DH, int64_t DW);

/*
 * 1-D convolution, Section 3 (the running example) and Section 4.6.2 equation (1-D), NWC input,
 * WCF filter:
 *     O[n,w,f] (+)= sum_{kw,c} I[n, w*SW + kw*DW, c] * Kf[kw,c,f]
 * I dense [N,W,C], Kf dense [KW,C,F], O dense [N,OW,F] with the same "valid" OW as above.
 * Arguments, workspace and errors as for lg_conv2d_nhwc_hwcf, of which this is the case
 * H = KH = 1 (the same kernel runs it).
 */
int lg_conv1d_nwc_wcf(const float *I, const float *Kf, float *O,
                      int64_t N, int64_t W, int64_t C, int64_t KW, int64_t F,
                      int64_t SW, int64_t DW,
                      int accumulate, void *workspace, size_t workspace_bytes, void *stream);
size_t lg_conv1d_workspace_bytes(int64_t N, int64_t W, int64_t C, int64_t KW, int64_t F,
                                 int64_t SW, int64_t DW);

/* Output extent used above for one spatial dimension; 0 when the window does not fit. */
int64_t lg_conv_out_extent(int64_t in, int64_t k, int64_t stride, int64_t dilation);

/*
 * Depthwise convolutions, Section 4.7:
 *   1-D  O[n,w,c]   (+)= sum_kw      I[n, w*SW + kw*DW, c] * Kf[kw,c]
 *   2-D  O[n,h,w,c] (+)= sum_{kh,kw} I[n, h*SH + kh*DH, w*SW + kw*DW, c] * Kf[kh,kw,c]
 * I dense [N,W,C] / [N,H,W,C]; Kf dense [KW,C] / [KH,KW,C]; O dense with the
 * same "valid" output extents as lg_conv2d_nhwc_hwcf.
 */
int lg_dwconv1d_nwc_wc(const float *I, const float *Kf, float *O,
                       int64_t N, int64_t W, int64_t C, int64_t KW,
                       int64_t SW, int64_t DW, int accumulate, void *stream);
int lg_dwconv2d_nhwc_hwc(const float *I, const float *Kf, float *O,
                         int64_t N, int64_t H, int64_t W, int64_t C,
                         int64_t KH, int64_t KW,
                         int64_t SH, int64_t SW, int64_t DH, int64_t DW,
                         int accumulate, void *stream);

/*
 * Reductions of a 2-D tensor to a 1-D tensor, Section 4.4 (RowRed2D, ColRed2D):
 *   lg_reduce_rows:  out[i] (+)= sum_j in[i,j]   out has R  entries
 *   lg_reduce_cols:  out[j] (+)= sum_i in[i,j]   out has Cn entries
 * `in` is R x Cn with row stride ld >= Cn.  Sums are fp32, formed as short
 * per-lane partial sums combined by trees (never one long running sum).
 * lg_reduce_cols splits the rows across workgroups and combines the partial
 * vectors from the workspace.  lg_reduce_rows gives every row one workgroup (one
 * wavefront when Cn < 4096) and needs no workspace; it fills the GPU once R is in
 * the hundreds, while a handful of very long rows occupy only as many compute units.
 * lg_reduce_rows_ws is the same operation with a workspace: when there are fewer
 * than 512 rows of at least 32768 elements it cuts every row into pieces, one
 * workgroup each, and adds the piece sums in a second pass (in ascending order of
 * position: the result does not depend on timing).  lg_reduce_rows_workspace_bytes
 * says how much it needs for a shape (0: it runs exactly as lg_reduce_rows and
 * workspace may be NULL); the workspace is device memory, 256-byte aligned, owned
 * by the caller, free for reuse once the call's work on the stream has finished;
 * missing, misaligned or too small is LG_ERR_WORKSPACE.
 */
int lg_reduce_rows(const float *in, float *out, int64_t R, int64_t Cn, int64_t ld,
                   int accumulate, void *stream);
int lg_reduce_rows_ws(const float *in, float *out, int64_t R, int64_t Cn, int64_t ld,
                      int accumulate, void *workspace, size_t workspace_bytes, void *stream);
size_t lg_reduce_rows_workspace_bytes(int64_t R, int64_t Cn);
int lg_reduce_cols(const float *in, float *out, int64_t R, int64_t Cn, int64_t ld,
                   int accumulate, void *workspace, size_t workspace_bytes, void *stream);
size_t lg_reduce_cols_workspace_bytes(int64_t R, int64_t Cn);

/*
 * lg_reduce_cols for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation,
 * arguments, results (bit for bit) and errors as lg_reduce_cols, minus the workspace: the partial
 * column sums go to a fixed 4 MiB array in device memory that belongs to the library (each GPU the
 * library runs on holds its own copy from the first call there until the process ends).  The call
 * allocates and frees nothing.  A shape whose partial sums need more than 4 MiB -- more than
 * lg_reduce_cols_workspace_bytes(R, Cn) = 4194304 -- is LG_ERR_UNSUPPORTED; nothing is enqueued
 * then.  All calls on one GPU share that array: calls that may overlap in time on one GPU (two
 * streams, two host threads) race on it and must be serialised by the caller; calls on one stream
 * are ordered by the stream.  Nothing in the array has to be cleared between calls: every partial
 * sum a call reads it has written itself.
 */
int lg_reduce_cols_static(const float *in, float *out, int64_t R, int64_t Cn, int64_t ld,
                          int accumulate, void *stream);

/*
 * 2-D transpose, Section 4.4 (Transpose2D):   out[j,i] = in[i,j]
 * `in` is R x Cn with row stride ld_in >= Cn; `out` is Cn x R with row stride
 * ld_out >= R.  Bit patterns are moved untouched (NaN payloads, signed zeros
 * and denormals survive).  In-place operation is rejected.
 */
int lg_transpose(const float *in, float *out, int64_t R, int64_t Cn,
                 int64_t ld_in, int64_t ld_out, void *stream);

/*
 * 2-D copy, Section 4.4 (Copy2D):   out[i,j] = in[i,j]
 * The paper's bandwidth yardstick; here the measured HBM ceiling the
 * memory-bound ops are quoted against.
 */
int lg_copy2d(const float *in, float *out, int64_t R, int64_t Cn,
              int64_t ld_in, int64_t ld_out, void *stream);

/*
 * Matrix-pipe yardstick (calibration, the compute counterpart of lg_copy2d): 512 workgroups of
 * four wavefronts, each wavefront issuing 4 * iters independent 32x32x2 fp32 MFMAs on registers
 * only, no memory traffic in the loop.  lg_mfma_probe_flops(iters) divided by the launch's
 * duration is the fp32 matrix rate this part sustains; the GEMM figures are quoted against it
 * beside the theoretical peak the paper uses for its compute-bound kernels (Section 4.3).
 * `out` receives lg_mfma_probe_out_elems() floats (one checksum per lane, so the work is
 * observable); out_elems is the caller's buffer length in elements and must be at least that.
 * 0 <= iters <= 2^22; anything else, or a short or null buffer, is LG_ERR_INVALID_ARG.
 */
int lg_mfma_probe(float *out, int64_t out_elems, int64_t iters, void *stream);
int64_t lg_mfma_probe_out_elems(void);
double lg_mfma_probe_flops(int64_t iters);

/*
 * HBM stream yardsticks (calibration, beside lg_copy2d): the paper quotes its bandwidth-bound
 * kernels against measured copy bandwidths and their read/write mixes (Section 4.3); these are
 * the three mixes on this part, with the launch shape and cache hints as parameters so that the
 * sweep behind a quoted ceiling can be repeated.
 *   mode 0  read   n floats of `in` are loaded and summed per lane; `out` is a sink of at least
 *                  1024 floats that is written only if a sum is NaN (never, for finite inputs)
 *   mode 1  write  n floats of `out` are overwritten with a constant pattern; `in` is ignored
 *   mode 2  copy   out[i] = in[i] for n floats
 * n is a multiple of 4 and both pointers are 16-byte aligned device pointers.  Every lane moves
 * `unroll` (1, 2, 4, 8) 128-bit words, `threads` (256, 512, 1024) apart, of its workgroup's
 * contiguous chunk.  hint bit 0: loads carry the non-temporal hint; bit 1: stores do.
 * Anything else is LG_ERR_INVALID_ARG; `in` overlapping what is written likewise.
 */
int lg_stream_probe(int mode, const float *in, float *out, int64_t n, int threads, int unroll, int hint,
                    void *stream);

/*
 * Batched 2-D transpose, Section 4.4: a transpose of more than two dimensions is a set of 2-D
 * transposes at various places in the tensor (the paper's example: [i,j,k,l] -> [k,j,l,i] is
 * j x k transposes of an i x l matrix).  For every b0 < B0, b1 < B1, i < R, j < Cn:
 *     out[b0*out_stride0 + b1*out_stride1 + j*ld_out + i] =
 *      in[b0*in_stride0  + b1*in_stride1  + i*ld_in  + j]
 * All strides in elements, >= 0; ld_in >= Cn, ld_out >= R.  B0, B1 <= 65535.  One launch.
 * Bit-exact data movement.  The output slices of different batches must not overlap each
 * other (not checked); in and out as a whole must not overlap (checked).
 */
int lg_transpose_batched(const float *in, float *out, int64_t R, int64_t Cn,
                         int64_t ld_in, int64_t ld_out,
                         int64_t B0, int64_t B1,
                         int64_t in_stride0, int64_t in_stride1,
                         int64_t out_stride0, int64_t out_stride1, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LG_H */
