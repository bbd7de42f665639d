/*
 * csrk — FP32 CSR sparse kernels for AMD Instinct MI355X (gfx950):
 *   SPMM     O = S . B                       (paper eq. (2), Algorithm 2)
 *   SDDMM    P = S (.) (A . B^T) on S's pattern  (paper eq. (1), Algorithm 1)
 *   FusedMM  O = (S (.) (A . B^T)) . C       (paper eq. (3), Algorithm 3)
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every pointer is a DEVICE pointer owned by the caller and valid on the
 *    device that is current when the call is made.  Nothing is copied to or
 *    from the host.
 *  - S is M x K in compressed sparse row form exactly as in the paper's section
 *    "Matrix Storage Layout" (Fig. 1): `rowptr` has M+1 int32 entries, 0-based,
 *    non-decreasing, rowptr[0] = 0 and rowptr[M] = nnz; `colidx` has nnz int32
 *    column indices in [0, K); `vals` has nnz FP32 values in the same order.
 *    Entries of a row may be in any order and may repeat (SPMM/FusedMM add
 *    repeated entries up, SDDMM yields one result per stored entry); explicitly
 *    stored zeros are ordinary entries.  The library reads nnz from rowptr[M] on
 *    the device; colidx, vals and P are never dereferenced when it is 0, so they
 *    may be NULL then.  Index contents are not validated by the compute calls: an
 *    out-of-range index or a decreasing rowptr is undefined behaviour (use
 *    csrk_validate_csr first when inputs are untrusted).
 *  - Dense matrices are FP32, row-major and contiguous (leading dimension = row
 *    length).
 *  - Calls are asynchronous: work is enqueued on `stream` and the call returns
 *    without synchronising.  Inputs must stay valid and unchanged, and outputs
 *    untouched, until the stream has passed the enqueued work.
 *  - Outputs are overwritten (there is no alpha/beta; Algorithm 2 starts from a
 *    zero row).  Rows of S with no entries give zero rows of O.  M == 0, N == 0,
 *    D == 0 or nnz == 0 are valid: with D == 0 every dot product is empty (0).
 *  - O must not overlap any input.  P may be the same array as vals (the
 *    paper's SDDMM overwrites the values of the sparse matrix in place).
 *  - Scratch.  SPMM and FusedMM need device memory beyond their operands for partial
 *    rows (8192 x N floats on an MI355X) or, when M is small and the reduction
 *    dimension is cut into up to 8 ranges, for partial outputs (at most 8 x M x N
 *    floats), plus a few flag words; SDDMM needs the flag words only.  Three ways to
 *    provide it:
 *      * spmm_csr / sddmm_csr / fusedmm_csr (and their planned and bfloat16 forms) use
 *        an area the library keeps per device.  It is allocated (hipMalloc, which
 *        synchronises) the first time it is needed, replaced when it has to grow (after
 *        a hipDeviceSynchronize), and kept until csrk_release_workspace or process exit.
 *        These calls take a process-wide lock for their duration and share the area:
 *        two of them in flight at once on different streams of one device would race
 *        on it, so serialise them on one stream.  This is the convenience path.
 *      * *_csr_ws take a workspace from the caller (csrk_workspace_bytes gives the
 *        size).  They allocate nothing, free nothing, never synchronise, take no lock
 *        and keep no state between calls: calls on different streams with different
 *        workspaces are independent, and every call can be captured in a HIP graph.
 *      * csrk_plan_reserve gives a plan a workspace of its own; planned calls that fit
 *        into it then behave like the *_csr_ws calls.
 *    Results do not depend on timing: partial rows and partial outputs are added in a
 *    fixed order.
 *  - Return value: CSRK_OK or an error code; csrk_last_error() then gives a
 *    message for the calling thread.  On error nothing has been enqueued.
 *  - Any N >= 1 and D >= 1 work.  Widths that are multiples of 4 with 16-byte
 *    aligned dense pointers take the fast (128-bit access) kernels.
 */
#ifndef CSRK_H
#define CSRK_H

#include <stddef.h>
#include <stdint.h>
#include <hip/hip_runtime_api.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int csrk_status;
#define CSRK_OK            0
#define CSRK_INVALID_ARG   1   /* negative size, null pointer where one is required, bad alignment */
#define CSRK_UNSUPPORTED   2   /* a size beyond what the kernels' 32-bit indexing covers */
#define CSRK_HIP_ERROR     3   /* a HIP runtime call failed; message has the HIP error string */
#define CSRK_WORKSPACE     4   /* the scratch area could not be allocated */

/*
 * SPMM, paper eq. (2) / Algorithm 2:
 *   O[i, :] = sum over stored entries j of row i of  vals[j] * B[colidx[j], :]
 * S is M x K (rowptr/colidx/vals), B is K x N, O is M x N (overwritten).
 * vals == NULL means every stored entry is 1 (the paper's all-ones matrix I_A).
 */
csrk_status spmm_csr(int M, int K, int N,
                     const int32_t *rowptr, const int32_t *colidx, const float *vals,
                     const float *B, float *O, hipStream_t stream);

/*
 * SDDMM, paper eq. (1) / Algorithm 1, with the sampled product scaled by S's
 * stored values:
 *   P[j] = vals[j] * <A[i, :], B[colidx[j], :]>   for every stored entry j of row i
 * A is M x D, B is K x D (used as B^T), P has nnz entries in the order of
 * colidx.  vals == NULL means an all-ones pattern, which is the paper's I_A.
 * P may alias vals (P == vals: the values are overwritten in place, as in the
 * paper's Algorithm 1); such a call keeps to the kernels that need no second
 * pass over vals - the LDS-tiled kernel only through sddmm_csr_plan, whose plan
 * vouches for the column order.  Partly overlapping P and vals are not allowed.
 */
csrk_status sddmm_csr(int M, int K, int D,
                      const int32_t *rowptr, const int32_t *colidx, const float *vals,
                      const float *A, const float *B, float *P, hipStream_t stream);

/*
 * FusedMM, paper eq. (3) / Algorithm 3: SDDMM followed by SPMM with the sampled
 * scores kept on chip (never written to device memory):
 *   O[i, :] = sum_j ( vals[j] * <A[i, :], B[colidx[j], :]> ) * C[colidx[j], :]
 * A is M x D, B is K x D, C is K x N, O is M x N (overwritten).  The paper has
 * D == N; here the dot length D and the output width N are independent.
 * vals == NULL means an all-ones pattern.
 */
csrk_status fusedmm_csr(int M, int K, int D, int N,
                        const int32_t *rowptr, const int32_t *colidx, const float *vals,
                        const float *A, const float *B, const float *C,
                        float *O, hipStream_t stream);

/*
 * fusedmm_csr for callers that cannot allocate: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and results as fusedmm_csr; the kernels' scratch is a fixed
 * area inside the library's device image (16 MB + 64 KB, held by every device the library runs on until the
 * process ends), so the call allocates and frees nothing, never synchronises and takes no lock beyond the one
 * that guards looking up the area's address the first time a device is used.  It serves outputs of up to 512
 * columns (8192 partial rows of N floats), and short matrices whose reduction dimension is cut into ranges only
 * while their partial outputs fit 16 MB; beyond that it returns CSRK_WORKSPACE with the sizes in the message and
 * enqueues nothing (fusedmm_csr_ws takes any size).  All calls on one device share the one area, which keeps
 * whatever the last call left in it (every call initialises what it reads): calls that overlap in time on one
 * device, on whatever streams, race - serialise them on one stream.
 */
csrk_status fusedmm_csr_static(int M, int K, int D, int N,
                               const int32_t *rowptr, const int32_t *colidx, const float *vals,
                               const float *A, const float *B, const float *C,
                               float *O, hipStream_t stream);

/*
 * The same three operations with the DENSE operands stored as bfloat16 (the upper 16
 * bits of an IEEE single, row-major like their FP32 counterparts): the variant the
 * paper names as future work (section "Conclusion").  The stored values of S, all
 * arithmetic and the outputs stay FP32: every bfloat16 is widened exactly, products
 * and sums are FP32 as in the calls above, so the result is what those calls give
 * on the widened operands.  Same argument rules; B / A, B / A, B, C are device
 * pointers to uint16_t.  These calls run the general kernels (half the bytes to
 * gather); there are no LDS-tiled bfloat16 kernels.
 */
csrk_status spmm_csr_bf16(int M, int K, int N,
                          const int32_t *rowptr, const int32_t *colidx, const float *vals,
                          const uint16_t *B, float *O, hipStream_t stream);
csrk_status sddmm_csr_bf16(int M, int K, int D,
                           const int32_t *rowptr, const int32_t *colidx, const float *vals,
                           const uint16_t *A, const uint16_t *B, float *P, hipStream_t stream);
csrk_status fusedmm_csr_bf16(int M, int K, int D, int N,
                             const int32_t *rowptr, const int32_t *colidx, const float *vals,
                             const uint16_t *A, const uint16_t *B, const uint16_t *C,
                             float *O, hipStream_t stream);

/*
 * The three operations on a workspace of the caller's (paper section "Overview of the
 * Algorithms": the same row algorithms; only where the kernels' scratch lives differs).
 *
 * csrk_workspace_bytes: host-only; *bytes receives the size that any call of the given
 * operation (CSRK_OP_*) and shape may need on the current device, whichever kernels it
 * takes (N is the output width, ignored for SDDMM; D is accepted for symmetry and does
 * not matter).  `workspace` is a DEVICE pointer to at least that many bytes, aligned to
 * 256 bytes (what hipMalloc returns), owned by the caller; its contents on entry do not
 * matter and are unspecified afterwards.  A call whose workspace is too small returns
 * CSRK_WORKSPACE, and the message names the size it needs; nothing has been enqueued then.
 * The call neither allocates nor frees nor synchronises, so it may be made while
 * `stream` is being captured into a HIP graph.  The workspace is in use until `stream`
 * has passed the enqueued work: two calls in flight at once need two workspaces.
 * All other arguments and the results are those of spmm_csr / sddmm_csr / fusedmm_csr.
 */
#define CSRK_OP_SPMM     1
#define CSRK_OP_SDDMM    2
#define CSRK_OP_FUSEDMM  3
csrk_status csrk_workspace_bytes(int op, int M, int K, int N, int D, size_t *bytes);
csrk_status spmm_csr_ws(int M, int K, int N,
                        const int32_t *rowptr, const int32_t *colidx, const float *vals,
                        const float *B, float *O,
                        void *workspace, size_t workspace_bytes, hipStream_t stream);
csrk_status sddmm_csr_ws(int M, int K, int D,
                         const int32_t *rowptr, const int32_t *colidx, const float *vals,
                         const float *A, const float *B, float *P,
                         void *workspace, size_t workspace_bytes, hipStream_t stream);
csrk_status fusedmm_csr_ws(int M, int K, int D, int N,
                           const int32_t *rowptr, const int32_t *colidx, const float *vals,
                           const float *A, const float *B, const float *C, float *O,
                           void *workspace, size_t workspace_bytes, hipStream_t stream);

/*
 * Which kernel family a call would take (the paper chooses NT and nchunks from the
 * shape, sections "SDDMM" and "SPMM"; here the choice is between kernel families).
 * Host-only: no device is touched, the number of compute units `cus` is given.  The
 * pattern is described by its number of stored entries and its longest row; columns
 * are taken to ascend strictly in every row, operands to be 16-byte aligned and
 * outputs not to alias inputs.  planned != 0: the choice of the *_plan calls.
 * *family (host pointer) receives one of CSRK_FAMILY_*.  Used by the regression test
 * that replays the choice against a recorded sweep of forced families.
 */
#define CSRK_FAMILY_GENERAL_SHARES 0  /* equal shares of the stored entries */
#define CSRK_FAMILY_GENERAL_ROWS   1  /* the same kernels dealing out whole rows (rows found even) */
#define CSRK_FAMILY_ROWS           2  /* whole-row kernels chosen by the host (small S) */
#define CSRK_FAMILY_TILED_NARROW   3  /* LDS-tiled, outputs of up to 128 columns (per launch) */
#define CSRK_FAMILY_TILED_WIDE     4  /* LDS-tiled, wider outputs */
#define CSRK_FAMILY_TILED_SDDMM    5  /* LDS-tiled SDDMM */
#define CSRK_FAMILY_SCHEDULE       6  /* a plan's schedule for uneven rows */
csrk_status csrk_explain_choice(int op, int cus, int M, int K, int N, int D, long long nnz,
                                int longest_row, int planned, int *family);

/*
 * Plans: the sparsity pattern analysed once, for callers that use one pattern many
 * times (training loops; the paper's row analysis - nnzr, NT, nchunks of sections
 * "SDDMM" and "SPMM" - depends on the pattern alone).  The calls above look at the
 * pattern on the device on every call: a row analysis (density, longest row) ahead
 * of or inside an LDS-tiled kernel, a column-order check inside it, and the general
 * kernel plus combine step launched behind it in case the device turns the tiled
 * kernel down.  A plan answers those questions once, on the host, so that a planned
 * call launches only the kernel that does the work (plus the combine step where the
 * method needs one).  Results are those of the unplanned calls.
 *
 * csrk_plan_create checks the structure like csrk_validate_csr (a pattern with
 * problems is refused with CSRK_INVALID_ARG), finds out whether every row's columns
 * are strictly ascending and whether the rows are even in length, and SYNCHRONISES
 * `stream`.  rowptr and colidx (device pointers, not copied) must stay alive and
 * UNCHANGED for as long as the plan is used; a planned call on a pattern changed
 * since has undefined results.  *out (host pointer) receives the plan, owned by the
 * caller until csrk_plan_destroy (NULL is accepted there).  A plan belongs to the
 * device that was current when it was made; it holds 32 bytes of device memory (plus the
 * workspace that csrk_plan_reserve may add, and the schedule described next).
 * Uneven rows (ordered columns, longest row > 2 * mean + 64; at least 256 rows and
 * K >= 1024): the plan also holds a SCHEDULE for the LDS-tiled kernels - rowptr is
 * read back to the host, the rows are sorted by length into blocks of 64 and every
 * block's K is cut into as many ranges as its share of the work asks for (the
 * paper's NT work-items per row, section "SDDMM", chosen per block of rows); about
 * 4 * M + 32 * (M / 64 + CUs) bytes of device memory.  Planned SPMM and FusedMM
 * (D <= 64) calls with outputs of 132 to 512 columns then run the tiled kernels over
 * that table instead of dealing the stored entries out in equal shares; partial
 * rows of cut blocks go through the scratch area and are added up in range order
 * (same bits every run).
 * csrk_plan_info reports what was found (any of the three host pointers may be
 * NULL).  The planned calls take the pattern and M, K from the plan; all other
 * arguments are as in spmm_csr / sddmm_csr / fusedmm_csr.
 */
typedef struct csrk_plan_s csrk_plan;
csrk_status csrk_plan_create(int M, int K, const int32_t *rowptr, const int32_t *colidx,
                             hipStream_t stream, csrk_plan **out);
/*
 * Gives the plan a workspace of its own, large enough for spmm_csr_plan and fusedmm_csr_plan
 * with outputs of up to max_N columns (and for sddmm_csr_plan): allocates it here
 * (hipMalloc; if the plan already had a smaller one, the device is synchronised and that one
 * freed), freed by csrk_plan_destroy.  Planned calls that fit into it use it instead of the
 * library's per-device area and then allocate nothing, never synchronise, take no lock and
 * may be captured in a HIP graph; calls that do not fit fall back to the per-device area.
 * Two calls on the same plan in flight at once on different streams would race on it.
 */
csrk_status csrk_plan_reserve(csrk_plan *plan, int max_N);
csrk_status csrk_plan_destroy(csrk_plan *plan);
csrk_status csrk_plan_info(const csrk_plan *plan, long long *nnz, int *sorted, int *even);
csrk_status spmm_csr_plan(const csrk_plan *plan, int N, const float *vals,
                          const float *B, float *O, hipStream_t stream);
csrk_status sddmm_csr_plan(const csrk_plan *plan, int D, const float *vals,
                           const float *A, const float *B, float *P, hipStream_t stream);
csrk_status fusedmm_csr_plan(const csrk_plan *plan, int D, int N, const float *vals,
                             const float *A, const float *B, const float *C,
                             float *O, hipStream_t stream);

/*
 * Debug helper for untrusted inputs (the paper's storage rules, Fig. 1): checks
 * on the device that rowptr[0] == 0, rowptr is non-decreasing and every colidx
 * is in [0, K).  Synchronises `stream`.  *problems receives a bit mask:
 * 1 rowptr[0] != 0, 2 rowptr decreases somewhere, 4 a column index is out of
 * range; *sorted receives 1 if the columns of every row are strictly ascending
 * (only meaningful when *problems == 0).  Either pointer may be NULL (host pointers).
 */
csrk_status csrk_validate_csr(int M, int K, const int32_t *rowptr, const int32_t *colidx,
                              hipStream_t stream, int *problems, int *sorted);

/*
 * Benchmark aid (not part of the paper's method; it mirrors the paper's practice of
 * timing each kernel on its own, section "Experiments").  csrk_profile_enable(n)
 * with n > 0 creates n pairs of HIP events; from then on every spmm_csr / sddmm_csr /
 * fusedmm_csr call (planned or not) records one pair on the call's stream around ALL kernel launches of
 * the call (the row analysis, the LDS-tiled kernel when one is tried, the general kernel
 * behind it - exactly one of the two does the work, the other returns at once - and the
 * combine pass of partial rows), until the pairs are used up.  csrk_profile_enable(0)
 * destroys the events and switches recording off.
 * csrk_profile_collect waits for the recorded pairs, writes up to `capacity`
 * elapsed times in milliseconds to ms[] and the operation of each to kinds[]
 * (1 SPMM, 2 SDDMM, 3 FusedMM; 11, 12, 13 for the bfloat16 variants) in call order, stores the number written in *count
 * and resets the recorder.  ms, kinds and count are host pointers.
 */
csrk_status csrk_profile_enable(int max_records);
csrk_status csrk_profile_collect(float *ms, int *kinds, int capacity, int *count);

/*
 * Measuring aids (not part of the paper's method; they serve its section "Performance Analysis": where the time of a
 * kernel goes).
 *
 * csrk_tile_phases runs a MEASURING BUILD of the 512-column LDS-tiled SPMM (op = CSRK_OP_SPMM: O = S.C, A and B
 * ignored) or FusedMM (CSRK_OP_FUSEDMM, D = 64) kernel once - the same code with a cycle counter read at every change
 * of phase - and returns, in cycles[0..7] (host array of 8 doubles), the mean number of shader-clock cycles a wavefront
 * spent in each phase over the whole call: [0] waiting at the barrier that ends a tile, [1] copying the next tile from
 * registers to LDS, [2] waiting at the barrier behind that copy, [3] issuing the loads of a tile, [4] the accumulate
 * stage (LDS reads and multiply-adds), [5] issuing the loads of the rows' next entries, [6] FusedMM's score stage,
 * [7] unused; *tiles receives the number of tiles per wavefront.  Needs N = 512, M a multiple of 64, ascending
 * columns; O is overwritten with the result.  Allocates and frees scratch of its own and SYNCHRONISES `stream`.  The
 * counter reads perturb what they measure by a few per cent.
 *
 * csrk_debug_row_rotation writes, for S = 0 .. 15 and every lane l of one wavefront, into out[S * 64 + l] (device,
 * 1024 floats) the number of the lane whose operand the row rotation by S of the kernels' rotated multiply-add hands
 * to lane l: the tiled SDDMM and FusedMM kernels are written for (l & ~15) | ((l - S) & 15).
 */
csrk_status csrk_tile_phases(int op, int M, int K, int D, int N,
                             const int32_t *rowptr, const int32_t *colidx, const float *vals,
                             const float *A, const float *B, const float *C, float *O,
                             hipStream_t stream, double *cycles, int *tiles);
csrk_status csrk_debug_row_rotation(float *out, hipStream_t stream);

/*
 * The machine rates the kernels are quoted against, measured on the current device by three small kernels of the
 * library's own (the paper's roofline, section "Performance Analysis", likewise takes its ceilings from what the
 * profiler measures on the device): *value receives
 *   CSRK_BENCH_HBM_COPY  GB/s of a 1 GiB device-to-device copy, bytes read plus bytes written;
 *   CSRK_BENCH_FMA_F32   TFLOP/s of a loop of independent plain FP32 multiply-adds (no packed FP32), 2 flops each;
 *   CSRK_BENCH_LDS_READ  TB/s of conflict-free 128-bit LDS reads in the tiled kernels' launch shape (one workgroup
 *                        of 16 wavefronts per CU, 2 KB rows of a 128 KB tile).
 * Best of five runs each.  Allocates and frees its buffers, synchronises the device, uses the default stream.
 * Returns a status only (no message is left for csrk_last_error).
 */
#define CSRK_BENCH_HBM_COPY  1
#define CSRK_BENCH_FMA_F32   2
#define CSRK_BENCH_LDS_READ  3
csrk_status csrk_microbench(int kind, double *value);

/* Frees the current device's scratch area of the plain entry points (synchronises the device). */
csrk_status csrk_release_workspace(void);

/* Message of the last error on the calling thread ("" if none). Host string owned by the library. */
const char *csrk_last_error(void);

/* Library version string, e.g. "csrk 0.1 gfx950". */
const char *csrk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CSRK_H */
