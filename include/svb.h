/*
 * svb -- singular values of a dense real matrix on one AMD MI355X (gfx950) by
 * the two-stage QR-based reduction of the paper (Section 3): dense -> band by
 * tiled Householder QR/LQ sweeps (Section 3.1, Algorithms 1 and 2), band ->
 * bidiagonal by bulge chasing (Section 3, second stage), bidiagonal ->
 * singular values by Sturm counts (Section 3, final stage; on the device by
 * default, on the host as in the paper on request).
 *
 * Plain C ABI: raw pointers and sizes only.  Every pointer is tagged [dev]
 * (device memory, accessible from the current HIP device) or [host].
 *
 * Conventions common to all entry points
 *   - Matrices are column-major: element (i,j) of A is A[i + j*lda], lda >= m.
 *     All index arithmetic is 64-bit.
 *   - The caller owns every buffer.  The library allocates no device memory;
 *     scratch space comes in through work_dev / work_bytes (size from
 *     svb_workspace_bytes), except for svb_gb2bd_noalloc, whose scratch is a
 *     fixed array inside the library's device image.
 *   - GPU work is ordered after what the HIP stream passed as `stream` (a
 *     hipStream_t cast to void*, NULL = the default stream) holds at the call,
 *     and that stream waits for it: stage 1 runs on two internal streams that
 *     are forked from and joined back to `stream` with events (the first
 *     level of every panel tree and the updates on one, the tree's upper
 *     levels beside them on the other), the rest on `stream`.
 *   - Return value: an svb_status.  On SVB_ERR_ARG / SVB_ERR_UNSUPPORTED /
 *     SVB_ERR_WORKSPACE nothing has been read or written.
 *   - dtype: SVB_F64, SVB_F32, and the storage-only types SVB_F16 / SVB_BF16
 *     (every sum is formed in f32, as the paper does for half precision,
 *     Section 4.3; the trailing update multiplies on the 16-bit matrix
 *     instructions with its f32 operands split into 16-bit terms, which keeps
 *     f32 accuracy; the band, the bidiagonal and the result are f32).
 *   - nb (the paper's TILESIZE): 32, 64 or 128; 0 lets the library choose
 *     (svb_choose_nb).
 *   - Magnitudes: entries may be anywhere in the finite range of the storage
 *     type.  svb_svdvals multiplies the matrix by a power of two first when its
 *     largest magnitude lies outside [2^-40, 2^40] (f32 arithmetic) or
 *     [2^-400, 2^400] (f64), because the kernels form sums of squares without
 *     scaling them, and multiplies the bidiagonal back.  An SVB_F16 matrix is
 *     scaled so that max|a| sqrt(m n) is about 2^11: the transformed matrix is
 *     written back in f16, where an entry can reach a column's norm.  The stage-split entry
 *     points svb_ge2gb / svb_gb2bd do not rescale: their inputs must keep
 *     sums of squares of n entries inside the arithmetic type's range (and an
 *     SVB_F16 matrix its Frobenius norm below 2^13).
 *     A NaN or an infinity in the input gives SVB_ERR_NONFINITE.
 *   - Calls that share a workspace, a matrix or a stream must not overlap, and
 *     calls into the library from different host threads must not overlap at
 *     all (the internal streams and events are per process).
 */
#ifndef SVB_H
#define SVB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SVB_F64 = 0, SVB_F32 = 1, SVB_F16 = 2, SVB_BF16 = 3 } svb_dtype;

typedef enum {
    SVB_OK = 0,
    SVB_ERR_ARG = 1,         /* null pointer, negative size, lda < m, ... */
    SVB_ERR_UNSUPPORTED = 2, /* nb / dtype outside the supported set, misaligned buffer */
    SVB_ERR_WORKSPACE = 3,   /* work_bytes smaller than svb_workspace_bytes says */
    SVB_ERR_DEVICE = 4,      /* a HIP call or a kernel-side consistency check failed */
    SVB_ERR_NOCONV = 5,      /* the bidiagonal solver did not converge */
    SVB_ERR_NONFINITE = 6    /* the input or the bidiagonal holds a NaN or an infinity */
} svb_status;

/*
 * Scratch requirements of svb_svdvals / svb_ge2gb for one problem (any m, n
 * >= 0; nb = 0 sizes for the tile size svb_choose_nb returns).
 * [host] dev_bytes, host_bytes: outputs (either may be NULL).  host_bytes is
 * always 0 (host scratch is allocated internally).  A matrix that is not a
 * whole number of tiles in both directions, or has m < n, is copied into the
 * workspace, which then includes room for the zero-padded copy.
 */
int svb_workspace_bytes(svb_dtype dt, int64_t m, int64_t n, int nb,
                        size_t* dev_bytes, size_t* host_bytes);

/*
 * The tile size that nb = 0 selects for an m x n matrix of type dt (the paper
 * tunes TILESIZE per matrix size and device, Section 4, Table 3), from timings
 * on MI355X, k = min(m, n): f32 arithmetic (SVB_F32, SVB_F16, SVB_BF16): 32 for
 * k < 1024, 64 up to 26624, 128 beyond; SVB_F64: 32 up to 2560, 64 beyond.
 * Returns 0 for invalid arguments.
 */
int svb_choose_nb(svb_dtype dt, int64_t m, int64_t n);

/*
 * All singular values of the m x n matrix A (Section 3, equation (1): the
 * diagonal of Sigma in A = U Sigma V^T), through stage 1, stage 2 and the
 * bidiagonal solve.  Any m, n >= 1.  The paper treats square matrices of whole
 * tiles (Algorithm 2) and names other shapes as future work (Section 5); here
 *   - m > n adds tile rows to the QR sweeps (the LQ sweeps stop at column n);
 *   - m < n is the transposed problem (same singular values);
 *   - a dimension that is not a multiple of nb is padded with zeros, which
 *     leaves the min(m, n) singular values unchanged and adds none to the
 *     output;
 *   the last two, and the first if m is not a multiple of nb, work on a copy
 *   of A inside the workspace.
 *   A_dev      [dev]  in/out: the matrix in storage type dt.  If m >= n and
 *                     both are multiples of nb it is DESTROYED (used as the
 *                     in-place work area of stage 1, like the paper's
 *                     banddiag!, Algorithm 2) and must be 16-byte aligned with
 *                     lda a multiple of 4 elements (2 for SVB_F64), else
 *                     SVB_ERR_UNSUPPORTED; otherwise it is only read and has
 *                     no alignment requirement.
 *   S_out_host [host] out: min(m,n) values, descending; double for SVB_F64,
 *                     float otherwise.
 *   nb                tile size of stage 1 = bandwidth handed to stage 2, or 0.
 *   work_dev   [dev]  scratch of at least svb_workspace_bytes(...) bytes,
 *                     256-byte aligned.
 * Blocking: returns after the result has been copied to S_out_host (one
 * stream synchronisation).  With the environment variable SVB_STAGE3=host the
 * bidiagonal is solved on the host (svb_bdsvals) instead of the device.
 */
int svb_svdvals(svb_dtype dt, int64_t m, int64_t n, void* A_dev, int64_t lda,
                void* S_out_host, int nb, void* work_dev, size_t work_bytes,
                void* stream);

/*
 * Stage 1 (Section 3.1, Algorithm 1, Figure 1): reduce A to an upper band
 * matrix with nb super-diagonals by alternating QR sweeps (diagonal tile made
 * upper triangular, tiles below annihilated) and LQ sweeps (tile right of the
 * diagonal made lower triangular, tiles to its right annihilated).  In place:
 * m >= n >= 1, both multiples of nb (nb in {32, 64, 128}, not 0), A_dev
 * 16-byte aligned, lda a multiple of 4 elements (2 for SVB_F64); anything
 * else returns SVB_ERR_UNSUPPORTED.
 *   band_dev [dev] out: packed band in the COMPUTE type (double for SVB_F64,
 *            float otherwise), ldab >= 3*nb rows by n columns: entry (i,j) of
 *            the n x n band matrix, -(2nb-1) <= i-j <= nb-1, lives at
 *            band[(i - j + 2*nb - 1) + j*ldab].  Entries outside the nb
 *            super-diagonals are written as zeros (room for stage 2's bulges).
 * Asynchronous: returns after enqueueing; A_dev is destroyed.
 */
int svb_ge2gb(svb_dtype dt, int64_t m, int64_t n, void* A_dev, int64_t lda, int nb,
              void* band_dev, int64_t ldab, void* work_dev, size_t work_bytes,
              void* stream);

/*
 * Stage 2 (Section 3, the second stage): reduce the packed upper band (layout
 * of svb_ge2gb, nb super-diagonals, nb in {8, 32, 64, 128}; band_dt = SVB_F64
 * or SVB_F32 is the type of the band entries; any n >= 0) to upper bidiagonal
 * form by bulge chasing.
 *   band_dev [dev] in/out: destroyed.
 *   d_dev    [dev] out: n diagonal entries, same type as the band.
 *   e_dev    [dev] out: n-1 super-diagonal entries (n slots are written).
 *   work_dev [dev] scratch of svb_gb2bd_workspace_bytes(n, nb) bytes (sweep
 *            tickets, error flags, one progress counter per sweep).
 * Asynchronous.  The sweeps are pipelined with bounded waits; should a wait
 * expire (it cannot unless the device is oversubscribed or faulty) d[0] is
 * set to NaN, which svb_bdsvals / svb_svdvals report as SVB_ERR_NONFINITE.
 */
int svb_gb2bd(svb_dtype band_dt, int64_t n, int nb, void* band_dev, int64_t ldab,
              void* d_dev, void* e_dev, void* work_dev, size_t work_bytes,
              void* stream);

/* Bytes of device scratch svb_gb2bd needs ([host] out). */
int svb_gb2bd_workspace_bytes(int64_t n, int nb, size_t* dev_bytes);

/*
 * svb_gb2bd for callers that can neither allocate device memory nor carry a
 * workspace (code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation): same arguments without work_dev / work_bytes, same
 * results.  The sweep counters live in a fixed 1 MiB array inside the
 * library's device image (one copy per device, held until the process ends),
 * which limits n to SVB_NOALLOC_MAX_N; larger n returns SVB_ERR_WORKSPACE.
 * Calls no allocating routine.  The counters a call uses are cleared by its
 * own kernels, so consecutive calls on one stream are independent; every call
 * on a device shares that device's array, so calls that overlap on one device
 * (different streams or threads) race and must be serialised by the caller.
 */
#define SVB_NOALLOC_MAX_N 131072
int svb_gb2bd_noalloc(svb_dtype band_dt, int64_t n, int nb, void* band_dev, int64_t ldab,
                      void* d_dev, void* e_dev, void* stream);

/*
 * Stage 3 (Section 3, final stage; the paper calls LAPACK on the CPU here):
 * singular values of the n x n upper bidiagonal (d, e), descending.
 * Host only, fp64, multi-threaded.
 *   d [host] n entries; e [host] n-1 entries; sigma [host] out, n entries.
 */
int svb_bdsvals(int64_t n, const double* d, const double* e, double* sigma);

/*
 * Stage 3 on the device (what svb_svdvals runs unless SVB_STAGE3=host): Sturm
 * counts by the differential stationary qd recurrence, each interval refined
 * by multisection (several lanes per singular value, one point of the
 * interval each).
 *   band_dt   SVB_F64 or SVB_F32: type of d, e and sigma.
 *   d_dev, e_dev [dev] in: n and n-1 entries (layout of svb_gb2bd's outputs).
 *   sigma_dev [dev] out: n values, descending.  Non-finite input gives NaNs.
 *   rel_tol   refinement stops at interval width rel_tol * sigma (0 = 2^-52 for
 *             SVB_F64 and 2^-29 for SVB_F32).
 *   work_dev  [dev] scratch of svb_bdsvals_dev_workspace_bytes(n) bytes.
 * Asynchronous.
 */
int svb_bdsvals_dev_workspace_bytes(int64_t n, size_t* dev_bytes);
int svb_bdsvals_dev(svb_dtype band_dt, int64_t n, const void* d_dev, const void* e_dev, void* sigma_dev,
                    double rel_tol, void* work_dev, size_t work_bytes, void* stream);

/*
 * Wall-clock seconds of the most recent svb_svdvals call of this process, in
 * the paper's four-way split (Figure 6): panel factorisation, trailing update,
 * band -> bidiagonal, bidiagonal -> values.  From HIP events on the caller's
 * stream (a host stage 3 from the host clock).  Panels and updates overlap on
 * two streams, so stage 1's wall time is split into the part covered by update
 * kernels (t_update) and the rest (t_panel: panel time that no update hides);
 * that split needs the per-kernel events of svb_profile_enable.  Without them
 * t_update holds the whole of stage 1 and t_panel is -1.  Staging and scaling
 * of the input count towards stage 1.  Any pointer may be NULL.
 */
int svb_last_timings(double* t_panel, double* t_update, double* t_stage2, double* t_stage3);

/*
 * Per-kernel timing for measurement.  When enabled, svb_ge2gb / svb_gb2bd /
 * svb_svdvals take the start and stop time stamps of every launch of the
 * kernel classes below with HIP events on the stream the kernel runs on and
 * svb_svdvals (or svb_profile_collect, after the caller synchronised the
 * stream) sums the elapsed times.  Off by default.
 *   kind: SVB_PROF_PANEL (domain QR of every tree level), SVB_PROF_UPDATE (the
 *   one-pass trailing update, first tree level: the launches whose flops are
 *   credited), SVB_PROF_UPDATE_UPPER (the same kernel on the tree levels above),
 *   SVB_PROF_BAND_REDUCE (stage 2, band -> 8 super-diagonals), SVB_PROF_NARROW
 *   (stage 2, 8 super-diagonals -> bidiagonal), SVB_PROF_STAGE3.
 *   seconds / launches / flops / bytes [host] out, any may be NULL: totals
 *   since the last svb_profile_enable(1); flops and bytes are the algorithmic
 *   counts of the launches (update: 2*rows*nb*cols per product, block read once
 *   and written once; band reduction: every nb x nb block read once and written
 *   once per block sweep; narrow chase: the band's 24 stored rows read once and
 *   written once per bundle of sweeps), not hardware counters.
 */
enum { SVB_PROF_PANEL = 0, SVB_PROF_UPDATE = 1, SVB_PROF_UPDATE_UPPER = 2, SVB_PROF_BAND_REDUCE = 3,
       SVB_PROF_NARROW = 4, SVB_PROF_STAGE3 = 5, SVB_PROF_KINDS = 6 };
int svb_profile_enable(int on);
int svb_profile_collect(void);
int svb_profile_get(int kind, double* seconds, int64_t* launches, double* flops, double* bytes);

/* Static, human-readable text for a status code. */
const char* svb_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SVB_H */
