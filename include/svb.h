/*
 * svb — singular values of a dense real matrix on one AMD MI355X (gfx950) by
 * the two-stage QR-based reduction of the paper (Section 3): dense -> band by
 * tiled Householder QR/LQ sweeps (Section 3.1, Algorithms 1 and 2), band ->
 * bidiagonal by bulge chasing (Section 3, second stage), bidiagonal ->
 * singular values on the host (Section 3, final stage).
 *
 * Plain C ABI: raw pointers and sizes only.  Every pointer is tagged [dev]
 * (device memory, accessible from the current HIP device) or [host].
 *
 * Conventions common to all entry points
 *   - Matrices are column-major: element (i,j) of A is A[i + j*lda], lda >= m.
 *     All index arithmetic is 64-bit.
 *   - The caller owns every buffer.  The library allocates no device memory;
 *     scratch space comes in through work_dev / work_bytes
 *     (size from svb_workspace_bytes).
 *   - GPU work is ordered after what the HIP stream passed as `stream` (a
 *     hipStream_t cast to void*, NULL = the default stream) holds at the call,
 *     and that stream waits for it: stage 1 runs on two internal streams that
 *     are forked from and joined back to `stream` with events (the panel tree
 *     on one, the updates it overlaps on the other), the rest on `stream`.
 *   - Return value: an svb_status.  On SVB_ERR_ARG / SVB_ERR_UNSUPPORTED /
 *     SVB_ERR_WORKSPACE nothing has been read or written.
 *   - Supported in this version: m == n, n a positive multiple of nb,
 *     nb in {32, 64, 128}, dtype f64 / f32 / f16 (f16 is storage only: every
 *     product and sum is formed in f32, as the paper does for half precision,
 *     Section 4.3).  Anything else returns SVB_ERR_UNSUPPORTED.
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
    SVB_ERR_UNSUPPORTED = 2, /* shape / nb / dtype outside the supported set */
    SVB_ERR_WORKSPACE = 3,   /* work_bytes smaller than svb_workspace_bytes says */
    SVB_ERR_DEVICE = 4,      /* a HIP call or a kernel-side consistency check failed */
    SVB_ERR_NOCONV = 5,      /* the bidiagonal solver did not converge */
    SVB_ERR_NONFINITE = 6    /* the bidiagonal holds a NaN or an infinity */
} svb_status;

/*
 * Scratch requirements of svb_svdvals / svb_ge2gb / svb_gb2bd for one problem.
 * [host] dev_bytes, host_bytes: outputs (either may be NULL).  host_bytes is
 * always 0 in this version (host scratch is allocated internally).
 */
int svb_workspace_bytes(svb_dtype dt, int64_t m, int64_t n, int nb,
                        size_t* dev_bytes, size_t* host_bytes);

/*
 * All singular values of the m x n matrix A (Section 3, equation (1): the
 * diagonal of Sigma in A = U Sigma V^T), through stage 1, stage 2 and the
 * host bidiagonal solve.
 *   A_dev      [dev]  in/out: the matrix in storage type dt; DESTROYED (used as
 *                     the in-place work area of stage 1, like the paper's
 *                     banddiag!, Algorithm 2).
 *   S_out_host [host] out: min(m,n) values, descending; double for SVB_F64,
 *                     float for SVB_F32 and SVB_F16.
 *   nb                tile size of stage 1 = bandwidth handed to stage 2
 *                     (the paper's TILESIZE).
 *   work_dev   [dev]  scratch of at least svb_workspace_bytes(...) bytes,
 *                     256-byte aligned.
 * Blocking: the stream is synchronised once before the host solve; on return
 * S_out_host is valid.
 */
int svb_svdvals(svb_dtype dt, int64_t m, int64_t n, void* A_dev, int64_t lda,
                void* S_out_host, int nb, void* work_dev, size_t work_bytes,
                void* stream);

/*
 * Stage 1 (Section 3.1, Algorithm 1, Figure 1): reduce A to an upper band
 * matrix with nb super-diagonals by alternating QR sweeps (diagonal tile made
 * upper triangular, tiles below annihilated) and LQ sweeps (tile right of the
 * diagonal made lower triangular, tiles to its right annihilated).
 *   band_dev [dev] out: packed band in the COMPUTE type (double for SVB_F64,
 *            float for SVB_F32 / SVB_F16), ldab >= 3*nb rows by n columns:
 *            entry (i,j) of the band matrix, -(2nb-1) <= i-j <= nb-1, lives at
 *            band[(i - j + 2*nb - 1) + j*ldab].  Entries outside the nb
 *            super-diagonals are written as zeros (room for stage 2's bulges).
 * Asynchronous: returns after enqueueing; A_dev is destroyed.
 */
int svb_ge2gb(svb_dtype dt, int64_t m, int64_t n, void* A_dev, int64_t lda, int nb,
              void* band_dev, int64_t ldab, void* work_dev, size_t work_bytes,
              void* stream);

/*
 * Stage 2 (Section 3, "second, memory-bound stage"): reduce the packed upper
 * band (layout of svb_ge2gb, nb super-diagonals, band_dt = SVB_F64 or SVB_F32
 * is the type of the band entries) to upper bidiagonal form by bulge chasing.
 *   band_dev [dev] in/out: destroyed.
 *   d_dev    [dev] out: n diagonal entries, same type as the band.
 *   e_dev    [dev] out: n-1 super-diagonal entries (n slots are written).
 *   work_dev [dev] scratch of svb_gb2bd_workspace_bytes(n, nb) bytes (sweep
 *            ticket, error flag, one progress counter per sweep).
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
 * Stage 3 (Section 3, final stage; the paper calls LAPACK on the CPU here):
 * singular values of the n x n upper bidiagonal (d, e), descending.
 * Host only, fp64, multi-threaded.
 *   d [host] n entries; e [host] n-1 entries; sigma [host] out, n entries.
 */
int svb_bdsvals(int64_t n, const double* d, const double* e, double* sigma);

/*
 * Stage 3 on the device: the Sturm counts of svb_bdsvals, each interval refined
 * by multisection (several lanes per singular value, one point of the interval
 * each), for callers that keep the bidiagonal in device memory
 * (svb_svdvals uses it unless the environment variable SVB_STAGE3=host is set).
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
 * Wall-clock seconds of the stages of the most recent svb_svdvals call of
 * this process (stages 1 and 2, and stage 3 when it runs on the device, from
 * HIP events on the caller's stream; a host stage 3 from the host clock).  Any
 * pointer may be NULL.
 */
int svb_last_timings(double* t_stage1, double* t_stage2, double* t_stage3);

/*
 * Per-kernel timing for measurement (the paper's Figure 6 reports the same
 * split: panel factorisation, trailing update, band -> bidiagonal).  When
 * enabled, svb_ge2gb / svb_gb2bd / svb_svdvals bracket every launch of the
 * kernel classes below with HIP events on the stream the kernel runs on and
 * svb_svdvals (or svb_profile_collect, after the caller synchronised the
 * stream) sums the elapsed times.  Off by default; costs two event records
 * per launch when on.
 *   kind: SVB_PROF_PANEL (gather + domain QR + R scatter), SVB_PROF_K1
 *   (W = Y^T C), SVB_PROF_K2 (C -= V W), SVB_PROF_FUSED (both products in one
 *   pass over the trailing matrix, the default), SVB_PROF_CHASE (stage 2).
 *   seconds / launches / flops / bytes [host] out, any may be NULL: totals
 *   since the last svb_profile_enable(1); flops and bytes are the algorithmic
 *   counts of the launches (2*rows*nb*cols per product; 3*n^2*nb*size for the
 *   chase), not hardware counters.
 */
enum { SVB_PROF_PANEL = 0, SVB_PROF_K1 = 1, SVB_PROF_K2 = 2, SVB_PROF_CHASE = 3, SVB_PROF_FUSED = 4,
       SVB_PROF_KINDS = 5 };
int svb_profile_enable(int on);
int svb_profile_collect(void);
int svb_profile_get(int kind, double* seconds, int64_t* launches, double* flops, double* bytes);

/* Static, human-readable text for a status code. */
const char* svb_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SVB_H */
