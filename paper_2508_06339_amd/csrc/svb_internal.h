// Internal declarations shared by the HIP translation units of libsvb.
// gfx950 only; wavefront size 64.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/svb.h"

namespace svb {

constexpr int kWave = 64;

// Storage <-> compute conversions.  f16 and bf16 are storage types only: products
// and sums are formed in f32 (the paper's treatment of half precision, Section 4.3).
typedef __hip_bfloat16 bf16_t;
template <typename T> struct compute_of { using type = T; };
template <> struct compute_of<__half> { using type = float; };
template <> struct compute_of<bf16_t> { using type = float; };

template <typename C, typename T> __device__ __forceinline__ C ld_as(const T* p) { return (C)(*p); }
template <> __device__ __forceinline__ float ld_as<float, __half>(const __half* p) { return __half2float(*p); }
template <typename T, typename C> __device__ __forceinline__ void st_as(T* p, C v) { *p = (T)v; }
template <> __device__ __forceinline__ void st_as<__half, float>(__half* p, float v) { *p = __float2half(v); }
template <> __device__ __forceinline__ float ld_as<float, bf16_t>(const bf16_t* p) { return __bfloat162float(*p); }
template <> __device__ __forceinline__ void st_as<bf16_t, float>(bf16_t* p, float v) { *p = __float2bfloat16(v); }

// Reciprocal and square root for reflector scalars: the hardware approximations (1 ulp,
// biased) refined by Newton steps.  A biased tau or scale would make every reflector
// non-orthogonal in the same direction, which adds up over a sweep.
__device__ __forceinline__ float newton_rcp(float x)
{
    const float r = __builtin_amdgcn_rcpf(x);
    return fmaf(r, fmaf(-x, r, 1.0f), r);
}
__device__ __forceinline__ double newton_rcp(double x)
{
    double r = __builtin_amdgcn_rcp(x);
    r = fma(r, fma(-x, r, 1.0), r);
    return fma(r, fma(-x, r, 1.0), r);
}
__device__ __forceinline__ float newton_sqrt(float x)   // x > 0, normal
{
    const float r = __builtin_amdgcn_rsqf(x);
    const float s = x * r;
    return fmaf(fmaf(-s, s, x), 0.5f * r, s);
}
__device__ __forceinline__ double newton_sqrt(double x)   // x > 0, normal
{
    const double r = __builtin_amdgcn_rsq(x), h = 0.5 * r;
    double s = x * r;
    s = fma(fma(-s, s, x), h, s);
    return fma(fma(-s, s, x), h, s);
}

// Geometry of one half-sweep's panel tree (Section 3.1: GEQRT on the first
// tile, then the tiles below are annihilated; here the tiles of a panel are
// grouped into domains that are factored independently and merged level by
// level, each level stacking the R factors of the level below).
struct Level {
    int chunks;        // number of nb-row chunks at this level
    int domains;       // ceil(chunks / g)
    int64_t stride;    // distance in panel rows between consecutive chunks: nb * g^level
    int64_t poff;      // element offset of this level's panel inside the panel buffers
    int64_t ldp;       // leading dimension of this level's panel = chunks * nb
};
constexpr int kMaxLevels = 12;

struct Orient {
    // address of trailing-matrix element (p, q): base + p*sp + q*sq, where p runs along
    // the panel direction (rows for a QR sweep, columns for an LQ sweep) and q
    // along the free direction.
    int64_t sp, sq;
};

// ---- stage 1, panel ---------------------------------------------------------
template <typename T, typename C>
void launch_panel_gather(const T* A, int64_t lda, int64_t row0, int64_t col0, bool lq,
                         int64_t len, int nb, C* P, int64_t ldp, hipStream_t s);

template <typename T, typename C>
void launch_panel_qr(int nb, C* P, int64_t ldp, C* Y, C* Tws, int chunks, int g,
                     C* Pnext, int64_t ldnext, const T* Asrc, int64_t lda, bool lq, C* band, int64_t ldab,
                     int64_t row0, int64_t col0, hipStream_t s, hipEvent_t done = nullptr, hipEvent_t start = nullptr);

// blocked register-resident domain QR (MFMA block reflectors inside the domain); domains of at
// most panel_blk_rows<C>() rows
// Asrc != nullptr: the panel is read straight from the matrix (Asrc = &A[row0, col0], QR / LQ
// orientation) instead of the work panel P; band != nullptr: R goes straight into the packed band
// (the last tree level) instead of Pnext.
template <typename C> struct PanelTreeArgs;
// tree (may be null, first level only): the upper levels run in launch_panel_tree beside this launch
template <typename T, typename C>
void launch_panel_blk(int nb, C* P, int64_t ldp, C* Tws, int chunks, int g, C* Pnext, int64_t ldnext,
                      const T* Asrc, int64_t lda, bool lq, C* band, int64_t ldab, int64_t row0, int64_t col0,
                      hipStream_t s, hipEvent_t done = nullptr, hipEvent_t start = nullptr,
                      int* out_flags = nullptr, int flag_base = 0, const PanelTreeArgs<C>* tree = nullptr);
template <typename C> int panel_blk_rows();
// Y = V T for every domain of a level (T: nb x nb per domain)
template <typename C>
void launch_panel_y_nb(int nb, const C* V, C* Y, const C* Tws, int64_t ldp, int64_t rows, int g, hipStream_t s);

// Every tree level above the first in one launch that runs beside the first level's kernel
// (launch_panel_blk with out_flags): a domain hands its R to the level above 16 rows at a time, as
// its block steps complete, and the level above follows one block step behind.
template <typename C> struct PanelTreeLevel {
    C* P; C* Tws; C* Pnext;   // the level's panel (stacked R factors, V on return), its T factors, the next level's panel
    int64_t ldp, ldnext;
    int chunks;               // nb-row factors stacked at this level
    int tiles;                // 16-row tiles of its tallest domain
    int first;                // ticket of its first domain
    int flags_in, flags_out;  // offsets of the flags of the level below / of this level
};
template <typename C> struct PanelTreeArgs {
    PanelTreeLevel<C> lv[kMaxLevels];
    int nl, total, g, lq;     // levels in this launch, workgroups, chunks per domain, orientation
    int* ticket;              // zero on entry
    int* flags;
    int* err;
    int flag_base, spin_limit;
    int* started;             // set to flag_base by the first level's kernel when it begins
    int start_spin;           // polls of `started` after which the upper levels' launch leaves its tickets to that kernel
    C* band; int64_t ldab, row0, col0;   // where the last level's R goes
};
template <typename C>
void launch_panel_tree(int nb, const PanelTreeArgs<C>& a, hipStream_t s, hipEvent_t start, hipEvent_t done);
void launch_fill_int(int* p, int n, int v, hipStream_t s);
template <typename C> void launch_tree_err(const int* err, C* band_entry, hipStream_t s);
// does the blocked kernel serve this (type, nb, chunks per domain)?  Then the first level needs no
// gathered copy of its panel and the last level no separate scatter of R.
template <typename C> bool panel_blk_serves(int nb, int g);

template <typename C>
void launch_scatter_r(const C* R, int64_t ldr, int nb, C* band, int64_t ldab,
                      int64_t row0, int64_t col0, bool lq, hipStream_t s);

template <typename C>
void launch_band_clear(C* band, int64_t ldab, int64_t n, hipStream_t s);

// ---- stage 1, trailing update ----------------------------------------------
// For every domain d of a tree level: W_d = Y_d^T C_d, then C_d -= V_d W_d (QR orientation; the
// LQ orientation is the same with p/q swapped), in one pass over the trailing matrix (W stays in
// registers); domains of at most fused_update_rows<C>() rows.  tri: the panel is a stack of upper
// triangular factors (tree levels above the first), whose structural zeros in V and Y are skipped.
// Tw: the domains' triangular factors (NB x NB each, column-major); if given (nb <= 64 only), Y is
// not read and W = T^T (V^T C) is formed inside the kernel.
template <typename T, typename C>
void launch_update_fused(int nb, bool lq, T* Cbase, int64_t lda, int64_t qlen, const C* V, const C* Y,
                         int64_t ldp, int chunks, int g, int64_t stride, bool tri, const C* Tw,
                         bool credited, hipStream_t s, bool half_ops = true);
template <typename C> int fused_update_rows();
// the same update for nb = 128 in f32 arithmetic on the 32 x 32 x 2 MFMA (domains of at most 512
// rows, qlen a multiple of 32)
template <typename T>
void launch_update_fused32(bool lq, T* Cbase, int64_t lda, int64_t qlen, const float* V, const float* Y,
                           int64_t ldp, int chunks, int g, int64_t stride, bool tri, bool credited, hipStream_t s);

// the same update for f16 / bf16 storage with both products on the 16-bit matrix instructions (f32
// accumulate; V, Y and W enter as sums of 16-bit terms), domains of at most 512 rows
template <typename T>
void launch_update_fused16(int nb, bool lq, T* Cbase, int64_t lda, int64_t qlen, const float* V, const float* Y,
                           int64_t ldp, int chunks, int g, int64_t stride, bool tri, const float* Tw, bool credited,
                           hipStream_t s);

// per-kernel timing hooks (no-ops unless profiling is enabled)
void prof_begin(int kind, hipStream_t s, double flops, double bytes);
void prof_end(hipStream_t s);
// For a single kernel: if profiling is on, hands out a pair of events for a launch that ties them
// to the kernel itself (hipExtLaunchKernelGGL's start and stop events: the kernel's own time
// stamps, no marker in the stream before or after it) and returns true.
bool prof_take(int kind, double flops, double bytes, hipEvent_t* start, hipEvent_t* stop);

// ---- preparation: staging copy, magnitude scan, scaling ------------------------
// factors (device, doubles): [0] = power of two the matrix is multiplied by before stage 1,
// [1] = its reciprocal (applied to the bidiagonal), [2] = largest magnitude found.
// S (mp x np, leading dimension lds, zero padded) = A (m x n) or, with transpose, A^T.
template <typename T>
void launch_stage_copy(const T* A, int64_t lda, int64_t m, int64_t n, bool transpose, T* S, int64_t lds,
                       int64_t mp, int64_t np, hipStream_t s);
// largest magnitude of the m x n matrix -> factors (NaN if an entry is not finite); then the
// matrix is multiplied by factors[0] where that is not 1
template <typename T>
void launch_scale_to_range(T* A, int64_t lda, int64_t m, int64_t n, double* factors, hipStream_t s);
// the same with the window given: scaled when the largest magnitude's binary exponent lies outside
// [lo_exp, hi_exp], so that it becomes target_exp
template <typename T>
void launch_scale_to_range(T* A, int64_t lda, int64_t m, int64_t n, double* factors, hipStream_t s, int lo_exp,
                           int hi_exp, int target_exp);
size_t scale_workspace_bytes();   // bytes behind `factors` (the factors and the scan's partial maxima)
// d, e (n entries each) multiplied by factors[1]
template <typename C>
void launch_rescale_bidiag(C* d, C* e, int64_t n, const double* factors, hipStream_t s);

// ---- stage 2 -----------------------------------------------------------------
template <typename C>
int run_chase(int64_t n, int nb, C* band, int64_t ldab, C* d, C* e,
              void* work, size_t work_bytes, hipStream_t s);
size_t chase_workspace_bytes(int64_t n, int nb);
template <typename C>
void launch_extract_bidiag(const C* band, int64_t ldab, int64_t n, int b, C* d, C* e, const int* ctrl,
                           const int* ctrl2, hipStream_t s);
// narrow band (8 super-diagonals) -> bidiagonal inside LDS windows; entry (i,j) at band[(i-j+ku) + j*ldab]
template <typename C>
int run_chase_narrow(int64_t n, C* band, int64_t ldab, int64_t ku, int* ctrl, hipStream_t s);
size_t chase_narrow_workspace_bytes(int64_t n);
// band of nb super-diagonals -> band of 8 (blocked chase, same storage); false / SVB_ERR_UNSUPPORTED
// where two nb x nb blocks do not fit in LDS
bool band_reduce_supported(int nb, size_t elem_size);
template <typename C>
int run_band_reduce(int64_t n, int nb, C* band, int64_t ldab, int* ctrl, hipStream_t s);
size_t band_reduce_workspace_bytes(int64_t n);

// ---- stage 3 (host) -----------------------------------------------------------
int host_bdsvals(int64_t n, const double* d, const double* e, double* sigma);

// ---- stage 3 (device) ---------------------------------------------------------
template <typename C>
// interval width on exit: rel_tol * max(sigma, floor_frac * bound on sigma_max)
int run_bdsvals_dev(int64_t n, const C* d, const C* e, C* sigma, void* work, double rel_tol, double floor_frac,
                    hipStream_t s);
size_t bdsvals_dev_workspace_bytes(int64_t n);

int env_int(const char* name, int dflt);

}  // namespace svb
