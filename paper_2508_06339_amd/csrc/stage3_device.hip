// Stage 3 on the device: singular values of the upper bidiagonal (d, e) by
// bisection (paper Section 3, final stage; the paper solves the bidiagonal on
// the CPU with LAPACK and names it the cheapest stage.  Once stages 1-2 run
// in tens of milliseconds a host solve dominates time-to-singular-values, so
// the same bisection that the host entry point svb_bdsvals performs is also
// available on the GPU).
//
// Count of singular values below x: with B^T B - x^2 I = L D L^T,
//   t_1 = -x^2,  D_j = d_j^2 + t_j,  t_{j+1} = -x^2 + e_j^2 * t_j / D_j,
// the number of negative D_j (the differential stationary qd form of the Sturm
// sequence: one division per row, n rows).  Squares are taken after scaling by
// the largest entry, always in fp64.  A first kernel counts at 4096 shared points of
// [0, bound]; every singular value then starts from the cell it falls in and is refined by
// multisection (several points per round, one lane each).
#include "svb_internal.h"

namespace svb {

namespace {

constexpr int kPrepThreads = 1024;

// ws[0] = scale, ws[1] = upper bound for sigma_max / scale; d2 = ws + 8, e2 = d2 + n.
template <typename C>
__global__ __launch_bounds__(kPrepThreads) void bd_prep_kernel(const C* __restrict__ d, const C* __restrict__ e,
                                                               int64_t n, double* __restrict__ ws)
{
    __shared__ double red[2][kPrepThreads / kWave];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double zmax = 0.0, bound = 0.0;
    bool bad = false;
    for (int64_t j = tid; j < n; j += kPrepThreads) {
        const double a = fabs((double)d[j]);
        const double b = j + 1 < n ? fabs((double)e[j]) : 0.0;
        const double bp = j > 0 ? fabs((double)e[j - 1]) : 0.0;
        bad = bad || !(a <= 1.79e308) || !(b <= 1.79e308);
        zmax = fmax(zmax, fmax(a, b));
        bound = fmax(bound, a + fmax(b, bp));
    }
    if (bad) { zmax = NAN; bound = NAN; }
    for (int off = 32; off > 0; off >>= 1) {
        const double z2 = __shfl_xor(zmax, off, kWave), b2 = __shfl_xor(bound, off, kWave);
        zmax = (zmax != zmax || z2 != z2) ? NAN : fmax(zmax, z2);
        bound = (bound != bound || b2 != b2) ? NAN : fmax(bound, b2);
    }
    if (lane == 0) { red[0][wave] = zmax; red[1][wave] = bound; }
    __syncthreads();
    zmax = 0.0; bound = 0.0;
    for (int w = 0; w < kPrepThreads / kWave; ++w) {
        const double z2 = red[0][w], b2 = red[1][w];
        zmax = (zmax != zmax || z2 != z2) ? NAN : fmax(zmax, z2);
        bound = (bound != bound || b2 != b2) ? NAN : fmax(bound, b2);
    }
    const double scale = zmax > 0.0 ? zmax : 1.0;  // NaN stays NaN through the comparisons below
    if (tid == 0) {
        ws[0] = (zmax != zmax) ? NAN : scale;
        ws[1] = bound / scale * (1.0 + 1e-14) + 1e-300;
    }
    double* d2 = ws + 8;
    double* e2 = d2 + n;
    for (int64_t j = tid; j < n; j += kPrepThreads) {
        const double a = (double)d[j] / scale;
        const double b = j + 1 < n ? (double)e[j] / scale : 0.0;
        d2[j] = a * a;
        e2[j] = b * b;
    }
}

constexpr int kGrid = 4096;   // points of the shared first partition of [0, bound]

__device__ __forceinline__ double lane_value(double v, int lane)
{
    const long long b = __builtin_bit_cast(long long, v);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffll), lane);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)(unsigned)lo);
}

// Number of singular values below x (x2 = x^2, one value per lane) by the recurrence in the
// header.  All 64 lanes of the wave walk the same rows, so the rows are fetched 64 at a time,
// one per lane, and handed round as wave-uniform scalars: no memory access sits on the
// dependent chain of the recurrence.  Rows past n are padded so that they never count.
__device__ __forceinline__ int64_t sturm_count(const double* __restrict__ d2, const double* __restrict__ e2,
                                               int64_t n, double x2)
{
    const int lane = threadIdx.x & (kWave - 1);
    const double pivmin = 1e-300;
    double t = -x2;
    int64_t cnt = 0;
    double dn = lane < n ? d2[lane] : 1e300, en = lane < n ? e2[lane] : 0.0;
    for (int64_t j0 = 0; j0 < n; j0 += kWave) {
        const double dj = dn, ej = en;
        const int64_t jn = j0 + kWave + lane;
        dn = jn < n ? d2[jn] : 1e300;
        en = jn < n ? e2[jn] : 0.0;
#pragma unroll
        for (int jj = 0; jj < kWave; ++jj) {
            const double dd = lane_value(dj, jj), ee = lane_value(ej, jj);
            double D = dd + t;
            if (fabs(D) < pivmin) D = -pivmin;
            cnt += D < 0.0 ? 1 : 0;
            double r = __builtin_amdgcn_rcp(D);      // reciprocal + one Newton step instead of a full division
            r = fma(r, fma(-D, r, 1.0), r);
            t = ee * (t * r) - x2;
        }
    }
    return cnt;
}

// counts at the points x_i = bound * i / kGrid, i = 1 .. kGrid - 1 (x_0 counts 0, x_kGrid counts n)
__global__ __launch_bounds__(64) void bd_grid_kernel(const double* __restrict__ ws, int64_t n, int* __restrict__ gcnt)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;   // 0 .. kGrid-1, all lanes stay active
    const double scale = ws[0], hi0 = ws[1];
    const double* __restrict__ d2 = ws + 8;
    const double* __restrict__ e2 = d2 + n;
    int64_t c = 0;
    if (scale == scale) {
        const double x = hi0 * ((double)i / kGrid);
        c = sturm_count(d2, e2, n, x * x);
    }
    gcnt[i] = i == 0 ? 0 : (int)min(c, n);
    if (i == 0) gcnt[kGrid] = (int)n;
}

// Multisection: P lanes per singular value, each counting at one of P equally spaced interior
// points of the value's current interval, which shrinks by P + 1 per round (P = 1 is plain
// bisection).  The Sturm recurrence is one long dependent chain per point and a wave costs the
// same whether it refines 64 values by 2 or 4 values by 17 per round, so while the compute
// units have waves to spare the extra points are free and the number of rounds drops.
template <typename C, int P>
__global__ __launch_bounds__(64) void bd_multisect_kernel(const double* __restrict__ ws, int64_t n,
                                                           C* __restrict__ sigma, double rel_tol,
                                                           double floor_frac, const int* __restrict__ gcnt)
{
    constexpr int VPW = kWave / P;   // values per wave
    const int lane = threadIdx.x, grp = lane / P, q = lane % P;
    const int64_t kraw = (int64_t)blockIdx.x * VPW + grp;  // ascending index
    const int64_t k = min(kraw, n - 1);   // surplus lanes repeat the last value: the wave stays whole
    const double scale = ws[0], hi0 = ws[1];
    const double* __restrict__ d2 = ws + 8;
    const double* __restrict__ e2 = d2 + n;
    if (scale != scale) {  // non-finite input: poison the output, the caller maps it to a status
        if (kraw < n && q == 0) sigma[n - 1 - k] = (C)NAN;
        return;
    }
    if (hi0 <= 2e-300) {   // all entries are zero (the bound is its own guard term): so are the values
        if (kraw < n && q == 0) sigma[n - 1 - k] = (C)0;
        return;
    }
    // first interval from the shared partition: gcnt[a] < k+1 <= gcnt[b] with b = a+1
    int a = 0, b = kGrid;
    while (b - a > 1) {
        const int m = (a + b) >> 1;
        if (gcnt[m] >= k + 1) b = m;
        else a = m;
    }
    double lo = hi0 * ((double)a / kGrid), hi = b == kGrid ? hi0 : hi0 * ((double)b / kGrid);
    const double frac = (double)(q + 1) / (P + 1);
    for (int it = 0; it < 200; ++it) {
        const double w = hi - lo, mid = 0.5 * (lo + hi);
        // width relative to the value, or to floor_frac times the bound on the largest value if that is more
        const bool open = (w > rel_tol * fmax(hi, floor_frac * hi0) + 1e-38 * hi0) && (mid > lo && mid < hi);
        if (!__any(open)) break;            // wave-uniform exit: the row hand-over needs every lane
        // this lane's point; rounding may put it on an end of the interval, where the count is known
        const double x = fmin(fmax(fma(w, frac, lo), lo), hi);
        const int64_t cnt = sturm_count(d2, e2, n, x * x);
        const bool above = x >= hi || (x > lo && cnt >= k + 1);   // the value lies below this point
        // the points of a value are ascending, so its lanes read: below .. below, above .. above
        const unsigned long long m = __ballot(above) >> (grp * P);
        const unsigned long long mine = P == 64 ? m : (m & ((1ull << P) - 1ull));
        const int f = mine ? __builtin_ctzll(mine) : P;          // first point above the value
        if (open) {
            // (the same expressions the lanes f - 1 and f evaluated their points with)
            const double nlo = f == 0 ? lo : fmin(fmax(fma(w, (double)f / (P + 1), lo), lo), hi);
            const double nhi = f == P ? hi : fmin(fmax(fma(w, (double)(f + 1) / (P + 1), lo), lo), hi);
            lo = nlo;
            hi = nhi;
        }
    }
    if (kraw < n && q == 0) sigma[n - 1 - k] = (C)(0.5 * (lo + hi) * scale);
}

}  // namespace

// doubles: scale, bound, 6 spare, d^2, e^2; then the counts at the partition points
size_t bdsvals_dev_workspace_bytes(int64_t n) { return (size_t)(8 + 2 * n) * sizeof(double) + (size_t)(kGrid + 8) * sizeof(int); }

template <typename C>
int run_bdsvals_dev(int64_t n, const C* d, const C* e, C* sigma, void* work, double rel_tol, double floor_frac,
                    hipStream_t s)
{
    double* ws = static_cast<double*>(work);
    hipLaunchKernelGGL((bd_prep_kernel<C>), dim3(1), dim3(kPrepThreads), 0, s, d, e, n, ws);
    int* gcnt = reinterpret_cast<int*>(ws + 8 + 2 * n);
    hipLaunchKernelGGL(bd_grid_kernel, dim3(kGrid / 64), dim3(64), 0, s, ws, n, gcnt);
    // points per value: as many as keep the launch at about two waves per SIMD
    int p = env_int("SVB_STAGE3_POINTS", 0);
    if (p <= 0) p = n <= 8192 ? 16 : (n <= 16384 ? 8 : (n <= 32768 ? 4 : (n <= 65536 ? 2 : 1)));
    auto launch = [&](auto kern, int pp) {
        const int vpw = kWave / pp;
        hipLaunchKernelGGL(kern, dim3((unsigned)((n + vpw - 1) / vpw)), dim3(64), 0, s, ws, n, sigma, rel_tol, floor_frac,
                           gcnt);
    };
    if (p >= 16) launch(bd_multisect_kernel<C, 16>, 16);
    else if (p >= 8) launch(bd_multisect_kernel<C, 8>, 8);
    else if (p >= 4) launch(bd_multisect_kernel<C, 4>, 4);
    else if (p >= 2) launch(bd_multisect_kernel<C, 2>, 2);
    else launch(bd_multisect_kernel<C, 1>, 1);
    return hipGetLastError() == hipSuccess ? SVB_OK : SVB_ERR_DEVICE;
}

template int run_bdsvals_dev<double>(int64_t, const double*, const double*, double*, void*, double, double, hipStream_t);
template int run_bdsvals_dev<float>(int64_t, const float*, const float*, float*, void*, double, double, hipStream_t);

}  // namespace svb
