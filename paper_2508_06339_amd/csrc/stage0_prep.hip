// Preparation of the input for stage 1 (nothing here is in the paper, whose kernels take a
// square matrix of whole tiles, Algorithm 2, and do not rescale, Section 3.2 "Accuracy"):
//   - staging copy: a matrix whose shape is not a whole number of tiles, or that is wider than
//     tall, is copied (transposed if wider than tall) into a zero-padded work matrix.  Rows and
//     columns of zeros stay exactly zero under every reflector of stage 1 (the reflector has a
//     zero there), so the band of the padded matrix is the band of the matrix itself followed by
//     zeros, and stage 2 runs on the leading min(m, n) columns only;
//   - magnitude scan and scaling: the panel kernels form sums of squares without scaling them, so
//     a matrix whose largest entry is far from 1 is multiplied by a power of two first (exact),
//     and the bidiagonal is multiplied back.
#include "svb_internal.h"

namespace svb {

namespace {

constexpr int kScanBlocks = 1024;   // partial maxima of the magnitude scan

// S(i, j) = A(i, j) (or A(j, i)) inside the matrix, zero in the padding; 32 x 32 tiles, block (32, 8)
template <typename T, bool TR>
__global__ __launch_bounds__(256) void stage_copy_kernel(const T* __restrict__ A, int64_t lda, int64_t m, int64_t n,
                                                         T* __restrict__ S, int64_t lds, int64_t mp, int64_t np)
{
    __shared__ T tile[32][33];
    const int64_t i0 = (int64_t)blockIdx.x * 32, j0 = (int64_t)blockIdx.y * 32;
    const int tx = threadIdx.x, ty = threadIdx.y;
    if (!TR) {
        for (int jj = ty; jj < 32; jj += 8) {
            const int64_t i = i0 + tx, j = j0 + jj;
            if (i < mp && j < np) S[i + j * lds] = (i < m && j < n) ? A[i + j * lda] : T(0.0f);
        }
    } else {
        // S(i, j) = A(j, i): read along A's columns (j runs fastest), write along S's
        for (int ii = ty; ii < 32; ii += 8) {
            const int64_t i = i0 + ii, j = j0 + tx;     // A(j, i)
            tile[ii][tx] = (j < m && i < n) ? A[j + i * lda] : T(0.0f);
        }
        __syncthreads();
        for (int jj = ty; jj < 32; jj += 8) {
            const int64_t i = i0 + tx, j = j0 + jj;
            if (i < mp && j < np) S[i + j * lds] = tile[tx][jj];
        }
    }
}

template <typename T> __device__ __forceinline__ double mag(const T* p)
{
    return fabs((double)ld_as<typename compute_of<T>::type, T>(p));
}

// NaN-propagating maximum of magnitudes (an infinity counts as not finite as well)
__device__ __forceinline__ double nmax(double a, double b) { return (a != a || b != b) ? NAN : fmax(a, b); }

template <typename T>
__global__ __launch_bounds__(256) void absmax_kernel(const T* __restrict__ A, int64_t lda, int64_t m, int64_t n,
                                                     double* __restrict__ partial)
{
    __shared__ double red[4];
    double v = 0.0;
    // a block takes whole columns, its threads run along a column (contiguous)
    for (int64_t j = blockIdx.x; j < n; j += gridDim.x)
        for (int64_t i = threadIdx.x; i < m; i += 256) v = nmax(v, mag<T>(&A[i + j * lda]));
    for (int off = 32; off > 0; off >>= 1) v = nmax(v, __shfl_xor(v, off, kWave));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        v = nmax(nmax(red[0], red[1]), nmax(red[2], red[3]));
        partial[blockIdx.x] = (v > 1.79e308) ? NAN : v;
    }
}

// limits of the largest magnitude beyond which the matrix is scaled: squares of the entries, summed
// over a column, must stay inside the arithmetic type's range with room to spare
template <typename T> struct ScaleRange { static constexpr int kExp = 40; };     // f32 arithmetic
template <> struct ScaleRange<double> { static constexpr int kExp = 400; };

template <typename T>
__global__ __launch_bounds__(256) void scale_kernel(T* __restrict__ A, int64_t lda, int64_t m, int64_t n,
                                                    const double* __restrict__ partial, int nparts,
                                                    double* __restrict__ factors, int lo_exp, int hi_exp, int target_exp)
{
    __shared__ double red[4];
    __shared__ double sh_f;
    double v = 0.0;
    for (int i = threadIdx.x; i < nparts; i += 256) v = nmax(v, partial[i]);
    for (int off = 32; off > 0; off >>= 1) v = nmax(v, __shfl_xor(v, off, kWave));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        v = nmax(nmax(red[0], red[1]), nmax(red[2], red[3]));
        double f = 1.0;
        if (v == v && v > 0.0) {
            int ex;
            (void)frexp(v, &ex);                       // v = frac * 2^ex, frac in [0.5, 1)
            if (ex > hi_exp || ex < lo_exp) f = ldexp(1.0, target_exp - ex);
        }
        sh_f = f;
        if (blockIdx.x == 0) {
            factors[0] = f;
            factors[1] = 1.0 / f;
            factors[2] = v;
        }
    }
    __syncthreads();
    const double f = sh_f;
    if (f == 1.0) return;
    for (int64_t j = blockIdx.x; j < n; j += gridDim.x)
        for (int64_t i = threadIdx.x; i < m; i += 256) {
            using C = typename compute_of<T>::type;
            T* p = &A[i + j * lda];
            st_as<T, C>(p, (C)((double)ld_as<C, T>(p) * f));
        }
}

template <typename C>
__global__ __launch_bounds__(256) void rescale_bidiag_kernel(C* __restrict__ d, C* __restrict__ e, int64_t n,
                                                             const double* __restrict__ factors)
{
    const double r = factors[1];
    if (r == 1.0) return;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        d[i] = (C)((double)d[i] * r);
        e[i] = (C)((double)e[i] * r);
    }
}

}  // namespace

template <typename T>
void launch_stage_copy(const T* A, int64_t lda, int64_t m, int64_t n, bool transpose, T* S, int64_t lds,
                       int64_t mp, int64_t np, hipStream_t s)
{
    dim3 grid((unsigned)((mp + 31) / 32), (unsigned)((np + 31) / 32)), block(32, 8);
    if (transpose) hipLaunchKernelGGL((stage_copy_kernel<T, true>), grid, block, 0, s, A, lda, m, n, S, lds, mp, np);
    else hipLaunchKernelGGL((stage_copy_kernel<T, false>), grid, block, 0, s, A, lda, m, n, S, lds, mp, np);
}

// factors: 8 doubles, followed by kScanBlocks partial maxima
template <typename T>
void launch_scale_to_range(T* A, int64_t lda, int64_t m, int64_t n, double* factors, hipStream_t s, int lo_exp,
                           int hi_exp, int target_exp)
{
    const int blocks = (int)(n < kScanBlocks ? (n < 1 ? 1 : n) : kScanBlocks);
    double* partial = factors + 8;
    hipLaunchKernelGGL((absmax_kernel<T>), dim3(blocks), dim3(256), 0, s, A, lda, m, n, partial);
    hipLaunchKernelGGL((scale_kernel<T>), dim3(blocks), dim3(256), 0, s, A, lda, m, n, partial, blocks, factors, lo_exp,
                       hi_exp, target_exp);
}
template <typename T>
void launch_scale_to_range(T* A, int64_t lda, int64_t m, int64_t n, double* factors, hipStream_t s)
{
    launch_scale_to_range<T>(A, lda, m, n, factors, s, -ScaleRange<T>::kExp, ScaleRange<T>::kExp, 0);
}

size_t scale_workspace_bytes() { return (size_t)(8 + kScanBlocks) * sizeof(double); }

template <typename C>
void launch_rescale_bidiag(C* d, C* e, int64_t n, const double* factors, hipStream_t s)
{
    int blocks = (int)((n + 255) / 256);
    if (blocks > 256) blocks = 256;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((rescale_bidiag_kernel<C>), dim3(blocks), dim3(256), 0, s, d, e, n, factors);
}

#define SVB_PREP_INST(T)                                                                                            \
    template void launch_stage_copy<T>(const T*, int64_t, int64_t, int64_t, bool, T*, int64_t, int64_t, int64_t, \
                                       hipStream_t);                                                                \
    template void launch_scale_to_range<T>(T*, int64_t, int64_t, int64_t, double*, hipStream_t);                   \
    template void launch_scale_to_range<T>(T*, int64_t, int64_t, int64_t, double*, hipStream_t, int, int, int);
SVB_PREP_INST(double)
SVB_PREP_INST(float)
SVB_PREP_INST(__half)
SVB_PREP_INST(bf16_t)
#undef SVB_PREP_INST
template void launch_rescale_bidiag<double>(double*, double*, int64_t, const double*, hipStream_t);
template void launch_rescale_bidiag<float>(float*, float*, int64_t, const double*, hipStream_t);

}  // namespace svb
