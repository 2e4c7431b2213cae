// Stage 2: band -> bidiagonal by bulge chasing (paper Section 3: "the second,
// memory-bound stage ... GPU-accelerated band-to-bidiagonal reduction"; the
// paper gives no algorithm, so this is the standard first-column chase).
//
// Packed band, b = nb super-diagonals on entry; entry (i,j) at
// band[(i - j + 2b - 1) + j*ldab], room for b-1 sub-diagonals and 2b-1
// super-diagonals of bulge.
//
// Sweep i (i = 0 .. n-3) makes row i bidiagonal and chases the fill-in off the
// matrix.  Step t of sweep i works at c0 = i + 1 + t*b with len = min(b, n-c0):
//   right reflector on columns c0 .. c0+len-1, built from row r (r = i for
//   t = 0, r = c0 - b otherwise), zeroing B(r, c0+1 ..); applied to rows
//   r+1 .. c0+len-1;
//   left reflector on rows c0 .. c0+len-1, built from column c0, zeroing
//   B(c0+1 .., c0); applied to columns c0+1 .. min(n-1, c0+len-1+b).
// Only the first row / column of each bulge is annihilated; the rest moves
// down the band with the following sweeps.
//
// Step (i+1, t) touches data of step (i, t+2) and nothing later of sweep i,
// so all steps with 3*i + t = const are independent: they are launched
// together, one workgroup per step, one launch per value of 3*i + t.
#include "svb_internal.h"

namespace svb {

template <typename C> __device__ __forceinline__ C wsum(C v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

template <typename C, int NT>
__device__ __forceinline__ C block_sum(C v, C* red)
{
    constexpr int NW = NT / kWave;
    v = wsum(v);
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = v;
    __syncthreads();
    C s = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) s += red[w];
    return s;
}

// Reflector scalars from pivot alpha and squared tail norm ss.
template <typename C>
__device__ __forceinline__ void reflector(C alpha, C ss, C& beta, C& tau, C& inv)
{
    if (ss == (C)0) {
        beta = alpha;
        tau = 0;
        inv = 0;
    } else {
        const C nrm = sqrt(alpha * alpha + ss);
        beta = alpha >= (C)0 ? -nrm : nrm;
        tau = (beta - alpha) / beta;
        inv = (C)1 / (alpha - beta);
    }
}

template <typename C, int NT>
__device__ void chase_step(C* __restrict__ band, int64_t ldab, int64_t n, int b, int64_t i, int64_t t,
                           C* vs, C* red)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    constexpr int NW = NT / kWave;
    const int64_t ku = 2 * (int64_t)b - 1;
#define BAND(r_, c_) band[((r_) - (c_) + ku) + (c_) * ldab]
    const int64_t c0 = i + 1 + t * b;
    const int len = (int)min((int64_t)b, n - c0);
    const int64_t r = (t == 0) ? i : c0 - b;

    // ---- right reflector from row r ---------------------------------------
    {
        C x = 0, ss = 0;
        if (tid < len) {
            x = BAND(r, c0 + tid);
            if (tid > 0) ss = x * x;
        }
        ss = block_sum<C, NT>(ss, red);
        if (tid == 0) vs[2 * b] = x;  // pivot
        __syncthreads();
        C beta, tau, inv;
        reflector<C>(vs[2 * b], ss, beta, tau, inv);
        if (tid < len) {
            vs[tid] = (tid == 0) ? (C)1 : x * inv;
            BAND(r, c0 + tid) = (tid == 0) ? beta : (C)0;
        }
        __syncthreads();
        if (tau != (C)0) {
            const int64_t rows = c0 + len - 1 - r;  // rows r+1 .. c0+len-1
            for (int64_t a = tid; a < rows; a += NT) {
                const int64_t q = r + 1 + a;
                C s = 0;
                for (int j = 0; j < len; ++j) s += vs[j] * BAND(q, c0 + j);
                s *= tau;
                for (int j = 0; j < len; ++j) BAND(q, c0 + j) -= s * vs[j];
            }
        }
        __syncthreads();
    }
    // ---- left reflector from column c0 --------------------------------------
    {
        C x = 0, ss = 0;
        if (tid < len) {
            x = BAND(c0 + tid, c0);
            if (tid > 0) ss = x * x;
        }
        ss = block_sum<C, NT>(ss, red);
        if (tid == 0) vs[2 * b] = x;
        __syncthreads();
        C beta, tau, inv;
        reflector<C>(vs[2 * b], ss, beta, tau, inv);
        if (tid < len) {
            vs[tid] = (tid == 0) ? (C)1 : x * inv;
            BAND(c0 + tid, c0) = (tid == 0) ? beta : (C)0;
        }
        __syncthreads();
        if (tau != (C)0) {
            const int64_t cend = min(n - 1, c0 + len - 1 + b);  // columns c0+1 .. cend
            for (int64_t c = c0 + 1 + wave; c <= cend; c += NW) {
                C s = 0;
                for (int a = lane; a < len; a += kWave) s += vs[a] * BAND(c0 + a, c);
                s = wsum(s) * tau;
                for (int a = lane; a < len; a += kWave) BAND(c0 + a, c) -= s * vs[a];
            }
        }
    }
#undef BAND
}

template <typename C, int NT>
__global__ __launch_bounds__(NT) void chase_wave_kernel(C* __restrict__ band, int64_t ldab, int64_t n,
                                                        int b, int64_t T, int64_t imin)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C* vs = reinterpret_cast<C*>(smem_raw);  // 2b + 1 entries
    __shared__ C red[NT / kWave];
    const int64_t i = imin + blockIdx.x;
    const int64_t t = T - 3 * i;
    chase_step<C, NT>(band, ldab, n, b, i, t, vs, red);
}

template <typename C>
__global__ __launch_bounds__(256) void extract_bidiag_kernel(const C* __restrict__ band, int64_t ldab,
                                                             int64_t n, int b, C* __restrict__ d,
                                                             C* __restrict__ e)
{
    const int64_t ku = 2 * (int64_t)b - 1;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        d[i] = band[ku + i * ldab];
        e[i] = (i + 1 < n) ? band[(ku - 1) + (i + 1) * ldab] : (C)0;
    }
}

size_t chase_workspace_bytes(int64_t /*n*/, int /*nb*/) { return 0; }

template <typename C>
int run_chase(int64_t n, int nb, C* band, int64_t ldab, C* d, C* e, void* /*work*/,
              size_t /*work_bytes*/, hipStream_t s)
{
    constexpr int NT = 256;
    const int64_t b = nb;
    if (n >= 3) {
        const int64_t Tmax = 3 * (n - 3);
        const size_t smem = (size_t)(2 * b + 2) * sizeof(C);
        for (int64_t T = 0; T <= Tmax; ++T) {
            // steps (i, t = T - 3i) with t >= 0 and i + 1 + t*b <= n - 2
            int64_t imax = T / 3;
            if (imax > n - 3) imax = n - 3;
            int64_t num = T * b - (n - 3);
            int64_t den = 3 * b - 1;
            int64_t imin = num <= 0 ? 0 : (num + den - 1) / den;
            if (imin > imax) continue;
            hipLaunchKernelGGL((chase_wave_kernel<C, NT>), dim3((unsigned)(imax - imin + 1)), dim3(NT),
                               smem, s, band, ldab, n, (int)b, T, imin);
        }
    }
    int blocks = (int)((n + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL((extract_bidiag_kernel<C>), dim3(blocks), dim3(256), 0, s, band, ldab, n, (int)b, d, e);
    return hipGetLastError() == hipSuccess ? SVB_OK : SVB_ERR_DEVICE;
}

template int run_chase<double>(int64_t, int, double*, int64_t, double*, double*, void*, size_t, hipStream_t);
template int run_chase<float>(int64_t, int, float*, int64_t, float*, float*, void*, size_t, hipStream_t);

}  // namespace svb
