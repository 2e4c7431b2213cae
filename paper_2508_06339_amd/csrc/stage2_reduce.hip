// Stage 2, first phase: band of B super-diagonals -> band of D = 8 super-diagonals
// (paper Section 3, second stage; the paper names a band-to-bidiagonal reduction without
// giving the algorithm, so this is a blocked bulge chase in the spirit of the successive
// band reduction literature; the second phase, D -> 1, is in stage2_narrow.hip).
//
// Block sweep s makes rows s*D .. s*D+D-1 final (at most D super-diagonals) and chases the
// fill down the band in steps of B columns.  Step t of sweep s works at c0 = (s+1)*D + t*B:
//   right: LQ of the D x B block X (rows rho .. rho+D-1, columns c0 .. c0+B-1; rho = s*D for
//          t = 0, rho = c0 - B otherwise); its D reflectors are applied from the right, as one
//          compact-WY block, to all other rows that have entries in those columns
//          (down to row c0+B-1), which fills the diagonal block Z (rows and columns c0 ..);
//   left:  QR of the first D columns of Z; the reflectors are applied from the left to the
//          other columns of Z and to the block right of it (A3), which becomes the next
//          step's upper block.
// Only D rows / columns of every bulge are annihilated per step; the rest moves down the band
// with the following sweeps.  Step (s+1, t) touches data of step (s, t+2) and nothing later of
// sweep s, so sweeps are pipelined three steps apart: one workgroup per sweep, sweeps drawn
// from a ticket counter, a progress counter per sweep, bounded waits (as in stage2_chase.hip).
//
// Per step the workgroup holds the upper block U (rows c0-B .., the previous step's A3) and Z
// stacked in LDS (2B x B); A3 is prefetched into registers at the start of the step and the
// next step's Z in the middle of it, and they take the place of U and Z once those have been
// written back, so every block is read once and written once per sweep.
//
// Packed band: entry (i,j) at band[(i - j + ku) + j*ldab], ku = 2B-1, ldab >= 3B.
#include "svb_internal.h"

namespace svb {

namespace {

constexpr int kSweepDone = 0x7fffffff;

template <typename C> __device__ __forceinline__ C rgld(const C* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename C> __device__ __forceinline__ void rgst(C* p, C v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// value of lane (l ^ pattern) through the data-parallel-primitive path (no LDS traffic)
template <int CTRL> __device__ __forceinline__ float dpp_get(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int CTRL> __device__ __forceinline__ double dpp_get(double v)
{
    const long long b = __builtin_bit_cast(long long, v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)(unsigned)lo);
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside groups of 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside rows of 16

// sum over the four lanes of a quad, result in all four
template <typename C> __device__ __forceinline__ C quad_allsum(C v)
{
    v += dpp_get<kDppXor1>(v);
    v += dpp_get<kDppXor2>(v);
    return v;
}
// value of one lane as a wave-uniform scalar
__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ double lane_value(double v, int lane)
{
    const long long b = __builtin_bit_cast(long long, v);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffll), lane);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)(unsigned)lo);
}
// lane 15 of the previous row of 16 (CTRL 0x142) / lane 31 (CTRL 0x143) for the rows in ROWS, 0 elsewhere
template <int CTRL, int ROWS> __device__ __forceinline__ float dpp_bcast(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWS, 0xF, false));
}
template <int CTRL, int ROWS> __device__ __forceinline__ double dpp_bcast(double v)
{
    const long long b = __builtin_bit_cast(long long, v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), CTRL, ROWS, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, ROWS, 0xF, false);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)(unsigned)lo);
}
// sum over the 64 lanes of a wave as a wave-uniform scalar: rows of 16 first, then row 0 into
// row 1 and row 2 into row 3, then rows 0+1 into rows 2 and 3; lane 63 holds the total
template <typename C> __device__ __forceinline__ C wave_sum(C v)
{
    v = quad_allsum(v);
    v += dpp_get<kDppHalfMirror>(v);
    v += dpp_get<kDppMirror>(v);
    v += dpp_bcast<0x142, 0xA>(v);
    v += dpp_bcast<0x143, 0xC>(v);
    return lane_value(v, 63);
}

__device__ __forceinline__ float rrcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ double rrcp(double x)
{
    double r = __builtin_amdgcn_rcp(x);
    r = fma(r, fma(-x, r, 1.0), r);
    return fma(r, fma(-x, r, 1.0), r);
}

// position of reflector-vector element e inside the V buffer (D values per element); the
// four segments of the long direction are shifted against each other so that the four
// parts of a line read different LDS banks
template <int B, int D> __device__ __forceinline__ int vidx(int e) { return e * D + (e / (B / 4)) * D; }

// D consecutive values of the V buffer with 16-byte LDS reads
template <int D> __device__ __forceinline__ void load_v(const float* v, float (&out)[D])
{
#pragma unroll
    for (int k = 0; k < D; k += 4) {
        const float4 t = *reinterpret_cast<const float4*>(v + k);
        out[k] = t.x; out[k + 1] = t.y; out[k + 2] = t.z; out[k + 3] = t.w;
    }
}
template <int D> __device__ __forceinline__ void load_v(const double* v, double (&out)[D])
{
#pragma unroll
    for (int k = 0; k < D; k += 2) {
        const double2 t = *reinterpret_cast<const double2*>(v + k);
        out[k] = t.x; out[k + 1] = t.y;
    }
}

// Householder factorisation of a D x B panel held in LDS, by one wave: panel element (k, e),
// k < D along the short and e < B along the long direction, lives at P[k*sk + e*se].
// Reflector k is built from line k, elements k .. B-1, and applied to lines k+1 .. D-1
// (H = I - tau v v^T, v_k = 1, beta = -sign(alpha)*norm).  On exit the panel holds the
// triangular factor (element (k,e) for e <= k, zeros beyond), Vs the vectors
// (Vs[vidx(e) + k]) and Ts the D x D upper triangular T of the compact-WY form
// H_0 H_1 .. H_{D-1} = I - V T V^T, row-major.  One D-vector reduction over the wave per
// reflector yields its norm, the products with the lines below and the products v_j^T v_k
// that T needs; the sums are wave-uniform scalars.
template <typename C, int B, int D>
__device__ __forceinline__ void panel_wave(C* P, int sk, int se, C* Vs, C* Ts)
{
    constexpr int QN = (B + kWave - 1) / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    C x[D][QN];
#pragma unroll
    for (int k = 0; k < D; ++k)
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            const int e = lane + kWave * q;
            x[k][q] = (e < B) ? P[k * sk + e * se] : (C)0;
        }
    const int tj = lane & (D - 1);   // this lane builds row tj of T as the reflectors appear
    C trow[D];
#pragma unroll
    for (int k = 0; k < D; ++k) {
        C p[D], colk[D];
#pragma unroll
        for (int j = 0; j < D; ++j) {
            C acc = 0;
#pragma unroll
            for (int q = 0; q < QN; ++q) {
                const int e = lane + kWave * q;
                acc += (e > k) ? x[j][q] * x[k][q] : (C)0;
            }
            p[j] = wave_sum(acc);
            colk[j] = lane_value(x[j][0], k);   // element k of every line
        }
        const C alpha = colk[k], ss = p[k];
        C beta, inv, tau;
        if (ss == (C)0) {
            beta = alpha; tau = 0; inv = 0;
        } else {
            const C nrm = sqrt(alpha * alpha + ss);
            beta = alpha >= (C)0 ? -nrm : nrm;
            tau = (beta - alpha) * rrcp(beta);
            inv = rrcp(alpha - beta);
        }
        // T(0:k,k) = -tau_k T(0:k,0:k) (V^T v_k), T(k,k) = tau_k; v_j^T v_k = v_j(k) + inv * p_j for j < k
        {
            C acc = 0;
#pragma unroll
            for (int i = 0; i < k; ++i) acc += trow[i] * (colk[i] + inv * p[i]);
            trow[k] = (k == tj) ? tau : (k > tj ? -tau * acc : (C)0);
        }
#pragma unroll
        for (int j = k + 1; j < D; ++j) {
            const C sj = tau * (colk[j] + inv * p[j]);
#pragma unroll
            for (int q = 0; q < QN; ++q) {
                const int e = lane + kWave * q;
                const C vk = (e == k) ? (C)1 : (e > k ? x[k][q] * inv : (C)0);
                x[j][q] -= sj * vk;
            }
        }
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            const int e = lane + kWave * q;
            if (e > k) x[k][q] *= inv;
            else if (e == k) x[k][q] = beta;
        }
    }
    // factor back into the panel, vectors to Vs
#pragma unroll
    for (int q = 0; q < QN; ++q) {
        const int e = lane + kWave * q;
        if (e < B) {
#pragma unroll
            for (int k = 0; k < D; ++k) {
                P[k * sk + e * se] = (e <= k) ? x[k][q] : (C)0;
                Vs[vidx<B, D>(e) + k] = (e < k) ? (C)0 : (e == k ? (C)1 : x[k][q]);
            }
        }
    }
    if (lane < D) {
#pragma unroll
        for (int k = 0; k < D; ++k) Ts[tj * D + k] = trow[k];
    }
}

// Applies the block reflector (Vs, Ts) to one line per quad of lanes: line elements
// base[e*es], e < B; the four lanes of a quad own a quarter of the line each.
// line <- line - ((line . V) T) V^T  (the same expression serves rows under a right
// transformation and columns under a left one: z_k = sum_{j<=k} w_j T(j,k) in both).
template <typename C, int B, int D>
__device__ __forceinline__ void apply_line(C* base, int es, bool valid, const C* Vs, const C* Ts)
{
    constexpr int SEG = B / 4;
    const int p = threadIdx.x & 3;
    const int rot = (SEG == 32 && p >= 2) ? 16 : 0;   // spreads the four parts over the LDS banks
    C w[D];
#pragma unroll
    for (int k = 0; k < D; ++k) w[k] = 0;
    if (valid) {
#pragma unroll 4
        for (int jj = 0; jj < SEG; ++jj) {
            const int e = p * SEG + ((jj + rot) & (SEG - 1));
            const C a = base[e * es];
            C v[D];
            load_v<D>(Vs + vidx<B, D>(e), v);
#pragma unroll
            for (int k = 0; k < D; ++k) w[k] += a * v[k];
        }
    }
#pragma unroll
    for (int k = 0; k < D; ++k) w[k] = quad_allsum(w[k]);
    C z[D];
#pragma unroll
    for (int k = 0; k < D; ++k) {
        C acc = 0;
#pragma unroll
        for (int j = 0; j <= k; ++j) acc += w[j] * Ts[j * D + k];
        z[k] = acc;
    }
    if (valid) {
#pragma unroll 4
        for (int jj = 0; jj < SEG; ++jj) {
            const int e = p * SEG + ((jj + rot) & (SEG - 1));
            C v[D];
            load_v<D>(Vs + vidx<B, D>(e), v);
            C a = base[e * es];
#pragma unroll
            for (int k = 0; k < D; ++k) a -= z[k] * v[k];
            base[e * es] = a;
        }
    }
}

template <typename C, int B, int D>
__global__ __launch_bounds__(8 * B) void band_reduce_kernel(C* __restrict__ band, int64_t ldab, int64_t n,
                                                            int* __restrict__ ctrl, int* __restrict__ progress,
                                                            int spin_limit)
{
    constexpr int NT = 8 * B, LD = 2 * B + 1, PER = B / 8;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C* S = reinterpret_cast<C*>(smem_raw);        // rows c0-B .. c0+B-1, columns c0 .. c0+B-1: S[row + col*LD]
    C* Vs = S + ((B * LD + 3) & ~3);              // (B + 4) * D
    C* Ts = Vs + (B + 4) * D;                     // D * D
    __shared__ int sh_s, sh_fail;
    const int tid = threadIdx.x;
    const int ii = tid % B, jj0 = tid / B;        // this thread's row and first column inside a block (column step 8)
    const int line = (tid >> 6) * 16 + ((tid & 63) >> 2);   // line of the apply phases
    const int64_t ku = 2 * (int64_t)B - 1;
#define BAND(r_, c_) band[((r_) - (c_) + ku) + (c_) * ldab]
#ifdef SVB_CHASE_TIMING
    unsigned long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, tlast = 0, nstep_acc = 0;
#define RMARK(slot_) do { if (tid == 0) { unsigned long long now_ = wall_clock64(); tacc[slot_] += now_ - tlast; tlast = now_; } } while (0)
#else
#define RMARK(slot_) do { } while (0)
#endif
    const int64_t nsweeps = (n - 1) / D;

    // Every thread-0-only section is followed by a barrier before the next one (no divergent
    // region spans a loop back-edge).
    for (;;) {
        if (tid == 0) {
            sh_s = atomicAdd(&ctrl[0], 1);
            sh_fail = __hip_atomic_load(&ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        const int64_t s = sh_s;
        bool failed = sh_fail != 0;
        __syncthreads();
        if (s >= nsweeps) break;
        const int64_t c00 = (s + 1) * D;
        const int nsteps = (int)((n - 1 - c00) / B) + 1;
        for (int t = 0; t < nsteps && !failed; ++t) {
            const int64_t c0 = c00 + (int64_t)t * B;
#ifdef SVB_CHASE_TIMING
            if (tid == 0) { tlast = wall_clock64(); ++nstep_acc; }
#endif
            if (s > 0) {
                if (tid == 0) {
                    const int need = t + 3;   // a finished sweep reports kSweepDone
                    int spins = 0;
                    while (__hip_atomic_load(&progress[s - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < need) {
                        if (++spins > spin_limit) {
                            atomicExch(&ctrl[1], 1);
                            sh_fail = 1;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(1);
                    }
                }
                __syncthreads();
                failed = sh_fail != 0;
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            }
            RMARK(0);
            if (!failed) {
                const int xoff = (t == 0) ? B - D : 0;
                C pre[PER];   // A3 of this step, then Z of the next one
                if (t == 0) {
                    // the sweep's own D rows and the first diagonal block, straight into LDS
                    C u0[PER], z0[PER];
#pragma unroll
                    for (int q = 0; q < PER; ++q) {
                        const int jj = jj0 + 8 * q;
                        const int64_t col = c0 + jj;
                        u0[q] = (ii >= B - D && col < n) ? rgld(&BAND(c0 - B + ii, col)) : (C)0;
                        z0[q] = (c0 + ii < n && col < n) ? rgld(&BAND(c0 + ii, col)) : (C)0;
                    }
#pragma unroll
                    for (int q = 0; q < PER; ++q) {
                        const int jj = jj0 + 8 * q;
                        S[ii + jj * LD] = u0[q];
                        S[B + ii + jj * LD] = z0[q];
                    }
                }
                // A3 of this step: requested now, used after the right half
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int jj = jj0 + 8 * q;
                    const int64_t col = c0 + B + jj;
                    pre[q] = (c0 + ii < n && col < n) ? rgld(&BAND(c0 + ii, col)) : (C)0;
                }
                __syncthreads();
                RMARK(1);
                // ---- right half: LQ of X, block reflector onto the rows below --------------
                if (tid < kWave) panel_wave<C, B, D>(S + xoff, 1, LD, Vs, Ts);
                __syncthreads();
                RMARK(2);
                {
                    const int row = xoff + D + line;
                    apply_line<C, B, D>(S + row, LD, row < 2 * B, Vs, Ts);
                }
                __syncthreads();
                RMARK(3);
                // U is final for this sweep: write it back, A3 takes its place
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int jj = jj0 + 8 * q;
                    const int64_t col = c0 + jj;
                    if (ii >= xoff && col < n) rgst(&BAND(c0 - B + ii, col), S[ii + jj * LD]);
                    S[ii + jj * LD] = pre[q];
                }
                // Z of the next step: requested now, used after the left half
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int jj = jj0 + 8 * q;
                    const int64_t col = c0 + B + jj;
                    pre[q] = (c0 + B + ii < n && col < n) ? rgld(&BAND(c0 + B + ii, col)) : (C)0;
                }
                __syncthreads();
                RMARK(4);
                // ---- left half: QR of Z's first D columns, block reflector onto Z and A3 ------
                if (tid < kWave) panel_wave<C, B, D>(S + B, LD, 1, Vs, Ts);
                __syncthreads();
                RMARK(5);
                {
                    const bool valid = line < 2 * B - D;
                    C* base = (line < B - D) ? S + B + (D + line) * LD : S + (line - (B - D)) * LD;
                    apply_line<C, B, D>(base, 1, valid, Vs, Ts);
                }
                __syncthreads();
                RMARK(6);
                // Z is final for this sweep; the next step's Z takes its place
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int jj = jj0 + 8 * q;
                    const int64_t col = c0 + jj;
                    if (c0 + ii < n && col < n) rgst(&BAND(c0 + ii, col), S[B + ii + jj * LD]);
                    S[B + ii + jj * LD] = pre[q];
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            }
            __syncthreads();
            if (tid == 0)
                __hip_atomic_store(&progress[s], (failed || t == nsteps - 1) ? kSweepDone : t + 1, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            RMARK(7);
        }
        if (failed) {
            if (tid == 0) __hip_atomic_store(&progress[s], kSweepDone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
    }
#ifdef SVB_CHASE_TIMING
    if (tid == 0) {
        unsigned long long* acc = reinterpret_cast<unsigned long long*>(ctrl + 8);
        for (int q = 0; q < 8; ++q) atomicAdd(&acc[q], tacc[q]);
        atomicAdd(&acc[8], nstep_acc);
    }
#endif
#undef RMARK
#undef BAND
}

__global__ __launch_bounds__(256) void reduce_clear_kernel(int* __restrict__ p, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

template <typename C, int B>
int launch_band_reduce(int64_t n, C* band, int64_t ldab, int* ctrl, hipStream_t s)
{
    constexpr int D = 8;
    constexpr size_t smem = sizeof(C) * (size_t)(((B * (2 * B + 1) + 3) & ~3) + (B + 4) * D + D * D);
    static_assert(smem <= 160 * 1024, "block pair does not fit in LDS");
    auto kern = band_reduce_kernel<C, B, D>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    const int64_t nsweeps = (n - 1) / D;
    const int64_t count = 64 + nsweeps + 1;
    const int cb = (int)((count + 255) / 256);
    hipLaunchKernelGGL(reduce_clear_kernel, dim3(cb > 256 ? 256 : cb), dim3(256), 0, s, ctrl, count);
    if (nsweeps <= 0) return SVB_OK;
    const int grid = (int)min((int64_t)env_int("SVB_REDUCE_GRID", 256), nsweeps);
    const int spin_limit = env_int("SVB_CHASE_SPIN", 1 << 20);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(8 * B), smem, s, band, ldab, n, ctrl, ctrl + 64, spin_limit);
    return hipGetLastError() == hipSuccess ? SVB_OK : SVB_ERR_DEVICE;
}

}  // namespace

// ctrl: 64 ints (ticket, error flag, timing slots) followed by one progress counter per block sweep
size_t band_reduce_workspace_bytes(int64_t n) { return (size_t)((64 + n / 8 + 8) * 4 + 255) / 256 * 256; }

bool band_reduce_supported(int nb, size_t elem_size)
{
    if (nb != 32 && nb != 64 && nb != 128) return false;
    return elem_size * ((size_t)nb * (2 * nb + 1) + (size_t)(nb + 4) * 8 + 64 + 4) <= 160 * 1024;
}

template <typename C>
int run_band_reduce(int64_t n, int nb, C* band, int64_t ldab, int* ctrl, hipStream_t s)
{
    if (nb == 32) return launch_band_reduce<C, 32>(n, band, ldab, ctrl, s);
    if (nb == 64) return launch_band_reduce<C, 64>(n, band, ldab, ctrl, s);
    if constexpr (sizeof(C) == 4) {
        if (nb == 128) return launch_band_reduce<C, 128>(n, band, ldab, ctrl, s);
    }
    return SVB_ERR_UNSUPPORTED;
}

template int run_band_reduce<double>(int64_t, int, double*, int64_t, int*, hipStream_t);
template int run_band_reduce<float>(int64_t, int, float*, int64_t, int*, hipStream_t);

}  // namespace svb
