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


// ---------------------------------------------------------------- pipelined chase
// One workgroup per sweep, sweeps pipelined along the band.  Workgroups take
// sweep numbers from a ticket counter, so a sweep is only ever waited for by
// later sweeps and its owner is already running: no co-residency assumption.
// Sweep i may run step t once sweep i-1 has finished step t+2 (see the region
// argument at the top of this file); progress[i] counts finished steps and is
// set to kDone when the sweep is complete.  Waits are bounded by spin_limit;
// on expiry the error flag is raised, every later sweep drains, and the
// extraction kernel poisons d[0] so the failure reaches the caller.
//
// Per step the workgroup keeps two B x B blocks in LDS (column-major, leading
// dimension B+1): X = the block above the diagonal block (its first row is
// the row being annihilated), Z = the diagonal block A2.  After the right
// reflector X is final and is written back while the block right of A2 (A3,
// prefetched into registers at the start of the step) takes its place; after
// the left reflector A2 is written back and A3 stays in LDS as the next step's X.

// Reflector from the strided vector src[0], src[inc], ... (len entries, first one the
// pivot), built by wave 0: vs <- v (v_0 = 1, zero beyond len), red[0] <- tau, and the vector
// itself is replaced by (beta, 0, ...).  Other waves pass through.
template <typename C, int B>
__device__ __forceinline__ void house_wave(C* src, int inc, int len, C* vs, C* red)
{
    if (threadIdx.x >= kWave) return;
    constexpr int PL = (B + kWave - 1) / kWave;
    const int lane = threadIdx.x;
    C x[PL];
    C ss = 0;
#pragma unroll
    for (int q = 0; q < PL; ++q) {
        const int idx = lane + q * kWave;
        x[q] = idx < len ? src[idx * inc] : (C)0;
        if (idx > 0) ss += x[q] * x[q];
    }
    ss = wsum(ss);
    const C alpha = __shfl(x[0], 0, kWave);
    C beta, tau, inv;
    reflector<C>(alpha, ss, beta, tau, inv);
#pragma unroll
    for (int q = 0; q < PL; ++q) {
        const int idx = lane + q * kWave;
        if (idx < B) {
            vs[idx] = idx < len ? ((idx == 0) ? (C)1 : x[q] * inv) : (C)0;
            src[idx * inc] = (idx == 0) ? beta : (C)0;
        }
    }
    if (lane == 0) red[0] = tau;
}

// Rows 1..B-1 of X and 0..B-1 of Z (column-major, leading dimension LD) get
// row <- row - tau (row . v) v.  A row is split over NT/(2B) threads.
template <typename C, int B, int NT>
__device__ __forceinline__ void apply_rows(C* X, C* Z, int LD, const C* vs, const C* red, C* part)
{
    constexpr int SPLIT = NT / (2 * B) > 0 ? NT / (2 * B) : 1, W = B / SPLIT;
    const C tau = red[0];
    const int tid = threadIdx.x, ridx = tid % (2 * B), h = tid / (2 * B);
    C* base = (ridx < B ? X + ridx : Z + (ridx - B)) + h * W * LD;
    const C* v = vs + h * W;
    C row[W];
    C s = 0;
#pragma unroll
    for (int j = 0; j < W; ++j) {
        row[j] = base[j * LD];
        s += v[j] * row[j];
    }
    if (SPLIT > 1) {
        part[tid] = s;
        __syncthreads();
        s = 0;
#pragma unroll
        for (int q = 0; q < SPLIT; ++q) s += part[ridx + q * 2 * B];
    }
    s *= tau;
    if (ridx != 0 && tau != (C)0) {
#pragma unroll
        for (int j = 0; j < W; ++j) base[j * LD] = row[j] - s * v[j];
    }
}

// Columns 1..B-1 of Z and 0..B-1 of X get col <- col - tau (v . col) v.
template <typename C, int B, int NT>
__device__ __forceinline__ void apply_cols(C* Z, C* X, int LD, const C* vs, const C* red, C* part)
{
    constexpr int SPLIT = NT / (2 * B) > 0 ? NT / (2 * B) : 1, W = B / SPLIT;
    const C tau = red[0];
    const int tid = threadIdx.x, cidx = tid % (2 * B), h = tid / (2 * B);
    C* col = (cidx < B ? Z + cidx * LD : X + (cidx - B) * LD) + h * W;
    const C* v = vs + h * W;
    C cv[W];
    C s = 0;
#pragma unroll
    for (int a = 0; a < W; ++a) {
        cv[a] = col[a];
        s += v[a] * cv[a];
    }
    if (SPLIT > 1) {
        part[tid] = s;
        __syncthreads();
        s = 0;
#pragma unroll
        for (int q = 0; q < SPLIT; ++q) s += part[cidx + q * 2 * B];
    }
    s *= tau;
    if (cidx != 0 && tau != (C)0) {
#pragma unroll
        for (int a = 0; a < W; ++a) col[a] = cv[a] - s * v[a];
    }
}

constexpr int kDone = 0x3fffffff;

// Band entries travel between workgroups (possibly on different XCDs, each with its own
// L2) while the kernel runs: they are read and written with device-scope accesses that
// bypass the non-coherent cache levels, so that no whole-cache write-back or invalidate
// is needed per step.
template <typename C> __device__ __forceinline__ C gld(const C* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename C> __device__ __forceinline__ void gst(C* p, C v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename C, int B, int NT>
__global__ __launch_bounds__(NT) void chase_persistent_kernel(C* __restrict__ band, int64_t ldab, int64_t n,
                                                              int* __restrict__ ctrl, int* __restrict__ progress,
                                                              int spin_limit)
{
    constexpr int LD = B + 1, NW = NT / kWave, CSTEP = NT / B;
    // A3 is prefetched into registers only while that stays cheap (B*B/NT values per thread)
    constexpr bool PREFETCH = (B * B / NT) <= 16;
    constexpr int PER = PREFETCH ? B * B / NT : 1;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C* X = reinterpret_cast<C*>(smem_raw);
    C* Z = X + B * LD;
    C* vs = Z + B * LD;
    C* red = vs + B;  // NW + 1
    C* part = red + NW + 1;  // NT
    __shared__ int sh_i, sh_fail;
    const int tid = threadIdx.x;
#ifdef SVB_CHASE_TIMING
    unsigned long long tacc[6] = {0, 0, 0, 0, 0, 0}, tlast = 0, nstep_acc = 0;
#define TMARK(slot_) do { if (tid == 0) { unsigned long long now_ = wall_clock64(); tacc[slot_] += now_ - tlast; tlast = now_; } } while (0)
#else
#define TMARK(slot_) do { } while (0)
#endif
    const int ii = tid % B, jj0 = tid / B;  // this thread's row and first column inside a block
    const int64_t ku = 2 * (int64_t)B - 1;
#define BAND(r_, c_) band[((r_) - (c_) + ku) + (c_) * ldab]

    // Every thread-0-only section below is followed by a barrier before the next one, so
    // that no divergent region ever spans a loop back-edge.
    for (;;) {
        if (tid == 0) {
            sh_i = atomicAdd(&ctrl[0], 1);
            sh_fail = __hip_atomic_load(&ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        const int64_t i = sh_i;
        bool failed = sh_fail != 0;
        __syncthreads();
        if (i > n - 3) break;
        const int nsteps = (int)((n - 3 - i) / B) + 1;
        for (int t = 0; t < nsteps && !failed; ++t) {
            const int64_t c0 = i + 1 + (int64_t)t * B;
            const int len = (int)min((int64_t)B, n - c0);
            const int na3 = (int)max((int64_t)0, min((int64_t)B, n - (c0 + B)));
#ifdef SVB_CHASE_TIMING
            if (tid == 0) { tlast = wall_clock64(); ++nstep_acc; }
#endif
            if (i > 0) {
                if (tid == 0) {
                    const int need = t + 3;
                    int spins = 0;
                    while (__hip_atomic_load(&progress[i - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < need) {
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
                TMARK(0);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            }
            TMARK(1);
            if (!failed) {
                // A2 -> Z, (first step) row i -> X, A3 -> registers.  All global loads are
                // issued before the first LDS write so that their latencies overlap.
                constexpr int ZPER = B * B / NT;
                C pre[PER];
                C zr[ZPER];
#pragma unroll
                for (int q = 0; q < ZPER; ++q) {
                    const int jj = jj0 + q * CSTEP;
                    zr[q] = (ii < len && jj < len) ? gld(&BAND(c0 + ii, c0 + jj)) : (C)0;
                }
                if (PREFETCH) {
#pragma unroll
                    for (int q = 0; q < PER; ++q) {
                        const int jj = jj0 + q * CSTEP;
                        pre[q] = (ii < len && jj < na3) ? gld(&BAND(c0 + ii, c0 + B + jj)) : (C)0;
                    }
                }
                if (t == 0) {
                    for (int jj = jj0; jj < B; jj += CSTEP) {
                        C xv = 0;
                        if (ii == 0 && jj < len) xv = gld(&BAND(i, c0 + jj));
                        X[ii + jj * LD] = xv;
                    }
                }
#pragma unroll
                for (int q = 0; q < ZPER; ++q) Z[ii + (jj0 + q * CSTEP) * LD] = zr[q];
                __syncthreads();
                TMARK(2);
                // right reflector from X row 0 (built by wave 0 alone: one barrier instead of a
                // block-wide reduction), applied to X rows 1.. and Z by all threads
                house_wave<C, B>(X, LD, len, vs, red);
                __syncthreads();
                apply_rows<C, B, NT>(X, Z, LD, vs, red, part);
                __syncthreads();
                TMARK(3);
                // X is final: write it back, A3 takes its place
                if (PREFETCH) {
#pragma unroll
                    for (int q = 0; q < PER; ++q) {
                        const int jj = jj0 + q * CSTEP;
                        const C v = X[ii + jj * LD];
                        if (jj < len) {
                            if (t == 0) {
                                if (ii == 0) gst(&BAND(i, c0 + jj), v);
                            } else {
                                gst(&BAND(c0 - B + ii, c0 + jj), v);
                            }
                        }
                        X[ii + jj * LD] = pre[q];
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < ZPER; ++q) {
                        const int jj = jj0 + q * CSTEP;
                        zr[q] = (ii < len && jj < na3) ? gld(&BAND(c0 + ii, c0 + B + jj)) : (C)0;
                    }
#pragma unroll
                    for (int q = 0; q < ZPER; ++q) {
                        const int jj = jj0 + q * CSTEP;
                        const C v = X[ii + jj * LD];
                        if (jj < len) {
                            if (t == 0) {
                                if (ii == 0) gst(&BAND(i, c0 + jj), v);
                            } else {
                                gst(&BAND(c0 - B + ii, c0 + jj), v);
                            }
                        }
                        X[ii + jj * LD] = zr[q];
                    }
                }
                __syncthreads();
                // left reflector from Z column 0, applied to Z columns 1.. and A3
                house_wave<C, B>(Z, 1, len, vs, red);
                __syncthreads();
                apply_cols<C, B, NT>(Z, X, LD, vs, red, part);
                __syncthreads();
                TMARK(4);
                // A2 is final for this sweep; after the last step so is A3
                for (int jj = jj0; jj < B; jj += CSTEP) {
                    if (ii < len && jj < len) gst(&BAND(c0 + ii, c0 + jj), Z[ii + jj * LD]);
                    if (t == nsteps - 1 && ii < len && jj < na3) gst(&BAND(c0 + ii, c0 + B + jj), X[ii + jj * LD]);
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            }
            __syncthreads();
            TMARK(5);
            if (tid == 0)
                __hip_atomic_store(&progress[i], (failed || t == nsteps - 1) ? kDone : t + 1, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
        }
        if (failed) {
            if (tid == 0) __hip_atomic_store(&progress[i], kDone, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
    }
#ifdef SVB_CHASE_TIMING
    if (tid == 0) {
        unsigned long long* acc = reinterpret_cast<unsigned long long*>(ctrl + 8);
        for (int q = 0; q < 6; ++q) atomicAdd(&acc[q], tacc[q]);
        atomicAdd(&acc[6], nstep_acc);
    }
#endif
#undef TMARK
#undef BAND
}


// Rows (or columns) of ONE B x B block: line <- line - tau (line . v) v for lines first..B-1.
// ROWS: a line is a row (stride LD), else a column (contiguous).  A line is split over NT/B threads.
template <typename C, int B, int NT, bool ROWS>
__device__ __forceinline__ void apply_one(C* buf, int LD, const C* vs, const C* red, C* part, int first)
{
    constexpr int SPLIT = NT / B, W = B / SPLIT;
    const C tau = red[0];
    const int tid = threadIdx.x, idx = tid % B, h = tid / B;
    C* base = ROWS ? buf + idx + h * W * LD : buf + idx * LD + h * W;
    const int inc = ROWS ? LD : 1;
    const C* v = vs + h * W;
    C line[W];
    C s = 0;
#pragma unroll
    for (int j = 0; j < W; ++j) {
        line[j] = base[j * inc];
        s += v[j] * line[j];
    }
    if (SPLIT > 1) {
        part[tid] = s;
        __syncthreads();
        s = 0;
#pragma unroll
        for (int q = 0; q < SPLIT; ++q) s += part[idx + q * B];
    }
    s *= tau;
    if (idx >= first && tau != (C)0) {
#pragma unroll
        for (int j = 0; j < W; ++j) base[j * inc] = line[j] - s * v[j];
    }
}

// Variant of the pipelined chase that keeps ONE B x B block in LDS (for block sizes of
// which two do not fit: f64 at B = 128).  Same pipeline protocol and the same arithmetic
// as chase_persistent_kernel; per step the single buffer holds, in turn, the block above
// the diagonal block (X), the diagonal block (A2) and the block right of it (A3), each
// loaded from and stored to the band once.
template <typename C, int B, int NT>
__global__ __launch_bounds__(NT) void chase_persistent_1buf_kernel(C* __restrict__ band, int64_t ldab, int64_t n,
                                                                   int* __restrict__ ctrl, int* __restrict__ progress,
                                                                   int spin_limit)
{
    constexpr int LD = B + 1, CSTEP = NT / B, PER = B * B / NT;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C* Wb = reinterpret_cast<C*>(smem_raw);
    C* vs = Wb + B * LD;
    C* red = vs + B;    // 2
    C* part = red + 2;  // NT
    __shared__ int sh_i, sh_fail;
    const int tid = threadIdx.x;
    const int ii = tid % B, jj0 = tid / B;
    const int64_t ku = 2 * (int64_t)B - 1;
#define BAND(r_, c_) band[((r_) - (c_) + ku) + (c_) * ldab]

    for (;;) {
        if (tid == 0) {
            sh_i = atomicAdd(&ctrl[0], 1);
            sh_fail = __hip_atomic_load(&ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        const int64_t i = sh_i;
        bool failed = sh_fail != 0;
        __syncthreads();
        if (i > n - 3) break;
        const int nsteps = (int)((n - 3 - i) / B) + 1;
        for (int t = 0; t < nsteps && !failed; ++t) {
            const int64_t c0 = i + 1 + (int64_t)t * B;
            const int len = (int)min((int64_t)B, n - c0);
            const int na3 = (int)max((int64_t)0, min((int64_t)B, n - (c0 + B)));
            if (i > 0) {
                if (tid == 0) {
                    const int need = t + 3;
                    int spins = 0;
                    while (__hip_atomic_load(&progress[i - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < need) {
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
            if (!failed) {
                C zr[PER];
                // A2 -> registers (its latency overlaps the work on X)
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int jj = jj0 + q * CSTEP;
                    zr[q] = (ii < len && jj < len) ? gld(&BAND(c0 + ii, c0 + jj)) : (C)0;
                }
                if (t == 0) {
                    for (int jj = jj0; jj < B; jj += CSTEP) {
                        C xv = 0;
                        if (ii == 0 && jj < len) xv = gld(&BAND(i, c0 + jj));
                        Wb[ii + jj * LD] = xv;
                    }
                    __syncthreads();
                }
                // right reflector from X row 0; X rows 1.. updated; X is final: store it
                house_wave<C, B>(Wb, LD, len, vs, red);
                __syncthreads();
                apply_one<C, B, NT, true>(Wb, LD, vs, red, part, 1);
                __syncthreads();
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int jj = jj0 + q * CSTEP;
                    const C v = Wb[ii + jj * LD];
                    if (jj < len) {
                        if (t == 0) {
                            if (ii == 0) gst(&BAND(i, c0 + jj), v);
                        } else {
                            gst(&BAND(c0 - B + ii, c0 + jj), v);
                        }
                    }
                    Wb[ii + jj * LD] = zr[q];   // A2 takes the buffer
                }
                __syncthreads();
                // A3 -> registers, then the right reflector on every row of A2
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int jj = jj0 + q * CSTEP;
                    zr[q] = (ii < len && jj < na3) ? gld(&BAND(c0 + ii, c0 + B + jj)) : (C)0;
                }
                apply_one<C, B, NT, true>(Wb, LD, vs, red, part, 0);
                __syncthreads();
                // left reflector from A2 column 0; columns 1.. updated; A2 is final: store it
                house_wave<C, B>(Wb, 1, len, vs, red);
                __syncthreads();
                apply_one<C, B, NT, false>(Wb, LD, vs, red, part, 1);
                __syncthreads();
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int jj = jj0 + q * CSTEP;
                    if (ii < len && jj < len) gst(&BAND(c0 + ii, c0 + jj), Wb[ii + jj * LD]);
                    Wb[ii + jj * LD] = zr[q];   // A3 takes the buffer
                }
                __syncthreads();
                // the left reflector on every column of A3, which stays as the next step's X
                apply_one<C, B, NT, false>(Wb, LD, vs, red, part, 0);
                __syncthreads();
                if (t == nsteps - 1) {
#pragma unroll
                    for (int q = 0; q < PER; ++q) {
                        const int jj = jj0 + q * CSTEP;
                        if (ii < len && jj < na3) gst(&BAND(c0 + ii, c0 + B + jj), Wb[ii + jj * LD]);
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            }
            __syncthreads();
            if (tid == 0)
                __hip_atomic_store(&progress[i], (failed || t == nsteps - 1) ? kDone : t + 1, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
        }
        if (failed) {
            if (tid == 0) __hip_atomic_store(&progress[i], kDone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
    }
#undef BAND
}

__global__ __launch_bounds__(256) void chase_ctrl_clear_kernel(int* __restrict__ ctrl, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (int64_t)gridDim.x * blockDim.x)
        ctrl[i] = 0;
}

template <typename C, int B>
static bool launch_chase_persistent(C* band, int64_t ldab, int64_t n, int* ctrl, hipStream_t s)
{
    constexpr size_t smem2 = sizeof(C) * (size_t)(2 * B * (B + 1) + B + 256 / kWave + 1 + 256);
    constexpr bool ONEBUF = smem2 > 150 * 1024;   // two blocks do not fit: single-buffer variant, 512 threads
    constexpr int NT = ONEBUF ? 512 : 256;
    constexpr size_t smem = ONEBUF ? sizeof(C) * (size_t)(B * (B + 1) + B + 2 + NT) : smem2;
    if (smem > 150 * 1024) return false;
    void (*kern)(C*, int64_t, int64_t, int*, int*, int);
    if (ONEBUF) kern = chase_persistent_1buf_kernel<C, B, ONEBUF ? 512 : 256>;
    else kern = chase_persistent_kernel<C, B, 256>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    const int64_t count = 64 + n;
    int cb = (int)((count + 255) / 256);
    hipLaunchKernelGGL(chase_ctrl_clear_kernel, dim3(cb > 1024 ? 1024 : cb), dim3(256), 0, s, ctrl, count);
    const int64_t sweeps = n - 2;
    const int grid = (int)min((int64_t)env_int("SVB_CHASE_GRID", 256), sweeps);
    const int spin_limit = env_int("SVB_CHASE_SPIN", 1 << 20);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), smem, s, band, ldab, n, ctrl, ctrl + 64, spin_limit);
    return true;
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
                                                             C* __restrict__ e, const int* __restrict__ ctrl,
                                                             const int* __restrict__ ctrl2)
{
    const bool bad = (ctrl != nullptr && ctrl[1] != 0) || (ctrl2 != nullptr && ctrl2[1] != 0);
    const int64_t ku = 2 * (int64_t)b - 1;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        d[i] = (bad && i == 0) ? (C)NAN : band[ku + i * ldab];
        e[i] = (i + 1 < n) ? band[(ku - 1) + (i + 1) * ldab] : (C)0;
    }
}

size_t chase_workspace_bytes(int64_t n, int /*nb*/) { return (size_t)((64 + n) * 4 + 255) / 256 * 256; }

template <typename C>
int run_chase(int64_t n, int nb, C* band, int64_t ldab, C* d, C* e, void* work,
              size_t /*work_bytes*/, hipStream_t s)
{
    constexpr int NT = 256;
    const int64_t b = nb;
    int* ctrl = static_cast<int*>(work);
    bool pipelined = false;
    if (n >= 3 && env_int("SVB_CHASE_IMPL", 1) != 0) {
        if (nb == 32) pipelined = launch_chase_persistent<C, 32>(band, ldab, n, ctrl, s);
        else if (nb == 64) pipelined = launch_chase_persistent<C, 64>(band, ldab, n, ctrl, s);
        else pipelined = launch_chase_persistent<C, 128>(band, ldab, n, ctrl, s);
    }
    if (n >= 3 && !pipelined) {
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
    hipLaunchKernelGGL((extract_bidiag_kernel<C>), dim3(blocks), dim3(256), 0, s, band, ldab, n, (int)b, d, e,
                       pipelined ? ctrl : (const int*)nullptr, (const int*)nullptr);
    return hipGetLastError() == hipSuccess ? SVB_OK : SVB_ERR_DEVICE;
}

template <typename C>
void launch_extract_bidiag(const C* band, int64_t ldab, int64_t n, int b, C* d, C* e, const int* ctrl,
                           const int* ctrl2, hipStream_t s)
{
    int blocks = (int)((n + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL((extract_bidiag_kernel<C>), dim3(blocks), dim3(256), 0, s, band, ldab, n, b, d, e, ctrl, ctrl2);
}
template void launch_extract_bidiag<double>(const double*, int64_t, int64_t, int, double*, double*, const int*, const int*, hipStream_t);
template void launch_extract_bidiag<float>(const float*, int64_t, int64_t, int, float*, float*, const int*, const int*, hipStream_t);

template int run_chase<double>(int64_t, int, double*, int64_t, double*, double*, void*, size_t, hipStream_t);
template int run_chase<float>(int64_t, int, float*, int64_t, float*, float*, void*, size_t, hipStream_t);

}  // namespace svb
