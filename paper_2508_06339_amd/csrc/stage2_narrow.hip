// Stage 2, narrow bands: band -> bidiagonal for a band of D = 8 super-diagonals
// (paper Section 3, second stage; the paper points to cache-efficient tile kernels and a
// communication-avoiding strategy without giving the algorithm).
//
// The chase itself is the one described in stage2_chase.hip (sweep i, step t at
// c0 = i + 1 + t*D: right reflector from row r on columns c0.., left reflector from column
// c0 on rows c0..; step t of sweep i+1 after step t+2 of sweep i).  What changes is where
// the hand-over between consecutive sweeps happens.  With one workgroup per sweep every
// hand-over goes through device memory, and the 3n dependent steps each pay that latency.
// Here a workgroup owns a BUNDLE of NW consecutive sweeps, four per wave (16 lanes each), and
// a sliding window of the band in LDS: a super-step is one HALF step (right or left reflector) of every
// sweep of the bundle, sweep w running 4w half steps behind sweep 0 (half step h of sweep i+1 needs
// half step h+3 of sweep i); a workgroup barrier separates super-steps, so the hand-over between the waves of a bundle
// is an LDS access.  Device memory is touched in chunks of CH = 8*D or 16*D columns: a chunk enters
// the window two groups (of 8 or 16 super-steps) before it is needed, and leaves it once the last
// wave has passed.  Bundles are pipelined over workgroups through a ticket counter and a
// per-bundle count of flushed columns (bounded waits, as in stage2_chase.hip).
//
// Packed band: entry (i,j) at band[(i - j + ku) + j*ldab]; ku >= 2D-1 and ldab >= ku + D.
#include "svb_internal.h"

namespace svb {

namespace {

constexpr int kAllFlushed = 0x7fffffff;

template <typename C> __device__ __forceinline__ C ngld(const C* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename C> __device__ __forceinline__ void ngst(C* p, C v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS hand-over inside a wave / between waves without waiting for outstanding global loads
// (a workgroup-scope fence would also drain vmcnt, i.e. stall on the chunk prefetch):
// s_waitcnt lgkmcnt(0) only (gfx9 encoding: vmcnt = 63, expcnt = 7, lgkmcnt = 0).
__device__ __forceinline__ void lds_wave_sync()
{
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
}
__device__ __forceinline__ void lds_block_sync()
{
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();
}

// Reciprocal with the hardware instruction (1 ulp) plus, for f64, one Newton step: the
// reflector scalars sit on the serial path of every step.
__device__ __forceinline__ float fast_rcp(float x)
{
    // hardware reciprocal (1 ulp, biased) refined by one Newton step: a biased tau or scale
    // makes every reflector slightly non-orthogonal in the same direction, which adds up
    const float r = __builtin_amdgcn_rcpf(x);
    return fmaf(r, fmaf(-x, r, 1.0f), r);
}
__device__ __forceinline__ double fast_rcp(double x)
{
    double r = __builtin_amdgcn_rcp(x);
    return fma(r, fma(-x, r, 1.0), r);
}

template <typename C>
__device__ __forceinline__ void nreflector(C alpha, C ss, C& beta, C& tau, C& inv)
{
    if (ss == (C)0) {
        beta = alpha; tau = 0; inv = 0;
    } else {
        const C nrm = sqrt(alpha * alpha + ss);
        beta = alpha >= (C)0 ? -nrm : nrm;
        tau = (beta - alpha) * fast_rcp(beta);
        inv = fast_rcp(alpha - beta);
    }
}

// One HALF step (the right reflector of step t if left == false, else its left reflector)
// for each of the four sweeps of a wave: lanes 16g .. 16g+15 work on the sweep of group g
// (its own i, t; act = false if that sweep has nothing to do now).  Consecutive sweeps are
// four half steps apart, so all sweeps of a bundle do the same kind of half step at a time.
// vbuf holds the pivot row / column of each group so that every lane can form the reflector.
template <typename C, int D, int WC>
__device__ __forceinline__ void narrow_half4(C* win, C* vbuf, int i, int t, bool left, bool act, int n)
{
    constexpr int RS = 3 * D;
    const int lane = threadIdx.x & 63, sub = lane & 15, grp = lane >> 4;
#define WIN(r_, c_) win[((c_) & (WC - 1)) * RS + ((r_) - (c_)) + 2 * D - 1]
    const int c0 = i + 1 + t * D;
    const int len = act ? min(D, n - c0) : 0;
    const int r = (t == 0) ? i : c0 - D;
    C* vb = vbuf + grp * D;
    C a[D];
    if (!left) {
        // right reflector from row r, applied to rows r+1 .. c0+len-1 (lane = row)
        const C x = (sub < len) ? WIN(r, c0 + sub) : (C)0;
        if (sub < D) vb[sub] = x;
        const int rows = c0 + len - 1 - r;
        const int q = r + 1 + sub;
        const bool mine = sub < rows;
#pragma unroll
        for (int jj = 0; jj < D; ++jj) a[jj] = (mine && jj < len) ? WIN(q, c0 + jj) : (C)0;
        lds_wave_sync();
        C v[D];
        C ss = 0;
#pragma unroll
        for (int jj = 0; jj < D; ++jj) {
            v[jj] = vb[jj];
            if (jj > 0) ss += v[jj] * v[jj];
        }
        C beta, tau, inv;
        nreflector<C>(v[0], ss, beta, tau, inv);
        v[0] = (C)1;
        C s = a[0];
#pragma unroll
        for (int jj = 1; jj < D; ++jj) {
            v[jj] *= inv;
            s += v[jj] * a[jj];
        }
        s *= tau;
        if (sub < len) WIN(r, c0 + sub) = (sub == 0) ? beta : (C)0;
        if (mine && tau != (C)0) {
#pragma unroll
            for (int jj = 0; jj < D; ++jj)
                if (jj < len) WIN(q, c0 + jj) = a[jj] - s * v[jj];
        }
    } else {
        // left reflector from column c0, applied to columns c0+1 .. min(n-1, c0+len-1+D) (lane = column)
        const C x = (sub < len) ? WIN(c0 + sub, c0) : (C)0;
        if (sub < D) vb[sub] = x;
        const int cols = act ? min(n - 1, c0 + len - 1 + D) - c0 : 0;
        const int c = c0 + 1 + sub;
        const bool mine = sub < cols;
#pragma unroll
        for (int jj = 0; jj < D; ++jj) a[jj] = (mine && jj < len) ? WIN(c0 + jj, c) : (C)0;
        lds_wave_sync();
        C v[D];
        C ss = 0;
#pragma unroll
        for (int jj = 0; jj < D; ++jj) {
            v[jj] = vb[jj];
            if (jj > 0) ss += v[jj] * v[jj];
        }
        C beta, tau, inv;
        nreflector<C>(v[0], ss, beta, tau, inv);
        v[0] = (C)1;
        C s = a[0];
#pragma unroll
        for (int jj = 1; jj < D; ++jj) {
            v[jj] *= inv;
            s += v[jj] * a[jj];
        }
        s *= tau;
        if (sub < len) WIN(c0 + sub, c0) = (sub == 0) ? beta : (C)0;
        if (mine && tau != (C)0) {
#pragma unroll
            for (int jj = 0; jj < D; ++jj)
                if (jj < len) WIN(c0 + jj, c) = a[jj] - s * v[jj];
        }
    }
#undef WIN
}

// The same half step for the common case: every active sweep of the wave is at least 2D
// columns away from the end of the matrix (full-length reflectors, full blocks) and, for a
// right reflector, its D columns do not straddle the wrap of the window.  Then every element
// a lane touches sits at a constant offset from one base address (consecutive columns of one
// row are RS - 1 apart, consecutive rows of one column 1 apart), each lane reads the pivot
// row / column itself (the 16 lanes of a sweep read the same addresses: a broadcast), and
// nothing but the row / column count needs a predicate.  H = I (tau = 0) falls out of the
// arithmetic: then s = 0 and the stores write back what was read.
template <typename C, int D, int WC, bool LEFT>
__device__ __forceinline__ void narrow_half4_fast(C* win, int i, int t, bool act)
{
    constexpr int RS = 3 * D, M = WC - 1;
    constexpr int SV = LEFT ? 1 : RS - 1;   // distance between consecutive elements of the pivot / of a lane's line
    const int sub = threadIdx.x & 15;
    const int c0 = i + 1 + t * D;
    C* pv;        // pivot element jj at pv[jj * SV]
    C* pa;        // this lane's row / column: element jj at pa[jj * SV]
    bool mine;
    if constexpr (!LEFT) {
        const int r = (t == 0) ? i : c0 - D;
        mine = act && sub < c0 + D - 1 - r;                 // rows r+1 .. c0+D-1
        pv = win + (c0 & M) * RS + (r - c0) + 2 * D - 1;    // (r, c0 + jj)
        pa = pv + 1 + sub;                                  // (r + 1 + sub, c0 + jj)
    } else {
        mine = act && sub < 2 * D - 1;                      // columns c0+1 .. c0+2D-1
        pv = win + (c0 & M) * RS + 2 * D - 1;               // (c0 + jj, c0)
        pa = win + ((c0 + 1 + sub) & M) * RS + 2 * D - 2 - sub;   // (c0 + jj, c0 + 1 + sub)
    }
    if (mine) {
        C v[D], a[D];
#pragma unroll
        for (int jj = 0; jj < D; ++jj) { v[jj] = pv[jj * SV]; a[jj] = pa[jj * SV]; }
        // sum of squares of the pivot's tail and its product with this lane's line, two chains
        // each, both independent of the reflector's scalars: the tail is used unscaled,
        //   H a = a - s (1, inv * tail),  s = tau (a_0 + inv * tail^T a_tail)
        C ssa = v[1] * v[1], ssb = v[2] * v[2], da = v[1] * a[1], db = v[2] * a[2];
#pragma unroll
        for (int jj = 3; jj < D; jj += 2) {
            ssa += v[jj] * v[jj];
            da += v[jj] * a[jj];
            if (jj + 1 < D) {
                ssb += v[jj + 1] * v[jj + 1];
                db += v[jj + 1] * a[jj + 1];
            }
        }
        const C ss = ssa + ssb;
        // the reflector without a branch: with ss = 0 the selects give H = I whatever the
        // discarded operands evaluate to
        const C alpha = v[0];
        const C x2 = alpha * alpha + ss;
        // the refined hardware square root wants a normal argument; sums of squares near the
        // underflow threshold (rare) take the library routine, for the whole wave
        constexpr C kTiny = sizeof(C) == 8 ? (C)1e-290 : (C)1e-30f;
        C nrm;
        if (__any(x2 < kTiny)) nrm = sqrt(x2); else nrm = newton_sqrt(x2);
        const C bc = alpha >= (C)0 ? -nrm : nrm;
        const bool ident = ss == (C)0;
        const C beta = ident ? alpha : bc;
        const C tau = ident ? (C)0 : (bc - alpha) * fast_rcp(bc);
        const C inv = ident ? (C)0 : fast_rcp(alpha - bc);
        const C s = tau * (a[0] + inv * (da + db));
        const C w = s * inv;
        if (sub < D) pv[sub * SV] = (sub == 0) ? beta : (C)0;
        pa[0] = a[0] - s;
#pragma unroll
        for (int jj = 1; jj < D; ++jj) pa[jj * SV] = a[jj] - w * v[jj];
    }
}

// One super-step of a wave: the half step h of each of its four sweeps, then the workgroup barrier.
template <typename C, int D, int WC, bool LEFT>
__device__ __forceinline__ void narrow_super_step(C* win, C* vbuf, int my_i, int h, bool have, int my_steps, int n)
{
    const bool act = have && h >= 0 && h < 2 * my_steps;
    const int tt = act ? (int)(h >> 1) : 0;
    const int c0 = my_i + 1 + tt * D;
    const bool fast = !act || (c0 + 2 * D <= n && (LEFT || (c0 & (WC - 1)) <= WC - D));
    if (__all(fast))
        narrow_half4_fast<C, D, WC, LEFT>(win, my_i, tt, act);
    else
        narrow_half4<C, D, WC>(win, vbuf, my_i, tt, LEFT, act, n);
    lds_block_sync();
}

template <typename C, int D, int NW, int WC, int GS>
__global__ __launch_bounds__(NW * 16) void chase_narrow_kernel(C* __restrict__ band, int64_t ldab, int64_t ku,
                                                               int64_t n, int* __restrict__ ctrl,
                                                               int* __restrict__ flushed, int spin_limit)
{
    constexpr int NT = NW * 16, RS = 3 * D, CH = GS * D;   // four sweeps per wave
    // GS lead steps (2*GS half steps) per group; sweep w runs 4w half steps = 2w steps behind sweep 0
    constexpr int LAGC = (2 * (NW - 1) + GS - 1) / GS;    // chunks the flush trails the load front by
    constexpr int PER = (CH * RS + NT - 1) / NT;
    static_assert((LAGC + 4) * CH <= WC, "window too small");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C* win = reinterpret_cast<C*>(smem_raw);  // WC columns x RS
    C* vbuf = win + WC * RS + (threadIdx.x >> 6) * 4 * D;
    __shared__ int sh_b, sh_fail;
    const int tid = threadIdx.x;
    const int slot = ((tid >> 6) << 2) + ((tid & 63) >> 4);   // which sweep of the bundle this lane works on
#ifdef SVB_CHASE_TIMING
    unsigned long long tacc[4] = {0, 0, 0, 0}, tlast = 0, ngrp = 0;
#define NMARK(slot_) do { if (tid == 0) { unsigned long long now_ = wall_clock64(); tacc[slot_] += now_ - tlast; tlast = now_; } } while (0)
#else
#define NMARK(slot_) do { } while (0)
#endif
    const int64_t nsweeps = n - 2;                         // sweeps 0 .. n-3
    const int64_t nbundles = (nsweeps + NW - 1) / NW;

    // element e of a chunk: column e / RS, storage row e % RS (row 3D-1 is unused padding)
    auto chunk_ptr = [&](int64_t col0, int e, bool& ok) -> C* {
        const int cl = e / RS, sr = e % RS;
        const int64_t j = col0 + cl;
        const int64_t i = j + sr - (2 * D - 1);
        ok = e < CH * RS && sr < RS - 1 && j < n && i >= 0 && i < n;
        return band + (i - j + ku) + j * ldab;
    };

    for (;;) {
        if (tid == 0) {
            sh_b = atomicAdd(&ctrl[0], 1);
            sh_fail = __hip_atomic_load(&ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        const int64_t b = sh_b;
        bool failed = sh_fail != 0;
        __syncthreads();
        if (b >= nbundles) break;
        const int64_t i0 = b * NW;
        const int64_t my_i = i0 + slot;
        const bool have = my_i <= n - 3;
        const int64_t my_steps = have ? (n - 3 - my_i) / D + 1 : 0;
        // half steps of this bundle: sweep 0 has the most steps, later sweeps start 4 half steps apart
        int64_t htot = 0;
        for (int w = 0; w < NW; ++w) {
            const int64_t iw = i0 + w;
            if (iw <= n - 3) htot = max(htot, (int64_t)4 * w + 2 * ((n - 3 - iw) / D + 1));
        }
        const int64_t ngroups = (htot + 2 * GS - 1) / (2 * GS);
        const int64_t nchunks = (n - i0 + CH - 1) / CH;    // chunks that hold columns < n

        // waits until the previous bundle has flushed every column below `upto`
        auto wait_prev = [&](int64_t upto) {
            if (b > 0) {
                if (tid == 0) {
                    const int need = (int)min(upto, n);
                    int spins = 0;
                    while (__hip_atomic_load(&flushed[b - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < need) {
                        if (++spins > spin_limit) {
                            atomicExch(&ctrl[1], 1);
                            sh_fail = 1;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
                __syncthreads();
                failed = failed || sh_fail != 0;
                // no cache invalidate: every band access is a device-scope atomic
            }
        };
        auto load_chunk_direct = [&](int64_t k) {
            const int64_t col0 = i0 + k * CH;
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int e = tid + q * NT;
                bool ok;
                C* p = chunk_ptr(col0, e, ok);
                if (e < CH * RS) win[(int)((col0 + e / RS) & (WC - 1)) * RS + e % RS] = ok ? ngld(p) : (C)0;
            }
        };
        auto flush_chunk = [&](int64_t k) {
            const int64_t col0 = i0 + k * CH;
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const int e = tid + q * NT;
                bool ok;
                C* p = chunk_ptr(col0, e, ok);
                if (ok) ngst(p, win[(int)((col0 + e / RS) & (WC - 1)) * RS + e % RS]);
            }
        };

        if (!failed) wait_prev(i0 + 2 * CH);
        if (!failed) {
            load_chunk_direct(0);
            if (nchunks > 1) load_chunk_direct(1);
        }
        __syncthreads();
        int64_t next_flush = 0;                            // first chunk not yet flushed
        for (int64_t g = 0; g < ngroups && !failed; ++g) {
            // chunk g+2 is requested now and lands in the window at the end of the group
            C pre[PER];
#ifdef SVB_CHASE_TIMING
            if (tid == 0) { tlast = wall_clock64(); ++ngrp; }
#endif
            const bool want = g + 2 < nchunks;
            if (want) wait_prev(i0 + (g + 3) * CH);
            if (failed) break;
            NMARK(0);
            if (want) {
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    bool ok;
                    C* p = chunk_ptr(i0 + (g + 2) * CH, tid + q * NT, ok);
                    pre[q] = ok ? ngld(p) : (C)0;
                }
            }
            for (int hp = 0; hp < GS; ++hp) {
                const int h = (int)g * 2 * GS + 2 * hp - 4 * slot;      // this sweep's half step (right, then left)
                narrow_super_step<C, D, WC, false>(win, vbuf, (int)my_i, h, have, (int)my_steps, (int)n);
                narrow_super_step<C, D, WC, true>(win, vbuf, (int)my_i, h + 1, have, (int)my_steps, (int)n);
            }
            NMARK(1);
            if (want) {
                const int64_t col0 = i0 + (g + 2) * CH;
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int e = tid + q * NT;
                    if (e < CH * RS) win[(int)((col0 + e / RS) & (WC - 1)) * RS + e % RS] = pre[q];
                }
            }
            NMARK(2);
            const int64_t f = g - LAGC;
            if (f >= 0 && f < nchunks) {
                flush_chunk(f);
                next_flush = f + 1;
                // the stores are device-scope atomics: once acknowledged (vmcnt = 0) they are
                // visible to every workgroup, no cache write-back is needed
                __builtin_amdgcn_s_waitcnt(0x0f70);
                __syncthreads();
                if (tid == 0)
                    __hip_atomic_store(&flushed[b], (int)min(i0 + (f + 1) * CH, (int64_t)kAllFlushed - 1),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
            NMARK(3);
        }
        if (!failed) {
            // everything that entered the window and has not been written back yet
            const int64_t last = min(nchunks, ngroups + 2);
            for (int64_t k = next_flush; k < last; ++k) flush_chunk(k);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        }
        __syncthreads();
        if (tid == 0) __hip_atomic_store(&flushed[b], kAllFlushed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
    }
#ifdef SVB_CHASE_TIMING
    if (tid == 0) {
        unsigned long long* acc = reinterpret_cast<unsigned long long*>(ctrl + 8);
        for (int q = 0; q < 4; ++q) atomicAdd(&acc[q], tacc[q]);
        atomicAdd(&acc[4], ngrp);
    }
#endif
#undef NMARK
}

__global__ __launch_bounds__(256) void narrow_clear_kernel(int* __restrict__ p, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0;
}

}  // namespace

// ctrl: 64 ints (ticket, error flag) followed by one flushed counter per bundle
size_t chase_narrow_workspace_bytes(int64_t n) { return (size_t)(64 + n / 8 + 8) * sizeof(int); }

template <typename C, int NW, int WC, int GS = 8>   // GS: super-steps per group (chunk = GS*D columns)
static int run_chase_narrow_nw(int64_t n, C* band, int64_t ldab, int64_t ku, int* ctrl, hipStream_t s)
{
    constexpr int D = 8;
    if (n < 3) return SVB_OK;
    const size_t smem = sizeof(C) * ((size_t)WC * 3 * D + (size_t)(NW / 4) * 4 * D);
    auto kern = chase_narrow_kernel<C, D, NW, WC, GS>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    const int64_t nbundles = (n - 2 + NW - 1) / NW;
    const int64_t count = 64 + nbundles + 1;
    int cb = (int)((count + 255) / 256);
    hipLaunchKernelGGL(narrow_clear_kernel, dim3(cb > 256 ? 256 : cb), dim3(256), 0, s, ctrl, count);
    const int grid = (int)min((int64_t)env_int("SVB_NARROW_GRID", 128), nbundles);
    const int spin_limit = env_int("SVB_CHASE_SPIN", 1 << 20);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 16), smem, s, band, ldab, ku, n, ctrl, ctrl + 64, spin_limit);
    return hipGetLastError() == hipSuccess ? SVB_OK : SVB_ERR_DEVICE;
}

template <typename C>
int run_chase_narrow(int64_t n, C* band, int64_t ldab, int64_t ku, int* ctrl, hipStream_t s)
{
    // Sweeps per bundle (four per wave) and super-steps per group.  A bundle follows its predecessor
    // by the chunks the window holds plus two, so the chain per sweep is shortest with as many sweeps
    // as the window takes and short groups; a group's fixed cost (flag, flush) sets the lower end.
    // Measured best: 48 sweeps in groups of 4 (f32, 1024-column window), 24 in groups of 4 (f64, 512).
    const int nw = env_int("SVB_NARROW_NW", sizeof(C) == 8 ? 24 : 48);
    const int gs = env_int("SVB_NARROW_GS", 4);
    if constexpr (sizeof(C) == 8) {
        if (nw == 16) return run_chase_narrow_nw<C, 16, 512>(n, band, ldab, ku, ctrl, s);
        return run_chase_narrow_nw<C, 24, 512, 4>(n, band, ldab, ku, ctrl, s);
    } else {
        if (nw == 16) return run_chase_narrow_nw<C, 16, 512>(n, band, ldab, ku, ctrl, s);
        if (nw == 32) return run_chase_narrow_nw<C, 32, 1024>(n, band, ldab, ku, ctrl, s);
        if (gs == 8) return run_chase_narrow_nw<C, 48, 1024>(n, band, ldab, ku, ctrl, s);
        return run_chase_narrow_nw<C, 48, 1024, 4>(n, band, ldab, ku, ctrl, s);
    }
}

template int run_chase_narrow<double>(int64_t, double*, int64_t, int64_t, int*, hipStream_t);
template int run_chase_narrow<float>(int64_t, float*, int64_t, int64_t, int*, hipStream_t);

}  // namespace svb
