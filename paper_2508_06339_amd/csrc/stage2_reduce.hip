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
// with the following sweeps.  Sweeps are pipelined: one workgroup per sweep, sweeps drawn from a
// ticket counter, a progress counter per sweep, bounded waits (as in stage2_chase.hip).  Of the
// blocks step (s+1, t) brings in, the one right of Z was last written by the right half of step
// (s, t+2) (that step's upper block) and the next diagonal block by its left half (the corner it
// shares with that step's Z); progress is therefore published per block (upper block final /
// whole step final) and a sweep follows its predecessor a little over two steps behind.
//
// Per step the workgroup holds the upper block U (rows c0-B .., the previous step's A3) and Z
// stacked in LDS (2B x B); a step's Z is requested at its start and A3 at the start of the left
// panel, as late as the panel factorisations still hide the latency (every request waits for the
// predecessor sweep), and they take the place of Z and U once those have been written back, so
// every block is read once and written once per sweep.  One wave factors the panels while the
// others do that traffic.
//
// Packed band: entry (i,j) at band[(i - j + ku) + j*ldab], ku = 2B-1, ldab >= 3B.
#include "svb_internal.h"
#include "mfma_frag.h"

namespace svb {

namespace {

constexpr int kSweepDone = 0x7fffffff;

// Workgroup barrier that orders LDS traffic only: s_waitcnt lgkmcnt(0) (gfx9 encoding:
// vmcnt = 63, expcnt = 7, lgkmcnt = 0), then s_barrier.  __syncthreads() would also wait for
// every outstanding global load and store, i.e. for the block prefetches that are meant to
// stay in flight across the phases of a step; visibility of global data between workgroups
// is handled separately (stores_done below, fences at the ends of a sweep).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();
}
// Every band access of this kernel is a device-scope atomic (written through to, and read
// from, the level all compute dies share), so publishing a step needs no cache write-back and
// consuming one no invalidate: the writer only waits until its stores have been acknowledged
// (s_waitcnt vmcnt(0)) before the barrier that precedes the progress store, and the reader
// issues its loads after the barrier that follows the progress load.
__device__ __forceinline__ void stores_done()
{
    __builtin_amdgcn_s_waitcnt(0x0f70);
}

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
constexpr int kDppRor8 = 0x128;       // lane i <-> i^8 inside rows of 16 (rotate by 8)

// Sums of eight per-lane values over the 64 lanes of a wave, as wave-uniform scalars.
// The first three stages halve the number of values while doubling the lanes summed
// (each lane keeps the half selected by one of its index bits and hands the other half to
// its partner: partners i^7 with bit 2, i^1 with bit 0, i^2 with bit 1), so that after them
// lane i holds, summed over its group of eight lanes, the value with index
// 4*bit1(i) + 2*bit0(i) + bit2(i); two more stages sum over the row of 16 and over the four rows.
template <typename C> __device__ __forceinline__ void wave_sum8(const C (&a)[8], C (&out)[8])
{
    const int lane = threadIdx.x & (kWave - 1);
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
    C b[4], c[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const C keep = b2 ? a[2 * j + 1] : a[2 * j], send = b2 ? a[2 * j] : a[2 * j + 1];
        b[j] = keep + dpp_get<kDppHalfMirror>(send);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const C keep = b0 ? b[2 * j + 1] : b[2 * j], send = b0 ? b[2 * j] : b[2 * j + 1];
        c[j] = keep + dpp_get<kDppXor1>(send);
    }
    const C keep = b1 ? c[1] : c[0], send = b1 ? c[0] : c[1];
    C v = keep + dpp_get<kDppXor2>(send);
    v += dpp_get<kDppRor8>(v);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = lane_value(v, ((i >> 1) & 1) + 2 * ((i >> 2) & 1) + 4 * (i & 1));
}

__device__ __forceinline__ float rrcp(float x)
{
    // hardware reciprocal (1 ulp, biased) refined by one Newton step: a biased tau or scale
    // makes every reflector slightly non-orthogonal in the same direction, which adds up
    const float r = __builtin_amdgcn_rcpf(x);
    return fmaf(r, fmaf(-x, r, 1.0f), r);
}
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
// that T needs; the sums are wave-uniform scalars.  D = 8.
// With G the panel lies in the packed band in device memory (device-scope accesses, elements
// e >= ne outside the matrix: read as zero, not written).
template <typename C, int B, int D, bool G = false>
__device__ __forceinline__ void panel_wave(C* P, int64_t sk, int64_t se, C* Vs, C* Ts, int ne = B)
{
    constexpr int QN = (B + kWave - 1) / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    C x[D][QN];
#pragma unroll
    for (int k = 0; k < D; ++k)
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            const int e = lane + kWave * q;
            if (G) x[k][q] = (e < ne) ? rgld(P + k * sk + e * se) : (C)0;
            else x[k][q] = (e < B) ? P[k * sk + e * se] : (C)0;
        }
    const int tj = lane & (D - 1);   // this lane builds row tj of T as the reflectors appear
    C trow[D];
#pragma unroll
    for (int k = 0; k < D; ++k) {
        C part[D], p[D], colk[D];
#pragma unroll
        for (int j = 0; j < D; ++j) {
            C acc = 0;
#pragma unroll
            for (int q = 0; q < QN; ++q) {
                const int e = lane + kWave * q;
                acc += (e > k) ? x[j][q] * x[k][q] : (C)0;
            }
            part[j] = acc;
            colk[j] = lane_value(x[j][0], k);   // element k of every line
        }
        wave_sum8(part, p);
        const C alpha = colk[k], ss = p[k];
        C beta, inv, tau;
        if (ss == (C)0) {
            beta = alpha; tau = 0; inv = 0;
        } else {
            // (alpha and ss are the same in every lane: a uniform branch.  The refined hardware
            // square root wants a normal argument; sums near the underflow threshold take the
            // library routine.)
            const C x2 = alpha * alpha + ss;
            const C nrm = x2 < (sizeof(C) == 8 ? (C)1e-290 : (C)1e-30f) ? sqrt(x2) : newton_sqrt(x2);
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
                if (G) {
                    if (e < ne) rgst(P + k * sk + e * se, (e <= k) ? x[k][q] : (C)0);
                } else {
                    P[k * sk + e * se] = (e <= k) ? x[k][q] : (C)0;
                }
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

// The block reflector (Vs, Ts) applied to SIXTEEN lines at once on MFMA, by one wave: element e
// of line n of the tile lives at base[e*es + n*ls] (LDS), e < B, lines n >= nvalid are left
// alone.  With Y(e, n) the tile's elements:
//     P = V^T Y  (16 x 16, rows 8.. zero),  Z = -T^T P,  Y += V Z
// (line <- line - ((line . V) T) V^T for every line, the expression of apply_line).  The
// first product contracts over e with Y as the B operand straight from LDS; the second and
// third use the accumulator registers of the previous one as their B operand (Frag).
template <typename C, int B, int D>
__device__ __forceinline__ void apply_tile(C* base, int es, int ls, int nvalid, const C* Vs, const C* Ts)
{
    using F = Frag<C>;
    typedef typename F::acc_t acc_t;
    const int lane = threadIdx.x & 63, i = lane & 15, gq = lane >> 4;
    const bool valid = i < nvalid;
    C* mine = base + i * ls;   // this lane's line (B / accumulator operands)
    acc_t p0, p1;
#pragma unroll
    for (int r = 0; r < 4; ++r) { p0[r] = 0; p1[r] = 0; }
#pragma unroll 8
    for (int s4 = 0; s4 < B / 4; ++s4) {
        const int k = 4 * s4 + gq;
        const C a = (i < D) ? Vs[vidx<B, D>(k) + i] : (C)0;   // A[m = i][k] = V(k, i)
        const C b = valid ? mine[k * es] : (C)0;              // B[k][n = i] = Y(k, i)
        if (s4 & 1) p1 = F::mma(a, b, p1);
        else p0 = F::mma(a, b, p0);
    }
    acc_t z;
#pragma unroll
    for (int r = 0; r < 4; ++r) { p0[r] += p1[r]; z[r] = 0; }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int kk = F::roff(r, gq);
        const C a = (i < D && kk < D) ? Ts[kk * D + i] : (C)0;   // A[m = i][kk] = T(kk, i)
        z = F::mma(a, p0[r], z);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) z[r] = -z[r];
#pragma unroll 2
    for (int e0 = 0; e0 < B; e0 += 16) {
        acc_t y;
#pragma unroll
        for (int r = 0; r < 4; ++r) y[r] = valid ? mine[(e0 + F::roff(r, gq)) * es] : (C)0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = F::roff(r, gq);
            if (F::roff(r, 0) < D) {   // some lane group still has a reflector index below D in this slot
                const C a = (j < D) ? Vs[vidx<B, D>(e0 + i) + j] : (C)0;   // A[m = i][j] = V(e0 + i, j)
                y = F::mma(a, z[r], y);
            }
        }
        if (valid) {
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[(e0 + F::roff(r, gq)) * es] = y[r];
        }
    }
}

// The same for a line of the packed band in device memory (device-scope accesses): elements
// base[e*es], e < ne, eight lanes per line (an eighth of the line each, held in registers
// between the two passes).  With IL the eight lanes own interleaved elements (e = 8*jj + p),
// which keeps their accesses together when the line is contiguous in memory.
template <typename C, int B, int D, bool IL>
__device__ __forceinline__ void apply_line_g(C* base, int64_t es, bool valid, int ne, const C* Vs, const C* Ts)
{
    constexpr int SEG = B / 8;
    const int p = threadIdx.x & 7;
    C a[SEG];
    C w[D];
#pragma unroll
    for (int k = 0; k < D; ++k) w[k] = 0;
    if (valid) {
#pragma unroll
        for (int jj = 0; jj < SEG; ++jj) {
            const int e = IL ? 8 * jj + p : p * SEG + jj;
            a[jj] = (e < ne) ? rgld(base + e * es) : (C)0;
        }
#pragma unroll
        for (int jj = 0; jj < SEG; ++jj) {
            const int e = IL ? 8 * jj + p : p * SEG + jj;
            C v[D];
            load_v<D>(Vs + vidx<B, D>(e), v);
#pragma unroll
            for (int k = 0; k < D; ++k) w[k] += a[jj] * v[k];
        }
    }
#pragma unroll
    for (int k = 0; k < D; ++k) {
        w[k] = quad_allsum(w[k]);
        w[k] += dpp_get<kDppHalfMirror>(w[k]);   // the other quad of the eight
    }
    C z[D];
#pragma unroll
    for (int k = 0; k < D; ++k) {
        C acc = 0;
#pragma unroll
        for (int j = 0; j <= k; ++j) acc += w[j] * Ts[j * D + k];
        z[k] = acc;
    }
    if (valid) {
#pragma unroll
        for (int jj = 0; jj < SEG; ++jj) {
            const int e = IL ? 8 * jj + p : p * SEG + jj;
            C v[D];
            load_v<D>(Vs + vidx<B, D>(e), v);
            C x = a[jj];
#pragma unroll
            for (int k = 0; k < D; ++k) x -= z[k] * v[k];
            if (e < ne) rgst(base + e * es, x);
        }
    }
}

// threads of the band reduction kernel: 8*B apply threads (four per line of a 2B-line pass),
// plus one extra wave for the panels where that still fits in a workgroup.  Blocks are moved
// by "traffic" waves, each lane keeping one block row: a wave covers 64 consecutive rows of
// CPG columns at a time and steps through the columns with a fixed stride, so that its
// addresses are a scalar base, advanced by a scalar per step, plus a fixed lane offset.
template <int B> struct ReduceShape {
    static constexpr bool EXTRA = 8 * B + kWave <= 1024;
    static constexpr int NT = EXTRA ? 8 * B + kWave : 8 * B;
    static constexpr int NWV = NT / kWave;
    static constexpr int PWV = EXTRA ? NWV - 1 : 0;               // the panel wave
    static constexpr int GPC = B >= kWave ? B / kWave : 1;        // 64-row groups per block column
    static constexpr int CPG = B >= kWave ? 1 : kWave / B;        // block columns per wave access
    static constexpr int NTW = (NWV - 1) / GPC * GPC;             // waves that move blocks
    static constexpr int JS = NTW / GPC * CPG;                    // column step of a traffic wave
    static constexpr int PER = (B + JS - 1) / JS;                 // accesses per traffic wave and block
};

// UG: only the diagonal block Z lives in LDS; the upper block U and the block right of Z are
// transformed where they lie, in the packed band in device memory (for element types of which
// two B x B blocks do not fit in LDS).
template <typename C, int B, int D, bool UG = false>
__global__ __launch_bounds__(ReduceShape<B>::NT) void band_reduce_kernel(C* __restrict__ band, int64_t ldab, int64_t n,
                                                                        int* __restrict__ ctrl,
                                                                        int* __restrict__ progress, int spin_limit)
{
    // The panel wave draws the sweep, waits for the predecessor, factors the two panels of a
    // step and publishes progress.  The traffic waves move the blocks between device memory
    // and LDS.  The panel wave's work overlaps the traffic: the right panel of step t with the
    // write-back of Z of step t-1, the left panel with the write-back of U.
    using SH = ReduceShape<B>;
    constexpr int LD = UG ? B + 1 : 2 * B + 1, PER = SH::PER, JS = SH::JS;
    constexpr int ZO = UG ? 0 : B;                // first row of Z inside S
    // block reflectors onto LDS lines: sixteen lines per wave on MFMA in f64 (half the FMA rate and
    // twice the LDS traffic of f32 make the line-per-quad form slow there), a line per quad in f32
    constexpr bool kTile = sizeof(C) == 8;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C* S = reinterpret_cast<C*>(smem_raw);        // rows c0-B .. c0+B-1 (UG: c0 ..), columns c0 .. c0+B-1: S[row + col*LD]
    C* Vs = S + ((B * LD + 3) & ~3);              // (B + 4) * D
    C* Ts = Vs + (B + 4) * D;                     // D * D
    __shared__ int sh_s, sh_fail, sh_back;   // sh_back: traffic waves whose stores of a block have been acknowledged
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave-uniform: scalar branches below
    const bool pw = wv == SH::PWV;
    const bool lead = tid == SH::PWV * kWave;                      // first lane of the panel wave
    const int tw = SH::EXTRA ? wv : wv - 1;                        // index among the traffic waves
    const bool traffic = !pw && tw < SH::NTW;
    const bool applies = tid < 8 * B;
    const int line = (tid >> 6) * 16 + (lane >> 2);                // line of the apply phases
    // this lane's block row and first block column
    const int ii = (tw % SH::GPC) * kWave + (B >= kWave ? lane : lane % B);
    const int jj0 = (tw / SH::GPC) * SH::CPG + (B >= kWave ? 0 : lane / B);
    const int ldm1 = (int)(ldab - 1);
    const int64_t ku = 2 * (int64_t)B - 1;
#ifdef SVB_CHASE_TIMING
    unsigned long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, tlast = 0, nstep_acc = 0;
#define RMARK(slot_) do { if (lead) { unsigned long long now_ = wall_clock64(); tacc[slot_] += now_ - tlast; tlast = now_; } } while (0)
#else
#define RMARK(slot_) do { } while (0)
#endif
    const int64_t nsweeps = (n - 1) / D;

    // A B x B block of the band whose first element is entry (r0, cb): this lane's first
    // element of it, and the numbers of its rows and columns that lie inside the matrix.
    struct Blk { C* p; int nrow, ncol; };
    auto block_at = [&](int64_t r0, int64_t cb) -> Blk {
        Blk k;
        k.p = band + ((r0 - cb + ku) + cb * ldab) + (ii + (int64_t)jj0 * ldm1);
        k.nrow = (int)max((int64_t)0, min((int64_t)B, n - r0));
        k.ncol = (int)max((int64_t)0, min((int64_t)B, n - cb));
        return k;
    };
    // access q of a block: element (ii, jj0 + q*JS), at k.p + q*JS*ldm1 in the band and at
    // lds0 + q*JS*LD in LDS; loads of elements outside the matrix read the band's first entry
    // and are masked where the value is consumed (masking at once would wait for the load)
    auto inside = [&](const Blk& k, int q) -> bool { return ii < k.nrow && jj0 + q * JS < k.ncol; };
    auto gload = [&](const Blk& k, int q, bool also) -> C {
        const C* p = (inside(k, q) && also) ? k.p + (int64_t)(q * JS) * ldm1 : band;
        return rgld(p);
    };
    auto gstore = [&](const Blk& k, int q, C v) { rgst(k.p + (int64_t)(q * JS) * ldm1, v); };
    // Progress of a sweep: 2k+1 once the upper block U of its step k is final in the band (and
    // every block of the steps before), 2k+2 once all blocks of step k are.
    // poll: the predecessor's progress, requested ahead of the work it is checked after;
    // wait_for: waits (one lane) until sweep s-1 has reached `need`, `seen` being an earlier
    // poll; an expired wait sets sh_fail
    auto poll = [&](int64_t s) -> int {
        return (lead && s > 0) ? __hip_atomic_load(&progress[s - 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
    };
    auto publish = [&](int64_t s, int value) {
        if (lead) __hip_atomic_store(&progress[s], value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    auto wait_for = [&](int64_t s, int need, int seen) {
        if (lead && s > 0 && seen < need) {
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
    };

    // A block written back by the traffic waves is published by the last of them to have its
    // stores acknowledged, not by the panel wave at the next barrier, which comes up to a
    // panel factorisation later: the successor sweep is waiting for exactly this.
    auto block_back = [&](int64_t s, int value) {
        stores_done();
        if (lane == 0) {
            const int arrived = atomicAdd(&sh_back, 1);
            if (arrived == SH::NTW - 1) {
                sh_back = 0;
                __hip_atomic_store(&progress[s], value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    };

    // Every single-lane section is followed by a barrier before the next one (no divergent
    // region spans a loop back-edge).
    for (;;) {
        if (lead) {
            sh_s = atomicAdd(&ctrl[0], 1);
            sh_fail = __hip_atomic_load(&ctrl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sh_back = 0;
        }
        __syncthreads();
        const int64_t s = sh_s;
        __syncthreads();
        if (s >= nsweeps) break;
        const int64_t c00 = (s + 1) * D;
        const int nsteps = (int)((n - 1 - c00) / B) + 1;
#ifdef SVB_CHASE_TIMING
        if (lead) tlast = wall_clock64();
#endif
        // ---- prologue: the sweep's own D rows and the first diagonal block, straight into LDS
        // (the first diagonal block was last touched by the predecessor's step 1)
        wait_for(s, 4, 0);
        __syncthreads();
        bool failed = sh_fail != 0;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        C pre[PER];   // traffic waves: A3 of the step, then Z of the next one
        if (!failed && traffic) {
            C u0[PER];
            const Blk ub = block_at(c00 - B, c00), zb = block_at(c00, c00);
            const int lds0 = ii + jj0 * LD;
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                if (!UG) u0[q] = gload(ub, q, ii >= B - D);
                pre[q] = gload(zb, q, true);
            }
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                if (jj0 + q * JS < B) {
                    if (!UG) S[lds0 + q * JS * LD] = (inside(ub, q) && ii >= B - D) ? u0[q] : (C)0;
                    S[ZO + lds0 + q * JS * LD] = inside(zb, q) ? pre[q] : (C)0;
                }
            }
        }
        __syncthreads();
        RMARK(7);
        int seen_next = 0;   // the predecessor's progress as polled during the previous step's last phase
        for (int t = 0; t < nsteps && !failed; ++t) {
            const int64_t c0 = c00 + (int64_t)t * B;
            const int xoff = (t == 0) ? B - D : 0;
            // opaque per-step copy: without it every LDS index below is hoisted out of the step
            // loop and held in (spilled) registers
            int lds0 = ii + jj0 * LD;
            asm volatile("" : "+v"(lds0));
#ifdef SVB_CHASE_TIMING
            if (lead) { tlast = wall_clock64(); ++nstep_acc; }
#endif
            if (t > 0) {
                // this step's Z (requested in S1) has a corner that the left half of the predecessor's
                // step t+1 wrote
                wait_for(s, 2 * t + 4, seen_next);
                lds_barrier();
                failed = sh_fail != 0;
                if (failed) break;
            }
            // ---- S1: right panel (LQ of X)  ||  Z of the previous step back, this step's Z in
            const int ncol = (int)min((int64_t)B, n - c0);                            // columns c0 .. inside the matrix
            const int64_t rho = (t == 0) ? c00 - D : c0 - B;                          // first row of X
            if (pw) {
                if (UG) panel_wave<C, B, D, true>(band + (rho - c0 + ku) + c0 * ldab, 1, ldm1, Vs, Ts, ncol);
                else panel_wave<C, B, D>(S + xoff, 1, LD, Vs, Ts);
            } else if (UG && traffic && t > 0) {
                // this step's Z is requested here (its registers would otherwise be live across the
                // in-band applies, which need theirs), the previous Z goes back meanwhile
                const Blk zp = block_at(c0 - B, c0 - B), zc = block_at(c0, c0);
#pragma unroll
                for (int q = 0; q < PER; ++q) pre[q] = gload(zc, q, true);
#pragma unroll
                for (int q = 0; q < PER; ++q)
                    if (inside(zp, q)) gstore(zp, q, S[lds0 + q * JS * LD]);
                // every block of step t-1 is final (the in-band stores of its last phase were
                // acknowledged before that phase's barrier)
                block_back(s, 2 * t);
#pragma unroll
                for (int q = 0; q < PER; ++q)
                    if (jj0 + q * JS < B) S[lds0 + q * JS * LD] = inside(zc, q) ? pre[q] : (C)0;
            } else if (traffic && t > 0) {
                // this step's Z is requested, the previous one goes back from LDS meanwhile and is
                // published, then the new one takes its place
                const Blk zp = block_at(c0 - B, c0 - B), zc = block_at(c0, c0);
#pragma unroll
                for (int q = 0; q < PER; ++q) pre[q] = gload(zc, q, true);
#pragma unroll
                for (int q = 0; q < PER; ++q)
                    if (inside(zp, q)) gstore(zp, q, S[ZO + lds0 + q * JS * LD]);
                block_back(s, 2 * t);   // every block of step t-1 is final
#pragma unroll
                for (int q = 0; q < PER; ++q)
                    if (jj0 + q * JS < B) S[ZO + lds0 + q * JS * LD] = inside(zc, q) ? pre[q] : (C)0;
            }
            RMARK(0);
            // UG: every wave's band stores of the previous step (and the panel's) are acknowledged
            // before the barrier that precedes the progress store
            if (UG) stores_done();
            lds_barrier();
            RMARK(1);
            RMARK(2);
            // ---- S3: block reflector onto the rows below X
            const int seen3 = UG ? 0 : poll(s);
            if (UG) {
                // (waves 0 .. 7: the rows of Z, in LDS, four lanes per line; waves 8 .. 15: rows D .. B-1
                // of U, in the band, eight lanes per line, two rounds; none in the first step, whose X
                // is the sweep's own rows)
                if (line < B) {
                    if (kTile) apply_tile<C, B, D>(S + 16 * wv, LD, 1, 16, Vs, Ts);
                    else apply_line<C, B, D>(S + line, LD, true, Vs, Ts);
                } else if (t > 0) {
#pragma unroll 1
                    for (int rd = 0; rd < 2; ++rd) {
                        const int row = D + rd * (B / 2) + (wv - 8) * 8 + (lane >> 3);
                        apply_line_g<C, B, D, false>(band + ((c0 - B + row) - c0 + ku) + c0 * ldab, ldm1,
                                                     row < B, ncol, Vs, Ts);
                    }
                    stores_done();
                }
            } else if (applies && kTile) {
                // sixteen rows per wave, from row xoff + D on
                const int row0 = xoff + D + 16 * wv;
                if (row0 < 2 * B) apply_tile<C, B, D>(S + row0, LD, 1, 2 * B - row0, Vs, Ts);
            } else if (applies) {
                const int row = xoff + D + line;
                apply_line<C, B, D>(S + row, LD, row < 2 * B, Vs, Ts);
            }
            lds_barrier();
            RMARK(3);
            if (UG) {
                publish(s, 2 * t + 1);   // U was transformed where it lies; the stores are acknowledged
            } else {
                // the block right of Z (requested in S4) was last touched by the right half of the
                // predecessor's step t+2, whose result is that step's upper block
                wait_for(s, 2 * t + 5, seen3);
                lds_barrier();
                failed = sh_fail != 0;
                if (failed) break;
            }
            // ---- S4: left panel (QR of Z's first D columns)  ||  A3 requested, U back, A3 in
            const int seen2 = UG ? poll(s) : 0;
            if (pw) {
                panel_wave<C, B, D>(S + ZO, LD, 1, Vs, Ts);
            } else if (!UG && traffic) {
                const Blk ub = block_at(c0 - B, c0), a3 = block_at(c0, c0 + B);
#pragma unroll
                for (int q = 0; q < PER; ++q) pre[q] = gload(a3, q, true);
#pragma unroll
                for (int q = 0; q < PER; ++q)
                    if (inside(ub, q) && ii >= xoff) gstore(ub, q, S[lds0 + q * JS * LD]);
                block_back(s, 2 * t + 1);   // U is final
#pragma unroll
                for (int q = 0; q < PER; ++q)
                    if (jj0 + q * JS < B) S[lds0 + q * JS * LD] = inside(a3, q) ? pre[q] : (C)0;
            }
            RMARK(4);
            lds_barrier();
            if (UG) {
                // the block right of Z (transformed where it lies in S5) was last touched by the right
                // half of the predecessor's step t+2, whose result is that step's upper block
                wait_for(s, 2 * t + 5, seen2);
                lds_barrier();
                failed = sh_fail != 0;
                if (failed) break;
            }
            RMARK(5);
            seen_next = poll(s);
            // ---- S5: block reflector onto the other columns of Z and onto A3
            if (UG) {
                // lines 0 .. B-1: columns D .. B-1 of Z, in LDS; lines B .. 2B-1: the columns of the
                // block right of Z, in the band
                if (line < B) {
                    if (kTile) apply_tile<C, B, D>(S + (D + 16 * wv) * LD, 1, LD, B - D - 16 * wv, Vs, Ts);
                    else apply_line<C, B, D>(S + (D + line) * LD, 1, line < B - D, Vs, Ts);
                } else {
                    const int nrow = (int)min((int64_t)B, n - c0);
#pragma unroll 1
                    for (int rd = 0; rd < 2; ++rd) {
                        const int64_t cg = c0 + B + rd * (B / 2) + (wv - 8) * 8 + (lane >> 3);
                        apply_line_g<C, B, D, true>(band + (c0 - cg + ku) + cg * ldab, 1, cg < n, nrow, Vs, Ts);
                    }
                    stores_done();
                }
            } else if (applies && kTile) {
                // waves 0 .. B/16-1: sixteen columns of Z each, from column D on; the others:
                // sixteen columns of the block right of Z each
                if (wv < B / 16) apply_tile<C, B, D>(S + B + (D + 16 * wv) * LD, 1, LD, B - D - 16 * wv, Vs, Ts);
                else apply_tile<C, B, D>(S + 16 * (wv - B / 16) * LD, 1, LD, 16, Vs, Ts);
            } else if (applies) {
                const bool valid = line < 2 * B - D;
                C* base = (line < B - D) ? S + B + (D + line) * LD : S + (line - (B - D)) * LD;
                apply_line<C, B, D>(base, 1, valid, Vs, Ts);
            }
            lds_barrier();
            RMARK(6);
        }
        // ---- epilogue: the last step's Z back (nothing is right of it)
        if (!failed && traffic) {
            const int64_t c0 = c00 + (int64_t)(nsteps - 1) * B;
            const Blk zl = block_at(c0, c0);
            const int lds0 = ii + jj0 * LD;
#pragma unroll
            for (int q = 0; q < PER; ++q)
                if (inside(zl, q)) gstore(zl, q, S[ZO + lds0 + q * JS * LD]);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        }
        __syncthreads();
        if (lead) __hip_atomic_store(&progress[s], kSweepDone, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
    }
#ifdef SVB_CHASE_TIMING
    if (lead) {
        unsigned long long* acc = reinterpret_cast<unsigned long long*>(ctrl + 8);
        for (int q = 0; q < 8; ++q) atomicAdd(&acc[q], tacc[q]);
        atomicAdd(&acc[8], nstep_acc);
    }
#endif
#undef RMARK
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
    // two blocks in LDS where they fit, otherwise only the diagonal block
    constexpr bool UG = sizeof(C) * (size_t)(((B * (2 * B + 1) + 3) & ~3) + (B + 4) * D + D * D) > 160 * 1024;
    constexpr int LD = UG ? B + 1 : 2 * B + 1;
    constexpr size_t smem = sizeof(C) * (size_t)(((B * LD + 3) & ~3) + (B + 4) * D + D * D);
    static_assert(smem <= 160 * 1024, "diagonal block does not fit in LDS");
    static_assert(!UG || ReduceShape<B>::NT == 1024, "one-block form: waves 0-7 on LDS lines, waves 8-15 on band lines");
    auto kern = band_reduce_kernel<C, B, D, UG>;
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
    hipLaunchKernelGGL(kern, dim3(grid), dim3(ReduceShape<B>::NT), smem, s, band, ldab, n, ctrl, ctrl + 64, spin_limit);
    return hipGetLastError() == hipSuccess ? SVB_OK : SVB_ERR_DEVICE;
}

}  // namespace

// ctrl: 64 ints (ticket, error flag, timing slots) followed by one progress counter per block sweep
size_t band_reduce_workspace_bytes(int64_t n) { return (size_t)((64 + n / 8 + 8) * 4 + 255) / 256 * 256; }

bool band_reduce_supported(int nb, size_t elem_size)
{
    (void)elem_size;
    return nb == 32 || nb == 64 || nb == 128;
}

template <typename C>
int run_band_reduce(int64_t n, int nb, C* band, int64_t ldab, int* ctrl, hipStream_t s)
{
    if (nb == 32) return launch_band_reduce<C, 32>(n, band, ldab, ctrl, s);
    if (nb == 64) return launch_band_reduce<C, 64>(n, band, ldab, ctrl, s);
    if (nb == 128) return launch_band_reduce<C, 128>(n, band, ldab, ctrl, s);
    return SVB_ERR_UNSUPPORTED;
}

template int run_band_reduce<double>(int64_t, int, double*, int64_t, int*, hipStream_t);
template int run_band_reduce<float>(int64_t, int, float*, int64_t, int*, hipStream_t);

}  // namespace svb
