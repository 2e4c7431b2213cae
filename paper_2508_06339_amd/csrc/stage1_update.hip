// Stage 1, trailing-matrix update (paper Section 3.1 Algorithm 1 lines 3/6,
// Section 3.2 "Trailing Submatrix Update", Algorithms 4 and 5).
//
// The paper applies the reflectors of a tile one at a time with scalar FMAs
// (Algorithm 5).  Here the reflectors of a whole domain are applied at once in
// compact-WY form: with Y = V T,
//     QR sweep:  C <- Q^T C = C - V (Y^T C)      (reflectors from the left)
//     LQ sweep:  C <- C Q   = C - (C Y) V^T      (reflectors from the right)
// i.e. two matrix products per domain: W = Y^T C (kernel K1), C -= V W
// (kernel K2).  Trailing-matrix element (p, q) lives at base + p*sp + q*sq;
// p runs along the panel direction, q along the free direction, so the LQ
// sweep is the QR sweep with (sp, sq) = (lda, 1) instead of (1, lda).
//
// A level's chunk ch covers panel rows ch*stride .. ch*stride + NB - 1
// (stride = NB at level 0, NB*g^L above: the rows that hold the R factors of
// the level below), and rows ch*NB .. of the level's V / Y panels.
#include <type_traits>

#include "svb_internal.h"
#include "mfma_gemm.h"

namespace svb {

// ------------------------------------------------------------------------
// Reference implementation with plain FMAs (selected with impl = 0; kept as
// the cross-check for the MFMA kernels).
// ------------------------------------------------------------------------
template <typename T, typename C, int NB, bool LQ>
__global__ __launch_bounds__(256) void k1_simple(const T* __restrict__ Cb, int64_t sp, int64_t sq,
                                                 int64_t qlen, const C* __restrict__ Y, int64_t ldp,
                                                 int chunks, int g, int64_t stride, C* __restrict__ W)
{
    constexpr int TQ = 64, TK = 32, PER = NB / 4;
    __shared__ C Ys[TK][NB + 1];
    __shared__ C Cs[TK][TQ + 1];
    const int d = blockIdx.y;
    const int64_t q0 = (int64_t)blockIdx.x * TQ;
    const int nch = min(g, chunks - d * g);
    const int t = threadIdx.x;
    const int q = t % TQ, grp = t / TQ;
    C acc[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) acc[u] = 0;
    for (int ch = 0; ch < nch; ++ch) {
        const int64_t chg = (int64_t)d * g + ch;
        for (int a0 = 0; a0 < NB; a0 += TK) {
            for (int idx = t; idx < TK * NB; idx += 256) {
                const int a = idx % TK, kk = idx / TK;
                Ys[a][kk] = Y[(chg * NB + a0 + a) + (int64_t)kk * ldp];
            }
            for (int idx = t; idx < TK * TQ; idx += 256) {
                int a, qq;
                if (LQ) { qq = idx % TQ; a = idx / TQ; } else { a = idx % TK; qq = idx / TK; }
                const int64_t p = chg * stride + a0 + a;
                C v = 0;
                if (q0 + qq < qlen) v = ld_as<C, T>(&Cb[p * sp + (q0 + qq) * sq]);
                Cs[a][qq] = v;
            }
            __syncthreads();
#pragma unroll 4
            for (int a = 0; a < TK; ++a) {
                const C c = Cs[a][q];
#pragma unroll
                for (int u = 0; u < PER; ++u) acc[u] += Ys[a][grp * PER + u] * c;
            }
            __syncthreads();
        }
    }
    if (q0 + q < qlen) {
        C* Wd = W + (int64_t)d * NB * qlen;
#pragma unroll
        for (int u = 0; u < PER; ++u) Wd[(grp * PER + u) + (q0 + q) * NB] = acc[u];
    }
}

template <typename T, typename C, int NB, bool LQ>
__global__ __launch_bounds__(256) void k2_simple(T* __restrict__ Cb, int64_t sp, int64_t sq,
                                                 int64_t qlen, const C* __restrict__ V, int64_t ldp,
                                                 int g, int64_t stride, const C* __restrict__ W)
{
    constexpr int TQ = 32, TK = 16, PER = NB / 8;
    __shared__ C Vs[TK][NB + 1];
    __shared__ C Ws[TK][TQ + 1];
    __shared__ C Os[NB][TQ + 1];
    const int64_t chg = blockIdx.y;
    const int d = (int)(chg / g);
    const int64_t q0 = (int64_t)blockIdx.x * TQ;
    const int t = threadIdx.x;
    const int q = t % TQ, grp = t / TQ;
    const C* Wd = W + (int64_t)d * NB * qlen;
    C acc[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) acc[u] = 0;
    for (int k0 = 0; k0 < NB; k0 += TK) {
        for (int idx = t; idx < TK * NB; idx += 256) {
            const int a = idx % NB, kk = idx / NB;
            Vs[kk][a] = V[(chg * NB + a) + (int64_t)(k0 + kk) * ldp];
        }
        for (int idx = t; idx < TK * TQ; idx += 256) {
            const int kk = idx % TK, qq = idx / TK;
            Ws[kk][qq] = (q0 + qq < qlen) ? Wd[(k0 + kk) + (q0 + qq) * NB] : (C)0;
        }
        __syncthreads();
#pragma unroll 4
        for (int kk = 0; kk < TK; ++kk) {
            const C w = Ws[kk][q];
#pragma unroll
            for (int u = 0; u < PER; ++u) acc[u] += Vs[kk][grp * PER + u] * w;
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) Os[grp * PER + u][q] = acc[u];
    __syncthreads();
    for (int idx = t; idx < NB * TQ; idx += 256) {
        int a, qq;
        if (LQ) { qq = idx % TQ; a = idx / TQ; } else { a = idx % NB; qq = idx / NB; }
        if (q0 + qq < qlen) {
            T* ptr = &Cb[(chg * stride + a) * sp + (q0 + qq) * sq];
            st_as<T, C>(ptr, ld_as<C, T>(ptr) - Os[a][qq]);
        }
    }
}

template <typename T, typename C, int NB, bool LQ>
static void update_simple(T* Cb, int64_t lda, int64_t qlen, const C* V, const C* Y, int64_t ldp,
                          int chunks, int g, int64_t stride, C* W, bool credited, hipStream_t s)
{
    // algorithmic work of one product: 2*rows*NB*cols flops; the matrix block is read once
    // by K1 and read + written by K2.  Levels above 0 are overhead of the tree: not credited.
    const double fl = credited ? 2.0 * chunks * NB * (double)NB * (double)qlen : 0.0;
    const double by = credited ? (double)chunks * NB * (double)qlen * sizeof(T) : 0.0;
    const int64_t sp = LQ ? lda : 1, sq = LQ ? 1 : lda;
    const int domains = (chunks + g - 1) / g;
    dim3 g1((unsigned)((qlen + 63) / 64), (unsigned)domains);
    prof_begin(SVB_PROF_K1, s, fl, by);
    hipLaunchKernelGGL((k1_simple<T, C, NB, LQ>), g1, dim3(256), 0, s, Cb, sp, sq, qlen, Y, ldp,
                       chunks, g, stride, W);
    prof_end(s);
    dim3 g2((unsigned)((qlen + 31) / 32), (unsigned)chunks);
    prof_begin(SVB_PROF_K2, s, fl, 2.0 * by);
    hipLaunchKernelGGL((k2_simple<T, C, NB, LQ>), g2, dim3(256), 0, s, Cb, sp, sq, qlen, V, ldp, g,
                       stride, W);
    prof_end(s);
}

// ------------------------------------------------------------------------
// MFMA implementation.
//
// One workgroup of 4 waves computes a TM x TN tile D = A_op * B_op with
// v_mfma_f32_32x32x2_f32 (f32 arithmetic) or v_mfma_f64_16x16x4_f64 (f64).
// Both operands are staged through LDS in k-major order (Xs[k][mn], row
// length odd), TK = 128 bytes of k per stage; the next stage's global loads
// are issued into registers before the current stage's MFMAs.  Tile roles
// are chosen so that the lanes of an accumulator register run along the
// direction in which the trailing matrix is contiguous in memory:
//   K1, both sweeps : D[q][kk] = sum_p C(p,q) Y(p,kk)     -> W[kk + q*NB]
//   K2, QR sweep    : D[q][p]  = sum_kk W(kk,q) V(p,kk)   -> C(p,q) -= D
//   K2, LQ sweep    : D[p][q]  = sum_kk V(p,kk) W(kk,q)   -> C(p,q) -= D
// ------------------------------------------------------------------------
// K1: D[q][kk] = sum over the domain's rows p of C(p,q) * Y(p,kk)
template <typename T, typename C, int NB, bool LQ>
struct K1Pol : TileShape<NB, false> {
    static constexpr bool A_KC = !LQ, B_KC = true, RMW = false;
    typedef T TA; typedef C TB; typedef C TD;
    static constexpr int TK = 128 / (int)sizeof(C);
    static constexpr int KPC = NB / TK;  // k-tiles per chunk
    const T* Cb; int64_t sp, sq, qlen, q0; const C* Y; int64_t ldp; int64_t ch0; int nch; int64_t stride; C* Wd;
    __device__ __forceinline__ int ktiles() const { return nch * KPC; }
    __device__ __forceinline__ const T* ptrA(int mn, int kt, int k) const
    {
        const int64_t q = q0 + mn;
        if (q >= qlen) return nullptr;
        const int64_t p = (ch0 + kt / KPC) * stride + (kt % KPC) * TK + k;
        return &Cb[p * sp + q * sq];
    }
    __device__ __forceinline__ const C* ptrB(int mn, int kt, int k) const
    {
        const int64_t row = (ch0 + kt / KPC) * NB + (kt % KPC) * TK + k;
        return &Y[row + (int64_t)mn * ldp];
    }
    __device__ __forceinline__ C* ptrD(int m, int n) const
    {
        const int64_t q = q0 + m;
        return q < qlen ? &Wd[n + q * NB] : nullptr;
    }
};

template <typename T, typename C, int NB, bool LQ>
__global__ __launch_bounds__(256) void k1_mfma(const T* __restrict__ Cb, int64_t sp, int64_t sq,
                                               int64_t qlen, const C* __restrict__ Y, int64_t ldp,
                                               int chunks, int g, int64_t stride, C* __restrict__ W)
{
    const int d = blockIdx.y;
    K1Pol<T, C, NB, LQ> pol;
    pol.Cb = Cb; pol.sp = sp; pol.sq = sq; pol.qlen = qlen; pol.q0 = (int64_t)blockIdx.x * 128;
    pol.Y = Y; pol.ldp = ldp; pol.ch0 = (int64_t)d * g; pol.nch = min(g, chunks - d * g);
    pol.stride = stride; pol.Wd = W + (int64_t)d * NB * qlen;
    gemm_tile<C>(pol);
}

// K2, QR sweep: D[q][p] = sum_kk W(kk,q) V(p,kk);  C(p,q) -= D
template <typename T, typename C, int NB>
struct K2QrPol : TileShape<NB, false> {
    static constexpr bool A_KC = true, B_KC = false, RMW = true;
    typedef C TA; typedef C TB; typedef T TD;
    static constexpr int TK = 128 / (int)sizeof(C);
    T* Cb; int64_t sp, sq, qlen, q0; const C* V; int64_t ldp; int64_t ch; int64_t stride; const C* Wd;
    __device__ __forceinline__ int ktiles() const { return NB / TK; }
    __device__ __forceinline__ const C* ptrA(int mn, int kt, int k) const
    {
        const int64_t q = q0 + mn;
        return q < qlen ? &Wd[(kt * TK + k) + q * NB] : nullptr;
    }
    __device__ __forceinline__ const C* ptrB(int mn, int kt, int k) const
    {
        return &V[(ch * NB + mn) + (int64_t)(kt * TK + k) * ldp];
    }
    __device__ __forceinline__ T* ptrD(int m, int n) const
    {
        const int64_t q = q0 + m;
        return q < qlen ? &Cb[(ch * stride + n) * sp + q * sq] : nullptr;
    }
};

// K2, LQ sweep: D[p][q] = sum_kk V(p,kk) W(kk,q);  C(p,q) -= D
template <typename T, typename C, int NB>
struct K2LqPol : TileShape<NB, true> {
    static constexpr bool A_KC = false, B_KC = true, RMW = true;
    typedef C TA; typedef C TB; typedef T TD;
    static constexpr int TK = 128 / (int)sizeof(C);
    T* Cb; int64_t sp, sq, qlen, q0; const C* V; int64_t ldp; int64_t ch; int64_t stride; const C* Wd;
    __device__ __forceinline__ int ktiles() const { return NB / TK; }
    __device__ __forceinline__ const C* ptrA(int mn, int kt, int k) const
    {
        return &V[(ch * NB + mn) + (int64_t)(kt * TK + k) * ldp];
    }
    __device__ __forceinline__ const C* ptrB(int mn, int kt, int k) const
    {
        const int64_t q = q0 + mn;
        return q < qlen ? &Wd[(kt * TK + k) + q * NB] : nullptr;
    }
    __device__ __forceinline__ T* ptrD(int m, int n) const
    {
        const int64_t q = q0 + n;
        return q < qlen ? &Cb[(ch * stride + m) * sp + q * sq] : nullptr;
    }
};

template <typename T, typename C, int NB, bool LQ>
__global__ __launch_bounds__(256) void k2_mfma(T* __restrict__ Cb, int64_t sp, int64_t sq, int64_t qlen,
                                               const C* __restrict__ V, int64_t ldp, int g,
                                               int64_t stride, const C* __restrict__ W, int sel)
{
    // sel 0: every chunk; 1: the first chunk of every domain (the rows the next panel and
    // the next tree level read); 2: all the others
    const int64_t y = blockIdx.y;
    const int64_t ch = sel == 0 ? y : (sel == 1 ? y * g : (y / (g - 1)) * g + 1 + y % (g - 1));
    typename std::conditional<LQ, K2LqPol<T, C, NB>, K2QrPol<T, C, NB>>::type pol;
    pol.Cb = Cb; pol.sp = sp; pol.sq = sq; pol.qlen = qlen; pol.q0 = (int64_t)blockIdx.x * 128;
    pol.V = V; pol.ldp = ldp; pol.ch = ch; pol.stride = stride;
    pol.Wd = W + (ch / g) * (int64_t)NB * qlen;
    gemm_tile<C>(pol);
}

template <typename T, typename C, int NB, bool LQ>
static void update_mfma(T* Cb, int64_t lda, int64_t qlen, const C* V, const C* Y, int64_t ldp,
                        int chunks, int g, int64_t stride, C* W, bool credited, int phase, hipStream_t s)
{
    const int64_t sp = LQ ? lda : 1, sq = LQ ? 1 : lda;
    const int domains = (chunks + g - 1) / g;
    const double fl = credited ? 2.0 * chunks * NB * (double)NB * (double)qlen : 0.0;
    const double by = credited ? (double)chunks * NB * (double)qlen * sizeof(T) : 0.0;
    const unsigned qt = (unsigned)((qlen + 127) / 128);
    if (phase != 2) {
        prof_begin(SVB_PROF_K1, s, fl, by);
        hipLaunchKernelGGL((k1_mfma<T, C, NB, LQ>), dim3(qt, (unsigned)domains), dim3(256), 0, s, Cb, sp, sq,
                           qlen, Y, ldp, chunks, g, stride, W);
        prof_end(s);
    }
    // phase 0: all of K2; 1: first chunks only; 2: the remaining chunks
    const int ny = phase == 0 ? chunks : (phase == 1 ? domains : chunks - domains);
    if (ny > 0) {
        const double share = (double)ny / chunks;
        prof_begin(SVB_PROF_K2, s, fl * share, 2.0 * by * share);
        hipLaunchKernelGGL((k2_mfma<T, C, NB, LQ>), dim3(qt, (unsigned)ny), dim3(256), 0, s, Cb, sp, sq,
                           qlen, V, ldp, g, stride, W, phase);
        prof_end(s);
    }
}

template <typename T, typename C, int NB>
static void update_nb(bool lq, T* Cb, int64_t lda, int64_t qlen, const C* V, const C* Y,
                      int64_t ldp, int chunks, int g, int64_t stride, C* W, int impl, bool credited,
                      int phase, hipStream_t s)
{
    if (impl == 0) {
        if (phase == 2) return;  // the plain kernels always do all of K2 in phase 0 / 1
        if (lq) update_simple<T, C, NB, true>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, W, credited, s);
        else update_simple<T, C, NB, false>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, W, credited, s);
    } else {
        if (lq) update_mfma<T, C, NB, true>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, W, credited, phase, s);
        else update_mfma<T, C, NB, false>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, W, credited, phase, s);
    }
}

template <typename T, typename C>
void launch_update(int nb, bool lq, T* Cbase, int64_t lda, int64_t qlen, const C* V, const C* Y,
                   int64_t ldp, int chunks, int g, int64_t stride, C* W, int impl, bool credited,
                   int phase, hipStream_t s)
{
    if (qlen <= 0) return;
    switch (nb) {
    case 32: update_nb<T, C, 32>(lq, Cbase, lda, qlen, V, Y, ldp, chunks, g, stride, W, impl, credited, phase, s); break;
    case 64: update_nb<T, C, 64>(lq, Cbase, lda, qlen, V, Y, ldp, chunks, g, stride, W, impl, credited, phase, s); break;
    default: update_nb<T, C, 128>(lq, Cbase, lda, qlen, V, Y, ldp, chunks, g, stride, W, impl, credited, phase, s); break;
    }
}

template void launch_update<double, double>(int, bool, double*, int64_t, int64_t, const double*, const double*, int64_t, int, int, int64_t, double*, int, bool, int, hipStream_t);
template void launch_update<float, float>(int, bool, float*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, float*, int, bool, int, hipStream_t);
template void launch_update<__half, float>(int, bool, __half*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, float*, int, bool, int, hipStream_t);

}  // namespace svb
