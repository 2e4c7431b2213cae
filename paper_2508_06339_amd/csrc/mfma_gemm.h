// Workgroup-level matrix product on MFMA, shared by the trailing update and
// the panel's Y = V T product.  gfx950, 4 waves per workgroup.
#pragma once

#include "svb_internal.h"

namespace svb {

template <typename C> struct Mfma;

template <> struct Mfma<float> {
    static constexpr int BM = 32, BN = 32, BK = 2, NACC = 16;
    typedef float acc_t __attribute__((ext_vector_type(16)));
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    // operand element held by lane l: (mn, k) = (l % 32, l / 32)
    static __device__ __forceinline__ int op_mn(int l) { return l & 31; }
    static __device__ __forceinline__ int op_k(int l) { return l >> 5; }
    // accumulator register i of lane l is D(row, col)
    static __device__ __forceinline__ int row(int i, int l) { return 8 * (i >> 2) + 4 * (l >> 5) + (i & 3); }
    static __device__ __forceinline__ int col(int l) { return l & 31; }
};

template <> struct Mfma<double> {
    static constexpr int BM = 16, BN = 16, BK = 4, NACC = 4;
    typedef double acc_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ acc_t run(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int op_mn(int l) { return l & 15; }
    static __device__ __forceinline__ int op_k(int l) { return l >> 4; }
    static __device__ __forceinline__ int row(int i, int l) { return 4 * i + (l >> 4); }
    static __device__ __forceinline__ int col(int l) { return l & 15; }
};

// 16-byte vectors of NV = 16 / sizeof(C) consecutive elements, read from / written to
// storage type T (a 4-element f16 vector is 8 bytes).
template <typename C, typename T> struct VecIO;
template <> struct VecIO<float, float> {
    typedef float raw_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ void ld(const float* p, float (&o)[4])
    {
        const raw_t v = *reinterpret_cast<const raw_t*>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    static __device__ __forceinline__ void st(float* p, const float (&o)[4])
    {
        raw_t v; v.x = o[0]; v.y = o[1]; v.z = o[2]; v.w = o[3];
        *reinterpret_cast<raw_t*>(p) = v;
    }
};
template <> struct VecIO<double, double> {
    typedef double raw_t __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void ld(const double* p, double (&o)[2])
    {
        const raw_t v = *reinterpret_cast<const raw_t*>(p);
        o[0] = v.x; o[1] = v.y;
    }
    static __device__ __forceinline__ void st(double* p, const double (&o)[2])
    {
        raw_t v; v.x = o[0]; v.y = o[1];
        *reinterpret_cast<raw_t*>(p) = v;
    }
};
template <> struct VecIO<float, __half> {
    typedef unsigned int raw_t __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void ld(const __half* p, float (&o)[4])
    {
        const raw_t v = *reinterpret_cast<const raw_t*>(p);
        const unsigned int lo = v.x, hi = v.y;
        __half2 a, b;
        __builtin_memcpy(&a, &lo, 4);
        __builtin_memcpy(&b, &hi, 4);
        o[0] = __low2float(a); o[1] = __high2float(a); o[2] = __low2float(b); o[3] = __high2float(b);
    }
    static __device__ __forceinline__ void st(__half* p, const float (&o)[4])
    {
        const __half2 a = __floats2half2_rn(o[0], o[1]), b = __floats2half2_rn(o[2], o[3]);
        unsigned int lo, hi;
        __builtin_memcpy(&lo, &a, 4);
        __builtin_memcpy(&hi, &b, 4);
        raw_t v;
        v.x = lo;
        v.y = hi;
        *reinterpret_cast<raw_t*>(p) = v;
    }
};

// bf16 is the upper half of an f32: conversion to f32 is a shift; conversion from f32 rounds to
// nearest even (NaN kept quiet)
template <> struct VecIO<float, bf16_t> {
    typedef unsigned int raw_t __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void ld(const bf16_t* p, float (&o)[4])
    {
        const raw_t v = *reinterpret_cast<const raw_t*>(p);
        o[0] = __builtin_bit_cast(float, v.x << 16);
        o[1] = __builtin_bit_cast(float, v.x & 0xffff0000u);
        o[2] = __builtin_bit_cast(float, v.y << 16);
        o[3] = __builtin_bit_cast(float, v.y & 0xffff0000u);
    }
    static __device__ __forceinline__ unsigned int rne(float f)
    {
        const unsigned int u = __builtin_bit_cast(unsigned int, f);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    static __device__ __forceinline__ void st(bf16_t* p, const float (&o)[4])
    {
        raw_t v;
        v.x = rne(o[0]) | (rne(o[1]) << 16);
        v.y = rne(o[2]) | (rne(o[3]) << 16);
        *reinterpret_cast<raw_t*>(p) = v;
    }
};

// Pol supplies: TM, TN, WM, WN; A_KC / B_KC (is the operand contiguous along k, or along
// its m / n index?); RMW; storage types TA, TB, TD; ktiles();
//   ptrA(mn, kt, k): address of NV consecutive elements of the A operand starting at tile
//     coordinates (mn, k) of k-tile kt -- consecutive along k if A_KC, else along mn --
//     or nullptr where the tile sticks out of the matrix (read as zeros); ptrB likewise;
//   ptrD(m, n): address of NV consecutive destination elements (m, n .. n+NV-1), or nullptr.
// All addresses must be 16-byte aligned (8 for f16 storage).
//
// Both operands are staged through LDS in k-major order (Xs[k][mn]); a k-contiguous
// operand is transposed on its way in (row length odd: conflict-free 4-byte writes), the
// other is copied with 16-byte writes.  The next k-tile's global loads are issued into
// registers before the current tile's MFMAs.  The accumulators leave through LDS, 32 tile
// rows at a time, so that every lane reads / writes 16 bytes and a wave covers whole
// contiguous runs of the destination.  With RMW the destination tile is read into
// registers before the k loop and (destination - product) is written.
template <typename C, typename Pol>
__device__ __forceinline__ void gemm_tile(const Pol& pol)
{
    using M = Mfma<C>;
    constexpr int NV = 16 / (int)sizeof(C);
    constexpr int TM = Pol::TM, TN = Pol::TN, WM = Pol::WM, WN = Pol::WN;
    constexpr int TK = 128 / (int)sizeof(C);
    constexpr int LDA = Pol::A_KC ? TM + 1 : TM + NV, LDB = Pol::B_KC ? TN + 1 : TN + NV, LDD = TN + NV;
    constexpr int WGN = TN / WN;
    static_assert((TM / WM) * WGN == 4, "4 waves per workgroup");
    constexpr int FM = WM / M::BM, FN = WN / M::BN;
    constexpr int NAV = TK * TM / NV / 256, NBV = TK * TN / NV / 256;
    static_assert(NAV >= 1 && NBV >= 1, "tile too small for 256 threads");
    constexpr int PR = 32;                       // tile rows per epilogue pass
    constexpr int NPASS = TM / PR, VPR = TN / NV, EPT = PR * VPR / 256;
    static_assert(EPT >= 1, "epilogue pass too small");
    constexpr int AB_ELEMS = TK * LDA + TK * LDB, D_ELEMS = PR * LDD;
    constexpr int SM_ELEMS = AB_ELEMS > D_ELEMS ? AB_ELEMS : D_ELEMS;
    __shared__ __align__(16) C smem[SM_ELEMS];
    C* As = smem;
    C* Bs = smem + TK * LDA;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    typename M::acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < M::NACC; ++r) acc[i][j][r] = 0;

    // destination tile, in the thread mapping of the epilogue
    C cin[Pol::RMW ? NPASS : 1][Pol::RMW ? EPT : 1][NV];
    if (Pol::RMW) {
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps)
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int v = tid + e * 256;
                const typename Pol::TD* ptr = pol.ptrD(ps * PR + v / VPR, (v % VPR) * NV);
                if (ptr) VecIO<C, typename Pol::TD>::ld(ptr, cin[ps][e]);
                else
#pragma unroll
                    for (int q = 0; q < NV; ++q) cin[ps][e][q] = 0;
            }
    }

    C ra[NAV][NV], rb[NBV][NV];
    auto fetch = [&](int kt) {
#pragma unroll
        for (int e = 0; e < NAV; ++e) {
            const int idx = tid + e * 256;
            const typename Pol::TA* ptr = Pol::A_KC ? pol.ptrA(idx / (TK / NV), kt, (idx % (TK / NV)) * NV)
                                                    : pol.ptrA((idx % (TM / NV)) * NV, kt, idx / (TM / NV));
            if (ptr) VecIO<C, typename Pol::TA>::ld(ptr, ra[e]);
            else
#pragma unroll
                for (int q = 0; q < NV; ++q) ra[e][q] = 0;
        }
#pragma unroll
        for (int e = 0; e < NBV; ++e) {
            const int idx = tid + e * 256;
            const typename Pol::TB* ptr = Pol::B_KC ? pol.ptrB(idx / (TK / NV), kt, (idx % (TK / NV)) * NV)
                                                    : pol.ptrB((idx % (TN / NV)) * NV, kt, idx / (TN / NV));
            if (ptr) VecIO<C, typename Pol::TB>::ld(ptr, rb[e]);
            else
#pragma unroll
                for (int q = 0; q < NV; ++q) rb[e][q] = 0;
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int e = 0; e < NAV; ++e) {
            const int idx = tid + e * 256;
            if (Pol::A_KC) {
                const int mn = idx / (TK / NV), k0 = (idx % (TK / NV)) * NV;
#pragma unroll
                for (int q = 0; q < NV; ++q) As[(k0 + q) * LDA + mn] = ra[e][q];
            } else {
                VecIO<C, C>::st(&As[(idx / (TM / NV)) * LDA + (idx % (TM / NV)) * NV], ra[e]);
            }
        }
#pragma unroll
        for (int e = 0; e < NBV; ++e) {
            const int idx = tid + e * 256;
            if (Pol::B_KC) {
                const int mn = idx / (TK / NV), k0 = (idx % (TK / NV)) * NV;
#pragma unroll
                for (int q = 0; q < NV; ++q) Bs[(k0 + q) * LDB + mn] = rb[e][q];
            } else {
                VecIO<C, C>::st(&Bs[(idx / (TN / NV)) * LDB + (idx % (TN / NV)) * NV], rb[e]);
            }
        }
    };

    const int nkt = pol.ktiles();
    fetch(0);
    for (int kt = 0; kt < nkt; ++kt) {
        stash();
        __syncthreads();
        if (kt + 1 < nkt) fetch(kt + 1);
        const int omn = M::op_mn(lane), ok = M::op_k(lane);
#pragma unroll
        for (int kk = 0; kk < TK; kk += M::BK) {
            C a[FM], b[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) a[i] = As[(kk + ok) * LDA + wm0 + i * M::BM + omn];
#pragma unroll
            for (int j = 0; j < FN; ++j) b[j] = Bs[(kk + ok) * LDB + wn0 + j * M::BN + omn];
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) acc[i][j] = M::run(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    // epilogue: PR tile rows per pass through LDS
    C* Ds = smem;
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            const int r0 = wm0 + i * M::BM;   // first tile row of accumulator block row i
            if (r0 >= ps * PR && r0 < (ps + 1) * PR) {
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int r = 0; r < M::NACC; ++r)
                        Ds[(r0 - ps * PR + M::row(r, lane)) * LDD + wn0 + j * M::BN + M::col(lane)] = acc[i][j][r];
            }
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int v = tid + e * 256;
            typename Pol::TD* ptr = pol.ptrD(ps * PR + v / VPR, (v % VPR) * NV);
            if (ptr) {
                C o[NV];
                VecIO<C, C>::ld(&Ds[(v / VPR) * LDD + (v % VPR) * NV], o);
                if (Pol::RMW) {
#pragma unroll
                    for (int q = 0; q < NV; ++q) o[q] = cin[Pol::RMW ? ps : 0][Pol::RMW ? e : 0][q] - o[q];
                }
                VecIO<C, typename Pol::TD>::st(ptr, o);
            }
        }
        __syncthreads();
    }
}

template <int NB, bool TRANSPOSED> struct TileShape;  // TRANSPOSED: TM = NB, TN = 128
template <> struct TileShape<128, false> { static constexpr int TM = 128, TN = 128, WM = 64, WN = 64; };
template <> struct TileShape<64, false>  { static constexpr int TM = 128, TN = 64,  WM = 64, WN = 32; };
template <> struct TileShape<32, false>  { static constexpr int TM = 128, TN = 32,  WM = 32, WN = 32; };
template <> struct TileShape<128, true>  { static constexpr int TM = 128, TN = 128, WM = 64, WN = 64; };
template <> struct TileShape<64, true>   { static constexpr int TM = 64,  TN = 128, WM = 32, WN = 64; };
template <> struct TileShape<32, true>   { static constexpr int TM = 32,  TN = 128, WM = 32, WN = 32; };


}  // namespace svb
