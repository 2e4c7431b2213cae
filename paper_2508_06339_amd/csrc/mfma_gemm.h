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

// Pol supplies: TM, TN, WM, WN, A_KC, B_KC (operand contiguous along k?),
// ktiles(), loadA(mn, kt, k), loadB(mn, kt, k), store(m, n, value) and RMW.
// With RMW the tile of the destination is read into registers before the k loop
// (loadC(m, n)), so that its latency hides behind the product, and
// store(m, n, c - value) writes the difference.
template <typename C, typename Pol>
__device__ __forceinline__ void gemm_tile(const Pol& pol)
{
    using M = Mfma<C>;
    constexpr int TM = Pol::TM, TN = Pol::TN, WM = Pol::WM, WN = Pol::WN;
    constexpr int TK = 128 / (int)sizeof(C);
    constexpr int LDA = TM + 1, LDB = TN + 1;
    constexpr int WGN = TN / WN;
    static_assert((TM / WM) * WGN == 4, "4 waves per workgroup");
    constexpr int FM = WM / M::BM, FN = WN / M::BN;
    constexpr int NA = TK * TM / 256, NBE = TK * TN / 256;
    __shared__ C As[TK * LDA];
    __shared__ C Bs[TK * LDB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
    typename M::acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < M::NACC; ++r) acc[i][j][r] = 0;

    typename M::acc_t cin[Pol::RMW ? FM : 1][Pol::RMW ? FN : 1];
    if (Pol::RMW) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < M::NACC; ++r)
                    cin[i][j][r] = pol.loadC(wm0 + i * M::BM + M::row(r, lane), wn0 + j * M::BN + M::col(lane));
    }

    C ra[NA], rb[NBE];
    auto fetch = [&](int kt) {
#pragma unroll
        for (int e = 0; e < NA; ++e) {
            const int idx = tid + e * 256;
            const int k = Pol::A_KC ? idx % TK : idx / TM;
            const int mn = Pol::A_KC ? idx / TK : idx % TM;
            ra[e] = pol.loadA(mn, kt, k);
        }
#pragma unroll
        for (int e = 0; e < NBE; ++e) {
            const int idx = tid + e * 256;
            const int k = Pol::B_KC ? idx % TK : idx / TN;
            const int mn = Pol::B_KC ? idx / TK : idx % TN;
            rb[e] = pol.loadB(mn, kt, k);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int e = 0; e < NA; ++e) {
            const int idx = tid + e * 256;
            const int k = Pol::A_KC ? idx % TK : idx / TM;
            const int mn = Pol::A_KC ? idx / TK : idx % TM;
            As[k * LDA + mn] = ra[e];
        }
#pragma unroll
        for (int e = 0; e < NBE; ++e) {
            const int idx = tid + e * 256;
            const int k = Pol::B_KC ? idx % TK : idx / TN;
            const int mn = Pol::B_KC ? idx / TK : idx % TN;
            Bs[k * LDB + mn] = rb[e];
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
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < M::NACC; ++r)
                pol.store(wm0 + i * M::BM + M::row(r, lane), wn0 + j * M::BN + M::col(lane),
                          Pol::RMW ? cin[Pol::RMW ? i : 0][Pol::RMW ? j : 0][r] - acc[i][j][r] : acc[i][j][r]);
}

template <int NB, bool TRANSPOSED> struct TileShape;  // TRANSPOSED: TM = NB, TN = 128
template <> struct TileShape<128, false> { static constexpr int TM = 128, TN = 128, WM = 64, WN = 64; };
template <> struct TileShape<64, false>  { static constexpr int TM = 128, TN = 64,  WM = 64, WN = 32; };
template <> struct TileShape<32, false>  { static constexpr int TM = 128, TN = 32,  WM = 32, WN = 32; };
template <> struct TileShape<128, true>  { static constexpr int TM = 128, TN = 128, WM = 64, WN = 64; };
template <> struct TileShape<64, true>   { static constexpr int TM = 64,  TN = 128, WM = 32, WN = 64; };
template <> struct TileShape<32, true>   { static constexpr int TM = 32,  TN = 128, WM = 32, WN = 32; };


}  // namespace svb
