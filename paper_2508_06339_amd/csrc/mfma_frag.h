// 16 x 16 x 4 MFMA fragments (gfx950) for kernels that keep a block of the
// matrix in accumulator registers and reuse those registers as an operand.
//
// One instruction computes D(16 x 16) += A(16 x 4) B(4 x 16).  Lane l = 16*gq + i
// supplies A[i][gq] and B[gq][i] and holds four entries of column i of D, in the
// rows roff(r, gq), r = 0..3.  Because the four k-slots of an instruction belong
// to the four lane groups gq, accumulator register r of a tile is at the same
// time a valid B operand: its k-slot gq carries row roff(r, gq) of the tile.
// A product whose contraction index runs over the rows of a register-resident
// tile therefore needs no data movement for that tile; the other operand is
// fetched in the matching order (Frag::ld4).
#pragma once

#include "svb_internal.h"
#include "mfma_gemm.h"

namespace svb {

template <typename C> struct Frag;

template <> struct Frag<float> {
    typedef float acc_t __attribute__((ext_vector_type(4)));
    static constexpr int NV = 4;  // elements per 16-byte vector
    static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int roff(int r, int gq) { return 4 * gq + r; }
    static constexpr bool kContig = true;  // roff(0..3, gq) are consecutive
    // a[r] = p[roff(r, gq)]; p 16-byte aligned
    static __device__ __forceinline__ void ld4(const float* p, int gq, float (&a)[4])
    {
        typedef float v4 __attribute__((ext_vector_type(4)));
        const v4 v = *reinterpret_cast<const v4*>(p + 4 * gq);
        a[0] = v.x; a[1] = v.y; a[2] = v.z; a[3] = v.w;
    }
    // p[roff(r, gq)] = a[r]
    static __device__ __forceinline__ void st4(float* p, int gq, const float (&a)[4])
    {
        typedef float v4 __attribute__((ext_vector_type(4)));
        v4 v; v.x = a[0]; v.y = a[1]; v.z = a[2]; v.w = a[3];
        *reinterpret_cast<v4*>(p + 4 * gq) = v;
    }
};

template <> struct Frag<double> {
    typedef double acc_t __attribute__((ext_vector_type(4)));
    static constexpr int NV = 2;
    static __device__ __forceinline__ acc_t mma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int roff(int r, int gq) { return 4 * r + gq; }
    static constexpr bool kContig = false;
    static __device__ __forceinline__ void ld4(const double* p, int gq, double (&a)[4])
    {
#pragma unroll
        for (int r = 0; r < 4; ++r) a[r] = p[4 * r + gq];
    }
    static __device__ __forceinline__ void st4(double* p, int gq, const double (&a)[4])
    {
#pragma unroll
        for (int r = 0; r < 4; ++r) p[4 * r + gq] = a[r];
    }
};

// ---- the four matrix entries a lane holds of one 16 x 16 tile: rows p0 + roff(r, gq), column q
template <typename T, typename C, bool LQ>
__device__ __forceinline__ typename Frag<C>::acc_t frag_load(const T* __restrict__ Cb, int64_t lda,
                                                             int64_t p0, int64_t q, int gq)
{
    using F = Frag<C>;
    typename F::acc_t c;
    if constexpr (!LQ && F::kContig) {
        C o[4];
        VecIO<C, T>::ld(&Cb[(p0 + 4 * gq) + q * lda], o);
        c[0] = o[0]; c[1] = o[1]; c[2] = o[2]; c[3] = o[3];
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t p = p0 + F::roff(r, gq);
            c[r] = ld_as<C, T>(LQ ? &Cb[p * lda + q] : &Cb[p + q * lda]);
        }
    }
    return c;
}

template <typename T, typename C, bool LQ>
__device__ __forceinline__ void frag_store(T* __restrict__ Cb, int64_t lda, int64_t p0, int64_t q, int gq,
                                           const typename Frag<C>::acc_t& c)
{
    using F = Frag<C>;
    if constexpr (!LQ && F::kContig) {
        const C o[4] = {c[0], c[1], c[2], c[3]};
        VecIO<C, T>::st(&Cb[(p0 + 4 * gq) + q * lda], o);
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t p = p0 + F::roff(r, gq);
            st_as<T, C>(LQ ? &Cb[p * lda + q] : &Cb[p + q * lda], c[r]);
        }
    }
}

}  // namespace svb
