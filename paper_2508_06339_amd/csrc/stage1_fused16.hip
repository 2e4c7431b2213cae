// Stage 1, trailing-matrix update in one pass for f16 / bf16 storage on the 16-bit matrix
// instructions (paper Section 3.1 Algorithm 1 lines 3/6; Section 3.2 "Trailing Submatrix Update",
// Algorithm 5; Section 4.3: half precision is stored in 16 bits and accumulated in f32).
//
// Same schedule as the f32 / f64 kernel (stage1_fused.hip): a workgroup owns the block
// C_d[:, strip] (all rows of one panel domain, 64 columns), each wave 16 of its columns in f32
// accumulators for the whole kernel,
//     W  = Y_d^T C      (or V_d^T C followed by W = T_d^T W)
//     C -= V_d W
// with both large products on v_mfma_f32_16x16x32_f16 / _bf16 (f32 accumulate).  A lane of such an
// instruction supplies eight consecutive k-slots; two 16-row accumulator tiles, converted to
// 16 bits and packed, are exactly that for a contraction over their 32 rows (slots 0-3: rows
// 4*gq .. 4*gq+3 of the first tile, slots 4-7: the same rows of the second), so the resident
// block and W again serve as operands without being moved.
//
// Precision.  The block is exact in its storage type, so it enters the first product unrounded.
// The reflectors V, Y (computed in f32 by the panel kernels) and W are split into a sum of 16-bit
// terms (two for f16, three for bf16) and the cross products that matter at f32 precision are
// accumulated, so the update is as accurate as the f32-operand kernel; the only rounding to 16 bits
// is the one the storage type imposes when the block is written back.  f16 terms hold magnitudes
// up to 65504 and lose bits below 6e-5; svb_svdvals scales f16 matrices into that range as it
// does the other types.
#include "svb_internal.h"
#include "mfma_frag.h"
#include "mfma_gemm.h"
#include <hip/hip_ext.h>
#include <type_traits>
#include <utility>

namespace svb {

namespace {

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): the stages of the kernel take
// their index as a constant, so that every register array is indexed statically whatever the size
// of the unrolled body
template <typename Fn, int... I>
__device__ __forceinline__ void static_for_impl(Fn&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename Fn> __device__ __forceinline__ void static_for(Fn&& f)
{
    static_for_impl(static_cast<Fn&&>(f), std::make_integer_sequence<int, N>{});
}

typedef float f4_t __attribute__((ext_vector_type(4)));
typedef float f2_t __attribute__((ext_vector_type(2)));

// 16-bit operand type of a storage type: vector types, number of terms of a split f32, the
// matrix instruction
template <typename T> struct Half16;
template <> struct Half16<__half> {
    typedef _Float16 e_t;
    typedef _Float16 v2_t __attribute__((ext_vector_type(2)));
    typedef _Float16 v4_t __attribute__((ext_vector_type(4)));
    typedef _Float16 v8_t __attribute__((ext_vector_type(8)));
    static constexpr int NS = 2;
    static __device__ __forceinline__ f4_t mma(v8_t a, v8_t b, f4_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};
template <> struct Half16<bf16_t> {
    typedef __bf16 e_t;
    typedef __bf16 v2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 v4_t __attribute__((ext_vector_type(4)));
    typedef __bf16 v8_t __attribute__((ext_vector_type(8)));
    static constexpr int NS = 3;
    static __device__ __forceinline__ f4_t mma(v8_t a, v8_t b, f4_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};

// x = s[0] + s[1] (+ s[2]) up to f32 rounding, every term representable in 16 bits
template <typename H> __device__ __forceinline__ void split4(const f4_t x, typename H::v4_t (&s)[H::NS])
{
    f4_t rest = x;
#pragma unroll
    for (int k = 0; k < H::NS; ++k) {
        s[k] = __builtin_convertvector(rest, typename H::v4_t);
        if (k + 1 < H::NS) rest -= __builtin_convertvector(s[k], f4_t);
    }
}
template <typename V8, typename V4> __device__ __forceinline__ V8 cat4(V4 a, V4 b)
{
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

template <int NB, int NS> struct Fused16Geom {
    static constexpr int NWV = 4, NT = NWV * 64, SW = NWV * 16;
    static constexpr int RC = 32;                 // rows of Y / V per LDS slice = rows of a tile pair
    static constexpr int MT = NB / 16;            // 16-row tiles of W
    static constexpr int KT = NB / 32;            // 32-slot steps of the second product
    // 16-bit parts (row lengths in 16-bit elements, multiples of 4: every operand fetch is 8 bytes)
    static constexpr int LDR = RC + 4;            // Y slice: [column][row]
    static constexpr int LDC = NB + 4;            // V slice: [row][column]
    static constexpr int PART = NB * LDR > RC * LDC ? NB * LDR : RC * LDC;   // one term of a slice
    // T slices stay f32: [column][row], row length NB + 4
    static constexpr int LDT = NB + 4;
    static constexpr size_t kHalfBytes = (size_t)NS * PART * 2;
    static constexpr size_t kTBytes = (size_t)RC * LDT * 4;
    static constexpr size_t kBufBytes = ((kHalfBytes > kTBytes ? kHalfBytes : kTBytes) + 15) / 16 * 16;
    static constexpr size_t kSmemBytes = 2 * kBufBytes;
    static constexpr int NLD = RC * NB / 4 / NT;  // 16-byte f32 vectors per thread and slice
    static_assert(NLD >= 1, "slice too small for the workgroup");
};

}  // namespace

// HT: 16-row tiles a wave holds (HT * 16 = rows of the largest domain).  TRI: the panel is a stack
// of upper triangular NB x NB factors (tree levels above the first): products with the 16-column
// blocks of V and Y that are entirely zero are skipped.  USET: the kernel is given the domains' T
// factors instead of Y and forms W = T^T (V^T C) itself (the small triangular product stays on the
// f32 instruction).
template <typename T, int NB, int HT, bool LQ, bool TRI, bool USET>
__global__ __launch_bounds__(256, 2) void update_fused16_kernel(T* __restrict__ Cb, int64_t lda, int64_t qlen,
                                                               const float* __restrict__ V, const float* __restrict__ Y,
                                                               int64_t ldp, int chunks, int g, int64_t stride,
                                                               int strips, int total, const float* __restrict__ Tw)
{
    using H = Half16<T>;
    using F = Frag<float>;
    using G = Fused16Geom<NB, H::NS>;
    typedef typename H::e_t e_t;
    typedef typename H::v4_t v4_t;
    typedef typename H::v8_t v8_t;
    constexpr int NS = H::NS, RC = G::RC, MT = G::MT, KT = G::KT, LDR = G::LDR, LDC = G::LDC, PART = G::PART, LDT = G::LDT,
                  NLD = G::NLD;
    constexpr int NCK = HT * 16 / RC;   // slices per product for a full domain
    constexpr int VPC = RC / 4;         // vectors per slice column
    extern __shared__ __align__(16) unsigned char smem_raw[];

    // every XCD gets a contiguous range of (domain, strip) tiles: the workgroups that share a
    // domain's V and Y mostly share an L2
    const int per = (total + 7) / 8;
    const int tile = (int)(blockIdx.x % 8) * per + (int)(blockIdx.x / 8);
    if (tile >= total) return;
    const int d = tile / strips, strip = tile % strips;

    const int nch = min(g, chunks - d * g);
    const int ntile = nch * NB / 16;   // 16-row tiles of this domain
    const int nck = nch * NB / RC;     // slices of this domain
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, gq = lane >> 4;
    const int64_t q = (int64_t)strip * G::SW + wave * 16 + i;
    const bool active = (int64_t)strip * G::SW + wave * 16 < qlen;   // qlen is a multiple of 16
    const int64_t prow0 = (int64_t)d * g * NB;

    auto tile_p = [&](int t) -> int64_t {
        return ((int64_t)d * g + (16 * t) / NB) * stride + (16 * t) % NB;
    };
    constexpr int PF = HT < 8 ? HT : (NB == 128 ? 4 : 8);   // tiles requested ahead (fewer where registers are short)
    f4_t c[HT];
    auto tile_ld = [&](int t) {
        if (active && t < ntile) c[t] = frag_load<T, float, LQ>(Cb, lda, tile_p(t), q, gq);
        else
#pragma unroll
            for (int r = 0; r < 4; ++r) c[t][r] = 0;
    };
    f4_t w[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) w[mt][r] = 0;

    // ---- slices of Y and V: global (f32) -> registers -> split -> LDS (16-bit terms)
    f4_t sreg[NLD];
    auto slice_ld = [&](const float* __restrict__ src, int ck) {
#pragma unroll
        for (int e = 0; e < NLD; ++e) {
            const int idx = tid + e * G::NT;
            const int rv = idx % VPC, col = idx / VPC;
            sreg[e] = *reinterpret_cast<const f4_t*>(&src[(prow0 + (int64_t)ck * RC + rv * 4) + (int64_t)col * ldp]);
        }
    };
    auto slice_st_y = [&](unsigned char* buf) {   // [column][row]
        e_t* hb = reinterpret_cast<e_t*>(buf);
#pragma unroll
        for (int e = 0; e < NLD; ++e) {
            const int idx = tid + e * G::NT;
            const int rv = idx % VPC, col = idx / VPC;
            v4_t s[NS];
            split4<H>(sreg[e], s);
#pragma unroll
            for (int k = 0; k < NS; ++k) *reinterpret_cast<v4_t*>(&hb[k * PART + col * LDR + rv * 4]) = s[k];
        }
    };
    auto slice_st_v = [&](unsigned char* buf) {   // [row][column]
        e_t* hb = reinterpret_cast<e_t*>(buf);
#pragma unroll
        for (int e = 0; e < NLD; ++e) {
            const int idx = tid + e * G::NT;
            const int rv = idx % VPC, col = idx / VPC;
            v4_t s[NS];
            split4<H>(sreg[e], s);
#pragma unroll
            for (int k = 0; k < NS; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) hb[k * PART + (rv * 4 + j) * LDC + col] = s[k][j];
        }
    };
    // T_d (column-major, NB x NB, upper triangular, f32): columns 32*ts .. 32*ts+31 are one
    // contiguous piece; in LDS [column][row]
    const float* Td = USET ? Tw + (int64_t)d * NB * NB : nullptr;
    auto tslice_ld = [&](int ts) {
#pragma unroll
        for (int e = 0; e < NLD; ++e)
            sreg[e] = *reinterpret_cast<const f4_t*>(&Td[(int64_t)ts * RC * NB + (int64_t)(tid + e * G::NT) * 4]);
    };
    auto tslice_st = [&](unsigned char* buf) {
        float* fb = reinterpret_cast<float*>(buf);
#pragma unroll
        for (int e = 0; e < NLD; ++e) {
            const int off = (tid + e * G::NT) * 4;
            const int kk = off / NB, j = off % NB;
            *reinterpret_cast<f4_t*>(&fb[kk * LDT + j]) = sreg[e];
        }
    };
    // barrier that orders LDS traffic only (the block's loads and stores stay in flight)
    auto lds_barrier = [] {
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
    };
    // eight k-slots of an operand: two groups of four consecutive 16-bit elements
    auto ld8 = [&](const e_t* p0, const e_t* p1) -> v8_t {
        return cat4<v8_t, v4_t>(*reinterpret_cast<const v4_t*>(p0), *reinterpret_cast<const v4_t*>(p1));
    };

    constexpr bool useT = USET;
    const float* __restrict__ Y1 = useT ? V : Y;   // operand of the first product
    constexpr int NTS = NB / RC;                   // slices of T
    // W as the second product's operand: its terms, per 32-row step
    v8_t wsp[KT][NS];
    auto split_w = [&] {
#pragma unroll
        for (int kk = 0; kk < KT; ++kk) {
            v4_t s0[NS], s1[NS];
            split4<H>(w[2 * kk], s0);
            split4<H>(w[2 * kk + 1], s1);
#pragma unroll
            for (int k = 0; k < NS; ++k) wsp[kk][k] = cat4<v8_t, v4_t>(s0[k], s1[k]);
        }
    };
    int cur = 0;
    slice_ld(Y1, 0);
#pragma unroll
    for (int t = 0; t < PF; ++t) tile_ld(t);
    slice_st_y(smem_raw);
    lds_barrier();
    static_for<2 * NCK>([&](auto stage) __attribute__((always_inline)) {
        constexpr int s = decltype(stage)::value;
        constexpr bool isV = s >= NCK;
        constexpr int ck = isV ? s - NCK : s;
        if (ck < nck) {
            const bool last = ck + 1 == nck;
            const bool have_next = !(isV && last);
            const bool nextT = !isV && last && useT;   // T's last column slice comes first
            const bool nextV = isV || last;
            if (nextT) tslice_ld(NTS - 1);
            else if (have_next) slice_ld(nextV ? V : Y1, last ? 0 : ck + 1);
            if (!isV) {
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
                    if (ck * 2 + tt + PF < HT) tile_ld(ck * 2 + tt + PF);
            }
            const e_t* hb = reinterpret_cast<const e_t*>(smem_raw + cur * G::kBufBytes);
            constexpr int t0 = 2 * ck, t1 = 2 * ck + 1;
            // first block column of V / Y that is not zero in the rows of this tile pair
            constexpr int rb0 = TRI ? (16 * t0 % NB) / 16 : 0;
            if (active) {
                if (!isV) {
                    // W += Y_slice^T C_slice: the block's two tiles, exact in 16 bits, are the B operand
                    const v8_t bc = cat4<v8_t, v4_t>(__builtin_convertvector(c[t0], v4_t),
                                                     __builtin_convertvector(c[t1], v4_t));
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        if (m >= rb0) {
#pragma unroll
                            for (int k = 0; k < NS; ++k) {
                                const e_t* p = hb + k * PART + (16 * m + i) * LDR + 4 * gq;
                                w[m] = H::mma(ld8(p, p + 16), bc, w[m]);
                            }
                        }
                    }
                    if (last && !useT) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) w[mt] = -w[mt];
                        split_w();
                    }
                } else {
                    // C_slice += V_slice (-W): the cross products of the terms that matter in f32
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt) {
                        const int t = t0 + tt;
                        const int rb = TRI ? (16 * t % NB) / 16 : 0;
#pragma unroll
                        for (int kk = 0; kk < KT; ++kk) {
                            if (2 * kk + 1 >= rb) {
                                v8_t a[NS];
#pragma unroll
                                for (int k = 0; k < NS; ++k) {
                                    const e_t* p = hb + k * PART + (16 * tt + i) * LDC + 32 * kk + 4 * gq;
                                    a[k] = ld8(p, p + 16);
                                }
#pragma unroll
                                for (int ka = 0; ka < NS; ++ka)
#pragma unroll
                                    for (int kw = 0; kw + ka < NS; ++kw) c[t] = H::mma(a[ka], wsp[kk][kw], c[t]);
                            }
                        }
                    }
                    frag_store<T, float, LQ>(Cb, lda, tile_p(t0), q, gq, c[t0]);
                    frag_store<T, float, LQ>(Cb, lda, tile_p(t1), q, gq, c[t1]);
                }
            }
            if (have_next) {
                unsigned char* nbuf = smem_raw + (cur ^ 1) * G::kBufBytes;
                if (nextT) tslice_st(nbuf);
                else if (nextV) slice_st_v(nbuf);
                else slice_st_y(nbuf);
            }
            lds_barrier();
            cur ^= 1;
            if (nextT) {
                // ---- W = -T^T W on the f32 instruction, tile rows from the last to the first: tile m of
                // the result needs tiles 0 .. m of the operand (T is upper triangular), still untouched
#pragma unroll
                for (int ts = NTS - 1; ts >= 0; --ts) {
                    if (ts > 0) tslice_ld(ts - 1);
                    else slice_ld(V, 0);
                    const float* tb = reinterpret_cast<const float*>(smem_raw + cur * G::kBufBytes);
                    if (active) {
#pragma unroll
                        for (int mm = RC / 16 - 1; mm >= 0; --mm) {
                            const int m = ts * (RC / 16) + mm;
                            f4_t acc;
#pragma unroll
                            for (int r = 0; r < 4; ++r) acc[r] = 0;
#pragma unroll
                            for (int mt = 0; mt <= m; ++mt) {
                                float a[4];
                                F::ld4(&tb[(16 * mm + i) * LDT + 16 * mt], gq, a);
#pragma unroll
                                for (int r = 0; r < 4; ++r) acc = F::mma(a[r], w[mt][r], acc);
                            }
                            w[m] = -acc;
                        }
                    }
                    unsigned char* nbuf = smem_raw + (cur ^ 1) * G::kBufBytes;
                    if (ts > 0) tslice_st(nbuf);
                    else slice_st_v(nbuf);
                    lds_barrier();
                    cur ^= 1;
                }
                split_w();
            }
        }
    });
}

template <typename T, int NB, int HT, bool LQ, bool TRI, bool USET>
static void launch_fused16(T* Cb, int64_t lda, int64_t qlen, const float* V, const float* Y, int64_t ldp, int chunks,
                           int g, int64_t stride, const float* Tw, bool credited, hipStream_t s)
{
    using G = Fused16Geom<NB, Half16<T>::NS>;
    auto kern = update_fused16_kernel<T, NB, HT, LQ, TRI, USET>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)G::kSmemBytes);
        attr_set = true;
    }
    const int domains = (chunks + g - 1) / g;
    const int strips = (int)((qlen + G::SW - 1) / G::SW);
    const int total = domains * strips;
    const int per = (total + 7) / 8;
    // credited: both products, 2 * rows * NB * cols flops each; the block is read once and written once
    const double rows = (double)chunks * NB;
    double fl = 4.0 * rows * NB * (double)qlen, by = 2.0 * rows * (double)qlen * sizeof(T);
    if (!credited) fl = by = 0.0;
    hipEvent_t ea = nullptr, eb = nullptr;
    if (prof_take(TRI ? SVB_PROF_UPDATE_UPPER : SVB_PROF_UPDATE, fl, by, &ea, &eb))
        hipExtLaunchKernelGGL(kern, dim3((unsigned)(per * 8)), dim3(G::NT), (uint32_t)G::kSmemBytes, s, ea, eb, 0u, Cb,
                              lda, qlen, V, Y, ldp, chunks, g, stride, strips, total, Tw);
    else
        hipLaunchKernelGGL(kern, dim3((unsigned)(per * 8)), dim3(G::NT), G::kSmemBytes, s, Cb, lda, qlen, V, Y, ldp,
                           chunks, g, stride, strips, total, Tw);
}

template <typename T, int NB, bool LQ, bool TRI>
static void launch_fused16_t(T* Cb, int64_t lda, int64_t qlen, const float* V, const float* Y, int64_t ldp, int chunks,
                             int g, int64_t stride, const float* Tw, bool credited, hipStream_t s)
{
    constexpr int HT = 32;   // 512 rows
    if constexpr (NB <= 64) {
        if (Tw != nullptr) {
            launch_fused16<T, NB, HT, LQ, TRI, true>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, Tw, credited, s);
            return;
        }
    }
    launch_fused16<T, NB, HT, LQ, TRI, false>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, nullptr, credited, s);
}

template <typename T>
void launch_update_fused16(int nb, bool lq, T* Cb, int64_t lda, int64_t qlen, const float* V, const float* Y,
                           int64_t ldp, int chunks, int g, int64_t stride, bool tri, const float* Tw, bool credited,
                           hipStream_t s)
{
    if (qlen <= 0) return;
#define SVB_F16_ARGS Cb, lda, qlen, V, Y, ldp, chunks, g, stride, Tw, credited, s
#define SVB_F16_CASE(NBV)                                                        \
    case NBV:                                                                    \
        if (lq && tri) launch_fused16_t<T, NBV, true, true>(SVB_F16_ARGS);      \
        else if (lq) launch_fused16_t<T, NBV, true, false>(SVB_F16_ARGS);       \
        else if (tri) launch_fused16_t<T, NBV, false, true>(SVB_F16_ARGS);      \
        else launch_fused16_t<T, NBV, false, false>(SVB_F16_ARGS);              \
        break;
    switch (nb) {
        SVB_F16_CASE(32)
        SVB_F16_CASE(64)
        SVB_F16_CASE(128)
    default: break;
    }
#undef SVB_F16_CASE
#undef SVB_F16_ARGS
}

template void launch_update_fused16<__half>(int, bool, __half*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, bool, const float*, bool, hipStream_t);
template void launch_update_fused16<bf16_t>(int, bool, bf16_t*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, bool, const float*, bool, hipStream_t);

}  // namespace svb
