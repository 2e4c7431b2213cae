// Stage 1, trailing-matrix update in one pass (paper Section 3.1 Algorithm 1
// lines 3/6; Section 3.2 "Trailing Submatrix Update", Algorithm 5: the fused
// TSMQR keeps the tile-row columns a thread owns in registers while it walks
// down the reflector tiles, so that every matrix entry is read once and
// written once).
//
// Same idea, with the domain's reflectors in compact-WY form (Y = V T) and the
// products on MFMA: a workgroup owns the block C_d[:, strip] (all rows of one
// panel domain, 64 columns of the trailing matrix; 128 for f64 at nb = 128), each of its waves keeps
// 16 of those columns in accumulator registers for the whole kernel:
//     W  = Y_d^T C      (contraction over the rows: C's registers are the B operand)
//     C -= V_d W        (W's registers are the B operand, C's the accumulators)
// Y_d and V_d stream through LDS in 32-row slices shared by the 4 waves
// (double buffered, one barrier per slice).  Given the domain's triangular factor T_d
// instead of Y_d, the kernel forms V_d^T C first and then W = T_d^T (V_d^T C) in place
// (T_d streams through the same buffers in slices of 32 columns, W's registers again
// the B operand), so that no Y has to be produced between the panel and its update.  The trailing matrix is read once
// and written once per tree level; W never leaves the registers.
//
// Trailing-matrix element (p, q) lives at Cb[p*sp + q*sq]; p runs along the
// panel direction.  QR sweep: (sp, sq) = (1, lda); LQ sweep: (lda, 1).
#include "svb_internal.h"
#include "mfma_frag.h"
#include "mfma_gemm.h"
#include <hip/hip_ext.h>

namespace svb {

namespace {

template <typename C, int NB> struct FusedGeom {
    // waves per workgroup (16 columns each): eight where the block and W leave room for only one
    // workgroup per compute unit (f64, nb = 128), so that a SIMD still has two waves to switch between
    static constexpr int NWV = (sizeof(C) == 8 && NB == 128) ? 8 : 4;
    static constexpr int NT = NWV * 64, SW = NWV * 16;   // threads, columns of a strip
    // rows of Y / V per LDS slice: every slice costs a fixed amount (its fetch, the wait for it, a
    // barrier) that at 32 rows exceeds its matrix instructions; 64 rows where registers and LDS allow
    static constexpr int RC = (sizeof(C) == 4 && NB == 64) ? 64 : 32;
    static constexpr int NV = Frag<C>::NV;
    static constexpr int MT = NB / 16;                    // 16-row tiles of W
    // row lengths chosen so that the operand fetches (16 lanes on 16 different rows) fall on
    // different LDS banks
    static constexpr int LDR = sizeof(C) == 4 ? RC + 4 : RC + 1;   // Y slice: [column][row]
    static constexpr int LDC = sizeof(C) == 4 ? NB + 4 : NB + 1;   // V slice: [row][column]
    static constexpr int BUF = NB * LDR > RC * LDC ? NB * LDR : RC * LDC;
    static constexpr int NLD = RC * NB / NV / NT;         // 16-byte vectors per thread and slice
    static_assert(NLD >= 1, "slice too small for the workgroup");
    static constexpr size_t kSmemBytes = 2 * (size_t)BUF * sizeof(C);
};

}  // namespace

// Optional phase timing (compile with -DSVB_FUSED_TIMING): thread 0 of workgroup 0 adds the
// shader-clock cycles of each phase to svb_fused_timing[slot].
#ifdef SVB_FUSED_TIMING
__device__ unsigned long long svb_fused_timing[8];
#define FT_MARK(slot_) do { if (tid == 0 && blockIdx.x == 0) { const unsigned long long now_ = clock64(); \
    atomicAdd(&svb_fused_timing[slot_], now_ - ft_last); ft_last = now_; } } while (0)
#else
#define FT_MARK(slot_) do { } while (0)
#endif

// HT: 16-row tiles a wave holds (HT * 16 = rows of the largest domain).
// Two workgroups per compute unit (one loads or stores its block while the other computes)
// wherever the block and W fit in 256 registers per lane.
// TRI: the panel is a stack of upper triangular NB x NB factors (every tree level above the
// first), so in every NB-row chunk of V and of Y = V T the 16 x 16 blocks below the block
// diagonal are exactly zero and their products are skipped.
// USET: the kernel is given the domains' T factors instead of Y (see the header of this file).
// FULL: the domain has all HT tiles and the strip all its columns: every count below is a constant
// and nothing in the stages is predicated.
template <typename T, typename C, int NB, int HT, bool LQ, bool TRI, bool USET, bool FULL>
__device__ __forceinline__ void update_fused_body(T* __restrict__ Cb, int64_t lda, int64_t qlen,
                                                  const C* __restrict__ V, const C* __restrict__ Y,
                                                  int64_t ldp, int chunks, int g, int64_t stride,
                                                  const int d, const int strip, const C* __restrict__ Tw)
{
    using F = Frag<C>;
    using G = FusedGeom<C, NB>;
    typedef typename F::acc_t acc_t;
    constexpr int RC = G::RC, NV = G::NV, MT = G::MT, LDR = G::LDR, LDC = G::LDC, BUF = G::BUF, NLD = G::NLD;
    constexpr int NCK = HT * 16 / RC;   // slices per product for a full domain
    constexpr int VPC = RC / NV;        // vectors per slice column
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C* smem = reinterpret_cast<C*>(smem_raw);

    const int nch = FULL ? HT * 16 / NB : min(g, chunks - d * g);
    const int ntile = FULL ? HT : nch * NB / 16;       // 16-row tiles of this domain
    const int nck = FULL ? NCK : nch * NB / RC;        // slices of this domain
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, gq = lane >> 4;
    const int64_t q = (int64_t)strip * G::SW + wave * 16 + i;
    const bool active = FULL || (int64_t)strip * G::SW + wave * 16 < qlen;   // qlen is a multiple of 16
    const int64_t prow0 = (int64_t)d * g * NB;                    // first row of the domain in V / Y

    // global p index of tile t: chunk (16t / NB) of the domain, offset (16t % NB) inside it
    auto tile_p = [&](int t) -> int64_t {
        return ((int64_t)d * g + (16 * t) / NB) * stride + (16 * t) % NB;
    };

    // The block is fetched tile by tile, PF tiles ahead of the first product's progress, and
    // written back tile by tile as the second product finishes with it, so that the memory
    // traffic runs under the MFMAs instead of before and after them.
    constexpr int PF = HT < 8 ? HT : 8;
    acc_t c[HT];
    auto tile_ld = [&](int t) {
        if (active && t < ntile) c[t] = frag_load<T, C, LQ>(Cb, lda, tile_p(t), q, gq);
        else
#pragma unroll
            for (int r = 0; r < 4; ++r) c[t][r] = 0;
    };
    acc_t w[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) w[mt][r] = 0;

    // ---- slices of Y and V: global -> registers -> LDS
    C sreg[NLD][NV];
    auto slice_ld = [&](const C* __restrict__ src, int ck) {
#pragma unroll
        for (int e = 0; e < NLD; ++e) {
            const int idx = tid + e * G::NT;
            const int rv = idx % VPC, col = idx / VPC;
            VecIO<C, C>::ld(&src[(prow0 + (int64_t)ck * RC + rv * NV) + (int64_t)col * ldp], sreg[e]);
        }
    };
    auto slice_st_y = [&](C* buf) {   // [column][row]
#pragma unroll
        for (int e = 0; e < NLD; ++e) {
            const int idx = tid + e * G::NT;
            const int rv = idx % VPC, col = idx / VPC;
            if constexpr (sizeof(C) == 4) {
                VecIO<C, C>::st(&buf[col * LDR + rv * NV], sreg[e]);
            } else {
#pragma unroll
                for (int j = 0; j < NV; ++j) buf[col * LDR + rv * NV + j] = sreg[e][j];
            }
        }
    };
    auto slice_st_v = [&](C* buf) {   // [row][column]
#pragma unroll
        for (int e = 0; e < NLD; ++e) {
            const int idx = tid + e * G::NT;
            const int rv = idx % VPC, col = idx / VPC;
#pragma unroll
            for (int j = 0; j < NV; ++j) buf[(rv * NV + j) * LDC + col] = sreg[e][j];
        }
    };

    // T_d (column-major, NB x NB, upper triangular): columns 32*ts .. 32*ts+31 are one contiguous
    // piece; in LDS [column][row] with the row length of a V slice
    const C* Td = USET ? Tw + (int64_t)d * NB * NB : nullptr;
    auto tslice_ld = [&](int ts) {
#pragma unroll
        for (int e = 0; e < NLD; ++e)
            VecIO<C, C>::ld(&Td[(int64_t)ts * RC * NB + (int64_t)(tid + e * G::NT) * NV], sreg[e]);
    };
    auto tslice_st = [&](C* buf) {
#pragma unroll
        for (int e = 0; e < NLD; ++e) {
            const int off = (tid + e * G::NT) * NV;
            const int kk = off / NB, j = off % NB;
            if constexpr (sizeof(C) == 4) {
                VecIO<C, C>::st(&buf[kk * LDC + j], sreg[e]);
            } else {
#pragma unroll
                for (int jj = 0; jj < NV; ++jj) buf[kk * LDC + j + jj] = sreg[e][jj];
            }
        }
    };

    // barrier that orders LDS traffic only (s_waitcnt lgkmcnt(0); s_barrier): __syncthreads()
    // would also wait for every outstanding global load and store
    auto lds_barrier = [] {
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
    };
#ifdef SVB_FUSED_TIMING
    unsigned long long ft_last = clock64();
#endif
    constexpr int vlo = 0;
    const int vhi = nck;
    constexpr bool useT = USET;                // (Tw is null otherwise)
    const C* __restrict__ Y1 = useT ? V : Y;   // operand of the first product
    constexpr int NTS = NB / RC;               // slices of T
    int cur = 0;
    slice_ld(Y1, 0);
#pragma unroll
    for (int t = 0; t < PF; ++t) tile_ld(t);
    slice_st_y(smem);
    lds_barrier();
    FT_MARK(0);
#pragma unroll
    for (int s = 0; s < 2 * NCK; ++s) {
        const bool isV = s >= NCK;
        const int ck = isV ? s - NCK : s;
        if (isV ? (ck >= vlo && ck < vhi) : ck < nck) {
            // the stage after this one: the next slice of the same product, or the second
            // product's first slice after the first product's last
            const bool last = ck + 1 == (isV ? vhi : nck);
            const bool have_next = !(isV && last);
            const bool nextT = !isV && last && useT;   // T's last column slice comes first
            const bool nextV = isV || last;
            if (nextT) tslice_ld(NTS - 1);
            else if (have_next) slice_ld(nextV ? V : Y1, last ? vlo : ck + 1);
            if (!isV) {
#pragma unroll
                for (int tt = 0; tt < RC / 16; ++tt)
                    if (ck * (RC / 16) + tt + PF < HT) tile_ld(ck * (RC / 16) + tt + PF);
            }
            const C* buf = smem + cur * BUF;
            FT_MARK(1);
            if (active) {
                if (!isV) {
                    // W += Y_slice^T C_slice
#pragma unroll
                    for (int tt = 0; tt < RC / 16; ++tt) {
                        const int t = ck * (RC / 16) + tt;
                        const int rb = TRI ? (16 * t % NB) / 16 : 0;   // first non-zero block column of this tile
                        // a few tiles of W at a time: consecutive MFMAs are independent
                        constexpr int MG = sizeof(C) == 8 ? 2 : (MT < 4 ? MT : 4);
#pragma unroll
                        for (int m0 = 0; m0 < MT; m0 += MG) {
                            C a[MG][4];
#pragma unroll
                            for (int m = 0; m < MG; ++m)
                                if (m0 + m >= rb) F::ld4(&buf[(16 * (m0 + m) + i) * LDR + 16 * tt], gq, a[m]);
#pragma unroll
                            for (int r = 0; r < 4; ++r)
#pragma unroll
                                for (int m = 0; m < MG; ++m)
                                    if (m0 + m >= rb) w[m0 + m] = F::mma(a[m][r], c[t][r], w[m0 + m]);
                        }
                    }
                    if (last && !useT) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) w[mt][r] = -w[mt][r];
                        }
                    }
                } else {
                    // C_slice += V_slice (-W), two tiles at a time (independent chains of instructions)
                    static_assert(RC % 32 == 0, "pairs of tiles");
#pragma unroll
                    for (int tp = 0; tp < RC / 32; ++tp) {
                        const int t0 = ck * (RC / 16) + 2 * tp, t1 = t0 + 1;
                        const int rb0 = TRI ? (16 * t0 % NB) / 16 : 0, rb1 = TRI ? (16 * t1 % NB) / 16 : 0;
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) {
                            C a0[4], a1[4];
                            if (mt >= rb0) F::ld4(&buf[(32 * tp + i) * LDC + 16 * mt], gq, a0);
                            if (mt >= rb1) F::ld4(&buf[(32 * tp + 16 + i) * LDC + 16 * mt], gq, a1);
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                if (mt >= rb0) c[t0] = F::mma(a0[r], w[mt][r], c[t0]);
                                if (mt >= rb1) c[t1] = F::mma(a1[r], w[mt][r], c[t1]);
                            }
                        }
                    }
                }
            }
            FT_MARK(isV ? 3 : 2);
            if (have_next) {
                C* nbuf = smem + (cur ^ 1) * BUF;
                if (nextT) tslice_st(nbuf);
                else if (nextV) slice_st_v(nbuf);
                else slice_st_y(nbuf);
            }
            // The finished tiles go back only now: loads and stores complete out of order with each
            // other, so a wait for the next slice (above) that found stores in flight would be a
            // wait for every one of them; issued here they have the whole next stage to complete.
            if (isV && active) {
#pragma unroll
                for (int tt = 0; tt < RC / 16; ++tt) {
                    const int t = ck * (RC / 16) + tt;
                    frag_store<T, C, LQ>(Cb, lda, tile_p(t), q, gq, c[t]);
                }
            }
            FT_MARK(4);
            lds_barrier();
            FT_MARK(5);
            cur ^= 1;
            if (nextT) {
                // ---- W = -T^T W, tile rows from the last to the first: tile m of the result needs
                // tiles 0 .. m of the operand (T is upper triangular), which are still untouched
#pragma unroll
                for (int ts = NTS - 1; ts >= 0; --ts) {
                    if (ts > 0) tslice_ld(ts - 1);
                    else slice_ld(V, vlo);
                    const C* tb = smem + cur * BUF;
                    if (active) {
#pragma unroll
                        for (int mm = RC / 16 - 1; mm >= 0; --mm) {
                            const int m = ts * (RC / 16) + mm;
                            acc_t acc;
#pragma unroll
                            for (int r = 0; r < 4; ++r) acc[r] = 0;
#pragma unroll
                            for (int mt = 0; mt <= m; ++mt) {
                                C a[4];
                                F::ld4(&tb[(16 * mm + i) * LDC + 16 * mt], gq, a);
#pragma unroll
                                for (int r = 0; r < 4; ++r) acc = F::mma(a[r], w[mt][r], acc);
                            }
#pragma unroll
                            for (int r = 0; r < 4; ++r) w[m][r] = -acc[r];
                        }
                    }
                    C* nbuf = smem + (cur ^ 1) * BUF;
                    if (ts > 0) tslice_st(nbuf);
                    else slice_st_v(nbuf);
                    lds_barrier();
                    cur ^= 1;
                }
            }
        }
    }
}
#undef FT_MARK

template <typename T, typename C, int NB, int HT, bool LQ, bool TRI, bool USET>
__global__ __launch_bounds__((FusedGeom<C, NB>::NT), (sizeof(C) == 8 && NB == 128) ? 1 : 2) void update_fused_kernel(T* __restrict__ Cb, int64_t lda, int64_t qlen,
                                                           const C* __restrict__ V, const C* __restrict__ Y,
                                                           int64_t ldp, int chunks, int g, int64_t stride,
                                                           int strips, int total, const C* __restrict__ Tw)
{
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): give every
    // XCD a contiguous range of tiles, so that the workgroups sharing a domain's V and Y
    // mostly share an L2 as well.
    const int per = (total + 7) / 8;
    const int tile = (int)(blockIdx.x % 8) * per + (int)(blockIdx.x / 8);
    if (tile >= total) return;
    const int d = tile / strips, strip = tile % strips;
    // (the predicate-free body exists for the QR orientation, whose accesses are 16-byte vectors;
    // in the LQ orientation, element by element, it does not fit the registers)
    if constexpr (!LQ && sizeof(C) == 4) {
        const bool full = g * NB == HT * 16 && chunks - d * g >= g && (int64_t)(strip + 1) * FusedGeom<C, NB>::SW <= qlen;
        if (full) {
            update_fused_body<T, C, NB, HT, LQ, TRI, USET, true>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, d, strip, Tw);
            return;
        }
    }
    update_fused_body<T, C, NB, HT, LQ, TRI, USET, false>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, d, strip, Tw);
}

template <typename T, typename C, int NB, int HT, bool LQ, bool TRI, bool USET>
static void launch_fused(T* Cb, int64_t lda, int64_t qlen, const C* V, const C* Y, int64_t ldp, int chunks,
                         int g, int64_t stride, const C* Tw, bool credited, hipStream_t s)
{
    using G = FusedGeom<C, NB>;
    auto kern = update_fused_kernel<T, C, NB, HT, LQ, TRI, USET>;
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
    // both products: 2 * rows * NB * cols flops each; the block is read once and written once
    const double rows = (double)chunks * NB;
    double fl = 4.0 * rows * NB * (double)qlen, by = 2.0 * rows * (double)qlen * sizeof(T);
    if (!credited) fl = by = 0.0;
    // profiling: the events are the kernel's own start and stop time stamps
    hipEvent_t ea = nullptr, eb = nullptr;
    if (prof_take(TRI ? SVB_PROF_UPDATE_UPPER : SVB_PROF_UPDATE, fl, by, &ea, &eb))
        hipExtLaunchKernelGGL(kern, dim3((unsigned)(per * 8)), dim3(G::NT), (uint32_t)G::kSmemBytes, s, ea, eb, 0u, Cb,
                              lda, qlen, V, Y, ldp, chunks, g, stride, strips, total, Tw);
    else
        hipLaunchKernelGGL(kern, dim3((unsigned)(per * 8)), dim3(G::NT), G::kSmemBytes, s, Cb, lda, qlen, V, Y, ldp,
                           chunks, g, stride, strips, total, Tw);
}

template <typename T, typename C, int NB, int HT, bool LQ, bool TRI>
static void launch_fused_t(T* Cb, int64_t lda, int64_t qlen, const C* V, const C* Y, int64_t ldp,
                           int chunks, int g, int64_t stride, const C* Tw, bool credited, hipStream_t s)
{
    // the form that applies T itself exists at nb <= 64 (at nb = 128 the extra accumulators do not
    // fit beside the block)
    if constexpr (NB <= 64) {
        if (Tw != nullptr) {
            launch_fused<T, C, NB, HT, LQ, TRI, true>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, Tw, credited, s);
            return;
        }
    }
    launch_fused<T, C, NB, HT, LQ, TRI, false>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, nullptr, credited, s);
}

template <typename C> constexpr int fused_tiles() { return sizeof(C) == 4 ? 32 : 16; }

// rows of the largest domain the one-pass kernel holds in registers
template <typename C> int fused_update_rows() { return fused_tiles<C>() * 16; }
template int fused_update_rows<float>();
template int fused_update_rows<double>();

template <typename T, typename C>
void launch_update_fused(int nb, bool lq, T* Cb, int64_t lda, int64_t qlen, const C* V, const C* Y,
                         int64_t ldp, int chunks, int g, int64_t stride, bool tri, const C* Tw,
                         bool credited, hipStream_t s, bool half_ops)
{
    if (qlen <= 0) return;
    if constexpr (sizeof(T) == 2) {
        // f16 / bf16 storage: both products on the 16-bit matrix instructions (half_ops = false keeps
        // the f32-operand kernels below)
        if (half_ops && g * nb <= 512) {
            launch_update_fused16<T>(nb, lq, Cb, lda, qlen, V, Y, ldp, chunks, g, stride, tri, Tw, credited, s);
            return;
        }
    }
    if constexpr (sizeof(C) == 4) {
        // nb = 128: the kernel built on the 32 x 32 x 2 instruction (SVB_UPDATE_MFMA32=0 keeps this file's)
        static const bool wide = env_int("SVB_UPDATE_MFMA32", 1) != 0;
        if (nb == 128 && Tw == nullptr && g * nb <= 512 && qlen % 32 == 0 && wide) {
            launch_update_fused32<T>(lq, Cb, lda, qlen, V, Y, ldp, chunks, g, stride, tri, credited, s);
            return;
        }
    }
    constexpr int HT = fused_tiles<C>();
#define SVB_FUSED_ARGS Cb, lda, qlen, V, Y, ldp, chunks, g, stride, Tw, credited, s
#define SVB_FUSED_CASE(NBV)                                                          \
    case NBV:                                                                        \
        if (lq && tri) launch_fused_t<T, C, NBV, HT, true, true>(SVB_FUSED_ARGS);   \
        else if (lq) launch_fused_t<T, C, NBV, HT, true, false>(SVB_FUSED_ARGS);    \
        else if (tri) launch_fused_t<T, C, NBV, HT, false, true>(SVB_FUSED_ARGS);   \
        else launch_fused_t<T, C, NBV, HT, false, false>(SVB_FUSED_ARGS);           \
        break;
    switch (nb) {
        SVB_FUSED_CASE(32)
        SVB_FUSED_CASE(64)
        SVB_FUSED_CASE(128)
    default: break;
    }
#undef SVB_FUSED_CASE
#undef SVB_FUSED_ARGS
}

template void launch_update_fused<float, float>(int, bool, float*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, bool, const float*, bool, hipStream_t, bool);
template void launch_update_fused<__half, float>(int, bool, __half*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, bool, const float*, bool, hipStream_t, bool);
template void launch_update_fused<bf16_t, float>(int, bool, bf16_t*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, bool, const float*, bool, hipStream_t, bool);
template void launch_update_fused<double, double>(int, bool, double*, int64_t, int64_t, const double*, const double*, int64_t, int, int, int64_t, bool, const double*, bool, hipStream_t, bool);

}  // namespace svb
