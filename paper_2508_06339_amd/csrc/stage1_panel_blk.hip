// Stage 1, panel factorisation of one domain, blocked (paper Section 3.2
// "Panel Factorization", Algorithm 3; Section 3.1 Algorithm 1 lines 2/4).
//
// The paper's GEQRT/TSQRT keep the tile in registers and apply every reflector
// to every column with scalar FMAs.  Here the domain (H = 16*HT rows, NB
// columns) also lives in registers, but in MFMA accumulator layout: wave w
// holds columns 16w .. 16w+15.  The columns are factored 16 at a time:
//   1. the owning wave hands its 16 columns to LDS;
//   2. all threads factor that 16-column block with Householder reflectors
//      (Algorithm 3's loop, the column split over row groups, two barriers per
//      reflector) -- the only part that works reflector by reflector;
//   3. the block's reflectors are applied to the columns right of it as ONE
//      block reflector on MFMA:  C_w -= V_b (T_b^T (V_b^T C_w));
//   4. the waves left of the block (whose registers now hold their own V)
//      form V_w^T V_b the same way, from which the domain's compact-WY factor
//      T grows by one block column:  T[0:b, b] = -T[0:b, 0:b] (V^T V_b) T_b.
// Outputs as for the other panel kernels: V explicit in place, R into the next
// level's panel, T for the Y = V T product.
//
// Reflector convention: H = I - tau v v^T, v_k = 1, beta = -sign(alpha)*norm,
// tau = (beta - alpha)/beta (Algorithm 3's 2x^2/(x^2+|tail|^2)); a zero tail
// gives tau = 0 instead of the paper's 10*eps rule.
#include "svb_internal.h"
#include "mfma_frag.h"
#include <hip/hip_ext.h>

namespace svb {

namespace {

template <typename C, int NB, int HT> struct PanelBlkGeom {
    static constexpr int NW = NB / 16, NT = NW * 64, H = HT * 16;
    static constexpr int RPT = (H / (4 * NW)) < 16 ? 16 : H / (4 * NW);   // rows per thread in step 2
    static constexpr int NRGU = H / RPT;                                  // row groups in use
    static constexpr int PAD = sizeof(C) == 4 ? 4 : 1;   // keeps 16 lanes on 16 rows off each other's banks
    static constexpr int LDB = H + PAD;                  // block columns: [column][row]
    static constexpr int LDT = 16 + PAD;                 // 16 x 16 blocks
    static constexpr int LDZ = NB + PAD;
    static constexpr int NBLK = NW * (NW + 1) / 2;       // blocks of the upper block triangle of T
    // LDS carve, in elements
    static constexpr int oBs = 0;
    static constexpr int oTs = oBs + 16 * LDB;           // T, block (bi, bj) row-major at blk(bi, bj) * 16 * LDT
    static constexpr int oZs = oTs + NBLK * 16 * LDT;    // Z = (V_w^T V_b) T_b, [column][row]
    static constexpr int oXs = oZs + 16 * LDZ;           // pivot column, two buffers
    static constexpr int XST = RPT + 4;                  // a row group's slot in the pivot-column buffer
    static constexpr int XSB = 4 * NW * XST;             // one buffer (padded: the four groups of a wave on different banks)
    static constexpr int oPart = oXs + 2 * XSB;          // partial inner products, [wave][column]
    static constexpr int oRowk = oPart + NW * 16;        // pivot row, two buffers
    static constexpr int oGs = oRowk + 2 * 16;           // v_c^T v_k inside the block, [k][c]
    static constexpr int oRs = oGs + 16 * 16;            // R block, [column][row]
    static constexpr int oTb = oRs + 16 * LDT;           // T_b, [column][row]
    static constexpr int oTau = oTb + 16 * LDT;
    static constexpr int kElems = oTau + 16;
    static constexpr size_t kSmemBytes = (size_t)kElems * sizeof(C);
    static_assert(RPT % 4 == 0 && NRGU <= 4 * NW, "row split");
    static_assert(kSmemBytes <= 160 * 1024, "LDS");
};

// N consecutive elements to / from 16-byte aligned LDS
template <typename C, int N> __device__ __forceinline__ void lds_ldn(const C* p, C (&o)[N])
{
    constexpr int NV = 16 / (int)sizeof(C);
#pragma unroll
    for (int j = 0; j < N; j += NV) {
        C t[NV];
        VecIO<C, C>::ld(p + j, t);
#pragma unroll
        for (int q = 0; q < NV; ++q) o[j + q] = t[q];
    }
}
template <typename C, int N> __device__ __forceinline__ void lds_stn(C* p, const C (&o)[N])
{
    constexpr int NV = 16 / (int)sizeof(C);
#pragma unroll
    for (int j = 0; j < N; j += NV) {
        C t[NV];
#pragma unroll
        for (int q = 0; q < NV; ++q) t[q] = o[j + q];
        VecIO<C, C>::st(p + j, t);
    }
}

// value of lane (l ^ 1) / (l ^ 2) inside quads of four lanes
template <int CTRL> __device__ __forceinline__ float quad_get(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int CTRL> __device__ __forceinline__ double quad_get(double v)
{
    const long long b = __builtin_bit_cast(long long, v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffll), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)(unsigned)lo);
}
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E;   // quad_perm [1,0,3,2] and [2,3,0,1]

__device__ __forceinline__ int tblk(int bi, int bj) { return bj * (bj + 1) / 2 + bi; }

}  // namespace

// Optional phase timing (compile with -DSVB_PANEL_TIMING): thread 0 of workgroup 0 adds the
// shader-clock cycles of each phase to svb_panel_timing[slot].
#ifdef SVB_PANEL_TIMING
__device__ unsigned long long svb_panel_timing[16];
#define PT_MARK(slot_) do { if (tid == 0 && blockIdx.x == 0) { const unsigned long long now_ = clock64(); \
    atomicAdd(&svb_panel_timing[slot_], now_ - pt_last); pt_last = now_; } } while (0)
#else
#define PT_MARK(slot_) do { } while (0)
#endif

// Where a panel comes from and where its R goes when they are not the work panels: the first
// tree level reads its panel straight from the matrix (QR sweep: element (i, j) of the panel is
// A[row0 + i, col0 + j]; LQ sweep: A[row0 + j, col0 + i]; Asrc points at A[row0, col0]), the
// last level writes its R -- a final piece of the band (Figure 1) -- straight into the packed
// band.  Null pointers select the work panels.
template <typename T, typename C> struct PanelEnds {
    const T* Asrc; int64_t lda; int lq;
    C* band; int64_t ldab, row0, col0;
};

// Hand-over of R between the levels of a panel tree that run at the same time (Section 3.1:
// the tile below is annihilated against the triangle above it -- here a stack of triangles
// against each other).  A domain's R is upper triangular, so its rows 16b .. 16b+15 are final as
// soon as the domain's block step b is done, and block step b of the level above needs exactly
// those rows of its stacked factors and nothing below them.  A domain therefore publishes R tile
// row by tile row (flag = base + number of block steps done), and the level above fetches tile
// row b of every chunk right before its own block step b: it runs one block step behind the level
// below instead of a whole level behind.
// The R tiles travel through device-scope accesses (written through to, and read from, the
// memory level all compute dies share), as the flags do: no cache write-back or invalidate.
struct TreeSync {
    const int* in_flags;   // flags of the level below, indexed by its domain (null: panel complete in memory)
    int* out_flag;         // this domain's flag (null: R is written when the domain is done)
    int base;              // value of a flag before the first block step of this half-sweep
    int spin_limit;        // polls before a wait gives up and raises *err
    int* err;
};
__device__ __forceinline__ int flag_ld(const int* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void flag_st(int* p, int v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// the four entries a lane holds of a 16 x 16 tile of a work panel, through device-scope accesses
template <typename C>
__device__ __forceinline__ typename Frag<C>::acc_t frag_load_dev(const C* P, int64_t ldp, int64_t p0, int64_t q, int gq)
{
    typename Frag<C>::acc_t c;
#pragma unroll
    for (int r = 0; r < 4; ++r)
        c[r] = __hip_atomic_load(&P[p0 + Frag<C>::roff(r, gq) + q * ldp], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return c;
}
template <typename C>
__device__ __forceinline__ void frag_store_dev(C* P, int64_t ldp, int64_t p0, int64_t q, int gq,
                                               const typename Frag<C>::acc_t& c)
{
#pragma unroll
    for (int r = 0; r < 4; ++r)
        __hip_atomic_store(&P[p0 + Frag<C>::roff(r, gq) + q * ldp], c[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// TRI: the panel is a stack of upper triangular NB x NB factors (tree levels above the first).
// Block b's reflectors are then exactly zero in every 16-row tile that lies below block row b
// of its chunk, and both products skip those tiles.
// PIN: the stacked factors arrive tile row by tile row from domains of the level below that are
// still running (TreeSync); d: the domain this workgroup factors.
template <typename T, typename C, int NB, int HT, bool TRI, bool PIN>
__device__ __forceinline__ void panel_blk_body(C* __restrict__ P, int64_t ldp,
                                               C* __restrict__ Tws, int chunks, int g,
                                               C* __restrict__ Pnext, int64_t ldnext,
                                               const PanelEnds<T, C>& ends, const int d, const TreeSync& sy)
{
    static_assert(!PIN || TRI, "only stacks of triangular factors arrive piecewise");
    using F = Frag<C>;
    using G = PanelBlkGeom<C, NB, HT>;
    typedef typename F::acc_t acc_t;
    constexpr int NW = G::NW, NT = G::NT, H = G::H, RPT = G::RPT, NRGU = G::NRGU, XST = G::XST, XSB = G::XSB;
    constexpr int LDB = G::LDB, LDT = G::LDT, LDZ = G::LDZ;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C* sm = reinterpret_cast<C*>(smem_raw);
    C* Bs = sm + G::oBs;
    C* Ts = sm + G::oTs;
    C* Zs = sm + G::oZs;
    C* xs = sm + G::oXs;
    C* part = sm + G::oPart;
    C* rowk = sm + G::oRowk;
    C* Gs = sm + G::oGs;
    C* Rs = sm + G::oRs;
    C* Tb = sm + G::oTb;
    C* taus = sm + G::oTau;

    const int nch = min(g, chunks - d * g);
    const int ntile = nch * NB / 16;              // 16-row tiles that exist (the rest reads as zero)
    C* Pd = P + (int64_t)d * g * NB;
    C* Td = Tws + (int64_t)d * NB * NB;
    C* Rd = Pnext + (int64_t)d * NB;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, gq = lane >> 4;      // MFMA fragment coordinates
    // step 2: column of the block and row group; the four row groups of a wave sit in one quad
    // of lanes, so their partial sums meet through DPP
    const int pc = lane >> 2, prg = 4 * wave + (lane & 3);
    const int64_t mycol = 16 * wave + i;

#ifdef SVB_PANEL_TIMING
    unsigned long long pt_last = clock64();
#endif
    acc_t c[HT];
#pragma unroll
    for (int t = 0; t < HT; ++t) {
        if (!PIN && t < ntile) {
            if (ends.Asrc) {
                const int64_t p0 = (int64_t)d * g * NB + 16 * t;
                c[t] = ends.lq ? frag_load<T, C, true>(ends.Asrc, ends.lda, p0, mycol, gq)
                               : frag_load<T, C, false>(ends.Asrc, ends.lda, p0, mycol, gq);
            } else {
                c[t] = frag_load<C, C, false>(Pd, ldp, 16 * t, mycol, gq);
            }
        }
        else
#pragma unroll
            for (int r = 0; r < 4; ++r) c[t][r] = 0;
    }
    for (int idx = tid; idx < G::NBLK * 16 * LDT; idx += NT) Ts[idx] = 0;

    PT_MARK(0);
    for (int b = 0; b < NW; ++b) {
        if constexpr (PIN) {
            // ---- 0. tile row b of every stacked factor, once the domain below has published it
            if (tid < nch) {
                const int need = sy.base + b + 1;
                int spins = 0;
                while (flag_ld(&sy.in_flags[d * g + tid]) < need) {
                    if (++spins > sy.spin_limit) {
                        atomicExch(sy.err, 1);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            __syncthreads();
            if (wave >= b) {
#pragma unroll
                for (int t = 0; t < HT; ++t)
                    if (t % NW == b && t < ntile) c[t] = frag_load_dev<C>(Pd, ldp, 16 * t, mycol, gq);
            }
        }
        // ---- 1. the owner's columns (rows 16b ..) to LDS
        if (wave == b) {
#pragma unroll
            for (int t = 0; t < HT; ++t)
                if (t >= b) {
                    const C o[4] = {c[t][0], c[t][1], c[t][2], c[t][3]};
                    F::st4(&Bs[i * LDB + 16 * t], gq, o);
                }
        }
        __syncthreads();
        PT_MARK(1);

        // ---- 2. Householder QR of the block: thread (pc, prg) holds rows 16b + prg*RPT + r of column pc
        const int rbase = 16 * b + prg * RPT;
        const bool rows_on = NRGU == 4 * NW || prg < NRGU;   // compile-time true unless row groups are spare
        // (a 16-byte vector never straddles row H: rbase and H are multiples of 16)
        constexpr bool kVecB = sizeof(C) == 4;   // f64 block columns have an odd row length
        C a[RPT];
        if (rows_on) {
            if constexpr (kVecB) {
#pragma unroll
                for (int r = 0; r < RPT; r += 4) {
                    C t4[4] = {0, 0, 0, 0};
                    if (rbase + r < H) lds_ldn<C, 4>(&Bs[pc * LDB + rbase + r], t4);
#pragma unroll
                    for (int q = 0; q < 4; ++q) a[r + q] = t4[q];
                }
            } else {
#pragma unroll
                for (int r = 0; r < RPT; ++r) a[r] = (rbase + r < H) ? Bs[pc * LDB + rbase + r] : (C)0;
            }
        } else {
#pragma unroll
            for (int r = 0; r < RPT; ++r) a[r] = 0;
        }
        C my_inv = 0;
        PT_MARK(2);
#pragma unroll
        for (int ki = 0; ki < 16; ++ki) {
            const int buf = ki & 1;
            if (prg == 0) rowk[buf * 16 + pc] = a[ki];
            if (pc == ki && rows_on) {
                C o[RPT];
#pragma unroll
                for (int r = 0; r < RPT; ++r) o[r] = (prg == 0 && r <= ki) ? (C)0 : a[r];
                lds_stn<C, RPT>(&xs[buf * XSB + prg * XST], o);
            }
            __syncthreads();
            C x[RPT];
            C p = 0;
            if (rows_on) {
                lds_ldn<C, RPT>(&xs[buf * XSB + prg * XST], x);
                C p4[4] = {0, 0, 0, 0};
#pragma unroll
                for (int r = 0; r < RPT; ++r) p4[r & 3] += x[r] * a[r];
                p = (p4[0] + p4[1]) + (p4[2] + p4[3]);
            } else {
#pragma unroll
                for (int r = 0; r < RPT; ++r) x[r] = 0;
            }
            p += quad_get<kQuadXor1>(p);
            p += quad_get<kQuadXor2>(p);
            if ((lane & 3) == 0) part[wave * 16 + pc] = p;
            __syncthreads();
            C D = 0, ss = 0;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                D += part[w * 16 + pc];
                ss += part[w * 16 + ki];
            }
            const C alpha = rowk[buf * 16 + ki], akc = rowk[buf * 16 + pc];
            C tau, beta, inv;
            if (ss == (C)0) {
                tau = 0; beta = alpha; inv = 0;
            } else {
                const C nrm = newton_sqrt(alpha * alpha + ss);
                beta = alpha >= (C)0 ? -nrm : nrm;
                tau = (beta - alpha) * newton_rcp(beta);
                inv = newton_rcp(alpha - beta);
            }
            const C wk = akc + inv * D;   // v_k^T (column pc), v_k's tail taken unscaled times inv
            const C f = tau * wk;
            if (prg == 0) {
                if (pc < ki) Gs[ki * 16 + pc] = my_inv * wk;   // v_pc^T v_k (v_pc's tail is stored unscaled)
                if (pc == ki) taus[ki] = tau;
            }
            if (pc == ki) my_inv = inv;
            if (prg == 0) a[ki] = (pc > ki) ? akc - f : ((pc == ki) ? beta : akc);
            if (pc > ki && tau != (C)0) {
                const C coef = f * inv;
#pragma unroll
                for (int r = 0; r < RPT; ++r) a[r] -= coef * x[r];   // x is zero at and above the pivot row
            }
        }
        PT_MARK(3);
        // explicit V block (unit diagonal, zeros above) back to LDS; R block aside
        if (rows_on) {
            C v[RPT];
#pragma unroll
            for (int r = 0; r < RPT; ++r) {
                const int rel = prg * RPT + r;
                v[r] = a[r] * my_inv;
                if (rel < 16) v[r] = rel < pc ? (C)0 : (rel == pc ? (C)1 : v[r]);
            }
            if constexpr (kVecB) {
#pragma unroll
                for (int r = 0; r < RPT; r += 4) {
                    const C t4[4] = {v[r], v[r + 1], v[r + 2], v[r + 3]};
                    if (rbase + r < H) lds_stn<C, 4>(&Bs[pc * LDB + rbase + r], t4);
                }
            } else {
#pragma unroll
                for (int r = 0; r < RPT; ++r)
                    if (rbase + r < H) Bs[pc * LDB + rbase + r] = v[r];
            }
        }
        if (prg == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) Rs[pc * LDT + r] = (r <= pc) ? a[r] : (C)0;
        }
        __syncthreads();
        PT_MARK(4);

        // ---- 3./4. first product with V_b (every wave but the owner); the owner builds T_b
        acc_t p1;
#pragma unroll
        for (int r = 0; r < 4; ++r) p1[r] = 0;
        if (wave == b) {
            // T_b: T[k][k] = tau_k, T[i][k] = -tau_k sum_{j=i}^{k-1} T[i][j] (v_j^T v_k); lane i keeps
            // row i in registers (zero left of the diagonal), so a column costs no exchange
            C trow[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                C acc = 0;
                if (k > 0) {
                    C gk[16];
                    lds_ldn<C, 16>(&Gs[k * 16], gk);
#pragma unroll
                    for (int j = 0; j < k; ++j) acc += trow[j] * gk[j];
                }
                const C tk = taus[k];
                trow[k] = (k == i) ? tk : (k > i ? -tk * acc : (C)0);
            }
            if (gq == 0) {
                C* Tbb = Ts + tblk(b, b) * 16 * LDT;
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    Tb[k * LDT + i] = trow[k];
                    Tbb[i * LDT + k] = trow[k];
                }
            }
        } else {
            // P1 = V_b^T C_w over rows 16b ..: C_w's registers are the B operand
            acc_t pa, pb;
#pragma unroll
            for (int r = 0; r < 4; ++r) { pa[r] = 0; pb[r] = 0; }
#pragma unroll
            for (int t = 0; t < HT; ++t) {
                if (t >= b && t < ntile && (!TRI || (t % (NB / 16)) <= b)) {
                    C o[4];
                    F::ld4(&Bs[i * LDB + 16 * t], gq, o);
                    if (t & 1) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) pb = F::mma(o[r], c[t][r], pb);
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r) pa = F::mma(o[r], c[t][r], pa);
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) p1[r] = pa[r] + pb[r];
        }
        __syncthreads();
        PT_MARK(5);

        // ---- right of the block: C_w -= V_b (T_b^T P1);  left of it: Z_w = (V_w^T V_b) T_b;
        //      the owner meanwhile reloads its registers
        if (wave == b) {
            // registers: tile b <- R block, tiles below <- V; V goes to global memory on the way
#pragma unroll
            for (int t = 0; t < HT; ++t) {
                if (t < ntile) {
                    if (t < b) {
                        acc_t z;
#pragma unroll
                        for (int r = 0; r < 4; ++r) z[r] = 0;
                        frag_store<C, C, false>(Pd, ldp, 16 * t, mycol, gq, z);
                    } else {
                        C o[4];
                        F::ld4(&Bs[i * LDB + 16 * t], gq, o);
                        acc_t v;
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = o[r];
                        frag_store<C, C, false>(Pd, ldp, 16 * t, mycol, gq, v);
                        if (t == b) {
                            F::ld4(&Rs[i * LDT], gq, o);
#pragma unroll
                            for (int r = 0; r < 4; ++r) v[r] = o[r];
                        }
                        c[t] = v;
                    }
                }
            }
        } else {
            C tb[4];
            F::ld4(&Tb[i * LDT], gq, tb);   // T_b[roff(r, gq)][i]
            if (wave > b) {
                acc_t w;
#pragma unroll
                for (int r = 0; r < 4; ++r) w[r] = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) w = F::mma(tb[r], p1[r], w);
#pragma unroll
                for (int r = 0; r < 4; ++r) w[r] = -w[r];
#pragma unroll
                for (int t = 0; t < HT; ++t) {
                    if (t >= b && t < ntile && (!TRI || (t % (NB / 16)) <= b)) {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            c[t] = F::mma(Bs[F::roff(r, gq) * LDB + 16 * t + i], w[r], c[t]);
                    }
                }
            } else {
                acc_t z;
#pragma unroll
                for (int r = 0; r < 4; ++r) z[r] = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) z = F::mma(p1[r], tb[r], z);
                const C o[4] = {z[0], z[1], z[2], z[3]};
                F::st4(&Zs[i * LDZ + 16 * wave], gq, o);
            }
        }
        if (sy.out_flag) {
            // rows 16b .. 16b+15 of R are final (no later block touches them): hand them over
            if (wave >= b) {
#pragma unroll
                for (int t = 0; t < NW; ++t)
                    if (t == b) frag_store_dev<C>(Rd, ldnext, 16 * t, mycol, gq, c[t]);
            }
            __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): the stores have been acknowledged
        }
        __syncthreads();
        if (sy.out_flag && tid == 0) flag_st(sy.out_flag, sy.base + b + 1);
        PT_MARK(6);

        // ---- T[wave, b] = - sum_{w2 = wave}^{b-1} T[wave, w2] Z_w2
        if (wave < b) {
            acc_t tn;
#pragma unroll
            for (int r = 0; r < 4; ++r) tn[r] = 0;
            for (int w2 = wave; w2 < b; ++w2) {
                C ta[4], zb[4];
                F::ld4(&Ts[tblk(wave, w2) * 16 * LDT + i * LDT], gq, ta);
                F::ld4(&Zs[i * LDZ + 16 * w2], gq, zb);
#pragma unroll
                for (int r = 0; r < 4; ++r) tn = F::mma(ta[r], zb[r], tn);
            }
            C* Tn = Ts + tblk(wave, b) * 16 * LDT;
#pragma unroll
            for (int r = 0; r < 4; ++r) Tn[F::roff(r, gq) * LDT + i] = -tn[r];
        }
    }

    PT_MARK(7);
    // R: rows 0 .. NB-1 of the factored domain, zero below the diagonal
#pragma unroll
    for (int t = 0; t < NW; ++t) {
        if (ends.band) {
            // upper triangle of R into the band: entry (ri, cj) of R is band entry
            // (row0 + ri, col0 + cj) in a QR sweep, (row0 + cj, col0 + ri) in an LQ sweep
            if (t <= wave) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int64_t ri = 16 * t + F::roff(r, gq), cj = mycol;
                    if (ri <= cj) {
                        const int64_t gi = ends.lq ? ends.row0 + cj : ends.row0 + ri;
                        const int64_t gj = ends.lq ? ends.col0 + ri : ends.col0 + cj;
                        ends.band[(gi - gj + 2 * NB - 1) + gj * ends.ldab] = c[t][r];
                    }
                }
            }
        } else if (!sy.out_flag) {
            acc_t v;
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = (t <= wave) ? c[t][r] : (C)0;
            frag_store<C, C, false>(Rd, ldnext, 16 * t, mycol, gq, v);
        }
    }
    __syncthreads();
    for (int idx = tid; idx < NB * NB; idx += NT) {
        const int ii = idx % NB, jj = idx / NB;
        const int bi = ii / 16, bj = jj / 16;
        Td[ii + jj * NB] = bi <= bj ? Ts[tblk(bi, bj) * 16 * LDT + (ii % 16) * LDT + (jj % 16)] : (C)0;
    }
    PT_MARK(8);
}
#undef PT_MARK

template <typename C> constexpr int panel_blk_tiles() { return sizeof(C) == 4 ? 32 : 16; }

template <typename C> int panel_blk_rows() { return panel_blk_tiles<C>() * 16; }
template int panel_blk_rows<float>();
template int panel_blk_rows<double>();

// One tree level: workgroup d factors domain d.  out_flags (may be null): the domains' hand-over
// flags for a level above that runs at the same time (TreeSync).
template <typename T, typename C, int NB, int HT, bool TRI>
__global__ __launch_bounds__(NB * 4) void panel_qr_blk_kernel(C* __restrict__ P, int64_t ldp,
                                                              C* __restrict__ Tws, int chunks, int g,
                                                              C* __restrict__ Pnext, int64_t ldnext,
                                                              PanelEnds<T, C> ends, int* out_flags, int flag_base)
{
    const int d = blockIdx.x;
    const TreeSync sy{nullptr, out_flags ? out_flags + d : nullptr, flag_base, 0, nullptr};
    panel_blk_body<T, C, NB, HT, TRI, false>(P, ldp, Tws, chunks, g, Pnext, ldnext, ends, d, sy);
}

// One domain of a tree level above the first: ticket tk of the upper levels' launch (tickets are
// numbered level by level, so the domains a workgroup waits for hold smaller tickets and are
// already running or done).
template <typename C, int NB>
__device__ __forceinline__ void panel_tree_item(const PanelTreeArgs<C>& a, const int tk)
{
    constexpr int HT = panel_blk_tiles<C>();
    int L = 0;
    while (L + 1 < a.nl && tk >= a.lv[L + 1].first) ++L;
    const PanelTreeLevel<C>& lv = a.lv[L];
    const int d = tk - lv.first;
    const bool last = L == a.nl - 1;
    const TreeSync sy{a.flags + lv.flags_in, last ? nullptr : a.flags + lv.flags_out + d, a.flag_base, a.spin_limit,
                      a.err};
    const PanelEnds<C, C> ends{nullptr, 0, a.lq, last ? a.band : nullptr, a.ldab, a.row0, a.col0};
    // a short stack near the top of the tree runs the body sized for it (fewer rows per thread in
    // the reflector steps, fewer tiles in the block products)
    if constexpr (HT / 4 * 16 >= NB) {
        if (lv.tiles <= HT / 4) {
            panel_blk_body<C, C, NB, HT / 4, true, true>(lv.P, lv.ldp, lv.Tws, lv.chunks, a.g, lv.Pnext, lv.ldnext, ends, d, sy);
            return;
        }
    }
    if constexpr (HT / 2 * 16 >= NB) {
        if (lv.tiles <= HT / 2) {
            panel_blk_body<C, C, NB, HT / 2, true, true>(lv.P, lv.ldp, lv.Tws, lv.chunks, a.g, lv.Pnext, lv.ldnext, ends, d, sy);
            return;
        }
    }
    panel_blk_body<C, C, NB, HT, true, true>(lv.P, lv.ldp, lv.Tws, lv.chunks, a.g, lv.Pnext, lv.ldnext, ends, d, sy);
}

// Every tree level above the first in one launch, running beside the first level's kernel, one
// ticket per workgroup.
// The launch must not occupy the machine while the first level's kernel cannot run (a tool that
// lets one kernel execute at a time would otherwise leave these workgroups waiting for flags that
// never move): a workgroup draws its ticket only once the first level's kernel has announced
// itself, and leaves without one if that does not happen within start_spin polls.  Tickets left
// undrawn are taken by the workgroups of the first level's kernel when they are done with their
// own domains (panel_first_kernel), so the tree is complete when that kernel is, whichever of the
// two launches ran first.
template <typename C, int NB>
__global__ __launch_bounds__(NB * 4) void panel_tree_kernel(PanelTreeArgs<C> a)
{
    __shared__ int sh_ticket;
    if (threadIdx.x == 0) {
        bool go = true;
        int spins = 0;
        while (flag_ld(a.started) < a.flag_base) {
            if (++spins > a.start_spin) {
                go = false;
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        sh_ticket = go ? atomicAdd(a.ticket, 1) : a.total;
    }
    __syncthreads();
    const int tk = sh_ticket;
    if (tk >= a.total) return;
    panel_tree_item<C, NB>(a, tk);
}

// The first tree level of a tree whose upper levels run in panel_tree_kernel beside it: workgroup
// d announces the kernel, factors domain d of the panel read straight from the matrix, handing
// its R over block step by block step, and then takes whatever tickets of the upper levels are
// still undrawn (none, unless the other launch could not run beside this one).
template <typename T, typename C, int NB>
__global__ __launch_bounds__(NB * 4) void panel_first_kernel(C* __restrict__ P, int64_t ldp, C* __restrict__ Tws,
                                                             int chunks, C* __restrict__ Pnext, int64_t ldnext,
                                                             PanelEnds<T, C> ends, int* out_flags, PanelTreeArgs<C> a)
{
    constexpr int HT = panel_blk_tiles<C>();
    __shared__ int sh_ticket;
    const int d = blockIdx.x;
    if (threadIdx.x == 0) flag_st(a.started, a.flag_base);
    const TreeSync sy{nullptr, out_flags + d, a.flag_base, 0, nullptr};
    panel_blk_body<T, C, NB, HT, false, false>(P, ldp, Tws, chunks, a.g, Pnext, ldnext, ends, d, sy);
    for (;;) {
        __syncthreads();
        if (threadIdx.x == 0) sh_ticket = flag_ld(a.ticket) < a.total ? atomicAdd(a.ticket, 1) : a.total;
        __syncthreads();
        const int tk = sh_ticket;
        if (tk >= a.total) break;
        panel_tree_item<C, NB>(a, tk);
    }
}

__global__ void fill_int_kernel(int* p, int n, int v)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = v;
}
// a raised error flag of the panel tree (an expired wait) becomes a NaN in the band, which the
// later stages carry into the result's status
template <typename C> __global__ void tree_err_kernel(const int* err, C* band_entry)
{
    if (*err) *band_entry = (C)NAN;
}

void launch_fill_int(int* p, int n, int v, hipStream_t s)
{
    if (n > 0) hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)((n + 255) / 256 < 64 ? (n + 255) / 256 : 64)), dim3(256), 0, s, p, n, v);
}
template <typename C> void launch_tree_err(const int* err, C* band_entry, hipStream_t s)
{
    hipLaunchKernelGGL(tree_err_kernel<C>, dim3(1), dim3(1), 0, s, err, band_entry);
}
template void launch_tree_err<float>(const int*, float*, hipStream_t);
template void launch_tree_err<double>(const int*, double*, hipStream_t);

template <typename C, int NB>
static void launch_tree_nb(const PanelTreeArgs<C>& a, hipStream_t s, hipEvent_t start, hipEvent_t done)
{
    using G = PanelBlkGeom<C, NB, panel_blk_tiles<C>()>;
    auto kern = panel_tree_kernel<C, NB>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)G::kSmemBytes);
        attr_set = true;
    }
    if (done)
        hipExtLaunchKernelGGL(kern, dim3((unsigned)a.total), dim3(G::NT), (uint32_t)G::kSmemBytes, s, start, done, 0u, a);
    else
        hipLaunchKernelGGL(kern, dim3((unsigned)a.total), dim3(G::NT), G::kSmemBytes, s, a);
}

template <typename C>
void launch_panel_tree(int nb, const PanelTreeArgs<C>& a, hipStream_t s, hipEvent_t start, hipEvent_t done)
{
    switch (nb) {
    case 32: launch_tree_nb<C, 32>(a, s, start, done); break;
    case 64: launch_tree_nb<C, 64>(a, s, start, done); break;
    default: launch_tree_nb<C, 128>(a, s, start, done); break;
    }
}
template void launch_panel_tree<float>(int, const PanelTreeArgs<float>&, hipStream_t, hipEvent_t, hipEvent_t);
template void launch_panel_tree<double>(int, const PanelTreeArgs<double>&, hipStream_t, hipEvent_t, hipEvent_t);

template <typename T, typename C, int NB, int HT, bool TRI>
static void launch_blk_ht(C* P, int64_t ldp, C* Tws, int chunks, int g, C* Pnext, int64_t ldnext,
                          const PanelEnds<T, C>& ends, int* out_flags, int flag_base, hipStream_t s,
                          hipEvent_t done, hipEvent_t start)
{
    using G = PanelBlkGeom<C, NB, HT>;
    auto kern = panel_qr_blk_kernel<T, C, NB, HT, TRI>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)G::kSmemBytes);
        attr_set = true;
    }
    const int domains = (chunks + g - 1) / g;
    // `done` (and `start`): events tied to this launch's own completion (and start): no separate
    // marker in the stream between this kernel and the next one
    if (done)
        hipExtLaunchKernelGGL(kern, dim3(domains), dim3(G::NT), (uint32_t)G::kSmemBytes, s, start, done, 0u, P, ldp,
                              Tws, chunks, g, Pnext, ldnext, ends, out_flags, flag_base);
    else
        hipLaunchKernelGGL(kern, dim3(domains), dim3(G::NT), G::kSmemBytes, s, P, ldp, Tws, chunks, g, Pnext, ldnext,
                           ends, out_flags, flag_base);
}

template <typename T, typename C, int NB>
static void launch_blk(C* P, int64_t ldp, C* Tws, int chunks, int g, C* Pnext, int64_t ldnext,
                       const PanelEnds<T, C>& ends, int* out_flags, int flag_base, const PanelTreeArgs<C>* tree,
                       hipStream_t s, hipEvent_t done, hipEvent_t start)
{
    constexpr int HT = panel_blk_tiles<C>();
    if (ends.Asrc && tree) {
        // first level of a tree whose upper levels run beside it
        using G = PanelBlkGeom<C, NB, HT>;
        auto kern = panel_first_kernel<T, C, NB>;
        static bool attr_set = false;
        if (!attr_set) {
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)G::kSmemBytes);
            attr_set = true;
        }
        const int domains = (chunks + g - 1) / g;
        if (done)
            hipExtLaunchKernelGGL(kern, dim3(domains), dim3(G::NT), (uint32_t)G::kSmemBytes, s, start, done, 0u, P, ldp,
                                  Tws, chunks, Pnext, ldnext, ends, out_flags, *tree);
        else
            hipLaunchKernelGGL(kern, dim3(domains), dim3(G::NT), G::kSmemBytes, s, P, ldp, Tws, chunks, Pnext, ldnext,
                               ends, out_flags, *tree);
        return;
    }
    // a panel that does not come from the matrix is a stack of triangular factors; near the top of
    // the tree such a stack is short, and a kernel sized for it (fewer rows per thread in the
    // reflector steps, fewer tiles in the block products) is faster than the full-height one
    if (ends.Asrc) {
        launch_blk_ht<T, C, NB, HT, false>(P, ldp, Tws, chunks, g, Pnext, ldnext, ends, out_flags, flag_base, s, done, start);
        return;
    }
    const int need = (chunks < g ? chunks : g) * NB / 16;   // tiles of the tallest domain
    if constexpr (HT / 4 * 16 >= NB) {
        if (need <= HT / 4) {
            launch_blk_ht<T, C, NB, HT / 4, true>(P, ldp, Tws, chunks, g, Pnext, ldnext, ends, out_flags, flag_base, s, done, start);
            return;
        }
    }
    if constexpr (HT / 2 * 16 >= NB) {
        if (need <= HT / 2) {
            launch_blk_ht<T, C, NB, HT / 2, true>(P, ldp, Tws, chunks, g, Pnext, ldnext, ends, out_flags, flag_base, s, done, start);
            return;
        }
    }
    launch_blk_ht<T, C, NB, HT, true>(P, ldp, Tws, chunks, g, Pnext, ldnext, ends, out_flags, flag_base, s, done, start);
}

template <typename T, typename C>
void launch_panel_blk(int nb, C* P, int64_t ldp, C* Tws, int chunks, int g, C* Pnext, int64_t ldnext,
                      const T* Asrc, int64_t lda, bool lq, C* band, int64_t ldab, int64_t row0, int64_t col0,
                      hipStream_t s, hipEvent_t done, hipEvent_t start, int* out_flags, int flag_base,
                      const PanelTreeArgs<C>* tree)
{
    const PanelEnds<T, C> ends{Asrc, lda, lq ? 1 : 0, band, ldab, row0, col0};
    switch (nb) {
    case 32: launch_blk<T, C, 32>(P, ldp, Tws, chunks, g, Pnext, ldnext, ends, out_flags, flag_base, tree, s, done, start); break;
    case 64: launch_blk<T, C, 64>(P, ldp, Tws, chunks, g, Pnext, ldnext, ends, out_flags, flag_base, tree, s, done, start); break;
    default: launch_blk<T, C, 128>(P, ldp, Tws, chunks, g, Pnext, ldnext, ends, out_flags, flag_base, tree, s, done, start); break;
    }
}

template void launch_panel_blk<float, float>(int, float*, int64_t, float*, int, int, float*, int64_t, const float*, int64_t, bool, float*, int64_t, int64_t, int64_t, hipStream_t, hipEvent_t, hipEvent_t, int*, int, const PanelTreeArgs<float>*);
template void launch_panel_blk<__half, float>(int, float*, int64_t, float*, int, int, float*, int64_t, const __half*, int64_t, bool, float*, int64_t, int64_t, int64_t, hipStream_t, hipEvent_t, hipEvent_t, int*, int, const PanelTreeArgs<float>*);
template void launch_panel_blk<bf16_t, float>(int, float*, int64_t, float*, int, int, float*, int64_t, const bf16_t*, int64_t, bool, float*, int64_t, int64_t, int64_t, hipStream_t, hipEvent_t, hipEvent_t, int*, int, const PanelTreeArgs<float>*);
template void launch_panel_blk<double, double>(int, double*, int64_t, double*, int, int, double*, int64_t, const double*, int64_t, bool, double*, int64_t, int64_t, int64_t, hipStream_t, hipEvent_t, hipEvent_t, int*, int, const PanelTreeArgs<double>*);

}  // namespace svb
