// Stage 1, panel factorisation (paper Section 3.1 Algorithm 1 lines 2/4 and
// Section 3.2 "Panel Factorization", Algorithm 3).
//
// A panel (the block column below a diagonal tile in a QR sweep, the block row
// right of it in an LQ sweep) is copied, transposed for LQ, into a contiguous
// work panel.  Its nb-row tiles ("chunks") are grouped into domains of g
// chunks; every domain is factored by one workgroup with Householder
// reflectors (GEQRT extended to several tiles), the R factors of the domains
// are stacked into the next level's panel and factored the same way (the
// role of TSQRT: annihilating tiles against an already triangular one), until
// one R is left.  Each domain also produces the compact-WY pair (V, Y = V T)
// that the trailing update applies with matrix products.
#include "svb_internal.h"
#include "mfma_gemm.h"

namespace svb {

template <typename C> __device__ __forceinline__ C wave_sum(C v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// ---------------------------------------------------------------- gather
// QR sweep: P[i, j] = A[row0 + i, col0 + j];  LQ sweep: P[i, j] = A[row0 + j, col0 + i]
// for i < len, j < nb.  Block (32, 8) moves a 32 x 32 tile through LDS so that
// both the read and the write run along contiguous memory.
template <typename T, typename C>
__global__ __launch_bounds__(256) void panel_gather_kernel(const T* __restrict__ A, int64_t lda,
                                                           int64_t row0, int64_t col0, int lq,
                                                           int64_t len, int nb,
                                                           C* __restrict__ P, int64_t ldp)
{
    __shared__ C tile[32][33];
    const int64_t i0 = (int64_t)blockIdx.x * 32;
    const int j0 = blockIdx.y * 32;
    const int tx = threadIdx.x, ty = threadIdx.y;
    if (!lq) {
        for (int jj = ty; jj < 32; jj += 8) {
            int64_t i = i0 + tx;
            if (i < len) P[i + (int64_t)(j0 + jj) * ldp] = ld_as<C, T>(&A[(row0 + i) + (col0 + j0 + jj) * lda]);
        }
    } else {
        // read: tx runs along j (rows of A, contiguous), ty along i (columns of A)
        for (int ii = ty; ii < 32; ii += 8) {
            int64_t i = i0 + ii;
            if (i < len) tile[ii][tx] = ld_as<C, T>(&A[(row0 + j0 + tx) + (col0 + i) * lda]);
        }
        __syncthreads();
        for (int jj = ty; jj < 32; jj += 8) {
            int64_t i = i0 + tx;
            if (i < len) P[i + (int64_t)(j0 + jj) * ldp] = tile[tx][jj];
        }
    }
}

template <typename T, typename C>
void launch_panel_gather(const T* A, int64_t lda, int64_t row0, int64_t col0, bool lq,
                         int64_t len, int nb, C* P, int64_t ldp, hipStream_t s)
{
    dim3 grid((unsigned)((len + 31) / 32), (unsigned)(nb / 32));
    dim3 block(32, 8);
    hipLaunchKernelGGL((panel_gather_kernel<T, C>), grid, block, 0, s, A, lda, row0, col0,
                       lq ? 1 : 0, len, nb, P, ldp);
}

// ---------------------------------------------------------------- domain QR
// One workgroup factors one domain (h = nch*NB rows, NB columns) in place in
// the work panel.  Per column k (Algorithm 3's loop): the tail norm, the
// reflector scalars, then every other column is visited once by one wave: a
// column right of k gets the rank-one update, a column left of k (already a
// reflector) yields the inner product needed for the next column of T.
// Reflector convention: H = I - tau v v^T, v_k = 1, beta = -sign(alpha)*norm,
// tau = (beta - alpha)/beta (equal to Algorithm 3's 2x^2/(x^2+|tail|^2)); a
// zero tail gives tau = 0 instead of the paper's 10*eps rule.
template <typename C, int NB, int NT>
__global__ __launch_bounds__(NT) void panel_qr_kernel(C* __restrict__ P, int64_t ldp,
                                                      C* __restrict__ Y, C* __restrict__ Tws,
                                                      int chunks, int g,
                                                      C* __restrict__ Pnext, int64_t ldnext)
{
    constexpr int NW = NT / kWave;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    C* vs = reinterpret_cast<C*>(smem_raw);  // h entries
    __shared__ C zs[NB];
    __shared__ C red[NW];

    const int d = blockIdx.x;
    const int nch = min(g, chunks - d * g);
    const int h = nch * NB;
    C* Pd = P + (int64_t)d * g * NB;
    C* Yd = Y + (int64_t)d * g * NB;
    C* Td = Tws + (int64_t)d * NB * NB;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;

    for (int k = 0; k < NB; ++k) {
        C* colk = Pd + (int64_t)k * ldp;
        // 1. squared norm of the tail, and the pivot
        C ss = 0;
        for (int i = k + 1 + tid; i < h; i += NT) {
            C x = colk[i];
            ss += x * x;
        }
        const C alpha = colk[k];
        ss = wave_sum(ss);
        if (lane == 0) red[wave] = ss;
        __syncthreads();
        ss = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) ss += red[w];
        C tau, beta, inv;
        if (ss == (C)0) {
            tau = 0;
            beta = alpha;
            inv = 0;
        } else {
            C nrm = sqrt(alpha * alpha + ss);
            beta = alpha >= (C)0 ? -nrm : nrm;
            tau = (beta - alpha) / beta;
            inv = (C)1 / (alpha - beta);
        }
        // 2. v = (0.., 1, tail/(alpha-beta)) to LDS and in place
        for (int i = tid; i < h; i += NT) {
            C v = (i < k) ? (C)0 : ((i == k) ? (C)1 : colk[i] * inv);
            vs[i] = v;
            if (i > k) colk[i] = v;
        }
        if (tid == 0) colk[k] = beta;
        __syncthreads();
        // 3. one wave per column
        const int i0 = (k / kWave) * kWave;
        for (int j = wave; j < NB; j += NW) {
            if (j == k) continue;
            C* colj = Pd + (int64_t)j * ldp;
            C dot = 0;
            for (int i = i0 + lane; i < h; i += kWave) dot += vs[i] * colj[i];
            dot = wave_sum(dot);
            if (j < k) {
                if (lane == 0) zs[j] = dot;
            } else {
                const C f = tau * dot;
                for (int i = i0 + lane; i < h; i += kWave) {
                    C v = vs[i];
                    if (v != (C)0) colj[i] -= f * v;
                }
            }
        }
        __syncthreads();
        // 4. column k of T: T[0:k,k] = -tau * T[0:k,0:k] * (V[:,0:k]^T v_k), T[k,k] = tau
        if (tid < k) {
            C acc = 0;
            for (int j = tid; j < k; ++j) acc += Td[tid + j * NB] * zs[j];
            Td[tid + k * NB] = -tau * acc;
        } else if (tid == k) {
            Td[k + k * NB] = tau;
        }
    }
    __syncthreads();
    // R (upper triangle of the top tile) becomes chunk d of the next level's panel
    for (int idx = tid; idx < NB * NB; idx += NT) {
        const int i = idx % NB, j = idx / NB;
        Pnext[((int64_t)d * NB + i) + (int64_t)j * ldnext] = (i <= j) ? Pd[i + (int64_t)j * ldp] : (C)0;
    }
    __syncthreads();
    // make V explicit: unit diagonal, zeros above it
    for (int idx = tid; idx < NB * NB; idx += NT) {
        const int i = idx % NB, j = idx / NB;
        if (i < j) Pd[i + (int64_t)j * ldp] = 0;
        else if (i == j) Pd[i + (int64_t)j * ldp] = 1;
    }
    __syncthreads();
    // Y = V T (T upper triangular)
    for (int i = tid; i < h; i += NT) {
        for (int k = 0; k < NB; ++k) {
            C acc = 0;
            for (int j = 0; j <= k; ++j) acc += Pd[i + (int64_t)j * ldp] * Td[j + k * NB];
            Yd[i + (int64_t)k * ldp] = acc;
        }
    }
}

// ---------------------------------------------------------------- domain QR, register resident
// The production panel kernel.  The whole domain (h <= HMAX = (NT/NB)*RPT rows,
// NB columns) lives in registers: thread (c, rg) = (tid % NB, tid / NB) holds
// rows rg*RPT .. rg*RPT+RPT-1 of column c (the paper's GEQRT, Algorithm 3, keeps
// one tile column per thread in the same way; here a column is additionally
// split over NT/NB threads, the role of the paper's SPLITK).  Per reflector k:
//   - the thread(s) of column k publish the pivot column in LDS, the row group
//     that owns row k publishes row k;
//   - every thread forms the inner product of its rows with the pivot column;
//     partial sums meet in LDS (column k's own sum is the squared tail norm);
//   - every thread derives beta, tau and updates its rows (Algorithm 3's
//     rho / rho' step); columns left of k record v_c^T v_k for the T factor.
// Two barriers per reflector; the reflector tails stay unscaled in registers
// (each column remembers its scale) until they are written out.  Reflectors are
// processed in blocks of 8 whose pivot rows sit at fixed register positions.
// Afterwards T is built in LDS from the recorded inner products (the LAPACK
// larft recurrence, rows in parallel) and written to Tws for the Y = V T product.
template <typename C, int NB, int RPT, int NT>
__global__ __launch_bounds__(NT) void panel_qr_reg_kernel(C* __restrict__ P, int64_t ldp,
                                                          C* __restrict__ Tws, int chunks, int g,
                                                          C* __restrict__ Pnext, int64_t ldnext)
{
    constexpr int NRG = NT / NB, HMAX = NRG * RPT, LT = NT / NB;  // LT lanes cooperate on one row of T
    extern __shared__ __align__(16) unsigned char smem_raw[];
    // G (NB x NB, column k holds v_c^T v_k for c < k) sits in LDS when it fits next to T,
    // otherwise in the second half of this domain's slot of Tws
    constexpr bool G_GLOBAL = sizeof(C) * (size_t)(NB * (NB + 1) + NB * NB) > 140 * 1024;
    C* Ts = reinterpret_cast<C*>(smem_raw);       // NB x (NB+1)
    C* Gs = G_GLOBAL ? Tws + ((int64_t)gridDim.x + blockIdx.x) * NB * NB : Ts + NB * (NB + 1);
    C* xs = Ts + NB * (NB + 1) + (G_GLOBAL ? 0 : NB * NB);  // 2 x HMAX
    C* part = xs + 2 * HMAX;                      // NRG x NB
    C* rowk = part + NRG * NB;                    // 2 x NB
    C* taus = rowk + 2 * NB;                      // NB

    const int d = blockIdx.x;
    const int nch = min(g, chunks - d * g);
    const int h = nch * NB;
    C* Pd = P + (int64_t)d * g * NB;
    C* Td = Tws + (int64_t)d * NB * NB;
    const int tid = threadIdx.x;
    const int c = tid % NB, rg = tid / NB, row0 = rg * RPT;

    C a[RPT];
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int row = row0 + r;
        a[r] = row < h ? Pd[row + (int64_t)c * ldp] : (C)0;
    }
    C my_inv = 0;

    // Reflectors are taken KB at a time.  Inside a block the pivot rows are registers
    // a[0] .. a[KB-1] of the row group that owns them (compile-time indices: a run-time
    // register index would cost a select per register and reflector); after the block those
    // KB rows are final, are written out, and the group's registers move down by KB.  The
    // pivot column is exchanged in register order (xs[row0 + i] belongs to a[i]), so the
    // moving frame of the pivot group never shows in an LDS index.
    constexpr int KB = 8;
    static_assert(RPT % KB == 0 && NB % KB == 0, "block of reflectors must divide the tile");
    for (int kb = 0; kb < NB / KB; ++kb) {
        const int rgk = (kb * KB) / RPT;          // row group that owns this block's pivot rows
#pragma unroll
        for (int ki = 0; ki < KB; ++ki) {
            const int k = kb * KB + ki;
            const int buf = ki & 1;
            if (rg == rgk) rowk[buf * NB + c] = a[ki];
            if (c == k) {
                if (rg == rgk) {
#pragma unroll
                    for (int r = 0; r < RPT; ++r) xs[buf * HMAX + row0 + r] = (r > ki) ? a[r] : (C)0;
                } else if (rg > rgk) {
#pragma unroll
                    for (int r = 0; r < RPT; ++r) xs[buf * HMAX + row0 + r] = a[r];
                }
            }
            __syncthreads();
            const bool below = rg >= rgk;
            C p = 0;
            if (below) {
#pragma unroll
                for (int r = 0; r < RPT; ++r) p += xs[buf * HMAX + row0 + r] * a[r];
            }
            part[rg * NB + c] = p;
            __syncthreads();
            C D = 0, ss = 0;
#pragma unroll
            for (int q = 0; q < NRG; ++q) {
                D += part[q * NB + c];
                ss += part[q * NB + k];
            }
            const C alpha = rowk[buf * NB + k], akc = rowk[buf * NB + c];
            C tau, beta, inv;
            if (ss == (C)0) {
                tau = 0; beta = alpha; inv = 0;
            } else {
                const C nrm = sqrt(alpha * alpha + ss);
                beta = alpha >= (C)0 ? -nrm : nrm;
                tau = (beta - alpha) / beta;
                inv = (C)1 / (alpha - beta);
            }
            const C w = akc + inv * D;   // v_k^T (column c)
            const C f = tau * w;
            if (rg == 0) {
                if (c < k) Gs[c + k * NB] = my_inv * w;   // v_c^T v_k (v_c's tail is stored unscaled)
                if (c == k) taus[k] = tau;
            }
            if (c == k) my_inv = inv;
            if (rg == rgk) a[ki] = (c > k) ? akc - f : ((c == k) ? beta : akc);
            if (c > k && below && tau != (C)0) {
                const C coef = f * inv;
                // the pivot column was published with zeros at and above the pivot row
#pragma unroll
                for (int r = 0; r < RPT; ++r) a[r] -= coef * xs[buf * HMAX + row0 + r];
            }
        }
        // rows kb*KB .. kb*KB+KB-1 are final: R part to the next level, V part (scaled tails,
        // unit diagonal, zeros above) in place; then the pivot group's registers move down
        if (rg == rgk) {
#pragma unroll
            for (int i = 0; i < KB; ++i) {
                const int row = kb * KB + i;
                if (row < h) {
                    Pnext[((int64_t)d * NB + row) + (int64_t)c * ldnext] = (row <= c) ? a[i] : (C)0;
                    Pd[row + (int64_t)c * ldp] = (row > c) ? a[i] * my_inv : ((row == c) ? (C)1 : (C)0);
                }
            }
#pragma unroll
            for (int r = 0; r < RPT - KB; ++r) a[r] = a[r + KB];
#pragma unroll
            for (int r = RPT - KB; r < RPT; ++r) a[r] = 0;
        }
    }
    // what is left in registers lies below the triangle: explicit V
    {
        constexpr int RGL = (NB - 1) / RPT;                 // last pivot group
        constexpr int LEFT = RPT - (NB - RGL * RPT);        // rows it still holds
        if (rg == RGL) {
#pragma unroll
            for (int r = 0; r < LEFT; ++r) {
                const int row = NB + r;
                if (row < h) Pd[row + (int64_t)c * ldp] = a[r] * my_inv;
            }
        } else if (rg > RGL) {
#pragma unroll
            for (int r = 0; r < RPT; ++r) {
                const int row = row0 + r;
                if (row < h) Pd[row + (int64_t)c * ldp] = a[r] * my_inv;
            }
        }
    }
    __syncthreads();
    // T: T[k][k] = tau_k, T[i][k] = -tau_k * sum_{j=i}^{k-1} T[i][j] G[j][k]  (i < k)
    {
        const int i = tid / LT, s = tid % LT;
        for (int j = s; j < NB; j += LT) Ts[i * (NB + 1) + j] = (j == i) ? taus[i] : (C)0;
        __syncthreads();
        for (int k = 1; k < NB; ++k) {
            C acc = 0;
            if (i < k)
                for (int j = i + s; j < k; j += LT) acc += Ts[i * (NB + 1) + j] * Gs[j + k * NB];
#pragma unroll
            for (int off = LT / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
            if (i < k && s == 0) Ts[i * (NB + 1) + k] = -taus[k] * acc;
            __syncthreads();
        }
        for (int idx = tid; idx < NB * NB; idx += NT) {
            const int ii = idx % NB, jj = idx / NB;
            Td[ii + jj * NB] = Ts[ii * (NB + 1) + jj];
        }
    }
}

template <typename C, int NB, int RPT, int NT>
static void launch_panel_reg(C* P, int64_t ldp, C* Tws, int chunks, int g, C* Pnext, int64_t ldnext,
                             hipStream_t s)
{
    constexpr int NRG = NT / NB, HMAX = NRG * RPT;
    constexpr bool G_GLOBAL = sizeof(C) * (size_t)(NB * (NB + 1) + NB * NB) > 140 * 1024;
    const size_t smem = sizeof(C) * (size_t)(NB * (NB + 1) + (G_GLOBAL ? 0 : NB * NB) + 2 * HMAX + NRG * NB + 2 * NB + NB);
    static bool attr_set = false;
    auto kern = panel_qr_reg_kernel<C, NB, RPT, NT>;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    const int domains = (chunks + g - 1) / g;
    hipLaunchKernelGGL(kern, dim3(domains), dim3(NT), smem, s, P, ldp, Tws, chunks, g, Pnext, ldnext);
}

// rows a register-resident domain can hold, 0 if this (type, nb) has no such kernel
template <typename C> int panel_reg_rows(int nb);
template <> int panel_reg_rows<float>(int nb) { return nb == 32 ? 512 : (nb == 64 ? 512 : 512); }
template <> int panel_reg_rows<double>(int nb) { return nb == 32 ? 512 : (nb == 64 ? 512 : 256); }

template <typename C> struct PanelRegDispatch;
template <> struct PanelRegDispatch<float> {
    static void run(int nb, float* P, int64_t ldp, float* Tws, int chunks, int g, float* Pn, int64_t ldn, hipStream_t s)
    {
        if (nb == 32) launch_panel_reg<float, 32, 32, 512>(P, ldp, Tws, chunks, g, Pn, ldn, s);
        else if (nb == 64) launch_panel_reg<float, 64, 64, 512>(P, ldp, Tws, chunks, g, Pn, ldn, s);
        else launch_panel_reg<float, 128, 64, 1024>(P, ldp, Tws, chunks, g, Pn, ldn, s);
    }
};
template <> struct PanelRegDispatch<double> {
    static void run(int nb, double* P, int64_t ldp, double* Tws, int chunks, int g, double* Pn, int64_t ldn, hipStream_t s)
    {
        if (nb == 32) launch_panel_reg<double, 32, 32, 512>(P, ldp, Tws, chunks, g, Pn, ldn, s);
        else if (nb == 64) launch_panel_reg<double, 64, 64, 512>(P, ldp, Tws, chunks, g, Pn, ldn, s);
        else launch_panel_reg<double, 128, 64, 512>(P, ldp, Tws, chunks, g, Pn, ldn, s);  // 4 row groups x 64 rows
    }
};

// ---------------------------------------------------------------- Y = V T on MFMA
// D[k][p] = sum_j T(j,k) V(p,j): lanes of an accumulator register run along p,
// so Y is written along its contiguous direction.
template <typename C, int NB>
struct YPol : TileShape<NB, true> {
    static constexpr bool A_KC = true, B_KC = false, RMW = false;
    typedef C TA; typedef C TB; typedef C TD;
    static constexpr int TK = 128 / (int)sizeof(C);
    const C* V; C* Y; const C* Td; int64_t ldp, p0, rows;
    __device__ __forceinline__ int ktiles() const { return NB / TK; }
    __device__ __forceinline__ const C* ptrA(int mn, int kt, int k) const { return &Td[(kt * TK + k) + mn * NB]; }
    __device__ __forceinline__ const C* ptrB(int mn, int kt, int k) const
    {
        const int64_t p = p0 + mn;
        return p < rows ? &V[p + (int64_t)(kt * TK + k) * ldp] : nullptr;
    }
    __device__ __forceinline__ C* ptrD(int m, int n) const
    {
        const int64_t p = p0 + n;
        return p < rows ? &Y[p + (int64_t)m * ldp] : nullptr;
    }
};

template <typename C, int NB>
__global__ __launch_bounds__(256) void panel_y_kernel(const C* __restrict__ V, C* __restrict__ Y,
                                                      const C* __restrict__ Tws, int64_t ldp,
                                                      int64_t rows, int g)
{
    YPol<C, NB> pol;
    pol.V = V; pol.Y = Y; pol.ldp = ldp; pol.p0 = (int64_t)blockIdx.x * 128; pol.rows = rows;
    pol.Td = Tws + (pol.p0 / NB / g) * (int64_t)NB * NB;
    gemm_tile<C>(pol);
}

template <typename C, int NB>
static void launch_panel_y(const C* V, C* Y, const C* Tws, int64_t ldp, int64_t rows, int g, hipStream_t s)
{
    hipLaunchKernelGGL((panel_y_kernel<C, NB>), dim3((unsigned)((rows + 127) / 128)), dim3(256), 0, s, V, Y,
                       Tws, ldp, rows, g);
}

template <typename C>
void launch_panel_y_nb(int nb, const C* V, C* Y, const C* Tws, int64_t ldp, int64_t rows, int g, hipStream_t s)
{
    if (nb == 32) launch_panel_y<C, 32>(V, Y, Tws, ldp, rows, g, s);
    else if (nb == 64) launch_panel_y<C, 64>(V, Y, Tws, ldp, rows, g, s);
    else launch_panel_y<C, 128>(V, Y, Tws, ldp, rows, g, s);
}
template void launch_panel_y_nb<float>(int, const float*, float*, const float*, int64_t, int64_t, int, hipStream_t);
template void launch_panel_y_nb<double>(int, const double*, double*, const double*, int64_t, int64_t, int, hipStream_t);

template <typename C> bool panel_blk_serves(int nb, int g)
{
    return env_int("SVB_PANEL_IMPL", 2) == 2 && panel_blk_rows<C>() >= g * nb && (g * nb) % 128 == 0;
}
template bool panel_blk_serves<float>(int, int);
template bool panel_blk_serves<double>(int, int);

template <typename T, typename C>
void launch_panel_qr(int nb, C* P, int64_t ldp, C* Y, C* Tws, int chunks, int g,
                     C* Pnext, int64_t ldnext, const T* Asrc, int64_t lda, bool lq, C* band, int64_t ldab,
                     int64_t row0, int64_t col0, hipStream_t s, hipEvent_t done, hipEvent_t start)
{
    const int impl = env_int("SVB_PANEL_IMPL", 2);
    // blocked register-resident kernel (2, default) or the reflector-at-a-time register kernel (1),
    // each followed by the MFMA Y product, when the domain fits (and 128-row Y tiles never
    // straddle two domains); otherwise the plain kernel below.  Only the blocked kernel reads the
    // matrix and writes the band itself (Asrc, band: null for the others).
    const bool blk = panel_blk_serves<C>(nb, g);
    if ((blk || (impl != 0 && panel_reg_rows<C>(nb) >= g * nb)) && (g * nb) % 128 == 0) {
        // `done` (an event tied to the completion of the level's last kernel) is served only where
        // the blocked kernel is that last kernel; otherwise it is recorded behind the level
        const bool tied = done && blk && Y == nullptr;
        if (blk) launch_panel_blk<T, C>(nb, P, ldp, Tws, chunks, g, Pnext, ldnext, Asrc, lda, lq, band, ldab, row0, col0, s,
                                        tied ? done : nullptr, tied ? start : nullptr);
        else PanelRegDispatch<C>::run(nb, P, ldp, Tws, chunks, g, Pnext, ldnext, s);
        const int64_t rows = (int64_t)chunks * nb;
        if (Y == nullptr) {   // the caller applies T itself
            if (done && !tied) (void)hipEventRecord(done, s);
            return;
        }
        if (nb == 32) launch_panel_y<C, 32>(P, Y, Tws, ldp, rows, g, s);
        else if (nb == 64) launch_panel_y<C, 64>(P, Y, Tws, ldp, rows, g, s);
        else launch_panel_y<C, 128>(P, Y, Tws, ldp, rows, g, s);
        if (done) (void)hipEventRecord(done, s);
        return;
    }
    const int domains = (chunks + g - 1) / g;
    const size_t smem = (size_t)g * nb * sizeof(C);
    constexpr int NT = 512;
    switch (nb) {
    case 32:
        hipLaunchKernelGGL((panel_qr_kernel<C, 32, NT>), dim3(domains), dim3(NT), smem, s, P, ldp, Y, Tws, chunks, g, Pnext, ldnext);
        break;
    case 64:
        hipLaunchKernelGGL((panel_qr_kernel<C, 64, NT>), dim3(domains), dim3(NT), smem, s, P, ldp, Y, Tws, chunks, g, Pnext, ldnext);
        break;
    default:
        hipLaunchKernelGGL((panel_qr_kernel<C, 128, NT>), dim3(domains), dim3(NT), smem, s, P, ldp, Y, Tws, chunks, g, Pnext, ldnext);
        break;
    }
    if (done) (void)hipEventRecord(done, s);
}

// ---------------------------------------------------------------- R -> band
// The last level's R is final: a QR sweep's R is the upper triangle of the
// diagonal tile, an LQ sweep's R^T the lower triangle of the tile right of it
// (Figure 1).  Together these triangles are exactly the band that stage 2
// receives, so they are written straight into the packed band.
template <typename C>
__global__ __launch_bounds__(256) void scatter_r_kernel(const C* __restrict__ R, int64_t ldr, int nb,
                                                        C* __restrict__ band, int64_t ldab,
                                                        int64_t row0, int64_t col0, int lq)
{
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < nb * nb; idx += gridDim.x * blockDim.x) {
        const int i = idx % nb, j = idx / nb;
        if (i > j) continue;
        const C r = R[i + (int64_t)j * ldr];
        const int64_t gi = lq ? row0 + j : row0 + i;
        const int64_t gj = lq ? col0 + i : col0 + j;
        band[(gi - gj + 2 * nb - 1) + gj * ldab] = r;
    }
}

template <typename C>
void launch_scatter_r(const C* R, int64_t ldr, int nb, C* band, int64_t ldab,
                      int64_t row0, int64_t col0, bool lq, hipStream_t s)
{
    hipLaunchKernelGGL((scatter_r_kernel<C>), dim3((nb * nb + 255) / 256), dim3(256), 0, s, R, ldr,
                       nb, band, ldab, row0, col0, lq ? 1 : 0);
}

template <typename C>
__global__ __launch_bounds__(256) void band_clear_kernel(C* __restrict__ band, int64_t total)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x)
        band[i] = 0;
}

template <typename C>
void launch_band_clear(C* band, int64_t ldab, int64_t n, hipStream_t s)
{
    const int64_t total = ldab * n;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL((band_clear_kernel<C>), dim3(blocks), dim3(256), 0, s, band, total);
}

// explicit instantiations
template void launch_panel_gather<double, double>(const double*, int64_t, int64_t, int64_t, bool, int64_t, int, double*, int64_t, hipStream_t);
template void launch_panel_gather<float, float>(const float*, int64_t, int64_t, int64_t, bool, int64_t, int, float*, int64_t, hipStream_t);
template void launch_panel_gather<__half, float>(const __half*, int64_t, int64_t, int64_t, bool, int64_t, int, float*, int64_t, hipStream_t);
template void launch_panel_gather<bf16_t, float>(const bf16_t*, int64_t, int64_t, int64_t, bool, int64_t, int, float*, int64_t, hipStream_t);
template void launch_panel_qr<double, double>(int, double*, int64_t, double*, double*, int, int, double*, int64_t, const double*, int64_t, bool, double*, int64_t, int64_t, int64_t, hipStream_t, hipEvent_t, hipEvent_t);
template void launch_panel_qr<float, float>(int, float*, int64_t, float*, float*, int, int, float*, int64_t, const float*, int64_t, bool, float*, int64_t, int64_t, int64_t, hipStream_t, hipEvent_t, hipEvent_t);
template void launch_panel_qr<__half, float>(int, float*, int64_t, float*, float*, int, int, float*, int64_t, const __half*, int64_t, bool, float*, int64_t, int64_t, int64_t, hipStream_t, hipEvent_t, hipEvent_t);
template void launch_panel_qr<bf16_t, float>(int, float*, int64_t, float*, float*, int, int, float*, int64_t, const bf16_t*, int64_t, bool, float*, int64_t, int64_t, int64_t, hipStream_t, hipEvent_t, hipEvent_t);
template void launch_scatter_r<double>(const double*, int64_t, int, double*, int64_t, int64_t, int64_t, bool, hipStream_t);
template void launch_scatter_r<float>(const float*, int64_t, int, float*, int64_t, int64_t, int64_t, bool, hipStream_t);
template void launch_band_clear<double>(double*, int64_t, int64_t, hipStream_t);
template void launch_band_clear<float>(float*, int64_t, int64_t, hipStream_t);

}  // namespace svb
