// Stage 1, trailing-matrix update in one pass, f32 arithmetic at nb = 128 on the 32 x 32 x 2 MFMA
// (paper Section 3.1 Algorithm 1 lines 3/6; Section 3.2 "Trailing Submatrix Update", Algorithm 5:
// the fused TSMQR keeps the columns a thread owns in registers while it walks down the reflector
// tiles, so that every matrix entry is read once and written once).
//
// Same scheme as stage1_fused.hip (W = Y_d^T C, then C -= V_d W, the block C_d[:, strip] resident
// in accumulator registers, Y_d and V_d streamed through LDS), rebuilt around
// v_mfma_f32_32x32x2_f32: on this machine a wave issues the 16 x 16 x 4 f32 instruction at no more
// than 80 % of the matrix pipe's rate and two waves per SIMD reach 80 % of the nominal peak, the
// 32 x 32 x 2 instruction 97 % (measured with register-only loops).  A 32 x 32 accumulator tile
// costs 16 registers, so a wave cannot hold 512 rows by 32 columns; the workgroup's block
// (512 rows, 64 columns) is split 2 x 2 instead: wave (rh, ch) keeps rows 256 rh .. 256 rh + 255,
// columns 32 ch .. 32 ch + 31 as eight tiles (128 registers).
//
//   * One instruction computes D(32 x 32) += A(32 x 2) B(2 x 32).  Lane l = 32 k + n supplies
//     A[n][k] and B[k][n] and holds column n of D: accumulator register i = 4 a + b is row
//     8 a + 4 k + b.  Register i of a tile is therefore a valid B operand whose two k-slots carry
//     rows 8 a + b and 8 a + 4 + b of the tile, and a product that contracts over the rows of a
//     register-resident tile needs no data movement for that tile; the other operand is fetched
//     in the matching order (four consecutive rows per 16-byte LDS read).
//   * First product, W = Y^T C: each wave forms the part of W (128 x 32, four tiles) that its 256
//     rows contribute; the two waves of a column half then add their parts through LDS.
//   * Second product, C -= V W: W's registers are the B operand (k-slots = rows of W), V supplies
//     32 rows by 2 columns per instruction.
//   * A stage is 32 instructions per wave: in the first product 16 rows of Y for each half of the
//     block (all 128 columns), in the second 32 rows of V for each half by 64 of its columns; the
//     two pieces of a stage share one LDS buffer of 20 KB, double buffered, one LDS-only barrier per
//     stage; the next stage's piece is fetched into registers before the current stage's products.
//
// Trailing-matrix element (p, q) lives at Cb[p*sp + q*sq]; p runs along the panel direction.
// QR sweep: (sp, sq) = (1, lda); LQ sweep: (lda, 1).
#include "svb_internal.h"
#include "mfma_gemm.h"
#include <hip/hip_ext.h>

namespace svb {

namespace {

#ifndef SVB_F32_OCC
#define SVB_F32_OCC 2
#endif
typedef float acc16_t __attribute__((ext_vector_type(16)));

constexpr int kNB = 128, kRows = 512, kHalf = 256, kStripCols = 64;
constexpr int kLdY = 20;                 // Y piece: [half][column 128][16 rows + 4]
constexpr int kLdV = 68;                 // V piece: [half][row 32][64 columns + 4]
constexpr int kYHalf = kNB * kLdY;       // 2560
constexpr int kVHalf = 32 * kLdV;        // 2176
constexpr int kBuf = 2 * kYHalf;         // elements per stage buffer (the larger of the two pieces)
constexpr int kExch = 4 * 32 * 64;       // W exchange: two tiles (32 registers) of each of the 4 waves
constexpr size_t kSmem32 = (size_t)(2 * kBuf + kExch) * sizeof(float);

__device__ __forceinline__ acc16_t mma32(float a, float b, acc16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Global memory goes through buffer instructions: a wave-uniform descriptor (base address in scalar
// registers), one 32-bit per-lane byte offset that is the same for every access of its kind, and a
// wave-uniform byte offset, so that address arithmetic stays on the scalar unit and costs one vector
// register per kind of access.
typedef unsigned u4v __attribute__((ext_vector_type(4)));
typedef unsigned u2v __attribute__((ext_vector_type(2)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base)
{
    // raw buffer (stride 0), 32-bit data format; the range check is left wide open (offsets are
    // proven in range by the caller)
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0xffffffff, 0x00020000);
}

// four consecutive elements / one element of storage type T at byte offset voff + soff
template <typename T> struct BufIO;
template <> struct BufIO<float> {
    static __device__ __forceinline__ void ld4(rsrc_t r, unsigned voff, unsigned soff, float (&o)[4])
    {
        // (the whole vector is reinterpreted at once: converting the four lanes one by one lets the
        // compiler narrow the load to its first lane)
        typedef float f4v __attribute__((ext_vector_type(4)));
        const f4v v = __builtin_bit_cast(f4v, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    static __device__ __forceinline__ void st4(rsrc_t r, unsigned voff, unsigned soff, const float (&o)[4])
    {
        typedef float f4v __attribute__((ext_vector_type(4)));
        f4v v; v.x = o[0]; v.y = o[1]; v.z = o[2]; v.w = o[3];
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4v, v), r, voff, soff, 0);
    }
    static __device__ __forceinline__ float ld1(rsrc_t r, unsigned voff, unsigned soff)
    {
        return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0));
    }
    static __device__ __forceinline__ void st1(rsrc_t r, unsigned voff, unsigned soff, float v)
    {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, voff, soff, 0);
    }
};
template <> struct BufIO<__half> {
    static __device__ __forceinline__ void ld4(rsrc_t r, unsigned voff, unsigned soff, float (&o)[4])
    {
        const u2v v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
        const unsigned lo = v.x, hi = v.y;
        __half2 a, b;
        __builtin_memcpy(&a, &lo, 4);
        __builtin_memcpy(&b, &hi, 4);
        o[0] = __low2float(a); o[1] = __high2float(a); o[2] = __low2float(b); o[3] = __high2float(b);
    }
    static __device__ __forceinline__ void st4(rsrc_t r, unsigned voff, unsigned soff, const float (&o)[4])
    {
        const __half2 a = __floats2half2_rn(o[0], o[1]), b = __floats2half2_rn(o[2], o[3]);
        u2v v;
        unsigned lo, hi;
        __builtin_memcpy(&lo, &a, 4);
        __builtin_memcpy(&hi, &b, 4);
        v.x = lo; v.y = hi;
        __builtin_amdgcn_raw_buffer_store_b64(v, r, voff, soff, 0);
    }
    static __device__ __forceinline__ float ld1(rsrc_t r, unsigned voff, unsigned soff)
    {
        const unsigned short u = __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
        __half h;
        __builtin_memcpy(&h, &u, 2);
        return __half2float(h);
    }
    static __device__ __forceinline__ void st1(rsrc_t r, unsigned voff, unsigned soff, float v)
    {
        const __half h = __float2half(v);
        unsigned short u;
        __builtin_memcpy(&u, &h, 2);
        __builtin_amdgcn_raw_buffer_store_b16(u, r, voff, soff, 0);
    }
};
template <> struct BufIO<bf16_t> {
    static __device__ __forceinline__ unsigned rne(float f) { return VecIO<float, bf16_t>::rne(f); }
    static __device__ __forceinline__ void ld4(rsrc_t r, unsigned voff, unsigned soff, float (&o)[4])
    {
        const u2v v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
        o[0] = __builtin_bit_cast(float, v.x << 16);
        o[1] = __builtin_bit_cast(float, v.x & 0xffff0000u);
        o[2] = __builtin_bit_cast(float, v.y << 16);
        o[3] = __builtin_bit_cast(float, v.y & 0xffff0000u);
    }
    static __device__ __forceinline__ void st4(rsrc_t r, unsigned voff, unsigned soff, const float (&o)[4])
    {
        u2v v;
        v.x = rne(o[0]) | (rne(o[1]) << 16);
        v.y = rne(o[2]) | (rne(o[3]) << 16);
        __builtin_amdgcn_raw_buffer_store_b64(v, r, voff, soff, 0);
    }
    static __device__ __forceinline__ float ld1(rsrc_t r, unsigned voff, unsigned soff)
    {
        const unsigned short u = __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
        return __builtin_bit_cast(float, (unsigned)u << 16);
    }
    static __device__ __forceinline__ void st1(rsrc_t r, unsigned voff, unsigned soff, float v)
    {
        __builtin_amdgcn_raw_buffer_store_b16((unsigned short)rne(v), r, voff, soff, 0);
    }
};

// The sixteen entries a lane holds of a 32 x 32 tile (register 4a + b: row 8a + 4k + b of the tile,
// column n).  r describes the memory from the tile's first element on; lane_off is the lane's byte
// offset inside a tile (QR: (4k + n*lda) elements, LQ: (4k*lda + n) elements), rowb the byte
// distance between consecutive rows in the LQ orientation.
template <typename T, bool LQ>
__device__ __forceinline__ acc16_t tile32_load(rsrc_t r, unsigned lane_off, unsigned rowb)
{
    acc16_t c;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        if constexpr (!LQ) {
            float o[4];
            BufIO<T>::ld4(r, lane_off, 8 * a * (unsigned)sizeof(T), o);
#pragma unroll
            for (int b = 0; b < 4; ++b) c[4 * a + b] = o[b];
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b) c[4 * a + b] = BufIO<T>::ld1(r, lane_off, (unsigned)(8 * a + b) * rowb);
        }
    }
    return c;
}

template <typename T, bool LQ>
__device__ __forceinline__ void tile32_store(rsrc_t r, unsigned lane_off, unsigned rowb, const acc16_t& c)
{
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        if constexpr (!LQ) {
            const float o[4] = {c[4 * a], c[4 * a + 1], c[4 * a + 2], c[4 * a + 3]};
            BufIO<T>::st4(r, lane_off, 8 * a * (unsigned)sizeof(T), o);
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b) BufIO<T>::st1(r, lane_off, (unsigned)(8 * a + b) * rowb, c[4 * a + b]);
        }
    }
}

__device__ __forceinline__ void ld4f(const float* p, float (&o)[4])
{
    typedef float v4 __attribute__((ext_vector_type(4)));
    const v4 v = *reinterpret_cast<const v4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
__device__ __forceinline__ void st4f(float* p, const float (&o)[4])
{
    typedef float v4 __attribute__((ext_vector_type(4)));
    v4 v; v.x = o[0]; v.y = o[1]; v.z = o[2]; v.w = o[3];
    *reinterpret_cast<v4*>(p) = v;
}

}  // namespace

// TRI: the panel is a stack of upper triangular 128 x 128 factors (tree levels above the first):
// in every chunk of V and of Y = V T the 32 x 32 blocks below the block diagonal are zero and their
// products are skipped.
// FULL: the domain has all 512 rows and the strip all 64 columns.  Then nothing in the body is
// predicated: every stage is straight-line code, and the waits for the staged pieces count exactly
// the memory operations issued after them instead of draining the queue.
template <typename T, bool LQ, bool TRI, bool FULL>
__device__ __forceinline__ void fused32_body(T* __restrict__ Cb, int64_t lda, int64_t qlen, const float* __restrict__ V,
                                             const float* __restrict__ Y, int64_t ldp, int chunks, int g,
                                             int64_t stride, int d, int strip, float* smem)
{
    float* exch = smem + 2 * kBuf;
    const int nch = FULL ? 4 : min(g, chunks - d * g);
    const int R = FULL ? kRows : nch * kNB;        // rows of this domain
    const int nst = FULL ? 16 : min(16, R / 16);   // stages per product: two per tile of the taller half
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave-uniform: scalar arithmetic below
    const int rh = wave >> 1, ch = wave & 1;
    const int n = lane & 31, k = lane >> 5;
    const int64_t q0 = (int64_t)strip * kStripCols + ch * 32;           // first column of this wave
    const unsigned lane_off = (LQ ? (unsigned)(4 * k * lda + n) : (unsigned)(4 * k + n * lda)) * (unsigned)sizeof(T);
    const unsigned rowb = (unsigned)lda * (unsigned)sizeof(T);
    const bool active = FULL || (int64_t)strip * kStripCols + ch * 32 < qlen;   // qlen is a multiple of 32
    const int64_t prow0 = (int64_t)d * g * kNB;                          // first row of the domain in V / Y

    // global p index of row r of the domain: chunk r / 128, offset r % 128 inside it
    auto row_p = [&](int r) -> int64_t { return ((int64_t)d * g + r / kNB) * stride + r % kNB; };

    // pointer to element (row r0 of the domain, first column of this wave)
    auto tile_base = [&](int r0) -> T* { return LQ ? Cb + row_p(r0) * lda + q0 : Cb + row_p(r0) + q0 * lda; };
    acc16_t c[8];
    auto tile_ld = [&](int t) {
        const int r0 = rh * kHalf + 32 * t;
        if (FULL || (active && r0 < R)) c[t] = tile32_load<T, LQ>(make_rsrc(tile_base(r0)), lane_off, rowb);
        else
#pragma unroll
            for (int i = 0; i < 16; ++i) c[t][i] = 0;
    };
    acc16_t w[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) w[mt][i] = 0;

    // ---- pieces of Y and V: global -> registers -> LDS (4 vectors of 4 per thread and stage)
    float sreg[4][4];
    // Y piece of stage s: rows 16 s .. 16 s + 15 of each half, all 128 columns.  Vector v = tid + 256 e:
    // four rows 4 (v % 4) .. of column (v / 4) % 128 of half v / 512 (e = 0, 1: upper half)
    const rsrc_t ry = make_rsrc(Y + prow0), rv_ = make_rsrc(V + prow0);
    const unsigned ldpb = (unsigned)ldp * 4u;
    const unsigned yoff = (unsigned)(4 * (tid & 3)) * 4u + (unsigned)(tid >> 2) * ldpb;          // e = 0
    const unsigned voff = (unsigned)(4 * (tid & 7)) * 4u + (unsigned)(tid >> 3) * ldpb;          // e = 0
    auto piece_ld_y = [&](int s) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int half = e >> 1;
            const int row = half * kHalf + 16 * s + 4 * (tid & 3);
            // e odd: columns 64 ..
            const unsigned so = (unsigned)(half * kHalf + 16 * s) * 4u + (unsigned)(e & 1) * 64u * ldpb;
            if (FULL || row < R) BufIO<float>::ld4(ry, yoff, so, sreg[e]);
            else
#pragma unroll
                for (int j = 0; j < 4; ++j) sreg[e][j] = 0;
        }
    };
    auto piece_st_y = [&](float* buf) {   // [half][column][row]
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int v = tid + e * 256;
            const int rv = v & 3, col = (v >> 2) & 127, half = v >> 9;
            st4f(&buf[half * kYHalf + col * kLdY + 4 * rv], sreg[e]);
        }
    };
    // V piece of stage s: rows 32 (s / 2) .. + 31 of each half, columns 64 (s % 2) .. + 63.  Vector
    // v = tid + 256 e: four rows 4 (v % 8) .. of column (v / 8) % 64 of half v / 512
    auto piece_ld_v = [&](int s) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int half = e >> 1;
            const int row = half * kHalf + 32 * (s >> 1) + 4 * (tid & 7);
            const unsigned so = (unsigned)(half * kHalf + 32 * (s >> 1)) * 4u +
                                (unsigned)(64 * (s & 1) + 32 * (e & 1)) * ldpb;
            if (FULL || row < R) BufIO<float>::ld4(rv_, voff, so, sreg[e]);
            else
#pragma unroll
                for (int j = 0; j < 4; ++j) sreg[e][j] = 0;
        }
    };
    auto piece_st_v = [&](float* buf) {   // [half][row][column]
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int v = tid + e * 256;
            const int rv = v & 7, col = (v >> 3) & 63, half = v >> 9;
#pragma unroll
            for (int j = 0; j < 4; ++j) buf[half * kVHalf + (4 * rv + j) * kLdV + col] = sreg[e][j];
        }
    };

    // barrier that orders LDS traffic only (s_waitcnt lgkmcnt(0); s_barrier): __syncthreads()
    // would also wait for every outstanding global load and store
    auto lds_barrier = [] {
        __builtin_amdgcn_s_waitcnt(0xc07f);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);   // the instruction scheduler keeps every stage to itself
    };

    int cur = 0;
    piece_ld_y(0);
    tile_ld(0);
    tile_ld(1);
    piece_st_y(smem);
    lds_barrier();

    // ---- first product: W += Y_piece^T C_piece, stage s = rows 16 s .. of each half
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        if (FULL || s < nst) {
            const bool last = s + 1 == nst;
            if (!last) piece_ld_y(s + 1);
            else piece_ld_v(0);
            if ((s & 1) == 0 && (s >> 1) + 2 < 8) tile_ld((s >> 1) + 2);
            __builtin_amdgcn_sched_barrier(0);   // the fetches stay in front of the products
            const float* buf = smem + cur * kBuf + rh * kYHalf;
            const int t = s >> 1, h8 = (s & 1) * 8;
            const int tl = TRI ? t % 4 : 0;            // block row of this tile inside its chunk
            __builtin_amdgcn_s_setprio(1);   // the wave inside its products goes first
            if (FULL || (active && rh * kHalf + 32 * t < R)) {
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) {
                    if (mt >= tl) {
                        float a0[4], a1[4];
                        ld4f(&buf[(32 * mt + n) * kLdY + 4 * k], a0);
                        ld4f(&buf[(32 * mt + n) * kLdY + 8 + 4 * k], a1);
#pragma unroll
                        for (int b = 0; b < 4; ++b) w[mt] = mma32(a0[b], c[t][h8 + b], w[mt]);
#pragma unroll
                        for (int b = 0; b < 4; ++b) w[mt] = mma32(a1[b], c[t][h8 + 4 + b], w[mt]);
                    }
                }
            }
            __builtin_amdgcn_s_setprio(0);
            float* nbuf = smem + (cur ^ 1) * kBuf;
            if (!last) piece_st_y(nbuf);
            else piece_st_v(nbuf);
            lds_barrier();
            cur ^= 1;
        }
    }

    // ---- the two row halves add their parts of W (two tiles at a time through LDS) and negate
    {
        typedef float v4 __attribute__((ext_vector_type(4)));
        v4* mine = reinterpret_cast<v4*>(exch) + (size_t)wave * 8 * 64;
        const v4* other = reinterpret_cast<const v4*>(exch) + (size_t)(wave ^ 2) * 8 * 64;
#pragma unroll
        for (int hp = 0; hp < 2; ++hp) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const acc16_t& x = w[2 * hp + mt];
                    v4 v; v.x = x[4 * a]; v.y = x[4 * a + 1]; v.z = x[4 * a + 2]; v.w = x[4 * a + 3];
                    mine[(mt * 4 + a) * 64 + lane] = v;
                }
            lds_barrier();
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const v4 v = other[(mt * 4 + a) * 64 + lane];
                    acc16_t& x = w[2 * hp + mt];
                    x[4 * a] = -(x[4 * a] + v.x);
                    x[4 * a + 1] = -(x[4 * a + 1] + v.y);
                    x[4 * a + 2] = -(x[4 * a + 2] + v.z);
                    x[4 * a + 3] = -(x[4 * a + 3] + v.w);
                }
            lds_barrier();
        }
    }

    // ---- second product: C_tile += V_piece (-W), stage s = tile s / 2, columns 64 (s % 2) .. of V
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        if (FULL || s < nst) {
            const bool last = s + 1 == nst;
            if (!last) piece_ld_v(s + 1);
            __builtin_amdgcn_sched_barrier(0);   // the fetches stay in front of the products
            const float* buf = smem + cur * kBuf + rh * kVHalf;
            const int t = s >> 1, jh = s & 1;
            const int tl = TRI ? t % 4 : 0;
            const bool mine = FULL || (active && rh * kHalf + 32 * t < R);
            __builtin_amdgcn_s_setprio(1);   // the wave inside its products goes first
            if (mine) {
#pragma unroll
                for (int ml = 0; ml < 2; ++ml) {
                    const int mt = 2 * jh + ml;
                    if (mt >= tl) {
#pragma unroll
                        for (int a = 0; a < 4; ++a) {
                            float av[4];
                            ld4f(&buf[n * kLdV + 32 * ml + 8 * a + 4 * k], av);
#pragma unroll
                            for (int b = 0; b < 4; ++b) c[t] = mma32(av[b], w[mt][4 * a + b], c[t]);
                        }
                    }
                }
                if (jh == 1) tile32_store<T, LQ>(make_rsrc(tile_base(rh * kHalf + 32 * t)), lane_off, rowb, c[t]);
            }
            __builtin_amdgcn_s_setprio(0);
            if (!last) {
                piece_st_v(smem + (cur ^ 1) * kBuf);
                lds_barrier();
                cur ^= 1;
            }
        }
    }
}

template <typename T, bool LQ, bool TRI>
__global__ __launch_bounds__(256, SVB_F32_OCC) void update_fused32_kernel(T* __restrict__ Cb, int64_t lda, int64_t qlen,
                                                                          const float* __restrict__ V,
                                                                          const float* __restrict__ Y, int64_t ldp,
                                                                          int chunks, int g, int64_t stride, int strips,
                                                                          int total)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* smem = reinterpret_cast<float*>(smem_raw);
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): give every XCD a
    // contiguous range of tiles, so that the workgroups sharing a domain's V and Y mostly share an L2.
    const int per = (total + 7) / 8;
    const int tile = (int)(blockIdx.x % 8) * per + (int)(blockIdx.x / 8);
    if (tile >= total) return;
    const int d = tile / strips, strip = tile % strips;
    const bool full = g == 4 && chunks - d * g >= 4 && (int64_t)(strip + 1) * kStripCols <= qlen;
    if (full) fused32_body<T, LQ, TRI, true>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, d, strip, smem);
    else fused32_body<T, LQ, TRI, false>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, d, strip, smem);
}

template <typename T, bool LQ, bool TRI>
static void launch_fused32(T* Cb, int64_t lda, int64_t qlen, const float* V, const float* Y, int64_t ldp, int chunks,
                           int g, int64_t stride, bool credited, hipStream_t s)
{
    auto kern = update_fused32_kernel<T, LQ, TRI>;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)kSmem32);
        attr_set = true;
    }
    const int domains = (chunks + g - 1) / g;
    const int strips = (int)((qlen + kStripCols - 1) / kStripCols);
    const int total = domains * strips;
    const int per = (total + 7) / 8;
    // both products: 2 * rows * nb * cols flops each; the block is read once and written once
    const double rows = (double)chunks * kNB;
    double fl = 4.0 * rows * kNB * (double)qlen, by = 2.0 * rows * (double)qlen * sizeof(T);
    if (!credited) fl = by = 0.0;
    // profiling: the events are the kernel's own start and stop time stamps
    hipEvent_t ea = nullptr, eb = nullptr;
    if (prof_take(TRI ? SVB_PROF_UPDATE_UPPER : SVB_PROF_UPDATE, fl, by, &ea, &eb))
        hipExtLaunchKernelGGL(kern, dim3((unsigned)(per * 8)), dim3(256), (uint32_t)kSmem32, s, ea, eb, 0u, Cb, lda,
                              qlen, V, Y, ldp, chunks, g, stride, strips, total);
    else
        hipLaunchKernelGGL(kern, dim3((unsigned)(per * 8)), dim3(256), kSmem32, s, Cb, lda, qlen, V, Y, ldp, chunks,
                           g, stride, strips, total);
}

// nb = 128, f32 arithmetic, domains of at most 512 rows (g <= 4); qlen a multiple of 32
template <typename T>
void launch_update_fused32(bool lq, T* Cb, int64_t lda, int64_t qlen, const float* V, const float* Y, int64_t ldp,
                           int chunks, int g, int64_t stride, bool tri, bool credited, hipStream_t s)
{
    if (qlen <= 0) return;
    if (lq && tri) launch_fused32<T, true, true>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, credited, s);
    else if (lq) launch_fused32<T, true, false>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, credited, s);
    else if (tri) launch_fused32<T, false, true>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, credited, s);
    else launch_fused32<T, false, false>(Cb, lda, qlen, V, Y, ldp, chunks, g, stride, credited, s);
}

template void launch_update_fused32<float>(bool, float*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, bool, bool, hipStream_t);
template void launch_update_fused32<__half>(bool, __half*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, bool, bool, hipStream_t);
template void launch_update_fused32<bf16_t>(bool, bf16_t*, int64_t, int64_t, const float*, const float*, int64_t, int, int, int64_t, bool, bool, hipStream_t);

}  // namespace svb
