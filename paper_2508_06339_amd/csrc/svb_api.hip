// C-ABI entry points and the host-side stage driver.
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "svb_internal.h"

namespace svb {

int env_int(const char* name, int dflt)
{
    const char* v = std::getenv(name);
    return (v && *v) ? std::atoi(v) : dflt;
}

namespace {

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

size_t compute_size(svb_dtype dt) { return dt == SVB_F64 ? 8 : 4; }
size_t storage_size(svb_dtype dt) { return dt == SVB_F64 ? 8 : (dt == SVB_F32 ? 4 : 2); }

int check_shape(svb_dtype dt, int64_t m, int64_t n, int nb)
{
    if (m < 0 || n < 0) return SVB_ERR_ARG;
    if (dt != SVB_F64 && dt != SVB_F32 && dt != SVB_F16) return SVB_ERR_UNSUPPORTED;
    if (nb != 32 && nb != 64 && nb != 128) return SVB_ERR_UNSUPPORTED;
    if (m != n || n <= 0 || n % nb != 0) return SVB_ERR_UNSUPPORTED;
    return SVB_OK;
}

// scratch of stage 2: counters of the band reduction (or of the one-phase chase, whichever
// is larger) followed by those of the narrow chase
size_t gb2bd_first_bytes(int64_t n, int nb)
{
    if (nb == 8) return 0;
    const size_t a = chase_workspace_bytes(n, nb), b = band_reduce_workspace_bytes(n);
    return align_up(a > b ? a : b);
}
size_t gb2bd_bytes(int64_t n, int nb)
{
    return gb2bd_first_bytes(n, nb) + align_up(chase_narrow_workspace_bytes(n));
}

// two-phase stage 2 (band -> 8 super-diagonals -> bidiagonal) unless switched off or unsupported
bool two_phase(int nb, size_t elem_size, int64_t n)
{
    return nb != 8 && n >= 3 && env_int("SVB_CHASE_IMPL", 2) == 2 && band_reduce_supported(nb, elem_size);
}

template <typename C>
int gb2bd_typed(int64_t n, int nb, C* band, int64_t ldab, C* d, C* e, void* work, size_t work_bytes, hipStream_t s)
{
    int* ctrl = static_cast<int*>(work);
    if (nb == 8) {
        // narrow band: bundles of sweeps inside LDS windows
        const int rc = run_chase_narrow<C>(n, band, ldab, 15, ctrl, s);
        launch_extract_bidiag<C>(band, ldab, n, 8, d, e, ctrl, nullptr, s);
        return rc;
    }
    if (two_phase(nb, sizeof(C), n)) {
        int* ctrl2 = reinterpret_cast<int*>(static_cast<unsigned char*>(work) + gb2bd_first_bytes(n, nb));
        int rc = run_band_reduce<C>(n, nb, band, ldab, ctrl, s);
        if (rc == SVB_OK) rc = run_chase_narrow<C>(n, band, ldab, 2 * (int64_t)nb - 1, ctrl2, s);
        launch_extract_bidiag<C>(band, ldab, n, nb, d, e, ctrl, ctrl2, s);
        return rc;
    }
    return run_chase<C>(n, nb, band, ldab, d, e, work, work_bytes, s);
}

// the update kernels move 16-byte vectors along both directions of A
bool aligned_for_vectors(const void* A, int64_t lda)
{
    return reinterpret_cast<uintptr_t>(A) % 16 == 0 && lda % 4 == 0;
}

// chunks-per-domain of the panel tree: as many nb-row tiles as the register-resident
// panel and update kernels hold (512 rows in f32, 256 in f64)
int domain_chunks(svb_dtype dt, int nb)
{
    int g = env_int("SVB_DOMAIN_CHUNKS", 0);
    if (g >= 2 && g <= 64) return g;
    return (dt == SVB_F64 ? 256 : 512) / nb;
}
constexpr int kMinDomainChunks = 2;  // workspace is sized for any g >= this

// Workspace layout (element counts in the compute type).
struct Carve {
    size_t panel_elems;  // V panels of all levels
    size_t w_elems;      // W of the largest level
    size_t t_elems;      // T factors of one level
    size_t band_elems, de_elems;
    size_t off_V[2], off_Y[2], off_W[2], off_T[2], off_band, off_d, off_e, off_sig, off_s3, off_err, total;
};

Carve carve(svb_dtype dt, int64_t n, int nb)
{
    Carve c{};
    const size_t cs = compute_size(dt);
    // levels shrink by >= kMinDomainChunks: sum of panel rows <= 2n (+ one chunk per level)
    c.panel_elems = (size_t)(2 * n + (int64_t)(kMaxLevels + 2) * nb) * nb;
    // W of every tree level: n^2/g * (1 + 1/g + ...) <= n^2 for g >= 2
    c.w_elems = (size_t)n * (size_t)n + (size_t)n * nb * (kMaxLevels + 1);
    c.t_elems = 2 * (size_t)(n / nb + 1) * nb * nb;  // T per domain, plus room for the v^T v products
    c.band_elems = (size_t)(3 * nb) * (size_t)n;
    c.de_elems = (size_t)n;
    size_t off = 0;
    // two sets: a half-sweep's deferred update still reads its set while the next panel is built
    for (int b = 0; b < 2; ++b) {
        c.off_V[b] = off; off += align_up(c.panel_elems * cs);
        c.off_Y[b] = off; off += align_up(c.panel_elems * cs);
        c.off_W[b] = off; off += align_up(c.w_elems * cs);
        c.off_T[b] = off; off += align_up(c.t_elems * cs);
    }
    c.off_band = off; off += align_up(c.band_elems * cs);
    c.off_d = off; off += align_up(c.de_elems * cs);
    c.off_e = off; off += align_up(c.de_elems * cs);
    c.off_sig = off; off += align_up(c.de_elems * cs);
    c.off_s3 = off; off += align_up(bdsvals_dev_workspace_bytes(n));
    c.off_err = off; off += 256;
    off += align_up(gb2bd_bytes(n, nb));
    c.total = off;
    return c;
}

int build_levels(int64_t len, int nb, int g, Level* lv)
{
    int nl = 0;
    int chunks = (int)(len / nb);
    int64_t stride = nb, poff = 0;
    for (;;) {
        Level& L = lv[nl];
        L.chunks = chunks;
        L.domains = (chunks + g - 1) / g;
        L.stride = stride;
        L.poff = poff;
        L.ldp = (int64_t)chunks * nb;
        poff += L.ldp * nb;
        ++nl;
        if (L.domains == 1 || nl == kMaxLevels) break;
        chunks = L.domains;
        stride *= g;
    }
    return nl;
}

struct Timings { double s1 = 0, s2 = 0, s3 = 0; } g_last;

// Optional per-kernel timing with events on the launching stream.
struct Profiler {
    struct Rec { int kind; hipEvent_t a, b; double flops, bytes; };
    bool on = false;
    std::vector<hipEvent_t> pool;
    std::vector<Rec> recs;
    double sec[SVB_PROF_KINDS] = {0}, flops[SVB_PROF_KINDS] = {0}, bytes[SVB_PROF_KINDS] = {0};
    int64_t count[SVB_PROF_KINDS] = {0};
    hipEvent_t get()
    {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        (void)hipEventCreate(&e);
        return e;
    }
    void begin(int kind, hipStream_t s, double fl, double by)
    {
        if (!on) return;
        Rec r{kind, get(), get(), fl, by};
        (void)hipEventRecord(r.a, s);
        recs.push_back(r);
    }
    void end(hipStream_t s)
    {
        if (!on) return;
        (void)hipEventRecord(recs.back().b, s);
    }
    bool take(int kind, double fl, double by, hipEvent_t* a, hipEvent_t* b)
    {
        if (!on) return false;
        Rec r{kind, get(), get(), fl, by};
        *a = r.a;
        *b = r.b;
        recs.push_back(r);
        return true;
    }
    void collect()
    {
        for (auto& r : recs) {
            float ms = 0;
            if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
                sec[r.kind] += ms * 1e-3;
                flops[r.kind] += r.flops;
                bytes[r.kind] += r.bytes;
                count[r.kind] += 1;
            }
            pool.push_back(r.a);
            pool.push_back(r.b);
        }
        recs.clear();
    }
    void reset()
    {
        collect();
        for (int k = 0; k < SVB_PROF_KINDS; ++k) { sec[k] = flops[k] = bytes[k] = 0; count[k] = 0; }
    }
} g_prof;

// Streams and events for the look-ahead (created once per process).  Stage 1 runs on two
// internal streams forked from the caller's stream and joined back to it: `m` carries the
// chain panel -> first part of the update -> next panel, `h` the deferred part of the update.
// `h` is confined to a subset of the compute units (SVB_HELPER_MASK_BITS of them, default 224
// of 256), so that the few workgroups of a panel kernel, each of which needs a compute unit
// of its own, find one free while the deferred update is running.  (A stream with a CU mask
// is an ordinary blocking stream: it would serialise with the NULL stream, which is why the
// chain does not run on the caller's stream itself.)
void g_la_release();
struct Lookahead {
    hipStream_t m = nullptr, h = nullptr, u = nullptr;
    hipEvent_t crit[2] = {nullptr, nullptr}, rest[2] = {nullptr, nullptr}, fork = nullptr, join = nullptr;
    // level pipeline: panel level L of a half-sweep done / its update done; the update stream's join
    hipEvent_t lvl[2][kMaxLevels] = {}, udone[2] = {nullptr, nullptr}, join_u = nullptr;
    bool ok = false, tried = false;
    static bool masked_stream(hipStream_t* st, int bits)
    {
        // bit i of a CU mask is compute unit i / 8 of XCD i % 8 (measured): clearing the top bits
        // takes the same number of CUs away from every XCD
        if (bits > 0 && bits < 256) {
            uint32_t mask[8];
            for (int w = 0; w < 8; ++w) {
                const int nb = bits - 32 * w;
                mask[w] = nb >= 32 ? 0xffffffffu : (nb <= 0 ? 0u : ((1u << nb) - 1u));
            }
            return hipExtStreamCreateWithCUMask(st, 8, mask) == hipSuccess;
        }
        return hipStreamCreateWithFlags(st, hipStreamNonBlocking) == hipSuccess;
    }
    bool init()
    {
        if (tried) return ok;
        tried = true;
        if (hipStreamCreateWithFlags(&m, hipStreamNonBlocking) != hipSuccess) return false;
        if (!masked_stream(&h, env_int("SVB_HELPER_MASK_BITS", 224))) return false;
        if (!masked_stream(&u, env_int("SVB_UPDATE_MASK_BITS", 256))) return false;
        // events between the two internal streams order kernels of one device against each other:
        // no system-scope fence (a cache write-back for the host's and other devices' benefit) is
        // needed when they are recorded, and it would sit on the critical path of every half-sweep
        const unsigned kInner = env_int("SVB_EVENT_FENCE", 0) ? hipEventDisableTiming
                                                              : (hipEventDisableTiming | hipEventDisableSystemFence);
        for (int i = 0; i < 2; ++i) {
            if (hipEventCreateWithFlags(&crit[i], kInner) != hipSuccess ||
                hipEventCreateWithFlags(&rest[i], kInner) != hipSuccess ||
                hipEventCreateWithFlags(&udone[i], kInner) != hipSuccess)
                return false;
            for (int L = 0; L < kMaxLevels; ++L)
                if (hipEventCreateWithFlags(&lvl[i][L], kInner) != hipSuccess) return false;
        }
        if (hipEventCreateWithFlags(&fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&join, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&join_u, hipEventDisableTiming) != hipSuccess)
            return false;
        ok = true;
        // released while the HIP runtime is still up (handlers registered later run earlier):
        // a CU-masked stream left to process teardown has crashed tools that hook the runtime
        std::atexit([] { g_la_release(); });
        return true;
    }
    void release()
    {
        if (!ok) return;
        ok = false;
        (void)hipStreamSynchronize(h);
        (void)hipStreamSynchronize(u);
        (void)hipStreamSynchronize(m);
        for (int i = 0; i < 2; ++i) {
            (void)hipEventDestroy(crit[i]);
            (void)hipEventDestroy(rest[i]);
            (void)hipEventDestroy(udone[i]);
            for (int L = 0; L < kMaxLevels; ++L) (void)hipEventDestroy(lvl[i][L]);
        }
        (void)hipEventDestroy(fork);
        (void)hipEventDestroy(join);
        (void)hipEventDestroy(join_u);
        (void)hipStreamDestroy(h);
        (void)hipStreamDestroy(u);
        (void)hipStreamDestroy(m);
    }
} g_la;
void g_la_release() { g_la.release(); }

// Stage 1 driver, level pipeline (the default with the one-pass update).  The tree levels of a
// panel depend on each other only through the R factors, not through the trailing matrix, so
// once level L of the panel is factored its update U_L can run while level L+1 is being factored.
// Two internal streams:   main: P0 P1 .. Pl Ul P0' ..      side: U0 .. Ul-1
// The last level's update and the next half-sweep's first panel follow the panel tree on the main
// stream: a dependency that crosses streams costs two to three times what one inside a stream
// does (measured), and for all but the largest trailing matrices the panel tree is the longer
// chain of a half-sweep.  (SVB_PIPELINE_LAYOUT=0: every update on the side stream.)
template <typename T, typename C>
int ge2gb_pipeline(int64_t n, T* A, int64_t lda, int nb, C* band, int64_t ldab, unsigned char* work,
                   const Carve& cv, int g, hipStream_t caller)
{
    const int64_t N = n / nb;
    Level lv[kMaxLevels];
    hipStream_t ms = g_la.m, ss = g_la.u;
    (void)hipEventRecord(g_la.fork, caller);
    (void)hipStreamWaitEvent(ms, g_la.fork, 0);
    (void)hipStreamWaitEvent(ss, g_la.fork, 0);
    launch_band_clear<C>(band, ldab, n, ms);
    C* Vb = reinterpret_cast<C*>(work + cv.off_V[0]);
    C* Yb = reinterpret_cast<C*>(work + cv.off_Y[0]);
    C* Tb = reinterpret_cast<C*>(work + cv.off_T[0]);
    const bool direct = panel_blk_serves<C>(nb, g);
    const int layout = env_int("SVB_PIPELINE_LAYOUT", 1);
    // a level's event is tied to the completion of its kernel instead of being recorded behind it
    // (one marker less in the main stream between two panel levels)
    const bool ext_events = env_int("SVB_EXT_EVENTS", 1) != 0;
    int hs = 0;
    bool side_pending = false;
    for (int64_t k = 0; k < N; ++k) {
        for (int half = 0; half < 2; ++half) {
            const bool lq = half == 1;
            if (lq && k == N - 1) break;
            const int set = hs & 1;
            const int64_t row0 = k * nb;
            const int64_t col0 = lq ? (k + 1) * nb : k * nb;
            const int64_t len = lq ? n - (k + 1) * nb : n - k * nb;
            const int64_t qlen = n - (k + 1) * nb;
            const int nl = build_levels(len, nb, g, lv);
            // every level keeps its own T factors until its update has run: the update applies
            // them itself (no Y = V T between a panel and its update) where they all fit
            int64_t toff[kMaxLevels], tsum = 0;
            for (int L = 0; L < nl; ++L) {
                toff[L] = tsum;
                tsum += (int64_t)lv[L].domains * nb * nb;
            }
            const bool useT = direct && nb <= 64 && tsum <= (int64_t)cv.t_elems && env_int("SVB_UPDATE_T", 1) != 0;
            const bool split = layout == 0 && qlen > 0;
            T* Cb = lq ? A + (k + 1) * nb + (k + 1) * nb * lda : A + k * nb + (k + 1) * nb * lda;
            // Factors level L on stream st and returns the event that fires when the level is done
            // (null if none was asked for).  Where the level is a single kernel the event is tied to
            // that kernel's completion instead of being recorded behind it, and with profiling on the
            // profiler's own stop event serves: no marker then separates two panel levels.
            auto panel = [&](int L, hipStream_t st, hipEvent_t done) -> hipEvent_t {
                const int64_t next_off = lv[L].poff + lv[L].ldp * nb;
                const int64_t ldnext = (int64_t)lv[L].domains * nb;
                const bool last = L == nl - 1;
                const bool single = ext_events && direct && useT;
                const double fl = L == 0 ? 2.0 * (double)len * nb * nb : 0.0;
                hipEvent_t ea = nullptr, eb = nullptr;
                const bool timed = single && prof_take(SVB_PROF_PANEL, fl, 0.0, &ea, &eb);
                if (!timed) g_prof.begin(SVB_PROF_PANEL, st, fl, 0.0);
                if (L == 0 && !direct)
                    launch_panel_gather<T, C>(A, lda, row0, col0, lq, len, nb, Vb + lv[0].poff, lv[0].ldp, st);
                launch_panel_qr<T, C>(nb, Vb + lv[L].poff, lv[L].ldp, useT ? (C*)nullptr : Yb + lv[L].poff,
                                      useT ? Tb + toff[L] : Tb, lv[L].chunks, g,
                                      Vb + next_off, ldnext, (direct && L == 0) ? A + row0 + col0 * lda : nullptr, lda, lq,
                                      (direct && last) ? band : nullptr, ldab, row0, col0, st,
                                      timed ? eb : (single ? done : nullptr), ea);
                if (last && !direct)
                    launch_scatter_r<C>(Vb + next_off, ldnext, nb, band, ldab, row0, col0, lq, st);
                if (!timed) g_prof.end(st);
                if (timed) return eb;
                if (done && !single) (void)hipEventRecord(done, st);
                return done;
            };
            auto update = [&](int L, hipStream_t st) {
                launch_update_fused<T, C>(nb, lq, Cb, lda, qlen, Vb + lv[L].poff, Yb + lv[L].poff, lv[L].ldp,
                                          lv[L].chunks, g, lv[L].stride, L > 0, 0, (C*)nullptr,
                                          useT ? Tb + toff[L] : (const C*)nullptr, L == 0, st);
            };
            if (side_pending) {
                // the previous half-sweep left its last update on the side stream
                (void)hipStreamWaitEvent(ms, g_la.udone[(hs - 1) & 1], 0);
                side_pending = false;
            }
            if (qlen <= 0) {
                for (int L = 0; L < nl; ++L) panel(L, ms, nullptr);
            } else if (split) {
                // every panel on the main stream, every update on the side stream
                for (int L = 0; L < nl; ++L) {
                    (void)hipStreamWaitEvent(ss, panel(L, ms, g_la.lvl[set][L]), 0);
                    update(L, ss);
                }
                (void)hipEventRecord(g_la.udone[set], ss);
                side_pending = true;
            } else {
                for (int L = 0; L < nl; ++L) {
                    const hipEvent_t ev = panel(L, ms, L < nl - 1 ? g_la.lvl[set][L] : nullptr);
                    if (L < nl - 1) {
                        (void)hipStreamWaitEvent(ss, ev, 0);
                        update(L, ss);
                    }
                }
                if (nl > 1) {
                    (void)hipEventRecord(g_la.udone[set], ss);
                    (void)hipStreamWaitEvent(ms, g_la.udone[set], 0);
                }
                update(nl - 1, ms);
            }
            ++hs;
        }
    }
    (void)hipEventRecord(g_la.join, ms);
    (void)hipEventRecord(g_la.join_u, ss);
    (void)hipStreamWaitEvent(caller, g_la.join, 0);
    (void)hipStreamWaitEvent(caller, g_la.join_u, 0);
    return hipGetLastError() == hipSuccess ? SVB_OK : SVB_ERR_DEVICE;
}

// Stage 1 driver.  Per half-sweep: panel tree on the caller's stream; then, level by
// level, K1 and the part of K2 that the next level and the next panel read (the first
// chunk of every domain); the rest of K2 (the bulk of its work) is handed to a helper
// stream and overlaps the next half-sweep's panel, which only touches the first chunk.
// The next half-sweep's K1 waits for it.
template <typename T, typename C>
int ge2gb_impl(int64_t n, T* A, int64_t lda, int nb, C* band, int64_t ldab, unsigned char* work,
               const Carve& cv, hipStream_t caller)
{
    const int g = domain_chunks(sizeof(C) == 8 ? SVB_F64 : SVB_F32, nb);
    // update: 2 = one pass over the trailing matrix per tree level (default, when the domain fits
    // the kernel's registers), 1 = two MFMA kernels with look-ahead, 0 = plain FMA kernels
    int impl = env_int("SVB_UPDATE_IMPL", 2);
    if (impl == 2 && g * nb > fused_update_rows<C>()) impl = 1;
    if (impl == 2 && env_int("SVB_PIPELINE", 1) != 0 && g_la.init())
        return ge2gb_pipeline<T, C>(n, A, lda, nb, band, ldab, work, cv, g, caller);
    const bool la = impl != 0 && env_int("SVB_LOOKAHEAD", 1) != 0 && g_la.init();
    const int64_t N = n / nb;
    Level lv[kMaxLevels];
    int64_t woff[kMaxLevels];
    // with look-ahead the work runs on the internal streams, forked from the caller's here and
    // joined back at the end
    hipStream_t s = caller;
    if (la) {
        s = g_la.m;
        (void)hipEventRecord(g_la.fork, caller);
        (void)hipStreamWaitEvent(s, g_la.fork, 0);
    }

    launch_band_clear<C>(band, ldab, n, s);
    int hs = 0;            // half-sweep counter: selects the buffer set and the events
    bool pending = false;  // deferred K2 work of the previous half-sweep is in flight on the helper stream
    for (int64_t k = 0; k < N; ++k) {
        for (int half = 0; half < 2; ++half) {
            const bool lq = half == 1;
            if (lq && k == N - 1) break;
            const int set = hs & 1;
            C* Vb = reinterpret_cast<C*>(work + cv.off_V[set]);
            C* Yb = reinterpret_cast<C*>(work + cv.off_Y[set]);
            C* Wb = reinterpret_cast<C*>(work + cv.off_W[set]);
            C* Tb = reinterpret_cast<C*>(work + cv.off_T[set]);
            // panel: QR -> rows k*nb.., columns k*nb..; LQ -> rows k*nb.., columns (k+1)*nb..
            const int64_t row0 = k * nb;
            const int64_t col0 = lq ? (k + 1) * nb : k * nb;
            const int64_t len = lq ? n - (k + 1) * nb : n - k * nb;
            const int nl = build_levels(len, nb, g, lv);
            g_prof.begin(SVB_PROF_PANEL, s, 2.0 * (double)len * nb * nb, 0.0);
            // the blocked panel kernel reads the first level's panel straight from the matrix and
            // writes the last level's R straight into the band; the other kernels go through a
            // gathered copy and a scatter
            const bool direct = panel_blk_serves<C>(nb, g);
            if (!direct) launch_panel_gather<T, C>(A, lda, row0, col0, lq, len, nb, Vb + lv[0].poff, lv[0].ldp, s);
            for (int L = 0; L < nl; ++L) {
                // the R factors of level L are stacked into level L+1's panel; the last
                // level's single R lands right behind it
                const int64_t next_off = lv[L].poff + lv[L].ldp * nb;
                const int64_t ldnext = (int64_t)lv[L].domains * nb;
                const bool last = L == nl - 1;
                launch_panel_qr<T, C>(nb, Vb + lv[L].poff, lv[L].ldp, Yb + lv[L].poff, Tb, lv[L].chunks, g,
                                      Vb + next_off, ldnext, (direct && L == 0) ? A + row0 + col0 * lda : nullptr, lda, lq,
                                      (direct && last) ? band : nullptr, ldab, row0, col0, s);
                if (last && !direct)
                    launch_scatter_r<C>(Vb + next_off, ldnext, nb, band, ldab, row0, col0, lq, s);
            }
            g_prof.end(s);
            // the previous half-sweep's deferred update must be complete before this one's K1
            if (pending) {
                (void)hipStreamWaitEvent(s, g_la.rest[(hs - 1) & 1], 0);
                pending = false;
            }
            // trailing matrix: QR -> rows k*nb.., columns (k+1)*nb..;  LQ -> rows (k+1)*nb.., columns (k+1)*nb..
            const int64_t qlen = n - (k + 1) * nb;
            if (qlen > 0) {
                T* Cb = lq ? A + (k + 1) * nb + (k + 1) * nb * lda : A + k * nb + (k + 1) * nb * lda;
                int64_t wo = 0;
                bool any_rest = false;
                for (int L = 0; L < nl; ++L) {
                    woff[L] = wo;
                    wo += (int64_t)lv[L].domains * nb * qlen;
                    any_rest = any_rest || lv[L].chunks > lv[L].domains;
                }
                // splitting pays once a launch is many rounds of workgroups; below that
                // both parts would take as long as the whole
                const bool big = impl != 2 || (int64_t)lv[0].domains * ((qlen + 63) / 64) >= env_int("SVB_LOOKAHEAD_MIN_TILES", 4096);
                const bool defer = la && any_rest && big;
                if (impl == 2) {
                    // one pass per level; with look-ahead split in two: the part the next panel
                    // waits for here, the rest on the helper stream under that panel
                    for (int L = 0; L < nl; ++L)
                        launch_update_fused<T, C>(nb, lq, Cb, lda, qlen, Vb + lv[L].poff, Yb + lv[L].poff,
                                                  lv[L].ldp, lv[L].chunks, g, lv[L].stride, L > 0, defer ? 1 : 0,
                                                  Wb + woff[L], (const C*)nullptr, L == 0, s);
                    if (defer) {
                        (void)hipEventRecord(g_la.crit[set], s);
                        (void)hipStreamWaitEvent(g_la.h, g_la.crit[set], 0);
                        for (int L = 0; L < nl; ++L)
                            if (lv[L].chunks > lv[L].domains)
                                launch_update_fused<T, C>(nb, lq, Cb, lda, qlen, Vb + lv[L].poff, Yb + lv[L].poff,
                                                          lv[L].ldp, lv[L].chunks, g, lv[L].stride, L > 0, 2,
                                                          Wb + woff[L], (const C*)nullptr, L == 0, g_la.h);
                        (void)hipEventRecord(g_la.rest[set], g_la.h);
                        pending = true;
                    }
                } else {
                for (int L = 0; L < nl; ++L)
                    launch_update<T, C>(nb, lq, Cb, lda, qlen, Vb + lv[L].poff, Yb + lv[L].poff, lv[L].ldp,
                                        lv[L].chunks, g, lv[L].stride, Wb + woff[L], impl, L == 0, defer ? 1 : 0, s);
                if (defer) {
                    (void)hipEventRecord(g_la.crit[set], s);
                    (void)hipStreamWaitEvent(g_la.h, g_la.crit[set], 0);
                    for (int L = 0; L < nl; ++L)
                        launch_update<T, C>(nb, lq, Cb, lda, qlen, Vb + lv[L].poff, Yb + lv[L].poff, lv[L].ldp,
                                            lv[L].chunks, g, lv[L].stride, Wb + woff[L], impl, L == 0, 2, g_la.h);
                    (void)hipEventRecord(g_la.rest[set], g_la.h);
                    pending = true;
                }
                }
            }
            ++hs;
        }
    }
    if (pending) (void)hipStreamWaitEvent(s, g_la.rest[(hs - 1) & 1], 0);
    if (la) {
        (void)hipEventRecord(g_la.join, s);
        (void)hipStreamWaitEvent(caller, g_la.join, 0);
    }
    return hipGetLastError() == hipSuccess ? SVB_OK : SVB_ERR_DEVICE;
}

int ge2gb_dispatch(svb_dtype dt, int64_t n, void* A, int64_t lda, int nb, void* band, int64_t ldab,
                   void* work, const Carve& cv, hipStream_t s)
{
    unsigned char* w = static_cast<unsigned char*>(work);
    switch (dt) {
    case SVB_F64: return ge2gb_impl<double, double>(n, (double*)A, lda, nb, (double*)band, ldab, w, cv, s);
    case SVB_F32: return ge2gb_impl<float, float>(n, (float*)A, lda, nb, (float*)band, ldab, w, cv, s);
    case SVB_F16: return ge2gb_impl<__half, float>(n, (__half*)A, lda, nb, (float*)band, ldab, w, cv, s);
    default: return SVB_ERR_UNSUPPORTED;
    }
}

}  // namespace

void prof_begin(int kind, hipStream_t s, double flops, double bytes) { g_prof.begin(kind, s, flops, bytes); }
void prof_end(hipStream_t s) { g_prof.end(s); }
bool prof_take(int kind, double flops, double bytes, hipEvent_t* start, hipEvent_t* stop)
{
    return g_prof.take(kind, flops, bytes, start, stop);
}

}  // namespace svb

using namespace svb;

extern "C" {

int svb_workspace_bytes(svb_dtype dt, int64_t m, int64_t n, int nb, size_t* dev_bytes, size_t* host_bytes)
{
    const int rc = check_shape(dt, m, n, nb);
    if (rc != SVB_OK) return rc;
    const Carve cv = carve(dt, n, nb);
    if (dev_bytes) *dev_bytes = cv.total;
    if (host_bytes) *host_bytes = 0;
    return SVB_OK;
}

int svb_ge2gb(svb_dtype dt, int64_t m, int64_t n, void* A_dev, int64_t lda, int nb, void* band_dev,
              int64_t ldab, void* work_dev, size_t work_bytes, void* stream)
{
    const int rc = check_shape(dt, m, n, nb);
    if (rc != SVB_OK) return rc;
    if (!A_dev || !band_dev || !work_dev || lda < m || ldab < 3 * (int64_t)nb) return SVB_ERR_ARG;
    if (!aligned_for_vectors(A_dev, lda) || reinterpret_cast<uintptr_t>(work_dev) % 256 != 0) return SVB_ERR_UNSUPPORTED;
    const Carve cv = carve(dt, n, nb);
    if (work_bytes < cv.total) return SVB_ERR_WORKSPACE;
    return ge2gb_dispatch(dt, n, A_dev, lda, nb, band_dev, ldab, work_dev, cv, (hipStream_t)stream);
}

int svb_gb2bd(svb_dtype band_dt, int64_t n, int nb, void* band_dev, int64_t ldab, void* d_dev,
              void* e_dev, void* work_dev, size_t work_bytes, void* stream)
{
    if (n < 0) return SVB_ERR_ARG;
    if (band_dt != SVB_F64 && band_dt != SVB_F32) return SVB_ERR_UNSUPPORTED;
    if (nb != 8 && nb != 32 && nb != 64 && nb != 128) return SVB_ERR_UNSUPPORTED;
    if (n == 0) return SVB_OK;
    if (!band_dev || !d_dev || !e_dev || ldab < 3 * (int64_t)nb) return SVB_ERR_ARG;
    if (work_bytes < gb2bd_bytes(n, nb)) return SVB_ERR_WORKSPACE;
    if (!work_dev) return SVB_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    const double cs = band_dt == SVB_F64 ? 8.0 : 4.0;
    prof_begin(SVB_PROF_CHASE, s, 6.0 * (double)n * (double)n * nb, 3.0 * (double)n * (double)n * nb * cs);
    int rc;
    if (band_dt == SVB_F64)
        rc = gb2bd_typed<double>(n, nb, (double*)band_dev, ldab, (double*)d_dev, (double*)e_dev, work_dev, work_bytes, s);
    else
        rc = gb2bd_typed<float>(n, nb, (float*)band_dev, ldab, (float*)d_dev, (float*)e_dev, work_dev, work_bytes, s);
    prof_end(s);
    return rc;
}

int svb_gb2bd_workspace_bytes(int64_t n, int nb, size_t* dev_bytes)
{
    if (n < 0 || !dev_bytes) return SVB_ERR_ARG;
    if (nb != 8 && nb != 32 && nb != 64 && nb != 128) return SVB_ERR_UNSUPPORTED;
    *dev_bytes = gb2bd_bytes(n, nb);
    return SVB_OK;
}

int svb_bdsvals_dev_workspace_bytes(int64_t n, size_t* dev_bytes)
{
    if (n < 0 || !dev_bytes) return SVB_ERR_ARG;
    *dev_bytes = bdsvals_dev_workspace_bytes(n);
    return SVB_OK;
}

int svb_bdsvals_dev(svb_dtype band_dt, int64_t n, const void* d_dev, const void* e_dev, void* sigma_dev,
                    double rel_tol, void* work_dev, size_t work_bytes, void* stream)
{
    if (n < 0) return SVB_ERR_ARG;
    if (band_dt != SVB_F64 && band_dt != SVB_F32) return SVB_ERR_UNSUPPORTED;
    if (n == 0) return SVB_OK;
    if (!d_dev || !e_dev || !sigma_dev || !work_dev || rel_tol < 0.0) return SVB_ERR_ARG;
    if (work_bytes < bdsvals_dev_workspace_bytes(n)) return SVB_ERR_WORKSPACE;
    if (rel_tol == 0.0) rel_tol = band_dt == SVB_F64 ? 0x1p-52 : 0x1p-29;
    hipStream_t s = (hipStream_t)stream;
    if (band_dt == SVB_F64)
        return run_bdsvals_dev<double>(n, (const double*)d_dev, (const double*)e_dev, (double*)sigma_dev, work_dev, rel_tol, 0.0, s);
    return run_bdsvals_dev<float>(n, (const float*)d_dev, (const float*)e_dev, (float*)sigma_dev, work_dev, rel_tol, 0.0, s);
}

int svb_bdsvals(int64_t n, const double* d, const double* e, double* sigma)
{
    return host_bdsvals(n, d, e, sigma);
}

int svb_svdvals(svb_dtype dt, int64_t m, int64_t n, void* A_dev, int64_t lda, void* S_out_host, int nb,
                void* work_dev, size_t work_bytes, void* stream)
{
    int rc = check_shape(dt, m, n, nb);
    if (rc != SVB_OK) return rc;
    if (!A_dev || !S_out_host || !work_dev || lda < m) return SVB_ERR_ARG;
    if (!aligned_for_vectors(A_dev, lda) || reinterpret_cast<uintptr_t>(work_dev) % 256 != 0) return SVB_ERR_UNSUPPORTED;
    const Carve cv = carve(dt, n, nb);
    if (work_bytes < cv.total) return SVB_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    unsigned char* w = static_cast<unsigned char*>(work_dev);
    void* band = w + cv.off_band;
    void* dd = w + cv.off_d;
    void* de = w + cv.off_e;
    const int64_t ldab = 3 * (int64_t)nb;
    const svb_dtype bdt = dt == SVB_F64 ? SVB_F64 : SVB_F32;

    hipEvent_t ev0, ev1, ev2;
    if (hipEventCreate(&ev0) != hipSuccess || hipEventCreate(&ev1) != hipSuccess ||
        hipEventCreate(&ev2) != hipSuccess)
        return SVB_ERR_DEVICE;
    (void)hipEventRecord(ev0, s);
    rc = ge2gb_dispatch(dt, n, A_dev, lda, nb, band, ldab, work_dev, cv, s);
    (void)hipEventRecord(ev1, s);
    if (rc == SVB_OK) {
        void* cw = w + cv.off_err + 256;
        rc = svb_gb2bd(bdt, n, nb, band, ldab, dd, de, cw, gb2bd_bytes(n, nb), s);
    }
    (void)hipEventRecord(ev2, s);
    const bool host3 = [] { const char* v = std::getenv("SVB_STAGE3"); return v && std::strcmp(v, "host") == 0; }();
    const size_t cs = compute_size(dt);
    double total3 = 0.0;
    hipEvent_t ev3 = nullptr;
    std::vector<double> hs((size_t)n);
    if (rc == SVB_OK && !host3) {
        // stage 3 on the device, then one copy of n values
        void* sig = w + cv.off_sig;
        // The two reductions leave every singular value with an absolute error of the order of
        // eps * sigma_max, so the bidiagonal's small values are refined to tol times an eighth of
        // the bound on sigma_max (2^-3 eps sigma_max in f64, 2^-9 in f32), not to tol times
        // themselves, which costs them two to three times as many rounds.
        const double tol = dt == SVB_F64 ? 0x1p-52 : 0x1p-29;
        const double floor_frac = env_int("SVB_STAGE3_RELATIVE", 0) ? 0.0 : 0.125;
        if (dt == SVB_F64)
            rc = run_bdsvals_dev<double>(n, (const double*)dd, (const double*)de, (double*)sig, w + cv.off_s3, tol,
                                         floor_frac, s);
        else
            rc = run_bdsvals_dev<float>(n, (const float*)dd, (const float*)de, (float*)sig, w + cv.off_s3, tol,
                                        floor_frac, s);
        if (hipEventCreate(&ev3) == hipSuccess) (void)hipEventRecord(ev3, s);
        if (rc == SVB_OK &&
            (hipMemcpyAsync(S_out_host, sig, (size_t)n * cs, hipMemcpyDeviceToHost, s) != hipSuccess ||
             hipStreamSynchronize(s) != hipSuccess))
            rc = SVB_ERR_DEVICE;
        if (rc == SVB_OK) {
            const bool bad = dt == SVB_F64 ? std::isnan(static_cast<double*>(S_out_host)[0])
                                           : std::isnan(static_cast<float*>(S_out_host)[0]);
            if (bad) rc = SVB_ERR_NONFINITE;
        }
    } else if (rc == SVB_OK) {
        std::vector<double> hd((size_t)n), he((size_t)n);
        std::vector<unsigned char> raw(2 * (size_t)n * cs);
        if (hipMemcpyAsync(raw.data(), dd, (size_t)n * cs, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipMemcpyAsync(raw.data() + (size_t)n * cs, de, (size_t)n * cs, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess) {
            rc = SVB_ERR_DEVICE;
        } else if (dt == SVB_F64) {
            std::memcpy(hd.data(), raw.data(), (size_t)n * 8);
            std::memcpy(he.data(), raw.data() + (size_t)n * 8, (size_t)n * 8);
        } else {
            const float* fd = reinterpret_cast<const float*>(raw.data());
            for (int64_t i = 0; i < n; ++i) {
                hd[(size_t)i] = fd[i];
                he[(size_t)i] = fd[n + i];
            }
        }
        const auto t3a = std::chrono::steady_clock::now();
        if (rc == SVB_OK) rc = host_bdsvals(n, hd.data(), he.data(), hs.data());
        total3 = std::chrono::duration<double>(std::chrono::steady_clock::now() - t3a).count();
        if (rc == SVB_OK) {
            if (dt == SVB_F64) std::memcpy(S_out_host, hs.data(), (size_t)n * 8);
            else
                for (int64_t i = 0; i < n; ++i) static_cast<float*>(S_out_host)[i] = (float)hs[(size_t)i];
        }
    } else {
        (void)hipStreamSynchronize(s);
    }
    float ms1 = 0, ms2 = 0;
    (void)hipEventElapsedTime(&ms1, ev0, ev1);
    (void)hipEventElapsedTime(&ms2, ev1, ev2);
    if (ev3) {
        float ms3 = 0;
        if (hipEventElapsedTime(&ms3, ev2, ev3) == hipSuccess) total3 = ms3 * 1e-3;
        (void)hipEventDestroy(ev3);
    }
    (void)hipEventDestroy(ev0);
    (void)hipEventDestroy(ev1);
    (void)hipEventDestroy(ev2);
    if (rc == SVB_OK && hipGetLastError() != hipSuccess) rc = SVB_ERR_DEVICE;
    if (g_prof.on) g_prof.collect();
    g_last.s1 = ms1 * 1e-3;
    g_last.s2 = ms2 * 1e-3;
    g_last.s3 = total3;
    return rc;
}

int svb_last_timings(double* t_stage1, double* t_stage2, double* t_stage3)
{
    if (t_stage1) *t_stage1 = g_last.s1;
    if (t_stage2) *t_stage2 = g_last.s2;
    if (t_stage3) *t_stage3 = g_last.s3;
    return SVB_OK;
}

int svb_profile_enable(int on)
{
    g_prof.reset();
    g_prof.on = on != 0;
    return SVB_OK;
}

int svb_profile_collect(void)
{
    g_prof.collect();
    return SVB_OK;
}

int svb_profile_get(int kind, double* seconds, int64_t* launches, double* flops, double* bytes)
{
    if (kind < 0 || kind >= SVB_PROF_KINDS) return SVB_ERR_ARG;
    if (seconds) *seconds = g_prof.sec[kind];
    if (launches) *launches = g_prof.count[kind];
    if (flops) *flops = g_prof.flops[kind];
    if (bytes) *bytes = g_prof.bytes[kind];
    return SVB_OK;
}

const char* svb_status_string(int status)
{
    switch (status) {
    case SVB_OK: return "ok";
    case SVB_ERR_ARG: return "invalid argument";
    case SVB_ERR_UNSUPPORTED: return "unsupported shape, tile size or dtype";
    case SVB_ERR_WORKSPACE: return "workspace too small";
    case SVB_ERR_DEVICE: return "HIP error";
    case SVB_ERR_NOCONV: return "bidiagonal solver did not converge";
    case SVB_ERR_NONFINITE: return "non-finite value in the bidiagonal";
    default: return "unknown status";
    }
}

}  // extern "C"
