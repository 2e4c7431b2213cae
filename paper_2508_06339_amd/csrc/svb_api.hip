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

bool dtype_ok(svb_dtype dt) { return dt == SVB_F64 || dt == SVB_F32 || dt == SVB_F16 || dt == SVB_BF16; }
bool nb_ok(int nb) { return nb == 32 || nb == 64 || nb == 128; }

// Tile size chosen when the caller passes nb = 0 (the paper tunes TILESIZE per size and
// hardware, Section 4 and Table 3).  From timings of svb_svdvals on MI355X at orders 1024 .. 24576:
// small tiles shorten the panel chain and stage 2, large tiles raise the arithmetic intensity of
// the trailing update, which only pays once the update dominates.  In f32 arithmetic nb = 64 is
// fastest from order 1024 up to about 20000 (16384: 365 ms against 410 ms at nb = 128), nb = 128
// beyond (24576: 842 ms against 854 ms); in f64, where a register-resident domain holds half as
// many rows, nb = 32 up to about 6000 (6144: 120 ms against 123 ms at nb = 64) and nb = 64 beyond
// (16384: 619 ms against 922 ms at nb = 128).
int choose_nb(svb_dtype dt, int64_t m, int64_t n)
{
    const int64_t k = m < n ? m : n;
    if (dt == SVB_F64) return k <= 2560 ? 32 : 64;
    if (k < 1024) return 32;
    return k <= 26624 ? 64 : 128;
}

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// The shape stage 1 works on: rows >= cols, both whole numbers of tiles.  `staged` says the input
// has to be copied (zero padded, transposed if it is wider than tall) into the workspace first.
struct Shape {
    int64_t rows, cols;   // of the matrix stage 1 factors (padded)
    int64_t k;            // min(m, n): number of singular values
    bool transpose, staged;
};
Shape shape_of(int64_t m, int64_t n, int nb)
{
    Shape sh{};
    sh.transpose = m < n;
    const int64_t r = sh.transpose ? n : m, c = sh.transpose ? m : n;
    sh.rows = round_up(r, nb);
    sh.cols = round_up(c, nb);
    sh.k = c;
    sh.staged = sh.transpose || sh.rows != r || sh.cols != c;
    return sh;
}

int check_shape(svb_dtype dt, int64_t m, int64_t n, int nb)
{
    if (m < 0 || n < 0) return SVB_ERR_ARG;
    if (!dtype_ok(dt) || !nb_ok(nb)) return SVB_ERR_UNSUPPORTED;
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

// Algorithmic bytes of the two stage-2 kernels: the band reduction reads and writes every nb x nb
// block once per block sweep (two blocks per step, about n/nb - 8s/nb steps in sweep s, n/8
// sweeps: n^2 nb / 4 elements each way in all ... counted as 2 * 2 * nb^2 per step); the narrow
// chase reads and writes the band's 24 stored rows from its first column on once per bundle.
double band_reduce_bytes(int64_t n, int nb, size_t cs)
{
    double steps = 0.0;
    for (int64_t s = 0; s < (n - 1) / 8; ++s) steps += (double)((n - 1 - (s + 1) * 8) / nb + 1);
    return steps * 4.0 * (double)nb * nb * (double)cs;
}
double narrow_bytes(int64_t n, size_t cs)
{
    const int64_t nw = cs == 8 ? 24 : 48;
    double cols = 0.0;
    for (int64_t i0 = 0; i0 < n - 2; i0 += nw) cols += (double)(n - i0);
    return cols * 24.0 * 2.0 * (double)cs;
}

template <typename C>
int gb2bd_typed(int64_t n, int nb, C* band, int64_t ldab, C* d, C* e, void* work, size_t work_bytes, hipStream_t s)
{
    int* ctrl = static_cast<int*>(work);
    if (nb == 8) {
        // narrow band: bundles of sweeps inside LDS windows
        prof_begin(SVB_PROF_NARROW, s, 0.0, narrow_bytes(n, sizeof(C)));
        const int rc = run_chase_narrow<C>(n, band, ldab, 15, ctrl, s);
        prof_end(s);
        launch_extract_bidiag<C>(band, ldab, n, 8, d, e, ctrl, nullptr, s);
        return rc;
    }
    if (two_phase(nb, sizeof(C), n)) {
        int* ctrl2 = reinterpret_cast<int*>(static_cast<unsigned char*>(work) + gb2bd_first_bytes(n, nb));
        prof_begin(SVB_PROF_BAND_REDUCE, s, 0.0, band_reduce_bytes(n, nb, sizeof(C)));
        int rc = run_band_reduce<C>(n, nb, band, ldab, ctrl, s);
        prof_end(s);
        if (rc == SVB_OK) {
            prof_begin(SVB_PROF_NARROW, s, 0.0, narrow_bytes(n, sizeof(C)));
            rc = run_chase_narrow<C>(n, band, ldab, 2 * (int64_t)nb - 1, ctrl2, s);
            prof_end(s);
        }
        launch_extract_bidiag<C>(band, ldab, n, nb, d, e, ctrl, ctrl2, s);
        return rc;
    }
    prof_begin(SVB_PROF_BAND_REDUCE, s, 0.0, 3.0 * (double)n * (double)n * nb * sizeof(C));
    const int rc = run_chase<C>(n, nb, band, ldab, d, e, work, work_bytes, s);
    prof_end(s);
    return rc;
}

// the update kernels move 16-byte vectors along both directions of A
bool aligned_for_vectors(const void* A, int64_t lda, svb_dtype dt)
{
    return reinterpret_cast<uintptr_t>(A) % 16 == 0 && lda % (dt == SVB_F64 ? 2 : 4) == 0;
}

// Environment switches, read once per process (they select kernel variants kept for testing and
// measurement; the launch loops consult this copy).
struct Switches {
    int domain_chunks, pipeline_layout, tree_spin, update_h16, ext_events, update_t, event_fence, stage3_host, stage3_relative, no_scale;
    bool loaded = false;
    void load()
    {
        domain_chunks = env_int("SVB_DOMAIN_CHUNKS", 0);
        pipeline_layout = env_int("SVB_PIPELINE_LAYOUT", 2);
        tree_spin = env_int("SVB_TREE_SPIN", 1 << 22);
        update_h16 = env_int("SVB_UPDATE_H16", 1);
        ext_events = env_int("SVB_EXT_EVENTS", 1);
        update_t = env_int("SVB_UPDATE_T", 1);
        event_fence = env_int("SVB_EVENT_FENCE", 0);
        const char* v = std::getenv("SVB_STAGE3");
        stage3_host = v && std::strcmp(v, "host") == 0;
        stage3_relative = env_int("SVB_STAGE3_RELATIVE", 0);
        no_scale = env_int("SVB_NO_SCALE", 0);
        loaded = true;
    }
} g_sw;
// (tests change the variables between calls: every entry point reloads them once, outside the
// launch loops)
const Switches& switches() { g_sw.load(); return g_sw; }

// chunks-per-domain of the panel tree: as many nb-row tiles as the register-resident
// panel and update kernels hold (512 rows in f32, 256 in f64)
int domain_chunks(svb_dtype dt, int nb, const Switches& sw)
{
    const int cap = (dt == SVB_F64 ? 256 : 512) / nb;
    const int g = sw.domain_chunks;
    if (g >= 2 && g <= cap) return g;
    return cap;
}
constexpr int kMinDomainChunks = 2;  // workspace is sized for any g >= this
constexpr size_t kTreeHead = 4;      // ints in front of the tickets of the panel tree's control block

// Workspace layout.  V, Y, T: the panels and factors of one half-sweep's tree (element counts in
// the compute type); stage: the zero-padded copy of an input that is not a whole number of tiles
// or is wider than tall (storage type).
struct Carve {
    size_t panel_elems, t_elems, band_elems, de_elems, stage_elems, tree_ints;
    size_t off_V, off_Y, off_T, off_band, off_d, off_e, off_sig, off_s3, off_fac, off_gb, off_tree, off_stage, total;
};

Carve carve(svb_dtype dt, const Shape& sh, int nb)
{
    Carve c{};
    const size_t cs = compute_size(dt);
    const int64_t rows = sh.rows, cols = sh.cols;
    // levels shrink by >= kMinDomainChunks: sum of panel rows <= 2 rows (+ one chunk per level)
    c.panel_elems = (size_t)(2 * rows + (int64_t)(kMaxLevels + 2) * nb) * nb;
    c.t_elems = 2 * (size_t)(rows / nb + 1) * nb * nb;  // T per domain, plus room for the v^T v products
    c.band_elems = (size_t)(3 * nb) * (size_t)cols;
    c.de_elems = (size_t)cols;
    c.stage_elems = sh.staged ? (size_t)rows * (size_t)cols : 0;
    // panel tree hand-over: error flag, one ticket counter per half-sweep, one flag per domain
    c.tree_ints = kTreeHead + 2 * (size_t)(cols / nb) + 2 + (size_t)(rows / nb) + kMaxLevels + 2;
    size_t off = 0;
    c.off_V = off; off += align_up(c.panel_elems * cs);
    c.off_Y = off; off += align_up(c.panel_elems * cs);
    c.off_T = off; off += align_up(c.t_elems * cs);
    c.off_band = off; off += align_up(c.band_elems * cs);
    c.off_d = off; off += align_up(c.de_elems * cs);
    c.off_e = off; off += align_up(c.de_elems * cs);
    c.off_sig = off; off += align_up(c.de_elems * cs);
    c.off_s3 = off; off += align_up(bdsvals_dev_workspace_bytes(sh.k));
    c.off_fac = off; off += align_up(scale_workspace_bytes());
    c.off_gb = off; off += align_up(gb2bd_bytes(sh.k, nb));
    c.off_tree = off; off += align_up(c.tree_ints * sizeof(int));
    c.off_stage = off; off += align_up(c.stage_elems * storage_size(dt));
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

struct Timings { double s1 = 0, s2 = 0, s3 = 0, upd = -1; } g_last;

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

// Streams and events of stage 1 (created once per process).  Stage 1 runs on two internal
// streams forked from the caller's stream and joined back to it: `m` carries the panel tree and
// the last level's update, `u` the updates of the levels below.  (The chain does not run on the
// caller's stream itself so that it never serialises with the NULL stream.)
void g_la_release();
struct Lookahead {
    hipStream_t m = nullptr, u = nullptr;
    hipEvent_t fork = nullptr, join = nullptr, join_u = nullptr;
    // level pipeline: panel level L of a half-sweep done / the side stream's updates done
    hipEvent_t lvl[2][kMaxLevels] = {}, udone[2] = {nullptr, nullptr};
    // stage boundaries of svb_svdvals, reused by every call
    hipEvent_t stage[4] = {nullptr, nullptr, nullptr, nullptr};
    bool ok = false, tried = false;
    bool init(const Switches& sw)
    {
        if (tried) return ok;
        tried = true;
        if (hipStreamCreateWithFlags(&m, hipStreamNonBlocking) != hipSuccess) return false;
        if (hipStreamCreateWithFlags(&u, hipStreamNonBlocking) != hipSuccess) return false;
        // events between the two internal streams order kernels of one device against each other:
        // no system-scope fence (a cache write-back for the host's and other devices' benefit) is
        // needed when they are recorded, and it would sit on the critical path of every half-sweep
        const unsigned kInner = sw.event_fence ? hipEventDisableTiming
                                               : (hipEventDisableTiming | hipEventDisableSystemFence);
        for (int i = 0; i < 2; ++i) {
            if (hipEventCreateWithFlags(&udone[i], kInner) != hipSuccess) return false;
            for (int L = 0; L < kMaxLevels; ++L)
                if (hipEventCreateWithFlags(&lvl[i][L], kInner) != hipSuccess) return false;
        }
        if (hipEventCreateWithFlags(&fork, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&join, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&join_u, hipEventDisableTiming) != hipSuccess)
            return false;
        for (int i = 0; i < 4; ++i)
            if (hipEventCreate(&stage[i]) != hipSuccess) return false;
        ok = true;
        // released while the HIP runtime is still up (handlers registered later run earlier)
        std::atexit([] { g_la_release(); });
        return true;
    }
    void release()
    {
        if (!ok) return;
        ok = false;
        (void)hipStreamSynchronize(u);
        (void)hipStreamSynchronize(m);
        for (int i = 0; i < 2; ++i) {
            (void)hipEventDestroy(udone[i]);
            for (int L = 0; L < kMaxLevels; ++L) (void)hipEventDestroy(lvl[i][L]);
        }
        (void)hipEventDestroy(fork);
        (void)hipEventDestroy(join);
        (void)hipEventDestroy(join_u);
        for (int i = 0; i < 4; ++i) (void)hipEventDestroy(stage[i]);
        (void)hipStreamDestroy(u);
        (void)hipStreamDestroy(m);
    }
} g_la;
void g_la_release() { g_la.release(); }

// Stage 1 driver (Section 3.1, Algorithms 1 and 2): for every tile column k a QR half-sweep
// (panel = block column k from the diagonal down, update = the columns right of it) and, but for
// the last one, an LQ half-sweep (panel = block row k right of the diagonal tile, update = the
// rows below it).  The matrix is rows x cols, rows >= cols, both whole numbers of tiles.
//
// Two internal streams.  The tree levels of a panel depend on each other only through the R
// factors, not through the trailing matrix.  Default (SVB_PIPELINE_LAYOUT=2): the first level's
// kernel K_A on the main stream, every level above it in one kernel K_B on the side stream, both
// started behind the previous half-sweep's last update and running side by side (K_B's levels one
// block step behind the level below, see stage1_panel_blk.hip); every update on the main stream,
//     main: K_A U0 [K_B done] U1 .. Ul K_A' ..      side: K_B
// so that a half-sweep costs K_A, its updates and their launch gaps.  Kept for testing: one launch
// per level, main: P0 P1 .. Pl Ul P0' .., side: U0 .. Ul-1 (=1), or every update on the side
// stream (=0).
template <typename T, typename C>
int ge2gb_pipeline(int64_t rows, int64_t cols, T* A, int64_t lda, int nb, C* band, int64_t ldab,
                   unsigned char* work, const Carve& cv, int g, const Switches& sw, hipStream_t caller)
{
    const int64_t N = cols / nb;
    Level lv[kMaxLevels];
    hipStream_t ms = g_la.m, ss = g_la.u;
    (void)hipEventRecord(g_la.fork, caller);
    (void)hipStreamWaitEvent(ms, g_la.fork, 0);
    (void)hipStreamWaitEvent(ss, g_la.fork, 0);
    launch_band_clear<C>(band, ldab, cols, ms);
    // control block of the panel tree: error flag, a ticket counter per half-sweep, a flag per domain
    int* const tree_err = reinterpret_cast<int*>(work + cv.off_tree);
    int* const tree_tickets = tree_err + kTreeHead;
    int* const tree_flags = tree_tickets + 2 * N + 2;
    launch_fill_int(tree_err, (int)cv.tree_ints, 0, ms);
    C* Vb = reinterpret_cast<C*>(work + cv.off_V);
    C* Yb = reinterpret_cast<C*>(work + cv.off_Y);
    C* Tb = reinterpret_cast<C*>(work + cv.off_T);
    const bool direct = panel_blk_serves<C>(nb, g);
    const int layout = sw.pipeline_layout;
    // a level's event is tied to the completion of its kernel instead of being recorded behind it
    // (one marker less in the main stream between two panel levels)
    const bool ext_events = sw.ext_events != 0;
    int hs = 0;
    bool side_pending = false;
    for (int64_t k = 0; k < N; ++k) {
        for (int half = 0; half < 2; ++half) {
            const bool lq = half == 1;
            if (lq && k == N - 1) break;
            const int set = hs & 1;
            const int64_t row0 = k * nb;
            const int64_t col0 = lq ? (k + 1) * nb : k * nb;
            // panel length (along the panel direction) and the extent of the trailing matrix
            // across it: a QR panel runs down the rows, its update covers the columns right of it;
            // an LQ panel runs along the columns, its update covers the rows below it
            const int64_t len = lq ? cols - (k + 1) * nb : rows - k * nb;
            const int64_t qlen = lq ? rows - (k + 1) * nb : cols - (k + 1) * nb;
            const int nl = build_levels(len, nb, g, lv);
            // every level keeps its own T factors until its update has run: the update applies
            // them itself (no Y = V T between a panel and its update) where they all fit
            int64_t toff[kMaxLevels], tsum = 0;
            for (int L = 0; L < nl; ++L) {
                toff[L] = tsum;
                tsum += (int64_t)lv[L].domains * nb * nb;
            }
            const bool useT = direct && nb <= 64 && tsum <= (int64_t)cv.t_elems && sw.update_t != 0;
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
                                          lv[L].chunks, g, lv[L].stride, L > 0,
                                          useT ? Tb + toff[L] : (const C*)nullptr, L == 0, st, sw.update_h16 != 0);
            };
            if (layout == 2 && direct && nl > 1 && tsum <= (int64_t)cv.t_elems) {
                // Tree in two launches that run side by side: the first level on the main stream, every
                // level above it in one kernel on the side stream, each level one block step behind the
                // level below (TreeSync in stage1_panel_blk.hip).  Every update follows on the main
                // stream: U0 needs the first level only, the others wait for the side stream.
                int foff[kMaxLevels], fsum = 0;
                for (int L = 0; L < nl; ++L) {
                    foff[L] = fsum;
                    fsum += lv[L].domains;
                }
                const int base = (hs + 1) * 64;
                (void)hipEventRecord(g_la.lvl[set][0], ms);   // behind the previous half-sweep's last update
                (void)hipStreamWaitEvent(ss, g_la.lvl[set][0], 0);
                PanelTreeArgs<C> ta{};
                int first = 0;
                for (int L = 1; L < nl; ++L) {
                    PanelTreeLevel<C>& t = ta.lv[L - 1];
                    t.P = Vb + lv[L].poff;
                    t.Tws = Tb + toff[L];
                    t.Pnext = Vb + lv[L].poff + lv[L].ldp * nb;
                    t.ldp = lv[L].ldp;
                    t.ldnext = (int64_t)lv[L].domains * nb;
                    t.chunks = lv[L].chunks;
                    t.tiles = (lv[L].chunks < g ? lv[L].chunks : g) * nb / 16;
                    t.first = first;
                    first += lv[L].domains;
                    t.flags_in = foff[L - 1];
                    t.flags_out = foff[L];
                }
                ta.nl = nl - 1; ta.total = first; ta.g = g; ta.lq = lq ? 1 : 0;
                ta.ticket = tree_tickets + hs; ta.flags = tree_flags; ta.err = tree_err;
                ta.flag_base = base; ta.spin_limit = sw.tree_spin;
                // (a few milliseconds of polls before the upper levels' launch leaves its tickets to the
                // first level's kernel: only a tool that runs one kernel at a time makes it wait that long)
                ta.started = tree_err + 1; ta.start_spin = 4096;
                ta.band = band; ta.ldab = ldab; ta.row0 = row0; ta.col0 = col0;
                // the first level; where Y = V T is wanted its completion is an event (tied to the kernel)
                // that the side stream's Y products wait for: the tree is complete when this kernel is
                hipEvent_t first_done = nullptr;
                {
                    hipEvent_t ea = nullptr, eb = nullptr;
                    const bool timed = prof_take(SVB_PROF_PANEL, 2.0 * (double)len * nb * nb, 0.0, &ea, &eb);
                    if (timed) first_done = eb;
                    else if (!useT) first_done = g_la.lvl[set][2];
                    launch_panel_blk<T, C>(nb, Vb + lv[0].poff, lv[0].ldp, Tb + toff[0], lv[0].chunks, g,
                                           Vb + lv[0].poff + lv[0].ldp * nb, (int64_t)lv[0].domains * nb,
                                           A + row0 + col0 * lda, lda, lq, nullptr, ldab, row0, col0, ms,
                                           (timed || ext_events) ? first_done : nullptr, ea, tree_flags + foff[0], base, &ta);
                    if (first_done && !timed && !ext_events) (void)hipEventRecord(first_done, ms);
                    if (!useT)
                        launch_panel_y_nb<C>(nb, Vb + lv[0].poff, Yb + lv[0].poff, Tb + toff[0], lv[0].ldp,
                                             (int64_t)lv[0].chunks * nb, g, ms);
                }
                hipEvent_t ea = nullptr, eb = nullptr;
                const bool timed = prof_take(SVB_PROF_PANEL, 0.0, 0.0, &ea, &eb);
                const bool tied = useT && (timed || ext_events);   // the tree is the side stream's last kernel
                hipEvent_t upper_done = timed ? eb : g_la.lvl[set][1];
                launch_panel_tree<C>(nb, ta, ss, ea, (tied || timed) ? upper_done : nullptr);
                if (!useT) {
                    (void)hipStreamWaitEvent(ss, first_done, 0);
                    for (int L = 1; L < nl; ++L)
                        launch_panel_y_nb<C>(nb, Vb + lv[L].poff, Yb + lv[L].poff, Tb + toff[L], lv[L].ldp,
                                             (int64_t)lv[L].chunks * nb, g, ss);
                }
                if (!tied) {
                    upper_done = g_la.lvl[set][1];
                    (void)hipEventRecord(upper_done, ss);
                }
                if (qlen > 0) update(0, ms);
                (void)hipStreamWaitEvent(ms, upper_done, 0);
                if (qlen > 0)
                    for (int L = 1; L < nl; ++L) update(L, ms);
                ++hs;
                continue;
            }
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
    launch_tree_err<C>(tree_err, band + (2 * nb - 1), ms);
    (void)hipEventRecord(g_la.join, ms);
    (void)hipEventRecord(g_la.join_u, ss);
    (void)hipStreamWaitEvent(caller, g_la.join, 0);
    (void)hipStreamWaitEvent(caller, g_la.join_u, 0);
    return hipGetLastError() == hipSuccess ? SVB_OK : SVB_ERR_DEVICE;
}

template <typename T, typename C>
int ge2gb_typed(svb_dtype dt, int64_t rows, int64_t cols, T* A, int64_t lda, int nb, C* band, int64_t ldab,
                unsigned char* work, const Carve& cv, const Switches& sw, hipStream_t s)
{
    if (!g_la.init(sw)) return SVB_ERR_DEVICE;
    const int g = domain_chunks(dt, nb, sw);
    return ge2gb_pipeline<T, C>(rows, cols, A, lda, nb, band, ldab, work, cv, g, sw, s);
}

int ge2gb_dispatch(svb_dtype dt, int64_t rows, int64_t cols, void* A, int64_t lda, int nb, void* band, int64_t ldab,
                   void* work, const Carve& cv, const Switches& sw, hipStream_t s)
{
    unsigned char* w = static_cast<unsigned char*>(work);
    switch (dt) {
    case SVB_F64: return ge2gb_typed<double, double>(dt, rows, cols, (double*)A, lda, nb, (double*)band, ldab, w, cv, sw, s);
    case SVB_F32: return ge2gb_typed<float, float>(dt, rows, cols, (float*)A, lda, nb, (float*)band, ldab, w, cv, sw, s);
    case SVB_F16: return ge2gb_typed<__half, float>(dt, rows, cols, (__half*)A, lda, nb, (float*)band, ldab, w, cv, sw, s);
    case SVB_BF16: return ge2gb_typed<bf16_t, float>(dt, rows, cols, (bf16_t*)A, lda, nb, (float*)band, ldab, w, cv, sw, s);
    default: return SVB_ERR_UNSUPPORTED;
    }
}

// staging copy and scaling, by storage type
void stage_copy_dispatch(svb_dtype dt, const void* A, int64_t lda, int64_t m, int64_t n, const Shape& sh, void* S,
                         hipStream_t s)
{
    switch (dt) {
    case SVB_F64: launch_stage_copy<double>((const double*)A, lda, m, n, sh.transpose, (double*)S, sh.rows, sh.rows, sh.cols, s); break;
    case SVB_F32: launch_stage_copy<float>((const float*)A, lda, m, n, sh.transpose, (float*)S, sh.rows, sh.rows, sh.cols, s); break;
    case SVB_F16: launch_stage_copy<__half>((const __half*)A, lda, m, n, sh.transpose, (__half*)S, sh.rows, sh.rows, sh.cols, s); break;
    default: launch_stage_copy<bf16_t>((const bf16_t*)A, lda, m, n, sh.transpose, (bf16_t*)S, sh.rows, sh.rows, sh.cols, s); break;
    }
}
void scale_dispatch(svb_dtype dt, void* A, int64_t lda, int64_t rows, int64_t cols, double* factors, hipStream_t s)
{
    switch (dt) {
    case SVB_F64: launch_scale_to_range<double>((double*)A, lda, rows, cols, factors, s); break;
    case SVB_F32: launch_scale_to_range<float>((float*)A, lda, rows, cols, factors, s); break;
    case SVB_BF16: launch_scale_to_range<bf16_t>((bf16_t*)A, lda, rows, cols, factors, s); break;
    default: {
        // f16 storage: the transformed matrix is written back in f16, and an entry of it can be as
        // large as a column's norm; the update's products W = Y^T C, bounded by a small multiple of
        // the Frobenius norm, are split into f16 terms as well.  So max|a| sqrt(rows cols) is
        // brought to about 2^11 (f16 holds 2^16; entries below 2^-24 of that flush to zero, far
        // below the storage type's rounding of the entries beside them)
        int e2 = 0;
        (void)std::frexp(std::sqrt((double)rows * (double)cols), &e2);   // sqrt(rows cols) <= 2^e2
        const int hi = 13 - e2;
        launch_scale_to_range<__half>((__half*)A, lda, rows, cols, factors, s, hi - 8, hi, hi - 2);
        break;
    }
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

// Scratch of svb_gb2bd_noalloc: part of the library's image on every device it runs on (each
// device holds its own copy at its own address until the process ends).  In host code the name is
// only a handle for hipGetSymbolAddress; kernels and memory operations get the looked-up pointer.
constexpr size_t kStaticScratchBytes = 1u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};

// device address of the current device's copy of the array (looked up once per device)
static int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SVB_ERR_DEVICE;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SVB_ERR_DEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SVB_OK;
}

extern "C" {

int svb_choose_nb(svb_dtype dt, int64_t m, int64_t n)
{
    if (m < 0 || n < 0 || !dtype_ok(dt)) return 0;
    return choose_nb(dt, m, n);
}

int svb_workspace_bytes(svb_dtype dt, int64_t m, int64_t n, int nb, size_t* dev_bytes, size_t* host_bytes)
{
    if (nb == 0 && m >= 0 && n >= 0 && dtype_ok(dt)) nb = choose_nb(dt, m, n);
    const int rc = check_shape(dt, m, n, nb);
    if (rc != SVB_OK) return rc;
    size_t total = 256;
    if (m > 0 && n > 0) total = carve(dt, shape_of(m, n, nb), nb).total;
    if (dev_bytes) *dev_bytes = total;
    if (host_bytes) *host_bytes = 0;
    return SVB_OK;
}

int svb_ge2gb(svb_dtype dt, int64_t m, int64_t n, void* A_dev, int64_t lda, int nb, void* band_dev,
              int64_t ldab, void* work_dev, size_t work_bytes, void* stream)
{
    const int rc = check_shape(dt, m, n, nb);
    if (rc != SVB_OK) return rc;
    // the stage-split entry point works in place: whole tiles, at least as many rows as columns
    if (m < n || m % nb != 0 || n % nb != 0 || n == 0) return SVB_ERR_UNSUPPORTED;
    if (!A_dev || !band_dev || !work_dev || lda < m || ldab < 3 * (int64_t)nb) return SVB_ERR_ARG;
    if (!aligned_for_vectors(A_dev, lda, dt) || reinterpret_cast<uintptr_t>(work_dev) % 256 != 0) return SVB_ERR_UNSUPPORTED;
    const Shape sh = shape_of(m, n, nb);
    const Carve cv = carve(dt, sh, nb);
    if (work_bytes < cv.total) return SVB_ERR_WORKSPACE;
    return ge2gb_dispatch(dt, m, n, A_dev, lda, nb, band_dev, ldab, work_dev, cv, switches(), (hipStream_t)stream);
}

static int gb2bd_checked(svb_dtype band_dt, int64_t n, int nb, void* band_dev, int64_t ldab, void* d_dev,
                         void* e_dev, void* work_dev, size_t work_bytes, hipStream_t s)
{
    if (band_dt == SVB_F64)
        return gb2bd_typed<double>(n, nb, (double*)band_dev, ldab, (double*)d_dev, (double*)e_dev, work_dev, work_bytes, s);
    return gb2bd_typed<float>(n, nb, (float*)band_dev, ldab, (float*)d_dev, (float*)e_dev, work_dev, work_bytes, s);
}

int svb_gb2bd(svb_dtype band_dt, int64_t n, int nb, void* band_dev, int64_t ldab, void* d_dev,
              void* e_dev, void* work_dev, size_t work_bytes, void* stream)
{
    if (n < 0) return SVB_ERR_ARG;
    if (band_dt != SVB_F64 && band_dt != SVB_F32) return SVB_ERR_UNSUPPORTED;
    if (nb != 8 && !nb_ok(nb)) return SVB_ERR_UNSUPPORTED;
    if (n == 0) return SVB_OK;
    if (!band_dev || !d_dev || !e_dev || ldab < 3 * (int64_t)nb) return SVB_ERR_ARG;
    if (work_bytes < gb2bd_bytes(n, nb)) return SVB_ERR_WORKSPACE;
    if (!work_dev) return SVB_ERR_ARG;
    return gb2bd_checked(band_dt, n, nb, band_dev, ldab, d_dev, e_dev, work_dev, work_bytes, (hipStream_t)stream);
}

int svb_gb2bd_noalloc(svb_dtype band_dt, int64_t n, int nb, void* band_dev, int64_t ldab, void* d_dev,
                      void* e_dev, void* stream)
{
    if (n < 0) return SVB_ERR_ARG;
    if (band_dt != SVB_F64 && band_dt != SVB_F32) return SVB_ERR_UNSUPPORTED;
    if (nb != 8 && !nb_ok(nb)) return SVB_ERR_UNSUPPORTED;
    if (n == 0) return SVB_OK;
    if (!band_dev || !d_dev || !e_dev || ldab < 3 * (int64_t)nb) return SVB_ERR_ARG;
    // the counters of the sweeps must fit the fixed array
    if (n > SVB_NOALLOC_MAX_N || gb2bd_bytes(n, nb) > kStaticScratchBytes) return SVB_ERR_WORKSPACE;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != SVB_OK) return rc;
    // (the kernels clear the counters they use at the start of every call)
    return gb2bd_checked(band_dt, n, nb, band_dev, ldab, d_dev, e_dev, ws, kStaticScratchBytes, (hipStream_t)stream);
}

int svb_gb2bd_workspace_bytes(int64_t n, int nb, size_t* dev_bytes)
{
    if (n < 0 || !dev_bytes) return SVB_ERR_ARG;
    if (nb != 8 && !nb_ok(nb)) return SVB_ERR_UNSUPPORTED;
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
    if (nb == 0 && m >= 0 && n >= 0 && dtype_ok(dt)) nb = choose_nb(dt, m, n);
    int rc = check_shape(dt, m, n, nb);
    if (rc != SVB_OK) return rc;
    if (m == 0 || n == 0) return SVB_OK;   // no singular values
    if (!A_dev || !S_out_host || !work_dev || lda < m) return SVB_ERR_ARG;
    if (reinterpret_cast<uintptr_t>(work_dev) % 256 != 0) return SVB_ERR_UNSUPPORTED;
    const Shape sh = shape_of(m, n, nb);
    // in place only where the kernels' 16-byte accesses are aligned
    if (!sh.staged && !aligned_for_vectors(A_dev, lda, dt)) return SVB_ERR_UNSUPPORTED;
    const Carve cv = carve(dt, sh, nb);
    if (work_bytes < cv.total) return SVB_ERR_WORKSPACE;
    const Switches& sw = switches();
    if (!g_la.init(sw)) return SVB_ERR_DEVICE;
    hipStream_t s = (hipStream_t)stream;
    unsigned char* w = static_cast<unsigned char*>(work_dev);
    void* band = w + cv.off_band;
    void* dd = w + cv.off_d;
    void* de = w + cv.off_e;
    double* factors = reinterpret_cast<double*>(w + cv.off_fac);
    const int64_t ldab = 3 * (int64_t)nb;
    const int64_t k = sh.k;
    const svb_dtype bdt = dt == SVB_F64 ? SVB_F64 : SVB_F32;
    const bool scaled = !sw.no_scale;

    hipEvent_t* ev = g_la.stage;
    (void)hipEventRecord(ev[0], s);
    // the matrix stage 1 works on: the caller's, or its zero-padded (transposed) copy
    void* A1 = A_dev;
    int64_t ld1 = lda;
    if (sh.staged) {
        A1 = w + cv.off_stage;
        ld1 = sh.rows;
        stage_copy_dispatch(dt, A_dev, lda, m, n, sh, A1, s);
    }
    if (scaled) scale_dispatch(dt, A1, ld1, sh.rows, sh.cols, factors, s);
    rc = ge2gb_dispatch(dt, sh.rows, sh.cols, A1, ld1, nb, band, ldab, work_dev, cv, sw, s);
    (void)hipEventRecord(ev[1], s);
    if (rc == SVB_OK) {
        // columns min(m, n) .. of the padded band are zero: stage 2 runs on the leading part
        rc = gb2bd_checked(bdt, k, nb, band, ldab, dd, de, w + cv.off_gb, gb2bd_bytes(k, nb), s);
        if (rc == SVB_OK && scaled) {
            if (bdt == SVB_F64) launch_rescale_bidiag<double>((double*)dd, (double*)de, k, factors, s);
            else launch_rescale_bidiag<float>((float*)dd, (float*)de, k, factors, s);
        }
    }
    (void)hipEventRecord(ev[2], s);
    const size_t cs = compute_size(dt);
    double total3 = 0.0;
    bool dev3 = false;
    if (rc == SVB_OK && !sw.stage3_host) {
        // stage 3 on the device, then one copy of k values
        void* sig = w + cv.off_sig;
        // The two reductions leave every singular value with an absolute error of the order of
        // eps * sigma_max, so the bidiagonal's small values are refined to tol times an eighth of
        // the bound on sigma_max (2^-3 eps sigma_max in f64, 2^-9 in f32), not to tol times
        // themselves, which costs them two to three times as many rounds.
        const double tol = dt == SVB_F64 ? 0x1p-52 : 0x1p-29;
        const double floor_frac = sw.stage3_relative ? 0.0 : 0.125;
        prof_begin(SVB_PROF_STAGE3, s, 0.0, 0.0);
        if (dt == SVB_F64)
            rc = run_bdsvals_dev<double>(k, (const double*)dd, (const double*)de, (double*)sig, w + cv.off_s3, tol,
                                         floor_frac, s);
        else
            rc = run_bdsvals_dev<float>(k, (const float*)dd, (const float*)de, (float*)sig, w + cv.off_s3, tol,
                                        floor_frac, s);
        prof_end(s);
        (void)hipEventRecord(ev[3], s);
        dev3 = true;
        if (rc == SVB_OK &&
            (hipMemcpyAsync(S_out_host, sig, (size_t)k * cs, hipMemcpyDeviceToHost, s) != hipSuccess ||
             hipStreamSynchronize(s) != hipSuccess))
            rc = SVB_ERR_DEVICE;
        if (rc == SVB_OK) {
            const bool bad = dt == SVB_F64 ? std::isnan(static_cast<double*>(S_out_host)[0])
                                           : std::isnan(static_cast<float*>(S_out_host)[0]);
            if (bad) rc = SVB_ERR_NONFINITE;
        }
    } else if (rc == SVB_OK) {
        std::vector<double> hd((size_t)k), he((size_t)k), hs((size_t)k);
        std::vector<unsigned char> raw(2 * (size_t)k * cs);
        if (hipMemcpyAsync(raw.data(), dd, (size_t)k * cs, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipMemcpyAsync(raw.data() + (size_t)k * cs, de, (size_t)k * cs, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess) {
            rc = SVB_ERR_DEVICE;
        } else if (dt == SVB_F64) {
            std::memcpy(hd.data(), raw.data(), (size_t)k * 8);
            std::memcpy(he.data(), raw.data() + (size_t)k * 8, (size_t)k * 8);
        } else {
            const float* fd = reinterpret_cast<const float*>(raw.data());
            for (int64_t i = 0; i < k; ++i) {
                hd[(size_t)i] = fd[i];
                he[(size_t)i] = fd[k + i];
            }
        }
        const auto t3a = std::chrono::steady_clock::now();
        if (rc == SVB_OK) rc = host_bdsvals(k, hd.data(), he.data(), hs.data());
        total3 = std::chrono::duration<double>(std::chrono::steady_clock::now() - t3a).count();
        if (rc == SVB_OK) {
            if (dt == SVB_F64) std::memcpy(S_out_host, hs.data(), (size_t)k * 8);
            else
                for (int64_t i = 0; i < k; ++i) static_cast<float*>(S_out_host)[i] = (float)hs[(size_t)i];
        }
    } else {
        (void)hipStreamSynchronize(s);
    }
    float ms1 = 0, ms2 = 0, ms3 = 0;
    (void)hipEventElapsedTime(&ms1, ev[0], ev[1]);
    (void)hipEventElapsedTime(&ms2, ev[1], ev[2]);
    if (dev3 && hipEventElapsedTime(&ms3, ev[2], ev[3]) == hipSuccess) total3 = ms3 * 1e-3;
    if (rc == SVB_OK && hipGetLastError() != hipSuccess) rc = SVB_ERR_DEVICE;
    g_last.s1 = ms1 * 1e-3;
    g_last.s2 = ms2 * 1e-3;
    g_last.s3 = total3;
    g_last.upd = -1.0;
    if (g_prof.on) {
        const double before = g_prof.sec[SVB_PROF_UPDATE] + g_prof.sec[SVB_PROF_UPDATE_UPPER];
        g_prof.collect();
        g_last.upd = g_prof.sec[SVB_PROF_UPDATE] + g_prof.sec[SVB_PROF_UPDATE_UPPER] - before;
    }
    return rc;
}

int svb_last_timings(double* t_panel, double* t_update, double* t_stage2, double* t_stage3)
{
    // stage 1's wall time, split into the part covered by update kernels and the rest (panel
    // factorisations that no update hides); the split needs the per-kernel events
    double upd = g_last.s1, pan = -1.0;
    if (g_last.upd >= 0.0) {
        upd = g_last.upd < g_last.s1 ? g_last.upd : g_last.s1;
        pan = g_last.s1 - upd;
    }
    if (t_panel) *t_panel = pan;
    if (t_update) *t_update = upd;
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
    case SVB_ERR_UNSUPPORTED: return "unsupported shape, tile size, alignment or dtype";
    case SVB_ERR_WORKSPACE: return "workspace too small";
    case SVB_ERR_DEVICE: return "HIP error";
    case SVB_ERR_NOCONV: return "bidiagonal solver did not converge";
    case SVB_ERR_NONFINITE: return "non-finite value in the input or the bidiagonal";
    default: return "unknown status";
    }
}

}  // extern "C"
