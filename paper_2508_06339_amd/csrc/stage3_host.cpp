// Stage 3 on the host (paper Section 3, final stage: bidiagonal to singular
// values, which the paper leaves to a CPU library, LAPACK; this library
// carries its own solver).
//
// Bisection on the Golub-Kahan tridiagonal (order 2n, zero diagonal,
// off-diagonals |d1|,|e1|,|d2|,...; its positive eigenvalues are the singular
// values).  Lanes of a SIMD batch bisect LANES neighbouring singular values at
// once with the same recurrence and different shifts; batches are spread over
// std::threads.  No convergence failure modes.
#include <algorithm>
#include <atomic>
#include <cfloat>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <thread>
#include <vector>

#include "../../include/svb.h"

namespace svb {

namespace {

constexpr int LANES = 16;

// For each lane l: number of negative pivots of (T - x[l] I), T the tridiagonal
// with zero diagonal and squared off-diagonals z2[0..nz-1].
__attribute__((target_clones("avx512f", "avx2", "default")))
void negcount_batch(const double* __restrict__ z2, int64_t nz, const double* __restrict__ x,
                    int64_t* __restrict__ cnt)
{
    const double piv = DBL_MIN;
    double q[LANES];
    int64_t c[LANES];
    for (int l = 0; l < LANES; ++l) {
        double v = -x[l];
        v = std::fabs(v) < piv ? -piv : v;
        q[l] = v;
        c[l] = v < 0.0 ? 1 : 0;
    }
    for (int64_t j = 0; j < nz; ++j) {
        const double zz = z2[j];
        for (int l = 0; l < LANES; ++l) {
            double v = -x[l] - zz / q[l];
            v = std::fabs(v) < piv ? -piv : v;
            q[l] = v;
            c[l] += v < 0.0 ? 1 : 0;
        }
    }
    for (int l = 0; l < LANES; ++l) cnt[l] = c[l];
}

}  // namespace

int host_bdsvals(int64_t n, const double* d, const double* e, double* sigma)
{
    if (n < 0 || (n > 0 && (!d || !sigma)) || (n > 1 && !e)) return SVB_ERR_ARG;
    if (n == 0) return SVB_OK;
    const int64_t nz = 2 * n - 1;
    std::vector<double> z2((size_t)nz);
    double zmax = 0.0, bound = 0.0, prev = 0.0;
    for (int64_t j = 0; j < nz; ++j) {
        const double z = std::fabs((j & 1) ? e[j / 2] : d[j / 2]);
        if (!std::isfinite(z)) return SVB_ERR_NONFINITE;
        zmax = std::max(zmax, z);
        bound = std::max(bound, prev + z);
        prev = z;
        z2[(size_t)j] = z;
    }
    bound = std::max(bound, prev);
    if (zmax == 0.0) {
        std::fill(sigma, sigma + n, 0.0);
        return SVB_OK;
    }
    for (auto& z : z2) {
        const double s = z / zmax;
        z = s * s;
    }
    const double hi0 = bound / zmax * (1.0 + 8.0 * DBL_EPSILON) + DBL_MIN;
    const int64_t nbatch = (n + LANES - 1) / LANES;
    std::atomic<int64_t> next{0};
    auto worker = [&]() {
        for (;;) {
            const int64_t bidx = next.fetch_add(1);
            if (bidx >= nbatch) break;
            // lanes handle ascending indices k0 .. k0+LANES-1 (clamped)
            double lo[LANES], hi[LANES], mid[LANES];
            int64_t want[LANES], cnt[LANES];
            for (int l = 0; l < LANES; ++l) {
                const int64_t k = std::min(bidx * LANES + l, n - 1);
                want[l] = n + k + 1;  // eigenvalue number n+k (0-based) lies below x iff count >= n+k+1
                lo[l] = 0.0;
                hi[l] = hi0;
            }
            for (int it = 0; it < 256; ++it) {
                bool active = false;
                for (int l = 0; l < LANES; ++l) {
                    mid[l] = 0.5 * (lo[l] + hi[l]);
                    if (hi[l] - lo[l] > 2.0 * DBL_EPSILON * hi[l] + 1e-38 && mid[l] > lo[l] && mid[l] < hi[l])
                        active = true;
                }
                if (!active) break;
                negcount_batch(z2.data(), nz, mid, cnt);
                for (int l = 0; l < LANES; ++l) {
                    if (!(mid[l] > lo[l] && mid[l] < hi[l])) continue;
                    if (cnt[l] >= want[l]) hi[l] = mid[l];
                    else lo[l] = mid[l];
                }
            }
            for (int l = 0; l < LANES; ++l) {
                const int64_t k = bidx * LANES + l;
                if (k < n) sigma[n - 1 - k] = 0.5 * (lo[l] + hi[l]) * zmax;
            }
        }
    };
    unsigned nt = std::thread::hardware_concurrency();
    if (const char* env = std::getenv("SVB_HOST_THREADS")) nt = (unsigned)std::max(1, std::atoi(env));
    if (nt == 0) nt = 1;
    nt = (unsigned)std::min<int64_t>(nt, std::min<int64_t>(nbatch, 64));
    if (nt <= 1) {
        worker();
    } else {
        std::vector<std::thread> pool;
        pool.reserve(nt);
        for (unsigned i = 0; i < nt; ++i) pool.emplace_back(worker);
        for (auto& th : pool) th.join();
    }
    return SVB_OK;
}

}  // namespace svb
