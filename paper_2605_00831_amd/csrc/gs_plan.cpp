// Hybrid recovery planner: how many leading chunks to recompute while the rest
// are reconstructed from survivors and parity (Alg. 2, get_recompute_units).
#include "../../include/ghostserve_ec.h"

#include <algorithm>
#include <cmath>

namespace {

bool bad(double v) { return !(v >= 0.0) || std::isinf(v); }

// time to recompute the first r chunks: chunk i costs base + growth*i
double recompute_time(const gs_recovery_costs &c, long r)
{
    return c.recompute_base_s * static_cast<double>(r) +
           c.recompute_growth_s * (static_cast<double>(r) * static_cast<double>(r - 1) / 2.0);
}

// time to bring back q chunks through the gather / H2D / reconstruct pipeline:
// the slowest stage paces it, the other two are paid once to fill and drain
double restore_time(const gs_recovery_costs &c, long q)
{
    if (q <= 0) return 0.0;
    const double stage = std::max(c.gather_s, std::max(c.h2d_s, c.reconstruct_s));
    const double fill = c.gather_s + c.h2d_s + c.reconstruct_s - stage;
    return c.restore_startup_s + fill + stage * static_cast<double>(q);
}

double makespan(const gs_recovery_costs &c, long n, long r)
{
    return std::max(recompute_time(c, r), restore_time(c, n - r));
}

}  // namespace

extern "C" int gs_recompute_units(int n_chunks, const gs_recovery_costs *costs, int *r_out, double *makespan_out)
{
    if (n_chunks < 0 || costs == nullptr || r_out == nullptr) return GS_EINVAL;
    const gs_recovery_costs &c = *costs;
    if (bad(c.recompute_base_s) || bad(c.recompute_growth_s) || bad(c.gather_s) || bad(c.h2d_s) ||
        bad(c.reconstruct_s) || bad(c.restore_startup_s))
        return GS_EINVAL;
    const long n = n_chunks;
    // recompute_time rises with r and restore_time falls, so the makespan is
    // minimised where they cross: find the first r with recompute >= restore
    long lo = 0, hi = n;  // invariant: answer in [lo, hi]
    while (lo < hi) {
        const long mid = lo + (hi - lo) / 2;
        if (recompute_time(c, mid) >= restore_time(c, n - mid)) hi = mid;
        else lo = mid + 1;
    }
    // the minimum is at the crossing or one step before it; prefer the smaller r on a tie
    long best = lo;
    if (lo > 0 && makespan(c, n, lo - 1) <= makespan(c, n, lo)) best = lo - 1;
    // dropping the restore pipeline altogether (r = n) saves its start-up cost
    if (makespan(c, n, n) < makespan(c, n, best)) best = n;
    *r_out = static_cast<int>(best);
    if (makespan_out) *makespan_out = makespan(c, n, best);
    return GS_OK;
}
