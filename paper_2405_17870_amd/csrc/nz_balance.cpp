// Host-side Load Balancer arithmetic: how a message should be shared among
// rails whose startup latency and bandwidth are known.
//
// Nezha (arXiv 2405.17870) Sec. 4.3: cold start sends everything over the best
// single rail (Eq. 4); hot start splits the message with shares alpha that sum
// to one and finishes when the slowest rail does (Eq. 5); the two states meet
// at the threshold size (Eq. 6); the shares are refined by descent on the hot
// latency (Eq. 7) from latency-derived starting shares (Eq. 8).
//
// Two routes to the shares are offered.  nz_balance_iterate is the paper's
// method: Eq. 8 starting shares, then steps of Eq. 7 until the data-length
// table no longer changes.  nz_balance writes down the point that descent
// converges to directly: the slowest-rail latency is minimal when every rail
// that takes part finishes at the same time T and every rail whose startup
// latency alone exceeds T sits out ("water filling" over the startup
// latencies); no iteration.
//
// Sec. 2.1.2 Eq. 2 (network efficiency) and Sec. 2.2.1 Eq. 3 (the real-time
// efficiency ratio that gates splitting) are evaluated at the end of the file.
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

#include "nz_internal.h"

namespace {

bool valid_model(const nz_rail_model *rails, uint32_t n_rails)
{
    if (rails == nullptr || n_rails == 0 || n_rails > NZ_MAX_RAILS) return false;
    for (uint32_t i = 0; i < n_rails; ++i) {
        if (!(rails[i].setup_s >= 0.0) || !std::isfinite(rails[i].setup_s)) return false;
        if (!(rails[i].bytes_per_s > 0.0) || !std::isfinite(rails[i].bytes_per_s)) return false;
    }
    return true;
}

// Rails in order of startup latency (index breaks ties).
std::vector<uint32_t> by_setup(const nz_rail_model *rails, uint32_t n_rails)
{
    std::vector<uint32_t> order(n_rails);
    std::iota(order.begin(), order.end(), 0u);
    std::stable_sort(order.begin(), order.end(),
                     [&](uint32_t x, uint32_t y) { return rails[x].setup_s < rails[y].setup_s; });
    return order;
}

// Integer weights that sum to exactly NZ_RATIO_SCALE: floors, then the leftover
// units to the largest remainders (lowest index among equals).
void shares_to_ratios(const double *share, uint32_t n_rails, uint32_t *ratios)
{
    const uint32_t total = NZ_RATIO_SCALE;
    double frac[NZ_MAX_RAILS];
    uint32_t given = 0;
    for (uint32_t i = 0; i < n_rails; ++i) {
        const double x = share[i] * total;
        double fl = std::floor(x);
        if (fl > total) fl = total;
        ratios[i] = (uint32_t)fl;
        frac[i] = x - fl;
        given += ratios[i];
    }
    while (given < total) {
        uint32_t pick = 0;
        for (uint32_t i = 1; i < n_rails; ++i)
            if (frac[i] > frac[pick]) pick = i;
        ratios[pick] += 1;
        frac[pick] = -1.0;
        ++given;
        bool any = false;
        for (uint32_t i = 0; i < n_rails; ++i) any = any || frac[i] >= 0.0;
        if (!any)
            for (uint32_t i = 0; i < n_rails; ++i) frac[i] = 0.0;
    }
    while (given > total) {  // only through floating-point excess in the shares
        uint32_t pick = 0;
        for (uint32_t i = 1; i < n_rails; ++i)
            if (ratios[i] > ratios[pick]) pick = i;
        ratios[pick] -= 1;
        --given;
    }
}

}  // namespace

extern "C" {

nz_status nz_balance(const nz_rail_model *rails, uint32_t n_rails, double msg_bytes, double *alpha,
                     uint32_t *ratios, double *t_cold, double *t_hot, uint32_t *best_rail, int *hot)
{
    if (n_rails > NZ_MAX_RAILS) return NZ_ERR_UNSUPPORTED;
    if (!valid_model(rails, n_rails) || !(msg_bytes >= 0.0) || !std::isfinite(msg_bytes))
        return NZ_ERR_INVALID_ARG;

    // Eq. 4.
    uint32_t best = 0;
    double cold = 0.0;
    for (uint32_t i = 0; i < n_rails; ++i) {
        const double t = rails[i].setup_s + msg_bytes / rails[i].bytes_per_s;
        if (i == 0 || t < cold) {
            cold = t;
            best = i;
        }
    }

    // Eq. 5 at its minimum: find the common finishing time T of the rails that
    // take part.  With the m lowest-latency rails taking part,
    //   sum_i (T - setup_i) * B_i = S   =>   T = (S + sum setup_i B_i) / sum B_i,
    // and rail m + 1 joins as long as its startup latency is below that T.
    const std::vector<uint32_t> order = by_setup(rails, n_rails);
    double sum_b = 0.0, sum_sb = 0.0, level = 0.0;
    uint32_t active = 0;
    for (uint32_t m = 0; m < n_rails; ++m) {
        const nz_rail_model &r = rails[order[m]];
        if (m > 0 && r.setup_s >= level) break;
        sum_b += r.bytes_per_s;
        sum_sb += r.setup_s * r.bytes_per_s;
        level = (msg_bytes + sum_sb) / sum_b;
        active = m + 1;
    }
    const bool is_hot = active > 1 && level < cold;

    std::vector<double> share(n_rails, 0.0);
    if (is_hot) {
        for (uint32_t m = 0; m < active; ++m) {
            const nz_rail_model &r = rails[order[m]];
            share[order[m]] = (level - r.setup_s) * r.bytes_per_s / msg_bytes;
        }
    } else {
        share[best] = 1.0;  // cold start: everything on the best single rail
    }

    if (alpha) std::copy(share.begin(), share.end(), alpha);
    if (ratios) shares_to_ratios(share.data(), n_rails, ratios);
    if (t_cold) *t_cold = cold;
    if (t_hot) *t_hot = is_hot ? level : cold;
    if (best_rail) *best_rail = best;
    if (hot) *hot = is_hot ? 1 : 0;
    return NZ_OK;
}

nz_status nz_balance_iterate(const nz_rail_model *rails, uint32_t n_rails, double msg_bytes,
                             uint32_t max_iterations, double *alpha, uint32_t *ratios, double *t_hot,
                             uint32_t *iterations)
{
    if (n_rails > NZ_MAX_RAILS) return NZ_ERR_UNSUPPORTED;
    if (!valid_model(rails, n_rails) || !(msg_bytes > 0.0) || !std::isfinite(msg_bytes))
        return NZ_ERR_INVALID_ARG;
    const uint32_t R = n_rails;
    const double S = msg_bytes;
    double a[NZ_MAX_RAILS], t[NZ_MAX_RAILS];

    // Eq. 8: each rail's latency T_i under a uniform split, T their sum; a
    // rail that is slow under the uniform split starts with a smaller share.
    if (R == 1) {
        a[0] = 1.0;
    } else {
        double total = 0.0;
        for (uint32_t i = 0; i < R; ++i) {
            t[i] = rails[i].setup_s + (S / R) / rails[i].bytes_per_s;
            total += t[i];
        }
        for (uint32_t i = 0; i < R; ++i) a[i] = (total - t[i]) / (total * (double)(R - 1));
    }

    // Eq. 7.  T_hot is the maximum over the rails that take part, so its
    // derivative is S / B on the slowest of them and zero elsewhere: a step
    // takes a share from the slowest rail.  The share goes to the rail that
    // would finish first (of all ways to keep the sum at one, the one that
    // raises T_hot least), and its size is the exact line search along that
    // direction: the two rails finish together.  A rail whose startup latency
    // alone reaches that common time hands over all it has and sits out.
    const double table_unit = 1.0 / (2.0 * NZ_RATIO_SCALE);  // half a unit of the data-length table
    uint32_t k = 0;
    for (; k < max_iterations && R > 1; ++k) {
        uint32_t w = R, f = R;
        for (uint32_t i = 0; i < R; ++i) {
            t[i] = rails[i].setup_s + a[i] * S / rails[i].bytes_per_s;
            if (a[i] > 0.0 && (w == R || t[i] > t[w])) w = i;
        }
        for (uint32_t i = 0; i < R; ++i)
            if (i != w && (f == R || t[i] < t[f])) f = i;
        if (!(t[f] < t[w])) break;  // nobody could take anything off the slowest rail
        const double bw = rails[w].bytes_per_s, bf = rails[f].bytes_per_s;
        const double meet = (bw * t[w] + bf * t[f]) / (bw + bf);
        if (rails[w].setup_s >= meet) {
            a[f] += a[w];
            a[w] = 0.0;
            continue;
        }
        const double delta = (t[w] - meet) * bw / S;
        if (delta < table_unit) break;  // the data-length table has converged
        a[w] -= delta;
        a[f] += delta;
    }

    double slowest = 0.0;
    for (uint32_t i = 0; i < R; ++i)
        if (a[i] > 0.0) slowest = std::max(slowest, rails[i].setup_s + a[i] * S / rails[i].bytes_per_s);
    if (alpha) std::copy(a, a + R, alpha);
    if (ratios) shares_to_ratios(a, R, ratios);
    if (t_hot) *t_hot = slowest;
    if (iterations) *iterations = k;
    return NZ_OK;
}

nz_status nz_balance_threshold(const nz_rail_model *rails, uint32_t n_rails, double *threshold_bytes)
{
    if (n_rails > NZ_MAX_RAILS) return NZ_ERR_UNSUPPORTED;
    if (!valid_model(rails, n_rails) || threshold_bytes == nullptr) return NZ_ERR_INVALID_ARG;
    if (n_rails == 1) {
        *threshold_bytes = std::numeric_limits<double>::infinity();
        return NZ_OK;
    }
    // Eq. 6: the two states give the same latency up to the size at which the
    // second rail starts to pay off: while the lowest-latency rail alone
    // finishes before the next rail could even start, (setup_2 - setup_1) * B_1.
    const std::vector<uint32_t> order = by_setup(rails, n_rails);
    const nz_rail_model &first = rails[order[0]], &second = rails[order[1]];
    *threshold_bytes = (second.setup_s - first.setup_s) * first.bytes_per_s;
    return NZ_OK;
}

nz_status nz_net_efficiency(const nz_rail_model *rail, double msg_bytes, double *delta)
{
    if (!valid_model(rail, 1) || delta == nullptr) return NZ_ERR_INVALID_ARG;
    if (!(msg_bytes > 0.0) || !std::isfinite(msg_bytes)) return NZ_ERR_INVALID_ARG;
    // Eq. 2, with numerator and denominator multiplied by S / B.
    const double wire = msg_bytes / rail->bytes_per_s;
    *delta = wire / (wire + rail->setup_s);
    return NZ_OK;
}

nz_status nz_efficiency_ratio(const nz_rail_model *rails, uint32_t n_rails, double msg_bytes,
                              const double *alpha, double *rho)
{
    if (n_rails > NZ_MAX_RAILS) return NZ_ERR_UNSUPPORTED;
    if (!valid_model(rails, n_rails) || rho == nullptr) return NZ_ERR_INVALID_ARG;
    if (!(msg_bytes > 0.0) || !std::isfinite(msg_bytes)) return NZ_ERR_INVALID_ARG;
    double total = 0.0;
    for (uint32_t i = 0; i < n_rails && alpha != nullptr; ++i) {
        if (!(alpha[i] >= 0.0) || !std::isfinite(alpha[i])) return NZ_ERR_INVALID_ARG;
        total += alpha[i];
    }
    if (alpha != nullptr && !(total > 0.0)) return NZ_ERR_INVALID_ARG;
    // S_i * delta_i / That_i of Eq. 3 is the rail's throughput on its own
    // volume: S_i / (T_setup_i + S_i / B_i).
    double fastest = 0.0, slowest = 0.0;
    bool any = false;
    for (uint32_t i = 0; i < n_rails; ++i) {
        const double volume = msg_bytes * (alpha ? alpha[i] / total : 1.0 / n_rails);
        if (!(volume > 0.0)) continue;
        const double rate = volume / (rails[i].setup_s + volume / rails[i].bytes_per_s);
        fastest = any ? std::max(fastest, rate) : rate;
        slowest = any ? std::min(slowest, rate) : rate;
        any = true;
    }
    *rho = fastest / slowest;
    return NZ_OK;
}

}  // extern "C"
