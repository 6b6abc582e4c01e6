// Host-only integer rules of the library: rank quantization (Section 2.1), rank formulas
// (eq. 6 / eq. 7) and the sequential-freezing schedule (Algorithm 2).  No device code here.
#include <cmath>
#include <cstddef>
#include <vector>
#include <cstdint>

#include "lrd.h"

extern "C" {

const char* lrd_status_string(lrd_status s)
{
    switch (s) {
        case LRD_OK: return "LRD_OK";
        case LRD_ERR_INVALID_ARG: return "LRD_ERR_INVALID_ARG";
        case LRD_ERR_UNSUPPORTED: return "LRD_ERR_UNSUPPORTED";
        case LRD_ERR_ALIGNMENT: return "LRD_ERR_ALIGNMENT";
        case LRD_ERR_WORKSPACE: return "LRD_ERR_WORKSPACE";
        case LRD_ERR_RUNTIME: return "LRD_ERR_RUNTIME";
    }
    return "LRD_ERR_UNKNOWN";
}

int32_t lrd_quantize_rank(int32_t r, int32_t multiple, int32_t mode, int32_t r_min, int32_t r_max)
{
    if (r < 1 || multiple < 1 || r_min > r_max) return -(int32_t)LRD_ERR_INVALID_ARG;
    const int64_t m = multiple, rr = r;
    int64_t q;
    switch (mode) {
        case LRD_ROUND_NEAREST: q = ((2 * rr + m) / (2 * m)) * m; break;  // half a step up, truncate
        case LRD_ROUND_DOWN: q = rr - rr % m; break;
        case LRD_ROUND_UP: q = rr + (m - rr % m) % m; break;
        default: return -(int32_t)LRD_ERR_INVALID_ARG;
    }
    // Admissible set: multiples of m inside [max(r_min,1), r_max].
    const int64_t floor_bound = r_min > 1 ? r_min : 1;
    const int64_t lowest = floor_bound + (m - floor_bound % m) % m;
    const int64_t highest = (int64_t)r_max - (int64_t)r_max % m;
    if (lowest > highest) return r;  // nothing admissible: leave the rank alone
    if (q < lowest) q = lowest;
    if (q > highest) q = highest;
    return (int32_t)q;
}

uint32_t lrd_freeze_mask(int32_t kind, int64_t epoch)
{
    const uint32_t outer = kind == LRD_KIND_TUCKER ? (LRD_FREEZE_L0 | LRD_FREEZE_L2) : LRD_FREEZE_L0;
    const bool odd = (epoch & 1) != 0;
    return odd ? (uint32_t)LRD_FREEZE_L1 : outer;
}

lrd_status lrd_tucker_rank(int64_t C, int64_t S, int32_t k, double alpha, double beta,
                           int32_t* r1, int32_t* r2)
{
    if (!r1 || !r2 || C < 1 || S < 1 || k < 1 || !(alpha > 0.0) || !(beta > 0.0))
        return LRD_ERR_INVALID_ARG;
    // eq. 6 solves  beta k^2 x^2 + (C + beta S) x = C S k^2 / alpha  for x = r1.
    const double kk = double(k) * double(k);
    const double quad = beta * kk, lin = double(C) + beta * double(S);
    const double rhs = double(C) * double(S) * kk / alpha;
    const double half_p = lin / (2.0 * quad);
    double x = -half_p + std::sqrt(half_p * half_p + rhs / quad);
    int64_t n = (int64_t)std::floor(x);
    // floor of the exact root: correct a root that rounding pushed across an integer
    auto params = [&](int64_t v) { return quad * double(v) * double(v) + lin * double(v); };
    if (params(n + 1) <= rhs) ++n;
    else if (n >= 1 && params(n) > rhs) --n;
    int64_t n2 = (int64_t)std::floor(beta * double(n));
    n = n < 1 ? 1 : (n > C ? C : n);
    n2 = n2 < 1 ? 1 : (n2 > S ? S : n2);
    *r1 = (int32_t)n;
    *r2 = (int32_t)n2;
    return LRD_OK;
}

int32_t lrd_svd_rank(int64_t in, int64_t out, double alpha)
{
    if (in < 1 || out < 1 || !(alpha > 0.0)) return -(int32_t)LRD_ERR_INVALID_ARG;
    const double x = (double(in) * double(out)) / (alpha * (double(in) + double(out)));
    int64_t n = (int64_t)std::floor(x);
    const int64_t cap = in < out ? in : out;
    n = n < 1 ? 1 : (n > cap ? cap : n);
    return (int32_t)n;
}

lrd_status lrd_select_rank(const double* times, int32_t r_min, int32_t r_max, double t_dense, double noise,
                           int32_t mode, int32_t* r_opt, int32_t* keep_decomposed)
{
    if (!times || !r_opt || !keep_decomposed) return LRD_ERR_INVALID_ARG;
    if (r_min < 1 || r_max < r_min) return LRD_ERR_INVALID_ARG;
    const bool require_faster = (mode & LRD_SELECT_REQUIRE_FASTER) != 0;
    mode &= ~int32_t(LRD_SELECT_REQUIRE_FASTER);
    if (mode != LRD_SELECT_FIRST_PEAK && mode != LRD_SELECT_ARGMAX) return LRD_ERR_INVALID_ARG;
    if (!std::isfinite(t_dense) || !std::isfinite(noise) || noise < 0.0) return LRD_ERR_INVALID_ARG;
    const size_t count = size_t(r_max - r_min) + 1;
    for (size_t i = 0; i < count; ++i)
        if (!std::isfinite(times[i])) return LRD_ERR_INVALID_ARG;

    // slope[i] = t(r_min + i + 1) - t(r_min + i): the increase of step time entering rank r_min + i + 1
    std::vector<double> slope(count > 1 ? count - 1 : 0);
    for (size_t i = 0; i + 1 < count; ++i) slope[i] = times[i + 1] - times[i];

    ptrdiff_t pick = -1;   // index into slope of the chosen drop
    if (mode == LRD_SELECT_FIRST_PEAK) {
        for (ptrdiff_t i = (ptrdiff_t)slope.size() - 1; i >= 0; --i) {
            if (slope[i] <= noise) continue;
            const bool above_ok = size_t(i) + 1 >= slope.size() || slope[i] >= slope[i + 1];
            const bool below_ok = i == 0 || slope[i] >= slope[i - 1];
            if (above_ok && below_ok) { pick = i; break; }
        }
    } else {
        for (ptrdiff_t i = (ptrdiff_t)slope.size() - 1; i >= 0; --i)
            if (slope[i] > noise && (pick < 0 || slope[i] > slope[pick])) pick = i;
    }
    int32_t chosen = pick < 0 ? r_max : r_min + (int32_t)pick;   // the rank just below the drop
    // optional extension (not in the paper): a pick that is not faster than the estimated rank is dropped
    if (require_faster && times[chosen - r_min] >= times[count - 1]) chosen = r_max;
    *r_opt = chosen;
    *keep_decomposed = times[chosen - r_min] < t_dense ? 1 : 0;
    return LRD_OK;
}

}  // extern "C"
