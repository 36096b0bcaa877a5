// Host-only parts of libhs that need no GPU: the admission-control predicate of the
// spatial partitions (paper Section IV-A) and the latency determinism metrics
// (Section V-A, warm-up / cool-down rule of Section VI).
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <utility>
#include <vector>

#include "hs.h"
#include "hs_internal.h"

namespace hs {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int xcd_count(int device_cus) { return std::max(1, device_cus / 32); }

hs_status admission_check(const uint32_t* claimed, const uint32_t* req_a, const uint32_t* req_b,
                          int n_words, int device_cus) {
  if (!req_a || !req_b || n_words < 1 || n_words > HS_MAX_CU_WORDS || device_cus < 1 ||
      device_cus > 32 * HS_MAX_CU_WORDS) {
    set_error("admission: bad arguments (n_words=%d, device_cus=%d)", n_words, device_cus);
    return HS_E_INVAL;
  }
  bool any_a = false, any_b = false;
  for (int w = 0; w < n_words; ++w) {
    any_a |= req_a[w] != 0;
    any_b |= req_b[w] != 0;
    const uint32_t req = req_a[w] | req_b[w];
    // bits naming CUs the device does not have
    uint32_t legal = 0;
    const int lo = 32 * w;
    if (device_cus >= lo + 32) legal = 0xffffffffu;
    else if (device_cus > lo) legal = (1u << (device_cus - lo)) - 1u;
    if (req & ~legal) {
      set_error("admission denied: request names a CU >= %d", device_cus);
      return HS_E_OVERSUBSCRIBED;
    }
    if (claimed && (req & claimed[w])) {
      set_error("admission denied: requested CUs are claimed by another application");
      return HS_E_OVERSUBSCRIBED;
    }
  }
  if (!any_a || !any_b) {
    set_error("admission denied: empty CU mask");
    return HS_E_OVERSUBSCRIBED;
  }
  // The device deals workgroups to all of its XCDs (32 CUs each) and CU i sits on XCD
  // i mod n_xcd: a mask that leaves an XCD without a CU cannot be bound to a queue.
  const int n_xcd = xcd_count(device_cus);
  for (int which = 0; which < 2; ++which) {
    const uint32_t* m = which ? req_b : req_a;
    for (int x = 0; x < n_xcd; ++x) {
      bool any = false;
      for (int cu = x; cu < 32 * n_words && cu < device_cus; cu += n_xcd)
        any = any || ((m[cu / 32] >> (cu % 32)) & 1u);
      if (!any) {
        set_error("admission: %s mask has no CU on XCD %d (CU i is on XCD i mod %d); "
                  "use whole groups of %d consecutive CUs", which ? "overlay" : "inference", x,
                  n_xcd, n_xcd);
        return HS_E_INVAL;
      }
    }
  }
  return HS_OK;
}

static double percentile_sorted(const std::vector<double>& s, double p) {
  const double pos = (double)(s.size() - 1) * p / 100.0;
  const size_t lo = (size_t)std::floor(pos);
  const size_t hi = std::min(lo + 1, s.size() - 1);
  return s[lo] + (s[hi] - s[lo]) * (pos - (double)lo);
}

}  // namespace hs

extern "C" {

const char* hs_last_error(void) { return hs::g_err; }
const char* hs_version(void) { return "libhs 0.1 (gfx950)"; }

hs_status hs_admission_check(const uint32_t* claimed_by_others, const uint32_t* req_infer,
                             const uint32_t* req_overlay, int n_words, int device_cus) {
  return hs::admission_check(claimed_by_others, req_infer, req_overlay, n_words, device_cus);
}

hs_status hs_latency_metrics_compute(const double* lat, size_t n, int trim,
                                     hs_latency_metrics* out) {
  if (!lat || !out) {
    hs::set_error("latency metrics: NULL argument");
    return HS_E_INVAL;
  }
  size_t t = 0;
  if (trim) t = std::min<size_t>(10, n / 6);
  if (n <= 2 * t) {
    hs::set_error("latency metrics: no samples left");
    return HS_E_INVAL;
  }
  std::vector<double> s(lat + t, lat + (n - t));
  std::sort(s.begin(), s.end());
  double sum = 0.0;
  for (double v : s) sum += v;
  const double mean = sum / (double)s.size();
  double ss = 0.0;
  for (double v : s) ss += (v - mean) * (v - mean);
  out->n = s.size();
  out->mean = mean;
  out->max = s.back();
  out->std = std::sqrt(ss / (double)s.size());
  out->p50 = hs::percentile_sorted(s, 50.0);
  out->p99 = hs::percentile_sorted(s, 99.0);
  out->tail = s.back() - hs::percentile_sorted(s, 95.0);
  out->flatness = hs::percentile_sorted(s, 90.0) - hs::percentile_sorted(s, 10.0);
  return HS_OK;
}

hs_status hs_mann_whitney_u(const double* a, size_t na, const double* b, size_t nb, hs_mwu* out) {
  if (!a || !b || !out || na == 0 || nb == 0) {
    hs::set_error("mann-whitney: NULL or empty sample");
    return HS_E_INVAL;
  }
  // pooled mid-ranks: sort (value, sample) pairs, give every run of equal values its mean rank
  std::vector<std::pair<double, int>> v;
  v.reserve(na + nb);
  for (size_t i = 0; i < na; ++i) v.emplace_back(a[i], 0);
  for (size_t i = 0; i < nb; ++i) v.emplace_back(b[i], 1);
  std::sort(v.begin(), v.end(),
            [](const std::pair<double, int>& x, const std::pair<double, int>& y) { return x.first < y.first; });
  const double N = (double)(na + nb);
  double rank_sum_a = 0.0, ties = 0.0;
  for (size_t i = 0; i < v.size();) {
    size_t j = i;
    while (j < v.size() && v[j].first == v[i].first) ++j;
    const double t = (double)(j - i);
    const double mid = 0.5 * ((double)(i + 1) + (double)j);     // ranks i+1 .. j
    for (size_t k = i; k < j; ++k)
      if (v[k].second == 0) rank_sum_a += mid;
    ties += t * t * t - t;
    i = j;
  }
  const double n = (double)na, m = (double)nb;
  const double u = rank_sum_a - n * (n + 1.0) / 2.0;
  const double mu = n * m / 2.0;
  const double var = N > 1.0 ? n * m / 12.0 * ((N + 1.0) - ties / (N * (N - 1.0))) : 0.0;
  const double d = u - mu;
  double z = 0.0;
  if (var > 0.0 && d != 0.0) z = (d - (d > 0.0 ? 0.5 : -0.5)) / std::sqrt(var);
  out->u = u;
  out->z = z;
  out->significant = std::fabs(z) > 1.96 ? 1 : 0;
  return HS_OK;
}

}  // extern "C"
