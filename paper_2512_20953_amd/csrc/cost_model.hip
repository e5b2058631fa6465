// Host-side cost-model arithmetic (include/ah_cost.h).  No device code.
#include "ah_cost.h"
#include "ah_stage.h"
#include "capi_util.h"

#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

using namespace ah;

extern "C" int ah_cost_layers_time(int n, const double* t_pow2, int n_pow2, double* out) {
  if (!t_pow2 || !out || n < 1 || n_pow2 < 1 || n_pow2 > 30) return set_error(AH_EINVAL, "ah_cost_layers_time: bad argument");
  if (n >> n_pow2) return set_error(AH_EINVAL, "ah_cost_layers_time: n = %d needs more than %d profiled powers of two", n, n_pow2);
  double t = 0.0;
  for (int i = 0; i < n_pow2; i++)
    if ((n >> i) & 1) t += t_pow2[i];
  *out = t;
  return AH_OK;
}

extern "C" int ah_cost_pipeline_time(const double* t, int P, int K, double* out) {
  if (!t || !out || P < 1 || K < 1) return set_error(AH_EINVAL, "ah_cost_pipeline_time: bad argument");
  double sum = 0.0, mx = 0.0;
  for (int i = 0; i < P; i++) {
    if (!(t[i] >= 0.0)) return set_error(AH_EINVAL, "ah_cost_pipeline_time: stage time %d is negative or NaN", i);
    sum += t[i];
    mx = std::max(mx, t[i]);
  }
  *out = sum + (K - 1) * mx;
  return AH_OK;
}

extern "C" int ah_cost_iteration_time(const double* t, const int* stages, int n_groups, int K, double t_sync, double* out) {
  if (!t || !stages || !out || n_groups < 1 || K < 1 || !(t_sync >= 0.0)) return set_error(AH_EINVAL, "ah_cost_iteration_time: bad argument");
  double worst = 0.0;
  const double* p = t;
  for (int j = 0; j < n_groups; j++) {
    double g;
    int rc = ah_cost_pipeline_time(p, stages[j], K, &g);
    if (rc) return rc;
    worst = std::max(worst, g);
    p += stages[j];
  }
  *out = worst + t_sync;
  return AH_OK;
}

extern "C" int ah_cost_idle_fractions(const double* t, int P, int K, double* idle, double* mean_idle) {
  if (!idle) return set_error(AH_EINVAL, "ah_cost_idle_fractions: idle is NULL");
  double total;
  int rc = ah_cost_pipeline_time(t, P, K, &total);
  if (rc) return rc;
  if (!(total > 0.0)) return set_error(AH_EINVAL, "ah_cost_idle_fractions: pipeline time is zero");
  double m = 0.0;
  for (int i = 0; i < P; i++) {
    idle[i] = 1.0 - K * t[i] / total;
    m += idle[i];
  }
  if (mean_idle) *mean_idle = m / P;
  return AH_OK;
}

extern "C" int ah_cost_partition_layers(int P, int n_layers, const double* t_layer, const double* mem_bytes, double fixed_per_layer,
                                        double act_per_layer, const int* in_flight, int* l_out, double* bottleneck) {
  if (!t_layer || !mem_bytes || !in_flight || !l_out || !bottleneck || P < 1 || n_layers < P || P > 4096 || n_layers > (1 << 20))
    return set_error(AH_EINVAL, "ah_cost_partition_layers: bad argument (need P >= 1 and n_layers >= P)");
  if (!(fixed_per_layer >= 0.0) || !(act_per_layer >= 0.0)) return set_error(AH_EINVAL, "ah_cost_partition_layers: negative byte counts");
  try {
  // largest layer count each stage can hold
  std::vector<long> cap(P);
  long cap_sum = 0;
  for (int i = 0; i < P; i++) {
    if (!(t_layer[i] > 0.0) || in_flight[i] < 1 || !(mem_bytes[i] >= 0.0)) return set_error(AH_EINVAL, "ah_cost_partition_layers: bad entry for stage %d", i);
    const double per = fixed_per_layer + act_per_layer * in_flight[i];
    long c = per > 0.0 ? (long)std::floor(mem_bytes[i] / per) : n_layers;
    c = std::min<long>(c, n_layers);
    if (c < 1) return set_error(AH_EUNSUPPORTED, "ah_cost_partition_layers: stage %d cannot hold one layer", i);
    cap[i] = c;
    cap_sum += c;
  }
  if (cap_sum < n_layers) return set_error(AH_EUNSUPPORTED, "ah_cost_partition_layers: the stages hold %ld layers in total, %d are needed", cap_sum, n_layers);
  // The optimum is one of the values l * t_layer[i].  For a candidate tau, stage i can take
  // min(cap_i, number of l with l * t_layer[i] <= tau) layers; tau is feasible when every stage can
  // take one and together they can take n_layers.  The counts use the same product as the candidates.
  auto fits = [&](int i, double tau) {  // largest l in [0, cap] with l * t <= tau
    const double q = std::floor(tau / t_layer[i]);
    long l = q >= (double)cap[i] ? cap[i] : q > 0.0 ? (long)q : 0;
    while (l < cap[i] && (double)(l + 1) * t_layer[i] <= tau) l++;  // the division may be off by one ulp either way
    while (l > 0 && (double)l * t_layer[i] > tau) l--;
    return l;
  };
  auto feasible = [&](double tau) {
    long total = 0;
    for (int i = 0; i < P; i++) {
      const long f = fits(i, tau);
      if (f < 1) return false;
      total += f;
    }
    return total >= n_layers;
  };
  // Feasibility grows with tau, so per stage the smallest feasible candidate l * t_layer[i] is found by bisection
  // over l (no list of all P * n_layers candidates is built); the optimum is the smallest of those.
  double tau = -1.0;
  for (int i = 0; i < P; i++) {
    if (!feasible((double)cap[i] * t_layer[i])) continue;  // none of this stage's candidates is feasible
    long lo = 1, hi = cap[i];
    while (lo < hi) {
      const long mid = (lo + hi) / 2;
      if (feasible((double)mid * t_layer[i])) hi = mid; else lo = mid + 1;
    }
    const double c = (double)lo * t_layer[i];
    if (tau < 0.0 || c < tau) tau = c;
  }
  if (tau < 0.0) return set_error(AH_EINVAL, "ah_cost_partition_layers: no feasible bottleneck (inconsistent stage times)");
  // every stage gets one layer; the rest goes to the earliest stages that still fit under tau
  long left = n_layers - P;
  for (int i = 0; i < P; i++) l_out[i] = 1;
  for (int i = 0; i < P && left > 0; i++) {
    const long extra = std::min(left, fits(i, tau) - 1);
    l_out[i] += (int)extra;
    left -= extra;
  }
  double worst = 0.0;
  for (int i = 0; i < P; i++) worst = std::max(worst, (double)l_out[i] * t_layer[i]);
  *bottleneck = worst;
  return AH_OK;
  } catch (const std::bad_alloc&) {
    return set_error(AH_ENOMEM, "ah_cost_partition_layers: out of host memory");
  } catch (...) {
    return set_error(AH_EINVAL, "ah_cost_partition_layers: unexpected failure");
  }
}
