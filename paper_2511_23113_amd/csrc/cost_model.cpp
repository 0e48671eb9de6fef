// Linear compute-time model of one partition: t = a * blocks + c * items + t0, fitted by least
// squares on per-partition samples (host only).
//
// Paper: Methodology, "Sparsity-aware Strategy Selection": the compute term of the latency
// equation is proportional to the dense-block count plus a constant, with constants fitted
// from profiles.  The per-item term is this build's addition (a persistent workgroup pays a
// fixed cost for every work item it starts).
#include <cmath>
#include <cstdint>
#include <string>

#include "dbsp.h"
#include "plan.hpp"

extern "C" int dbsp_fit_cost_model(const int64_t* blocks, const int64_t* items, const double* time, int32_t n,
                                   double* a, double* c, double* t0, double* rms_residual) {
  if (!blocks || !items || !time || !a || !c || !t0) return dbsp_set_error(DBSP_EINVAL, "dbsp_fit_cost_model: null pointer");
  if (n < 3) return dbsp_set_error(DBSP_EINVAL, "dbsp_fit_cost_model: at least 3 samples are needed");
  // centred normal equations: the intercept drops out, leaving a 2x2 system for (a, c)
  long double mb = 0, mi = 0, mt = 0;
  for (int32_t k = 0; k < n; ++k) {
    if (!std::isfinite(time[k])) return dbsp_set_error(DBSP_EINVAL, "dbsp_fit_cost_model: non-finite time sample");
    mb += blocks[k];
    mi += items[k];
    mt += time[k];
  }
  mb /= n; mi /= n; mt /= n;
  long double sbb = 0, sii = 0, sbi = 0, sbt = 0, sit = 0;
  for (int32_t k = 0; k < n; ++k) {
    const long double db = blocks[k] - mb, di = items[k] - mi, dt = time[k] - mt;
    sbb += db * db; sii += di * di; sbi += db * di; sbt += db * dt; sit += di * dt;
  }
  const long double det = sbb * sii - sbi * sbi;
  if (!(sbb > 0) || !(sii > 0) || !(det > 1e-12L * sbb * sii))
    return dbsp_set_error(DBSP_EINVAL, "dbsp_fit_cost_model: the samples do not determine the three constants "
                                       "(blocks or items constant, or proportional to each other)");
  const long double fa = (sbt * sii - sit * sbi) / det;
  const long double fc = (sit * sbb - sbt * sbi) / det;
  const long double f0 = mt - fa * mb - fc * mi;
  *a = (double)fa; *c = (double)fc; *t0 = (double)f0;
  if (rms_residual) {
    long double ss = 0;
    for (int32_t k = 0; k < n; ++k) {
      const long double r = time[k] - (fa * blocks[k] + fc * items[k] + f0);
      ss += r * r;
    }
    *rms_residual = (double)std::sqrt((double)(ss / n));
  }
  return DBSP_OK;
}
