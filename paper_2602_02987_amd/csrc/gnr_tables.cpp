// Host-side sampler tables of the simulator: length quantile tables, Poisson arrival-count
// thresholds, class-mix thresholds. Integer tables only reach the device, so the device never
// evaluates a transcendental and every random decision is an integer comparison.
//
// Definitions (they fix the encoding, so any implementation of them yields the same integers):
//  * length table: entry j = min{k in [1,32768] : F(k) >= (j+0.5)/65536}, with
//      geometric  F(k) = -expm1(k*log1p(-1/mean))      (Pr(X>=k) = (1-p)^(k-1), paper EC, geometric check)
//      lognormal  F(k) = erfc(-z/sqrt2)/2, z = (log(k+0.5)-log(median))/sigma  (rounded to nearest, clamped)
//  * patience table (abandonment): the geometric length table with mean 1/(1 - e^(-theta*dt)), the mean computed
//      as 1.0 / -expm1(-theta*dt): Pr(patience >= m steps) = e^(-theta*dt*(m-1))
//  * arrival thresholds for a per-server, per-step mean m = Lambda*dt*(1+amp*sin(2*pi*row/period)):
//      t0 = q(e^-m), t1 = q(e^-m + m e^-m), t2 = q((e^-m + m e^-m) + m^2 e^-m/2), q(p) = floor(p*2^32)
//      clamped to [0, 2^32-1]; the count is the number of thresholds the random word reaches.
//  * class thresholds: q(sum_{i<=k} lambda_i / Lambda), partial sums in class order.
#include "gnr_internal.h"

#include <cmath>

namespace gnr {

static uint32_t quantise32(double p)
{
  double v = std::floor(p * 4294967296.0);
  if (v < 0.0) return 0u;
  if (v > 4294967295.0) return 0xFFFFFFFFu;
  return static_cast<uint32_t>(v);
}

namespace {
struct Geometric {
  double log_q;  // log(1 - p)
  bool degenerate;
  explicit Geometric(double mean) : log_q(0.0), degenerate(false)
  {
    const double p = 1.0 / mean;
    if (p >= 1.0) degenerate = true; else log_q = std::log1p(-p);
  }
  double cdf(int k) const { return degenerate ? 1.0 : -std::expm1(static_cast<double>(k) * log_q); }
};
struct LogNormal {
  double mu, sigma;
  LogNormal(double median, double s) : mu(std::log(median)), sigma(s) {}
  double cdf(int k) const
  {
    const double z = (std::log(static_cast<double>(k) + 0.5) - mu) / sigma;
    return 0.5 * std::erfc(-z * M_SQRT1_2);
  }
};
template <class Law> void fill_quantiles(const Law &law, uint16_t *out)
{
  int k = 1;
  for (int j = 0; j < kTableSize; ++j) {
    const double u = (static_cast<double>(j) + 0.5) / 65536.0;
    while (k < kMaxLen && law.cdf(k) < u) ++k;
    out[j] = static_cast<uint16_t>(k);
  }
}
}  // namespace

int build_length_table(int law, double p0, double p1, const uint16_t *user, uint16_t *out)
{
  switch (law) {
    case SIM_CONST: {
      long long v = std::llround(p0);
      v = v < 1 ? 1 : (v > kMaxLen ? kMaxLen : v);
      for (int j = 0; j < kTableSize; ++j) out[j] = static_cast<uint16_t>(v);
      return SIM_OK;
    }
    case SIM_GEOMETRIC:
      if (!(p0 > 0.0)) return SIM_EINVAL;
      fill_quantiles(Geometric(p0), out);
      return SIM_OK;
    case SIM_LOGNORMAL:
      if (!(p0 > 0.0) || !(p1 > 0.0)) return SIM_EINVAL;
      fill_quantiles(LogNormal(p0, p1), out);
      return SIM_OK;
    case SIM_TABLE:
      if (!user) return SIM_EINVAL;
      for (int j = 0; j < kTableSize; ++j) {
        if (user[j] < 1 || user[j] > kMaxLen) return SIM_EINVAL;
        out[j] = user[j];
      }
      return SIM_OK;
    default:
      return SIM_EINVAL;
  }
}

uint32_t probability_threshold(double p) { return quantise32(p); }

// A class selection weight as an integer: the nearest multiple of 2^-20, but never zero, so that a class whose
// weight is zero is still served when no other class waits (each pool stays work-conserving).
uint32_t selection_weight_units(double w)
{
  const double v = std::floor(w * 1048576.0 + 0.5);
  return v < 1.0 ? 1u : (v > 1048576.0 ? 1048576u : static_cast<uint32_t>(v));
}

int build_patience_table(double theta, double dt_seconds, uint16_t *out)
{
  if (!(theta > 0.0) || !(dt_seconds > 0.0) || !std::isfinite(theta)) return SIM_EINVAL;
  return build_length_table(SIM_GEOMETRIC, 1.0 / -std::expm1(-theta * dt_seconds), 0.0, nullptr, out);
}

double total_rate(const sim_class *cls, int K)
{
  double lam = 0.0;
  for (int k = 0; k < K; ++k) lam += cls[k].lambda;
  return lam;
}

void build_arrival_row(double lam, int64_t dt_ns, double amp, int64_t period, int64_t row, uint32_t thr[3])
{
  const double dts = static_cast<double>(dt_ns) * 1e-9;
  double mod = 1.0;
  if (period > 0) {
    const double ph = 2.0 * M_PI * static_cast<double>(row) / static_cast<double>(period);
    mod = 1.0 + amp * std::sin(ph);
  }
  double m = lam * dts * mod;
  if (m < 0.0) m = 0.0;
  const double p0 = std::exp(-m);
  const double p1 = p0 * m;
  const double p2 = p1 * m * 0.5;
  thr[0] = quantise32(p0);
  thr[1] = quantise32(p0 + p1);
  thr[2] = quantise32((p0 + p1) + p2);
}

void build_class_thresholds(const sim_class *cls, int K, uint32_t *thr)
{
  const double lam = total_rate(cls, K);
  double acc = 0.0;
  for (int k = 0; k < kMaxK; ++k) thr[k] = 0xFFFFFFFFu;
  for (int k = 0; k + 1 < K; ++k) {
    acc += cls[k].lambda;
    thr[k] = lam > 0.0 ? quantise32(acc / lam) : 0xFFFFFFFFu;
  }
}

}  // namespace gnr
