// Host side of the sampling plan: how many mask rows, which coalition sizes, and
// the regression weight of each size class.
//
// Follows the paper's sample-distribution equation (rho_s = (n-1)/(s(n-s)),
// k_s proportional to rho_s) and its complementary pairing. A pair class s
// (1 <= s <= floor(n/2)) holds the sizes (s, n-s); its mass is 2*rho_s, or rho_s
// when 2s == n. The K sampled pairs are split by cumulative rounding so that the
// classes sum to K exactly and pairs are laid out by ascending size. A row of
// size s weighs rho_s / (number of emitted rows of size s), so each represented
// size carries its whole kernel mass; under enumeration this is the Shapley
// kernel weight itself. (Option: every sampled row weighs 1 instead, the
// importance-sampling form, since the allocation already follows rho_s.)
//
// Every operation that decides an integer is a single IEEE double + * / or floor
// (no fused multiply-add: build with -ffp-contract=off), so the boundaries are
// reproducible bit for bit.
#include <cmath>

#include "internal.h"

static double rho_mass(int64_t n, int64_t s) {
  return (double)(n - 1) / ((double)s * (double)(n - s));
}

extern "C" int ds_sample_plan(int64_t n, int64_t n_samples, int64_t* k_out, int32_t* enumerated_out) {
  if (n < 0 || n_samples < 0) return DS_EINVAL;
  int enumerate = (n <= DS_ENUM_MAX_PLAYERS && n_samples >= ((int64_t)1 << n)) ? 1 : 0;
  int64_t k = enumerate ? ((int64_t)1 << n) : 2 * (n_samples / 2);
  if (k_out) *k_out = k;
  if (enumerated_out) *enumerated_out = enumerate;
  return DS_OK;
}

int ds_make_plan(ds_ctx* ctx, int64_t n, int64_t n_samples, ds_plan* plan, int weighting, int saturate) {
  if (n < 2) return ds_fail(ctx, DS_EINVAL, "sampling needs at least 2 players (n=%lld)", (long long)n);
  if (n > 0x7fffffffLL) return ds_fail(ctx, DS_EINVAL, "too many players (n=%lld)", (long long)n);
  int32_t enumerate;
  int64_t k;
  ds_sample_plan(n, n_samples, &k, &enumerate);
  if (!enumerate && n_samples < 4)
    return ds_fail(ctx, DS_EINVAL, "n_samples must be at least 4 (got %lld)", (long long)n_samples);
  plan->n = n;
  plan->k = k;
  plan->K = k / 2 - 1;
  plan->H = n / 2;
  plan->enumerate = enumerate;
  const int64_t H = plan->H, K = plan->K;
  plan->wtab.assign(H + 1, 0.0f);
  plan->b.assign(H + 1, 0);
  plan->enum_upto = 0;
  if (saturate && weighting != DS_WEIGHT_CLASS_MASS)
    return ds_fail(ctx, DS_EINVAL, "saturated size classes need the class-mass weighting");
  if (enumerate) {
    double binom = 1.0;  // C(n, s), exact in double for n <= 24
    for (int64_t s = 1; s <= H; ++s) {
      binom = binom * (double)(n - s + 1) / (double)s;
      plan->wtab[s] = (float)(rho_mass(n, s) / binom);
    }
    return DS_OK;
  }
  // Option `saturate`: a class that is allotted at least as many pairs as it has coalitions (q_s >= C(n, s)) is
  // enumerated (every s-subset once) and the pairs this frees go to the classes that are left, by the same
  // cumulative rounding; the test moves on to the next class (C(n, s) grows and the allotment shrinks with s, so
  // the enumerated classes are 1..enum_upto). The class 2s == n is never enumerated this way.
  std::vector<double> c(H + 1, 0.0);
  int64_t enum_upto = 0, used = 0, cap_prev = 1;  // cap_prev = C(n, enum_upto)
  for (;;) {
    double acc = 0.0;
    for (int64_t s = enum_upto + 1; s <= H; ++s) {
      double r = rho_mass(n, s);
      acc = acc + ((2 * s == n) ? r : 2.0 * r);
      c[s] = acc;
    }
    const double T = acc;
    for (int64_t s = enum_upto + 1; s < H; ++s)
      plan->b[s] = used + (int64_t)std::floor((double)(K - used) * (c[s] / T) + 0.5);
    plan->b[H] = K;
    const int64_t s1 = enum_upto + 1;
    if (!saturate || s1 > H || 2 * s1 >= n) break;
    const __int128 cap = (__int128)cap_prev * (__int128)(n - s1 + 1) / (__int128)s1;  // C(n, s1), exact
    if (cap > (__int128)(plan->b[s1] - used)) break;
    enum_upto = s1;
    used += (int64_t)cap;
    cap_prev = (int64_t)cap;
    plan->b[s1] = used;
  }
  plan->enum_upto = enum_upto;
  for (int64_t s = 1; s <= H; ++s) {
    int64_t m = (plan->b[s] - plan->b[s - 1]) * ((2 * s == n) ? 2 : 1);
    if (m > 0) plan->wtab[s] = weighting == DS_WEIGHT_UNIFORM ? 1.0f : (float)(rho_mass(n, s) / (double)m);
  }
  return DS_OK;
}

extern "C" int ds_plan_tables(int64_t n, int64_t n_samples, int64_t* b, float* wtab) {
  return ds_plan_tables_ex(n, n_samples, nullptr, b, wtab, nullptr);
}

extern "C" int ds_plan_tables_ex(int64_t n, int64_t n_samples, const ds_options* opts, int64_t* b, float* wtab,
                                 int64_t* enum_upto) {
  if (n < 2 || n > 0x7fffffffLL || n_samples < 0) return DS_EINVAL;
  ds_plan plan;
  int rc = ds_make_plan(nullptr, n, n_samples, &plan, opts ? opts->weighting : DS_WEIGHT_CLASS_MASS, opts ? opts->saturate : 0);
  if (enum_upto) *enum_upto = plan.enum_upto;
  if (rc != DS_OK) return rc;
  for (int64_t s = 0; s <= plan.H; ++s) {
    if (b) b[s] = plan.b[s];
    if (wtab) wtab[s] = plan.wtab[s];
  }
  return DS_OK;
}
