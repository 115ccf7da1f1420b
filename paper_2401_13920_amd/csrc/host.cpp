// Host-only part of liblocmoe: status strings, descriptor validation, the scalar capacity
// formulas of Section 3.2.3 (Lemma 3, Theorem 1) and the workspace size.
#include <atomic>
#include <charconv>
#include <cmath>
#include <cstdlib>
#include <limits>

#include "common.h"

namespace locmoe {

int check_desc(const locmoe_desc* p) {
  if (!p) return LOCMOE_ERR_NULL;
  if (p->T < 1 || p->d < 1 || p->E < 1 || p->N < 1 || p->h < 1) return LOCMOE_ERR_SHAPE;
  if (p->E > 1024 || p->N > p->E) return LOCMOE_ERR_SHAPE;
  if (p->d % p->E != 0) return LOCMOE_ERR_SHAPE;  // Eq. 4 needs equal blocks of d/n features
  if (p->d % 8 != 0 || p->h % 8 != 0) return LOCMOE_ERR_SHAPE;
  if (p->C < 1) return LOCMOE_ERR_ARG;
  if (p->x_dtype != LOCMOE_F32 && p->x_dtype != LOCMOE_BF16) return LOCMOE_ERR_ARG;
  if (p->relu != 0 && p->relu != 1) return LOCMOE_ERR_ARG;
  if (p->w_packed != 0 && p->w_packed != 1) return LOCMOE_ERR_ARG;
  if ((int64_t)p->E * (int64_t)p->C > (int64_t)std::numeric_limits<int32_t>::max()) return LOCMOE_ERR_SHAPE;
  return LOCMOE_OK;
}

int cu_count() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

namespace {

// Continued fraction of the regularized incomplete beta function (DLMF 8.17.22), evaluated
// with the modified Lentz recurrence.  Converges quickly for x < (a+1)/(a+b+2).
double beta_cf(double a, double b, double x) {
  const double tiny = 1e-300;
  double c = 1.0, dd = 1.0 - (a + b) * x / (a + 1.0);
  if (std::fabs(dd) < tiny) dd = tiny;
  dd = 1.0 / dd;
  double f = dd;
  for (int m = 1; m <= 100000; ++m) {
    const double m2 = 2.0 * m;
    double num = m * (b - m) * x / ((a + m2 - 1.0) * (a + m2));  // even term
    dd = 1.0 + num * dd; if (std::fabs(dd) < tiny) dd = tiny; dd = 1.0 / dd;
    c = 1.0 + num / c;   if (std::fabs(c) < tiny) c = tiny;
    f *= dd * c;
    num = -(a + m) * (a + b + m) * x / ((a + m2) * (a + m2 + 1.0));  // odd term
    dd = 1.0 + num * dd; if (std::fabs(dd) < tiny) dd = tiny; dd = 1.0 / dd;
    c = 1.0 + num / c;   if (std::fabs(c) < tiny) c = tiny;
    const double step = dd * c;
    f *= step;
    if (std::fabs(step - 1.0) < 1e-16) break;
  }
  return f;
}

// I_x(a,b), 0 <= x <= 1.
double reg_inc_beta(double a, double b, double x) {
  if (x <= 0.0) return 0.0;
  if (x >= 1.0) return 1.0;
  const double lnpre = std::lgamma(a + b) - std::lgamma(a) - std::lgamma(b) + a * std::log(x) + b * std::log1p(-x);
  const double pre = std::exp(lnpre);
  if (x < (a + 1.0) / (a + b + 2.0)) return pre * beta_cf(a, b, x) / a;
  return 1.0 - pre * beta_cf(b, a, 1.0 - x) / b;
}

// Lemma 3 written as the upper tail I_{1-delta^2}((d-1)/2, 1/2), which keeps precision when
// the probability is tiny.
double p_delta(int d, double delta) { return reg_inc_beta(0.5 * (d - 1), 0.5, 1.0 - delta * delta); }

// ceil(cf * T / E) for the empirical capacity of Section 3.2.3, with the capacity factor read as the decimal
// number the caller wrote: the shortest decimal that rounds to the given double (1.1 means 11/10, not the double
// next to it), and the product and quotient formed exactly in integers, so that the plain ceiling of the paper's
// formula is taken of the plain value (cf = 1.1, T = 100, E = 10 gives 11; a product that is an integer gives that
// integer; anything above it, however little, gives the next one).  cf > 0 and finite; the result is clamped to
// [1, T] here already.
int ceil_cf_tokens_per_expert(double cf, int T, int E) {
  const double approx = cf * (double)T / (double)E;
  if (approx < 0.25) return 1;               // the exact value is below 1 as well
  if (approx > (double)T + 1.0) return T;    // ... above T as well
  char buf[64];
  const auto res = std::to_chars(buf, buf + sizeof buf - 1, cf, std::chars_format::scientific);
  *res.ptr = 0;
  // "d.ddde[+-]xx" -> digits D and a power of ten: cf = D * 10^p10
  unsigned __int128 D = 0;
  int frac_digits = 0;
  const char* q = buf;
  bool after_point = false;
  for (; *q && *q != 'e'; ++q) {
    if (*q == '.') { after_point = true; continue; }
    D = D * 10 + (unsigned)(*q - '0');
    if (after_point) ++frac_digits;
  }
  const int p10 = (*q == 'e' ? std::atoi(q + 1) : 0) - frac_digits;
  // 0.25 E/T <= cf <= (T+1) E/T bounds p10 to [-27, 13]: every product below fits in 128 bits
  unsigned __int128 num = D * (unsigned __int128)(unsigned)T, den = (unsigned __int128)(unsigned)E;
  for (int i = 0; i < p10; ++i) num *= 10;
  for (int i = 0; i < -p10; ++i) den *= 10;
  const unsigned __int128 c = (num + den - 1) / den;
  if (c < 1) return 1;
  return c > (unsigned __int128)(unsigned)T ? T : (int)c;
}

}  // namespace
}  // namespace locmoe

using namespace locmoe;

extern "C" {

const char* locmoe_status_string(int status) {
  switch (status) {
    case LOCMOE_OK: return "ok";
    case LOCMOE_ERR_NULL: return "null pointer";
    case LOCMOE_ERR_SHAPE: return "bad shape";
    case LOCMOE_ERR_ARG: return "bad argument";
    case LOCMOE_ERR_WORKSPACE: return "workspace missing or too small";
    case LOCMOE_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

int locmoe_p_delta(int32_t d, double delta, double* p) {
  if (!p) return LOCMOE_ERR_NULL;
  if (d < 2) return LOCMOE_ERR_SHAPE;
  if (!(delta >= 0.0 && delta <= 1.0)) return LOCMOE_ERR_ARG;
  *p = p_delta(d, delta);
  return LOCMOE_OK;
}

int locmoe_capacity_min(int32_t E, int32_t d, double delta, int32_t form, double* ec_min) {
  if (!ec_min) return LOCMOE_ERR_NULL;
  if (E < 1 || d < 2) return LOCMOE_ERR_SHAPE;
  if (!(delta > 0.0 && delta < 1.0) || form < 0 || form > 2) return LOCMOE_ERR_ARG;
  const double inf = std::numeric_limits<double>::infinity();
  const double y = delta * delta * d / (2.0 - delta * delta);
  double v;
  if (form == 0) {
    const double p = p_delta(d, delta);
    v = p > 0.0 ? 1.0 / (E * p) : inf;
  } else if (form == 1) {
    const double c = std::erfc(std::sqrt(y));
    v = c > 0.0 ? 1.0 / (E * c) : inf;
  } else {
    v = std::exp(y) / E;  // overflows to +inf by itself
  }
  *ec_min = v;
  return LOCMOE_OK;
}

int locmoe_capacity(int32_t T, int32_t E, int32_t d, double cf, double delta, int32_t* C) {
  if (!C) return LOCMOE_ERR_NULL;
  if (T < 1 || E < 1 || d < 2) return LOCMOE_ERR_SHAPE;
  if (!(cf >= 0.0) || std::isinf(cf)) return LOCMOE_ERR_ARG;
  double bound;
  const int st = locmoe_capacity_min(E, d, delta, 1, &bound);
  if (st != LOCMOE_OK) return st;
  double rows = bound >= (double)T ? (double)T : std::ceil(bound);
  if (cf > 0.0) rows = std::fmax(rows, (double)ceil_cf_tokens_per_expert(cf, T, E));
  rows = std::fmin(std::fmax(rows, 1.0), (double)T);
  *C = (int32_t)rows;
  return LOCMOE_OK;
}

size_t locmoe_workspace_bytes(const locmoe_desc* p) {
  if (check_desc(p) != LOCMOE_OK) return 0;
  // route: per block E counts + E probability sums + N home counts + 1 locality count
  const size_t route = (size_t)kRouteMaxBlocks * ((size_t)p->E * 8 + (size_t)p->N * 4 + 4);
  // dispatch: per block of tokens, E counts
  const size_t blocks = (size_t)ceil_div(p->T, kDispatchTokensPerBlock);
  const size_t disp = blocks * (size_t)p->E * 4;
  const size_t need = route > disp ? route : disp;
  return (need + 255) & ~(size_t)255;
}

}  // extern "C"
