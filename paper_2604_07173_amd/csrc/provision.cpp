// Cache provisioning for the tail-TTFT target (Sec. 4.2, Eq. 1-4, Algorithm 1): the smallest
// number M of resident adapters for which the Immediate Admissibility Rate reaches alpha.
// Host code only (fp64); no device work.
//
// Model: adapter i is hit lambda_i = LB * p_i times per global batch on average; it is taken to
// be resident with probability q_i = Pr[Poisson(lambda_i) > tau*] (Eq. 2), where tau* makes the
// q_i sum to M (Eq. 3).  A request for adapter i is admitted at once if i is resident or, if not,
// when the other adapters hold at most M - 1 slots (Eq. 4); the number of slots the others hold
// is a sum of independent Bernoulli(q_j) variables.
//
// Eq. 2 writes the Poisson tail for integer tau; Eq. 3 needs a continuous tau, so the tail is
// taken as the regularized lower incomplete gamma function P(tau + 1, lambda), which agrees
// with Eq. 2 at the integers.
//
// Instead of one dynamic programme per adapter over the other N - 1 (N^3 per candidate M), the
// distribution of all N Bernoulli variables is built once per M and adapter i is divided out
// again, which is the same distribution by construction: with f = all N, g = all but i,
//   f[k] = g[k] (1 - q_i) + g[k-1] q_i.
// The division runs upwards from g[0] when q_i <= 1/2 and downwards from g[N-1] otherwise, so
// the recurrence always divides by the larger of (1 - q_i, q_i) and errors shrink as it goes.
#include <cmath>
#include <cstddef>
#include <limits>
#include <vector>

#include "../../include/lora_provision.h"

namespace {

// regularized lower incomplete gamma P(a, x), a > 0, x >= 0
double gamma_p(double a, double x)
{
    if (x <= 0.0) return 0.0;
    const double lg = std::lgamma(a);
    if (x < a + 1.0) {
        // series: P = e^-x x^a / Gamma(a) * sum_n x^n / (a (a+1) ... (a+n))
        double term = 1.0 / a, sum = term, ap = a;
        for (int n = 0; n < 100000; ++n) {
            ap += 1.0;
            term *= x / ap;
            sum += term;
            if (std::fabs(term) < std::fabs(sum) * 1e-17) break;
        }
        return sum * std::exp(-x + a * std::log(x) - lg);
    }
    // continued fraction for Q = 1 - P (modified Lentz)
    const double tiny = 1e-300;
    double b = x + 1.0 - a, c = 1.0 / tiny, d = 1.0 / b, h = d;
    for (int n = 1; n < 100000; ++n) {
        const double an = -n * (n - a);
        b += 2.0;
        d = an * d + b;
        if (std::fabs(d) < tiny) d = tiny;
        c = b + an / c;
        if (std::fabs(c) < tiny) c = tiny;
        d = 1.0 / d;
        const double delta = d * c;
        h *= delta;
        if (std::fabs(delta - 1.0) < 1e-16) break;
    }
    return 1.0 - std::exp(-x + a * std::log(x) - lg) * h;
}

// Q(lambda, tau) = Pr[Poisson(lambda) > tau], tau >= -1 real
double poisson_tail(double lambda, double tau)
{
    if (lambda <= 0.0) return 0.0;
    if (tau <= -1.0) return 1.0;
    return gamma_p(tau + 1.0, lambda);
}

double sum_tail(const std::vector<double> &lambda, double tau)
{
    double s = 0.0;
    for (double l : lambda) s += poisson_tail(l, tau);
    return s;
}

// tau* of Eq. 3 by bisection (the sum decreases in tau)
double solve_threshold(const std::vector<double> &lambda, int M)
{
    int n_pos = 0;
    for (double l : lambda) n_pos += l > 0.0 ? 1 : 0;
    if (M >= n_pos) return -1.0;
    double lo = -1.0, hi = 1.0;
    while (sum_tail(lambda, hi) > M) hi = 2.0 * hi + 1.0;
    for (int it = 0; it < 200; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (sum_tail(lambda, mid) > M) lo = mid;
        else hi = mid;
    }
    return 0.5 * (lo + hi);
}

int check_inputs(const double *p, int N, double LB)
{
    if (!p || N < 1) return LORA_PROVISION_ERR_INVALID_ARG;
    if (!(LB > 0.0) || !std::isfinite(LB)) return LORA_PROVISION_ERR_INVALID_ARG;
    double s = 0.0;
    for (int i = 0; i < N; ++i) {
        if (!(p[i] >= 0.0) || !std::isfinite(p[i])) return LORA_PROVISION_ERR_INVALID_ARG;
        s += p[i];
    }
    if (std::fabs(s - 1.0) > 1e-6) return LORA_PROVISION_ERR_NOT_A_DISTRIBUTION;
    return LORA_PROVISION_OK;
}

double iar_of(const double *p, int N, double LB, int M, double *tau_out, double *q_out)
{
    std::vector<double> lambda(N), q(N);
    for (int i = 0; i < N; ++i) lambda[i] = LB * p[i];
    const double tau = solve_threshold(lambda, M);
    for (int i = 0; i < N; ++i) q[i] = poisson_tail(lambda[i], tau);
    if (tau_out) *tau_out = tau;
    if (q_out)
        for (int i = 0; i < N; ++i) q_out[i] = q[i];

    // f[k] = Pr[exactly k of all N adapters resident]
    std::vector<double> f(N + 1, 0.0), g(N + 1, 0.0);
    f[0] = 1.0;
    for (int j = 0; j < N; ++j) {
        for (int k = j + 1; k >= 1; --k) f[k] = f[k] * (1.0 - q[j]) + f[k - 1] * q[j];
        f[0] *= 1.0 - q[j];
    }
    double total = 0.0;
    for (int i = 0; i < N; ++i) {
        if (p[i] == 0.0) continue;
        // g = the distribution without adapter i (N - 1 variables: g[0 .. N-1])
        const double qi = q[i];
        if (qi <= 0.5) {
            g[0] = f[0] / (1.0 - qi);
            for (int k = 1; k < N; ++k) g[k] = (f[k] - g[k - 1] * qi) / (1.0 - qi);
        } else {
            g[N - 1] = f[N] / qi;
            for (int k = N - 1; k >= 1; --k) g[k - 1] = (f[k] - g[k] * (1.0 - qi)) / qi;
        }
        double p_free = 0.0;
        for (int k = 0; k < M && k < N; ++k) p_free += g[k];
        if (p_free > 1.0) p_free = 1.0;
        if (p_free < 0.0) p_free = 0.0;
        total += p[i] * (qi + (1.0 - qi) * p_free);
    }
    return total;
}

}  // namespace

extern "C" {

int lora_provision_iar(const double *p, int N, double LB, int M, double *iar, double *tau,
                       double *q)
{
    const int rc = check_inputs(p, N, LB);
    if (rc != LORA_PROVISION_OK) return rc;
    if (M < 1 || M > N || !iar) return LORA_PROVISION_ERR_INVALID_ARG;
    *iar = iar_of(p, N, LB, M, tau, q);
    return LORA_PROVISION_OK;
}

int lora_provision_min_cache(const double *p, int N, double LB, double alpha, int *M_star,
                             double *iar_at_M)
{
    const int rc = check_inputs(p, N, LB);
    if (rc != LORA_PROVISION_OK) return rc;
    if (!(alpha > 0.0) || alpha > 1.0 || !M_star) return LORA_PROVISION_ERR_INVALID_ARG;
    double value = 0.0;
    for (int M = 1; M <= N; ++M) {
        value = iar_of(p, N, LB, M, nullptr, nullptr);
        if (value >= alpha) {
            *M_star = M;
            if (iar_at_M) *iar_at_M = value;
            return LORA_PROVISION_OK;
        }
    }
    *M_star = N;              // IAR(N) = 1 up to rounding; alpha <= 1
    if (iar_at_M) *iar_at_M = value;
    return LORA_PROVISION_OK;
}

int64_t lora_provision_memory_bytes(int M, int64_t adapter_bytes)
{
    if (M < 0 || adapter_bytes < 0) return -1;
    return (int64_t)M * adapter_bytes;
}

}  // extern "C"
