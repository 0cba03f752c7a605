// Host side of the controller: latency predictor (App. C) and per-step planner (sections 3.3, 3.4).
#include "taper_admission.h"

#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstdint>
#include <new>
#include <string>
#include <vector>

namespace taper {
int set_error(int code, const std::string& msg);  // taper_api.cpp
}
using taper::set_error;

namespace {

// Least squares of an n x 3 system by Householder reflections; columns are scaled to
// unit max-abs first (L_context is ~1e6 times n_tokens), which keeps the rank test meaningful.
int ols3(int64_t n, const double* x1, const double* x2, const double* y, double beta[3]) {
    if (n < 3) return set_error(TAPER_EINVAL, "need at least 3 observations");
    double s1 = 0, s2 = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (!std::isfinite(x1[i]) || !std::isfinite(x2[i]) || !std::isfinite(y[i]))
            return set_error(TAPER_EINVAL, "observation is not finite");
        s1 = std::max(s1, std::fabs(x1[i]));
        s2 = std::max(s2, std::fabs(x2[i]));
    }
    if (s1 == 0 || s2 == 0) return set_error(TAPER_EINVAL, "observations do not determine the coefficients");
    std::vector<double> A((size_t)n * 3), b(y, y + n);
    for (int64_t i = 0; i < n; ++i) {
        A[3 * i] = 1.0;
        A[3 * i + 1] = x1[i] / s1;
        A[3 * i + 2] = x2[i] / s2;
    }
    double R[3][3] = {};
    for (int k = 0; k < 3; ++k) {
        double norm = 0;
        for (int64_t i = k; i < n; ++i) norm += A[3 * i + k] * A[3 * i + k];
        norm = std::sqrt(norm);
        if (norm < 1e-12 * std::sqrt((double)n)) return set_error(TAPER_EINVAL, "observations do not determine the coefficients");
        const double alpha = A[3 * k + k] > 0 ? -norm : norm;
        // v = x - alpha e_k, stored in place
        A[3 * k + k] -= alpha;
        double vnorm2 = 0;
        for (int64_t i = k; i < n; ++i) vnorm2 += A[3 * i + k] * A[3 * i + k];
        R[k][k] = alpha;
        for (int j = k + 1; j < 3; ++j) {
            double dot = 0;
            for (int64_t i = k; i < n; ++i) dot += A[3 * i + k] * A[3 * i + j];
            const double f = 2.0 * dot / vnorm2;
            for (int64_t i = k; i < n; ++i) A[3 * i + j] -= f * A[3 * i + k];
            R[k][j] = A[3 * k + j];
        }
        double dot = 0;
        for (int64_t i = k; i < n; ++i) dot += A[3 * i + k] * b[i];
        const double f = 2.0 * dot / vnorm2;
        for (int64_t i = k; i < n; ++i) b[i] -= f * A[3 * i + k];
    }
    // rank test relative to the largest pivot
    const double big = std::max({std::fabs(R[0][0]), std::fabs(R[1][1]), std::fabs(R[2][2])});
    for (int k = 0; k < 3; ++k)
        if (std::fabs(R[k][k]) < 1e-10 * big) return set_error(TAPER_EINVAL, "observations do not determine the coefficients");
    double z[3];
    for (int k = 2; k >= 0; --k) {
        double v = b[k];
        for (int j = k + 1; j < 3; ++j) v -= R[k][j] * z[j];
        z[k] = v / R[k][k];
    }
    beta[0] = z[0];
    beta[1] = z[1] / s1;
    beta[2] = z[2] / s2;
    return TAPER_OK;
}

double eval(const taper_predictor& p, double n, double L) { return p.a + p.b * n + p.c * L; }

int mape(const taper_predictor& p, int64_t n, const double* x1, const double* x2, const double* y, double* out) {
    if (n < 1) return set_error(TAPER_EINVAL, "no observations");
    double acc = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (y[i] == 0 || !std::isfinite(y[i])) return set_error(TAPER_EINVAL, "observed latency is zero or not finite");
        acc += std::fabs(eval(p, x1[i], x2[i]) - y[i]) / std::fabs(y[i]);
    }
    *out = acc / (double)n * 100.0;
    return TAPER_OK;
}

}  // namespace

struct taper_window {
    int32_t capacity = 0, size = 0, head = 0;  // head = slot of the next push
    std::vector<double> n, L, t;
};

extern "C" {

int taper_predictor_fit(int64_t n, const double* n_tokens, const double* l_context, const double* t_ms,
                        taper_predictor* out, double* mape_pct) {
    if (!n_tokens || !l_context || !t_ms || !out) return set_error(TAPER_EINVAL, "null argument");
    double beta[3];
    if (int rc = ols3(n, n_tokens, l_context, t_ms, beta)) return rc;
    out->a = beta[0];
    out->b = beta[1];
    out->c = beta[2];
    if (mape_pct) return mape(*out, n, n_tokens, l_context, t_ms, mape_pct);
    return TAPER_OK;
}

int taper_predictor_fit_monotone(int64_t n, const double* n_tokens, const double* l_context, const double* t_ms,
                                 taper_predictor* out, double* mape_pct) {
    if (!n_tokens || !l_context || !t_ms || !out) return set_error(TAPER_EINVAL, "null argument");
    double beta[3];
    if (int rc = ols3(n, n_tokens, l_context, t_ms, beta)) return rc;
    if (beta[1] < 0 || beta[2] < 0) {
        // Two sign constraints: the minimiser has one or both of them active.  Each active set is a smaller
        // least-squares problem in closed form; the best feasible one is the constrained minimiser (the
        // objective is convex, so a feasible stationary point on a face is the minimum over that face).
        double sn = 0, sL = 0, st = 0, snn = 0, sLL = 0, snt = 0, sLt = 0;
        const double N = (double)n;
        for (int64_t i = 0; i < n; ++i) {
            sn += n_tokens[i];
            sL += l_context[i];
            st += t_ms[i];
        }
        const double mn = sn / N, mL = sL / N, mt = st / N;
        for (int64_t i = 0; i < n; ++i) {  // centred sums: well conditioned for regressors of any magnitude
            const double dn = n_tokens[i] - mn, dL = l_context[i] - mL, dt = t_ms[i] - mt;
            snn += dn * dn;
            sLL += dL * dL;
            snt += dn * dt;
            sLt += dL * dt;
        }
        auto rss = [&](double a_, double b_, double c_) {
            double acc = 0;
            for (int64_t i = 0; i < n; ++i) {
                const double e = a_ + b_ * n_tokens[i] + c_ * l_context[i] - t_ms[i];
                acc += e * e;
            }
            return acc;
        };
        double best[3] = {mt, 0.0, 0.0};  // both active: the mean
        double best_rss = rss(best[0], 0.0, 0.0);
        if (snn > 0) {  // c = 0: line in n_tokens
            const double b_ = snt / snn;
            if (b_ >= 0) {
                const double a_ = mt - b_ * mn, v = rss(a_, b_, 0.0);
                if (v < best_rss) best[0] = a_, best[1] = b_, best[2] = 0.0, best_rss = v;
            }
        }
        if (sLL > 0) {  // b = 0: line in L_context
            const double c_ = sLt / sLL;
            if (c_ >= 0) {
                const double a_ = mt - c_ * mL, v = rss(a_, 0.0, c_);
                if (v < best_rss) best[0] = a_, best[1] = 0.0, best[2] = c_, best_rss = v;
            }
        }
        beta[0] = best[0], beta[1] = best[1], beta[2] = best[2];
    }
    out->a = beta[0];
    out->b = beta[1];
    out->c = beta[2];
    if (mape_pct) return mape(*out, n, n_tokens, l_context, t_ms, mape_pct);
    return TAPER_OK;
}

double taper_predictor_eval(const taper_predictor* p, double n_tokens, double l_context) {
    return p ? eval(*p, n_tokens, l_context) : NAN;
}

int taper_predictor_mape(const taper_predictor* p, int64_t n, const double* n_tokens, const double* l_context,
                         const double* t_ms, double* mape_pct) {
    if (!p || !n_tokens || !l_context || !t_ms || !mape_pct) return set_error(TAPER_EINVAL, "null argument");
    return mape(*p, n, n_tokens, l_context, t_ms, mape_pct);
}

int taper_window_create(int32_t capacity, taper_window** out) {
    if (!out || capacity < 3) return set_error(TAPER_EINVAL, "window capacity must be at least 3");
    taper_window* w = new (std::nothrow) taper_window;
    if (!w) return set_error(TAPER_ENOMEM, "window allocation failed");
    w->capacity = capacity;
    w->n.resize(capacity);
    w->L.resize(capacity);
    w->t.resize(capacity);
    *out = w;
    return TAPER_OK;
}

void taper_window_destroy(taper_window* w) { delete w; }

int taper_window_push(taper_window* w, double n_tokens, double l_context, double t_ms) {
    if (!w) return set_error(TAPER_EINVAL, "null window");
    w->n[w->head] = n_tokens;
    w->L[w->head] = l_context;
    w->t[w->head] = t_ms;
    w->head = (w->head + 1) % w->capacity;
    w->size = std::min(w->size + 1, w->capacity);
    return TAPER_OK;
}

int32_t taper_window_size(const taper_window* w) { return w ? w->size : 0; }

int taper_window_fit(const taper_window* w, taper_predictor* out, double* mape_pct) {
    if (!w || !out) return set_error(TAPER_EINVAL, "null argument");
    return taper_predictor_fit(w->size, w->n.data(), w->L.data(), w->t.data(), out, mape_pct);
}

int taper_window_fit_monotone(const taper_window* w, taper_predictor* out, double* mape_pct) {
    if (!w || !out) return set_error(TAPER_EINVAL, "null argument");
    return taper_predictor_fit_monotone(w->size, w->n.data(), w->L.data(), w->t.data(), out, mape_pct);
}

int taper_admit_step(const taper_predictor* T, int32_t n_requests, const int64_t* base_context, const double* slack_ms,
                     const int32_t* branch_start, const int64_t* branch_context, const double* weight,
                     const double* utility_table, const taper_admission_options* opts, int32_t* granted,
                     taper_admission_result* result) {
    if (!T || !base_context || !slack_ms || !branch_start || !opts || !granted || !result)
        return set_error(TAPER_EINVAL, "null argument");
    if (n_requests < 1) return set_error(TAPER_EINVAL, "no requests");
    if (!(opts->rho > 0.0 && opts->rho <= 1.0)) return set_error(TAPER_EINVAL, "rho must be in (0, 1]");
    if (!(T->b >= 0.0 && T->c >= 0.0) || !std::isfinite(T->a)) return set_error(TAPER_EINVAL, "predictor must be monotone (b, c >= 0)");
    const int kind = opts->utility_kind;
    if (kind < TAPER_UTILITY_LINEAR || kind > TAPER_UTILITY_TABLE) return set_error(TAPER_EINVAL, "unknown utility kind");
    if (kind == TAPER_UTILITY_TABLE && !utility_table) return set_error(TAPER_EINVAL, "utility table missing");
    if (branch_start[0] != 0) return set_error(TAPER_EINVAL, "branch_start[0] must be 0");
    int64_t n = n_requests, L = 0;
    double min_slack = INFINITY;
    for (int r = 0; r < n_requests; ++r) {
        if (base_context[r] < 0) return set_error(TAPER_ELEN, "negative context length");
        if (branch_start[r + 1] < branch_start[r]) return set_error(TAPER_EINVAL, "branch_start must not decrease");
        if (std::isnan(slack_ms[r])) return set_error(TAPER_EINVAL, "slack is not a number");
        L += base_context[r];
        min_slack = std::min(min_slack, slack_ms[r]);
    }
    if (branch_start[n_requests] > 0 && !branch_context) return set_error(TAPER_EINVAL, "branch_context missing");
    for (int i = 0; i < branch_start[n_requests]; ++i)
        if (branch_context[i] < 0) return set_error(TAPER_ELEN, "negative context length");

    auto utility = [&](int r, int k) -> double {
        if (kind == TAPER_UTILITY_TABLE) return utility_table[(int64_t)branch_start[r] + r + k];
        const double w = weight ? weight[r] : 1.0;
        return kind == TAPER_UTILITY_LINEAR ? w * (double)k : w * std::log2(1.0 + (double)k);
    };

    const double t0 = eval(*T, (double)n, (double)L);
    const double budget = t0 + opts->rho * std::max(0.0, min_slack - t0);
    // The candidates: one record per request that still has a ready branch and has not been pruned, holding
    // what the next round needs of it -- the context its next branch would add and what that branch is worth.
    // Only the record of the request that was just widened changes between rounds.
    struct Candidate {
        int32_t request;
        int64_t next_context;
        double gain;  // u(k + 1) - u(k) at the request's current k
    };
    std::vector<Candidate> cand;
    cand.reserve(n_requests);
    for (int r = 0; r < n_requests; ++r) {
        granted[r] = 0;
        if (branch_start[r + 1] > branch_start[r])
            cand.push_back({r, branch_context[branch_start[r]], utility(r, 1) - utility(r, 0)});
    }
    double t_step = t0;
    int64_t evals = 0, admitted = 0;
    while (!cand.empty()) {
        // one sweep: price every candidate's widened step, let those over the budget go for good (T only grows),
        // remember the best ratio among the rest (the earliest request on a tie)
        size_t kept = 0, best = SIZE_MAX;
        double best_score = 0, best_t = 0;
        for (size_t q = 0; q < cand.size(); ++q) {
            const double t_w = eval(*T, (double)(n + 1), (double)(L + cand[q].next_context));
            ++evals;
            if (t_w > budget) continue;
            const double score = cand[q].gain / (1e-9 + std::max(0.0, t_w - t_step));
            if (best == SIZE_MAX || score > best_score) {
                best = kept;
                best_score = score;
                best_t = t_w;
            }
            cand[kept++] = cand[q];
        }
        cand.resize(kept);
        if (best == SIZE_MAX || !(best_score > 0)) break;
        Candidate& c = cand[best];
        const int r = c.request;
        n += 1;
        L += c.next_context;
        t_step = best_t;
        ++admitted;
        const int k = ++granted[r];
        if (k >= branch_start[r + 1] - branch_start[r]) {
            cand.erase(cand.begin() + (ptrdiff_t)best);  // (keeps the index order the tie rule needs)
        } else {
            c.next_context = branch_context[branch_start[r] + k];
            c.gain = utility(r, k + 1) - utility(r, k);
        }
    }
    result->t0_ms = t0;
    result->budget_ms = budget;
    result->t_pred_ms = t_step;
    result->n_tokens = n;
    result->l_context = L;
    result->evaluations = evals;
    result->admitted = admitted;
    return TAPER_OK;
}

}  // extern "C"
