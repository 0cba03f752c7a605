// Host side of the controller: latency predictor (App. C) and per-step planner (sections 3.3, 3.4).
#include "taper_admission.h"

#include <algorithm>
#include <cmath>
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
    std::vector<int> live;
    for (int r = 0; r < n_requests; ++r) {
        granted[r] = 0;
        if (branch_start[r + 1] > branch_start[r]) live.push_back(r);
    }
    double t_step = t0;
    int64_t evals = 0, admitted = 0;
    while (!live.empty()) {
        int best = -1;
        double best_score = 0, best_t = 0;
        int64_t best_L = 0;
        size_t kept = 0;
        for (size_t q = 0; q < live.size(); ++q) {
            const int r = live[q];
            const int64_t L_w = L + branch_context[branch_start[r] + granted[r]];
            const double t_w = eval(*T, (double)(n + 1), (double)L_w);
            ++evals;
            if (t_w > budget) continue;  // pruned for good
            live[kept++] = r;
            const double du = utility(r, granted[r] + 1) - utility(r, granted[r]);
            const double score = du / (1e-9 + std::max(0.0, t_w - t_step));
            if (best < 0 || score > best_score) {
                best = r;
                best_score = score;
                best_t = t_w;
                best_L = L_w;
            }
        }
        live.resize(kept);
        if (best < 0 || !(best_score > 0)) break;
        n += 1;
        L = best_L;
        t_step = best_t;
        ++granted[best];
        ++admitted;
        if (granted[best] >= branch_start[best + 1] - branch_start[best])
            live.erase(std::find(live.begin(), live.end(), best));
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
