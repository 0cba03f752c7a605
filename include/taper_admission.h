/*
 * taper_admission -- the controller side that the decode-step attention serves:
 * the latency predictor T(S) of the paper's App. C and the per-step admission of
 * §3.3 (slack budget) and §3.4 (greedy planner).  Host-only, plain C, float64;
 * every pointer is host memory owned by the caller and only read or written
 * during the call.  Functions return 0 or a negative taper_status (taper_attn.h);
 * taper_last_error() gives the message.
 */
#ifndef TAPER_ADMISSION_H
#define TAPER_ADMISSION_H

#include <stdint.h>

#include "taper_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * T(S) = a + b * n_tokens + c * L_context, milliseconds (App. C "Predictor
 * formulation"): n_tokens = sequences in the step (one new token each),
 * L_context = their aggregate context length.  The second regressor may be any
 * other per-step aggregate (e.g. unique KV tokens when prefixes are shared); the
 * arithmetic is the same.
 */
typedef struct {
    double a, b, c;
} taper_predictor;

/*
 * Ordinary least squares over n observed steps (App. C "Fitting").  Solved by
 * Householder QR of the column-scaled n x 3 design matrix.  TAPER_EINVAL when
 * n < 3, a value is not finite, or the observations do not determine all three
 * coefficients (e.g. every step has the same batch size).
 * mape_pct (may be NULL) receives the fit's mean absolute percentage error over
 * the same observations (App. C "Accuracy"); observations with t_ms == 0 are
 * rejected.
 */
TAPER_API int taper_predictor_fit(int64_t n, const double *n_tokens, const double *l_context, const double *t_ms,
                                  taper_predictor *out, double *mape_pct);

/*
 * The same fit under b >= 0 and c >= 0 (App. C "Monotonicity": the predictor is monotone in admitted
 * branches because b and c are positive; the planner's pruning rule relies on it and taper_admit_step
 * refuses a predictor that is not).  Noisy or small observation sets -- a rolling window of steps that
 * are all launch-bound, say -- can give ordinary least squares a negative slope; this form returns the
 * least-squares solution over the region b, c >= 0 instead (equal to the ordinary one whenever that is
 * inside it; otherwise one or both coefficients are exactly 0 and the rest is refitted), so a refresh
 * never hands the planner a model it cannot use.  Same errors as taper_predictor_fit.
 */
TAPER_API int taper_predictor_fit_monotone(int64_t n, const double *n_tokens, const double *l_context,
                                           const double *t_ms, taper_predictor *out, double *mape_pct);

TAPER_API double taper_predictor_eval(const taper_predictor *p, double n_tokens, double l_context);

/* Mean absolute percentage error of p over n observations (App. C "Accuracy"). */
TAPER_API int taper_predictor_mape(const taper_predictor *p, int64_t n, const double *n_tokens, const double *l_context,
                                   const double *t_ms, double *mape_pct);

/*
 * Rolling refresh (App. C "Fitting": the most recent 200 observed step
 * latencies).  A window keeps the last `capacity` observations; fit() runs the
 * OLS above over what it holds.
 */
typedef struct taper_window taper_window;
TAPER_API int taper_window_create(int32_t capacity, taper_window **out);
TAPER_API void taper_window_destroy(taper_window *w);
TAPER_API int taper_window_push(taper_window *w, double n_tokens, double l_context, double t_ms);
TAPER_API int32_t taper_window_size(const taper_window *w);
TAPER_API int taper_window_fit(const taper_window *w, taper_predictor *out, double *mape_pct);
/* The refresh a planner should use: taper_predictor_fit_monotone over the window. */
TAPER_API int taper_window_fit_monotone(const taper_window *w, taper_predictor *out, double *mape_pct);

/* Utility curve u_r(k) of §3.3: what k opportunistic branches are worth to request r. */
typedef enum {
    TAPER_UTILITY_LINEAR = 0,  /* u(k) = weight * k                 (throughput-oriented)   */
    TAPER_UTILITY_CONCAVE = 1, /* u(k) = weight * log2(1 + k)       (fairness-oriented)     */
    TAPER_UTILITY_TABLE = 2    /* u(k) = utility_table[...][k], caller-supplied              */
} taper_utility_kind;

typedef struct {
    double rho;           /* fraction of the residual slack to spend, in (0, 1]  (§3.3)     */
    int32_t utility_kind; /* taper_utility_kind                                             */
    int32_t reserved;
} taper_admission_options;

typedef struct {
    double t0_ms;        /* T(S_0): predicted latency of the protected composition          */
    double budget_ms;    /* T0 + rho * max(0, min_r slack_r - T0)                            */
    double t_pred_ms;    /* predicted latency of the composition returned                    */
    int64_t n_tokens;    /* of the composition returned                                      */
    int64_t l_context;
    int64_t evaluations; /* calls of T made while widening                                   */
    int64_t admitted;    /* sum of granted[]                                                 */
} taper_admission_result;

/*
 * One planner invocation (§3.4; budget of §3.3).  Starts from the protected
 * composition S_0 -- one token per request: n_requests tokens and the sum of
 * base_context[] -- and repeatedly admits the ready branch with the largest
 * marginal utility per marginal predicted latency,
 *     (u_r(k+1) - u_r(k)) / (1e-9 + max(0, T(widened) - T(step))),
 * among the requests whose widened step still satisfies T <= budget.  A request
 * whose next branch does not fit is not looked at again (T is monotone).
 * Requests are scanned in index order; on equal score the lower index wins.
 * Stops when no request is left or the best score is <= 0.
 *
 *   base_context[r]   context length of request r's protected continuation
 *   slack_ms[r]       d_r(t) - t: time left until r's next-token deadline; the
 *                     budget uses the minimum over ALL requests
 *   branch_start[r]   CSR (n_requests + 1 entries) into branch_context[]
 *   branch_context[]  context length of each ready branch, per request in the
 *                     order they would be admitted
 *   weight[r]         utility weight (may be NULL = 1); ignored for TABLE
 *   utility_table[]   for TABLE: per request u_r(0..ready_r), laid out with the
 *                     CSR table_start[r] = branch_start[r] + r (ready_r + 1
 *                     entries each); NULL otherwise
 *   granted[r]        out: opportunistic branches admitted for request r
 *
 * TAPER_EINVAL on null pointers, rho outside (0, 1], negative lengths, a
 * non-monotone CSR, non-finite slack, or b < 0 or c < 0 in the predictor (the
 * pruning rule needs T monotone in admitted branches).
 */
TAPER_API int taper_admit_step(const taper_predictor *T, int32_t n_requests, const int64_t *base_context,
                               const double *slack_ms, const int32_t *branch_start, const int64_t *branch_context,
                               const double *weight, const double *utility_table,
                               const taper_admission_options *opts, int32_t *granted, taper_admission_result *result);

#ifdef __cplusplus
}
#endif
#endif /* TAPER_ADMISSION_H */
