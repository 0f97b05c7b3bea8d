// Freeze decision on the stream of plasticity scores (Section 4.2 "How to
// Decide Layer Freezing", Eq. 2 and Algorithm 1 of the paper).  Host code
// only; the state lives in a caller-owned struct.
#include <cmath>
#include <limits>
#include "../../include/egeria.h"

namespace {

const double kNaN = std::numeric_limits<double>::quiet_NaN();

void reset_module(egeria_freeze_state *st)
{
    st->stale = 0;
    st->n_raw = 0;
    st->n_smooth = 0;
    st->n_first_slopes = 0;
    st->max_first_slope = 0.0;
    st->has_T = st->T_user > 0.0 ? 1 : 0;
    st->T = st->T_user > 0.0 ? st->T_user : kNaN;
}

// Mean of the last min(W, n) values of a ring that has seen n values (Eq. 2).
double window_mean(const double *ring, int64_t n, int W)
{
    const int m = (int)(n < W ? n : W);
    double sum = 0.0;
    for (int k = m; k >= 1; --k) sum += ring[(n - k) % EGERIA_FREEZE_MAX_W];   // oldest first
    return sum / (double)m;
}

// Least-squares slope of the last m = min(max(W, 2), n) ring values against 0 .. m-1.
double window_slope(const double *ring, int64_t n, int W)
{
    const int w2 = W < 2 ? 2 : W;
    const int m = (int)(n < w2 ? n : w2);
    const double xbar = 0.5 * (double)(m - 1);
    double ybar = 0.0;
    for (int k = 0; k < m; ++k) ybar += ring[(n - m + k) % EGERIA_FREEZE_MAX_W];
    ybar /= (double)m;
    double sxy = 0.0, sxx = 0.0;
    for (int k = 0; k < m; ++k) {
        const double dx = (double)k - xbar;
        sxy += dx * (ring[(n - m + k) % EGERIA_FREEZE_MAX_W] - ybar);
        sxx += dx * dx;
    }
    return sxy / sxx;
}

}  // namespace

extern "C" {

egeria_status egeria_freeze_init(egeria_freeze_state *st, int32_t n_modules, int32_t W, double T, int32_t lr_annealing)
{
    if (!st || n_modules < 1 || W < 1 || W > EGERIA_FREEZE_MAX_W || T != T) return EGERIA_ERR_INVALID_ARG;
    st->n_modules = n_modules;
    st->front = 0;
    st->W = W;
    st->lr_annealing = lr_annealing ? 1 : 0;
    st->has_lr_ref = 0;
    st->lr_ref = 0.0;
    st->T_user = T > 0.0 ? T : 0.0;
    for (int i = 0; i < EGERIA_FREEZE_MAX_W; ++i) st->raw[i] = st->smooth[i] = 0.0;
    reset_module(st);
    return EGERIA_OK;
}

egeria_status egeria_freeze_observe(egeria_freeze_state *st, double p, double lr, egeria_freeze_decision *out)
{
    if (!st || !out) return EGERIA_ERR_INVALID_ARG;
    if (st->n_modules < 1 || st->W < 1 || st->W > EGERIA_FREEZE_MAX_W || st->front < 0 || st->front >= st->n_modules)
        return EGERIA_ERR_INVALID_ARG;
    int action = EGERIA_FREEZE_NONE;
    double smoothed = kNaN, slope = kNaN;
    if (st->front < st->n_modules - 1) {
        if (st->stale < st->W) {
            st->raw[st->n_raw % EGERIA_FREEZE_MAX_W] = p;
            st->n_raw += 1;
            smoothed = window_mean(st->raw, st->n_raw, st->W);
            st->smooth[st->n_smooth % EGERIA_FREEZE_MAX_W] = smoothed;
            st->n_smooth += 1;
            if (st->n_smooth < 2) {
                st->stale = 0;
            } else {
                slope = window_slope(st->smooth, st->n_smooth, st->W);
                if (!st->has_T) {
                    const double a = std::fabs(slope);
                    if (st->n_first_slopes == 0 || a > st->max_first_slope) st->max_first_slope = a;
                    st->n_first_slopes += 1;
                    if (st->n_first_slopes == 3) {
                        st->T = 0.2 * st->max_first_slope;
                        st->has_T = 1;
                    }
                }
                if (st->has_T && std::fabs(slope) < st->T) st->stale += 1;
                else st->stale = 0;
            }
        } else {
            if (st->front == 0) {
                st->lr_ref = lr;
                st->has_lr_ref = 1;
            }
            st->front += 1;
            reset_module(st);
            action = EGERIA_FREEZE_FREEZE;
        }
    }
    if (st->lr_annealing && st->front > 0 && st->has_lr_ref && lr <= 0.1 * st->lr_ref * (1.0 + 1e-12)) {
        st->front = 0;
        st->W = st->W / 2 > 1 ? st->W / 2 : 1;
        st->has_lr_ref = 0;
        reset_module(st);
        action = EGERIA_FREEZE_UNFREEZE_ALL;
    }
    out->action = action;
    out->front = st->front;
    out->stale = st->stale;
    out->W = st->W;
    out->smoothed = smoothed;
    out->slope = slope;
    out->T = st->has_T ? st->T : kNaN;
    return EGERIA_OK;
}

}  // extern "C"
