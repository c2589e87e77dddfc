// Batch-duration model (Sec. 4.2, Eq. 9): host-side least-squares fit of measured batch durations
// against the batch's size measure (uncached prefill tokens, or decode requests), and the prediction
// a scheduler makes from it.  No device work.
#include <cmath>

#include "relserve.h"

extern "C" {

int32_t relserve_duration_fit(const double* units, const double* seconds, int32_t n, relserve_duration_model* out) {
    if (!units || !seconds || !out) return RELSERVE_ERR_NULL_POINTER;
    if (n < 2) return RELSERVE_ERR_BAD_ARGUMENT;
    // centred sums in extended precision: token counts reach 1e4 while durations are ~1e-3, and the
    // uncentred normal equations would lose half of the digits
    long double mu = 0, ms = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (!std::isfinite(units[i]) || !std::isfinite(seconds[i])) return RELSERVE_ERR_BAD_ARGUMENT;
        mu += units[i];
        ms += seconds[i];
    }
    mu /= n;
    ms /= n;
    long double sxx = 0, sxy = 0, syy = 0;
    for (int32_t i = 0; i < n; ++i) {
        const long double du = units[i] - mu, ds = seconds[i] - ms;
        sxx += du * du;
        sxy += du * ds;
        syy += ds * ds;
    }
    if (sxx == 0) return RELSERVE_ERR_BAD_ARGUMENT;   // every batch has the same size: no slope
    const long double alpha = sxy / sxx, beta = ms - alpha * mu;
    long double ssr = 0;
    for (int32_t i = 0; i < n; ++i) {
        const long double r = seconds[i] - (alpha * units[i] + beta);
        ssr += r * r;
    }
    out->alpha = (double)alpha;
    out->beta = (double)beta;
    out->r2 = syy == 0 ? (ssr == 0 ? 1.0 : 0.0) : (double)(1 - ssr / syy);
    out->n = n;
    return RELSERVE_OK;
}

int32_t relserve_duration_predict(const relserve_duration_model* model, double units, double* seconds) {
    if (!model || !seconds) return RELSERVE_ERR_NULL_POINTER;
    *seconds = model->alpha * units + model->beta;
    return RELSERVE_OK;
}

}  // extern "C"
