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

// ---- Priority Estimation Model (Sec. 4.2: Algorithm 1 and Eq. 10) ----
// One walk over the requests in order.  State: tokens of the open prefill batch, requests of the open decode
// group, tokens held on the GPU since the last decode-to-completion.
namespace {
struct PemWalk {
    int32_t out_len;
    int32_t* prefill_utok;                 // optional outputs
    int32_t* group_req;
    const relserve_duration_model* mp;     // optional: the lines to sum
    const relserve_duration_model* md;
    int32_t n_prefill = 0, n_groups = 0;
    int64_t p_tok = 0, accum = 0;
    int32_t p_req = 0, d_req = 0;
    double seconds = 0;

    void close_prefill() {
        if (p_req > 0) {
            if (prefill_utok) prefill_utok[n_prefill] = (int32_t)p_tok;
            if (mp) seconds += mp->alpha * (double)p_tok + mp->beta;
            ++n_prefill;
        }
        p_tok = 0;
        p_req = 0;
    }
    void decode_to_completion() {
        if (d_req > 0) {
            if (group_req) group_req[n_groups] = d_req;
            if (md) seconds += (double)out_len * (md->alpha * (double)d_req + md->beta);
            ++n_groups;
        }
        d_req = 0;
        accum = 0;
    }
};

int32_t pem_walk(const int32_t* utok, const uint8_t* decodes, int32_t n, int32_t out_len, const relserve_pem_limits* lim,
                 int32_t* prefill_batch_of, int32_t* decode_group_of, PemWalk& w) {
    if (n < 0 || out_len < 0 || !lim || lim->cap < 0 || lim->max_num_seqs < 1 || lim->max_num_batched_tokens < 1)
        return RELSERVE_ERR_BAD_ARGUMENT;
    if (n > 0 && !utok) return RELSERVE_ERR_NULL_POINTER;
    for (int32_t i = 0; i < n; ++i)
        if (utok[i] < 0) return RELSERVE_ERR_BAD_ARGUMENT;
    for (int32_t i = 0; i < n; ++i) {
        const bool dec = !decodes || decodes[i] != 0;
        if ((int64_t)utok[i] + w.accum > lim->cap || w.d_req + (dec ? 1 : 0) > lim->max_num_seqs) {
            w.close_prefill();
            w.decode_to_completion();
        }
        if ((int64_t)utok[i] + w.p_tok > lim->max_num_batched_tokens) w.close_prefill();
        if (prefill_batch_of) prefill_batch_of[i] = utok[i] > 0 ? w.n_prefill : -1;
        if (decode_group_of) decode_group_of[i] = dec ? w.n_groups : -1;
        if (utok[i] > 0) {
            w.p_tok += utok[i];
            ++w.p_req;
        }
        if (dec) ++w.d_req;
        w.accum += utok[i];
    }
    w.close_prefill();
    w.decode_to_completion();
    return RELSERVE_OK;
}
}  // namespace

extern "C" {

int32_t relserve_batch_decompose(const int32_t* utok, const uint8_t* decodes, int32_t n, int32_t out_len,
                                 const relserve_pem_limits* limits, int32_t* prefill_batch_of, int32_t* decode_group_of,
                                 int32_t* prefill_utok, int32_t* n_prefill, int32_t* group_req, int32_t* n_groups) {
    if (!limits || !n_prefill || !n_groups) return RELSERVE_ERR_NULL_POINTER;
    PemWalk w{out_len, prefill_utok, group_req, nullptr, nullptr};
    if (int32_t rc = pem_walk(utok, decodes, n, out_len, limits, prefill_batch_of, decode_group_of, w)) return rc;
    *n_prefill = w.n_prefill;
    *n_groups = w.n_groups;
    return RELSERVE_OK;
}

int32_t relserve_pem_estimate(const int32_t* utok, const uint8_t* decodes, int32_t n, int32_t out_len,
                              const relserve_pem_limits* limits, const relserve_duration_model* prefill,
                              const relserve_duration_model* decode, double* seconds) {
    if (!limits || !prefill || !decode || !seconds) return RELSERVE_ERR_NULL_POINTER;
    PemWalk w{out_len, nullptr, nullptr, prefill, decode};
    if (int32_t rc = pem_walk(utok, decodes, n, out_len, limits, nullptr, nullptr, w)) return rc;
    *seconds = w.seconds;
    return RELSERVE_OK;
}

}  // extern "C"

// ---- Adaptive Batch Arranger decision (Sec. 4.3, Eq. 14-17) and starvation rule (Sec. 4.2, Eq. 13) ----
extern "C" {

int32_t relserve_aba_decide(const relserve_aba_input* in, const relserve_duration_model* prefill,
                            const relserve_duration_model* decode, int32_t* decision, double* delta) {
    if (!in || !prefill || !decode || !decision) return RELSERVE_ERR_NULL_POINTER;
    if (in->n_running_reqs < 0 || in->cand_prefill_reqs < 0 || in->cand_prefill_utok < 0 || in->cand_prefill_out_len < 0 ||
        in->n_running_relqueries < 0 || in->n_waiting_relqueries < 0)
        return RELSERVE_ERR_BAD_ARGUMENT;
    if (delta) *delta = 0.0;
    if (in->n_running_reqs == 0 && in->cand_prefill_reqs == 0) { *decision = RELSERVE_ABA_IDLE; return RELSERVE_OK; }
    if (in->n_running_reqs == 0) { *decision = RELSERVE_ABA_PREFILL; return RELSERVE_OK; }
    if (in->cand_prefill_reqs == 0) { *decision = RELSERVE_ABA_DECODE; return RELSERVE_OK; }
    if (in->m_running >= in->m_waiting) { *decision = RELSERVE_ABA_PREFILL; return RELSERVE_OK; }   // preemption / same relQuery
    // transitional case: latency added to the running relQueries against latency saved for the waiting ones
    if (in->n_running_relqueries < 1 || !in->running_out_len) return RELSERVE_ERR_BAD_ARGUMENT;
    const double l_prefill = prefill->alpha * (double)in->cand_prefill_utok + prefill->beta;
    double d_plus = l_prefill * (double)in->n_running_relqueries;
    int32_t max_ol = 0;
    for (int32_t i = 0; i < in->n_running_relqueries; ++i) {
        const int32_t ol = in->running_out_len[i];
        if (ol < 0) return RELSERVE_ERR_BAD_ARGUMENT;
        d_plus += decode->alpha * (double)in->cand_prefill_reqs * (double)(ol < in->cand_prefill_out_len ? ol : in->cand_prefill_out_len);
        if (ol > max_ol) max_ol = ol;
    }
    const double d_minus = (double)in->n_waiting_relqueries * decode->beta *
                           (double)(in->cand_prefill_out_len < max_ol ? in->cand_prefill_out_len : max_ol);
    const double d = d_plus - d_minus;
    if (delta) *delta = d;
    *decision = d < 0 ? RELSERVE_ABA_PREFILL : RELSERVE_ABA_DECODE;
    return RELSERVE_OK;
}

int32_t relserve_starved_priority(double priority, double waiting_seconds, int32_t n_requests_submitted, double threshold,
                                  double* out) {
    if (!out) return RELSERVE_ERR_NULL_POINTER;
    if (n_requests_submitted < 1) return RELSERVE_ERR_BAD_ARGUMENT;
    *out = waiting_seconds / (double)n_requests_submitted > threshold ? 0.0 : priority;
    return RELSERVE_OK;
}

}  // extern "C"

// ---- the rest of the scheduler's per-iteration arithmetic (Sec. 3 Eq. 6-7; Sec. 4.2 Eq. 11-12; Sec. 4.3 candidates) ----
extern "C" {

int32_t relserve_static_priority(const int32_t* tok, int32_t n, int32_t out_len, const relserve_duration_model* l1,
                                 const relserve_duration_model* l2, double* priority) {
    if (!l1 || !l2 || !priority) return RELSERVE_ERR_NULL_POINTER;
    if (n < 0 || out_len < 0) return RELSERVE_ERR_BAD_ARGUMENT;
    if (n > 0 && !tok) return RELSERVE_ERR_NULL_POINTER;
    double sum = 0.0;
    for (int32_t i = 0; i < n; ++i) {
        if (tok[i] < 0) return RELSERVE_ERR_BAD_ARGUMENT;
        sum += (l1->alpha * (double)tok[i] + l1->beta) + (l2->alpha * (double)out_len + l2->beta);   // Eq. 6, summed as Eq. 7
    }
    *priority = sum;
    return RELSERVE_OK;
}

int32_t relserve_utok_estimate(const int32_t* tok, int32_t n, const int32_t* sample_tok, const int32_t* sample_utok,
                               int32_t n_sample, int32_t* utok_out) {
    if (n < 0 || n_sample < 1) return RELSERVE_ERR_BAD_ARGUMENT;
    if (!sample_tok || !sample_utok || (n > 0 && (!tok || !utok_out))) return RELSERVE_ERR_NULL_POINTER;
    int64_t su = 0, st = 0;
    for (int32_t i = 0; i < n_sample; ++i) {
        if (sample_tok[i] < 0 || sample_utok[i] < 0 || sample_utok[i] > sample_tok[i]) return RELSERVE_ERR_BAD_ARGUMENT;
        su += sample_utok[i];
        st += sample_tok[i];
    }
    if (st == 0) return RELSERVE_ERR_BAD_ARGUMENT;
    const double ratio = (double)su / (double)st;                      // cache miss ratio of the sample
    for (int32_t i = 0; i < n; ++i) {
        if (tok[i] < 0) return RELSERVE_ERR_BAD_ARGUMENT;
        utok_out[i] = (int32_t)__builtin_nearbyint((double)tok[i] * ratio);   // ties to even
    }
    return RELSERVE_OK;
}

int32_t relserve_priority_reuse(int32_t n_submitted, int32_t n_waiting_before, int32_t n_waiting_now, int32_t* reuse) {
    if (!reuse) return RELSERVE_ERR_NULL_POINTER;
    if (n_submitted < 1 || n_waiting_before < 0 || n_waiting_now < 0 || n_waiting_before > n_submitted ||
        n_waiting_now > n_waiting_before)
        return RELSERVE_ERR_BAD_ARGUMENT;
    *reuse = (n_waiting_before == n_submitted && n_waiting_now == n_submitted) ? 1 : 0;
    return RELSERVE_OK;
}

int32_t relserve_prefill_candidate(const int32_t* utok, int32_t n, int64_t tokens_free, int32_t seqs_free,
                                   int32_t tokens_in_batch, int32_t max_num_batched_tokens, int32_t* n_taken,
                                   int64_t* tokens_taken) {
    if (!n_taken || !tokens_taken) return RELSERVE_ERR_NULL_POINTER;
    if (n < 0 || tokens_in_batch < 0 || max_num_batched_tokens < 1) return RELSERVE_ERR_BAD_ARGUMENT;
    if (n > 0 && !utok) return RELSERVE_ERR_NULL_POINTER;
    int32_t taken = 0;
    int64_t toks = 0;
    for (int32_t i = 0; i < n; ++i) {
        const int64_t u = utok[i];
        if (u < 0) return RELSERVE_ERR_BAD_ARGUMENT;
        if (seqs_free - taken < 1 || u > tokens_free - toks) break;                                    // max_num_seqs, cap
        if (tokens_in_batch + toks + u > max_num_batched_tokens && (taken > 0 || tokens_in_batch > 0)) break;
        ++taken;
        toks += u;
    }
    *n_taken = taken;
    *tokens_taken = toks;
    return RELSERVE_OK;
}

}  // extern "C"

