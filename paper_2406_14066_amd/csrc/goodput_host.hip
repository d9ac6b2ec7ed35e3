// Host-side speculation control: the goodput model and the search for the proposed
// length (arXiv 2406.14066, Section 4.1 "Using Goodput for Speculation", Eq. 1-4, and
// Section 4.2's listing "Finding k to maximize goodput").  Plain host code: nothing
// here touches the GPU.
#include "spec_verify.h"

#include <math.h>

extern "C" {

double spec_expected_generated_len(double alpha, int32_t k)
{
    if (!(alpha >= 0.0 && alpha <= 1.0) || k < 0) return NAN;
    // Eq. 4 as the finite geometric sum 1 + a + ... + a^k: no cancellation near a = 1
    double sum = 0.0, term = 1.0;
    for (int j = 0; j <= k; ++j) {
        sum += term;
        term *= alpha;
    }
    return sum;
}

double spec_predict_latency(const spec_latency_model *model, double n_context, double n_batched)
{
    if (model == nullptr) return NAN;
    return model->c_context * n_context + model->c_batched * n_batched + model->c_fixed;   // Eq. 3
}

// Least squares for Eq. 3: normal equations of the centred problem (two unknowns), then
// the constant from the means.  Centring keeps the 2x2 system well conditioned when the
// token counts are in the thousands.
spec_status spec_fit_latency(const double *n_context, const double *n_batched, const double *seconds, int32_t n,
                             spec_latency_model *model)
{
    if (n_context == nullptr || n_batched == nullptr || seconds == nullptr || model == nullptr || n < 3)
        return SPEC_EINVAL;
    double mc = 0.0, mb = 0.0, mt = 0.0;
    for (int i = 0; i < n; ++i) { mc += n_context[i]; mb += n_batched[i]; mt += seconds[i]; }
    mc /= n; mb /= n; mt /= n;
    double scc = 0.0, sbb = 0.0, scb = 0.0, sct = 0.0, sbt = 0.0;
    for (int i = 0; i < n; ++i) {
        const double c = n_context[i] - mc, b = n_batched[i] - mb, t = seconds[i] - mt;
        scc += c * c; sbb += b * b; scb += c * b; sct += c * t; sbt += b * t;
    }
    const double det = scc * sbb - scb * scb;
    if (!(det > 1e-12 * scc * sbb) || !(scc > 0.0) || !(sbb > 0.0)) return SPEC_EINVAL;   // dependent columns
    model->c_context = (sct * sbb - sbt * scb) / det;
    model->c_batched = (sbt * scc - sct * scb) / det;
    model->c_fixed = mt - model->c_context * mc - model->c_batched * mb;
    return SPEC_OK;
}

void spec_acceptance_update(spec_acceptance_tracker *tracker, int64_t accepted, int64_t attempted, double decay)
{
    if (tracker == nullptr || attempted <= 0 || accepted < 0 || accepted > attempted) return;
    if (!(decay > 0.0 && decay <= 1.0)) decay = 1.0;
    tracker->accepted_weighted = tracker->accepted_weighted * decay + (double)accepted;
    tracker->attempted_weighted = tracker->attempted_weighted * decay + (double)attempted;
}

double spec_acceptance_rate(const spec_acceptance_tracker *tracker, double prior)
{
    if (tracker == nullptr || !(tracker->attempted_weighted > 0.0)) return prior;
    return tracker->accepted_weighted / tracker->attempted_weighted;
}

int32_t spec_argmax_goodput(const spec_goodput_args *a, double *goodput_per_k)
{
    if (a == nullptr || a->B < 1 || a->max_k < 0 || a->max_k > SPEC_K_MAX || a->context_len == nullptr ||
        a->alpha == nullptr)
        return -1;
    double n_context = 0.0;
    for (int b = 0; b < a->B; ++b) {
        if (a->context_len[b] < 0) return -1;
        n_context += (double)a->context_len[b];
    }
    const int n_alpha = a->alpha_per_request ? a->B : 1;
    for (int i = 0; i < n_alpha; ++i)
        if (!(a->alpha[i] >= 0.0 && a->alpha[i] <= 1.0)) return -1;

    int best_k = -1;
    double best = -1.0;
    for (int k = 0; k <= a->max_k; ++k) {
        if (goodput_per_k != nullptr) goodput_per_k[k] = NAN;
        const int64_t new_tokens = (int64_t)a->B * (k + 1);
        if (a->free_kv_tokens >= 0 && new_tokens > a->free_kv_tokens) continue;   // would not fit in the KV cache
        double generated = 0.0;
        if (a->alpha_per_request) {
            for (int b = 0; b < a->B; ++b) generated += spec_expected_generated_len(a->alpha[b], k);
        } else {
            generated = (double)a->B * spec_expected_generated_len(a->alpha[0], k);
        }
        double seconds = spec_predict_latency(&a->target, n_context, (double)new_tokens);   // Eq. 2: T_target ...
        if (k > 0)                                                                           // ... + T_draft
            seconds += a->draft_is_model ? (double)k * spec_predict_latency(&a->draft, n_context, (double)a->B)
                                         : a->draft_fixed_seconds;
        if (!(seconds > 0.0)) return -1;   // a model that predicts no time at all is unusable
        const double goodput = generated / seconds;   // Eq. 1
        if (goodput_per_k != nullptr) goodput_per_k[k] = goodput;
        if (goodput > best) { best = goodput; best_k = k; }
    }
    return best_k;
}

}  // extern "C"
