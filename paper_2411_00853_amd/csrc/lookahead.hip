// Host-side lookahead controller of spec_decode.h: per-sequence acceptance estimates with
// exponential forgetting and the K that maximises predicted tokens per millisecond.  No device code.
#include <cmath>
#include <vector>

#include "common.h"
#include "../../include/spec_decode.h"

using namespace specv;

struct spec_lookahead {
    spec_lookahead_cfg cfg;
    std::vector<double> tested, kept;
};

namespace {
double alpha_of(const spec_lookahead* c, int b)
{
    return (c->kept[b] + c->cfg.prior_accept * c->cfg.prior_weight) / (c->tested[b] + c->cfg.prior_weight);
}
}  // namespace

extern "C" int spec_lookahead_init(const spec_lookahead_cfg* cfg, int32_t batch, spec_lookahead** out)
{
    if (!cfg || !out) return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_init: NULL argument");
    if (batch < 1 || batch > SPEC_MAX_BATCH) return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_init: batch outside 1..%d", SPEC_MAX_BATCH);
    if (cfg->k_min < 1 || cfg->k_max < cfg->k_min || cfg->k_max > SPEC_MAX_LOOKAHEAD)
        return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_init: need 1 <= k_min <= k_max <= %d", SPEC_MAX_LOOKAHEAD);
    if (!(cfg->draft_ms >= 0.0) || !(cfg->verify_ms > 0.0) || !(cfg->verify_ms_per_token >= 0.0))
        return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_init: costs must be non-negative and verify_ms positive");
    if (!(cfg->forget > 0.0 && cfg->forget <= 1.0) || !(cfg->prior_accept >= 0.0 && cfg->prior_accept <= 1.0)
        || !(cfg->prior_weight > 0.0))
        return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_init: forget in (0,1], prior_accept in [0,1], prior_weight > 0");
    spec_lookahead* c = new spec_lookahead();
    c->cfg = *cfg;
    c->tested.assign(batch, 0.0);
    c->kept.assign(batch, 0.0);
    *out = c;
    return SPEC_OK;
}

extern "C" void spec_lookahead_destroy(spec_lookahead* c) { delete c; }

extern "C" int spec_lookahead_update(spec_lookahead* c, const int32_t* n_accepted, int32_t K)
{
    if (!c || !n_accepted) return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_update: NULL argument");
    if (K < 1 || K > SPEC_MAX_LOOKAHEAD) return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_update: K outside 1..%d", SPEC_MAX_LOOKAHEAD);
    for (size_t b = 0; b < c->tested.size(); ++b) {
        const int a = n_accepted[b];
        if (a < 0) continue;
        if (a > K) return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_update: n_accepted[%zu] = %d exceeds K = %d", b, a, K);
        const int tested = a + 1 < K ? a + 1 : K;
        c->tested[b] = c->cfg.forget * c->tested[b] + (double)tested;
        c->kept[b] = c->cfg.forget * c->kept[b] + (double)a;
    }
    return SPEC_OK;
}

namespace {
// the K with the best predicted tokens per millisecond, and that rate
int best_k(const spec_lookahead* c, double* rate_out)
{
    int best_k = c->cfg.k_min;
    double best = -1.0;
    for (int K = c->cfg.k_min; K <= c->cfg.k_max; ++K) {
        double tokens = 0.0;
        for (size_t b = 0; b < c->tested.size(); ++b) {
            const double al = alpha_of(c, (int)b);
            tokens += al < 1.0 ? (1.0 - std::pow(al, (double)(K + 1))) / (1.0 - al) : (double)(K + 1);
        }
        const double rate = tokens / ((double)K * c->cfg.draft_ms + c->cfg.verify_ms + (double)K * c->cfg.verify_ms_per_token);
        if (rate > best) {
            best = rate;
            best_k = K;
        }
    }
    if (rate_out) *rate_out = best;
    return best_k;
}
}  // namespace

extern "C" int32_t spec_lookahead_next(const spec_lookahead* c)
{
    if (!c) return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_next: NULL argument");
    return best_k(c, nullptr);
}

extern "C" int32_t spec_lookahead_next_per_seq(const spec_lookahead* c, int32_t* K_out)
{
    if (!c || !K_out) return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_next_per_seq: NULL argument");
    double rate = 0.0;
    const int K = best_k(c, &rate);
    const double worth = rate * c->cfg.verify_ms_per_token / (double)c->tested.size();
    for (size_t b = 0; b < c->tested.size(); ++b) {
        const double al = alpha_of(c, (int)b);
        int kb = 1;                               // one proposal is always tested
        double reach = 1.0;                       // alpha_b^k
        for (int k = 1; k <= K; ++k) {
            reach *= al;
            if (reach >= worth) kb = k;
            else break;
        }
        K_out[b] = kb;
    }
    return K;
}

extern "C" int spec_lookahead_update_per_seq(spec_lookahead* c, const int32_t* n_accepted, const int32_t* K_per_seq)
{
    if (!c || !n_accepted || !K_per_seq) return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_update_per_seq: NULL argument");
    for (size_t b = 0; b < c->tested.size(); ++b) {
        const int a = n_accepted[b], K = K_per_seq[b];
        if (K < 0 || K > SPEC_MAX_LOOKAHEAD)
            return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_update_per_seq: K_per_seq[%zu] = %d outside 0..%d", b, K, SPEC_MAX_LOOKAHEAD);
        if (a > K) return fail(SPEC_ERR_INVALID_ARG, "spec_lookahead_update_per_seq: n_accepted[%zu] = %d exceeds K = %d", b, a, K);
    }
    for (size_t b = 0; b < c->tested.size(); ++b) {
        const int a = n_accepted[b], K = K_per_seq[b];
        if (a < 0) continue;
        const int tested = a + 1 < K ? a + 1 : K;
        c->tested[b] = c->cfg.forget * c->tested[b] + (double)tested;
        c->kept[b] = c->cfg.forget * c->kept[b] + (double)a;
    }
    return SPEC_OK;
}

extern "C" double spec_lookahead_accept(const spec_lookahead* c, int32_t b)
{
    if (!c || b < 0 || (size_t)b >= c->tested.size()) return std::nan("");
    return alpha_of(c, b);
}
