// Host-only part of the C ABI: the outage-constrained link model and the early-exit ladder of
// Sec. II-D.2 (Eq. (comm_latency), Eq. (epsilon_rstar), Algorithm 2).  Scalar fp64 code; it makes
// no HIP call.  The sizes it reasons about are what tsq_blob_info reports for blobs that
// tsq_compress / tsq_compress_batch wrote.
#include <cmath>
#include <limits>

#include "tsq.h"

namespace {

bool link_ok(const tsq_link *l) {
    return l && l->bandwidth_hz > 0.0 && l->snr > 0.0 && l->outage > 0.0 && l->outage < 1.0 &&
           std::isfinite(l->bandwidth_hz) && std::isfinite(l->snr);
}

// P_o(R) = 1 - exp(-(2^(R/W) - 1) / gamma), through expm1 so that small arguments keep their digits
double outage_probability(const tsq_link &l, double rate) {
    const double x = (std::exp2(rate / l.bandwidth_hz) - 1.0) / l.snr;
    return -std::expm1(-x);
}

// ceil(ln eps / ln P_o): transmissions after which the residual outage is at most eps
double transmissions(const tsq_link &l, double rate) {
    const double po = outage_probability(l, rate);
    if (!(po < 1.0)) return std::numeric_limits<double>::infinity();   // every transmission fails
    if (!(po > 0.0)) return 1.0;                                       // none fails
    const double n = std::ceil(std::log(l.outage) / std::log(po));
    return n < 1.0 ? 1.0 : n;
}

double latency(const tsq_link &l, double bits, double rate) {
    if (bits <= 0.0) return 0.0;
    return bits / rate * transmissions(l, rate);
}

}  // namespace

extern "C" {

double tsq_link_outage_probability(const tsq_link *link, double rate) {
    if (!link_ok(link) || !(rate >= 0.0)) return std::numeric_limits<double>::quiet_NaN();
    return outage_probability(*link, rate);
}

double tsq_link_latency(const tsq_link *link, double bits, double rate) {
    if (!link_ok(link) || !(rate > 0.0) || !(bits >= 0.0)) return std::numeric_limits<double>::quiet_NaN();
    return latency(*link, bits, rate);
}

double tsq_link_best_rate(const tsq_link *link, double rate_lo, double rate_hi, uint32_t steps) {
    if (!link_ok(link) || !(rate_lo > 0.0) || !(rate_hi >= rate_lo) || steps == 0)
        return std::numeric_limits<double>::quiet_NaN();
    // Eq. (comm_latency) without its ceiling is D_tx * ln(1/eps) / (R * ln(1 / P_o(R))): the rate that
    // makes it smallest maximises R * ln(1 / P_o(R)).  Uniform grid of steps + 1 rates; the first best wins.
    double best = rate_lo, vbest = -1.0;
    for (uint32_t i = 0; i <= steps; ++i) {
        const double r = rate_lo + (rate_hi - rate_lo) * ((double)i / (double)steps);
        const double v = r * -std::log(outage_probability(*link, r));
        if (v > vbest) { vbest = v; best = r; }
    }
    return best;
}

tsq_status tsq_early_exit_decide(const tsq_exit_input *in, tsq_exit_decision *out) {
    if (!in || !out || !link_ok(&in->link) || !(in->rate > 0.0) || !(in->deadline >= 0.0) || !in->compute_latency ||
        !in->hidden_prefix_bits || !(in->raw_bits >= 0.0) || !(in->compressed_bits_with_kv >= 0.0))
        return TSQ_ERR_INVALID_ARG;
    const tsq_link &l = in->link;
    uint32_t w = in->tokens;
    const double lc = in->compute_latency[w];
    // as it is
    double t = lc + latency(l, in->raw_bits, in->rate);
    out->tokens = w; out->with_kv = 1; out->action = TSQ_EXIT_CONTINUE; out->latency = t;
    if (t <= in->deadline) return TSQ_OK;
    // compressed, cache included
    t = lc + latency(l, in->compressed_bits_with_kv, in->rate);
    out->action = TSQ_EXIT_COMPRESSED; out->latency = t;
    if (t <= in->deadline) return TSQ_OK;
    // compressed, hidden state only
    t = lc + latency(l, (double)in->hidden_prefix_bits[w], in->rate);
    out->action = TSQ_EXIT_WITHOUT_KV; out->with_kv = 0; out->latency = t;
    if (t <= in->deadline) return TSQ_OK;
    // fewer tokens
    out->action = TSQ_EXIT_FEWER_TOKENS;
    while (t > in->deadline && w > 0) {
        --w;
        t = in->compute_latency[w] + latency(l, (double)in->hidden_prefix_bits[w], in->rate);
    }
    out->tokens = w; out->latency = t;
    return TSQ_OK;
}

tsq_status tsq_early_exit_walk(const tsq_exit_walk_input *in, tsq_exit_walk_result *out) {
    if (!in || !out || !link_ok(&in->link) || !(in->rate > 0.0) || !(in->deadline >= 0.0) || !in->compute_latency ||
        !in->bits || in->layers == 0)
        return TSQ_ERR_INVALID_ARG;
    const tsq_link &l = in->link;
    const double D = in->deadline;
    tsq_status st = TSQ_OK;
    uint32_t steps = 0;
    // L_t of Eq. (total) for what the callbacks say; a size or a time that is negative or NaN ends the walk
    auto total = [&](uint32_t w_time, uint32_t w, uint32_t layer, int32_t ikv, int32_t compressed, uint32_t keep) {
        const double lc = in->compute_latency(w_time, layer, in->user);
        const double bits = in->bits(w, layer, ikv, compressed, keep, in->user);
        if (!(lc >= 0.0) || !(bits >= 0.0)) { st = TSQ_ERR_INVALID_ARG; return 0.0; }
        return lc + latency(l, bits, in->rate);
    };
    auto done = [&](int32_t action, int32_t ikv, uint32_t w, uint32_t layer, uint32_t keep, double t) {
        out->action = action; out->with_kv = ikv; out->tokens = w; out->layer = layer;
        out->sent_tokens = keep; out->steps = steps; out->latency = t;
        return st;
    };
    int32_t ikv = 1;
    for (uint32_t w = 1; w <= in->max_tokens; ++w)
        for (uint32_t layer = 1; layer <= in->layers; ++layer) {
            ++steps;                                           // the caller's forward pass up to `layer` for token w
            double t = total(w, w, layer, ikv, 0, w);
            if (st != TSQ_OK) return st;
            if (!(t > D)) continue;
            t = total(w, w, layer, ikv, 1, w);                 // TabQ(T_w; I_kv)
            if (st != TSQ_OK) return st;
            if (t <= D) return done(TSQ_EXIT_COMPRESSED, ikv, w, layer, w, t);
            ikv = 0;
            t = total(w, w, layer, 0, 1, w);
            if (st != TSQ_OK) return st;
            if (t > D) {
                uint32_t keep = w;
                while (t > D && keep > 0) {
                    --keep;
                    t = total(keep, w, layer, 0, 1, keep);
                    if (st != TSQ_OK) return st;
                }
                return done(TSQ_EXIT_FEWER_TOKENS, 0, w, layer, keep, t);
            }
        }
    const double t = total(in->max_tokens, in->max_tokens, in->layers, ikv, 1, in->max_tokens);
    if (st != TSQ_OK) return st;
    return done(TSQ_EXIT_COMPLETED, ikv, in->max_tokens, in->layers, in->max_tokens, t);
}

}  // extern "C"
