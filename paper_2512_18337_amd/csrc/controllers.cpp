// Host-side controllers of the serving loop.
//
//   speculation depth   spec_choose_k / spec_switch_frontier turn a measured cost table of the verification step
//                       and an acceptance probability into the depth that commits most tokens per unit of time and
//                       into the context / batch thresholds beyond which no depth pays; spec_adaptive_k is the
//                       threshold test itself (Sec. 5.4.2, adaptive switch; Alg. 4 step 4).
//   admission           agentsched_pick scores the waiting queue under the current KV-cache pressure and returns
//                       the best request that fits (Alg. 3).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "agentsam.h"

namespace {

// ---- speculation depth -----------------------------------------------------------------------------------------
// Tokens a step with `depth` drafts commits on average when every draft is accepted with probability p,
// independently, and acceptance stops at the first rejection: the token the target model emits anyway plus the
// accepted prefix, 1 + p + p^2 + ... + p^depth (summed term by term: exact for p = 1, no cancellation near it).
double committed_tokens(int depth, double p) {
    double term = 1.0, total = 1.0;
    for (int j = 1; j <= depth; ++j) {
        term *= p;
        total += term;
    }
    return total;
}

// What a step with `depth` drafts costs: the measured time of this path plus the layers outside it, which stream
// their weights once (a floor that does not depend on the rows) until the rows make them compute-bound.
double step_cost(double t_path, int depth, int batch, double other_floor, double other_per_row) {
    const double rows = (double)batch * (1.0 + depth);
    return t_path + std::max(other_floor, other_per_row * rows);
}

// index of the depth with the highest committed tokens per unit of cost (the shallower one on equal rates)
int best_depth(const int32_t *depths, const double *t_path, int n, double p, int batch, double other_floor,
               double other_per_row, double *rate_out) {
    int best = -1;
    double best_rate = 0.0;
    for (int i = 0; i < n; ++i) {
        const double rate = committed_tokens(depths[i], p) / step_cost(t_path[i], depths[i], batch, other_floor, other_per_row);
        if (best < 0 || rate > best_rate || (rate == best_rate && depths[i] < depths[best])) {
            best = i;
            best_rate = rate;
        }
    }
    if (rate_out) *rate_out = best_rate;
    return best;
}

bool valid_table(const int32_t *depths, const double *t, int n) {
    for (int i = 0; i < n; ++i) {
        if (depths[i] < 0 || !(t[i] > 0.0) || !std::isfinite(t[i])) return false;
        if (i > 0 && depths[i] <= depths[i - 1]) return false;
    }
    return n >= 1 && depths[0] == 0;
}

// ---- admission ---------------------------------------------------------------------------------------------------
double logistic(double x) {
    if (x >= 0.0) return 1.0 / (1.0 + std::exp(-x));
    const double e = std::exp(x);
    return e / (1.0 + e);
}

// The price of a KV block under the queue's pressure, and how far the cost of a request has moved from "its prompt
// length" (no pressure: shortest job first) to "the new blocks it needs" (full pressure).
struct Pressure {
    double price;            // in [0, price_max]
    double prompt_weight;    // 1 - price / price_max, in [0, 1]: the share of "prompt length" in a request's cost
};

Pressure queue_pressure(int64_t free_blocks, int64_t reusable_total, int64_t demand_total, double price_max,
                        double steepness, double eps) {
    const double capacity = (double)std::max<int64_t>(0, free_blocks - reusable_total);
    const double load = (double)demand_total / (capacity + eps);
    Pressure pr;
    pr.price = price_max * logistic(steepness * (load - 1.0));
    pr.prompt_weight = std::min(1.0, std::max(0.0, 1.0 - pr.price / price_max));
    return pr;
}

}  // namespace

extern "C" {

int spec_adaptive_k(int32_t batch, int64_t context_len, int32_t k, int32_t batch_threshold,
                    int64_t context_threshold, int32_t *k_out) {
    if (!k_out) return AGENTSAM_ERR_NULL;
    if (batch < 0 || context_len < 0 || k < 0) return AGENTSAM_ERR_ARG;
    *k_out = (context_len > context_threshold || batch > batch_threshold) ? 0 : k;
    return AGENTSAM_OK;
}

int spec_choose_k(const int32_t *k_values, const double *t_step, int32_t n, double p_accept, int32_t batch,
                  double other_floor, double other_per_row, int32_t *k_star, double *gain) {
    if (!k_values || !t_step || !k_star) return AGENTSAM_ERR_NULL;
    if (n < 1 || batch < 1 || !(p_accept >= 0.0 && p_accept <= 1.0) || !(other_floor >= 0.0) || !(other_per_row >= 0.0))
        return AGENTSAM_ERR_ARG;
    if (!valid_table(k_values, t_step, n)) return AGENTSAM_ERR_ARG;
    double rate = 0.0;
    const int i = best_depth(k_values, t_step, n, p_accept, batch, other_floor, other_per_row, &rate);
    *k_star = k_values[i];
    if (gain) *gain = rate * step_cost(t_step[0], 0, batch, other_floor, other_per_row);   // a plain step commits one token
    return AGENTSAM_OK;
}

int spec_switch_frontier(const int32_t *batches, int32_t n_batches, const int64_t *contexts, int32_t n_contexts,
                         const int32_t *k_values, int32_t n_k, const double *t_step, double p_accept,
                         double other_floor, double other_per_row, int32_t *k_star, int64_t *context_threshold,
                         int32_t *batch_threshold) {
    if (!batches || !contexts || !k_values || !t_step || !k_star || !context_threshold || !batch_threshold)
        return AGENTSAM_ERR_NULL;
    if (n_batches < 1 || n_contexts < 1 || n_k < 1 || !(p_accept >= 0.0 && p_accept <= 1.0) || !(other_floor >= 0.0) ||
        !(other_per_row >= 0.0))
        return AGENTSAM_ERR_ARG;
    for (int i = 0; i < n_batches; ++i)
        if (batches[i] < 1 || (i > 0 && batches[i] <= batches[i - 1])) return AGENTSAM_ERR_ARG;
    for (int j = 0; j < n_contexts; ++j)
        if (contexts[j] < 0 || (j > 0 && contexts[j] <= contexts[j - 1])) return AGENTSAM_ERR_ARG;
    for (int i = 0; i < n_batches; ++i)
        for (int j = 0; j < n_contexts; ++j) {
            const double *cell = t_step + ((int64_t)i * n_contexts + j) * n_k;
            if (!valid_table(k_values, cell, n_k)) return AGENTSAM_ERR_ARG;
            k_star[i * n_contexts + j] =
                k_values[best_depth(k_values, cell, n_k, p_accept, batches[i], other_floor, other_per_row, nullptr)];
        }
    // the largest grid value up to which speculation pays without interruption (-1: not even at the smallest)
    for (int i = 0; i < n_batches; ++i) {
        int64_t upto = -1;
        for (int j = 0; j < n_contexts && k_star[i * n_contexts + j] > 0; ++j) upto = contexts[j];
        context_threshold[i] = upto;
    }
    for (int j = 0; j < n_contexts; ++j) {
        int32_t upto = -1;
        for (int i = 0; i < n_batches && k_star[i * n_contexts + j] > 0; ++i) upto = batches[i];
        batch_threshold[j] = upto;
    }
    return AGENTSAM_OK;
}

int agentsched_pick(int64_t free_blocks, const int64_t *hit, const int64_t *need, const int64_t *prompt_tok,
                    const double *wait, int64_t n, double lambda_max, double k, double eps, double a, double b,
                    double c, int32_t tokens_per_block, double *lambda_out, double *score, int64_t *picked) {
    if (!lambda_out || !picked) return AGENTSAM_ERR_NULL;
    if (n < 0 || free_blocks < 0 || tokens_per_block < 1 || !(lambda_max > 0.0) || !(eps > 0.0)) return AGENTSAM_ERR_ARG;
    if (n > 0 && (!hit || !need || !prompt_tok || !wait)) return AGENTSAM_ERR_NULL;
    int64_t reusable_total = 0, demand_total = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (hit[i] < 0 || need[i] < 0 || prompt_tok[i] < 0) return AGENTSAM_ERR_ARG;
        reusable_total += hit[i];
        demand_total += need[i];
    }
    const Pressure pr = queue_pressure(free_blocks, reusable_total, demand_total, lambda_max, k, eps);
    *lambda_out = pr.price;
    // one pass over the queue: reward for cached blocks, price on the request's cost, reward for waiting; the best
    // request that fits is tracked on the way (a later request must score strictly higher to replace an earlier one)
    const double block_price = b + pr.price;
    int64_t best = -1;
    double best_score = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double prompt_blocks = (double)prompt_tok[i] / (double)tokens_per_block;
        const double cost_blocks = pr.prompt_weight * prompt_blocks + (1.0 - pr.prompt_weight) * (double)need[i];
        const double s = a * (double)hit[i] - block_price * cost_blocks + c * wait[i];
        if (score) score[i] = s;
        if (need[i] <= free_blocks && (best < 0 || s > best_score)) {
            best = i;
            best_score = s;
        }
    }
    *picked = best;
    return AGENTSAM_OK;
}

}  // extern "C"
