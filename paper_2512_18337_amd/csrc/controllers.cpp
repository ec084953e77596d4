// Host-side controllers of the serving loop: the adaptive speculation switch (paper Sec. 5.4.2,
// "Adaptive switch for speculative decoding"; Alg. 4 step 4) and the AgentSched pick (Alg. 3).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <new>
#include <numeric>
#include <vector>

#include "agentsam.h"

extern "C" {

int spec_adaptive_k(int32_t batch, int64_t context_len, int32_t k, int32_t batch_threshold,
                    int64_t context_threshold, int32_t *k_out) {
    if (!k_out) return AGENTSAM_ERR_NULL;
    if (batch < 0 || context_len < 0 || k < 0) return AGENTSAM_ERR_ARG;
    *k_out = (context_len > context_threshold || batch > batch_threshold) ? 0 : k;
    return AGENTSAM_OK;
}

int agentsched_pick(int64_t free_blocks, const int64_t *hit, const int64_t *need, const int64_t *prompt_tok,
                    const double *wait, int64_t n, double lambda_max, double k, double eps, double a, double b,
                    double c, int32_t tokens_per_block, double *lambda_out, double *score, int64_t *picked) {
    if (!lambda_out || !picked) return AGENTSAM_ERR_NULL;
    if (n < 0 || free_blocks < 0 || tokens_per_block < 1 || !(lambda_max > 0.0) || !(eps > 0.0)) return AGENTSAM_ERR_ARG;
    if (n > 0 && (!hit || !need || !prompt_tok || !wait)) return AGENTSAM_ERR_NULL;
    // Step 2: pressure on the capacity left once the queue's cached blocks are counted in
    int64_t H = 0, D = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (hit[i] < 0 || need[i] < 0 || prompt_tok[i] < 0) return AGENTSAM_ERR_ARG;
        H += hit[i];
        D += need[i];
    }
    const int64_t U = std::max<int64_t>(0, free_blocks - H);
    const double z = (double)D / ((double)U + eps);
    const double x = k * (z - 1.0);
    const double sig = x >= 0 ? 1.0 / (1.0 + std::exp(-x)) : std::exp(x) / (1.0 + std::exp(x));
    const double lam = lambda_max * sig;
    *lambda_out = lam;
    // Step 3: between shortest-job-first (no pressure) and KV-aware (full pressure)
    const double sjf_mix = std::min(1.0, std::max(0.0, 1.0 - lam / lambda_max));
    std::vector<double> local;
    double *sc = score;
    try {
        if (!sc) { local.resize((size_t)n); sc = local.data(); }
        for (int64_t i = 0; i < n; ++i) {
            const double need_tok = (double)prompt_tok[i] / (double)tokens_per_block;
            const double need_eff = sjf_mix * need_tok + (1.0 - sjf_mix) * (double)need[i];
            sc[i] = a * (double)hit[i] - (b + lam) * need_eff + c * wait[i];
        }
        // Step 4: the best-scoring request whose new blocks fit (earlier request on equal scores)
        int64_t best = -1;
        for (int64_t i = 0; i < n; ++i)
            if (need[i] <= free_blocks && (best < 0 || sc[i] > sc[best])) best = i;
        *picked = best;
    } catch (const std::bad_alloc &) {
        return AGENTSAM_ERR_NOMEM;
    }
    return AGENTSAM_OK;
}

}  // extern "C"
