"""Oracle of the AgentSched pick (paper Alg. 3) and of the adaptive speculation switch (Alg. 4, step 4).

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain Python / float64, one request at a time, in
the order and notation of the algorithms.  Readings where the paper is silent: sigma is the logistic
function; a request is feasible when the new blocks it needs fit into the free blocks; ties in score go
to the earlier request; the constants a, b, c, k, lambda_max, epsilon are parameters (the paper prints
none); the integral state and the gains k_P, k_I, beta listed among the parameters are not used by the
printed update, so they are not used here.
"""
from __future__ import annotations

import math


def agentsched_oracle(free_blocks, hit, need, prompt_tok, wait, lambda_max, k, eps, a, b, c, tokens_per_block):
    """Returns (lambda, scores, picked index or -1)."""
    n = len(hit)
    # Step 2: shadow price from the pressure on the effective capacity
    H = sum(int(x) for x in hit)
    U = max(0, int(free_blocks) - H)
    D = sum(int(x) for x in need)
    z = D / (U + eps)
    x = k * (z - 1.0)
    if x >= 0:
        sig = 1.0 / (1.0 + math.exp(-x))
    else:
        ex = math.exp(x)
        sig = ex / (1.0 + ex)
    lam = lambda_max * sig
    # Step 3: scores
    sjf_mix = min(1.0, max(0.0, 1.0 - lam / lambda_max))
    scores = []
    for i in range(n):
        need_tok = prompt_tok[i] / tokens_per_block
        need_eff = sjf_mix * need_tok + (1.0 - sjf_mix) * need[i]
        scores.append(a * hit[i] - (b + lam) * need_eff + c * wait[i])
    # Step 4: first feasible candidate in descending score order
    order = sorted(range(n), key=lambda i: (-scores[i], i))
    picked = -1
    for i in order:
        if need[i] <= free_blocks:
            picked = i
            break
    return lam, scores, picked


def adaptive_k_oracle(batch, context_len, k, batch_threshold, context_threshold):
    """Alg. 4 step 4: no speculation beyond either threshold."""
    if context_len > context_threshold or batch > batch_threshold:
        return 0
    return k
