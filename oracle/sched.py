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


def expected_committed_oracle(k, p):
    """Tokens one speculative step commits on average (Sec. 5.4.2: drafts are checked in order and the first
    mismatch ends the accepted prefix; the main model's own next token is always committed).  Each draft is
    accepted with probability p, independently: a prefix of a < k drafts has probability p^a (1-p), all k
    have p^k, and a prefix of a drafts commits a + 1 tokens."""
    total = 0.0
    for a in range(k + 1):
        prob = p ** a * ((1.0 - p) if a < k else 1.0)
        total += prob * (a + 1)
    return total


def choose_k_oracle(k_values, t_step, p, batch=1, other_floor=0.0, other_per_row=0.0):
    """The depth with the most committed tokens per unit of cost (the smaller on equal rates), and that rate over
    the rate without speculation.  Cost of a step with k drafts: t_step[k] + max(other_floor, other_per_row *
    batch * (1 + k)) (Alg. 4 step 4: speculate only while it pays)."""
    def rate(i):
        cost = t_step[i] + max(other_floor, other_per_row * batch * (1 + k_values[i]))
        return expected_committed_oracle(k_values[i], p) / cost
    rates = [rate(i) for i in range(len(k_values))]
    best = max(range(len(k_values)), key=lambda i: (rates[i], -k_values[i]))
    return k_values[best], rates[best] / rates[0]


def switch_frontier_oracle(batches, contexts, k_values, t_step, p, other_floor=0.0, other_per_row=0.0):
    """choose_k_oracle at every (batch, context) grid point (t_step[i][j][:] is that point's table), and for each
    batch the largest context up to which speculation pays without interruption (-1: none), likewise per context."""
    kstar = [[choose_k_oracle(k_values, t_step[i][j], p, batches[i], other_floor, other_per_row)[0]
              for j in range(len(contexts))] for i in range(len(batches))]
    ctx_thr = []
    for i in range(len(batches)):
        upto = -1
        for j in range(len(contexts)):
            if kstar[i][j] == 0:
                break
            upto = contexts[j]
        ctx_thr.append(upto)
    batch_thr = []
    for j in range(len(contexts)):
        upto = -1
        for i in range(len(batches)):
            if kstar[i][j] == 0:
                break
            upto = batches[i]
        batch_thr.append(upto)
    return kstar, ctx_thr, batch_thr
