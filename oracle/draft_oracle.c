/*
 * CPU oracle for the AgentSAM draft lookup.  TEST INFRASTRUCTURE ONLY: it is
 * called by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg, never by the product path, and shares no code with the HIP library.
 *
 * What it computes (paper Sec. 5.4.2, "Algorithm design"; Alg. 4 step
 * FollowTransitions): given the current verified suffix of a session (the
 * window q of its most recent tokens) and an indexed token memory T, find a
 * matching continuation of a specified length k.  A suffix automaton reaches
 * exactly the result of the plain definition below, so the oracle is that
 * definition written out as a brute-force backward scan:
 *
 *   - an end position e of T is ELIGIBLE when a continuation exists there:
 *     e+1 < N and T[e+1] != SEP;
 *   - for every eligible e, count how many tokens T[e], T[e-1], ... agree with
 *     q[m-1], q[m-2], ... (the common-suffix length, at most m);
 *   - the answer is the eligible e with the longest common suffix, the largest
 *     such e on ties (most recent occurrence); match_len is that length;
 *   - the draft is T[e+1], T[e+2], ... up to k tokens, stopping before N and
 *     before a SEP;
 *   - if the best length is below min_match (or 0) nothing is proposed:
 *     match_len = 0, match_end = -1, n_draft = 0.
 *
 * Readings the paper leaves open (which occurrence, what happens at the tail
 * of the memory, separators between sessions) are fixed as above.
 */
#include <stdint.h>

void draft_oracle(const int32_t *T, int64_t N, int32_t sep,
                  const int32_t *q, int32_t m, int32_t k, int32_t min_match,
                  int32_t *draft /* [k] */, int32_t *n_draft,
                  int32_t *match_len, int64_t *match_end)
{
    int32_t best_len = 0;
    int64_t best_end = -1;
    for (int64_t e = 0; e < N; ++e) {
        if (!(e + 1 < N && T[e + 1] != sep))
            continue;                       /* no continuation after e */
        int32_t L = 0;
        while (L < m && e - L >= 0 && T[e - L] == q[m - 1 - L])
            ++L;
        if (L > 0 && L >= best_len) {       /* e ascends: ties go to the later e */
            best_len = L;
            best_end = e;
        }
    }
    for (int32_t j = 0; j < k; ++j)
        draft[j] = -1;
    *n_draft = 0;
    if (best_len < min_match || best_len == 0) {
        *match_len = 0;
        *match_end = -1;
        return;
    }
    *match_len = best_len;
    *match_end = best_end;
    int32_t n = 0;
    while (n < k && best_end + 1 + n < N && T[best_end + 1 + n] != sep) {
        draft[n] = T[best_end + 1 + n];
        ++n;
    }
    *n_draft = n;
}

/* Batch form: session b searches memory T[mem_off[b] .. mem_off[b+1]) with
 * window q[b, m - q_len[b] .. m) (windows are right-aligned in a [B, m] array).
 * match_end is relative to the session's own memory. */
void draft_oracle_batch(const int32_t *T, const int64_t *mem_begin, const int64_t *mem_end, int32_t sep,
                        const int32_t *q, const int32_t *q_len, int32_t B, int32_t m,
                        int32_t k, int32_t min_match,
                        int32_t *draft /* [B,k] */, int32_t *n_draft, int32_t *match_len,
                        int64_t *match_end)
{
    for (int32_t b = 0; b < B; ++b) {
        int32_t ql = q_len[b];
        draft_oracle(T + mem_begin[b], mem_end[b] - mem_begin[b], sep,
                     q + (int64_t)b * m + (m - ql), ql, k, min_match,
                     draft + (int64_t)b * k, n_draft + b, match_len + b, match_end + b);
    }
}
