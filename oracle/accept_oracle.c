/*
 * CPU oracle for greedy acceptance.  TEST INFRASTRUCTURE ONLY (called by the
 * tests, the smoke check and the benchmark's CPU-baseline leg; never by the
 * product path; shares no code with the HIP library).
 *
 * Alg. 4, "Validate with main LLM; commit matched prefix"; Sec. 5.4.1 calls the
 * acceleration lossless, so the committed tokens are exactly what greedy
 * decoding would have produced.  Written as a scalar loop:
 *
 *   tgt[b,i]      = the lowest index attaining the maximum of logits[b,i,:]
 *                   (a NaN never wins; a row with no finite maximum gives 0)
 *   a_b           = number of leading drafts j < n_draft[b] with draft[b,j] == tgt[b,j]
 *   out[b,0..a_b] = tgt[b,0..a_b]  (accepted drafts and the bonus token), rest -1
 *
 * Logits arrive as float32; bf16 logits are widened exactly by the caller, so
 * every comparison sees the stored value.
 */
#include <stdint.h>
#include <math.h>

void accept_oracle(const float *logits, const int32_t *draft, const int32_t *n_draft,
                   int32_t B, int32_t k, int64_t V,
                   int32_t *accept_len, int32_t *out_tokens /* [B,1+k] */, int32_t *tgt /* [B,1+k] */)
{
    const int32_t R = 1 + k;
    for (int32_t b = 0; b < B; ++b) {
        for (int32_t i = 0; i < R; ++i) {
            const float *row = logits + ((int64_t)b * R + i) * V;
            double best_v = -INFINITY;
            int64_t best = 0;
            for (int64_t v = 0; v < V; ++v) {
                double x = (double)row[v];
                if (x > best_v) {           /* strict: first maximum wins; NaN compares false */
                    best_v = x;
                    best = v;
                }
            }
            tgt[(int64_t)b * R + i] = (int32_t)best;
        }
        int32_t a = 0;
        while (a < n_draft[b] && a < k && draft[(int64_t)b * k + a] == tgt[(int64_t)b * R + a])
            ++a;
        accept_len[b] = a;
        for (int32_t i = 0; i < R; ++i)
            out_tokens[(int64_t)b * R + i] = (i <= a) ? tgt[(int64_t)b * R + i] : -1;
    }
}
